"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This package holds input generators only: circuit DAGs and leaf weights.  None of
the evaluation arithmetic (neither the oracle's nor the GPU library's) lives here.
"""
from .circuits import (AND, FALSE, LIT, OR, TRUE, Circuit, CircuitBuilder, layered_random,
                       obdd_from_cnf, parse_text_circuit, random_3cnf, tautology, tiny_ddnnf)
from .weights import P_FLOOR, as_inputs, leaf_probs
from .configs import CONFIGS, make_config

__all__ = ["AND", "FALSE", "LIT", "OR", "TRUE", "Circuit", "CircuitBuilder", "layered_random",
           "obdd_from_cnf", "parse_text_circuit", "random_3cnf", "tautology", "tiny_ddnnf",
           "P_FLOOR", "as_inputs", "leaf_probs", "CONFIGS", "make_config"]
