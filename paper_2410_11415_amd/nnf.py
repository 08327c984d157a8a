"""Reader for circuits in the textual ``.nnf`` format written by d-DNNF compilers (c2d, Dsharp, d4's
legacy output): one node per line, children before parents, the last node is the root.

    nnf <nodes> <edges> <variables>
    L <literal>                     literal, +-(1-based variable)
    A <k> <c1> ... <ck>             AND of earlier lines (0-based); ``A 0`` is TRUE
    O <j> <k> <c1> ... <ck>         OR; j is the decision variable or 0; ``O 0 0`` is FALSE

This is input plumbing only: it produces the arrays ``klay_build`` takes (paper Section 2: an NNF
circuit as linked nodes).  Nothing is evaluated here.
"""
from __future__ import annotations

import numpy as np

LIT, AND, OR, TRUE, FALSE = 0, 1, 2, 3, 4


def parse_nnf(text: str):
    """Returns ``(num_vars, node_type, node_lit, child_ptr, child_idx, roots)`` for ``Circuit(*...)``."""
    lines = [ln.split() for ln in text.splitlines() if ln.strip() and not ln.lstrip().startswith("c")]
    if not lines or lines[0][0] != "nnf" or len(lines[0]) != 4:
        raise ValueError("not an nnf file: missing 'nnf <nodes> <edges> <vars>' header")
    n_nodes, n_edges, n_vars = (int(x) for x in lines[0][1:])
    body = lines[1:]
    if len(body) != n_nodes:
        raise ValueError("nnf header announces %d nodes, file has %d" % (n_nodes, len(body)))
    node_type = np.zeros(n_nodes, dtype=np.uint8)
    node_lit = np.zeros(n_nodes, dtype=np.int32)
    child_ptr = np.zeros(n_nodes + 1, dtype=np.int64)
    kids: list[int] = []
    for i, tok in enumerate(body):
        kind = tok[0]
        if kind == "L":
            lit = int(tok[1])
            if lit == 0 or abs(lit) > n_vars:
                raise ValueError("line %d: literal %d out of range" % (i + 2, lit))
            node_type[i], node_lit[i] = LIT, lit
        elif kind in ("A", "O"):
            args = [int(x) for x in tok[1:]]
            if kind == "O":
                args = args[1:]                      # drop the decision variable
            if not args or args[0] != len(args) - 1:
                raise ValueError("line %d: child count does not match" % (i + 2))
            ch = args[1:]
            if any(c < 0 or c >= i for c in ch):
                raise ValueError("line %d: child must be an earlier line" % (i + 2))
            if not ch:
                node_type[i] = TRUE if kind == "A" else FALSE
            else:
                node_type[i] = AND if kind == "A" else OR
                kids.extend(ch)
        else:
            raise ValueError("line %d: unknown node kind %r" % (i + 2, kind))
        child_ptr[i + 1] = len(kids)
    if len(kids) != n_edges:
        raise ValueError("nnf header announces %d edges, file has %d" % (n_edges, len(kids)))
    child_idx = np.asarray(kids, dtype=np.int32)
    roots = np.array([n_nodes - 1], dtype=np.int32)
    return n_vars, node_type, node_lit, child_ptr, child_idx, roots


def load_nnf(path: str):
    with open(path) as f:
        return parse_nnf(f.read())
