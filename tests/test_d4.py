"""The d4 text reader: a hand-written decision-DNNF of (A and B) or C loads to a circuit with that
function's weighted model count and models.  No GPU needed."""
import itertools

import numpy as np
import pytest

from oracle import oracle
from paper_2410_11415_amd import Circuit
from paper_2410_11415_amd.d4 import load_d4, parse_d4
from tests.conftest import GOLDEN


def test_hand_written_d4():
    arr = load_d4(GOLDEN + "/a_and_b_or_c.d4")
    assert arr[0] == 3
    p = np.random.default_rng(0).uniform(0.05, 0.95, size=(5, 3))
    ref = p[:, 2] + (1 - p[:, 2]) * p[:, 0] * p[:, 1]
    np.testing.assert_allclose(oracle.forward(*arr, p, oracle.REAL)[:, 0], ref, rtol=1e-14)
    for a, b, c in itertools.product((0.0, 1.0), repeat=3):
        assert oracle.forward(*arr, np.array([[a, b, c]]), oracle.REAL)[0, 0] == float((a and b) or c)
    k = Circuit.from_d4(GOLDEN + "/a_and_b_or_c.d4", device=-1)
    assert k.info()["num_roots"] == 1 and k.info()["dag_nodes"] == 7       # 4 literals, AND(A, B), AND(-C, .), OR


def test_empty_nodes_shared_children_and_errors():
    # an OR without arcs is false, an AND without arcs is true; a child used twice is one node
    arr = parse_d4("o 1 0\no 2 0\na 3 0\no 4 0\n1 2 1 0\n1 3 -1 0\n1 4 2 0\n4 3 -2 0\n", num_vars=3)
    assert arr[0] == 3
    # = (x1 and false) or (-x1 and true) or (x2 and (-x2 and true)): value (1 - p1) + p2 (1 - p2)
    v = oracle.forward(*arr, np.array([[0.3, 0.6, 0.5]]), oracle.REAL)[0, 0]
    assert v == pytest.approx(0.7 + 0.6 * 0.4)
    for bad in ("o 2 0\n", "o 1 0\n1 2 0\n", "o 1 0\no 1 0\n", "x 1 0\n", "o 1 0\nt 2 0\n1 2 0 0\n", "o 1 0\nt 2 0\n1 2 3\n",
                "t 1 0\nt 2 0\n1 2 0\n", "o 1 0\no 2 0\n1 2 0\n2 1 0\n"):
        with pytest.raises(ValueError):
            parse_d4(bad)
    with pytest.raises(ValueError):
        parse_d4("o 1 0\nt 2 0\n1 2 5 0\n", num_vars=2)
