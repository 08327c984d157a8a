"""The .sdd text reader: a hand-written diagram of (A and B) or C loads to a circuit with that
function's weighted model count and models.  No GPU needed."""
import itertools

import numpy as np
import pytest

from oracle import oracle
from paper_2410_11415_amd import Circuit
from paper_2410_11415_amd.sdd import load_sdd, parse_sdd
from tests.conftest import GOLDEN


def test_hand_written_sdd():
    arr = load_sdd(GOLDEN + "/a_and_b_or_c.sdd")
    assert arr[0] == 3
    p = np.random.default_rng(0).uniform(0.05, 0.95, size=(5, 3))
    ref = p[:, 0] * p[:, 1] + (1 - p[:, 0] * p[:, 1]) * p[:, 2]
    np.testing.assert_allclose(oracle.forward(*arr, p, oracle.REAL)[:, 0], ref, rtol=1e-14)
    # every assignment: the circuit is the indicator of (A and B) or C
    for a, b, c in itertools.product((0.0, 1.0), repeat=3):
        v = oracle.forward(*arr, np.array([[a, b, c]]), oracle.REAL)[0, 0]
        assert v == float((a and b) or c)
    k = Circuit(*arr, device=-1)
    assert k.info()["num_roots"] == 1 and k.num_layers == 4       # OR(AND(A,B), AND(OR(AND(A,-B), -A), C))
    k2 = Circuit.from_sdd(GOLDEN + "/a_and_b_or_c.sdd", device=-1)
    assert k2.layer_sizes()[0].tolist() == k.layer_sizes()[0].tolist()


def test_order_of_lines_constants_and_errors():
    # parents before children, a true root element, more variables than mentioned
    arr = parse_sdd("sdd 4\nD 3 1 2 0 2 1 2\nL 0 0 1\nL 1 0 -1\nT 2\n", num_vars=4)
    assert arr[0] == 4
    assert oracle.forward(*arr, np.array([[0.3, 0.5, 0.5, 0.5]]), oracle.REAL)[0, 0] == pytest.approx(1.0)
    assert parse_sdd("sdd 1\nF 0\n")[1].tolist() == [4]
    for bad in ("sdd 2\nL 0 0 1\n", "L 0 0 1\n", "sdd 1\nL 0 0 0\n", "sdd 1\nD 0 1 1 0 5\n", "sdd 2\nL 0 0 1\nL 1 0 2\n",
                "sdd 2\nL 0 0 1\nL 0 0 2\n", "sdd 1\nX 0\n", "sdd 2\nD 0 1 1 1 1\nD 1 1 1 0 0\n"):
        with pytest.raises(ValueError):
            parse_sdd(bad)
    with pytest.raises(ValueError):
        parse_sdd("sdd 1\nL 0 0 3\n", num_vars=2)
