"""The .nnf text reader: the hand-written file of the paper's running example (Section 2, Figure 1b)
loads to a circuit with the figure's value, model count and layer structure.  No GPU needed."""
import numpy as np
import pytest

from oracle import oracle
from paper_2410_11415_amd import Circuit
from paper_2410_11415_amd.nnf import load_nnf, parse_nnf
from tests.conftest import GOLDEN


def test_fig1b_nnf_file(golden):
    arr = load_nnf(GOLDEN + "/fig1b_ddnnf.nnf")
    ref = golden("fig1b_ddnnf.txt")
    assert arr[0] == 4 and arr[1].shape[0] == 15 and arr[4].shape[0] == 16
    p = np.random.default_rng(0).uniform(0.05, 0.95, size=(6, 4))
    np.testing.assert_allclose(oracle.forward(*arr, p, oracle.REAL), oracle.forward(*ref.arrays(), p, oracle.REAL),
                               rtol=1e-14)
    assert oracle.forward(*arr, np.full((1, 4), 0.5), oracle.REAL)[0, 0] == pytest.approx(13 / 16)
    k = Circuit(*arr, device=-1)
    nodes, edges = k.layer_sizes()
    assert nodes.tolist() == [8, 7, 6, 3, 1] and edges[1:].tolist() == [9, 8, 6, 3]


def test_constants_and_errors():
    arr = parse_nnf("nnf 4 2 1\nA 0\nO 0 0\nL -1\nO 1 2 0 2\n")
    assert arr[1].tolist() == [3, 4, 0, 2] and arr[4].tolist() == [0, 2]
    assert oracle.forward(*arr, np.array([[0.3]]), oracle.REAL)[0, 0] == pytest.approx(1.7)
    for bad in ("nnf 1 0 1\nX 1\n", "nnf 2 1 1\nL 1\nA 1 1\n", "nnf 1 0 1\nL 2\n", "nnf 2 0 1\nL 1\n", "L 1\n",
                "nnf 2 2 1\nL 1\nA 1 0\n", "nnf 2 1 1\nL 1\nA 2 0\n"):
        with pytest.raises(ValueError):
            parse_nnf(bad)
