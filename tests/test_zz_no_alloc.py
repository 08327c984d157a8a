"""klay_forward_static, the entry point that allocates nothing (its workspace is a fixed array in
device memory), against klay_forward: same kernels, so the outputs must be bit-identical; both are
also held to the oracle's tolerance.  Two calls in a row, the second on a smaller input, show that
nothing a call leaves behind in the shared array leaks into the next."""
import numpy as np
import pytest

from klay_synth import as_inputs, make_config
from tests.gpu_util import assert_log_close, assert_real_close, oracle_eval

pytestmark = pytest.mark.gpu

REAL, LOG, MAXLOG = 0, 1, 2


@pytest.fixture(scope="module")
def klay():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2410_11415_amd as pkg
    pkg.load()
    return pkg


def _both(klay, k, w32, semiring):
    import torch
    w = torch.from_numpy(np.ascontiguousarray(w32)).cuda()
    B = w.shape[0]
    out_s = torch.full((B, k.num_roots), float("nan"), dtype=torch.float32, device="cuda")
    out_d = torch.full((B, k.num_roots), float("nan"), dtype=torch.float32, device="cuda")
    klay.klay_forward_static(k._h, w.data_ptr(), B, out_s.data_ptr(), semiring, torch.cuda.current_stream().cuda_stream)
    klay.klay_forward(k._h, w.data_ptr(), B, out_d.data_ptr(), semiring, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return out_s.cpu().numpy(), out_d.cpu().numpy()


def test_static_forward_matches_forward_twice_in_a_row_second_call_smaller(klay):
    big, p_big, _ = make_config("layered_100k", seed=4, scale=0.4, batch=96)       # split rows, tail kernel, 4-byte tiles
    small, p_small, _ = make_config("layered_100k", seed=5, scale=0.05, batch=7)   # lane groups, far fewer rows
    kb = klay.Circuit(*big.arrays(), device=0)
    ks = klay.Circuit(*small.arrays(), device=0)
    assert kb.workspace_bytes(96, False) <= klay.binding.KLAY_STATIC_WORKSPACE_BYTES
    for k, c, p in ((kb, big, p_big), (ks, small, p_small), (kb, big, p_big[:33])):
        for s in (LOG, REAL, MAXLOG):
            w32 = as_inputs(p, s != REAL)
            got_s, got_d = _both(klay, k, w32, s)
            np.testing.assert_array_equal(got_s, got_d)
            ref, _ = oracle_eval(c, w32, s)
            (assert_real_close if s == REAL else assert_log_close)(got_s, ref, "static forward")
    kb.close(); ks.close()


def test_static_forward_leaves_the_handles_own_forward_state_alone(klay):
    """a klay_forward that is still to be differentiated survives a static call on the same handle;
    a static call alone gives klay_backward nothing to differentiate"""
    import torch
    c, p, _ = make_config("layered_100k", seed=6, scale=0.1, batch=40)
    w32 = as_inputs(p, True)
    k = klay.Circuit(*c.arrays(), device=0)
    w = torch.from_numpy(w32).cuda()
    dout = torch.ones((40, k.num_roots), device="cuda")
    with pytest.raises(klay.KlayError) as e:
        k.forward_static(w, LOG)
        klay.klay_backward(k._h, dout.data_ptr(), torch.empty((40, k.num_vars), device="cuda").data_ptr(), 0)
    assert e.value.status == 5
    out = k.forward(w, LOG)
    g0 = k.backward(dout).clone()
    k.forward(w, LOG)
    other = k.forward_static((w * 2).contiguous(), LOG)
    g1 = k.backward(dout)
    torch.cuda.synchronize()
    assert torch.equal(g0, g1) and not torch.equal(other, out)
    k.close()


def test_static_forward_refuses_what_does_not_fit(klay):
    import torch
    c, p, _ = make_config("layered_100k", seed=0, scale=1.0, batch=8)
    k = klay.Circuit(*c.arrays(), device=0)
    B = 512
    assert k.workspace_bytes(B, False) > klay.binding.KLAY_STATIC_WORKSPACE_BYTES
    w = torch.zeros((B, k.num_vars), device="cuda")
    with pytest.raises(klay.KlayError) as e:
        k.forward_static(w, LOG)
    assert e.value.status == 3 and "fixed buffer" in str(e.value)
    # the handle still works, also statically at a size that fits
    w32 = as_inputs(p, True)
    got_s, got_d = _both(klay, k, w32, LOG)
    np.testing.assert_array_equal(got_s, got_d)
    k.close()
