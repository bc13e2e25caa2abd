"""GPU parity of attn_bwd_wgrad (the paper's own output, g = dL/dX = A_1^T p A_2) against the oracle.

Without mask and with scale 1 the reference is the oracle's step-by-step evaluation of the paper's
no-cache algorithm (App. C.1).  With a causal mask or another scale there is no such listing in the
paper; the reference is then the definition composed from pinned oracle pieces: queries A_1 X and
values A_3 Y as float64 products, the oracle forward and backward, and g = A_1^T dQ.
"""
import numpy as np
import pytest

from oracle import attn_oracle as orc
from paper_2410_09397_amd import synth
from tests import helpers

pytestmark = pytest.mark.gpu

# g sums n terms built from bf16-rounded queries, values, O and dQ: same gate as the other bf16 outputs
TOL = helpers.TOL["bf16"]


def _run_gpu(w, inp, scale, causal):
    import torch
    from paper_2410_09397_amd import attn
    dev = {k: helpers.to_dev(v, "bf16") for k, v in inp.items()}
    g = attn.attn_bwd_wgrad(dev["A1"], dev["A2"], dev["A3"], dev["X"], dev["Y"], dev["dO"], scale=scale, causal=causal)
    torch.cuda.synchronize()
    return g.cpu().numpy().astype(np.float64)


def _composed_reference(inp, b, h, scale, causal):
    A1, A2, A3, dO = (inp[k][b, h].astype(np.float64) for k in ("A1", "A2", "A3", "dO"))
    X, Y = inp["X"][b, h].astype(np.float64), inp["Y"][b, h].astype(np.float64)
    Q, V = (A1 @ X)[None, None], (A3 @ Y)[None, None]
    K, G = A2[None, None], dO[None, None]
    O, LSE = orc.attn_fwd(Q, K, V, scale, causal=causal)
    dQ, _, _ = orc.attn_bwd(Q, K, V, O, G, LSE, scale, causal=causal)
    return A1.T @ dQ[0, 0]


@pytest.mark.parametrize("n,d,heads", [(256, 64, 2), (320, 128, 2), (1100, 128, 1), (64, 64, 3), (300, 256, 2)])
def test_wgrad_matches_the_papers_algorithm(n, d, heads):
    w = synth.workload(2).small(batch=1, heads=heads, n=n, d=d)
    inp = synth.make_wgrad_inputs(w)
    g = _run_gpu(w, inp, 1.0, False)
    assert g.shape == (1, heads, d, d)
    for h in range(heads):
        ref, _, _, _ = orc.wgrad(inp["A1"][0, h], inp["A2"][0, h], inp["A3"][0, h], inp["dO"][0, h],
                                      inp["X"][0, h], inp["Y"][0, h])
        assert helpers.rel_err(g[0, h], ref) <= TOL


@pytest.mark.parametrize("n,d,scale,causal", [(384, 128, 1.0, True), (200, 64, 0.7, False), (2112, 128, 1.3, True), (1100, 256, 0.9, True)])
def test_wgrad_with_scale_and_causal_mask(n, d, scale, causal):
    w = synth.workload(3).small(batch=2, heads=2, n=n, d=d)
    inp = synth.make_wgrad_inputs(w)
    g = _run_gpu(w, inp, scale, causal)
    for b, h in ((0, 0), (1, 1)):
        assert helpers.rel_err(g[b, h], _composed_reference(inp, b, h, scale, causal)) <= TOL


def test_wgrad_is_deterministic():
    w = synth.workload(3).small(batch=1, heads=4, n=2048, d=128)
    inp = synth.make_wgrad_inputs(w)
    assert np.array_equal(_run_gpu(w, inp, 1.0, True), _run_gpu(w, inp, 1.0, True))


def test_wgrad_of_an_empty_sequence_is_zero():
    import torch
    from paper_2410_09397_amd import attn
    z = torch.empty((1, 2, 0, 64), dtype=torch.bfloat16, device="cuda")
    wts = torch.ones((1, 2, 64, 64), dtype=torch.bfloat16, device="cuda")
    g = torch.full((1, 2, 64, 64), 7.0, dtype=torch.float32, device="cuda")
    attn.attn_bwd_wgrad(z, z, z, wts, wts, z, out=g)
    torch.cuda.synchronize()
    assert torch.count_nonzero(g).item() == 0


def test_wgrad_at_the_bench_shape_one_head_against_the_oracle():
    """Workload 3's shape (b2 h32 n8192 d128, causal), as `bench.py --wgrad` launches it; one head is checked
    against the composed float64 reference (about 10 s of host work)."""
    w = synth.workload(3)
    inp = synth.make_wgrad_inputs(w)
    g = _run_gpu(w, inp, 1.0, True)
    assert np.isfinite(g).all()
    b, h = 1, 17
    assert helpers.rel_err(g[b, h], _composed_reference(inp, b, h, 1.0, True)) <= TOL
