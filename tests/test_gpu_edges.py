"""Sequence lengths around every tile edge of the kernels (1, 31 ... 257 rows), on each bf16 path and the fp32 one,
dense and causal: forward and isolated backward against the oracle; and properties of the gradients that hold at any
size, checked at the full size of the benchmark workloads where the oracle can only sample rows."""
import numpy as np
import pytest

from paper_2410_09397_amd import synth
from tests.helpers import LSE_TOL, check, oracle_reference, to_dev, to_np

pytestmark = pytest.mark.gpu

EDGE_LENGTHS = (1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 193, 255, 257)


@pytest.mark.parametrize("d,dtype", [(64, "bf16"), (128, "bf16"), (256, "bf16"), (512, "bf16"), (40, "f32")])
def test_lengths_around_tile_edges(d, dtype):
    from paper_2410_09397_amd import attn
    for k, n in enumerate(EDGE_LENGTHS):
        for causal in (False, True):
            w = synth.Workload("edge_d%d_n%d%s" % (d, n, "_causal" if causal else ""), 400 + k, 1, 2, n, d, dtype,
                               causal=causal)
            print("case", w.name, flush=True)
            inp = synth.make_inputs(w)
            ref = oracle_reference(w, inp)
            Q, K, V, dO = (to_dev(inp[t], dtype) for t in ("Q", "K", "V", "dO"))
            O, LSE = attn.attn_fwd(Q, K, V, w.scale, causal=causal)
            check(w.name, "O", to_np(O), ref["O"], dtype)
            assert np.abs(to_np(LSE) - ref["LSE"]).max() <= LSE_TOL[dtype] * max(1.0, np.abs(ref["LSE"]).max())
            O_in, LSE_in = to_dev(ref["O_in"], dtype), to_dev(ref["LSE_in"], "f32")
            grads = attn.attn_bwd(Q, K, V, O_in, dO, LSE_in, w.scale, causal=causal)
            for name, g, r in zip(("dQ", "dK", "dV"), grads, ref["iso"]):
                check(w.name + " isolated", name, to_np(g), r, dtype)


@pytest.mark.parametrize("index", [2, 3, 4, 5])
def test_gradient_invariants_at_full_size(index):
    """Rows of f sum to 1 and rows of p sum to 0 (App. B.4), whatever the mask, so for every (batch, head) pair
    the column sums of dV equal those of dO, and <dQ, Q> = <dK, K> (both are scale * sum_ij p_ij s_ij / scale).
    Every element of the three outputs enters these sums (the sampled-row comparison with the oracle in
    test_gpu_fullsize.py sees 40 rows per tensor); observed: 7e-5 .. 1.4e-4 and 4e-6 .. 3e-5."""
    import torch
    from paper_2410_09397_amd import attn
    w = synth.workload(index)
    print("case invariants", w.name, flush=True)
    inp = synth.make_inputs(w)
    Q, K, V, dO = (to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO"))
    mask = attn.BlockMask(inp["keep"], w.block, w.n) if w.sparse else None
    O, LSE = attn.attn_fwd(Q, K, V, w.scale, causal=w.causal, mask=mask)
    if mask is not None:
        dQ, dK, dV = attn.attn_bwd_blocksparse(Q, K, V, O, dO, LSE, w.scale, mask, causal=w.causal)
    else:
        dQ, dK, dV = attn.attn_bwd(Q, K, V, O, dO, LSE, w.scale, causal=w.causal)
    torch.cuda.synchronize()
    f64 = lambda t: t.double()
    # column sums: n terms of unit size each, bf16 outputs -> errors of order 2^-9 * sqrt(n) against sums of order sqrt(n)
    sv, sg = f64(dV).sum(dim=2), f64(dO).sum(dim=2)
    err = float((sv - sg).abs().max() / sg.abs().max())
    print("invariant %s: column sums of dV against dO, max-normalised %.3e" % (w.name, err), flush=True)
    assert err <= 1e-3
    a, b = (f64(dQ) * f64(Q)).sum(dim=(2, 3)), (f64(dK) * f64(K)).sum(dim=(2, 3))
    # the two inner products are sums of n d terms with both signs: compare against the sum of magnitudes
    size = (f64(dQ).abs() * f64(Q).abs()).sum(dim=(2, 3))
    err2 = float(((a - b).abs() / size).max())
    print("invariant %s: <dQ,Q> against <dK,K>, relative to sum |dQ||Q| %.3e" % (w.name, err2), flush=True)
    assert err2 <= 3e-4
