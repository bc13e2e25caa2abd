"""Full-size parity: the five workloads of the metric at their real sizes, launched exactly as
bench.py launches them (forward, then backward chained on the GPU's own O and LSE).

The oracle cannot run whole problems of this size, so it computes (a) the complete forward
(O, LSE) of a few sampled heads, (b) dQ for sampled query rows and dK, dV for sampled key rows
of those heads, each from its plain definition, and the GPU result is compared element by
element on those samples.  Two identities that hold at any size are checked on every head:
column sums of dV equal column sums of dO (rows of f sum to 1), and <dQ, Q> = <dK, K>.
"""
import numpy as np
import pytest

from oracle import attn_oracle as orc
from paper_2410_09397_amd import synth
from tests.helpers import LSE_TOL, TOL, rel_err, to_dev, to_np

pytestmark = pytest.mark.gpu


def sample_rows(w, rng, count=40):
    edges = [0, 1, w.n - 1, w.n - 2, 63, 64, 127, 128, w.n // 2 - 1, w.n // 2]
    rows = set(r for r in edges if 0 <= r < w.n)
    rows.update(rng.integers(0, w.n, size=count).tolist())
    return np.array(sorted(rows), dtype=np.int32)


@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_workload_at_full_size(index):
    check_at_full_size(synth.workload(index), index)


# Shapes beyond the five workloads, at sizes where every kernel runs many tiles per workgroup: the fused
# kernels at d = 256 (one wave per SIMD), the four-phase path at d = 1024, block masks with the causal rule on
# top, and one mask per (batch, head) pair.
MORE = [
    synth.Workload("full_d256_causal", 71, 1, 4, 4096, 256, "bf16", causal=True),
    synth.Workload("full_d1024", 72, 1, 2, 2048, 1024, "bf16"),
    synth.Workload("full_d128_sparse_causal", 73, 1, 4, 8192, 128, "bf16", sparse=True, causal=True, extra_frac=0.3),
    synth.Workload("full_d128_masks_per_head", 74, 2, 2, 4096, 128, "bf16", sparse=True, extra_frac=0.25,
                   per_head_masks=True),
]


@pytest.mark.parametrize("w", MORE, ids=lambda w: w.name)
def test_more_shapes_at_scale(w):
    check_at_full_size(w, w.index)


def check_at_full_size(w, index):
    import torch
    from paper_2410_09397_amd import attn
    print("workload", w, flush=True)
    inp = synth.make_inputs(w)
    Q, K, V, dO = (to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO"))
    mask = attn.BlockMask(inp["keep"], w.block, w.n) if w.sparse else None
    O, LSE = attn.attn_fwd(Q, K, V, w.scale, causal=w.causal, mask=mask)
    if mask is not None:
        dQ, dK, dV = attn.attn_bwd_blocksparse(Q, K, V, O, dO, LSE, w.scale, mask, causal=w.causal)
    else:
        dQ, dK, dV = attn.attn_bwd(Q, K, V, O, dO, LSE, w.scale, causal=w.causal)
    torch.cuda.synchronize()
    tol, ltol = TOL[w.dtype], LSE_TOL[w.dtype]

    # identities on every head (fp32 reductions on the device; bf16 outputs carry rounding noise)
    sum_dv, sum_do = dV.float().sum(2), dO.float().sum(2)
    assert (sum_dv - sum_do).abs().max().item() <= tol * max(1.0, sum_do.abs().max().item())
    qdq = (dQ.float() * Q.float()).sum((2, 3))
    kdk = (dK.float() * K.float()).sum((2, 3))
    scale_ref = (dQ.float().abs() * Q.float().abs()).sum((2, 3))
    assert ((qdq - kdk).abs() / scale_ref).max().item() <= tol

    rng = np.random.default_rng(1000 + index)
    bh = w.batch * w.heads
    heads = sorted({0, bh - 1, int(rng.integers(0, bh))})
    per_head = inp["keep"] is not None and np.asarray(inp["keep"]).ndim == 3
    for lin in heads:
        b, h = divmod(lin, w.heads)
        m = dict(causal=w.causal, keep=inp["keep"][lin] if per_head else inp["keep"], block=w.block)
        q, k, v, g = (inp[t][b, h] for t in ("Q", "K", "V", "dO"))
        rO, rL = orc.attn_fwd(q[None, None], k[None, None], v[None, None], w.scale, **m)
        assert rel_err(to_np(O[b, h]), rO[0, 0]) <= tol, ("O", lin)
        assert np.abs(to_np(LSE[b, h]) - rL[0, 0]).max() <= ltol * max(1.0, np.abs(rL).max()), ("LSE", lin)
        q_rows, k_rows = sample_rows(w, rng), sample_rows(w, rng)
        rdQ, rdK, rdV = orc.attn_bwd_sampled(q, k, v, rO[0, 0], g, rL[0, 0], w.scale, q_rows, k_rows, **m)
        assert rel_err(to_np(dQ[b, h])[q_rows], rdQ) <= tol, ("dQ", lin)
        assert rel_err(to_np(dK[b, h])[k_rows], rdK) <= tol, ("dK", lin)
        assert rel_err(to_np(dV[b, h])[k_rows], rdV) <= tol, ("dV", lin)
        print("head", lin, "ok", flush=True)
