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
from tests.helpers import LSE_TOL, TOL, check, round_storage, to_dev, to_np

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
    # the longest sequence the tests run: 512 streamed tiles per workgroup
    synth.Workload("full_d128_n32768_causal", 75, 1, 1, 32768, 128, "bf16", causal=True),
    # more than 256 blocks per mask: the block-order lists come from the two-step kernels, not the fused one
    synth.Workload("full_d64_n33000_sparse", 76, 1, 1, 33000, 64, "bf16", sparse=True, extra_frac=0.02),
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
        check("%s head %d" % (w.name, lin), "O", to_np(O[b, h]), rO[0, 0], w.dtype)
        assert np.abs(to_np(LSE[b, h]) - rL[0, 0]).max() <= ltol * max(1.0, np.abs(rL).max()), ("LSE", lin)
        q_rows, k_rows = sample_rows(w, rng), sample_rows(w, rng)
        rdQ, rdK, rdV = orc.attn_bwd_sampled(q, k, v, rO[0, 0], g, rL[0, 0], w.scale, q_rows, k_rows, **m)
        check("%s head %d" % (w.name, lin), "dQ", to_np(dQ[b, h])[q_rows], rdQ, w.dtype, chained=True)
        check("%s head %d" % (w.name, lin), "dK", to_np(dK[b, h])[k_rows], rdK, w.dtype, chained=True)
        check("%s head %d" % (w.name, lin), "dV", to_np(dV[b, h])[k_rows], rdV, w.dtype, chained=True)
        print("head", lin, "ok", flush=True)


def test_isolated_backward_at_full_size_workload_3():
    """The backward alone at the size the metric is quoted on: O and LSE come from the oracle (O rounded
    to bf16, LSE to fp32), for every head, and both sides consume those same arrays; sampled rows of three
    heads are compared element by element."""
    import torch
    from paper_2410_09397_amd import attn
    w = synth.workload(3)
    print("workload", w, "isolated backward", flush=True)
    inp = synth.make_inputs(w)
    rO, rL = orc.attn_fwd(inp["Q"], inp["K"], inp["V"], w.scale, causal=True)
    O_in = round_storage(rO, w.dtype)
    L_in = rL.astype(np.float32)
    print("oracle forward done", flush=True)
    Q, K, V, dO = (to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO"))
    dQ, dK, dV = attn.attn_bwd(Q, K, V, to_dev(O_in, w.dtype), dO, to_dev(L_in, "f32"), w.scale, causal=True)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3003)
    bh = w.batch * w.heads
    for lin in sorted({0, bh - 1, int(rng.integers(0, bh))}):
        b, h = divmod(lin, w.heads)
        q_rows, k_rows = sample_rows(w, rng), sample_rows(w, rng)
        rdQ, rdK, rdV = orc.attn_bwd_sampled(inp["Q"][b, h], inp["K"][b, h], inp["V"][b, h], O_in[b, h], inp["dO"][b, h],
                                             L_in[b, h], w.scale, q_rows, k_rows, causal=True)
        check("cfg3 isolated head %d" % lin, "dQ", to_np(dQ[b, h])[q_rows], rdQ, w.dtype)
        check("cfg3 isolated head %d" % lin, "dK", to_np(dK[b, h])[k_rows], rdK, w.dtype)
        check("cfg3 isolated head %d" % lin, "dV", to_np(dV[b, h])[k_rows], rdV, w.dtype)
