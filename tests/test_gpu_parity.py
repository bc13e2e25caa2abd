"""GPU parity: the HIP path, called through the C ABI, against the float64 CPU oracle on the
same seeded inputs, element by element, at sizes the oracle finishes in seconds and that
span several tiles and ragged tails."""
import numpy as np
import pytest

from paper_2410_09397_amd import synth
from tests.helpers import LSE_TOL, TOL, check, oracle_reference, rel_err, to_dev, to_np

pytestmark = pytest.mark.gpu


def W(name, index, b, h, n, d, dtype, **kw):
    return synth.Workload(name, index, b, h, n, d, dtype, **kw)


CASES = [
    # the fp32 workload as specified, and ragged fp32 shapes (generic fp32-FMA kernels)
    synth.workload(1),
    W("f32_ragged", 11, 2, 2, 77, 40, "f32"),
    W("f32_ragged_causal", 12, 1, 3, 131, 24, "f32", causal=True),
    W("f32_blocks16", 13, 1, 2, 100, 32, "f32", sparse=True, block=16, extra_frac=0.3),
    W("f32_blocks16_causal", 14, 1, 2, 90, 16, "f32", sparse=True, causal=True, block=16, extra_frac=0.5),
    # bf16 MFMA kernels, d = 64
    W("bf16_d64", 21, 1, 2, 384, 64, "bf16"),
    W("bf16_d64_ragged_causal", 22, 2, 1, 333, 64, "bf16", causal=True),
    W("bf16_d64_tiny", 23, 1, 1, 5, 64, "bf16"),
    # bf16 MFMA kernels, d = 128
    W("bf16_d128_causal", 31, 1, 2, 512, 128, "bf16", causal=True, dO_std=0.1),
    W("bf16_d128_ragged", 32, 1, 3, 200, 128, "bf16"),
    W("bf16_d128_8heads", 33, 2, 4, 256, 128, "bf16", causal=True),
    # odd numbers of streamed tiles (the mask-free tiles run two at a time, one is left over)
    W("bf16_d128_5tiles", 34, 1, 2, 320, 128, "bf16"),
    W("bf16_d64_7tiles_causal", 35, 1, 2, 448, 64, "bf16", causal=True),
    W("bf16_d128_9tiles_ragged", 36, 1, 1, 570, 128, "bf16"),
    # block-sparse, 128 x 128 blocks
    W("bf16_d128_sparse", 41, 1, 2, 1024, 128, "bf16", sparse=True, extra_frac=0.3),
    W("bf16_d128_sparse_ragged", 42, 1, 1, 1000, 128, "bf16", sparse=True, extra_frac=0.15),
    W("bf16_d64_sparse_causal", 43, 1, 2, 768, 64, "bf16", sparse=True, causal=True, extra_frac=0.5),
    W("bf16_d128_sparse_causal_ragged", 44, 1, 2, 1100, 128, "bf16", sparse=True, causal=True, extra_frac=0.4),
    # one mask per (batch, head) pair: fused kernels and the generic ones
    W("bf16_d128_masks_per_head", 45, 2, 3, 900, 128, "bf16", sparse=True, extra_frac=0.3, per_head_masks=True),
    W("bf16_d64_masks_per_head_causal", 46, 1, 4, 640, 64, "bf16", sparse=True, causal=True, extra_frac=0.5,
      per_head_masks=True),
    W("f32_masks_per_head_blocks16", 47, 2, 2, 100, 32, "f32", sparse=True, block=16, extra_frac=0.3,
      per_head_masks=True),
    # d = 256 (fused kernels, one wave per SIMD) and the large head dimensions (small-cache regime)
    W("bf16_d512", 51, 1, 2, 384, 512, "bf16"),
    W("bf16_d512_ragged_causal", 52, 1, 1, 200, 512, "bf16", causal=True),
    W("bf16_d256", 53, 1, 2, 256, 256, "bf16"),
    W("bf16_d256_sparse_ragged", 60, 1, 2, 700, 256, "bf16", sparse=True, extra_frac=0.3),
    W("bf16_d256_sparse_causal", 61, 1, 1, 512, 256, "bf16", sparse=True, causal=True, extra_frac=0.5),
    W("bf16_d512_causal_5blocks", 54, 1, 2, 640, 512, "bf16", causal=True, dO_std=0.1),
    W("bf16_d256_ragged_causal", 55, 2, 1, 333, 256, "bf16", causal=True),
    # single rows and a few rows on every bf16 path
    W("bf16_d128_one_row", 62, 1, 2, 1, 128, "bf16", causal=True),
    W("bf16_d256_three_rows", 63, 2, 1, 3, 256, "bf16"),
    W("bf16_d512_one_row", 64, 1, 1, 1, 512, "bf16"),
    W("bf16_d1024_65_rows_causal", 65, 1, 1, 65, 1024, "bf16", causal=True),
    W("bf16_d1024", 58, 1, 1, 256, 1024, "bf16"),
    W("bf16_d1024_ragged_causal", 59, 1, 2, 150, 1024, "bf16", causal=True),
    # shapes only the generic fp32-FMA kernels take: bf16 with d outside {64,128,256,512},
    # d = 512 under a block mask, and a block edge other than 128
    W("bf16_d96_generic", 56, 1, 2, 150, 96, "bf16", causal=True),
    W("bf16_d512_sparse_generic", 57, 1, 1, 256, 512, "bf16", sparse=True, block=64, extra_frac=0.4),
]


def gpu_mask(w, inp):
    from paper_2410_09397_amd import attn
    return attn.BlockMask(inp["keep"], w.block, w.n) if inp["keep"] is not None else None


def gpu_bwd(w, mask, *args):
    from paper_2410_09397_amd import attn
    if mask is not None:
        return attn.attn_bwd_blocksparse(*args, w.scale, mask, causal=w.causal)
    return attn.attn_bwd(*args, w.scale, causal=w.causal)


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_forward_and_backward_match_oracle(w):
    from paper_2410_09397_amd import attn
    print("case", w, flush=True)
    inp = synth.make_inputs(w)
    ref = oracle_reference(w, inp)
    Q, K, V, dO = (to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO"))
    mask = gpu_mask(w, inp)
    tol, ltol = TOL[w.dtype], LSE_TOL[w.dtype]

    O, LSE = attn.attn_fwd(Q, K, V, w.scale, causal=w.causal, mask=mask)
    check(w.name, "O", to_np(O), ref["O"], w.dtype)
    assert np.abs(to_np(LSE) - ref["LSE"]).max() <= ltol * max(1.0, np.abs(ref["LSE"]).max())

    # backward in isolation: both sides consume the same rounded O and fp32 LSE
    O_in, LSE_in = to_dev(ref["O_in"], w.dtype), to_dev(ref["LSE_in"], "f32")
    grads = gpu_bwd(w, mask, Q, K, V, O_in, dO, LSE_in)
    for name, g, r in zip(("dQ", "dK", "dV"), grads, ref["iso"]):
        check(w.name + " isolated", name, to_np(g), r, w.dtype)

    # chained after the GPU forward, against the oracle's exact chain
    grads = gpu_bwd(w, mask, Q, K, V, O, dO, LSE)
    for name, g, r in zip(("dQ", "dK", "dV"), grads, ref["exact"]):
        check(w.name + " chained", name, to_np(g), r, w.dtype, chained=True)


def _run_all(w, inp, keep, causal):
    import torch
    from paper_2410_09397_amd import attn
    Q, K, V, dO = (to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO"))
    mask = attn.BlockMask(keep, w.block, w.n) if keep is not None else None
    O, LSE = attn.attn_fwd(Q, K, V, w.scale, causal=causal, mask=mask)
    if mask is not None:
        g = attn.attn_bwd_blocksparse(Q, K, V, O, dO, LSE, w.scale, mask, causal=causal)
    else:
        g = attn.attn_bwd(Q, K, V, O, dO, LSE, w.scale, causal=causal)
    torch.cuda.synchronize()
    return [t.cpu() for t in (O, LSE, *g)]


@pytest.mark.parametrize("d,dtype,block", [(128, "bf16", 128), (64, "bf16", 128), (256, "bf16", 128), (32, "f32", 64)])
def test_mask_logic_is_bit_exact(d, dtype, block):
    """An all-ones block mask must reproduce the dense result bit for bit, and a lower
    triangular block mask combined with the causal rule must reproduce causal bit for bit:
    the mask only selects which tiles are visited, it never changes their arithmetic."""
    import torch
    n = block * 4 - (block // 4)
    w = W("maskbits", 61, 1, 2, n, d, dtype)
    inp = synth.make_inputs(w)
    nblk = w.nblk
    dense = _run_all(w, inp, None, False)
    ones = _run_all(w, inp, np.ones((nblk, nblk), np.uint8), False)
    for a, b in zip(dense, ones):
        assert torch.equal(a, b)
    causal = _run_all(w, inp, None, True)
    tri = _run_all(w, inp, np.tril(np.ones((nblk, nblk), np.uint8)), True)
    for a, b in zip(causal, tri):
        assert torch.equal(a, b)


@pytest.mark.parametrize("scale", [-0.11, 0.0, 0.35])
@pytest.mark.parametrize("d,dtype", [(128, "bf16"), (64, "bf16"), (256, "bf16"), (512, "bf16"), (48, "f32")])
def test_unusual_scales(scale, d, dtype):
    """scale is any finite float: negative (the forward moves its sign into Q) and zero (uniform
    attention over the visible keys) must match the oracle like the usual 1/sqrt(d)."""
    from oracle import attn_oracle as orc
    from paper_2410_09397_amd import attn
    w = W("scale", 70, 1, 2, 200, d, dtype, causal=True)
    inp = synth.make_inputs(w)
    Q, K, V, dO = (to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO"))
    O, LSE = attn.attn_fwd(Q, K, V, scale, causal=True)
    dQ, dK, dV = attn.attn_bwd(Q, K, V, O, dO, LSE, scale, causal=True)
    rO, rL = orc.attn_fwd(inp["Q"], inp["K"], inp["V"], scale, causal=True)
    rg = orc.attn_bwd(inp["Q"], inp["K"], inp["V"], rO, inp["dO"], rL, scale, causal=True)
    tol = TOL[dtype]
    assert rel_err(to_np(O), rO) <= tol
    assert np.abs(to_np(LSE) - rL).max() <= LSE_TOL[dtype] * max(1.0, np.abs(rL).max())
    for name, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), rg):
        den = max(np.abs(r).max(), 1e-30)
        assert np.abs(to_np(g) - r).max() <= tol * den + (1e-6 if scale == 0.0 else 0.0), name


def test_backward_is_deterministic():
    """No atomics anywhere: two runs give bit-identical dQ, dK, dV."""
    import torch
    w = W("determinism", 62, 1, 4, 640, 128, "bf16", causal=True)
    inp = synth.make_inputs(w)
    a = _run_all(w, inp, None, True)
    b = _run_all(w, inp, None, True)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("d,dtype,n", [(64, "bf16", 300), (128, "bf16", 300), (256, "bf16", 200), (512, "bf16", 300),
                                       (96, "bf16", 150), (40, "f32", 150)])
def test_strided_layout_matches_contiguous(d, dtype, n):
    """[batch, n, heads, d] storage viewed as [batch, heads, n, d] gives the same bits, on every path:
    fused (d = 64, 128, 256), four-phase (512) and the generic fp32-FMA kernels (bf16 d = 96, fp32)."""
    import torch
    from paper_2410_09397_amd import attn
    w = W("strided", 63, 2, 3, n, d, dtype, causal=True)
    inp = synth.make_inputs(w)
    cont = [to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO")]
    perm = [t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in cont]
    assert perm[0].stride() != cont[0].stride()
    Oc, Lc = attn.attn_fwd(*cont[:3], w.scale, causal=True)
    Op = torch.empty_like(perm[0])
    Lp = torch.empty_like(Lc)
    attn.attn_fwd(*perm[:3], w.scale, causal=True, out=(Op, Lp))
    assert torch.equal(Oc, Op) and torch.equal(Lc, Lp)
    gc = attn.attn_bwd(*cont[:3], Oc, cont[3], Lc, w.scale, causal=True)
    outs = tuple(torch.empty_like(perm[0]) for _ in range(3))
    attn.attn_bwd(*perm[:3], Op, perm[3], Lp, w.scale, causal=True, out=outs)
    for a, b in zip(gc, outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("d,dtype", [(128, "bf16"), (512, "bf16"), (48, "f32")])
def test_call_on_a_non_default_stream(d, dtype):
    """Everything a call launches goes to the stream it is given: run on a side stream (default
    priority) while the current stream holds other work, the results equal those of the current stream."""
    import torch
    from paper_2410_09397_amd import attn
    w = W("stream", 66, 1, 2, 700, d, dtype, causal=True)
    inp = synth.make_inputs(w)
    Q, K, V, dO = (to_dev(inp[t], w.dtype) for t in ("Q", "K", "V", "dO"))
    O0, L0 = attn.attn_fwd(Q, K, V, w.scale, causal=True)
    g0 = attn.attn_bwd(Q, K, V, O0, dO, L0, w.scale, causal=True)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    filler = torch.randn(2048, 2048, device="cuda")
    for _ in range(4):
        filler = filler @ filler * 1e-3  # keeps the current stream busy meanwhile
    O1, L1 = torch.empty_like(O0), torch.empty_like(L0)
    g1 = tuple(torch.empty_like(Q) for _ in range(3))
    attn.attn_fwd(Q, K, V, w.scale, causal=True, stream=side, out=(O1, L1))
    attn.attn_bwd(Q, K, V, O1, dO, L1, w.scale, causal=True, stream=side, out=g1)
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(O0, O1) and torch.equal(L0, L1)
    for a, b in zip(g0, g1):
        assert torch.equal(a, b)


def test_empty_and_fully_masked_rows():
    """n = 0 is a valid no-op; a query-block row that keeps nothing gives O = 0, LSE = -inf
    and zero gradients, as in the oracle."""
    import torch
    from oracle import attn_oracle as orc
    from paper_2410_09397_amd import attn
    z = torch.empty(1, 2, 0, 64, dtype=torch.bfloat16, device="cuda")
    O, LSE = attn.attn_fwd(z, z, z, 1.0)
    assert O.numel() == 0 and LSE.numel() == 0
    attn.attn_bwd(z, z, z, O, z, LSE, 1.0)

    w = W("emptyrow", 64, 1, 1, 384, 64, "bf16", block=128)
    inp = synth.make_inputs(w)
    keep = np.array([[1, 1, 0], [0, 0, 0], [1, 0, 1]], np.uint8)
    O, LSE, dQ, dK, dV = _run_all(w, inp, keep, False)
    assert torch.all(O[0, 0, 128:256] == 0) and torch.all(torch.isneginf(LSE[0, 0, 128:256]))
    assert torch.all(dQ[0, 0, 128:256] == 0)
    rO, rL = orc.attn_fwd(inp["Q"], inp["K"], inp["V"], w.scale, keep=keep, block=128)
    rg = orc.attn_bwd(inp["Q"], inp["K"], inp["V"], rO, inp["dO"], rL, w.scale, keep=keep, block=128)
    assert rel_err(to_np(O), rO) <= TOL["bf16"]
    for g, r in zip((dQ, dK, dV), rg):
        assert rel_err(to_np(g), r) <= TOL["bf16"]

    # the same on the generic fp32 kernels (block edge 16): rows 16..31 keep nothing
    w = W("emptyrow_generic", 67, 1, 2, 48, 24, "f32", block=16)
    inp = synth.make_inputs(w)
    O, LSE, dQ, dK, dV = _run_all(w, inp, keep, False)
    assert torch.all(O[:, :, 16:32] == 0) and torch.all(torch.isneginf(LSE[:, :, 16:32]))
    assert torch.all(dQ[:, :, 16:32] == 0)
    rO, rL = orc.attn_fwd(inp["Q"], inp["K"], inp["V"], w.scale, keep=keep, block=16)
    rg = orc.attn_bwd(inp["Q"], inp["K"], inp["V"], rO, inp["dO"], rL, w.scale, keep=keep, block=16)
    assert rel_err(to_np(O), rO) <= TOL["f32"]
    for g, r in zip((dQ, dK, dV), rg):
        assert rel_err(to_np(g), r) <= TOL["f32"]
