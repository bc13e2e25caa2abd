"""CPU-only checks of the boundary: the shared library loads, exports exactly what the header
declares, rejects bad arguments before any launch, and the host-side mask logic is right."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2410_09397_amd import attn, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names += re.findall(r"\b(attn_[a-z_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    L = attn.lib()
    decl = declared_functions()
    assert sorted(decl) == sorted(attn.EXPORTS)
    for name in decl:
        assert hasattr(L, name), name


def test_status_strings():
    assert attn.status_str(attn.ATTN_OK) == "ok"
    assert len({attn.status_str(s) for s in range(5)}) == 5


def desc(**kw):
    base = dict(batch=1, heads=1, n=128, d=64, scale=0.125, causal=0, dtype=attn.ATTN_BF16,
                stride_b=128 * 64, stride_h=128 * 64, stride_n=64)
    base.update(kw)
    return attn.attn_desc(**base)


P = 0x1000  # a non-null, 16-byte aligned fake device address: never dereferenced by a rejected call


def call_fwd(d, mask=None, ptrs=(P, P, P, P, P)):
    return attn.lib().attn_fwd(ctypes.byref(d) if d is not None else None, mask, *ptrs, P, 1 << 40, None)


def call_bwd(d, ptrs=(P,) * 9, ws=P, ws_bytes=1 << 30):
    return attn.lib().attn_bwd(ctypes.byref(d) if d is not None else None, *ptrs, ws, ws_bytes, None)


@pytest.mark.parametrize("kw,status", [
    (dict(n=-1), attn.ATTN_ERR_INVALID_ARG),
    (dict(d=0), attn.ATTN_ERR_INVALID_ARG),
    (dict(causal=2), attn.ATTN_ERR_INVALID_ARG),
    (dict(scale=float("nan")), attn.ATTN_ERR_INVALID_ARG),
    (dict(stride_n=32), attn.ATTN_ERR_INVALID_ARG),
    (dict(stride_n=68), attn.ATTN_ERR_INVALID_ARG),      # bf16 rows must stay 16-byte aligned
    (dict(dtype=7), attn.ATTN_ERR_UNSUPPORTED),
    (dict(d=2048, stride_n=2048), attn.ATTN_ERR_UNSUPPORTED),
    (dict(d=1024, stride_n=1024, dtype=attn.ATTN_F32), attn.ATTN_ERR_UNSUPPORTED),  # bf16 large-d path only
    (dict(d=768, stride_n=768), attn.ATTN_ERR_UNSUPPORTED),
    (dict(stride_n=1 << 22), attn.ATTN_ERR_UNSUPPORTED),   # row offsets inside a tile are 32-bit
    (dict(d=60, stride_n=64), attn.ATTN_ERR_UNSUPPORTED),  # bf16 needs d % 8 == 0
])
def test_bad_descriptors_are_rejected_before_launch(kw, status):
    d = desc(**kw)
    assert call_fwd(d) == status
    assert call_bwd(d) == status
    assert attn.lib().attn_workspace_bytes(ctypes.byref(d), None) == 0


def test_null_and_misaligned_pointers_and_workspace():
    d = desc()
    assert call_fwd(None) == attn.ATTN_ERR_INVALID_ARG
    assert call_fwd(d, ptrs=(P, None, P, P, P)) == attn.ATTN_ERR_INVALID_ARG
    assert call_fwd(d, ptrs=(P + 2, P, P, P, P)) == attn.ATTN_ERR_INVALID_ARG
    assert call_bwd(d, ptrs=(P,) * 8 + (None,)) == attn.ATTN_ERR_INVALID_ARG
    need = attn.lib().attn_workspace_bytes(ctypes.byref(d), None)
    assert need >= 128 * 4
    assert call_bwd(d, ws=None) == attn.ATTN_ERR_WORKSPACE
    assert call_bwd(d, ws_bytes=need - 1) == attn.ATTN_ERR_WORKSPACE
    # block-sparse entry point without a mask
    assert attn.lib().attn_bwd_blocksparse(ctypes.byref(d), None, *(P,) * 9, P, 1 << 30, None) == attn.ATTN_ERR_INVALID_ARG
    # mask whose block count does not match n
    m = attn.attn_blockmask(128, 3, P, P, P, P)
    assert call_fwd(d, mask=ctypes.byref(m)) == attn.ATTN_ERR_INVALID_ARG


def call_wgrad(d, ptrs=(P,) * 7, ws=P, ws_bytes=1 << 40):
    return attn.lib().attn_bwd_wgrad(ctypes.byref(d) if d is not None else None, *ptrs, ws, ws_bytes, None)


def test_wgrad_entry_point_validates_before_launch():
    L = attn.lib()
    d = desc()
    need = L.attn_wgrad_workspace_bytes(ctypes.byref(d))
    # Q, V, O, dQ in bf16, LSE and delta rows, one chunk of partial products
    assert need >= 4 * 128 * 64 * 2 + 2 * 128 * 4 + 64 * 64 * 4
    assert call_wgrad(None) == attn.ATTN_ERR_INVALID_ARG
    assert call_wgrad(d, ptrs=(P, P, P, None, P, P, P)) == attn.ATTN_ERR_INVALID_ARG
    assert call_wgrad(d, ptrs=(P, P, P, P, P, P + 4, P)) == attn.ATTN_ERR_INVALID_ARG
    assert call_wgrad(d, ws=None) == attn.ATTN_ERR_WORKSPACE
    assert call_wgrad(d, ws_bytes=need - 1) == attn.ATTN_ERR_WORKSPACE
    for kw in (dict(dtype=attn.ATTN_F32), dict(d=512, stride_n=512, stride_h=128 * 512, stride_b=128 * 512),
               dict(stride_n=128, stride_h=128 * 128, stride_b=128 * 128)):  # fp32, d > 256, padded rows
        bad = desc(**kw)
        assert call_wgrad(bad) == attn.ATTN_ERR_UNSUPPORTED
        assert L.attn_wgrad_workspace_bytes(ctypes.byref(bad)) == 0
    assert call_wgrad(desc(batch=0), ptrs=(None,) * 7, ws=None, ws_bytes=0) == attn.ATTN_OK
    assert call_wgrad(desc(n=0), ptrs=(None,) * 7, ws=None, ws_bytes=0) == attn.ATTN_ERR_INVALID_ARG  # g is written


def test_empty_problem_is_ok_without_touching_pointers():
    d = desc(n=0)
    assert call_fwd(d, ptrs=(None,) * 5) == attn.ATTN_OK
    assert call_bwd(d, ptrs=(None,) * 9, ws=None, ws_bytes=0) == attn.ATTN_OK


def test_blockmask_validate_and_csr_csc():
    keep = synth.block_mask(16, 3, 7, 5)
    assert keep.sum(1).tolist() == [4] * 16 and np.all(np.diag(keep) == 1)
    rp, ci, cp, ri = attn.csr_csc_from_dense(keep)
    # brute force: both orientations list exactly the kept pairs, ascending
    for i in range(16):
        assert ci[rp[i]:rp[i + 1]].tolist() == [j for j in range(16) if keep[i, j]]
        assert ri[cp[i]:cp[i + 1]].tolist() == [r for r in range(16) if keep[r, i]]
    v = attn.attn_blockmask_validate
    assert v(128, 16, 2048, rp, ci, cp, ri) == attn.ATTN_OK
    assert v(128, 16, 2000, rp, ci, cp, ri) == attn.ATTN_OK       # ragged last block
    assert v(128, 16, 2049, rp, ci, cp, ri) == attn.ATTN_ERR_INVALID_ARG
    bad = ci.copy(); bad[1], bad[0] = ci[0], ci[1]                # unsorted row
    assert v(128, 16, 2048, rp, bad, cp, ri) == attn.ATTN_ERR_INVALID_ARG
    bad = ci.copy(); bad[0] = 16                                  # out of range
    assert v(128, 16, 2048, rp, bad, cp, ri) == attn.ATTN_ERR_INVALID_ARG
    other = attn.csr_csc_from_dense(np.roll(keep, 1, axis=0))    # orientations disagree
    assert v(128, 16, 2048, rp, ci, other[2], other[3]) == attn.ATTN_ERR_INVALID_ARG
    bad = rp.copy(); bad[3] = bad[2] - 1                          # non-monotone pointer
    assert v(128, 16, 2048, bad, ci, cp, ri) == attn.ATTN_ERR_INVALID_ARG
    assert v(0, 16, 2048, rp, ci, cp, ri) == attn.ATTN_ERR_INVALID_ARG
    # a stack of masks, one per (batch, head) pair: pointer arrays continue from mask to mask
    stack = np.stack([keep, np.roll(keep, 3, axis=1) | np.eye(16, dtype=keep.dtype), np.eye(16, dtype=keep.dtype)])
    srp, sci, scp, sri = attn.csr_csc_from_dense(stack)
    assert len(srp) == 3 * 17 and srp[17] == srp[16] and srp[-1] == len(sci) == len(sri)
    assert v(128, 16, 2048, srp, sci, scp, sri, nmasks=3) == attn.ATTN_OK
    bad = srp.copy(); bad[17:34] += 1                             # second mask does not continue the first
    assert v(128, 16, 2048, bad, sci, scp, sri, nmasks=3) == attn.ATTN_ERR_INVALID_ARG
    swapped = attn.csr_csc_from_dense(stack[[0, 2, 1]])           # orientations of masks 1 and 2 disagree
    assert v(128, 16, 2048, srp, sci, swapped[2], swapped[3], nmasks=3) == attn.ATTN_ERR_INVALID_ARG
    # the number of masks must be 1 or batch * heads
    d = desc(n=2048, heads=2, stride_h=2048 * 64, stride_b=2 * 2048 * 64)
    m = attn.attn_blockmask(128, 16, P, P, P, P, 3)
    assert call_fwd(d, mask=ctypes.byref(m)) == attn.ATTN_ERR_INVALID_ARG


def test_synthetic_inputs_are_reproducible_and_rounded():
    import torch
    w = synth.workload(2).small(batch=1, heads=2, n=64)
    a, b = synth.make_inputs(w), synth.make_inputs(w)
    for t in ("Q", "K", "V", "dO"):
        assert np.array_equal(a[t], b[t])
        # storage rounding agrees with torch's round-to-nearest-even bf16 cast
        back = torch.from_numpy(a[t]).to(torch.bfloat16).float().numpy()
        assert np.array_equal(back, a[t])
    assert not np.array_equal(a["Q"], a["K"])
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32)
    assert np.array_equal(synth.round_to_bf16(x), torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    w3 = synth.workload(3).small(batch=1, heads=1, n=4096)
    assert abs(synth.make_inputs(w3)["dO"].std() - 0.1) < 5e-3
    w5 = synth.workload(5)
    assert w5.extra_blocks == 13 and abs(w5.kept_fraction() - 1792 / 16384) < 1e-12
    assert abs(w5.bwd_flops() - 6.013e11) / 6.013e11 < 1e-3
    assert abs(synth.workload(3).bwd_flops() - 2.749e12) / 2.749e12 < 1e-3


def test_mfma_ceiling_rejects_bad_arguments_before_launch():
    L = attn.lib()
    flops = ctypes.c_double(0.0)
    assert L.attn_mfma_ceiling(0, 0, P, ctypes.byref(flops), None) == attn.ATTN_ERR_INVALID_ARG
    assert L.attn_mfma_ceiling(5000000, 0, P, ctypes.byref(flops), None) == attn.ATTN_ERR_INVALID_ARG
    assert L.attn_mfma_ceiling(100, 0, None, ctypes.byref(flops), None) == attn.ATTN_ERR_INVALID_ARG
    assert L.attn_mfma_ceiling(100, 0, P, None, None) == attn.ATTN_ERR_INVALID_ARG
