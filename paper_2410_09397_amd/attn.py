"""ctypes binding of libattn_mi355x.so: argument marshalling only.

Every function here has the name and meaning of the C entry point it wraps (see
include/attn_mi355x.h).  PyTorch supplies device memory and the current HIP stream; all
arithmetic runs in the library's kernels.  There is no CPU fallback: if the shared library
is missing, loading raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn_mi355x.so")

ATTN_OK, ATTN_ERR_INVALID_ARG, ATTN_ERR_UNSUPPORTED, ATTN_ERR_WORKSPACE, ATTN_ERR_DEVICE = range(5)
ATTN_F32, ATTN_BF16 = 0, 1
(ATTN_BWD_AUTO, ATTN_BWD_TWO_KERNEL, ATTN_BWD_ONEPASS_K64, ATTN_BWD_ONEPASS_K128, ATTN_BWD_PART_DQ,
 ATTN_BWD_PART_DKDV, ATTN_BWD_FOUR_PHASE, ATTN_BWD_SPLIT_D) = range(8)

EXPORTS = ("attn_workspace_bytes", "attn_fwd", "attn_bwd", "attn_bwd_noalloc", "attn_bwd_blocksparse",
           "attn_wgrad_workspace_bytes", "attn_bwd_wgrad", "attn_blockmask_validate", "attn_mfma_ceiling",
           "attn_status_str")


class attn_desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("n", ctypes.c_int32),
                ("d", ctypes.c_int32), ("scale", ctypes.c_float), ("causal", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("bwd_tiling", ctypes.c_int32), ("stride_b", ctypes.c_int64),
                ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64)]


class attn_blockmask(ctypes.Structure):
    _fields_ = [("block", ctypes.c_int32), ("nblk", ctypes.c_int32),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p),
                ("col_ptr", ctypes.c_void_p), ("row_idx", ctypes.c_void_p), ("nmasks", ctypes.c_int32)]


class AttnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s" % (where, status_str(status)))


_lib = None


def lib():
    """The loaded shared library (raises OSError if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("libattn_mi355x.so is not built: run `python -m paper_2410_09397_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, dp, mp = ctypes.c_void_p, ctypes.POINTER(attn_desc), ctypes.POINTER(attn_blockmask)
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.attn_workspace_bytes.restype = ctypes.c_size_t
        L.attn_workspace_bytes.argtypes = [dp, mp]
        L.attn_fwd.restype = ctypes.c_int
        L.attn_fwd.argtypes = [dp, mp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.attn_bwd.restype = ctypes.c_int
        L.attn_bwd.argtypes = [dp] + [vp] * 9 + [vp, ctypes.c_size_t, vp]
        L.attn_bwd_noalloc.restype = ctypes.c_int
        L.attn_bwd_noalloc.argtypes = [dp] + [vp] * 9 + [vp]
        L.attn_bwd_blocksparse.restype = ctypes.c_int
        L.attn_bwd_blocksparse.argtypes = [dp, mp] + [vp] * 9 + [vp, ctypes.c_size_t, vp]
        L.attn_wgrad_workspace_bytes.restype = ctypes.c_size_t
        L.attn_wgrad_workspace_bytes.argtypes = [dp]
        L.attn_bwd_wgrad.restype = ctypes.c_int
        L.attn_bwd_wgrad.argtypes = [dp] + [vp] * 7 + [vp, ctypes.c_size_t, vp]
        L.attn_blockmask_validate.restype = ctypes.c_int
        L.attn_blockmask_validate.argtypes = [ctypes.c_int32] * 4 + [i32p] * 4
        L.attn_mfma_ceiling.restype = ctypes.c_int
        L.attn_mfma_ceiling.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.attn_status_str.restype = ctypes.c_char_p
        L.attn_status_str.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_str(status):
    return lib().attn_status_str(int(status)).decode()


def csr_csc_from_dense(keep):
    """Host int32 arrays (row_ptr, col_idx, col_ptr, row_idx) of an [nblk, nblk] 0/1 matrix, or of a stack
    [nmasks, nblk, nblk] of them in the concatenated form of include/attn_mi355x.h (pointer arrays of
    nblk + 1 entries per mask that index the concatenated index arrays)."""
    keep = np.asarray(keep) != 0
    stack = keep[None] if keep.ndim == 2 else keep
    nblk = stack.shape[1]
    row_ptr, col_idx, col_ptr, row_idx = [], [], [], []
    start = 0
    for k in stack:
        rp = np.zeros(nblk + 1, np.int64)
        rp[1:] = np.cumsum(k.sum(1))
        cp = np.zeros(nblk + 1, np.int64)
        cp[1:] = np.cumsum(k.sum(0))
        row_ptr.append(rp + start)
        col_ptr.append(cp + start)
        col_idx.append(np.nonzero(k)[1])
        row_idx.append(np.nonzero(k.T)[1])
        start += int(rp[-1])
    cat = lambda parts: np.concatenate(parts).astype(np.int32)
    return cat(row_ptr), cat(col_idx), cat(col_ptr), cat(row_idx)


def attn_blockmask_validate(block, nblk, n, row_ptr, col_idx, col_ptr, row_idx, nmasks=1):
    """Status code of the host-side structural check of a block mask (numpy int32 arrays)."""
    i32p = ctypes.POINTER(ctypes.c_int32)
    arrs = [np.ascontiguousarray(a, dtype=np.int32) if a is not None else None
            for a in (row_ptr, col_idx, col_ptr, row_idx)]
    ptrs = [a.ctypes.data_as(i32p) if a is not None else None for a in arrs]
    return lib().attn_blockmask_validate(int(block), int(nblk), int(n), int(nmasks), *ptrs)


class BlockMask:
    """Device copies of a block mask in both compressed orientations.  `keep` is [nblk, nblk] (one
    pattern for all batches and heads) or [batch * heads, nblk, nblk] (one per pair)."""

    def __init__(self, keep, block, n, device="cuda"):
        import torch
        keep = np.asarray(keep)
        self.block, self.n = int(block), int(n)
        self.nblk = int(keep.shape[-1])
        self.nmasks = 1 if keep.ndim == 2 else int(keep.shape[0])
        self.host = csr_csc_from_dense(keep)
        st = attn_blockmask_validate(self.block, self.nblk, self.n, *self.host, nmasks=self.nmasks)
        if st != ATTN_OK:
            raise AttnError(st, "attn_blockmask_validate")
        self.dev = [torch.from_numpy(a).to(device) for a in self.host]
        self.c = attn_blockmask(self.block, self.nblk, *[t.data_ptr() for t in self.dev], self.nmasks)


def _desc(x, scale, causal, tiling=ATTN_BWD_AUTO):
    import torch
    if x.dim() != 4 or x.stride(3) != 1:
        raise ValueError("expected a [batch, heads, n, d] tensor with unit stride along d")
    dt = {torch.float32: ATTN_F32, torch.bfloat16: ATTN_BF16}[x.dtype]
    b, h, n, d = x.shape
    return attn_desc(b, h, n, d, float(scale), int(bool(causal)), dt, int(tiling), x.stride(0), x.stride(1),
                     x.stride(2))


def _same_layout(ref, *others):
    for t in others:
        if t.shape != ref.shape or t.stride() != ref.stride() or t.dtype != ref.dtype or t.device != ref.device:
            raise ValueError("all [batch, heads, n, d] tensors must share shape, strides, dtype and device")


def _stream(stream):
    import torch
    return (stream if stream is not None else torch.cuda.current_stream()).cuda_stream


def attn_workspace_bytes(desc, mask=None):
    return lib().attn_workspace_bytes(ctypes.byref(desc), ctypes.byref(mask.c) if mask is not None else None)


def _workspace(desc, mask, workspace, device, stream=None):
    """The caller's workspace, or a fresh one.  A fresh one is allocated on the stream the kernels will
    run on: torch's allocator may hand a freed block to later work of the allocating stream only, so the
    block cannot be reused while these kernels still read it."""
    import torch
    if workspace is None:
        nbytes = max(attn_workspace_bytes(desc, mask), 256)
        if stream is not None:
            with torch.cuda.stream(stream):
                workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        else:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return workspace


def attn_fwd(Q, K, V, scale, causal=False, mask=None, stream=None, out=None, workspace=None):
    """O, LSE = forward(Q, K, V) on the GPU.  Q, K, V: cuda tensors [batch, heads, n, d]."""
    import torch
    _same_layout(Q, K, V)
    desc = _desc(Q, scale, causal)
    workspace = _workspace(desc, mask, workspace, Q.device, stream)
    O = out[0] if out is not None else torch.empty_like(Q)
    LSE = out[1] if out is not None else torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    _same_layout(Q, O)
    st = lib().attn_fwd(ctypes.byref(desc), ctypes.byref(mask.c) if mask is not None else None,
                        Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(),
                        workspace.data_ptr(), workspace.numel(), _stream(stream))
    if st != ATTN_OK:
        raise AttnError(st, "attn_fwd")
    return O, LSE


def _bwd(name, Q, K, V, O, dO, LSE, scale, causal, mask, stream, out, workspace, tiling):
    import torch
    _same_layout(Q, K, V, O, dO)
    desc = _desc(Q, scale, causal, tiling)
    dQ, dK, dV = out if out is not None else (torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q))
    _same_layout(Q, dQ, dK, dV)
    if LSE.dtype != torch.float32 or not LSE.is_contiguous() or LSE.shape != Q.shape[:3]:
        raise ValueError("LSE must be a contiguous float32 [batch, heads, n] tensor")
    workspace = _workspace(desc, mask, workspace, Q.device, stream)
    args = [Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), LSE.data_ptr(),
            dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(stream)]
    if name == "attn_bwd":
        st = lib().attn_bwd(ctypes.byref(desc), *args)
    else:
        st = lib().attn_bwd_blocksparse(ctypes.byref(desc), ctypes.byref(mask.c), *args)
    if st != ATTN_OK:
        raise AttnError(st, name)
    return dQ, dK, dV


def attn_bwd(Q, K, V, O, dO, LSE, scale, causal=False, stream=None, out=None, workspace=None,
             tiling=ATTN_BWD_AUTO):
    """dQ, dK, dV from the forward's O and LSE (no block mask)."""
    return _bwd("attn_bwd", Q, K, V, O, dO, LSE, scale, causal, None, stream, out, workspace, tiling)


def attn_bwd_noalloc(Q, K, V, O, dO, LSE, scale, out, causal=False, stream=None, tiling=ATTN_BWD_AUTO):
    """attn_bwd with the library's fixed device scratch: the caller passes inputs and the outputs
    out = (dQ, dK, dV); nothing is allocated here or in the library."""
    import torch
    _same_layout(Q, K, V, O, dO, *out)
    desc = _desc(Q, scale, causal, tiling)
    if LSE.dtype != torch.float32 or not LSE.is_contiguous() or LSE.shape != Q.shape[:3]:
        raise ValueError("LSE must be a contiguous float32 [batch, heads, n] tensor")
    st = lib().attn_bwd_noalloc(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                dO.data_ptr(), LSE.data_ptr(), out[0].data_ptr(), out[1].data_ptr(),
                                out[2].data_ptr(), _stream(stream))
    if st != ATTN_OK:
        raise AttnError(st, "attn_bwd_noalloc")
    return out


def attn_bwd_blocksparse(Q, K, V, O, dO, LSE, scale, mask, causal=False, stream=None, out=None, workspace=None,
                         tiling=ATTN_BWD_AUTO):
    """dQ, dK, dV under a BlockMask."""
    return _bwd("attn_bwd_blocksparse", Q, K, V, O, dO, LSE, scale, causal, mask, stream, out, workspace, tiling)


def attn_wgrad_workspace_bytes(desc):
    return lib().attn_wgrad_workspace_bytes(ctypes.byref(desc))


def attn_bwd_wgrad(A1, A2, A3, X, Y, dO, scale=1.0, causal=False, stream=None, out=None, workspace=None):
    """g = dL/dX [batch, heads, d, d] (float32) of the paper's loss: queries A1 X, keys A2, values A3 Y."""
    import torch
    _same_layout(A1, A2, A3, dO)
    _same_layout(X, Y)
    desc = _desc(A1, scale, causal)
    b, h, n, d = A1.shape
    if tuple(X.shape) != (b, h, d, d) or not X.is_contiguous() or not Y.is_contiguous() or X.dtype != A1.dtype:
        raise ValueError("X and Y must be contiguous [batch, heads, d, d] tensors of the inputs' dtype")
    g = out if out is not None else torch.empty((b, h, d, d), dtype=torch.float32, device=A1.device)
    if workspace is None:
        nbytes = max(attn_wgrad_workspace_bytes(desc), 256)
        if stream is not None:  # see _workspace
            with torch.cuda.stream(stream):
                workspace = torch.empty(nbytes, dtype=torch.uint8, device=A1.device)
        else:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=A1.device)
    st = lib().attn_bwd_wgrad(ctypes.byref(desc), A1.data_ptr(), A2.data_ptr(), A3.data_ptr(), X.data_ptr(),
                              Y.data_ptr(), dO.data_ptr(), g.data_ptr(), workspace.data_ptr(), workspace.numel(),
                              _stream(stream))
    if st != ATTN_OK:
        raise AttnError(st, "attn_bwd_wgrad")
    return g


def attn_mfma_ceiling(iters, operands=0, stream=None):
    """Launches the register-only MFMA loop (include/attn_mi355x.h).  Returns (clock, flops): a
    device float tensor that holds the shader clock in GHz once the stream is synchronised, and
    the number of floating-point operations of the launch."""
    import torch
    clock = torch.zeros(1, dtype=torch.float32, device="cuda")
    flops = ctypes.c_double(0.0)
    st = lib().attn_mfma_ceiling(int(iters), int(operands), clock.data_ptr(), ctypes.byref(flops),
                                 _stream(stream))
    if st != ATTN_OK:
        raise AttnError(st, "attn_mfma_ceiling")
    return clock, flops.value
