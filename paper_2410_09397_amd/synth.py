"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no attention arithmetic: it draws numbers, rounds them to the storage
dtype and draws block masks.  Both the GPU path and the CPU oracle are fed from here.

The generator is counter based (numpy's Philox keyed by seed, workload index and tensor
index), so a tensor's values do not depend on the order in which tensors are drawn.
"""
from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 241009397
TENSOR_IDS = {"Q": 0, "K": 1, "V": 2, "dO": 3, "mask": 4, "A1": 5, "A2": 6, "A3": 7, "X": 8, "Y": 9}


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    batch: int
    heads: int
    n: int
    d: int
    dtype: str            # "f32" or "bf16": storage type of Q, K, V, O, dO and the gradients
    causal: bool = False
    sparse: bool = False  # block-sparse mask: diagonal block + `extra_blocks` others per row
    block: int = 128
    extra_frac: float = 0.10
    dO_std: float = 1.0
    per_head_masks: bool = False  # block-sparse: a different mask for every (batch, head) pair

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.d))

    @property
    def nblk(self):
        return (self.n + self.block - 1) // self.block

    @property
    def extra_blocks(self):
        """Non-diagonal key blocks kept per query-block row (fixed count, not Bernoulli)."""
        return int(round(self.extra_frac * (self.nblk - 1))) if self.sparse else 0

    def kept_fraction(self):
        """Fraction of the n x n score matrix counted as visible when quoting FLOPs
        (causal is counted as one half; the exact share is (n + 1) / 2n)."""
        if self.sparse:
            # with the causal rule on top: half of the diagonal block and, in expectation, half of the others
            return (1 + self.extra_blocks) / self.nblk * (0.5 if self.causal else 1.0)
        if self.causal:
            return 0.5
        return 1.0

    def bwd_flops(self):
        """Algorithmic backward FLOPs: five n x n x d contractions over visible pairs."""
        return 10.0 * self.batch * self.heads * self.n * self.n * self.d * self.kept_fraction()

    def fwd_flops(self):
        return 4.0 * self.batch * self.heads * self.n * self.n * self.d * self.kept_fraction()

    def small(self, **kw):
        """A reduced copy (same structure, smaller sizes) for oracle-speed parity cases."""
        return replace(self, **kw)


# The five workloads the metric is defined on.
WORKLOADS = [
    Workload("cfg1_f32_n256_d64", 1, 1, 1, 256, 64, "f32"),
    Workload("cfg2_bf16_n2048_d64", 2, 4, 16, 2048, 64, "bf16"),
    Workload("cfg3_bf16_n8192_d128_causal", 3, 2, 32, 8192, 128, "bf16", causal=True, dO_std=0.1),
    Workload("cfg4_bf16_n4096_d512_larged", 4, 1, 8, 4096, 512, "bf16"),
    Workload("cfg5_bf16_n16384_d128_blocksparse", 5, 1, 16, 16384, 128, "bf16", sparse=True),
]


def workload(index):
    return WORKLOADS[index - 1]


def reshaped(w, shape):
    """Workload `w` with sizes replaced from a "batch,heads,n,d[,causal]" string (for sweeps over n or d that keep
    the value distributions and the mask kind of `w`); the name says what was changed."""
    parts = [int(x) for x in shape.split(",")]
    if len(parts) not in (4, 5):
        raise ValueError("shape must be batch,heads,n,d[,causal]")
    b, h, n, d = parts[:4]
    causal = bool(parts[4]) if len(parts) == 5 else w.causal
    return replace(w, name="%s_as_b%d_h%d_n%d_d%d%s" % (w.name.split("_")[0], b, h, n, d, "_causal" if causal else ""),
                   batch=b, heads=h, n=n, d=d, causal=causal)


def with_density(w, extra_frac):
    """Block-sparse workload `w` with another share of non-diagonal key blocks kept per query-block row."""
    if not w.sparse:
        raise ValueError("density applies to the block-sparse workload")
    return replace(w, name="%s_extra%g" % (w.name, extra_frac), extra_frac=float(extra_frac))


def _rng(seed, workload_index, tensor_id):
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 8) ^ int(workload_index), int(tensor_id)]))


def round_to_bf16(x):
    """float32 -> nearest bfloat16 (ties to even), returned widened back to float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = (u + (((u >> 16) & 1) + 0x7FFF)) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def normal(shape, std, seed, workload_index, tensor, dtype):
    """iid N(0, std^2) as float32, already rounded to the storage dtype."""
    x = _rng(seed, workload_index, TENSOR_IDS[tensor]).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x = x * np.float32(std)
    return round_to_bf16(x) if dtype == "bf16" else x


def block_mask(nblk, extra, seed, workload_index, pair=0):
    """[nblk, nblk] uint8: the diagonal block plus `extra` distinct other key blocks per
    query-block row, drawn without replacement, uniformly, from the seeded stream (one stream
    per (batch, head) pair when every pair has its own mask)."""
    rng = _rng(seed, workload_index, TENSOR_IDS["mask"] + 16 * int(pair))
    keep = np.zeros((nblk, nblk), dtype=np.uint8)
    for i in range(nblk):
        keep[i, i] = 1
        others = np.delete(np.arange(nblk), i)
        if extra > 0:
            keep[i, rng.choice(others, size=min(extra, nblk - 1), replace=False)] = 1
    return keep


def make_inputs(w, seed=BASE_SEED):
    """Q, K, V, dO as float32 numpy arrays [batch, heads, n, d] holding storage-dtype values,
    plus `keep` (None unless the workload is block sparse)."""
    shape = (w.batch, w.heads, w.n, w.d)
    out = {t: normal(shape, w.dO_std if t == "dO" else 1.0, seed, w.index, t, w.dtype)
           for t in ("Q", "K", "V", "dO")}
    if w.sparse and w.per_head_masks:
        out["keep"] = np.stack([block_mask(w.nblk, w.extra_blocks, seed, w.index, pair=m)
                                for m in range(w.batch * w.heads)])
    else:
        out["keep"] = block_mask(w.nblk, w.extra_blocks, seed, w.index) if w.sparse else None
    return out


def make_wgrad_inputs(w, seed=BASE_SEED):
    """Inputs of the weight-gradient entry point: A1, A2, A3, dO [batch, heads, n, d] ~ N(0, 1)
    (dO with the workload's std), X [batch, heads, d, d] ~ N(0, 1 / d^2) so that the scores
    <A1 X, A2> have unit variance without a 1/sqrt(d) factor, and Y ~ N(0, 1 / d) so that the values
    A3 Y do.  float32 arrays holding storage-dtype values."""
    shape, wshape = (w.batch, w.heads, w.n, w.d), (w.batch, w.heads, w.d, w.d)
    out = {t: normal(shape, 1.0, seed, w.index, t, w.dtype) for t in ("A1", "A2", "A3")}
    out["dO"] = normal(shape, w.dO_std, seed, w.index, "dO", w.dtype)
    out["X"] = normal(wshape, 1.0 / w.d, seed, w.index, "X", w.dtype)
    out["Y"] = normal(wshape, w.d ** -0.5, seed, w.index, "Y", w.dtype)
    return out
