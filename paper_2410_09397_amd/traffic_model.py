"""Host-side replay of tile schedules: how many bytes each schedule moves between memory and the
chip when nothing but the workgroup's own LDS and registers is a cache.

No attention arithmetic here, only loops over tiles that add up sizes.  Two groups:
  * the paper's two schedules, counted in elements as its lemmas do (App. C: four phases over
    B x B blocks; App. D, phase 2: row blocks of B_r outermost, column blocks of B_c inside, the
    d x d result resident), so that the counts can be set against Thm 4.1 / 4.3;
  * the schedules of this library's backward tilings, counted in bytes per (batch, head) pair,
    so that they can be set against the HBM bytes that rocprofv3 measures (the difference is what
    the 4 MB L2 of an XCD absorbs: tiles re-read by workgroups that run at the same time).
"""
import math


def _ceil(a, b):
    return -(-a // b)


# ------------------------------------------------------------------- the paper's schedules
def paper_small_cache(n, d, B):
    """(reads, writes) in elements of the four-phase scheme over B x B blocks (App. C), ragged
    edges included: every blocked product reads two blocks per k-step and writes its block once,
    the elementwise passes read and write n x n."""
    def blocks(m):
        return [min(B, m - a) for a in range(0, m, B)]

    def product(m, nn, k):  # C[m x nn] = A[m x k] B[k x nn]
        rd = sum(mi * kk + kk * nj for mi in blocks(m) for nj in blocks(nn) for kk in blocks(k))
        return rd, m * nn

    rd = wr = 0
    for shape in ((n, d, d), (n, n, d), (n, d, d), (n, n, d), (d, n, n), (d, d, n)):
        r, w_ = product(*shape)
        rd += r
        wr += w_
    rd += n * n + (n * n + n) + 4 * n * n  # exp / row sums; normalisation (reads l); phase 3 reads f, q twice
    wr += (n * n + n) + n * n + n * n      # A and l; f; p
    return rd, wr


def paper_large_cache_phase2(n, d, M):
    """(reads, writes) in elements of phase 2 of the large-cache algorithm (App. D) with the block
    sizes it prescribes, B_r = min(ceil(M / 4d), d) and B_c = ceil(M / 4d): per row block the rows of
    S, O, dO, A_1 and l; per (row block, column block) the rows of h and A_2; g (d x d) written once."""
    b_c = _ceil(M, 4 * d)
    b_r = min(b_c, d)
    rd = 0
    for i0 in range(0, n, b_r):
        bi = min(b_r, n - i0)
        rd += 4 * bi * d + bi
        for j0 in range(0, n, b_c):
            rd += 2 * min(b_c, n - j0) * d
    return rd, d * d


# ---------------------------------------------------------------- this library's schedules
def _visible_tiles(n, owner0, owner_rows, tile, causal, owner_is_key):
    """Start rows of the streamed tiles that a block of owner rows visits."""
    if not causal:
        return list(range(0, n, tile))
    if owner_is_key:   # queries from the tile that holds the first owned key on
        return list(range((owner0 // tile) * tile, n, tile))
    return list(range(0, min(n, owner0 + owner_rows), tile))  # keys up to the last owned query


def two_kernel(n, d, causal=False, es=2, key_block=64, query_block=128, tile=64):
    """Bytes per head of the two-kernel tiling: the query-block owner (dQ, and v on the way) and the
    key-block owner (dK, dV).  Returns a dict with 'read', 'written' and the share that is streamed
    (re-read once per owner block)."""
    rd = wr = streamed = 0
    for i0 in range(0, n, query_block):      # dQ kernel: resident Q, dO, O rows; streams K, V
        rows = min(query_block, n - i0)
        rd += 3 * rows * d * es + rows * 4   # Q, dO, O, LSE
        for j0 in _visible_tiles(n, i0, rows, tile, causal, False):
            t = 2 * min(tile, n - j0) * d * es
            rd += t
            streamed += t
        wr += rows * d * es + rows * 4       # dQ, v
    for j0 in range(0, n, key_block):        # dK/dV kernel: resident K, V rows; streams Q, dO, LSE, v
        rows = min(key_block, n - j0)
        rd += 2 * rows * d * es
        for i0 in _visible_tiles(n, j0, rows, tile, causal, True):
            r = min(tile, n - i0)
            t = 2 * r * d * es + 2 * r * 4
            rd += t
            streamed += t
        wr += 2 * rows * d * es
    return {"read": rd, "written": wr, "streamed": streamed}


def one_pass(n, d, causal=False, es=2, key_block=128, tile=64):
    """Bytes per head of the one-pass tiling: prep (v and the zeroed fp32 dQ array), the key-block
    owner that adds its dQ tiles with fp32 atomics (each addition is a write of 4 bytes per element to
    the memory side), and the final scaling pass."""
    rd = 2 * n * d * es                       # prep: O, dO
    wr = n * 4 + n * d * 4                    # v, zeroed dQ array
    streamed = atomics = 0
    for j0 in range(0, n, key_block):
        rows = min(key_block, n - j0)
        rd += 3 * rows * d * es               # K, V rows and the K^T fragments
        for i0 in _visible_tiles(n, j0, rows, tile, causal, True):
            r = min(tile, n - i0)
            t = 2 * r * d * es + 2 * r * 4
            rd += t
            streamed += t
            atomics += r * d * 4
        wr += 2 * rows * d * es
    rd += n * d * 4                           # scaling pass reads the fp32 array
    wr += n * d * es                          # and writes dQ
    return {"read": rd, "written": wr + atomics, "streamed": streamed, "atomics": atomics}


def split_d(n, d, causal=False, es=2, block=32):
    """Bytes per head of the fused split-d tiling: 32-row owners on both sides, 32-row streamed tiles."""
    out = two_kernel(n, d, causal, es, key_block=block, query_block=block, tile=block)
    out["read"] += n * d * es  # v comes from a row-sum kernel of its own, which reads dO once more (and O instead of the owner)
    return out


def four_phase(n, d, causal=False, es=2, score_q=128, score_k=256, prod_m=256, prod_n=128):
    """Bytes per head of the four-phase path: the row-sum kernel, the score kernel (tiles of 128 queries x
    256 keys, S and then dP with a k-loop over d each, f and p written as n x n bf16 matrices, n padded to 256)
    and the three products with a k-loop over n (tiles of 256 x 128 outputs)."""
    npad = _ceil(n, 256) * 256
    rd = 2 * n * d * es
    wr = n * 4
    tiles = 0
    for i0 in range(0, npad, score_q):
        for j0 in range(0, npad, score_k):
            if causal and j0 > i0 + score_q - 1:
                continue
            tiles += 1
    rd += tiles * (2 * (score_q + score_k) * d * es + 2 * score_q * 4)   # Q, dO, K, V chunks of the tile; LSE, v
    wr += tiles * 2 * score_q * score_k * es                             # f, p
    streamed = tiles * 2 * (score_q + score_k) * d * es
    for _ in range(3):                                             # dV = f^T dO, dK = p^T Q, dQ = p K
        out_tiles = _ceil(npad, prod_m) * _ceil(d, prod_n)
        k_len = npad * (0.5 if causal else 1.0)                    # the invisible half of f / p is skipped
        rd += out_tiles * (prod_m + prod_n) * k_len * es
        streamed += out_tiles * (prod_m + prod_n) * k_len * es
        wr += n * d * es
    return {"read": rd, "written": wr, "streamed": streamed}


def theorem_1_1_bytes(n, d, M_bytes, es=2, causal=False):
    """Both branches of Thm 1.1 in the Q / K / V form of Table 1 (constant 1), in bytes, for a cache of
    M_bytes: (large-cache branch n^2 d^2 / M, small-cache branch n^2 d / sqrt(M))."""
    M = M_bytes / es
    frac = 0.5 if causal else 1.0
    return es * n * n * d * d / M * frac, es * n * n * d / math.sqrt(M) * frac
