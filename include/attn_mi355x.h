/*
 * attn_mi355x.h -- C ABI of libattn_mi355x.so: exact softmax attention, forward and backward,
 * for AMD MI355X (gfx950).
 *
 * What is computed (arXiv 2410.09397, "On Fine-Grained I/O Complexity of Attention Backward
 * Passes"; the paper's S = A_1 X, A_2, h = A_3 Y are the Q, K, V of this interface):
 *   forward  (Sec. 3.1, forward definition; App. B.4, definitions of A, l, f, O)
 *       s_ij = scale * <Q_i, K_j> over visible (i, j);  l_i = sum_j exp(s_ij);
 *       O_i = sum_j exp(s_ij) / l_i * V_j;              LSE_i = log l_i
 *   backward (App. B.4, definitions of q and p; Sec. 3.1, backward gradient; the tiling follows
 *             the large-cache phase-2 algorithm of App. D for d <= 256 and the four-phase
 *             small-cache algorithm of App. C for d > 256)
 *       f_ij = exp(s_ij - LSE_i);  v_i = <dO_i, O_i>;  q_ij = <dO_i, V_j>;  p_ij = f_ij (q_ij - v_i)
 *       dV_j = sum_i f_ij dO_i;  dK_j = scale sum_i p_ij Q_i;  dQ_i = scale sum_j p_ij K_j
 * The paper has no scale and no mask; scale multiplies Q K^T, and a pair (i, j) is visible iff
 * (!causal || j <= i) and, when a block mask is given, the mask keeps block (i/block, j/block).
 * A query with no visible key gets O = 0, LSE = -inf and contributes no gradient.
 *
 * Conventions
 *   - Every tensor pointer is DEVICE memory owned by the caller.  Q, K, V, O, dO, dQ, dK, dV are
 *     [batch, heads, n, d] with element strides (stride_b, stride_h, stride_n, 1), the same for
 *     all of them; LSE is contiguous [batch, heads, n] float.  Outputs are overwritten.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream);
 *     calls return without synchronising.  The library allocates no device memory and keeps no
 *     state between calls (attn_bwd_noalloc alone keeps the device address of its scratch array,
 *     per GPU, behind a mutex); scratch comes from the caller's workspace (attn_workspace_bytes).
 *     Entry points may be called from several host threads at once.
 *   - Arguments are validated on the host before anything is launched; a failed call launches
 *     nothing and leaves outputs untouched.  batch * heads * n == 0 is a valid empty call.
 *   - Supported: d a multiple of 8 for ATTN_BF16 (pointers and strides 16-byte aligned), any d
 *     for ATTN_F32, 1 <= d <= 512.  ATTN_BF16 runs bf16-MFMA kernels with fp32 accumulation for
 *     d in {64, 128, 256} (block masks: block == 128; fused, nothing n x n leaves the chip) and
 *     for d in {512, 1024} without block mask and n <= 32768 (four-phase path through the
 *     workspace; d = 1024 is supported there only); every other supported case, ATTN_F32 always,
 *     runs fp32 FMA kernels.
 */
#ifndef ATTN_MI355X_H
#define ATTN_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ATTN_OK = 0,
    ATTN_ERR_INVALID_ARG = 1, /* null pointer, negative size, misaligned stride, malformed mask */
    ATTN_ERR_UNSUPPORTED = 2, /* valid request outside the supported set (d, dtype) */
    ATTN_ERR_WORKSPACE = 3,   /* workspace missing or smaller than attn_workspace_bytes() */
    ATTN_ERR_DEVICE = 4       /* the HIP runtime reported an error at launch */
} attn_status;

typedef enum { ATTN_F32 = 0, ATTN_BF16 = 1 } attn_dtype;

/*
 * Tilings of the bf16 backward.  All compute the same gradients; they
 * differ in which block stays on chip, i.e. in the cache size M they need and in the traffic they
 * cause (the trade-off of Thm 1.1 / Sec. 4), and exist side by side so that it can be measured.
 *   ATTN_BWD_AUTO          the library's choice (the fastest measured for the shape)
 *   ATTN_BWD_TWO_KERNEL    a query-block owner forms dQ and a key-block owner forms dK, dV; both
 *                          recompute f and p (14 d multiply-adds per pair for 10 d counted); no
 *                          atomics, every output bit-reproducible; d in {64, 128, 256}
 *   ATTN_BWD_ONEPASS_K64   one key-block owner (64 keys) forms all five products once and adds its
 *   ATTN_BWD_ONEPASS_K128  dQ tiles with fp32 atomic adds into a zeroed array in the workspace,
 *                          which a last kernel scales and rounds to bf16 (K128: 128 keys per owner,
 *                          half the atomic volume); dK, dV bit-reproducible, dQ up to the order of
 *                          the additions; d in {64, 128}
 *   ATTN_BWD_PART_DQ       measurement aids: one kernel of ATTN_BWD_TWO_KERNEL alone, so that a caller
 *   ATTN_BWD_PART_DKDV     can time it with events of its own.  PART_DQ writes dQ (and v into the
 *                          workspace) and leaves dK, dV untouched; PART_DKDV writes dK, dV, leaves dQ
 *                          untouched and reads the v (and, under a block mask, nothing else) that an
 *                          earlier TWO_KERNEL or PART_DQ call left in the same workspace
 *   ATTN_BWD_FOUR_PHASE    the four-phase small-cache scheme of App. C (f and p through the workspace) at
 *                          a head dimension where the fused kernels are the default: d in {128, 256}
 *                          (it is what d in {512, 1024} run anyway); no block mask, n <= 32768
 *   ATTN_BWD_SPLIT_D       fused kernels whose owned block is 32 rows with the contraction over d split
 *                          over the waves of a workgroup: the fused alternative where the four-phase
 *                          scheme is the default, d = 512 (also d = 256); no block mask; bit-reproducible
 * A tiling that does not exist for the shape gives ATTN_ERR_UNSUPPORTED; the generic fp32 kernels
 * ignore the field, and so does the forward.
 */
typedef enum {
    ATTN_BWD_AUTO = 0,
    ATTN_BWD_TWO_KERNEL = 1,
    ATTN_BWD_ONEPASS_K64 = 2,
    ATTN_BWD_ONEPASS_K128 = 3,
    ATTN_BWD_PART_DQ = 4,
    ATTN_BWD_PART_DKDV = 5,
    ATTN_BWD_FOUR_PHASE = 6,
    ATTN_BWD_SPLIT_D = 7
} attn_bwd_tiling;

typedef struct {
    int32_t batch, heads, n, d;
    float scale;        /* multiplies Q K^T; callers usually pass 1/sqrt(d) */
    int32_t causal;     /* 0 or 1: key j visible to query i iff j <= i */
    int32_t dtype;      /* attn_dtype of Q, K, V, O, dO, dQ, dK, dV */
    int32_t bwd_tiling; /* attn_bwd_tiling; 0 unless a particular tiling is to be measured */
    int64_t stride_b, stride_h, stride_n; /* in elements; the d axis has stride 1; stride_n < 2^22 */
} attn_desc;

/*
 * Block mask: an nblk x nblk pattern of kept blocks, nblk = ceil(n / block), in both compressed
 * orientations (DEVICE int32 arrays, caller owned):
 *   row_ptr[nblk+1], col_idx[nnz]: key blocks kept for each query-block row, ascending;
 *   col_ptr[nblk+1], row_idx[nnz]: query blocks kept for each key-block column, ascending.
 * The two must describe the same set; attn_blockmask_validate checks host copies.
 * nmasks == 0 or 1: one pattern shared by all (batch, head) pairs.  nmasks == batch * heads: one
 * pattern per pair, mask m = b * heads + h; the arrays are the concatenations of the per-mask
 * arrays, row_ptr and col_ptr with nblk + 1 entries per mask that index the concatenated col_idx
 * and row_idx directly (entry 0 of mask m equals entry nblk of mask m - 1; mask 0 starts at 0).
 * (The paper's sparse bound, Thm 4.5, only counts non-zero entries: it covers both.)
 */
typedef struct {
    int32_t block;
    int32_t nblk;
    const int32_t *row_ptr, *col_idx;
    const int32_t *col_ptr, *row_idx;
    int32_t nmasks;
} attn_blockmask;

/* Bytes of device scratch that attn_fwd, attn_bwd and attn_bwd_blocksparse need for `desc`
 * (one figure that covers all three; 0 if desc or mask is invalid).  For d <= 256 it holds the
 * [batch, heads, n] row sums v (under a block mask also two lists of ceil(n / 128) block indices:
 * the order in which the workgroups take the blocks) and, for the one-pass tilings, the fp32
 * [batch, heads, n, d] array in which dQ is summed; for d > 256 (App. C path) the row sums and
 * the n x n matrices f and p of every (batch, head) in bf16, with n rounded up to 256. */
size_t attn_workspace_bytes(const attn_desc *desc, const attn_blockmask *mask /* nullable */);

/* Forward: writes O [batch, heads, n, d] and LSE [batch, heads, n].  `mask` may be NULL.
 * `workspace` is read only when d > 256 and may be NULL otherwise. */
attn_status attn_fwd(const attn_desc *desc, const attn_blockmask *mask, const void *Q,
                     const void *K, const void *V, void *O, float *LSE, void *workspace,
                     size_t workspace_bytes, void *stream);

/* Backward without block mask: dQ, dK, dV from Q, K, V, the forward's O and LSE, and dO. */
attn_status attn_bwd(const attn_desc *desc, const void *Q, const void *K, const void *V,
                     const void *O, const void *dO, const float *LSE, void *dQ, void *dK,
                     void *dV, void *workspace, size_t workspace_bytes, void *stream);

/*
 * attn_bwd for callers that cannot allocate or pass device scratch (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same result as
 * attn_bwd, with the scratch taken from a fixed array of ATTN_NOALLOC_SCRATCH_BYTES that the
 * library holds on every GPU it runs on until the process ends.  It calls no hipMalloc, hipFree or
 * other allocating routine.  A desc whose attn_workspace_bytes(desc, NULL) exceeds the array gives
 * ATTN_ERR_WORKSPACE and launches nothing (d <= 256 needs 4 bytes per (batch, head, query) for the
 * two-kernel tiling: 2 Mi rows fit).  Every call on one GPU uses that GPU's one array, which keeps
 * the previous call's contents (nothing in it has to start at zero: every kernel writes what it
 * later reads): calls that overlap in time on one GPU, on whatever streams, race.
 */
#define ATTN_NOALLOC_SCRATCH_BYTES (8u << 20)
attn_status attn_bwd_noalloc(const attn_desc *desc, const void *Q, const void *K, const void *V,
                             const void *O, const void *dO, const float *LSE, void *dQ, void *dK,
                             void *dV, void *stream);

/* Backward under a block mask (the sparse setting of Sec. 4.3; the paper gives bounds for it,
 * no algorithm).  `mask` must not be NULL.  Gradients of fully masked key rows are zero. */
attn_status attn_bwd_blocksparse(const attn_desc *desc, const attn_blockmask *mask,
                                 const void *Q, const void *K, const void *V, const void *O,
                                 const void *dO, const float *LSE, void *dQ, void *dK, void *dV,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Weight gradient of the paper's loss (Def. 3.2 and the backward gradient of Sec. 3.1; the
 * no-cache algorithm of App. C.1 states the same product step by step): with
 *     S = A_1 X (queries), A_2 (keys), h = A_3 Y (values), f, q, p as above,
 *     g = dL/dX = scale * A_1^T p A_2            one d x d matrix per (batch, head), float32.
 * A_1, A_2, A_3 and dO are [batch, heads, n, d] (here contiguous: stride_n == d, stride_h ==
 * n * d, stride_b == heads * n * d), X and Y are contiguous [batch, heads, d, d], row-major
 * (X[k][c]: input feature k, output feature c), g is contiguous [batch, heads, d, d].  dO is the
 * gradient of the loss with respect to the attention output (the paper's O - E).
 * The two projections, the forward, the dQ part of the backward and the product A_1^T dQ all run
 * on the device; queries, values, O and dQ pass through the workspace in bf16.
 * Supported: ATTN_BF16, d in {64, 128, 256}, no block mask; anything else -> ATTN_ERR_UNSUPPORTED.
 * attn_wgrad_workspace_bytes returns 0 for an invalid or unsupported desc.
 */
size_t attn_wgrad_workspace_bytes(const attn_desc *desc);
attn_status attn_bwd_wgrad(const attn_desc *desc, const void *A1, const void *A2, const void *A3,
                           const void *X, const void *Y, const void *dO, float *g,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Checks HOST copies of a block mask (nmasks patterns, 0 counts as 1): monotone pointers that
 * continue from one pattern to the next, strictly ascending in-range indices,
 * nblk == ceil(n / block), and that the two orientations of every pattern hold the same pairs. */
attn_status attn_blockmask_validate(int32_t block, int32_t nblk, int32_t n, int32_t nmasks,
                                    const int32_t *row_ptr, const int32_t *col_idx,
                                    const int32_t *col_ptr, const int32_t *row_idx);

/*
 * Measurement aid (no part of the attention path; the paper has no counterpart): launches a
 * register-only loop of independent dense bf16 MFMAs (32x32x16) on every CU, two waves per SIMD,
 * `iters` iterations of 8 MFMAs per wave.  `operands`: 0 = random bf16 operands held in registers,
 * 1 = all-zero operands, 2 = random operands with the B operand of every MFMA read from LDS as a fresh
 * 1 KB fragment requested one MFMA ahead (what the attention kernels do), 3 = as 2 plus four fp32
 * multiply-adds and one exponential per MFMA (about the vector arithmetic of the backward kernels),
 * 4 = the instruction stream of one wave of the dK / dV kernel per 64 x 64 tile at d = 128 with every
 * dependency taken out (per 32 MFMAs: 16 ds_read_b128 and 32 ds_read_b64_tr_b16 fragment reads, 16
 * exponentials, 64 multiply-adds, 16 bf16 packs, 8 LDS writes, 8 KB of global_load_lds tile copy out of
 * a 1 MB window, two workgroup barriers); `iters` still counts 8 MFMAs, a tile is four of them.
 * The rate it sustains is the ceiling of any kernel built on that instruction for operands of
 * that kind: under matrix load the shader clock follows the power the data's switching activity
 * draws.  Asynchronous on `stream`; the caller times it.
 *   clock_ghz  DEVICE float[1], caller owned: shader clock seen by one workgroup over the run
 *              (cycle counter against the 100 MHz constant-rate counter), valid after the stream
 *              has been synchronised
 *   flops      HOST double[1]: floating-point operations the launch executes
 * Errors: ATTN_ERR_INVALID_ARG (iters outside 1 .. 4 000 000, i.e. about a second of GPU time;
 * operands outside 0 .. 4; null pointers), ATTN_ERR_DEVICE.
 */
attn_status attn_mfma_ceiling(int32_t iters, int32_t operands, float *clock_ghz, double *flops,
                              void *stream);

/* Static description of a status code. */
const char *attn_status_str(attn_status s);

#ifdef __cplusplus
}
#endif
#endif /* ATTN_MI355X_H */
