// Large-d path (d in {512, 1024}; the kernels also take 256): the regime where a d x d working set no longer fits the
// per-CU LDS and register budget (the paper's small-cache case, M = o(d^2)).  It follows the
// four-phase small-cache algorithm of App. C: square tiles with the contraction loop split
// into chunks, and the n x n matrices f (here P) and p (here dS) written to memory between
// the phases:
//   scores kernel : per tile S^T = K Q^T with a k-loop over d-chunks, f = exp(S - LSE); then dP^T = V dO^T
//                   with a second k-loop and p = f o (q - v) (phases 1 to 3; one sweep over the tile
//                   because v = rowsum(dO o O) is precomputed) -> P, dS in HBM
//   gemm kernel   : dV = P^T dO, dK = scale dS^T Q, dQ = scale dS K as tiled products with the
//                   k-loop over n (phase 4 written for dQ/dK/dV instead of A_1^T p A_2)
// The forward uses the same kernels: partial row statistics of S per 64-key chunk, a combine
// step for LSE, P = exp(S - LSE) written to HBM, and O = P V.
#include <type_traits>

#include "attn_common.hpp"
#include "attn_internal.hpp"

namespace attn {

// Scores kernel, tiles of 128 queries x 256 keys, four waves with a 128 x 64 block (4 x 2 accumulators) each; a
// k-step needs 32-column chunks of two operands (24 KB), and three LDS stages (copies two steps ahead) fit two
// workgroups on a CU.  Accumulator: lane <-> query, register <-> key.  Modes:
//   kStats    row maximum and sum of exp of S per 64-key chunk (the forward's first sweep)
//   kProbs    P = exp(S - LSE) written to the workspace (the forward's second sweep)
//   kBackward P and dS.  The two products of a tile are formed one after the other - S^T over all of d, then dP^T
//             over all of d - so that the wave can hold its block of the one in progress: 256 x 128 tiles move 384 bytes
//             from memory per MFMA instead of the 512 of 128 x 128 tiles with both products at once.  Between the
//             passes P stays in registers, rounded to bf16 as it is stored (dS = P (dP - delta) uses that rounded P).
enum ScoreMode { kStats = 0, kProbs = 1, kBackward = 2 };
constexpr int kScoreStage = (256 + 128) * 32 * 2, kScoreLds = 3 * kScoreStage;
template <int MODE>
__global__ void __launch_bounds__(kThreads, 2) ld_scores_kernel(LargeDParams p) {
    constexpr int BK = 32, kKeys = 256;
    constexpr int kTileK = kKeys * BK * 2, kTileQ = 128 * BK * 2, kStage = kScoreStage;
    constexpr int kOutTile = 128 * kKeys * 2;  // a [128 queries][256 keys] bf16 tile staged for the stores
    static_assert(kOutTile <= 3 * kStage, "the staged tile reuses the stages");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;  // keys 128 wm .., queries 64 wn ..
    const int nbq = p.npad / 128, nbk = p.npad / kKeys;
    int bh, kb, qb;
    {   // XCD-contiguous tile order, regions of 8 query tiles x 1024 keys (as in the forward modes)
        constexpr int kPerRegionRow = 1024 / kKeys;
        const int per_head = nbq * nbk, total = per_head * p.batch * p.heads;
        int t = blockIdx.x;
        if ((total & 7) == 0) t = (t >> 3) + (t & 7) * (total >> 3);
        bh = t / per_head;
        const int tile = t % per_head;
        if ((nbq & 7) == 0 && nbk % kPerRegionRow == 0) {
            const int region = tile / (8 * kPerRegionRow), in = tile % (8 * kPerRegionRow);
            const int rpr = nbk / kPerRegionRow;
            qb = (region / rpr) * 8 + in / kPerRegionRow;
            kb = (region % rpr) * kPerRegionRow + in % kPerRegionRow;
        } else {
            qb = tile / nbk;
            kb = tile % nbk;
        }
    }
    if (p.causal && kb * kKeys > qb * 128 + 127) return;  // wholly above the diagonal: never read
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const int k0 = kb * kKeys, q0 = qb * 128;
    const long ld = p.stride_n;

    TileLoader<BK, kKeys, 4> copy_k;
    TileLoader<BK, 128, 4> copy_q;
    copy_k.init(tid, ld);
    copy_q.init(tid, ld);
    constexpr int kCopiesPerFetch = (kTileK + kTileQ) / (1024 * 4);  // per wave
    int rk[BK / 16], rq[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        rk[ks] = tile_off<BK>(128 * wm + l32, 2 * ks + h);
        rq[ks] = tile_off<BK>(64 * wn + l32, 2 * ks + h) + kTileK;
    }
    const int chunks = p.d / BK;

    f32x16 c[4][2];
    // one product over all of d: rows of gA (keys) x rows of gB (queries), three stages
    auto product = [&](const __bf16* gA, const __bf16* gB) {
#pragma unroll
        for (int tm = 0; tm < 4; ++tm)
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int i = 0; i < 16; ++i) c[tm][tn][i] = 0.f;
        auto fetch = [&](int kc, int stage) {
            char* b = smem + stage * kStage;
            copy_k.load(gA + kc * BK, ld, k0, p.n, b, tid);
            copy_q.load(gB + kc * BK, ld, q0, p.n, b + kTileK, tid);
        };
        fetch(0, 0);
        if (chunks > 1) {
            fetch(1, 1);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerFetch) : "memory");
        } else {
            wait_direct_loads();
        }
        __syncthreads();
        auto step = [&](int kc, auto stage_index) {
            constexpr int si = decltype(stage_index)::value, so = si * kStage;
            const bool more = kc + 2 < chunks;
            if (more) fetch(kc + 2, (si + 2) % 3);
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                // the key fragments one ahead of their MFMAs, two live at a time (the accumulators and the packed P of
                // the first pass leave room for little else)
                bf16x8 b[2], a = FragOffsets<BK>::read(smem, rk[ks], so);
#pragma unroll
                for (int t = 0; t < 2; ++t) b[t] = FragOffsets<BK>::read(smem, rq[ks], so + 32 * t * (BK * 2));
#pragma unroll
                for (int tm = 0; tm < 4; ++tm) {
                    bf16x8 a_next = a;
                    if (tm + 1 < 4) a_next = FragOffsets<BK>::read(smem, rk[ks], so + 32 * (tm + 1) * (BK * 2));
#pragma unroll
                    for (int tn = 0; tn < 2; ++tn) c[tm][tn] = mfma32(a, b[tn], c[tm][tn]);
                    a = a_next;
                }
            }
            if (more) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerFetch) : "memory");
            else wait_direct_loads();
            __syncthreads();
        };
        int kc = 0;
        for (; kc + 3 <= chunks; kc += 3) {
            step(kc, std::integral_constant<int, 0>{});
            step(kc + 1, std::integral_constant<int, 1>{});
            step(kc + 2, std::integral_constant<int, 2>{});
        }
        if (kc < chunks) {
            step(kc, std::integral_constant<int, 0>{});
            if (kc + 1 < chunks) step(kc + 1, std::integral_constant<int, 1>{});
        }
    };
    // the whole tile from LDS ([query][key] rows, swizzled chunks) to a matrix in the workspace, in whole rows
    auto store_tile = [&](__bf16* M) {
        __syncthreads();
        constexpr int kChunks = kKeys / 8, kRowsPerPass = kThreads / kChunks;  // 8 rows per pass
        const int cc = tid % kChunks;
        // the lane's addresses are formed here, not carried in registers through the product loop in front
        int q_first = q0;
        asm volatile("" : "+s"(q_first));
#pragma unroll 4
        for (int r0 = 0; r0 < 128; r0 += kRowsPerPass) {
            const int row = r0 + tid / kChunks;
            const long off = ((long)bh * p.npad + q_first + row) * p.npad + k0 + 8 * cc;
            *reinterpret_cast<u32x4*>(M + off) = *reinterpret_cast<const u32x4*>(smem + tile_off<kKeys>(row, cc));
        }
        __syncthreads();  // the stages are free again
    };

    // ---- pass 1: S^T
    product(p.K + base, p.Q + base);
    const float cs = p.scale * kLog2e;
    const bool need_mask = (p.causal && k0 + kKeys - 1 > q0) || (k0 + kKeys > p.n);
    if constexpr (MODE == kStats) {
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const int q = q0 + 64 * wn + 32 * tn + l32;
#pragma unroll
            for (int half = 0; half < 2; ++half) {  // the two 64-key chunks of this wave's 128 keys
                float x[2][16];
                float mx = -__builtin_inff();
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float v = c[2 * half + t][tn][i] * cs;
                        const int key = k0 + 128 * wm + 64 * half + 32 * t + acc_row(i, h);
                        if (need_mask && (key >= p.n || (p.causal && key > q))) v = -__builtin_inff();
                        x[t][i] = v;
                        mx = fmaxf(mx, v);
                    }
                mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                const float m_use = mx == -__builtin_inff() ? 0.f : mx;
                float sum = 0.f;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(x[t][i] - m_use);
                sum += __shfl_xor(sum, 32, 64);
                if (q < p.n && h == 0) {
                    const long o = ((long)bh * (2 * nbq) + k0 / 64 + 2 * wm + half) * p.n + q;  // [bh][chunk][query]
                    p.stat_m[o] = mx;
                    p.stat_l[o] = sum;
                }
            }
        }
        return;
    }
    // P (bf16): written out and, in the backward, kept packed in registers
    uint32_t pk[MODE == kBackward ? 4 : 1][2][8];
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
        const int q = q0 + 64 * wn + 32 * tn + l32;
        const bool q_ok = q < p.n;
        const float lse2 = q_ok ? (MODE == kBackward ? p.LSE : p.LSEout)[(long)bh * p.n + q] * kLog2e : __builtin_inff();
        char* prow = smem + (64 * wn + 32 * tn + l32) * (kKeys * 2);
#pragma unroll
        for (int tm = 0; tm < 4; ++tm)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int key = k0 + 128 * wm + 32 * tm + 8 * g + 4 * h;
                float pv[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float v = __builtin_amdgcn_exp2f(c[tm][tn][4 * g + r] * cs - lse2);
                    if (lse2 == -__builtin_inff()) v = 0.f;  // a fully masked row has LSE = -inf
                    if (need_mask && (key + r >= p.n || (p.causal && key + r > q))) v = 0.f;
                    pv[r] = v;
                }
                u32x2 a;
                a[0] = pack_bf16(pv[0], pv[1]);
                a[1] = pack_bf16(pv[2], pv[3]);
                if constexpr (MODE == kBackward) {
                    pk[tm][tn][2 * g] = a[0];
                    pk[tm][tn][2 * g + 1] = a[1];
                }
                const int slot = (((16 * wm + 4 * tm + g) ^ swz<kKeys>(64 * wn + 32 * tn + l32)) << 4) + 8 * h;
                *reinterpret_cast<u32x2*>(prow + slot) = a;
            }
    }
    store_tile(p.P);
    if constexpr (MODE != kBackward) return;

    // ---- pass 2: dP^T -> dS = P (dP - delta)
    product(p.V + base, p.dO + base);
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
        const int q = q0 + 64 * wn + 32 * tn + l32;
        const float dl = q < p.n ? p.delta[(long)bh * p.n + q] : 0.f;  // (P is 0 in rows past n)
        char* prow = smem + (64 * wn + 32 * tn + l32) * (kKeys * 2);
#pragma unroll
        for (int tm = 0; tm < 4; ++tm)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float dv[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t word = pk[tm][tn][2 * g + (r >> 1)];
                    const float pv = __builtin_bit_cast(float, (r & 1) ? (word & 0xffff0000u) : (word << 16));
                    dv[r] = pv * (c[tm][tn][4 * g + r] - dl);
                }
                u32x2 a;
                a[0] = pack_bf16(dv[0], dv[1]);
                a[1] = pack_bf16(dv[2], dv[3]);
                const int slot = (((16 * wm + 4 * tm + g) ^ swz<kKeys>(64 * wn + 32 * tn + l32)) << 4) + 8 * h;
                *reinterpret_cast<u32x2*>(prow + slot) = a;
            }
    }
    store_tile(p.dS);
}

// LSE from the per-chunk statistics.  A workgroup takes 16 rows; 16 threads per row each fold every 16th chunk into a
// running (maximum, sum) pair, and the 16 pairs of a row are folded through LDS (one thread per row alone spent its time
// waiting for one load after the other).  Statistics are [bh][chunk][query]: threads that stand for consecutive
// queries read consecutive floats.
constexpr int kCombineRows = 16, kCombineParts = kThreads / kCombineRows;
__global__ void __launch_bounds__(kThreads) ld_lse_combine_kernel(LargeDParams p) {
    __shared__ float part_m[kCombineParts][kCombineRows], part_l[kCombineParts][kCombineRows];
    const int rl = threadIdx.x % kCombineRows, g = threadIdx.x / kCombineRows;
    const long rows = (long)p.batch * p.heads * p.n;
    const long r = (long)blockIdx.x * kCombineRows + rl;
    const bool ok = r < rows;
    const int q = ok ? (int)(r % p.n) : 0;
    const int nb = p.npad / 128;
    const int chunks = ok ? 2 * (p.causal ? q / 128 + 1 : nb) : 0;
    const long pitch = p.n;
    const long head = ok ? (r / p.n) * (2 * nb) * pitch + q : 0;
    float M = -__builtin_inff(), L = 0.f;
    for (int c = g; c < chunks; c += kCombineParts) {
        const float mc = p.stat_m[head + c * pitch], lc = p.stat_l[head + c * pitch];
        if (mc != -__builtin_inff()) {
            const float top = fmaxf(M, mc);
            L = L * __builtin_amdgcn_exp2f(M - top) + lc * __builtin_amdgcn_exp2f(mc - top);  // (exp2(-inf) = 0 at the start)
            M = top;
        }
    }
    part_m[g][rl] = M;
    part_l[g][rl] = L;
    __syncthreads();
    if (g != 0 || !ok) return;
    for (int k = 1; k < kCombineParts; ++k) {
        const float mk = part_m[k][rl], lk = part_l[k][rl];
        if (mk != -__builtin_inff()) {
            const float top = fmaxf(M, mk);
            L = L * __builtin_amdgcn_exp2f(M - top) + lk * __builtin_amdgcn_exp2f(mk - top);
            M = top;
        }
    }
    p.LSEout[r] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * kLn2 : -__builtin_inff();
}

// C[m][n] = alpha * sum_k A(m, k) B(k, n): 128 x 128 output tile per workgroup, k-loop over the
// sequence.  A is one of the n x n matrices in the workspace (row pitch npad): read as stored
// ([m][k], A_KMAJOR = false: dQ = dS K, O = P V) or transposed ([k][m], A_KMAJOR = true:
// dV = P^T dO, dK = dS^T Q).  B is an [n, d] tensor, k along its rows.  Under the causal rule
// the k-range of a tile shrinks to the blocks the scores kernel wrote.
struct GemmArgs {
    const __bf16* A;  // workspace matrix, [bh][npad][npad]
    const __bf16* B;  // [b, h, n, d] tensor
    __bf16* C;        // [b, h, n, d] tensor
    float alpha;
};

// Output tile of the product kernel: 256 rows x 128 columns per workgroup, a 128 x 64 block (4 x 2
// accumulators) per wave: six fragments from LDS feed eight MFMAs, and a k-step of 32 moves 24 KB
// from global memory for 64 MFMAs.  (With 128 x 128 tiles the copies alone, at the 64 B/clk that
// the vector memory path delivers per CU, took as long as the MFMAs.)
constexpr int kGemmBK = 32, kGemmM = 256;
template <bool A_KMAJOR>
__global__ void __launch_bounds__(kThreads, 2) ld_gemm_kernel(LargeDParams p, GemmArgs g) {
    constexpr int BK = kGemmBK, TM = kGemmM;
    constexpr int kTileA = TM * BK * 2, kTileB = 128 * BK * 2, kStage = kTileA + kTileB;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, uniform
    const int wm = w >> 1, wn = w & 1;
    // 1-D grid, XCD-contiguous like the scores kernel: the column tiles of one (head, row block)
    // follow one another on one XCD and share its copy of the A operand
    int bh, mb, n0;
    {
        const int nt = (p.d + 127) / 128, mbs = p.npad / TM, total = nt * mbs * p.batch * p.heads;
        int t = blockIdx.x;
        if ((total & 7) == 0) t = (t >> 3) + (t & 7) * (total >> 3);
        n0 = (t % nt) * 128;
        mb = (t / nt) % mbs;
        bh = t / (nt * mbs);
    }
    const int m0 = mb * TM;
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const __bf16* gA = g.A + (long)bh * p.npad * p.npad;  // npad x npad, zero beyond n
    const __bf16* gB = g.B + base;
    int k_begin = 0, k_end = p.npad;
    if (p.causal) {
        if (A_KMAJOR) k_begin = m0;   // queries at or after this key block
        else k_end = m0 + TM;         // keys at or before this query block
    }

    f32x16 c[4][2];
#pragma unroll
    for (int tm = 0; tm < 4; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) c[tm][tn][i] = 0.f;
    // Operand tiles go straight from global memory into the LDS stage that was last read one
    // step ago.  Rows of B past n repeat the last row; they meet columns (rows, if A is read
    // transposed) of A that are zero.  Lane offsets of the copies and of the fragment reads are
    // computed once; the k-loop runs three steps per iteration so that the stage offsets are
    // immediates.
    TileLoader<TM, BK> copy_at;   // A read transposed: BK rows of TM columns
    TileLoader<BK, TM> copy_a;    // A as stored: TM rows of BK columns
    TileLoader<128, BK> copy_b;
    if (A_KMAJOR) copy_at.init(tid, p.npad);
    else copy_a.init(tid, p.npad);
    copy_b.init(tid, p.stride_n);
    auto fetch = [&](int k, int stage) {
        char* at = smem + stage * kStage;
        if (A_KMAJOR) copy_at.load(gA + m0 + (long)k * p.npad, at);
        else copy_a.load(gA + k + (long)m0 * p.npad, at);
        copy_b.load(gB + n0, p.stride_n, k, p.n, at + kTileA, tid);
    };
    // A read transposed: one register pair per 32-row tile t.  A as stored: one register per k-step, the 16-byte
    // chunk 2 ks + h of this lane's row (the 32-row tiles are immediates apart); B is then fetched with its k index
    // in the same natural order.  (Reading A in 8-byte halves to match the other order cost 44 % LDS bank conflicts.)
    int ra[4][2], rc[BK / 16], rb[2][2];
    {
        FragOffsets<TM> fa;
        FragOffsets<128> fb;
        fa.init(lane);
        fb.init(lane);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            ra[t][0] = fa.tr(4 * wm + t, 0);
            ra[t][1] = fa.tr(4 * wm + t, 1);
        }
        // A as stored: whole 16-byte chunks of this lane's row (k in natural order), chunk 2 ks + h
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) rc[ks] = tile_off<BK>(128 * wm + l32, 2 * ks + h);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int half = 0; half < 2; ++half)
                rb[t][half] = (A_KMAJOR ? fb.tr(2 * wn + t, half) : FragOffsets<128>::tr_natural(lane, 2 * wn + t, half)) + kTileA;
    }
    // Three stages: the copies of step k + 2 are issued while step k is multiplied, so two steps' worth of bytes
    // (48 KB per workgroup) are in flight; with two stages the product kernels waited for memory at every step.
    constexpr int kCopiesPerFetch = (kTileA + kTileB) / (1024 * 4);  // per wave
    fetch(k_begin, 0);
    if (k_begin + BK < k_end) {
        fetch(k_begin + BK, 1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerFetch) : "memory");
    } else {
        wait_direct_loads();
    }
    __syncthreads();
    auto step = [&](int k, auto stage_index) {
        constexpr int si = decltype(stage_index)::value, so = si * kStage;
        const bool more = k + 2 * BK < k_end;
        if (more) fetch(k + 2 * BK, (si + 2) % 3);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 a[4], b[2];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (A_KMAJOR) {
                    a[t] = FragOffsets<TM>::read_t(smem, ra[t][0], ra[t][1], 16 * ks, so);
                } else {
                    a[t] = FragOffsets<BK>::read(smem, rc[ks], so + 32 * t * (BK * 2));
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
                b[t] = A_KMAJOR ? FragOffsets<128>::read_t(smem, rb[t][0], rb[t][1], 16 * ks, so)
                                : FragOffsets<128>::read_t_natural(smem, rb[t][0], rb[t][1], 16 * ks, so);
#pragma unroll
            for (int tm = 0; tm < 4; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn) c[tm][tn] = mfma32(a[tm], b[tn], c[tm][tn]);
        }
        // step k + 1 must have landed; the copies just issued may stay in flight
        if (more) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kCopiesPerFetch) : "memory");
        else wait_direct_loads();
        __syncthreads();
    };
    int k = k_begin;
    for (; k + 3 * BK <= k_end; k += 3 * BK) {
        step(k, std::integral_constant<int, 0>{});
        step(k + BK, std::integral_constant<int, 1>{});
        step(k + 2 * BK, std::integral_constant<int, 2>{});
    }
    if (k < k_end) {
        step(k, std::integral_constant<int, 0>{});
        if (k + BK < k_end) step(k + BK, std::integral_constant<int, 1>{});
    }
    // accumulator: lane <-> output column, register <-> output row
#pragma unroll
    for (int tm = 0; tm < 4; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const int col = n0 + 64 * wn + 32 * tn + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = m0 + 128 * wm + 32 * tm + acc_row(i, h);
                if (row < p.n && col < p.d) g.C[base + (long)row * p.stride_n + col] = (__bf16)(c[tm][tn][i] * g.alpha);
            }
        }
}

static hipError_t set_lds(const void* fn, int bytes) {
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

constexpr int kGemmLds = 3 * (kGemmM + 128) * kGemmBK * 2;  // three stages of an A and a B tile (72 KB: two workgroups per CU)
template <bool A_KMAJOR>
static void run_gemm(const LargeDParams& p, const __bf16* A, const __bf16* B, __bf16* C, float alpha,
                     hipStream_t stream) {
    const dim3 grid((unsigned)(((p.d + 127) / 128) * (p.npad / kGemmM) * p.batch * p.heads));
    GemmArgs g{A, B, C, alpha};
    hipLaunchKernelGGL(ld_gemm_kernel<A_KMAJOR>, grid, dim3(kThreads), kGemmLds, stream, p, g);
}

// LDS sizes of the large-d kernels on the current device (set on every call: cheap, and per device).
hipError_t configure_larged() {
    hipError_t e = set_lds(reinterpret_cast<const void*>(ld_scores_kernel<kStats>), kScoreLds);
    if (e == hipSuccess) e = set_lds(reinterpret_cast<const void*>(ld_scores_kernel<kProbs>), kScoreLds);
    if (e == hipSuccess) e = set_lds(reinterpret_cast<const void*>(ld_scores_kernel<kBackward>), kScoreLds);
    if (e == hipSuccess) e = set_lds(reinterpret_cast<const void*>(ld_gemm_kernel<true>), kGemmLds);
    if (e == hipSuccess) e = set_lds(reinterpret_cast<const void*>(ld_gemm_kernel<false>), kGemmLds);
    return e;
}

hipError_t launch_larged(bool backward, const LargeDParams& p, hipStream_t stream) {
    const hipError_t ce = configure_larged();
    if (ce != hipSuccess) return ce;
    const unsigned bh = (unsigned)(p.batch * p.heads);
    const unsigned nbq = (unsigned)(p.npad / 128);
    const dim3 sgrid(nbq * (unsigned)(p.npad / 256) * bh);  // score tiles: 128 queries x 256 keys
    const dim3 block(kThreads);
    if (!backward) {
        hipLaunchKernelGGL(ld_scores_kernel<kStats>, sgrid, block, kScoreLds, stream, p);
        const long rows = (long)bh * p.n;
        hipLaunchKernelGGL(ld_lse_combine_kernel, dim3((unsigned)((rows + kCombineRows - 1) / kCombineRows)), block, 0, stream, p);
        hipLaunchKernelGGL(ld_scores_kernel<kProbs>, sgrid, block, kScoreLds, stream, p);
        run_gemm<false>(p, p.P, p.V, p.Oout, 1.f, stream);
    } else {
        hipLaunchKernelGGL(ld_scores_kernel<kBackward>, sgrid, block, kScoreLds, stream, p);
        run_gemm<true>(p, p.P, p.dO, p.dV, 1.f, stream);
        run_gemm<true>(p, p.dS, p.Q, p.dK, p.scale, stream);
        run_gemm<false>(p, p.dS, p.K, p.dQ, p.scale, stream);
    }
    return hipGetLastError();
}

}  // namespace attn
