// Fused backward kernels for d <= 256 (the regime where a d x d working set fits on chip; d = 256
// runs with one wave per SIMD and up to 512 registers per lane):
//   dQ      : one workgroup owns a block of 128 queries and streams key tiles; its prologue also
//             forms delta = rowsum(dO o O) (second matrix form of p, App. B.4) for those queries
//   dK, dV  : one workgroup owns a block of 64 keys and streams query tiles
//   (delta_kernel, the stand-alone row sum, serves the large-d path)
// Per tile pair this is the inner body of the paper's large-cache phase-2 algorithm (App. D):
// q = dO h^T, A = S A_2^T, f = exp(A) / l, p = f o q - diag(v) f, followed by the three
// products that use f and p.  The resident operand is the owned block, so dK/dV (resp. dQ)
// accumulate in registers with no atomics and no n x n matrix ever leaves the chip.
#include <type_traits>

#include "attn_common.hpp"
#include "attn_internal.hpp"

namespace attn {

// --------------------------------------------------------------------------------- delta
// min(d / 8, 64) consecutive lanes share one row (16-byte chunks; a lane takes every 64th chunk when
// the row has more than 64); the row sum is a shuffle reduction inside that lane group.  d / 8 must
// be a power of two.
__global__ void __launch_bounds__(kThreads) delta_kernel(FusedParams p, int d) {
    const int cpr = d >> 3;             // chunks per row
    const int lpr = cpr < 64 ? cpr : 64;  // lanes per row
    const long rows = (long)p.batch * p.heads * p.n;
    const long f = (long)blockIdx.x * kThreads + threadIdx.x;
    const long r = f / lpr;
    const int c = (int)(f % lpr);
    float acc = 0.f;
    if (r < rows) {
        const int bh = (int)(r / p.n), i = (int)(r % p.n);
        const long off = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h + (long)i * p.stride_n;
        for (int cc = c; cc < cpr; cc += lpr) {
            const bf16x8 o = *reinterpret_cast<const bf16x8*>(p.O + off + cc * 8);
            const bf16x8 g = *reinterpret_cast<const bf16x8*>(p.dO + off + cc * 8);
#pragma unroll
            for (int t = 0; t < 8; ++t) acc += (float)o[t] * (float)g[t];
        }
    }
    for (int m = lpr >> 1; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
    if (r < rows && c == 0) p.delta[r] = acc;
}

// --------------------------------------------------------------------------- block order
// order[r] = the block with the r-th longest list (ties: lower index first).  Workgroups are
// dispatched in index order, so taking the long lists first keeps the tail of a launch short
// when the lists of a block mask differ in length, and workgroups that run at the same time walk
// through the streamed blocks together (their re-reads then hit in L2).  Two steps: the list
// lengths that count (entries the causal rule removes do not), then one thread per block ranks
// its length against all others (nblk^2 comparisons).
__global__ void __launch_bounds__(kThreads) block_len_kernel(const int32_t* ptr_all, const int32_t* idx, int nblk,
                                                            int causal, int column_lists, int32_t* len_all) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= nblk) return;
    const int32_t* ptr = ptr_all + (long)blockIdx.y * (nblk + 1);  // mask blockIdx.y
    int32_t* len = len_all + (long)blockIdx.y * nblk;
    const int first = ptr[i];
    int count = ptr[i + 1] - first;
    if (causal) {
        if (column_lists) count -= causal_col_skip(idx, first, count, i);
        else count = causal_row_entries(idx, first, count, i);
    }
    len[i] = count;
}
__global__ void __launch_bounds__(kThreads) block_order_kernel(const int32_t* len_all, int nblk, int32_t* order_all) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= nblk) return;
    const int32_t* len = len_all + (long)blockIdx.y * nblk;
    int32_t* order = order_all + (long)blockIdx.y * nblk;
    const int mine = len[i];
    int rank = 0;
    for (int k = 0; k < nblk; ++k) {
        const int other = len[k];
        rank += (other > mine || (other == mine && k < i)) ? 1 : 0;
    }
    order[rank] = i;
}

// Both steps, for the row lists and the column lists of a mask, in one launch when a mask has at most
// kOrderFusedBlocks blocks: workgroup (mask, kind) keeps the lengths in LDS and ranks them there (four small
// launches in front of the backward kernels cost as much as 2 % of a block-sparse call).
constexpr int kOrderFusedBlocks = 256;
__global__ void __launch_bounds__(kThreads) block_order_fused_kernel(const int32_t* row_ptr, const int32_t* col_idx,
                                                                    const int32_t* col_ptr, const int32_t* row_idx,
                                                                    int nblk, int causal, int32_t* order_q,
                                                                    int32_t* order_k, int first_kind) {
    __shared__ int32_t len[kOrderFusedBlocks];
    const int kind = first_kind + blockIdx.y;  // 0: row lists (query blocks), 1: column lists (key blocks)
    const int32_t* ptr = (kind ? col_ptr : row_ptr) + (long)blockIdx.x * (nblk + 1);  // mask blockIdx.x
    const int32_t* idx = kind ? row_idx : col_idx;
    int32_t* order = (kind ? order_k : order_q) + (long)blockIdx.x * nblk;
    for (int i = threadIdx.x; i < nblk; i += kThreads) {
        const int first = ptr[i];
        int count = ptr[i + 1] - first;
        if (causal) {
            if (kind) count -= causal_col_skip(idx, first, count, i);
            else count = causal_row_entries(idx, first, count, i);
        }
        len[i] = count;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nblk; i += kThreads) {
        const int mine = len[i];
        int rank = 0;
        for (int k = 0; k < nblk; ++k) {
            const int other = len[k];
            rank += (other > mine || (other == mine && k < i)) ? 1 : 0;
        }
        order[rank] = i;
    }
}

// ------------------------------------------------------------------------------- dK, dV
// A workgroup owns 64 keys and streams 64-query tiles; per tile its 4 waves work in two phases:
//   phase 1: wave (wk, wx) computes S^T and dP^T for key half wk and query half wx, with the
//            resident K / V fragments as A operands (lane <-> query, so lse2 and delta are
//            per-lane scalars), then P and dS go to LDS as bf16 tiles [query][key];
//   phase 2: wave (wk, wx) accumulates dV^T (wx = 0) or dK^T (wx = 1) for the d-half wk and all
//            64 keys over the 64 queries, as a block of accumulators in which every fragment
//            read from LDS feeds two MFMAs; P / dS (B operands) and dO^T / Q^T (A operands)
//            are all read with transposing LDS loads.
// Keeping K, V and both gradients of 128 keys in the registers of one workgroup instead (no LDS
// round trip for P and dS) needs more than 256 registers per lane at d = 128, i.e. one wave per
// SIMD; that variant was measured at 60 % of this one's speed at d = 128 and 91 % at d = 64.
// Wave priorities per phase: the two waves that share a SIMD compete for one matrix pipe and
// fall into step; ranking phase 1 above phase 2 above the exponentials lets one of them run ahead
// (measured: 2 % faster than without priorities, 3 % faster than with the exponentials in the middle).
constexpr int kPrioPhase1 = 3, kPrioSoftmax = 0, kPrioPhase2 = 1;
template <int D>
__global__ void __launch_bounds__(kThreads, D <= 128 ? 2 : 1) bwd_dkdv_kernel(FusedParams p) {
    constexpr int BR = 64, BC = 64, KS = D / 16, MT = D / 32;
    constexpr int kTileBytes = BR * D * 2;
    constexpr int kStageBytes = 2 * kTileBytes;
    constexpr int kPBytes = BC * BR * 2;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, uniform
    const int wk = w & 1, wx = w >> 1;
    // with an order list the grid has both halves of every 128-key block (the last one may lie
    // past n) and the blocks come longest list first
    const int key_blocks = p.order ? 2 * ((p.n + 127) / 128) : (p.n + BC - 1) / BC;
    int bh, j;
    decode_block(blockIdx.x, key_blocks, p.batch * p.heads, bh, j);
    if (p.order) {
        j = 2 * p.order[(long)bh * p.order_stride + (j >> 1)] + (j & 1);
        if (j * BC >= p.n) return;
    }
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const long ld = p.stride_n;
    const int j0 = j * BC;
    const float* lse_g = p.LSE + (long)bh * p.n;
    const float* delta_g = p.delta + (long)bh * p.n;

    int n_it, t0 = 0, lp0 = 0;
    if (p.list_ptr) {
        const int32_t* lptr = p.list_ptr + (long)bh * p.list_stride;  // this (batch, head)'s mask
        lp0 = lptr[j0 / 128];
        int entries = lptr[j0 / 128 + 1] - lp0;
        if (p.causal) {
            const int skip = causal_col_skip(p.list_idx, lp0, entries, j0 / 128);
            lp0 += skip;
            entries -= skip;
        }
        n_it = entries * (128 / BR);
    } else {
        t0 = p.causal ? j0 / BR : 0;
        n_it = (p.n + BR - 1) / BR - t0;
    }
    auto tile_start = [&](int it) -> int { return tile_start_row<BR>(p.list_idx, lp0, t0, it); };

    const int key = j0 + 32 * wk + l32;
    bf16x8 kf[KS], vf[KS];
    {
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = zero;
            vf[ks] = zero;
            if (key < p.n) {
                kf[ks] = *reinterpret_cast<const bf16x8*>(p.K + base + (long)key * ld + 16 * ks + 8 * h);
                vf[ks] = *reinterpret_cast<const bf16x8*>(p.V + base + (long)key * ld + 16 * ks + 8 * h);
            }
        }
    }
    // phase-2 role of this wave: wx = 0 accumulates dV^T (from P and dO^T), wx = 1 dK^T (from dS
    // and Q^T), each for all 64 keys and the half wk of d: a 2 x 2 block of accumulators, so that
    // every fragment read from LDS feeds two MFMAs
    constexpr int MH = MT / 2;
    f32x16 acc[MH][2];
#pragma unroll
    for (int m = 0; m < MH; ++m)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][kt][i] = 0.f;

    const float c = p.scale * kLog2e;
    // Row i0 + 32 wx + l32 of the tile being fetched.  The loaded values are not touched until
    // the next iteration, so nothing waits on the copies in flight behind them.
    float lse_raw = 0.f, delta_raw = 0.f;
    bool row_ok = false;
    TileLoader<D, BR> loader;
    loader.init(tid, ld);
    auto fetch_rows = [&](int i0) {
        const int q = i0 + 32 * wx + l32;
        row_ok = q < p.n;
        lse_raw = lse_g[min(q, p.n - 1)];
        delta_raw = delta_g[min(q, p.n - 1)];
    };
    auto fetch = [&](int i0, int stage_off) {
        char* s = smem + stage_off;
        loader.load(p.Q + base, ld, i0, p.n, s, tid);
        loader.load(p.dO + base, ld, i0, p.n, s + kTileBytes, tid);
        fetch_rows(i0);
    };
    int i0_next = n_it > 0 ? tile_start(0) : 0;
    if (n_it > 0) fetch(i0_next, 0);
    wait_direct_loads();
    __syncthreads();

#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        settle(kf[ks]);
        settle(vf[ks]);
    }
    FragOffsets<D> fo;    // Q / dO tiles
    FragOffsets<BC> fp;   // P / dS tiles
    fo.init(lane);
    fp.init(lane);
    constexpr int kPOff = 2 * kStageBytes, kDsOff = kPOff + kPBytes;
    // This lane's 8-byte slot of group g in the [query][key] tiles: p_wr ^ (g << 4).  The two
    // 8-byte halves of a chunk swap places in odd rows: rows 2k and 2k+1 share their swizzle
    // term and are 128 bytes apart, so without the swap the 16 lanes that write together would
    // hit every bank twice.  The transposed reads apply the same swap per lane.
    const int p_wr = tile_off<BC>(32 * wx + l32, 4 * wk) + 8 * (h ^ (l32 & 1));
    fp.tr0 ^= (((lane & 15) >> 2) & 1) << 3;
    // Address registers of everything this wave reads from or writes to LDS, relative to the
    // stage (all wave-dependent tile choices folded in): a fetch is then a register plus an
    // immediate, with no vector arithmetic in the loop.
    //   q_rm[ks]     Q rows 32 wx + l32 (phase 1; the dO tile is kTileBytes further)
    //   a_tr[m][.]   phase-2 A operand: dO^T (wx = 0) or Q^T (wx = 1), columns 32 (MH wk + m) ..
    //   b_tr[kt][.]  phase-2 B operand: P (wx = 0) or dS (wx = 1), keys 32 kt ..
    //   p_slot[g]    this lane's slot in the P tile (the dS tile is kPBytes further)
    int q_rm[KS], a_tr[MT / 2][2], b_tr[2][2], p_slot[4];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) q_rm[ks] = fo.rm(ks) + 32 * wx * (D * 2);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int m = 0; m < MT / 2; ++m) a_tr[m][half] = fo.tr((MT / 2) * wk + m, half) + (wx == 0 ? kTileBytes : 0);
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) b_tr[kt][half] = fp.tr(kt, half) + (wx == 0 ? kPOff : kDsOff);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) p_slot[g] = kPOff + (p_wr ^ (g << 4));
    // One streamed query tile (two barriers).  `masked` selects the copy of phase 1 that applies
    // the causal bound.
    auto tile = [&](auto stage_off, int it, int i0, bool skip, auto masked) {
        const float lse_cur = row_ok ? lse_raw * kLog2e : __builtin_inff();
        const float delta_cur = row_ok ? delta_raw : 0.f;
        const int q_off = stage_off;  // Q tile; the dO tile follows it
        // The copies of the next tile go into the stage that was last read before barrier B of the
        // previous tile.  In the mask-free body they are issued one by one between the MFMAs of
        // phase 1 (a wave that issues all of them at once waits until the copy path, 64 B per
        // cycle and CU, has taken them: ~750 cycles per tile in front of the first MFMA; 1.5 % faster).
        bool spread = false;
        const __bf16* next_q = nullptr;
        const __bf16* next_g = nullptr;
        char* next_stage = smem + (kStageBytes - q_off);
        if (it + 1 < n_it) {
            i0_next = tile_start(it + 1);
            spread = !decltype(masked)::value && !skip && i0_next + BR <= p.n;
            if (spread) {
                next_q = p.Q + base + (long)i0_next * ld;
                next_g = p.dO + base + (long)i0_next * ld;
                fetch_rows(i0_next);
            } else {
                fetch(i0_next, kStageBytes - q_off);
            }
        }
        __builtin_amdgcn_s_setprio(kPrioPhase1);
        if (!skip) {
            // ---- phase 1: S^T, dP^T for (key half wk) x (query half wx); the resident K / V
            // fragments serve as A operands, so a lane holds one query and lse2 / delta are scalars
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
            {
                // Q and dO fragments are requested kAhead k-steps before the MFMAs that use them
                // (left to itself the compiler requests each pair right in front of its MFMAs and
                // every pair waits out the LDS latency: measured 3 % slower)
                constexpr int kAhead = 2;
                bf16x8 fq[KS], fg[KS];
#pragma unroll
                for (int ks = 0; ks < kAhead; ++ks) {
                    fq[ks] = FragOffsets<D>::read(smem, q_rm[ks], q_off);
                    fg[ks] = FragOffsets<D>::read(smem, q_rm[ks], q_off + kTileBytes);
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {  // two independent accumulation chains, interleaved
                    __builtin_amdgcn_sched_barrier(0);
                    if (ks + kAhead < KS) {
                        fq[ks + kAhead] = FragOffsets<D>::read(smem, q_rm[ks + kAhead], q_off);
                        fg[ks + kAhead] = FragOffsets<D>::read(smem, q_rm[ks + kAhead], q_off + kTileBytes);
                    }
                    s = mfma32(kf[ks], fq[ks], s);
                    dp = mfma32(vf[ks], fg[ks], dp);
                    if (spread) {  // 2 kInst copies over KS k-steps: one per step for d = 64 and 128
                        constexpr int kPer = TileLoader<D, BR>::kInst;
                        static_assert(2 * kPer == KS, "one copy per k-step");
                        if (ks < kPer) loader.load_one(ks, next_q, next_stage);
                        else loader.load_one(ks - kPer, next_g, next_stage + kTileBytes);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(kPrioSoftmax);
            // key j0 + 32 wk + 8g + 4h + r is visible to this lane's query iff 8g + r <= lim
            // (the masked body also serves unpaired tiles of unmasked runs)
            const int lim = p.causal ? i0 + 32 * wx + l32 - j0 - 32 * wk - 4 * h : 0x7fffffff;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float pv[4], dsv[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int i = 4 * g + r;
                    float v = __builtin_amdgcn_exp2f(s[i] * c - lse_cur);
                    if constexpr (decltype(masked)::value) v = (8 * g + r > lim) ? 0.f : v;
                    pv[r] = v;
                    dsv[r] = v * (dp[i] - delta_cur);
                }
                // [query][key] tiles: four consecutive keys of this lane's query
                u32x2 a, b;
                a[0] = pack_bf16(pv[0], pv[1]);
                a[1] = pack_bf16(pv[2], pv[3]);
                b[0] = pack_bf16(dsv[0], dsv[1]);
                b[1] = pack_bf16(dsv[2], dsv[3]);
                *reinterpret_cast<u32x2*>(smem + p_slot[g]) = a;
                *reinterpret_cast<u32x2*>(smem + p_slot[g] + kPBytes) = b;
            }
        }
        lds_barrier();  // P, dS visible; the tile copies for the next iteration stay in flight
        __builtin_amdgcn_s_setprio(kPrioPhase2);
        if (!skip) {
            // ---- phase 2: dV^T = dO^T P (wx = 0) or dK^T = Q^T dS (wx = 1) for d half wk over the
            // 64 queries and 64 keys
            bf16x8 at[2][MH], bt[2][2];
            auto request = [&](int ks) {
#pragma unroll
                for (int m = 0; m < MH; ++m)
                    at[ks & 1][m] = FragOffsets<D>::read_t(smem, a_tr[m][0], a_tr[m][1], 16 * ks, q_off);
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
                    bt[ks & 1][kt] = FragOffsets<BC>::read_t(smem, b_tr[kt][0], b_tr[kt][1], 16 * ks);
            };
            request(0);
#pragma unroll
            for (int ks = 0; ks < BR / 16; ++ks) {  // fragments of the next 16 queries requested ahead
                if (ks + 1 < BR / 16) request(ks + 1);
#pragma unroll
                for (int m = 0; m < MH; ++m)
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        // boustrophedon order: consecutive MFMAs share an operand (A, then B, then A);
                        // with both operands changing between the second and third one the kernel
                        // measured 3 % slower
                        const int kt = (m & 1) ? 1 - kk : kk;
                        acc[m][kt] = mfma32(at[ks & 1][m], bt[ks & 1][kt], acc[m][kt]);
                    }
            }
        }
        wait_direct_loads();
        __syncthreads();
    };
    // Query tiles come in ascending order: under the causal rule the ones that straddle the
    // diagonal (or lie wholly above it) are the first, then everything is visible.  The visible
    // ones go two at a time through a body whose LDS stage offsets are compile-time constants;
    // the masked body (run-time stage) also takes the tile that makes the pairs start at an even
    // index and the one left over at the end.
    int it = 0;
    for (; it < n_it; ++it) {
        const int i0 = i0_next;
        if (!(p.causal && i0 < j0 + BC - 1) && !(it & 1)) break;
        tile((it & 1) * kStageBytes, it, i0, i0 + BR - 1 < j0, std::true_type{});
    }
    for (; it + 2 <= n_it; it += 2) {
        tile(std::integral_constant<int, 0>{}, it, i0_next, false, std::false_type{});
        tile(std::integral_constant<int, kStageBytes>{}, it + 1, i0_next, false, std::false_type{});
    }
    for (; it < n_it; ++it) tile((it & 1) * kStageBytes, it, i0_next, false, std::true_type{});

    const float f = wx == 0 ? 1.f : p.scale;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
        const int okey = j0 + 32 * kt + l32;  // accumulator column
        if (okey < p.n) {
            __bf16* row = (wx == 0 ? p.dV : p.dK) + base + (long)okey * ld + 32 * MH * wk;
#pragma unroll
            for (int m = 0; m < MH; ++m)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 a;
                    a[0] = pack_bf16(acc[m][kt][4 * g + 0] * f, acc[m][kt][4 * g + 1] * f);
                    a[1] = pack_bf16(acc[m][kt][4 * g + 2] * f, acc[m][kt][4 * g + 3] * f);
                    *reinterpret_cast<u32x2*>(row + 32 * m + 8 * g + 4 * h) = a;
                }
        }
    }
}

// ----------------------------------------------------------------------------------- dQ
// Wave w owns queries i0 + 32w .. +31: their Q and dO rows stay in registers as B operands.
// Per key tile (64 keys, two halves T):
//   S^T[T] = K_T Q_w^T, dP^T[T] = V_T dO_w^T        accumulator: lane <-> query, register <-> key
//   dS^T = P^T (dP^T - delta)                        per-lane scalars lse2, delta
//   dQ_w^T += K_T^T dS^T                             K^T from transposed LDS reads
template <int D, int QT>
__global__ void __launch_bounds__(kThreads, D == 64 ? 4 : (QT == 1 && D <= 128 ? 2 : 1)) bwd_dq_kernel(FusedParams p) {
    constexpr int BR = 128 * QT, BC = 64, KS = D / 16, MT = D / 32;
    constexpr int kTileBytes = BC * D * 2;
    constexpr int kStageBytes = 2 * kTileBytes;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, uniform
    const int q_blocks = (p.n + BR - 1) / BR;
    int bh, blk;
    decode_block(blockIdx.x, q_blocks, p.batch * p.heads, bh, blk);
    // longest rows first: under the causal rule the last blocks, under a block mask by the order list
    const int ib = p.order ? p.order[(long)bh * p.order_stride + blk] : (p.causal ? q_blocks - 1 - blk : blk);
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const long ld = p.stride_n;
    const int i0 = ib * BR;
    const int w0 = i0 + 32 * QT * w;  // first query of this wave

    int n_it, lp0 = 0;
    if (p.list_ptr) {  // block lists are per 128 queries: only with QT == 1
        const int32_t* lptr = p.list_ptr + (long)bh * p.list_stride;  // this (batch, head)'s mask
        lp0 = lptr[ib];
        int entries = lptr[ib + 1] - lp0;
        if (p.causal) entries = causal_row_entries(p.list_idx, lp0, entries, ib);
        n_it = entries * (128 / BC);
    } else {
        const int k_end = p.causal ? min(p.n, i0 + BR) : p.n;
        n_it = (k_end + BC - 1) / BC;
    }
    auto tile_start = [&](int it) -> int { return tile_start_row<BC>(p.list_idx, lp0, 0, it); };

    // K and V tiles go straight from global memory into the LDS stage that was last read one
    // iteration ago; rows past n repeat the last row and are masked below.
    TileLoader<D, BC> loader;
    loader.init(tid, ld);
    auto fetch = [&](int j0, int stage) {
        char* s = smem + stage * kStageBytes;
        loader.load(p.K + base, ld, j0, p.n, s, tid);
        loader.load(p.V + base, ld, j0, p.n, s + kTileBytes, tid);
    };
    // the first tile is requested before the resident rows, so that the two latencies overlap
    int j0_next = n_it > 0 ? tile_start(0) : 0;
    if (n_it > 0) fetch(j0_next, 0);

    // resident operands: QT tiles of 32 queries per wave
    int q[QT];
    bf16x8 qf[QT][KS], gf[QT][KS];
    float lse2[QT], dl[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        q[t] = w0 + 32 * t + l32;
        const bool ok = q[t] < p.n;
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[t][ks] = zero;
            gf[t][ks] = zero;
            if (ok) {
                qf[t][ks] = *reinterpret_cast<const bf16x8*>(p.Q + base + (long)q[t] * ld + 16 * ks + 8 * h);
                gf[t][ks] = *reinterpret_cast<const bf16x8*>(p.dO + base + (long)q[t] * ld + 16 * ks + 8 * h);
            }
        }
        lse2[t] = ok ? p.LSE[(long)bh * p.n + q[t]] * kLog2e : __builtin_inff();
        // delta = rowsum(dO o O) of this lane's query: the dO fragments are at hand, the O row is
        // read once here (and nowhere else in the backward); the two lane halves hold the two
        // halves of every 16-element chunk.  The dK / dV kernel, which runs after this one,
        // takes delta from the workspace.
        float dsum = 0.f;
        if (ok) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 of = *reinterpret_cast<const bf16x8*>(p.O + base + (long)q[t] * ld + 16 * ks + 8 * h);
#pragma unroll
                for (int e = 0; e < 8; ++e) dsum += (float)of[e] * (float)gf[t][ks][e];
            }
        }
        dsum += __shfl_xor(dsum, 32, 64);
        dl[t] = ok ? dsum : 0.f;
        if (ok && h == 0) p.delta[(long)bh * p.n + q[t]] = dsum;
    }

    f32x16 dq[QT][MT];
#pragma unroll
    for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i) dq[t][mt][i] = 0.f;

    const float c = p.scale * kLog2e;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            settle(qf[t][ks]);
            settle(gf[t][ks]);
        }
        settle(lse2[t]);
        settle(dl[t]);
    }
    // -delta of this lane's query in all 16 registers of an accumulator block: the dP^T chains start
    // from it (C operand of their first MFMA), so dP^T - delta costs no vector instruction per tile.
    // Not at d = 64: there the kernel is built for four workgroups per CU (128 registers) and the
    // 16 extra registers would spill (measured: 12 -> 332 bytes of scratch per lane, four times slower).
    constexpr bool kDeltaInAcc = D >= 128;
    f32x16 ndl[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
#pragma unroll
        for (int i = 0; i < 16; ++i) ndl[t][i] = kDeltaInAcc ? -dl[t] : 0.f;
    }
    FragOffsets<D> lane_offsets;
    lane_offsets.init(lane);
    FragAddrs<D> fo;
    fo.init(lane_offsets);
    wait_direct_loads();
    __syncthreads();

    // One streamed tile.  `masked` selects the copy of the body that applies the causal / tail
    // bound; the other copy has no mask arithmetic at all.  Every K, V and K^T fragment read
    // from LDS feeds QT MFMAs (one per resident query tile).
    // Wave priorities per phase (see the forward kernel): score MFMAs, then the dQ MFMAs, the
    // exponentials last.
    constexpr int kPrioScores = 2, kPrioSoftmax = 0, kPrioDq = 1;
    auto tile = [&](auto stage_off, int j0, auto masked) {
        const int k_off = stage_off;  // K tile; the V tile follows it
        // the two 32-key halves one after the other: half the score registers live at a time
#pragma unroll
        for (int T = 0; T < 2; ++T) {
            __builtin_amdgcn_s_setprio(kPrioScores);
            f32x16 st[QT], dpt[QT];
#pragma unroll
            for (int t = 0; t < QT; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i) st[t][i] = 0.f;
#pragma unroll
            for (int t = 0; t < QT; ++t) dpt[t] = ndl[t];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {  // independent accumulation chains, interleaved
                const bf16x8 kfr = fo.frag(smem, k_off, 32 * T, ks);
                const bf16x8 vfr = fo.frag(smem, k_off + kTileBytes, 32 * T, ks);
#pragma unroll
                for (int t = 0; t < QT; ++t) {
                    st[t] = mfma32(kfr, qf[t][ks], st[t]);
                    dpt[t] = mfma32(vfr, gf[t][ks], dpt[t]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(kPrioSoftmax);
            bf16x8 dsb[QT][2], kt[2][MT];
#pragma unroll
            for (int t = 0; t < QT; ++t) {
                // key j0 + 32T + 8g + 4h + r is visible iff 8g + r <= lim (one per-lane bound)
                const int lim = (p.causal ? min(q[t], p.n - 1) : p.n - 1) - j0 - 32 * T - 4 * h;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float pv = __builtin_amdgcn_exp2f(st[t][i] * c - lse2[t]);
                    if constexpr (decltype(masked)::value) pv = (8 * (i >> 2) + (i & 3) > lim) ? 0.f : pv;
                    dpt[t][i] = kDeltaInAcc ? pv * dpt[t][i] : pv * (dpt[t][i] - dl[t]);
                }
#pragma unroll
                for (int ss = 0; ss < 2; ++ss) dsb[t][ss] = acc_to_operand(dpt[t], ss);
            }
            __builtin_amdgcn_s_setprio(kPrioDq);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) kt[0][mt] = fo.frag_t(smem, k_off, mt, 32 * T);
#pragma unroll
            for (int ss = 0; ss < 2; ++ss) {  // K^T fragments of the next 16 keys requested ahead
                if (ss == 0) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) kt[1][mt] = fo.frag_t(smem, k_off, mt, 32 * T + 16);
                }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int t = 0; t < QT; ++t) dq[t][mt] = mfma32(kt[ss][mt], dsb[t][ss], dq[t][mt]);
            }
            __builtin_amdgcn_sched_barrier(0);  // the next half starts after this one is issued
        }
    };
    // Tiles come in ascending key order, so those that need the bound (they straddle the
    // diagonal or the end of the sequence) are the last ones.  Mask-free tiles go two at a time
    // through a body whose LDS stage offsets are compile-time constants (fragment addresses are
    // then a precomputed register plus an immediate); the rest takes the masked body with a
    // run-time stage.  Waves may leave the first loop at different tiles; both loops run the same
    // fetches and barriers.
    auto needs_mask = [&](int j0) { return (p.causal && (j0 + BC - 1 > w0)) || (j0 + BC > p.n); };
    int it = 0;
    for (; it + 2 <= n_it; it += 2) {
        const int ja = j0_next, jb = tile_start(it + 1);
        if (needs_mask(ja) || needs_mask(jb)) break;
        j0_next = jb;
        fetch(jb, 1);
        tile(std::integral_constant<int, 0>{}, ja, std::false_type{});
        wait_direct_loads();
        __syncthreads();
        if (it + 2 < n_it) {
            j0_next = tile_start(it + 2);
            fetch(j0_next, 0);
        }
        tile(std::integral_constant<int, kStageBytes>{}, jb, std::false_type{});
        wait_direct_loads();
        __syncthreads();
    }
    for (; it < n_it; ++it) {
        const int j0 = j0_next;
        if (it + 1 < n_it) {
            j0_next = tile_start(it + 1);
            fetch(j0_next, (it + 1) & 1);
        }
        // causal: this wave's last query precedes the tile's first key -> nothing visible
        if (!(p.causal && (w0 + 32 * QT - 1 < j0))) tile((it & 1) * kStageBytes, j0, std::true_type{});
        wait_direct_loads();
        __syncthreads();
    }

#pragma unroll
    for (int t = 0; t < QT; ++t) {
        if (q[t] < p.n) {
            __bf16* row = p.dQ + base + (long)q[t] * ld;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 a;
                    a[0] = pack_bf16(dq[t][mt][4 * g + 0] * p.scale, dq[t][mt][4 * g + 1] * p.scale);
                    a[1] = pack_bf16(dq[t][mt][4 * g + 2] * p.scale, dq[t][mt][4 * g + 3] * p.scale);
                    *reinterpret_cast<u32x2*>(row + 32 * mt + 8 * g + 4 * h) = a;
                }
        }
    }
}

// ------------------------------------------------------------------------------ launchers
void launch_delta(const FusedParams& p, int d, hipStream_t stream) {
    const long lanes = (long)p.batch * p.heads * p.n * (d / 8 < 64 ? d / 8 : 64);
    hipLaunchKernelGGL(delta_kernel, dim3((unsigned)((lanes + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream, p, d);
}

template <int D>
static hipError_t launch_bwd(const FusedParams& p, const int32_t* csr_ptr, const int32_t* csr_idx,
                             const int32_t* csc_ptr, const int32_t* csc_idx, hipStream_t stream, bool dq_only,
                             int32_t* order_scratch, int onepass_keys, float* dq_acc, bool dkdv_only) {
    const int bh = p.batch * p.heads;
    const bool onepass = onepass_keys != 0 && !dq_only;

    constexpr int kv_lds = 2 * (2 * 64 * D * 2) + 2 * 64 * 64 * 2;  // two stages of Q, dO; P and dS
    constexpr int q_lds = 2 * (2 * 64 * D * 2);
    const void* kv_fn = reinterpret_cast<const void*>(bwd_dkdv_kernel<D>);
    // set on every call (the attribute belongs to the current device, and the call is cheap)
    if (!onepass) {
        hipError_t e = hipFuncSetAttribute(kv_fn, hipFuncAttributeMaxDynamicSharedMemorySize, kv_lds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dq_kernel<D, 1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, q_lds);
        if (e != hipSuccess) return e;
    }
    const int blocks128 = (p.n + 127) / 128;
    int32_t* order_q = nullptr;
    int32_t* order_k = nullptr;
    const int masks = p.list_stride ? bh : 1;  // one mask per (batch, head), or one for all
    if (order_scratch && csr_ptr && csc_ptr && masks <= 65535) {  // (grid.y limit; beyond it: ascending order)
        order_q = order_scratch;
        order_k = order_scratch + (long)masks * blocks128;
        int32_t* len = order_scratch + 2L * masks * blocks128;
        const dim3 og((unsigned)((blocks128 + kThreads - 1) / kThreads), (unsigned)masks);
        const bool want_q = !onepass && !dkdv_only, want_k = !dq_only;
        if (blocks128 <= kOrderFusedBlocks) {
            if (want_q || want_k)
                hipLaunchKernelGGL(block_order_fused_kernel, dim3((unsigned)masks, want_q && want_k ? 2u : 1u),
                                   dim3(kThreads), 0, stream, csr_ptr, csr_idx, csc_ptr, csc_idx, blocks128, p.causal,
                                   order_q, order_k, want_q ? 0 : 1);
        } else {
            if (want_q) {
                hipLaunchKernelGGL(block_len_kernel, og, dim3(kThreads), 0, stream, csr_ptr, csr_idx, blocks128, p.causal, 0, len);
                hipLaunchKernelGGL(block_order_kernel, og, dim3(kThreads), 0, stream, len, blocks128, order_q);
            }
            if (want_k) {
                hipLaunchKernelGGL(block_len_kernel, og, dim3(kThreads), 0, stream, csc_ptr, csc_idx, blocks128, p.causal, 1, len);
                hipLaunchKernelGGL(block_order_kernel, og, dim3(kThreads), 0, stream, len, blocks128, order_k);
            }
        }
    }
    if (onepass) {
        FusedParams pk = p;
        pk.list_ptr = csc_ptr;
        pk.list_idx = csc_idx;
        pk.order = order_k;
        pk.order_stride = p.list_stride ? blocks128 : 0;
        return launch_bwd_onepass(D, onepass_keys, pk, dq_acc, stream);
    }
    FusedParams pq = p;
    pq.list_ptr = csr_ptr;
    pq.list_idx = csr_idx;
    pq.order = order_q;
    pq.order_stride = p.list_stride ? blocks128 : 0;
    // One query tile per wave and two workgroups per CU.  (QT = 2, i.e. one wave per SIMD with every
    // LDS fragment feeding two MFMAs, halves the LDS traffic but measured 20 % slower at d = 128:
    // with a single wave per SIMD the softmax arithmetic no longer overlaps another wave's MFMAs.)
    if (!dkdv_only)
        hipLaunchKernelGGL((bwd_dq_kernel<D, 1>), dim3((unsigned)(blocks128 * bh)), dim3(kThreads), q_lds, stream, pq);
    if (dq_only) return hipGetLastError();
    FusedParams pk = p;
    pk.list_ptr = csc_ptr;
    pk.list_idx = csc_idx;
    pk.order = order_k;
    pk.order_stride = p.list_stride ? blocks128 : 0;
    const int key_blocks = order_k ? 2 * blocks128 : (p.n + 63) / 64;
    hipLaunchKernelGGL(bwd_dkdv_kernel<D>, dim3((unsigned)(key_blocks * bh)), dim3(kThreads), kv_lds, stream, pk);
    return hipGetLastError();
}

hipError_t launch_bwd_fused(int d, const FusedParams& p, const int32_t* csr_ptr, const int32_t* csr_idx,
                            const int32_t* csc_ptr, const int32_t* csc_idx, hipStream_t stream, bool dq_only,
                            int32_t* order_scratch, int onepass_keys, float* dq_acc, bool dkdv_only) {
    switch (d) {
        case 64: return launch_bwd<64>(p, csr_ptr, csr_idx, csc_ptr, csc_idx, stream, dq_only, order_scratch, onepass_keys, dq_acc, dkdv_only);
        case 128: return launch_bwd<128>(p, csr_ptr, csr_idx, csc_ptr, csc_idx, stream, dq_only, order_scratch, onepass_keys, dq_acc, dkdv_only);
        case 256: return launch_bwd<256>(p, csr_ptr, csr_idx, csc_ptr, csc_idx, stream, dq_only, order_scratch, 0, nullptr, dkdv_only);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace attn
