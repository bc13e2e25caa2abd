// One-pass backward for d in {64, 128}: every visible (query tile, key block) pair is visited once
// and all five products of the pair are formed there (10 d multiply-adds per pair, nothing is
// recomputed).  This is the inner body of the paper's large-cache phase-2 algorithm (App. D) with
// the key block as the resident operand:
//   q = dO h^T, A = S A_2^T, f = exp(A) / l, p = f o q - diag(v) f       (App. B.4)
//   dV_j += f^T dO_i,  dK_j += p^T Q_i     accumulate in the registers of the workgroup that owns
//                                          the key block (no atomics, bit-reproducible)
//   dQ_i += p A_2j                         the `p A_2` factor of the backward gradient (Sec. 3.1):
//                                          a sum over key blocks, i.e. over workgroups; each
//                                          workgroup adds its 64 x d tile with fp32 atomic adds
//                                          into a zeroed [batch * heads, n, d] array
// Three launches: bwd_prep_kernel (v = rowsum(dO o O), and zeroes the fp32 dQ array),
// bwd_onepass_kernel, bwd_dq_store_kernel (scale, round to bf16, strided store).
// The order of the atomic additions is not fixed, so dQ can differ in its last bits from run to
// run; dK and dV cannot.
#include <type_traits>

#include "attn_common.hpp"
#include "attn_internal.hpp"

namespace attn {

// ------------------------------------------------------------------------ prep: v and zero
// min(d / 8, 64) consecutive lanes share one row (16-byte chunks of O and dO); each lane also
// clears the 32 bytes of the fp32 dQ array that face its chunk.
__global__ void __launch_bounds__(kThreads) bwd_prep_kernel(FusedParams p, int d, float* dq_acc) {
    const int cpr = d >> 3;
    const int lpr = cpr < 64 ? cpr : 64;
    const long rows = (long)p.batch * p.heads * p.n;
    const long f = (long)blockIdx.x * kThreads + threadIdx.x;
    const long r = f / lpr;
    const int c = (int)(f % lpr);
    float acc = 0.f;
    if (r < rows) {
        const int bh = (int)(r / p.n), i = (int)(r % p.n);
        const long off = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h + (long)i * p.stride_n;
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        for (int cc = c; cc < cpr; cc += lpr) {
            const bf16x8 o = *reinterpret_cast<const bf16x8*>(p.O + off + 8 * cc);
            const bf16x8 g = *reinterpret_cast<const bf16x8*>(p.dO + off + 8 * cc);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += (float)o[e] * (float)g[e];
            f32x4* z = reinterpret_cast<f32x4*>(dq_acc + r * d + 8 * cc);
            z[0] = zero;
            z[1] = zero;
        }
    }
    for (int m = lpr >> 1; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
    if (r < rows && c == 0) p.delta[r] = acc;
}

// ------------------------------------------------------------------------ dQ: fp32 -> bf16
// One lane per 8 elements: dQ = bf16(scale * sum).
__global__ void __launch_bounds__(kThreads) bwd_dq_store_kernel(FusedParams p, int d, const float* dq_acc) {
    const int cpr = d >> 3;
    const long chunks = (long)p.batch * p.heads * p.n * cpr;
    const long f = (long)blockIdx.x * kThreads + threadIdx.x;
    if (f >= chunks) return;
    const long r = f / cpr;
    const int c = (int)(f % cpr);
    const int bh = (int)(r / p.n), i = (int)(r % p.n);
    const long off = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h + (long)i * p.stride_n;
    const f32x4* src = reinterpret_cast<const f32x4*>(dq_acc + r * d + 8 * c);
    const f32x4 a = src[0], b = src[1];
    u32x4 o;
    o[0] = pack_bf16(a[0] * p.scale, a[1] * p.scale);
    o[1] = pack_bf16(a[2] * p.scale, a[3] * p.scale);
    o[2] = pack_bf16(b[0] * p.scale, b[1] * p.scale);
    o[3] = pack_bf16(b[2] * p.scale, b[3] * p.scale);
    *reinterpret_cast<u32x4*>(p.dQ + off + 8 * c) = o;
}

// ----------------------------------------------------------------------------- one pass
// A workgroup of eight waves owns BC = 32 NKB keys (NKB = 4: 128 keys; NKB = 2: 64) and streams
// 64-query tiles, last tile first: under the causal rule every workgroup of a head then starts at the
// same query tile and walks towards its own diagonal, so the workgroups that run together read the
// same Q and dO rows and add into the same dQ rows at about the same time (they share an L2: all
// workgroups of a (batch, head) pair run on one XCD).
// The waves split into two roles that work on consecutive tiles at the same time, one wave of each
// role per SIMD, so that one role's exponentials run beside the other role's MFMAs:
//   waves 0-3, tile t:     S^T and dP^T for one 32-key block (resident K / V fragments as A operands;
//                          lane <-> query, so LSE and v are per-lane scalars), f and p, written to
//                          LDS as bf16 [query][key] tiles (two buffers, t even / odd); these waves
//                          also issue the global -> LDS copies of the Q and dO tiles (three stages:
//                          tile t + 1 arrives while tile t is used here and tile t - 1 below);
//   waves 4-7, tile t - 1: dQ tile = p A_2j (p row-major from LDS as A operand, K^T fragments as B
//                          operand in registers), added to the fp32 dQ array at once so that the
//                          additions are under way during the rest; then dV^T += dO^T f or
//                          dK^T += Q^T p for one half of d and all keys of the block (MH x NKB
//                          accumulators, all operands read with transposing LDS loads).
// One workgroup barrier per tile hands tile t from the first role to the second.
template <int D, int NKB>
__global__ void __launch_bounds__(512, 1) bwd_onepass_kernel(FusedParams p, float* dq_acc) {
    constexpr int BR = 64, BC = 32 * NKB, KS = D / 16, MT = D / 32, MH = MT / 2;
    constexpr int NQ = NKB / 2;       // 32-query blocks per wave of the first role
    constexpr int KB = BC / 16;       // k-steps of the dQ product
    constexpr int NB = MT / 2;        // dQ blocks (32 queries x 32 columns) per wave of the second role
    constexpr int kTileBytes = BR * D * 2;
    constexpr int kStageBytes = 2 * kTileBytes;  // Q tile, dO tile
    constexpr int kPBytes = BR * BC * 2;
    constexpr int kPOff = 3 * kStageBytes;       // two buffers of (f tile, p tile) follow the three stages
    constexpr bool kSwap = BC == 64;  // 128-byte rows: the two 8-byte halves of a chunk swap in odd rows (see p_wr)
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    constexpr int kSub = 128 / BC;  // owned blocks per 128-key block of a mask
    const int blocks128 = (p.n + 127) / 128;
    const int key_blocks = p.order ? kSub * blocks128 : (p.n + BC - 1) / BC;
    int bh, j;
    decode_block(blockIdx.x, key_blocks, p.batch * p.heads, bh, j);
    if (p.order) {
        j = kSub * p.order[(long)bh * p.order_stride + j / kSub] + j % kSub;
        if (j * BC >= p.n) return;
    }
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const long ld = p.stride_n;
    const int j0 = j * BC;

    // the streamed query tiles: entry r of the ascending sequence, taken from the last one down
    int n_it, t0 = 0, lp0 = 0;
    if (p.list_ptr) {
        const int32_t* lptr = p.list_ptr + (long)bh * p.list_stride;
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
    const int r_top = n_it - 1;
    auto tile_start = [&](int it) -> int { return tile_start_row<BR>(p.list_idx, lp0, t0, r_top - it); };
    // the second 64 keys of a mask's diagonal block see nothing of that block's first 64 queries
    if (p.causal && n_it > 0 && tile_start(n_it - 1) + BR - 1 < j0) --n_it;

    FragOffsets<D> fo;   // Q / dO tiles
    FragOffsets<BC> fp;  // f / p tiles
    fo.init(lane);
    fp.init(lane);

    if (w < 4) {
        // ================================================================ first role: f and p
        const int kb = w % NKB, qb0 = (w / NKB) * NQ;
        const float* lse_g = p.LSE + (long)bh * p.n;
        const float* delta_g = p.delta + (long)bh * p.n;
        const int key = j0 + 32 * kb + l32;
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
        const float c = p.scale * kLog2e;
        float lse_raw[NQ], delta_raw[NQ];
        bool row_ok[NQ];
        TileLoader<D, BR, 4> loader;
        loader.init(tid, ld);
        auto fetch_rows = [&](int i0) {
#pragma unroll
            for (int t = 0; t < NQ; ++t) {
                const int q = i0 + 32 * (qb0 + t) + l32;
                row_ok[t] = q < p.n;
                lse_raw[t] = lse_g[min(q, p.n - 1)];
                delta_raw[t] = delta_g[min(q, p.n - 1)];
            }
        };
        auto fetch = [&](int i0, int stage_off) {
            char* s = smem + stage_off;
            loader.load(p.Q + base, ld, i0, p.n, s, tid);
            loader.load(p.dO + base, ld, i0, p.n, s + kTileBytes, tid);
            fetch_rows(i0);
        };
        int i0_next = n_it > 0 ? tile_start(0) : 0;
        if (n_it > 0) fetch(i0_next, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            settle(kf[ks]);
            settle(vf[ks]);
        }
        wait_direct_loads();
        __builtin_amdgcn_s_barrier();  // tile 0 is in LDS

        // This lane's 8-byte slot of group g in the [query][key] tiles: p_wr ^ (g << 4).  With
        // 128-byte rows (BC = 64) rows 2k and 2k+1 share their swizzle term, so the 16 lanes that
        // write together would hit every bank twice: there the two 8-byte halves of a chunk swap
        // places in odd rows, and every read of those tiles applies the same swap.
        const int p_wr = tile_off<BC>(32 * qb0 + l32, 4 * kb) + 8 * (kSwap ? (h ^ (l32 & 1)) : h);
        const int q_rm0 = fo.rm0 + 32 * qb0 * (D * 2);

        auto tile = [&](int it, int i0, auto masked) {
            const int st = (it % 3) * kStageBytes;                  // this tile's Q / dO stage
            const int pb = kPOff + (it & 1) * (2 * kPBytes);        // this tile's f / p buffer
            float lse_cur[NQ], delta_cur[NQ];
#pragma unroll
            for (int t = 0; t < NQ; ++t) {
                lse_cur[t] = row_ok[t] ? lse_raw[t] * kLog2e : __builtin_inff();
                delta_cur[t] = row_ok[t] ? delta_raw[t] : 0.f;
            }
            // the copies of the next tile go into the stage that the second role left two barriers
            // ago; whole tiles are copied one instruction per k-step between the MFMAs
            bool spread = false;
            const __bf16* next_q = nullptr;
            const __bf16* next_g = nullptr;
            char* next_stage = smem + ((it + 1) % 3) * kStageBytes;
            if (it + 1 < n_it) {
                i0_next = tile_start(it + 1);
                spread = i0_next + BR <= p.n;
                if (spread) {
                    next_q = p.Q + base + (long)i0_next * ld;
                    next_g = p.dO + base + (long)i0_next * ld;
                    fetch_rows(i0_next);
                } else {
                    fetch(i0_next, ((it + 1) % 3) * kStageBytes);
                }
            }
            __builtin_amdgcn_s_setprio(2);
            f32x16 s[NQ], dp[NQ];
#pragma unroll
            for (int t = 0; t < NQ; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i) { s[t][i] = 0.f; dp[t][i] = 0.f; }
            {
                constexpr int kAhead = 2;
                bf16x8 fq[KS][NQ], fg[KS][NQ];
                auto request = [&](int ks) {
                    const int a = (q_rm0 ^ (ks << 5)) + st;
#pragma unroll
                    for (int t = 0; t < NQ; ++t) {
                        fq[ks][t] = *reinterpret_cast<const bf16x8*>(smem + a + 32 * t * (D * 2));
                        fg[ks][t] = *reinterpret_cast<const bf16x8*>(smem + a + 32 * t * (D * 2) + kTileBytes);
                    }
                };
#pragma unroll
                for (int ks = 0; ks < kAhead; ++ks) request(ks);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    __builtin_amdgcn_sched_barrier(0);
                    if (ks + kAhead < KS) request(ks + kAhead);
#pragma unroll
                    for (int t = 0; t < NQ; ++t) {
                        s[t] = mfma32(kf[ks], fq[ks][t], s[t]);
                        dp[t] = mfma32(vf[ks], fg[ks][t], dp[t]);
                    }
                    if (spread) {
                        constexpr int kPer = TileLoader<D, BR, 4>::kInst;
                        static_assert(2 * kPer <= KS, "at most one copy per k-step");
                        if (ks < kPer) loader.load_one(ks, next_q, next_stage);
                        else if (ks < 2 * kPer) loader.load_one(ks - kPer, next_g, next_stage + kTileBytes);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int t = 0; t < NQ; ++t) {
                // key j0 + 32 kb + 8g + 4h + r is visible to this lane's query iff 8g + r <= lim
                const int lim = p.causal ? i0 + 32 * (qb0 + t) + l32 - j0 - 32 * kb - 4 * h : 0x7fffffff;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float pv[4], dsv[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i = 4 * g + r;
                        float v = __builtin_amdgcn_exp2f(s[t][i] * c - lse_cur[t]);
                        if constexpr (decltype(masked)::value) v = (8 * g + r > lim) ? 0.f : v;
                        pv[r] = v;
                        dsv[r] = v * (dp[t][i] - delta_cur[t]);
                    }
                    u32x2 a, b;
                    a[0] = pack_bf16(pv[0], pv[1]);
                    a[1] = pack_bf16(pv[2], pv[3]);
                    b[0] = pack_bf16(dsv[0], dsv[1]);
                    b[1] = pack_bf16(dsv[2], dsv[3]);
                    const int slot = pb + (p_wr ^ (g << 4)) + 32 * t * (BC * 2);
                    *reinterpret_cast<u32x2*>(smem + slot) = a;
                    *reinterpret_cast<u32x2*>(smem + slot + kPBytes) = b;
                }
            }
            // f, p of this tile and the copies of the next tile are complete: hand over
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        };
        // descending query order: a tile that reaches past n comes first, those that straddle the
        // diagonal last; only they take the body with the bound
        for (int it = 0; it < n_it; ++it) {
            const int i0 = i0_next;
            if (p.causal && i0 < j0 + BC - 1) tile(it, i0, std::true_type{});
            else tile(it, i0, std::false_type{});
        }
        return;
    }

    // ============================================================ second role: dQ, dK, dV
    const int cw = w - 4;
    const int which = cw & 1, dh = cw >> 1;           // dV (0) or dK (1); half of d
    const int db = cw % MT, qb0 = (cw / MT) * NB;     // dQ: 32 columns of d, first 32-query block
    float* dq_head = dq_acc + (long)bh * p.n * D;
    // K^T fragments (B operand of p A_2j): column 32 db + l32 of keys j0 + 16 ks + 8 h .. + 7.  Keys
    // past n read the last row and are zeroed afterwards (all loads are issued before any is used).
    bf16x8 ktf[KB];
    {
        const unsigned short* kcol = reinterpret_cast<const unsigned short*>(p.K) + base + 32 * db + l32;
        unsigned short e[KB][8];
#pragma unroll
        for (int ks = 0; ks < KB; ++ks)
#pragma unroll
            for (int t = 0; t < 8; ++t) e[ks][t] = kcol[(long)min(j0 + 16 * ks + 8 * h + t, p.n - 1) * ld];
#pragma unroll
        for (int ks = 0; ks < KB; ++ks) {
            u32x4 r;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int kk = j0 + 16 * ks + 8 * h + 2 * t;
                const unsigned lo = kk < p.n ? e[ks][2 * t] : 0u, hi = kk + 1 < p.n ? e[ks][2 * t + 1] : 0u;
                r[t] = lo | (hi << 16);
            }
            ktf[ks] = __builtin_bit_cast(bf16x8, r);
        }
    }
    f32x16 acc[MH][NKB];
#pragma unroll
    for (int m = 0; m < MH; ++m)
#pragma unroll
        for (int kt = 0; kt < NKB; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][kt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KB; ++ks) settle(ktf[ks]);
    __builtin_amdgcn_s_barrier();  // matches the first role's "tile 0 is in LDS"

    if (kSwap) fp.tr0 ^= (((lane & 15) >> 2) & 1) << 3;
    // row-major fetch of p (A operand of the dQ product): row l32 of a 32-query block, chunk h
    const int ds_rm = kPBytes + fp.rm0 + (kSwap ? 8 * (l32 & 1) : 0) + qb0 * 32 * (BC * 2);
    const int a_tr0 = fo.tr0 + (which == 0 ? kTileBytes : 0);  // dO^T (dV) or Q^T (dK)
    const int b_tr0 = fp.tr0 + (which == 0 ? 0 : kPBytes);     // f (dV) or p (dK)
    // dQ rows of this lane: query 32 (qb0 + b) + 8 (i / 4) + 4 h + i % 4 of the tile, column 32 db + l32
    const int dq_lane = (32 * qb0 + 4 * h) * D + 32 * db + l32;
    __builtin_amdgcn_s_setprio(1);

    for (int it = 0; it < n_it; ++it) {
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // tile `it` is ready
        const int i0 = tile_start(it);
        const int st = (it % 3) * kStageBytes;
        const int pb = kPOff + (it & 1) * (2 * kPBytes);
        {
            // ---- dQ tile = p A_2j, added to the fp32 array
            f32x16 dq[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) dq[b][i] = 0.f;
            bf16x8 pf[KB][NB];
            auto request = [&](int ks) {
                const int a0 = (ds_rm ^ (ks << 5)) + pb;
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    if constexpr (kSwap) {
                        const u32x2 lo = *reinterpret_cast<const u32x2*>(smem + a0 + b * 32 * (BC * 2));
                        const u32x2 hi = *reinterpret_cast<const u32x2*>(smem + (a0 ^ 8) + b * 32 * (BC * 2));
                        const u32x4 r = {lo[0], lo[1], hi[0], hi[1]};
                        pf[ks][b] = __builtin_bit_cast(bf16x8, r);
                    } else {
                        pf[ks][b] = *reinterpret_cast<const bf16x8*>(smem + a0 + b * 32 * (BC * 2));
                    }
                }
            };
            constexpr int kAhead = 2;
#pragma unroll
            for (int ks = 0; ks < kAhead; ++ks) request(ks);
#pragma unroll
            for (int ks = 0; ks < KB; ++ks) {
                __builtin_amdgcn_sched_barrier(0);
                if (ks + kAhead < KB) request(ks + kAhead);
#pragma unroll
                for (int b = 0; b < NB; ++b) dq[b] = mfma32(pf[ks][b], ktf[ks], dq[b]);
            }
            __builtin_amdgcn_sched_barrier(0);
            float* dst = dq_head + (long)i0 * D + dq_lane;
            if (i0 + BR <= p.n) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        __hip_atomic_fetch_add(dst + (32 * b + 8 * (i >> 2) + (i & 3)) * D, dq[b][i], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
            } else {  // the tile reaches past n
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int row = 32 * b + 8 * (i >> 2) + (i & 3);  // + 32 qb0 + 4 h: in dq_lane
                        if (i0 + 32 * qb0 + 4 * h + row < p.n)
                            __hip_atomic_fetch_add(dst + row * D, dq[b][i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        {
            // ---- dV^T += dO^T f (which = 0) or dK^T += Q^T p (which = 1)
            bf16x8 at[2][MH], bt[2][NKB];
            auto request = [&](int ks) {
#pragma unroll
                for (int m = 0; m < MH; ++m) {
                    const int a = (a_tr0 ^ ((MH * dh + m) << 6)) + st;
                    at[ks & 1][m] = FragOffsets<D>::read_t(smem, a, a ^ 32, 16 * ks);
                }
#pragma unroll
                for (int kt = 0; kt < NKB; ++kt) {
                    const int b = (b_tr0 ^ (kt << 6)) + pb;
                    bt[ks & 1][kt] = FragOffsets<BC>::read_t(smem, b, b ^ 32, 16 * ks);
                }
            };
            request(0);
#pragma unroll
            for (int ks = 0; ks < BR / 16; ++ks) {
                __builtin_amdgcn_sched_barrier(0);
                if (ks + 1 < BR / 16) request(ks + 1);
#pragma unroll
                for (int m = 0; m < MH; ++m)
#pragma unroll
                    for (int kk = 0; kk < NKB; ++kk) {
                        const int kt = (m & 1) ? NKB - 1 - kk : kk;  // consecutive MFMAs share an operand
                        acc[m][kt] = mfma32(at[ks & 1][m], bt[ks & 1][kt], acc[m][kt]);
                    }
            }
        }
    }

    const float f = which == 0 ? 1.f : p.scale;
#pragma unroll
    for (int kt = 0; kt < NKB; ++kt) {
        const int okey = j0 + 32 * kt + l32;
        if (okey < p.n) {
            __bf16* row = (which == 0 ? p.dV : p.dK) + base + (long)okey * ld + 32 * MH * dh;
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

// ------------------------------------------------------------------------------ launcher
template <int D, int NKB>
static hipError_t launch_onepass_t(const FusedParams& p, float* dq_acc, hipStream_t stream) {
    constexpr int lds = 3 * (2 * 64 * D * 2) + 2 * (2 * 64 * (32 * NKB) * 2);
    const void* fn = reinterpret_cast<const void*>(bwd_onepass_kernel<D, NKB>);
    // set on every call (the attribute belongs to the current device, and the call is cheap)
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    const int bh = p.batch * p.heads;
    const long rows = (long)bh * p.n;
    const int lpr = D / 8 < 64 ? D / 8 : 64;
    hipLaunchKernelGGL(bwd_prep_kernel, dim3((unsigned)((rows * lpr + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       stream, p, D, dq_acc);
    constexpr int BC = 32 * NKB;
    const int blocks128 = (p.n + 127) / 128;
    const int key_blocks = p.order ? (128 / BC) * blocks128 : (p.n + BC - 1) / BC;
    hipLaunchKernelGGL((bwd_onepass_kernel<D, NKB>), dim3((unsigned)(key_blocks * bh)), dim3(512), lds, stream, p,
                       dq_acc);
    hipLaunchKernelGGL(bwd_dq_store_kernel, dim3((unsigned)((rows * (D / 8) + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, stream, p, D, dq_acc);
    return hipGetLastError();
}

hipError_t launch_bwd_onepass(int d, int key_block, const FusedParams& p, float* dq_acc, hipStream_t stream) {
    if (d == 64 && key_block == 64) return launch_onepass_t<64, 2>(p, dq_acc, stream);
    if (d == 64 && key_block == 128) return launch_onepass_t<64, 4>(p, dq_acc, stream);
    if (d == 128 && key_block == 64) return launch_onepass_t<128, 2>(p, dq_acc, stream);
    if (d == 128 && key_block == 128) return launch_onepass_t<128, 4>(p, dq_acc, stream);
    return hipErrorInvalidValue;
}

}  // namespace attn
