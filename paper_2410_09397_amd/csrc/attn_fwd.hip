// Fused forward for d <= 256 (d = 256: one wave per SIMD): O = diag(l)^{-1} exp(scale Q K^T) V and LSE = log l (forward
// definition, Sec. 3.1; A, l, f, O of App. B.4), evaluated per block of 128 queries with a
// running maximum so that no n x n matrix is formed.  The paper gives no forward algorithm;
// the streaming-softmax tiling is prior art, the kernel is written for gfx950.
#include <type_traits>

#include "attn_common.hpp"
#include "attn_internal.hpp"

namespace attn {

// Wave w owns queries i0 + 32w .. +31 (Q rows resident in registers as B operands).
// Per key tile (64 keys, two halves T):
//   S^T[T] = K_T Q_w^T                 accumulator: lane <-> query, register <-> key
//   m, l   : running row maximum and sum, one scalar per lane (both lane halves of a query
//            see the same maximum; their partial sums are added at the end)
//   O_w^T += V_T^T P^T                 V^T from transposed LDS reads, P^T straight from registers
// Workgroups per CU: 4 at d = 64 (128 registers per lane; measured 5-6 % faster than 3 per CU at 134
// registers on a grid of 1024 workgroups), 2 at d = 128, 1 at d = 256.
template <int D>
__global__ void __launch_bounds__(kThreads, D == 64 ? 4 : (D <= 128 ? 2 : 1)) fwd_kernel(FusedParams p) {
    constexpr int BR = 128, BC = 64, KS = D / 16, MT = D / 32;
    constexpr int kTileBytes = BC * D * 2;
    constexpr int kStageBytes = 2 * kTileBytes;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, uniform
    const int q_blocks = (p.n + BR - 1) / BR;
    int bh, blk;
    decode_block(blockIdx.x, q_blocks, p.batch * p.heads, bh, blk);
    const int ib = p.causal ? q_blocks - 1 - blk : blk;  // causal: longest rows first
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const long ld = p.stride_n;
    const int i0 = ib * BR;

    int n_it, lp0 = 0;
    if (p.list_ptr) {
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
    // the first tile is requested before the resident Q rows, so that the two latencies overlap
    int j0_next = n_it > 0 ? tile_start(0) : 0;
    if (n_it > 0) fetch(j0_next, 0);

    const int q = i0 + 32 * w + l32;
    const bool q_ok = q < p.n;
    bf16x8 qf[KS];
    {
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = zero;
            if (q_ok) qf[ks] = *reinterpret_cast<const bf16x8*>(p.Q + base + (long)q * ld + 16 * ks + 8 * h);
        }
    }

    f32x16 o[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[mt][i] = 0.f;
    float m_run = -__builtin_inff();  // running maximum of scale * log2(e) * s
    float l_run = 0.f;                // this lane's share of sum exp2(scaled s - m_run)

    // Scores are kept raw in the accumulators and scaled inside the exponential: with
    // cs = |scale| log2(e) > 0 the row maximum commutes with the scaling.  A negative scale is
    // moved into Q (sign flip of the resident fragments), a zero scale becomes a denormal-sized
    // positive one so that masked (-inf) scores stay -inf.
    const float cs = fmaxf(fabsf(p.scale) * kLog2e, 1.17549435e-38f);
    if (p.scale < 0.f) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 v = __builtin_bit_cast(u32x4, qf[ks]);
            v ^= 0x80008000u;
            qf[ks] = __builtin_bit_cast(bf16x8, v);
        }
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) settle(qf[ks]);
    FragOffsets<D> lane_offsets;
    lane_offsets.init(lane);
    FragAddrs<D> fo;
    fo.init(lane_offsets);
    wait_direct_loads();
    __syncthreads();

    // One streamed tile; `masked` selects the copy of the body that applies the causal / tail bound.
    // Wave priorities: the two waves that share a SIMD tend to fall into step (they compete for
    // the same matrix pipe, so both reach the end of a phase, and its LDS latency, together).
    // Ranking the phases - score MFMAs first, then the PV MFMAs, the exponentials last - lets one
    // wave run ahead while the other fills the gaps (measured: 5-7 % faster at d = 128).
    constexpr int kPrioScores = 2, kPrioSoftmax = 0, kPrioPV = 1;
    auto tile = [&](auto stage_off, int j0, auto masked) {
        const int k_off = stage_off;  // K tile; the V tile follows it
        __builtin_amdgcn_s_setprio(kPrioScores);
        f32x16 st[2];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int i = 0; i < 16; ++i) st[T][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int T = 0; T < 2; ++T) st[T] = mfma32(fo.frag(smem, k_off, 32 * T, ks), qf[ks], st[T]);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(kPrioSoftmax);
        if constexpr (decltype(masked)::value) {
            // key j0 + 32T + 8g + 4h + r is visible iff 32T + 8g + r <= lim (one per-lane bound)
            const int lim = (p.causal ? min(q, p.n - 1) : p.n - 1) - j0 - 4 * h;
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    st[T][i] = (32 * T + 8 * (i >> 2) + (i & 3) > lim) ? -__builtin_inff() : st[T][i];
        }
        // maximum (IEEE-754-2019, v_maximum3_f32) instead of fmaxf: for fmaxf the compiler first
        // canonicalises every accumulator value (one extra VALU instruction each, for signalling
        // NaNs).  Two chains of three-input maxima over the 32 values of this lane.
        float mxa = max3(st[0][0], st[0][1], st[0][2]), mxb = max3(st[1][0], st[1][1], st[1][2]);
#pragma unroll
        for (int i = 3; i < 15; i += 2) {
            mxa = max3(mxa, st[0][i], st[0][i + 1]);
            mxb = max3(mxb, st[1][i], st[1][i + 1]);
        }
        float mx = max3(mxa, mxb, __builtin_elementwise_maximum(st[0][15], st[1][15]));
        mx = __builtin_elementwise_maximum(mx, __shfl_xor(mx, 32, 64));
        // The reference point m_run of the exponentials only has to be close to the row maximum,
        // not equal to it: it moves (and O, l are rescaled) only when the maximum has grown by
        // more than kSlack, so p = exp2(s - m_run) stays below 2^kSlack and the final O / l and
        // m_run + log2(l) are unchanged.  After the first tiles of a row this almost never
        // happens, which saves the 16 MT + 1 multiplications per lane and tile of the rescaling.
        constexpr float kSlack = 8.f;
        const float cand = mx * cs;
        const bool grow = cand > m_run + kSlack;  // also the first finite maximum after -inf
        const float m_new = grow ? cand : m_run;
        const float m_use = (m_new == -__builtin_inff()) ? 0.f : m_new;  // nothing visible yet
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {  // some row's reference moved: rescale
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
            l_run *= alpha;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[mt][i] *= alpha;
        }
        m_run = m_new;
        float sum = 0.f;
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float pv = __builtin_amdgcn_exp2f(fmaf(st[T][i], cs, -m_use));
                st[T][i] = pv;
                sum += pv;
            }
        l_run += sum;
        bf16x8 pb[2][2];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int ss = 0; ss < 2; ++ss) pb[T][ss] = acc_to_operand(st[T], ss);
        __builtin_amdgcn_s_setprio(kPrioPV);
        // O^T += V^T P^T in four groups of 16 keys; the V^T fragments of the next group are
        // requested before the MFMAs of the current one so that LDS latency hides behind them
        bf16x8 va[2][MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) va[0][mt] = fo.frag_t(smem, k_off + kTileBytes, mt, 0);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (g + 1 < 4) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    va[(g + 1) & 1][mt] = fo.frag_t(smem, k_off + kTileBytes, mt, 16 * (g + 1));
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) o[mt] = mfma32(va[g & 1][mt], pb[g >> 1][g & 1], o[mt]);
        }
    };
    // Tiles come in ascending key order, so those that need the bound (they straddle the
    // diagonal or the end of the sequence) are the last ones.  Mask-free tiles go two at a time
    // through a body whose LDS stage offsets are compile-time constants (fragment addresses are
    // then a precomputed register plus an immediate: no vector arithmetic per fetch); the rest
    // takes the masked body with a run-time stage.  Waves may leave the first loop at different
    // tiles; both loops run the same fetches and barriers.
    auto needs_mask = [&](int j0) { return (p.causal && (j0 + BC - 1 > i0 + 32 * w)) || (j0 + BC > p.n); };
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
        if (!(p.causal && (i0 + 32 * w + 31 < j0))) tile((it & 1) * kStageBytes, j0, std::true_type{});
        wait_direct_loads();
        __syncthreads();
    }

    const float l = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = l > 0.f ? 1.f / l : 0.f;
    if (q_ok) {
        __bf16* row = p.Oout + base + (long)q * ld;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 a;
                a[0] = pack_bf16(o[mt][4 * g + 0] * inv, o[mt][4 * g + 1] * inv);
                a[1] = pack_bf16(o[mt][4 * g + 2] * inv, o[mt][4 * g + 3] * inv);
                *reinterpret_cast<u32x2*>(row + 32 * mt + 8 * g + 4 * h) = a;
            }
        if (h == 0)
            p.LSEout[(long)bh * p.n + q] = l > 0.f ? (m_run + __builtin_amdgcn_logf(l)) * kLn2 : -__builtin_inff();
    }
}

template <int D>
static hipError_t launch_fwd(const FusedParams& p, const int32_t* csr_ptr, const int32_t* csr_idx,
                             hipStream_t stream) {
    constexpr int lds = 2 * (2 * 64 * D * 2);
    // set on every call: the attribute belongs to the current device, and the call is cheap
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fwd_kernel<D>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    FusedParams pf = p;
    pf.list_ptr = csr_ptr;
    pf.list_idx = csr_idx;
    const int blocks = (p.n + 127) / 128 * p.batch * p.heads;
    hipLaunchKernelGGL(fwd_kernel<D>, dim3((unsigned)blocks), dim3(kThreads), lds, stream, pf);
    return hipGetLastError();
}

hipError_t launch_fwd_fused(int d, const FusedParams& p, const int32_t* csr_ptr, const int32_t* csr_idx,
                            hipStream_t stream) {
    switch (d) {
        case 64: return launch_fwd<64>(p, csr_ptr, csr_idx, stream);
        case 128: return launch_fwd<128>(p, csr_ptr, csr_idx, stream);
        case 256: return launch_fwd<256>(p, csr_ptr, csr_idx, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace attn
