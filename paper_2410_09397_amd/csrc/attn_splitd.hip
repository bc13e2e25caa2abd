// Fused backward for head dimensions whose rows no longer fit one wave's registers (d = 512): the
// alternative to the four-phase path of App. C in the small-cache regime.  Nothing n x n leaves the
// chip: this is still the inner body of the large-cache phase-2 algorithm (App. D), with the owned
// block shrunk to 32 rows so that its d-wide operands and accumulators fit, and with the contraction
// over d split over the four waves of the workgroup:
//   wave w holds columns [w d/4, (w+1) d/4) of the owned rows and forms the partial products
//   S^T and dP^T of a 32 x 32 tile over those columns; the partials are exchanged through LDS, each
//   wave sums the quarter of the tile it owns (8 keys x 32 queries), turns it into f and p (App. B.4)
//   and writes them as bf16 [query][key] tiles; then every wave multiplies the whole f / p tile
//   with its own d/4 columns of the streamed tile.
// Two roles (one launch each, both recompute f and p as the two-kernel tiling for d <= 256 does):
//   key owner   (dK, dV): resident K, V fragments, streams Q, dO;  dV^T += dO^T f, dK^T += Q^T p
//   query owner (dQ)    : resident Q, dO fragments, streams K, V;  dQ^T += K^T p^T
// v = rowsum(dO o O) comes from delta_kernel, as on the four-phase path.  No atomics: bit-reproducible.
#include "attn_common.hpp"
#include "attn_internal.hpp"

namespace attn {

namespace {

// [32][32] bf16 tile, 64-byte rows, no swizzle (2 KB: conflicts cost nothing next to the d-wide tiles)
__device__ __forceinline__ int small_off(int row, int col) { return row * 64 + col * 2; }

// B operand with lane <-> column col and k <-> rows in the order of FragOffsets::read_t
// (element t of half h <-> row row16 + 8 (t / 4) + 4 h + t % 4): transposing reads of the small tile.
__device__ __forceinline__ bf16x8 small_frag_t(const char* tile, int row16, int lane) {
    const int s = lane & 15;
    const int row = row16 + 4 * (lane >> 5) + (s >> 2);
    const int col = 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(tile + small_off(row, col)));
    i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(tile + small_off(row + 8, col)));
    typedef short i16x8 __attribute__((ext_vector_type(8)));
    i16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// B operand with lane <-> row and k along the row, in that same k order
// (element t of half h <-> column 16 ks + 8 (t / 4) + 4 h + t % 4).
__device__ __forceinline__ bf16x8 small_frag_perm(const char* tile, int ks, int lane) {
    const int row = lane & 31, h = lane >> 5;
    const u32x2 lo = *reinterpret_cast<const u32x2*>(tile + small_off(row, 16 * ks + 4 * h));
    const u32x2 hi = *reinterpret_cast<const u32x2*>(tile + small_off(row, 16 * ks + 8 + 4 * h));
    const u32x4 r = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, r);
}

}  // namespace

constexpr int kKeyOwner = 0, kQueryOwner = 1;

template <int D, int ROLE>
__global__ void __launch_bounds__(kThreads, 1) bwd_splitd_kernel(FusedParams p) {
    constexpr int BO = 32, BS = 32;            // owned rows, streamed rows per tile
    constexpr int DQ = D / 4, KSQ = DQ / 16, MQ = DQ / 32;  // this wave's columns: k-steps, 32-column blocks
    constexpr int kTileBytes = BS * D * 2;     // one streamed operand tile
    constexpr int kStageBytes = 2 * kTileBytes;
    constexpr int kPartOff = 2 * kStageBytes;  // partial sums: [owner wave][sender 0..2][S, dP][4 registers][64 lanes]
    constexpr int kPartBytes = 4 * 3 * 8 * 64 * 4;
    constexpr int kPOff = kPartOff + kPartBytes, kDsOff = kPOff + 2048;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blocks = (p.n + BO - 1) / BO;
    int bh, blk;
    decode_block(blockIdx.x, blocks, p.batch * p.heads, bh, blk);
    // longest sweeps first under the causal rule: the first key blocks, the last query blocks
    if (ROLE == kQueryOwner && p.causal) blk = blocks - 1 - blk;
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const long ld = p.stride_n;
    const int o0 = blk * BO;  // first owned row
    const float* lse_g = p.LSE + (long)bh * p.n;
    const float* delta_g = p.delta + (long)bh * p.n;

    // streamed tiles: queries from the diagonal on (key owner), keys up to the diagonal (query owner)
    int t_first = 0, n_it;
    if (ROLE == kKeyOwner) {
        t_first = p.causal ? o0 / BS : 0;
        n_it = (p.n + BS - 1) / BS - t_first;
    } else {
        const int end = p.causal ? min(p.n, o0 + BO) : p.n;
        n_it = (end + BS - 1) / BS;
    }
    const __bf16* X = ROLE == kKeyOwner ? p.Q : p.K;   // streamed operands
    const __bf16* Y = ROLE == kKeyOwner ? p.dO : p.V;
    const __bf16* RA = ROLE == kKeyOwner ? p.K : p.Q;  // resident operands
    const __bf16* RB = ROLE == kKeyOwner ? p.V : p.dO;

    TileLoader<D, BS> loader;
    loader.init(tid, ld);
    auto fetch = [&](int r0, int stage) {
        char* s = smem + stage * kStageBytes;
        loader.load(X + base, ld, r0, p.n, s, tid);
        loader.load(Y + base, ld, r0, p.n, s + kTileBytes, tid);
    };
    if (n_it > 0) fetch(t_first * BS, 0);

    // resident fragments: row o0 + l32, columns DQ w + 16 ks + 8 h .. + 7
    const int orow = o0 + l32;
    bf16x8 ra[KSQ], rb[KSQ];
    {
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) {
            ra[ks] = zero;
            rb[ks] = zero;
            if (orow < p.n) {
                ra[ks] = *reinterpret_cast<const bf16x8*>(RA + base + (long)orow * ld + DQ * w + 16 * ks + 8 * h);
                rb[ks] = *reinterpret_cast<const bf16x8*>(RB + base + (long)orow * ld + DQ * w + 16 * ks + 8 * h);
            }
        }
    }
    // accumulators: key owner dV^T and dK^T, query owner dQ^T, for this wave's d / 4 rows and the 32 owned rows
    constexpr int NACC = ROLE == kKeyOwner ? 2 : 1;
    f32x16 acc[NACC][MQ];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int m = 0; m < MQ; ++m)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][m][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KSQ; ++ks) {
        settle(ra[ks]);
        settle(rb[ks]);
    }
    const float c = p.scale * kLog2e;
    // query owner: this lane's query is fixed
    float lse_res = 0.f, delta_res = 0.f;
    if (ROLE == kQueryOwner) {
        lse_res = orow < p.n ? lse_g[orow] * kLog2e : __builtin_inff();
        delta_res = orow < p.n ? delta_g[orow] : 0.f;
        settle(lse_res);
        settle(delta_res);
    }
    FragOffsets<D> fo;
    fo.init(lane);
    wait_direct_loads();
    __syncthreads();

    for (int it = 0; it < n_it; ++it) {
        const int s0 = (t_first + it) * BS;  // first streamed row of this tile
        const int st = (it & 1) * kStageBytes;
        if (it + 1 < n_it) fetch(s0 + BS, (it + 1) & 1);
        // this lane's query and its row scalars
        const int query = ROLE == kKeyOwner ? s0 + l32 : orow;
        float lse2 = lse_res, dl = delta_res;
        if (ROLE == kKeyOwner) {
            lse2 = query < p.n ? lse_g[query] * kLog2e : __builtin_inff();
            dl = query < p.n ? delta_g[query] : 0.f;
        }
        // ---- partial S^T and dP^T over this wave's columns (register <-> key, lane <-> query)
        f32x16 s, dp;
#pragma unroll
        for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) {
            const bf16x8 xf = FragOffsets<D>::read(smem, fo.rm(KSQ * w + ks), st);
            const bf16x8 yf = FragOffsets<D>::read(smem, fo.rm(KSQ * w + ks), st + kTileBytes);
            if (ROLE == kKeyOwner) {  // A = resident keys, B = streamed queries
                s = mfma32(ra[ks], xf, s);
                dp = mfma32(rb[ks], yf, dp);
            } else {                  // A = streamed keys, B = resident queries
                s = mfma32(xf, ra[ks], s);
                dp = mfma32(yf, rb[ks], dp);
            }
        }
        // ---- exchange: registers 4u .. 4u+3 (keys 8u + 4h + r) go to wave u
        float own_s[4], own_dp[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u == w) {
#pragma unroll
                for (int r = 0; r < 4; ++r) { own_s[r] = s[4 * u + r]; own_dp[r] = dp[4 * u + r]; }
            } else {
                float* slot = reinterpret_cast<float*>(smem + kPartOff) + ((u * 3 + ((w - u - 1) & 3)) * 8) * 64 + lane;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    slot[r * 64] = s[4 * u + r];
                    slot[(4 + r) * 64] = dp[4 * u + r];
                }
            }
        }
        lds_barrier();
        {
            const float* mine = reinterpret_cast<const float*>(smem + kPartOff) + (w * 3 * 8) * 64 + lane;
#pragma unroll
            for (int v = 0; v < 3; ++v)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    own_s[r] += mine[(v * 8 + r) * 64];
                    own_dp[r] += mine[(v * 8 + 4 + r) * 64];
                }
        }
        // ---- f and p of this wave's 8 keys x 32 queries; pairs outside the mask or the sequence are zero
        {
            const int key0 = (ROLE == kKeyOwner ? o0 : s0) + 8 * w + 4 * h;
            float pv[4], dsv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int key = key0 + r;
                const bool visible = key < p.n && query < p.n && (!p.causal || key <= query);
                const float f = visible ? __builtin_amdgcn_exp2f(own_s[r] * c - lse2) : 0.f;
                pv[r] = f;
                dsv[r] = f * (own_dp[r] - dl);
            }
            u32x2 a, b;
            a[0] = pack_bf16(pv[0], pv[1]);
            a[1] = pack_bf16(pv[2], pv[3]);
            b[0] = pack_bf16(dsv[0], dsv[1]);
            b[1] = pack_bf16(dsv[2], dsv[3]);
            const int off = small_off(l32, 8 * w + 4 * h);  // [query][key]
            *reinterpret_cast<u32x2*>(smem + kPOff + off) = a;
            *reinterpret_cast<u32x2*>(smem + kDsOff + off) = b;
        }
        lds_barrier();
        // ---- products with the whole f / p tile, over this wave's d / 4 columns of the streamed tile
        if (ROLE == kKeyOwner) {
#pragma unroll
            for (int k2 = 0; k2 < BS / 16; ++k2) {  // contraction over the 32 queries
                const bf16x8 pf = small_frag_t(smem + kPOff, 16 * k2, lane);
                const bf16x8 dsf = small_frag_t(smem + kDsOff, 16 * k2, lane);
#pragma unroll
                for (int m = 0; m < MQ; ++m) {
                    const int a = fo.tr(MQ * w + m, 0), b = fo.tr(MQ * w + m, 1);
                    const bf16x8 gt = FragOffsets<D>::read_t(smem, a, b, 16 * k2, st + kTileBytes);  // dO^T
                    const bf16x8 qt = FragOffsets<D>::read_t(smem, a, b, 16 * k2, st);               // Q^T
                    acc[0][m] = mfma32(gt, pf, acc[0][m]);
                    acc[NACC - 1][m] = mfma32(qt, dsf, acc[NACC - 1][m]);
                }
            }
        } else {
#pragma unroll
            for (int k2 = 0; k2 < BS / 16; ++k2) {  // contraction over the 32 keys
                const bf16x8 dsf = small_frag_perm(smem + kDsOff, k2, lane);
#pragma unroll
                for (int m = 0; m < MQ; ++m) {
                    const bf16x8 kt = FragOffsets<D>::read_t(smem, fo.tr(MQ * w + m, 0), fo.tr(MQ * w + m, 1), 16 * k2, st);
                    acc[0][m] = mfma32(kt, dsf, acc[0][m]);
                }
            }
        }
        wait_direct_loads();
        __syncthreads();
    }

    // ---- store: accumulator column <-> owned row, register <-> column of d
    if (orow < p.n) {
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
            __bf16* out = ROLE == kKeyOwner ? (a == 0 ? p.dV : p.dK) : p.dQ;
            const float f = (ROLE == kKeyOwner && a == 0) ? 1.f : p.scale;
            __bf16* row = out + base + (long)orow * ld + DQ * w;
#pragma unroll
            for (int m = 0; m < MQ; ++m)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 v;
                    v[0] = pack_bf16(acc[a][m][4 * g + 0] * f, acc[a][m][4 * g + 1] * f);
                    v[1] = pack_bf16(acc[a][m][4 * g + 2] * f, acc[a][m][4 * g + 3] * f);
                    *reinterpret_cast<u32x2*>(row + 32 * m + 8 * g + 4 * h) = v;
                }
        }
    }
}

template <int D>
static hipError_t launch_splitd_t(const FusedParams& p, hipStream_t stream) {
    constexpr int lds = 2 * (2 * 32 * D * 2) + 4 * 3 * 8 * 64 * 4 + 2 * 2048;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_splitd_kernel<D, kKeyOwner>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_splitd_kernel<D, kQueryOwner>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    launch_delta(p, D, stream);
    const unsigned grid = (unsigned)(((p.n + 31) / 32) * p.batch * p.heads);
    hipLaunchKernelGGL((bwd_splitd_kernel<D, kQueryOwner>), dim3(grid), dim3(kThreads), lds, stream, p);
    hipLaunchKernelGGL((bwd_splitd_kernel<D, kKeyOwner>), dim3(grid), dim3(kThreads), lds, stream, p);
    return hipGetLastError();
}

hipError_t launch_bwd_splitd(int d, const FusedParams& p, hipStream_t stream) {
    switch (d) {
        case 256: return launch_splitd_t<256>(p, stream);
        case 512: return launch_splitd_t<512>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace attn
