// Weight gradient of the paper's attention loss (Def. 3.2 and the gradient theorem of Sec. 3.1;
// no-cache and large-cache algorithms of App. C.1 / App. D):
//     S = A_1 X (the queries), K = A_2, h = A_3 Y (the values),
//     g = dL/dX = A_1^T p A_2                                   (d x d per batch and head)
// With dQ = scale * p A_2 from the query-owner backward kernel this is g = A_1^T dQ: the two
// projections in front of the attention kernels and one product with the contraction over n
// behind them.  The paper accumulates T = A_1^T p block by block and multiplies by A_2 at the
// end; here p A_2 is what the dQ kernel already accumulates per query block, so the d x d
// accumulator of the paper's phase 2 turns into the split-n product below.
//   proj_kernel          Out = A W        [n x d] [d x d] -> bf16, one 128-row block per workgroup
//   wgrad_partial_kernel part_c = A_1[c]^T dQ[c] for a chunk c of rows -> fp32 [d x d]
//   wgrad_reduce_kernel  g = sum_c part_c  (fixed order: bit-reproducible)
#include <cstring>

#include "attn_common.hpp"
#include "attn_internal.hpp"

namespace attn {

namespace {

constexpr int kChunkRows = 1024;  // rows of one partial product

// Out^T = W^T A^T: wave w owns rows 32w .. +31 of the block; W^T fragments (A operands) come
// from transposed LDS reads of the row-major W tile, the rows of A (B operands) straight from
// global memory in the k order of those reads.
template <int D>
__global__ void __launch_bounds__(kThreads) proj_kernel(const __bf16* A, const __bf16* W, __bf16* Out, int n,
                                                        int bh_total) {
    constexpr int KS = D / 16, MT = D / 32;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blocks = (n + 127) / 128;
    const int bh = blockIdx.x / blocks, blk = blockIdx.x % blocks;
    if (bh >= bh_total) return;
    const __bf16* a_head = A + (long)bh * n * D;
    load_tile_direct<D, D>(W + (long)bh * D * D, D, 0, D, smem, tid);
    const int row = blk * 128 + 32 * w + l32;
    const bool ok = row < n;
    // element t of half h of k-step ks <-> input feature 16 ks + 8 (t / 4) + 4h + t % 4
    bf16x8 af[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        u32x2 lo = {0, 0}, hi = {0, 0};
        if (ok) {
            lo = *reinterpret_cast<const u32x2*>(a_head + (long)row * D + 16 * ks + 4 * h);
            hi = *reinterpret_cast<const u32x2*>(a_head + (long)row * D + 16 * ks + 8 + 4 * h);
        }
        const u32x4 r = {lo[0], lo[1], hi[0], hi[1]};
        af[ks] = __builtin_bit_cast(bf16x8, r);
    }
    wait_direct_loads();
    __syncthreads();
    FragOffsets<D> fo;
    fo.init(lane);
    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = mfma32(fo.frag_t(smem, 0, mt, 16 * ks), af[ks], acc[mt]);
    if (ok) {
        __bf16* out = Out + ((long)bh * n + row) * D;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 v;
                v[0] = pack_bf16(acc[mt][4 * g + 0], acc[mt][4 * g + 1]);
                v[1] = pack_bf16(acc[mt][4 * g + 2], acc[mt][4 * g + 3]);
                *reinterpret_cast<u32x2*>(out + 32 * mt + 8 * g + 4 * h) = v;
            }
    }
}

// part[bh][c] = A_1[rows of chunk c]^T dQ[rows of chunk c]: 64-row tiles of both operands are
// streamed through LDS (two stages); both operands of every MFMA are transposed reads (the
// contraction runs over the tiles' rows).  Waves form a 2 x 2 grid over the d x d output.
template <int D>
__global__ void __launch_bounds__(kThreads, D <= 128 ? 2 : 1) wgrad_partial_kernel(const __bf16* A1, const __bf16* dQ, float* part,
                                                                    int n, int chunks) {
    constexpr int BR = 64, TW = D / 64;  // 32 x 32 output tiles per wave and dimension
    constexpr int kTileBytes = BR * D * 2, kStageBytes = 2 * kTileBytes;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = w >> 1, wj = w & 1;
    const int bh = blockIdx.x / chunks, c = blockIdx.x % chunks;
    const __bf16* a_head = A1 + (long)bh * n * D;
    const __bf16* q_head = dQ + (long)bh * n * D;
    const int r_begin = c * kChunkRows, r_end = min(n, r_begin + kChunkRows);
    const int n_it = (r_end - r_begin + BR - 1) / BR;

    f32x16 acc[TW][TW];
#pragma unroll
    for (int x = 0; x < TW; ++x)
#pragma unroll
        for (int y = 0; y < TW; ++y)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[x][y][i] = 0.f;

    TileLoader<D, BR> loader;
    loader.init(tid, D);
    auto fetch = [&](int it, int stage) {
        char* s = smem + stage * kStageBytes;
        loader.load(a_head, D, r_begin + it * BR, n, s, tid);
        loader.load(q_head, D, r_begin + it * BR, n, s + kTileBytes, tid);
    };
    if (n_it > 0) fetch(0, 0);
    wait_direct_loads();
    __syncthreads();
    FragOffsets<D> fo;
    fo.init(lane);
    for (int it = 0; it < n_it; ++it) {
        if (it + 1 < n_it) fetch(it + 1, (it + 1) & 1);
        const int off = (it & 1) * kStageBytes;
        const int r0 = r_begin + it * BR;
        const bool tail = r0 + BR > n;  // rows at or past n repeat the last row: drop them
#pragma unroll
        for (int ks = 0; ks < BR / 16; ++ks) {
            bf16x8 a[TW], b[TW];
#pragma unroll
            for (int x = 0; x < TW; ++x) {
                a[x] = fo.frag_t(smem, off, TW * wi + x, 16 * ks);
                if (tail) {
#pragma unroll
                    for (int t = 0; t < 8; ++t)
                        if (r0 + 16 * ks + 8 * (t >> 2) + 4 * h + (t & 3) >= n) a[x][t] = (__bf16)0.f;
                }
            }
#pragma unroll
            for (int y = 0; y < TW; ++y) b[y] = fo.frag_t(smem, off + kTileBytes, TW * wj + y, 16 * ks);
#pragma unroll
            for (int x = 0; x < TW; ++x)
#pragma unroll
                for (int y = 0; y < TW; ++y) acc[x][y] = mfma32(a[x], b[y], acc[x][y]);
        }
        wait_direct_loads();
        __syncthreads();
    }
    // accumulator: lane <-> output column, register <-> output row
    float* out = part + ((long)bh * chunks + c) * D * D;
#pragma unroll
    for (int x = 0; x < TW; ++x)
#pragma unroll
        for (int y = 0; y < TW; ++y) {
            const int col = 32 * (TW * wj + y) + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) out[(long)(32 * (TW * wi + x) + acc_row(i, h)) * D + col] = acc[x][y][i];
        }
}

__global__ void __launch_bounds__(kThreads) wgrad_reduce_kernel(const float* part, float* g, int chunks, int dd,
                                                               long total) {
    const long e = (long)blockIdx.x * kThreads + threadIdx.x;
    if (e >= total) return;
    const long bh = e / dd, r = e % dd;
    float s = 0.f;
    for (int c = 0; c < chunks; ++c) s += part[(bh * chunks + c) * dd + r];
    g[e] = s;
}

template <int D>
hipError_t run(const WgradParams& p, hipStream_t stream) {
    const int bh = p.batch * p.heads;
    const int blocks = (p.n + 127) / 128, chunks = wgrad_chunks(p.n);
    constexpr int proj_lds = D * D * 2, part_lds = 2 * 2 * 64 * D * 2;
    {  // set on every call: the attributes belong to the current device, and the calls are cheap
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(proj_kernel<D>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, proj_lds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad_partial_kernel<D>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, part_lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(proj_kernel<D>, dim3((unsigned)(blocks * bh)), dim3(kThreads), proj_lds, stream, p.A1, p.X, p.Q,
                       p.n, bh);
    hipLaunchKernelGGL(proj_kernel<D>, dim3((unsigned)(blocks * bh)), dim3(kThreads), proj_lds, stream, p.A3, p.Y, p.V,
                       p.n, bh);
    FusedParams f;
    memset(&f, 0, sizeof(f));
    f.stride_n = D;
    f.stride_h = (long)p.n * D;
    f.stride_b = (long)p.heads * p.n * D;
    f.batch = p.batch;
    f.heads = p.heads;
    f.n = p.n;
    f.scale = p.scale;
    f.causal = p.causal;
    f.Q = p.Q;
    f.K = p.A2;
    f.V = p.V;
    f.Oout = p.O;
    f.LSEout = p.LSE;
    hipError_t e = launch_fwd_fused(D, f, nullptr, nullptr, stream);
    if (e != hipSuccess) return e;
    f.O = p.O;
    f.dO = p.dO;
    f.LSE = p.LSE;
    f.delta = p.delta;
    f.dQ = p.dQ;
    e = launch_bwd_fused(D, f, nullptr, nullptr, nullptr, nullptr, stream, /*dq_only=*/true);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(wgrad_partial_kernel<D>, dim3((unsigned)(chunks * bh)), dim3(kThreads), part_lds, stream, p.A1,
                       p.dQ, p.partial, p.n, chunks);
    const long total = (long)bh * D * D;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       stream, p.partial, p.g, chunks, D * D, total);
    return hipGetLastError();
}

}  // namespace

int wgrad_chunks(int n) { return (n + kChunkRows - 1) / kChunkRows; }

hipError_t launch_wgrad_zero(int d, int bh, float* g, hipStream_t stream) {
    const long total = (long)bh * d * d;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       stream, nullptr, g, 0, d * d, total);
    return hipGetLastError();
}

hipError_t launch_wgrad_fused(int d, const WgradParams& p, hipStream_t stream) {
    switch (d) {
        case 64: return run<64>(p, stream);
        case 128: return run<128>(p, stream);
        case 256: return run<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace attn
