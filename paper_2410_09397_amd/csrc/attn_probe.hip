// Measurement aid, not part of the attention path: the rate at which the device sustains dense
// bf16 MFMAs on given operand data.  The 2.5 PFLOP/s peak assumes 2.4 GHz; under matrix load the
// clock follows the power the operands' switching activity draws, so the rate that a kernel's
// roofline fraction can be read against depends on the data.  A register-only loop of
// independent v_mfma_f32_32x32x16_bf16 chains (two waves per SIMD on every CU, no memory traffic)
// is the ceiling for any kernel built on that instruction.
#include <hip/hip_runtime.h>

#include "attn_common.hpp"
#include "../../include/attn_mi355x.h"

namespace attn {

namespace {

constexpr int kProbeBlocksPerCu = 2, kProbeLds = 64 * 1024;  // 64 KB of LDS pins two workgroups to a CU
constexpr int kProbeMfmaPerIter = 8;

__device__ __forceinline__ unsigned mix(unsigned x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// two bf16 values with random sign and mantissa and magnitude in [0.5, 2)
__device__ __forceinline__ unsigned random_bf16x2(unsigned seed) {
    const unsigned r = mix(seed);
    const unsigned lo = 0x3f00u | (r & 0x80ffu);
    const unsigned hi = 0x3f00u | ((r >> 16) & 0x80ffu);
    return lo | (hi << 16);
}

// MODE 0: operands stay in registers.  MODE 1: the B operand of every MFMA is a fresh 1 KB fragment read from LDS
// (ds_read_b128 per lane, conflict-free), which is what the attention kernels do.  MODE 2: in addition one exponential
// and four other fp32 instructions per MFMA, independent of one another: about the vector arithmetic of the
// backward kernels per MFMA.
template <int MODE>
__global__ void __launch_bounds__(kThreads) mfma_ceiling_kernel(float* result, int iters, int zero_operands) {
    extern __shared__ char smem[];
    const int tid = threadIdx.x;
    u32x4 au, bu;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        au[i] = zero_operands ? 0u : random_bf16x2(tid * 31u + i + blockIdx.x * 7919u);
        bu[i] = zero_operands ? 0u : random_bf16x2(tid * 57u + i + 99u);
    }
    const bf16x8 a = __builtin_bit_cast(bf16x8, au);
    bf16x8 b = __builtin_bit_cast(bf16x8, bu);
    if (MODE >= 1) {  // 8 fragments of 1 KB per wave in LDS, random (or zero) like the register operands
#pragma unroll
        for (int j = 0; j < kProbeMfmaPerIter; ++j) {
            u32x4 v;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = zero_operands ? 0u : random_bf16x2(tid * 131u + j * 17u + i);
            *reinterpret_cast<u32x4*>(smem + (j * kThreads + tid) * 16) = v;
        }
        __syncthreads();
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    float v[kProbeMfmaPerIter];
#pragma unroll
    for (int j = 0; j < kProbeMfmaPerIter; ++j) v[j] = 0.37f + tid * 1e-3f + j;
    bf16x8 b_next = b;
    if (MODE >= 1) b_next = *reinterpret_cast<const bf16x8*>(smem + tid * 16);
    const long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < kProbeMfmaPerIter; ++j) {
            if (MODE >= 1) {  // a read per MFMA, requested one MFMA ahead (as the kernels do) and not hoisted out of the loop
                b = b_next;
                b_next = *reinterpret_cast<const bf16x8*>(smem + (((j + 1) % kProbeMfmaPerIter) * kThreads + tid) * 16);
                asm volatile("" : "+v"(b));
            }
            acc[j & 3] = mfma32(a, b, acc[j & 3]);
            if (MODE >= 2) {  // independent of one another and of the MFMAs: v[j] is touched once per iteration
                const float e = __builtin_amdgcn_exp2f(v[j] * 0.5f - 1.f);
                v[j] = (e - 0.25f) * v[j] + 0.3f;
                v[(j + 4) & 7] = v[(j + 4) & 7] * 0.999f + 0.001f;
                asm volatile("" : "+v"(v[j]));
            }
        }
        if ((it & 1023) == 1023) {  // the sums are random walks: pull them back now and then
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[j][i] *= 1e-3f;
        }
    }
    // shader clock in GHz: cycle counter against the 100 MHz constant-rate counter
    if (tid == 0 && blockIdx.x == gridDim.x / 2)
        result[0] = (float)((double)(clock64() - c0) / (double)(wall_clock64() - w0)) * 0.1f;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kProbeMfmaPerIter; ++j) s += v[j];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    if (s == 12345.678f) smem[tid] = 1;  // keeps the accumulators (and the LDS allocation) alive
}

// The tile loop of the dK / dV kernel with everything that makes it wait taken out: one iteration issues what one wave
// issues for a 64 x 64 tile at d = 128 - 32 MFMAs, the first 16 with one ds_read_b128 fragment each (phase 1), the last
// 16 with two ds_read_b64_tr_b16 fragments each (phase 2), 16 exponentials, 64 fp32 multiply-adds, 16 bf16 packs, 8
// 8-byte LDS writes, its quarter (8 KB) of the 32 KB tile copy with global_load_lds_dwordx4, two workgroup barriers -
// but no instruction depends on a result of this iteration: the vector arithmetic works on its own registers, the
// fragments are always there, the copied bytes (from a 1 MB window that stays in L2) are never read.  What is left is
// the issue cost of the instruction mix; the real kernel adds the waits for operands.
constexpr int kSkeletonLds = 72 * 1024;       // 32 KB of fragments, 32 KB copy target, 8 KB for the writes; two workgroups per CU
constexpr int kSkeletonWindowTiles = 32;      // 32 KB tiles
static __device__ __align__(256) unsigned char skeleton_src[kSkeletonWindowTiles * 32768];
__global__ void __launch_bounds__(kThreads, 2) tile_skeleton_kernel(float* result, const unsigned char* src, int tiles) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    u32x4 au;
#pragma unroll
    for (int i = 0; i < 4; ++i) au[i] = random_bf16x2(tid * 31u + i + blockIdx.x * 7919u);
    const bf16x8 a = __builtin_bit_cast(bf16x8, au);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = random_bf16x2(tid * 131u + j * 17u + i);
        *reinterpret_cast<u32x4*>(smem + (j * kThreads + tid) * 16) = v;
    }
    __syncthreads();
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    float e[16], v[32];
    unsigned pk[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        e[j] = 0.37f + tid * 1e-3f + j;
        pk[j] = 0;
    }
#pragma unroll
    for (int j = 0; j < 32; ++j) v[j] = 0.11f + tid * 1e-3f + j;
    auto fragment = [&](int j) -> bf16x8 {  // j < 16: one 16-byte read; otherwise two transposing 8-byte reads
        const char* p = smem + ((j & 7) * kThreads + tid) * 16;
        if ((j & 31) >= 16) {
            const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(p));
            const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 ATTN_LDS*)(p + 8));
            typedef short i16x8 __attribute__((ext_vector_type(8)));
            return __builtin_bit_cast(bf16x8, (i16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
        return *reinterpret_cast<const bf16x8*>(p);
    };
    bf16x8 b, b_next = fragment(0);
    const unsigned copy_dst = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(ATTN_LDS char*)(smem + 32768)) + w * 8192;
    const unsigned voff = lane * 16;
    unsigned pos = (blockIdx.x * 7u) % kSkeletonWindowTiles;
    const long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < tiles; ++it) {
        pos = (pos + 1) % kSkeletonWindowTiles;
        // the tile address is uniform: hand it to the copies as a scalar pair
        const unsigned long long ta = reinterpret_cast<unsigned long long>(src + (size_t)pos * 32768 + w * 8192);
        // (the builtin returns a signed int: both halves go through unsigned, or the low half would sign-extend
        // into the high one)
        const unsigned ta_lo = __builtin_amdgcn_readfirstlane((unsigned)ta);
        const unsigned ta_hi = __builtin_amdgcn_readfirstlane((unsigned)(ta >> 32));
        const unsigned long long tile = ((unsigned long long)ta_hi << 32) | ta_lo;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            b = b_next;
            b_next = fragment(j + 1);
            asm volatile("" : "+v"(b));
            acc[j & 3] = mfma32(a, b, acc[j & 3]);
            if (j % 4 == 0)  // this wave's 8 KB of the tile copy, 1 KB per instruction
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                             :
                             : "s"(copy_dst + (j / 4) * 1024), "v"(voff + (j / 4) * 1024), "s"(tile)
                             : "memory", "m0");
            if (j % 2 == 0) {
                e[j / 2] = __builtin_amdgcn_exp2f(e[j / 2]);
                asm volatile("" : "+v"(e[j / 2]));
                pk[j / 2] = pack_bf16(v[j], v[j + 1]);
                asm volatile("" : "+v"(pk[j / 2]));
            }
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int i = (2 * j + x) & 31;
                v[i] = v[i] * 0.999f + 0.001f;
                asm volatile("" : "+v"(v[i]));
            }
            if (j % 4 == 3) {
                u32x2 t;
                t[0] = pk[(j / 4) * 2];
                t[1] = pk[(j / 4) * 2 + 1];
                *reinterpret_cast<u32x2*>(smem + 65536 + (((j / 4) & 3) * kThreads + tid) * 8) = t;
            }
            if (j == 15) lds_barrier();
        }
        wait_direct_loads();
        lds_barrier();
        if ((it & 255) == 255) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[j][i] *= 1e-3f;
        }
    }
    if (tid == 0 && blockIdx.x == gridDim.x / 2)
        result[0] = (float)((double)(clock64() - c0) / (double)(wall_clock64() - w0)) * 0.1f;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) s += e[j] + (float)pk[j];
#pragma unroll
    for (int j = 0; j < 32; ++j) s += v[j];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    if (s == 12345.678f) smem[tid] = 1;
}

}  // namespace

}  // namespace attn

namespace {

// `iters` iterations of 8 MFMAs, as in the other variants: a tile of the skeleton is four of them
attn_status launch_tile_skeleton(int iters, float* clock_ghz, double* flops, hipStream_t s) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ATTN_ERR_DEVICE;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return ATTN_ERR_DEVICE;
    void* src = nullptr;  // the array lives once per device: ask for the current device's copy every time
    if (hipGetSymbolAddress(&src, HIP_SYMBOL(attn::skeleton_src)) != hipSuccess || !src) return ATTN_ERR_DEVICE;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(attn::tile_skeleton_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, attn::kSkeletonLds) != hipSuccess)
        return ATTN_ERR_DEVICE;
    const int tiles = (iters + 3) / 4, blocks = attn::kProbeBlocksPerCu * cus;
    hipLaunchKernelGGL(attn::tile_skeleton_kernel, dim3((unsigned)blocks), dim3(attn::kThreads), attn::kSkeletonLds, s,
                       clock_ghz, static_cast<const unsigned char*>(src), tiles);
    if (hipGetLastError() != hipSuccess) return ATTN_ERR_DEVICE;
    *flops = (double)blocks * (attn::kThreads / 64) * 32.0 * (double)tiles * 2.0 * 32 * 32 * 16;
    return ATTN_OK;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

attn_status attn_mfma_ceiling(int32_t iters, int32_t operands, float* clock_ghz, double* flops, void* stream) {
    if (iters < 1 || iters > 4000000 || !clock_ghz || !flops) return ATTN_ERR_INVALID_ARG;  // <= about 1 s of GPU time
    if (operands < 0 || operands > 4) return ATTN_ERR_INVALID_ARG;
    if (operands == 4) return launch_tile_skeleton(iters, clock_ghz, flops, static_cast<hipStream_t>(stream));
    const int zero_operands = operands == 1, mode = operands >= 2 ? operands - 1 : 0;
    const void* fn = mode == 0   ? reinterpret_cast<const void*>(attn::mfma_ceiling_kernel<0>)
                     : mode == 1 ? reinterpret_cast<const void*>(attn::mfma_ceiling_kernel<1>)
                                 : reinterpret_cast<const void*>(attn::mfma_ceiling_kernel<2>);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ATTN_ERR_DEVICE;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return ATTN_ERR_DEVICE;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, attn::kProbeLds) != hipSuccess)
        return ATTN_ERR_DEVICE;
    const int blocks = attn::kProbeBlocksPerCu * cus;
    const dim3 grid((unsigned)blocks), block(attn::kThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mode == 0) hipLaunchKernelGGL(attn::mfma_ceiling_kernel<0>, grid, block, attn::kProbeLds, s, clock_ghz, iters, zero_operands);
    else if (mode == 1) hipLaunchKernelGGL(attn::mfma_ceiling_kernel<1>, grid, block, attn::kProbeLds, s, clock_ghz, iters, zero_operands);
    else hipLaunchKernelGGL(attn::mfma_ceiling_kernel<2>, grid, block, attn::kProbeLds, s, clock_ghz, iters, zero_operands);
    if (hipGetLastError() != hipSuccess) return ATTN_ERR_DEVICE;
    // 32 x 32 x 16 multiply-adds per MFMA and wave
    *flops = (double)blocks * (attn::kThreads / 64) * attn::kProbeMfmaPerIter * (double)iters * 2.0 * 32 * 32 * 16;
    return ATTN_OK;
}

}  // extern "C"
#pragma GCC visibility pop
