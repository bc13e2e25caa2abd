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
    const long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < kProbeMfmaPerIter; ++j) {
            if (MODE >= 1) {
                b = *reinterpret_cast<const bf16x8*>(smem + (j * kThreads + tid) * 16);
                asm volatile("" : "+v"(b));  // a read per MFMA: not hoisted out of the loop
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

}  // namespace

}  // namespace attn

#pragma GCC visibility push(default)
extern "C" {

attn_status attn_mfma_ceiling(int32_t iters, int32_t operands, float* clock_ghz, double* flops, void* stream) {
    if (iters < 1 || iters > 4000000 || !clock_ghz || !flops) return ATTN_ERR_INVALID_ARG;  // <= about 1 s of GPU time
    if (operands < 0 || operands > 3) return ATTN_ERR_INVALID_ARG;
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
