// Host-side launcher declarations shared between the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "attn_common.hpp"

namespace attn {

// Fused bf16 paths, d in {64, 128}.  csr_* / csc_* are device pointers or nullptr (dense).
hipError_t launch_fwd_fused(int d, const FusedParams& p, const int32_t* csr_ptr, const int32_t* csr_idx,
                            hipStream_t stream);
hipError_t launch_bwd_fused(int d, const FusedParams& p, const int32_t* csr_ptr, const int32_t* csr_idx,
                            const int32_t* csc_ptr, const int32_t* csc_idx, hipStream_t stream);

// Arguments of the generic fp32-arithmetic kernels (any n, d <= 512, any mask block edge).
struct GenericParams {
    const void *Q, *K, *V, *O_in, *dO;
    void *O, *dQ, *dK, *dV;
    const float* LSE_in;
    float* LSE_out;
    float* delta;
    long stride_b, stride_h, stride_n;
    int batch, heads, n, d;
    float scale;
    int causal;
    const int32_t *csr_ptr, *csr_idx, *csc_ptr, *csc_idx;  // nullptr = dense
    int block;
};
hipError_t launch_generic(bool is_bf16, bool backward, const GenericParams& p, hipStream_t stream);

}  // namespace attn
