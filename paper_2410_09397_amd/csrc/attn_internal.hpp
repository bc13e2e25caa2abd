// Host-side launcher declarations shared between the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "attn_common.hpp"

namespace attn {

// Fused bf16 paths, d in {64, 128, 256}.  csr_* / csc_* are device pointers or nullptr (dense).
hipError_t launch_fwd_fused(int d, const FusedParams& p, const int32_t* csr_ptr, const int32_t* csr_idx,
                            hipStream_t stream);
// dq_only: run the query-owner kernel alone (dQ and delta), for callers that need neither dK nor dV;
// dkdv_only: run the key-owner kernel alone (it reads the delta an earlier call left in p.delta).
// order_scratch: under a block mask, 3 * ceil(n / 128) int32 per mask of device scratch for the order in
// which the workgroups take the blocks (longest list first), or nullptr (ascending order).
// onepass_keys: 0 = the two-kernel tiling; 64 or 128 = the one-pass tiling with that many keys per
// workgroup, which sums dQ in dq_acc, an fp32 [batch * heads, n, d] array of device scratch.
hipError_t launch_bwd_fused(int d, const FusedParams& p, const int32_t* csr_ptr, const int32_t* csr_idx,
                            const int32_t* csc_ptr, const int32_t* csc_idx, hipStream_t stream,
                            bool dq_only = false, int32_t* order_scratch = nullptr, int onepass_keys = 0,
                            float* dq_acc = nullptr, bool dkdv_only = false);
// The three launches of the one-pass tiling (d = 64: key_block 64; d = 128: 64 or 128); p.list_*, p.order
// describe the key-block columns of a block mask (or are null).
hipError_t launch_bwd_onepass(int d, int key_block, const FusedParams& p, float* dq_acc, hipStream_t stream);

// Fused split-d backward (bf16, d in {256, 512}, no block mask): delta kernel, query-owner and key-owner launches.
hipError_t launch_bwd_splitd(int d, const FusedParams& p, hipStream_t stream);

// delta[b, h, i] = sum_k dO_ik O_ik for bf16 tensors (p.O, p.dO, p.delta), any d % 8 == 0.
void launch_delta(const FusedParams& p, int d, hipStream_t stream);

// Arguments of the large-d path (bf16, d in {512, 1024}, no block mask).  P and dS are n x n
// matrices per (batch, head) with row pitch npad = n rounded up to 256, in the workspace.
struct LargeDParams {
    const __bf16 *Q, *K, *V, *dO;
    __bf16 *Oout, *dQ, *dK, *dV;
    const float* LSE;   // backward input
    float* LSEout;      // forward output
    const float* delta; // backward: rowsum(dO o O)
    __bf16 *P, *dS;
    float *stat_m, *stat_l;  // forward: per 64-key chunk row maximum and sum, [bh][npad / 64][n]
    long stride_b, stride_h, stride_n;
    int batch, heads, n, d, npad;
    float scale;
    int causal;
};
hipError_t configure_larged();  // kernel attributes; call before anything of a large-d call is launched
hipError_t launch_larged(bool backward, const LargeDParams& p, hipStream_t stream);

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
    int mask_stride;  // entries between the pointer arrays of consecutive (batch, head) masks; 0 = one shared mask
};
hipError_t launch_generic(bool is_bf16, bool backward, const GenericParams& p, hipStream_t stream);

// Weight gradient g = A_1^T dQ of the paper's loss (bf16, d in {64, 128, 256}, contiguous tensors).
// Q, V, O, dQ are [b, h, n, d] bf16 scratch, LSE and delta [b, h, n] fp32, partial
// [b * h, wgrad_chunks(n), d, d] fp32; X, Y are [b, h, d, d] bf16, g is [b, h, d, d] fp32.
struct WgradParams {
    const __bf16 *A1, *A2, *A3, *X, *Y, *dO;
    float* g;
    __bf16 *Q, *V, *O, *dQ;
    float *LSE, *delta, *partial;
    int batch, heads, n;
    float scale;
    int causal;
};
int wgrad_chunks(int n);
hipError_t launch_wgrad_fused(int d, const WgradParams& p, hipStream_t stream);
hipError_t launch_wgrad_zero(int d, int bh, float* g, hipStream_t stream);  // n == 0: g = 0

}  // namespace attn
