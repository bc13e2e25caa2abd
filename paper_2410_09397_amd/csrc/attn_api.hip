// C ABI of libattn_mi355x.so: host-side validation and dispatch.  No device memory is
// allocated here and nothing is launched before every argument has been checked.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/attn_mi355x.h"
#include "attn_internal.hpp"

// Device scratch of attn_bwd_noalloc: one copy per GPU the library runs on, held until the process
// ends.  Host code never uses this name as an address; it asks the runtime for the device address.
static __device__ __align__(256) unsigned char scratch[ATTN_NOALLOC_SCRATCH_BYTES];

namespace {

using attn::FusedParams;
using attn::GenericParams;
using attn::LargeDParams;

enum class Path { kFused, kLargeD, kGeneric, kSplitD, kNone };

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

attn_status check_desc(const attn_desc* d) {
    if (!d) return ATTN_ERR_INVALID_ARG;
    if (d->batch < 0 || d->heads < 0 || d->n < 0 || d->d < 1) return ATTN_ERR_INVALID_ARG;
    if (d->causal != 0 && d->causal != 1) return ATTN_ERR_INVALID_ARG;
    if (!std::isfinite(d->scale)) return ATTN_ERR_INVALID_ARG;
    if (d->dtype != ATTN_F32 && d->dtype != ATTN_BF16) return ATTN_ERR_UNSUPPORTED;
    if (d->d > 512 && !(d->dtype == ATTN_BF16 && d->d == 1024)) return ATTN_ERR_UNSUPPORTED;
    if (d->dtype == ATTN_BF16 && d->d % 8 != 0) return ATTN_ERR_UNSUPPORTED;
    if (d->stride_n < d->d || d->stride_h < 0 || d->stride_b < 0) return ATTN_ERR_INVALID_ARG;
    if (d->dtype == ATTN_BF16 && (d->stride_n % 8 || d->stride_h % 8 || d->stride_b % 8))
        return ATTN_ERR_INVALID_ARG;
    // the tile copies address a tile's rows with 32-bit byte offsets from its first row
    if (d->stride_n >= (int64_t)1 << 22) return ATTN_ERR_UNSUPPORTED;
    if (d->bwd_tiling < ATTN_BWD_AUTO || d->bwd_tiling > ATTN_BWD_SPLIT_D) return ATTN_ERR_INVALID_ARG;
    return ATTN_OK;
}

attn_status check_mask(const attn_desc* d, const attn_blockmask* m) {
    if (!m) return ATTN_OK;
    if (m->block < 1 || m->nblk < 0) return ATTN_ERR_INVALID_ARG;
    if ((long)m->nblk != ((long)d->n + m->block - 1) / m->block) return ATTN_ERR_INVALID_ARG;
    if (!m->row_ptr || !m->col_idx || !m->col_ptr || !m->row_idx) return ATTN_ERR_INVALID_ARG;
    if (m->nmasks != 0 && m->nmasks != 1 && (long)m->nmasks != (long)d->batch * d->heads) return ATTN_ERR_INVALID_ARG;
    return ATTN_OK;
}

bool is_empty(const attn_desc* d) { return (long)d->batch * d->heads * d->n == 0; }

Path pick_path(const attn_desc* d, const attn_blockmask* m) {
    if (d->dtype == ATTN_BF16 && (d->d == 64 || d->d == 128 || d->d == 256) && (!m || m->block == 128))
        return Path::kFused;
    if (d->dtype == ATTN_BF16 && (d->d == 512 || d->d == 1024) && !m && d->n <= 32768)
        return Path::kLargeD;
    return Path::kGeneric;
}

// The tiling the fused backward runs with: the caller's choice where it exists for the shape (0 if it
// does not), else the library's.
int pick_tiling(const attn_desc* d) {
    switch (d->bwd_tiling) {
        case ATTN_BWD_TWO_KERNEL:
        case ATTN_BWD_PART_DQ:
        case ATTN_BWD_PART_DKDV: return d->bwd_tiling;
        case ATTN_BWD_ONEPASS_K64: return (d->d == 64 || d->d == 128) ? ATTN_BWD_ONEPASS_K64 : 0;
        case ATTN_BWD_ONEPASS_K128: return (d->d == 64 || d->d == 128) ? ATTN_BWD_ONEPASS_K128 : 0;
        default: return ATTN_BWD_TWO_KERNEL;
    }
}
bool is_onepass(int tiling) { return tiling == ATTN_BWD_ONEPASS_K64 || tiling == ATTN_BWD_ONEPASS_K128; }

// d = 1024 exists on the large-d path only (the generic kernels stop at 512).
attn_status check_path(const attn_desc* d, const attn_blockmask* m) {
    return (d->d > 512 && pick_path(d, m) != Path::kLargeD) ? ATTN_ERR_UNSUPPORTED : ATTN_OK;
}

// The path of the backward: the caller can ask for the four-phase scheme at head dimensions where the
// fused kernels are the default, and for the fused split-d kernels where the four-phase scheme is.
Path bwd_path(const attn_desc* d, const attn_blockmask* m) {
    const bool plain = d->dtype == ATTN_BF16 && !m;
    if (d->bwd_tiling == ATTN_BWD_FOUR_PHASE)
        return plain && d->n <= 32768 && (d->d == 128 || d->d == 256 || d->d == 512 || d->d == 1024) ? Path::kLargeD
                                                                                                       : Path::kNone;
    if (d->bwd_tiling == ATTN_BWD_SPLIT_D) return plain && (d->d == 256 || d->d == 512) ? Path::kSplitD : Path::kNone;
    if (check_path(d, m) != ATTN_OK) return Path::kNone;
    const Path path = pick_path(d, m);
    return (path == Path::kFused && pick_tiling(d) == 0) ? Path::kNone : path;
}

size_t delta_bytes(const attn_desc* d) { return round_up((size_t)d->batch * d->heads * d->n * sizeof(float), 256); }
// two lists of 128-row block indices (query blocks, key blocks) and one of list lengths for the masked fused backward
int mask_count(const attn_blockmask* m) { return m && m->nmasks > 1 ? m->nmasks : 1; }
size_t order_bytes(const attn_desc* d, const attn_blockmask* m) {
    return round_up((size_t)mask_count(m) * 3 * (((size_t)d->n + 127) / 128) * sizeof(int32_t), 256);
}
// the fp32 [batch, heads, n, d] array in which the one-pass tilings sum dQ
size_t dq_acc_bytes(const attn_desc* d) {
    return round_up((size_t)d->batch * d->heads * d->n * d->d * sizeof(float), 256);
}
// Workspace layout of the fused backward: [delta][block order lists (masked only)][fp32 dQ (one-pass only)]
size_t fused_bytes(const attn_desc* d, const attn_blockmask* m) {
    return delta_bytes(d) + (m ? order_bytes(d, m) : 0) + (is_onepass(pick_tiling(d)) ? dq_acc_bytes(d) : 0);
}

// Workspace layout of the large-d path.  Backward: [delta][P][dS]; forward: [stat_m][stat_l][P].
size_t npad_of(const attn_desc* d) { return round_up((size_t)d->n, 256); }  // the product kernels' row block
size_t nn_bytes(const attn_desc* d) { return (size_t)d->batch * d->heads * npad_of(d) * npad_of(d) * 2; }
size_t stat_bytes(const attn_desc* d) {
    return round_up((size_t)d->batch * d->heads * d->n * (npad_of(d) / 64) * sizeof(float), 256);
}

LargeDParams larged_params(const attn_desc* d) {
    LargeDParams p;
    std::memset(&p, 0, sizeof(p));
    p.stride_b = d->stride_b;
    p.stride_h = d->stride_h;
    p.stride_n = d->stride_n;
    p.batch = d->batch;
    p.heads = d->heads;
    p.n = d->n;
    p.d = d->d;
    p.npad = (int)npad_of(d);
    p.scale = d->scale;
    p.causal = d->causal;
    return p;
}

FusedParams fused_params(const attn_desc* d) {
    FusedParams p;
    std::memset(&p, 0, sizeof(p));
    p.stride_b = d->stride_b;
    p.stride_h = d->stride_h;
    p.stride_n = d->stride_n;
    p.batch = d->batch;
    p.heads = d->heads;
    p.n = d->n;
    p.scale = d->scale;
    p.causal = d->causal;
    return p;
}

GenericParams generic_params(const attn_desc* d, const attn_blockmask* m) {
    GenericParams p;
    std::memset(&p, 0, sizeof(p));
    p.stride_b = d->stride_b;
    p.stride_h = d->stride_h;
    p.stride_n = d->stride_n;
    p.batch = d->batch;
    p.heads = d->heads;
    p.n = d->n;
    p.d = d->d;
    p.scale = d->scale;
    p.causal = d->causal;
    p.block = 1;
    if (m) {
        p.csr_ptr = m->row_ptr;
        p.csr_idx = m->col_idx;
        p.csc_ptr = m->col_ptr;
        p.csc_idx = m->row_idx;
        p.block = m->block;
        p.mask_stride = m->nmasks > 1 ? m->nblk + 1 : 0;
    }
    return p;
}

attn_status bwd_impl(const attn_desc* desc, const attn_blockmask* mask, const void* Q, const void* K,
                     const void* V, const void* O, const void* dO, const float* LSE, void* dQ, void* dK,
                     void* dV, void* workspace, size_t workspace_bytes, void* stream) {
    attn_status st = check_desc(desc);
    if (st != ATTN_OK) return st;
    st = check_mask(desc, mask);
    if (st != ATTN_OK) return st;
    const Path path = bwd_path(desc, mask);
    if (path == Path::kNone) return ATTN_ERR_UNSUPPORTED;
    if (is_empty(desc)) return ATTN_OK;
    if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV) return ATTN_ERR_INVALID_ARG;
    if (desc->dtype == ATTN_BF16 && !(aligned16(Q) && aligned16(K) && aligned16(V) && aligned16(O) &&
                                      aligned16(dO) && aligned16(dQ) && aligned16(dK) && aligned16(dV)))
        return ATTN_ERR_INVALID_ARG;
    const size_t need = attn_workspace_bytes(desc, mask);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return ATTN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (path) {
        case Path::kSplitD: {
            FusedParams p = fused_params(desc);
            p.Q = static_cast<const __bf16*>(Q);
            p.K = static_cast<const __bf16*>(K);
            p.V = static_cast<const __bf16*>(V);
            p.O = static_cast<const __bf16*>(O);
            p.dO = static_cast<const __bf16*>(dO);
            p.dQ = static_cast<__bf16*>(dQ);
            p.dK = static_cast<__bf16*>(dK);
            p.dV = static_cast<__bf16*>(dV);
            p.LSE = LSE;
            p.delta = static_cast<float*>(workspace);
            e = attn::launch_bwd_splitd(desc->d, p, s);
            break;
        }
        case Path::kFused: {
            FusedParams p = fused_params(desc);
            p.Q = static_cast<const __bf16*>(Q);
            p.K = static_cast<const __bf16*>(K);
            p.V = static_cast<const __bf16*>(V);
            p.O = static_cast<const __bf16*>(O);
            p.dO = static_cast<const __bf16*>(dO);
            p.dQ = static_cast<__bf16*>(dQ);
            p.dK = static_cast<__bf16*>(dK);
            p.dV = static_cast<__bf16*>(dV);
            p.LSE = LSE;
            p.delta = static_cast<float*>(workspace);
            p.list_stride = mask && mask->nmasks > 1 ? mask->nblk + 1 : 0;
            char* ws = static_cast<char*>(workspace);
            int32_t* order = mask ? reinterpret_cast<int32_t*>(ws + delta_bytes(desc)) : nullptr;
            const int tiling = pick_tiling(desc);
            float* dq_acc = is_onepass(tiling)
                                ? reinterpret_cast<float*>(ws + delta_bytes(desc) + (mask ? order_bytes(desc, mask) : 0))
                                : nullptr;
            e = attn::launch_bwd_fused(desc->d, p, mask ? mask->row_ptr : nullptr, mask ? mask->col_idx : nullptr,
                                       mask ? mask->col_ptr : nullptr, mask ? mask->row_idx : nullptr, s,
                                       tiling == ATTN_BWD_PART_DQ, order,
                                       tiling == ATTN_BWD_ONEPASS_K64 ? 64 : tiling == ATTN_BWD_ONEPASS_K128 ? 128 : 0,
                                       dq_acc, tiling == ATTN_BWD_PART_DKDV);
            break;
        }
        case Path::kLargeD: {
            if (attn::configure_larged() != hipSuccess) return ATTN_ERR_DEVICE;  // before the first launch
            char* ws = static_cast<char*>(workspace);
            FusedParams fp = fused_params(desc);
            fp.O = static_cast<const __bf16*>(O);
            fp.dO = static_cast<const __bf16*>(dO);
            fp.delta = reinterpret_cast<float*>(ws);
            attn::launch_delta(fp, desc->d, s);
            LargeDParams p = larged_params(desc);
            p.Q = static_cast<const __bf16*>(Q);
            p.K = static_cast<const __bf16*>(K);
            p.V = static_cast<const __bf16*>(V);
            p.dO = static_cast<const __bf16*>(dO);
            p.dQ = static_cast<__bf16*>(dQ);
            p.dK = static_cast<__bf16*>(dK);
            p.dV = static_cast<__bf16*>(dV);
            p.LSE = LSE;
            p.delta = fp.delta;
            p.P = reinterpret_cast<__bf16*>(ws + delta_bytes(desc));
            p.dS = reinterpret_cast<__bf16*>(ws + delta_bytes(desc) + nn_bytes(desc));
            e = attn::launch_larged(true, p, s);
            break;
        }
        default: {
            GenericParams p = generic_params(desc, mask);
            p.Q = Q;
            p.K = K;
            p.V = V;
            p.O_in = O;
            p.dO = dO;
            p.dQ = dQ;
            p.dK = dK;
            p.dV = dV;
            p.LSE_in = LSE;
            p.delta = static_cast<float*>(workspace);
            e = attn::launch_generic(desc->dtype == ATTN_BF16, true, p, s);
            break;
        }
    }
    return e == hipSuccess ? ATTN_OK : ATTN_ERR_DEVICE;
}

// Weight-gradient entry point: bf16, d in {64, 128, 256}, contiguous [batch, heads, n, d] tensors.
attn_status wgrad_check(const attn_desc* d) {
    const attn_status st = check_desc(d);
    if (st != ATTN_OK) return st;
    if (d->dtype != ATTN_BF16 || (d->d != 64 && d->d != 128 && d->d != 256)) return ATTN_ERR_UNSUPPORTED;
    if (!is_empty(d) && (d->stride_n != d->d || d->stride_h != (int64_t)d->n * d->d ||
                         d->stride_b != (int64_t)d->heads * d->n * d->d))
        return ATTN_ERR_UNSUPPORTED;
    return ATTN_OK;
}

// Workspace of the weight gradient: [Q][V][O][dQ] bf16 tensors, [LSE][delta] rows, [partial products].
struct WgradLayout {
    size_t q, v, o, dq, lse, delta, partial, total;
};
WgradLayout wgrad_layout(const attn_desc* d) {
    const size_t bh = (size_t)d->batch * d->heads;
    const size_t t = round_up(bh * d->n * d->d * 2, 256), r = round_up(bh * d->n * sizeof(float), 256);
    WgradLayout l;
    l.q = 0;
    l.v = t;
    l.o = 2 * t;
    l.dq = 3 * t;
    l.lse = 4 * t;
    l.delta = 4 * t + r;
    l.partial = 4 * t + 2 * r;
    l.total = l.partial + round_up(bh * attn::wgrad_chunks(d->n) * d->d * d->d * sizeof(float), 256);
    return l;
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};
hipError_t scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

size_t attn_workspace_bytes(const attn_desc* desc, const attn_blockmask* mask) {
    if (check_desc(desc) != ATTN_OK || check_mask(desc, mask) != ATTN_OK || check_path(desc, mask) != ATTN_OK) return 0;
    if (is_empty(desc)) return 256;
    // the forward goes by d alone; the backward also by the tiling asked for (one that does not exist
    // for the shape is refused by the backward itself and needs nothing here)
    const size_t fwd = pick_path(desc, mask) == Path::kLargeD ? 2 * stat_bytes(desc) + nn_bytes(desc) : 0;
    size_t bwd = delta_bytes(desc);
    switch (bwd_path(desc, mask)) {
        case Path::kLargeD: bwd = delta_bytes(desc) + 2 * nn_bytes(desc); break;
        case Path::kFused: bwd = fused_bytes(desc, mask); break;
        default: break;
    }
    return bwd > fwd ? bwd : fwd;
}

attn_status attn_fwd(const attn_desc* desc, const attn_blockmask* mask, const void* Q, const void* K,
                     const void* V, void* O, float* LSE, void* workspace, size_t workspace_bytes, void* stream) {
    attn_status st = check_desc(desc);
    if (st != ATTN_OK) return st;
    st = check_mask(desc, mask);
    if (st != ATTN_OK) return st;
    st = check_path(desc, mask);
    if (st != ATTN_OK) return st;
    if (is_empty(desc)) return ATTN_OK;
    if (!Q || !K || !V || !O || !LSE) return ATTN_ERR_INVALID_ARG;
    if (desc->dtype == ATTN_BF16 && !(aligned16(Q) && aligned16(K) && aligned16(V) && aligned16(O)))
        return ATTN_ERR_INVALID_ARG;
    const Path path = pick_path(desc, mask);
    // the forward's own share of attn_workspace_bytes: row statistics and the matrix f
    if (path == Path::kLargeD &&
        (!workspace || workspace_bytes < 2 * stat_bytes(desc) + nn_bytes(desc) || !aligned16(workspace)))
        return ATTN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (path) {
        case Path::kFused: {
            FusedParams p = fused_params(desc);
            p.Q = static_cast<const __bf16*>(Q);
            p.K = static_cast<const __bf16*>(K);
            p.V = static_cast<const __bf16*>(V);
            p.Oout = static_cast<__bf16*>(O);
            p.LSEout = LSE;
            p.list_stride = mask && mask->nmasks > 1 ? mask->nblk + 1 : 0;
            e = attn::launch_fwd_fused(desc->d, p, mask ? mask->row_ptr : nullptr, mask ? mask->col_idx : nullptr, s);
            break;
        }
        case Path::kLargeD: {
            char* ws = static_cast<char*>(workspace);
            LargeDParams p = larged_params(desc);
            p.Q = static_cast<const __bf16*>(Q);
            p.K = static_cast<const __bf16*>(K);
            p.V = static_cast<const __bf16*>(V);
            p.Oout = static_cast<__bf16*>(O);
            p.LSEout = LSE;
            p.stat_m = reinterpret_cast<float*>(ws);
            p.stat_l = reinterpret_cast<float*>(ws + stat_bytes(desc));
            p.P = reinterpret_cast<__bf16*>(ws + 2 * stat_bytes(desc));
            e = attn::launch_larged(false, p, s);
            break;
        }
        default: {
            GenericParams p = generic_params(desc, mask);
            p.Q = Q;
            p.K = K;
            p.V = V;
            p.O = O;
            p.LSE_out = LSE;
            e = attn::launch_generic(desc->dtype == ATTN_BF16, false, p, s);
            break;
        }
    }
    return e == hipSuccess ? ATTN_OK : ATTN_ERR_DEVICE;
}

attn_status attn_bwd(const attn_desc* desc, const void* Q, const void* K, const void* V, const void* O,
                     const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                     size_t workspace_bytes, void* stream) {
    return bwd_impl(desc, nullptr, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, stream);
}

attn_status attn_bwd_noalloc(const attn_desc* desc, const void* Q, const void* K, const void* V, const void* O,
                             const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* stream) {
    attn_status st = check_desc(desc);
    if (st != ATTN_OK) return st;
    if (bwd_path(desc, nullptr) == Path::kNone) return ATTN_ERR_UNSUPPORTED;
    if (is_empty(desc)) return ATTN_OK;
    if (attn_workspace_bytes(desc, nullptr) > (size_t)ATTN_NOALLOC_SCRATCH_BYTES) return ATTN_ERR_WORKSPACE;
    void* ptr = nullptr;
    if (scratch_address(&ptr) != hipSuccess) return ATTN_ERR_DEVICE;
    return bwd_impl(desc, nullptr, Q, K, V, O, dO, LSE, dQ, dK, dV, ptr, ATTN_NOALLOC_SCRATCH_BYTES, stream);
}

attn_status attn_bwd_blocksparse(const attn_desc* desc, const attn_blockmask* mask, const void* Q,
                                 const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                                 void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                                 void* stream) {
    if (!mask) return ATTN_ERR_INVALID_ARG;
    return bwd_impl(desc, mask, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, stream);
}

size_t attn_wgrad_workspace_bytes(const attn_desc* desc) {
    if (wgrad_check(desc) != ATTN_OK) return 0;
    if (is_empty(desc)) return 256;
    const WgradLayout l = wgrad_layout(desc);
    return l.total;
}

attn_status attn_bwd_wgrad(const attn_desc* desc, const void* A1, const void* A2, const void* A3, const void* X,
                           const void* Y, const void* dO, float* g, void* workspace, size_t workspace_bytes,
                           void* stream) {
    attn_status st = wgrad_check(desc);
    if (st != ATTN_OK) return st;
    if ((long)desc->batch * desc->heads == 0) return ATTN_OK;
    if (desc->n == 0) {  // a sum over no rows: g = 0
        if (!g || !aligned16(g)) return ATTN_ERR_INVALID_ARG;
        const hipError_t e0 = attn::launch_wgrad_zero(desc->d, desc->batch * desc->heads, g,
                                                      static_cast<hipStream_t>(stream));
        return e0 == hipSuccess ? ATTN_OK : ATTN_ERR_DEVICE;
    }
    if (!A1 || !A2 || !A3 || !X || !Y || !dO || !g) return ATTN_ERR_INVALID_ARG;
    if (!(aligned16(A1) && aligned16(A2) && aligned16(A3) && aligned16(X) && aligned16(Y) && aligned16(dO) &&
          aligned16(g)))
        return ATTN_ERR_INVALID_ARG;
    const WgradLayout l = wgrad_layout(desc);
    if (!workspace || workspace_bytes < l.total || !aligned16(workspace)) return ATTN_ERR_WORKSPACE;
    char* ws = static_cast<char*>(workspace);
    attn::WgradParams p;
    std::memset(&p, 0, sizeof(p));
    p.A1 = static_cast<const __bf16*>(A1);
    p.A2 = static_cast<const __bf16*>(A2);
    p.A3 = static_cast<const __bf16*>(A3);
    p.X = static_cast<const __bf16*>(X);
    p.Y = static_cast<const __bf16*>(Y);
    p.dO = static_cast<const __bf16*>(dO);
    p.g = g;
    p.Q = reinterpret_cast<__bf16*>(ws + l.q);
    p.V = reinterpret_cast<__bf16*>(ws + l.v);
    p.O = reinterpret_cast<__bf16*>(ws + l.o);
    p.dQ = reinterpret_cast<__bf16*>(ws + l.dq);
    p.LSE = reinterpret_cast<float*>(ws + l.lse);
    p.delta = reinterpret_cast<float*>(ws + l.delta);
    p.partial = reinterpret_cast<float*>(ws + l.partial);
    p.batch = desc->batch;
    p.heads = desc->heads;
    p.n = desc->n;
    p.scale = desc->scale;
    p.causal = desc->causal;
    const hipError_t e = attn::launch_wgrad_fused(desc->d, p, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? ATTN_OK : ATTN_ERR_DEVICE;
}

attn_status attn_blockmask_validate(int32_t block, int32_t nblk, int32_t n, int32_t nmasks, const int32_t* row_ptr,
                                    const int32_t* col_idx, const int32_t* col_ptr, const int32_t* row_idx) {
    if (block < 1 || nblk < 0 || n < 0 || nmasks < 0) return ATTN_ERR_INVALID_ARG;
    if ((long)nblk != ((long)n + block - 1) / block) return ATTN_ERR_INVALID_ARG;
    if (!row_ptr || !col_ptr || (nblk > 0 && (!col_idx || !row_idx))) return ATTN_ERR_INVALID_ARG;
    if (row_ptr[0] != 0 || col_ptr[0] != 0) return ATTN_ERR_INVALID_ARG;
    std::vector<unsigned char> keep((size_t)nblk * nblk);
    const int masks = nmasks > 1 ? nmasks : 1;
    for (int m = 0; m < masks; ++m) {
        const int32_t* rp = row_ptr + (size_t)m * (nblk + 1);
        const int32_t* cp = col_ptr + (size_t)m * (nblk + 1);
        // the lists of mask m continue where those of mask m - 1 end
        if (m > 0 && (rp[0] != rp[-1] || cp[0] != cp[-1])) return ATTN_ERR_INVALID_ARG;
        for (int a = 0; a < nblk; ++a) {
            if (rp[a + 1] < rp[a] || cp[a + 1] < cp[a]) return ATTN_ERR_INVALID_ARG;
            if (rp[a + 1] - rp[a] > nblk || cp[a + 1] - cp[a] > nblk) return ATTN_ERR_INVALID_ARG;
        }
        if (rp[nblk] != cp[nblk] || rp[0] != cp[0]) return ATTN_ERR_INVALID_ARG;
        std::fill(keep.begin(), keep.end(), 0);
        for (int i = 0; i < nblk; ++i)
            for (int a = rp[i]; a < rp[i + 1]; ++a) {
                const int j = col_idx[a];
                if (j < 0 || j >= nblk) return ATTN_ERR_INVALID_ARG;
                if (a > rp[i] && col_idx[a - 1] >= j) return ATTN_ERR_INVALID_ARG;
                keep[(size_t)i * nblk + j] = 1;
            }
        for (int j = 0; j < nblk; ++j)
            for (int a = cp[j]; a < cp[j + 1]; ++a) {
                const int i = row_idx[a];
                if (i < 0 || i >= nblk) return ATTN_ERR_INVALID_ARG;
                if (a > cp[j] && row_idx[a - 1] >= i) return ATTN_ERR_INVALID_ARG;
                if (!keep[(size_t)i * nblk + j]) return ATTN_ERR_INVALID_ARG;
            }
    }
    return ATTN_OK;
}

const char* attn_status_str(attn_status s) {
    switch (s) {
        case ATTN_OK: return "ok";
        case ATTN_ERR_INVALID_ARG: return "invalid argument";
        case ATTN_ERR_UNSUPPORTED: return "unsupported configuration";
        case ATTN_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case ATTN_ERR_DEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
#pragma GCC visibility pop
