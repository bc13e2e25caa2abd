// Generic exact-arithmetic path: fp32 FMA only (no matrix cores, no reduced precision), any n,
// any d <= 512, any block edge for the block mask.  It serves the fp32 storage type and shapes
// the tiled bf16 kernels do not cover.  One wavefront owns one row; lanes split the other
// sequence dimension for the score-like quantities and the feature dimension for the outputs.
// Formulas: A, l, f, O, q, p of App. B.4 with the scale, mask and log-sum-exp readings.
#include "attn_common.hpp"
#include "attn_internal.hpp"

namespace attn {

constexpr int kMaxD = 512;
constexpr int kCols = kMaxD / 64;  // output columns per lane

template <typename T> __device__ __forceinline__ float ldf(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void stf(T* p, float v) { *p = (T)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}

template <typename T>
__device__ __forceinline__ float dot_row(const float* a_lds, const T* b, int d) {
    float s = 0.f;
    for (int k = 0; k < d; ++k) s = fmaf(a_lds[k], ldf(b + k), s);
    return s;
}

// Visible range of the other index for row r: ranges are whole blocks of the list (or one
// range 0..n when dense), clipped by the causal rule.  `row_is_query` picks the rule's side.
struct Ranges {
    const int32_t *ptr, *idx;
    int block, n, causal;
    __device__ __forceinline__ int count(int r) const { return ptr ? ptr[r / block + 1] - ptr[r / block] : 1; }
    __device__ __forceinline__ void get(int r, int a, bool row_is_query, int& lo, int& hi) const {
        lo = 0;
        hi = n;
        if (ptr) {
            const int b = idx[ptr[r / block] + a];
            lo = b * block;
            hi = min(n, lo + block);
        }
        if (causal) {
            if (row_is_query) hi = min(hi, r + 1);  // keys j <= i
            else lo = max(lo, r);                   // queries i >= j
        }
    }
};

template <typename T>
__global__ void __launch_bounds__(kThreads) generic_fwd_kernel(GenericParams p) {
    __shared__ float qs[4][kMaxD];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long rows = (long)p.batch * p.heads * p.n;
    const long r_raw = (long)blockIdx.x * 4 + w;
    const bool active = r_raw < rows;  // idle waves redo the last row and store nothing
    const long r = active ? r_raw : rows - 1;
    const int bh = (int)(r / p.n), i = (int)(r % p.n);
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const T *Q = (const T*)p.Q + base, *K = (const T*)p.K + base, *V = (const T*)p.V + base;
    T* O = (T*)p.O + base;
    for (int k = lane; k < p.d; k += 64) qs[w][k] = ldf(Q + (long)i * p.stride_n + k);
    __syncthreads();
    const Ranges rg{p.csr_ptr ? p.csr_ptr + (long)bh * p.mask_stride : nullptr, p.csr_idx, p.block, p.n, p.causal};
    const int nr = rg.count(i);
    float m = -__builtin_inff();
    for (int a = 0; a < nr; ++a) {
        int lo, hi;
        rg.get(i, a, true, lo, hi);
        for (int j = lo + lane; j < hi; j += 64) m = fmaxf(m, p.scale * dot_row(qs[w], K + (long)j * p.stride_n, p.d));
    }
    m = wave_max(m);
    float acc[kCols];
#pragma unroll
    for (int u = 0; u < kCols; ++u) acc[u] = 0.f;
    float l = 0.f;
    if (m != -__builtin_inff()) {
        for (int a = 0; a < nr; ++a) {
            int lo, hi;
            rg.get(i, a, true, lo, hi);
            for (int j0 = lo; j0 < hi; j0 += 64) {
                const int j = j0 + lane;
                float e = 0.f;
                if (j < hi) e = expf(p.scale * dot_row(qs[w], K + (long)j * p.stride_n, p.d) - m);
                l += e;
                const int cnt = min(64, hi - j0);
                for (int jj = 0; jj < cnt; ++jj) {
                    const float ej = __shfl(e, jj, 64);
#pragma unroll
                    for (int u = 0; u < kCols; ++u) {
                        const int k = lane + 64 * u;
                        if (k < p.d) acc[u] = fmaf(ej, ldf(V + (long)(j0 + jj) * p.stride_n + k), acc[u]);
                    }
                }
            }
        }
        l = wave_sum(l);
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int u = 0; u < kCols; ++u) {
        const int k = lane + 64 * u;
        if (active && k < p.d) stf(O + (long)i * p.stride_n + k, acc[u] * inv);
    }
    if (active && lane == 0) p.LSE_out[r] = l > 0.f ? m + logf(l) : -__builtin_inff();
}

template <typename T>
__global__ void __launch_bounds__(kThreads) generic_delta_kernel(GenericParams p) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long rows = (long)p.batch * p.heads * p.n;
    const long r_raw = (long)blockIdx.x * 4 + w;
    const bool active = r_raw < rows;  // idle waves redo the last row and store nothing
    const long r = active ? r_raw : rows - 1;
    const int bh = (int)(r / p.n), i = (int)(r % p.n);
    const long off = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h + (long)i * p.stride_n;
    float s = 0.f;
    for (int k = lane; k < p.d; k += 64) s = fmaf(ldf((const T*)p.O_in + off + k), ldf((const T*)p.dO + off + k), s);
    s = wave_sum(s);
    if (active && lane == 0) p.delta[r] = s;
}

// dQ_i = scale sum_j p_ij K_j, one wavefront per query row.
template <typename T>
__global__ void __launch_bounds__(kThreads) generic_dq_kernel(GenericParams p) {
    __shared__ float qs[4][kMaxD], gs[4][kMaxD];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long rows = (long)p.batch * p.heads * p.n;
    const long r_raw = (long)blockIdx.x * 4 + w;
    const bool active = r_raw < rows;  // idle waves redo the last row and store nothing
    const long r = active ? r_raw : rows - 1;
    const int bh = (int)(r / p.n), i = (int)(r % p.n);
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const T *Q = (const T*)p.Q + base, *K = (const T*)p.K + base, *V = (const T*)p.V + base, *G = (const T*)p.dO + base;
    for (int k = lane; k < p.d; k += 64) {
        qs[w][k] = ldf(Q + (long)i * p.stride_n + k);
        gs[w][k] = ldf(G + (long)i * p.stride_n + k);
    }
    __syncthreads();
    const float lse = p.LSE_in[r], v = p.delta[r];
    const Ranges rg{p.csr_ptr ? p.csr_ptr + (long)bh * p.mask_stride : nullptr, p.csr_idx, p.block, p.n, p.causal};
    const int nr = rg.count(i);
    float acc[kCols];
#pragma unroll
    for (int u = 0; u < kCols; ++u) acc[u] = 0.f;
    if (lse != -__builtin_inff()) {
        for (int a = 0; a < nr; ++a) {
            int lo, hi;
            rg.get(i, a, true, lo, hi);
            for (int j0 = lo; j0 < hi; j0 += 64) {
                const int j = j0 + lane;
                float pp = 0.f;
                if (j < hi) {
                    const float f = expf(p.scale * dot_row(qs[w], K + (long)j * p.stride_n, p.d) - lse);
                    pp = f * (dot_row(gs[w], V + (long)j * p.stride_n, p.d) - v);
                }
                const int cnt = min(64, hi - j0);
                for (int jj = 0; jj < cnt; ++jj) {
                    const float pj = __shfl(pp, jj, 64);
#pragma unroll
                    for (int u = 0; u < kCols; ++u) {
                        const int k = lane + 64 * u;
                        if (k < p.d) acc[u] = fmaf(pj, ldf(K + (long)(j0 + jj) * p.stride_n + k), acc[u]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kCols; ++u) {
        const int k = lane + 64 * u;
        if (active && k < p.d) stf((T*)p.dQ + base + (long)i * p.stride_n + k, acc[u] * p.scale);
    }
}

// dK_j = scale sum_i p_ij Q_i, dV_j = sum_i f_ij dO_i, one wavefront per key row.
template <typename T>
__global__ void __launch_bounds__(kThreads) generic_dkdv_kernel(GenericParams p) {
    __shared__ float ks[4][kMaxD], vs[4][kMaxD];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long rows = (long)p.batch * p.heads * p.n;
    const long r_raw = (long)blockIdx.x * 4 + w;
    const bool active = r_raw < rows;  // idle waves redo the last row and store nothing
    const long r = active ? r_raw : rows - 1;
    const int bh = (int)(r / p.n), j = (int)(r % p.n);
    const long base = (long)(bh / p.heads) * p.stride_b + (long)(bh % p.heads) * p.stride_h;
    const T *Q = (const T*)p.Q + base, *K = (const T*)p.K + base, *V = (const T*)p.V + base, *G = (const T*)p.dO + base;
    const float* lse = p.LSE_in + (long)bh * p.n;
    const float* dl = p.delta + (long)bh * p.n;
    for (int k = lane; k < p.d; k += 64) {
        ks[w][k] = ldf(K + (long)j * p.stride_n + k);
        vs[w][k] = ldf(V + (long)j * p.stride_n + k);
    }
    __syncthreads();
    const Ranges rg{p.csc_ptr ? p.csc_ptr + (long)bh * p.mask_stride : nullptr, p.csc_idx, p.block, p.n, p.causal};
    const int nr = rg.count(j);
    float ak[kCols], av[kCols];
#pragma unroll
    for (int u = 0; u < kCols; ++u) { ak[u] = 0.f; av[u] = 0.f; }
    for (int a = 0; a < nr; ++a) {
        int lo, hi;
        rg.get(j, a, false, lo, hi);
        // chunks start on multiples of 64 so that dense and block-list runs sum in the same order
        for (int i0 = lo & ~63; i0 < hi; i0 += 64) {
            const int i = i0 + lane;
            float f = 0.f, pp = 0.f;
            if (i >= lo && i < hi && lse[i] != -__builtin_inff()) {
                f = expf(p.scale * dot_row(ks[w], Q + (long)i * p.stride_n, p.d) - lse[i]);
                pp = f * (dot_row(vs[w], G + (long)i * p.stride_n, p.d) - dl[i]);
            }
            const int cnt = min(64, hi - i0);
            for (int ii = 0; ii < cnt; ++ii) {
                const float fi = __shfl(f, ii, 64), pi = __shfl(pp, ii, 64);
#pragma unroll
                for (int u = 0; u < kCols; ++u) {
                    const int k = lane + 64 * u;
                    if (k < p.d) {
                        av[u] = fmaf(fi, ldf(G + (long)(i0 + ii) * p.stride_n + k), av[u]);
                        ak[u] = fmaf(pi, ldf(Q + (long)(i0 + ii) * p.stride_n + k), ak[u]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kCols; ++u) {
        const int k = lane + 64 * u;
        if (active && k < p.d) {
            stf((T*)p.dK + base + (long)j * p.stride_n + k, ak[u] * p.scale);
            stf((T*)p.dV + base + (long)j * p.stride_n + k, av[u]);
        }
    }
}

template <typename T>
static hipError_t run_generic(const GenericParams& p, bool backward, hipStream_t stream) {
    const long rows = (long)p.batch * p.heads * p.n;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(kThreads);
    if (!backward) {
        hipLaunchKernelGGL(generic_fwd_kernel<T>, grid, block, 0, stream, p);
    } else {
        hipLaunchKernelGGL(generic_delta_kernel<T>, grid, block, 0, stream, p);
        hipLaunchKernelGGL(generic_dq_kernel<T>, grid, block, 0, stream, p);
        hipLaunchKernelGGL(generic_dkdv_kernel<T>, grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_generic(bool is_bf16, bool backward, const GenericParams& p, hipStream_t stream) {
    if (p.d > kMaxD) return hipErrorInvalidValue;
    return is_bf16 ? run_generic<__bf16>(p, backward, stream) : run_generic<float>(p, backward, stream);
}

}  // namespace attn
