// Exercises the host-side validation of libattn_mi355x (no GPU needed: every call here is either
// a pure host function or is rejected before anything is launched).  Built by
// tests/test_sanitizers.py with the host pass of attn_api.hip under AddressSanitizer and UBSan.
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/attn_mi355x.h"

static int fails = 0;
#define EXPECT(cond)                                            \
    do {                                                        \
        if (!(cond)) {                                          \
            std::printf("FAILED line %d: %s\n", __LINE__, #cond); \
            ++fails;                                            \
        }                                                       \
    } while (0)

static attn_desc make_desc(int b, int h, int n, int d, int dtype) {
    attn_desc x;
    std::memset(&x, 0, sizeof(x));
    x.batch = b; x.heads = h; x.n = n; x.d = d;
    x.scale = 0.125f; x.causal = 0; x.dtype = dtype; x.bwd_tiling = ATTN_BWD_AUTO;
    x.stride_n = d; x.stride_h = (int64_t)n * d; x.stride_b = (int64_t)h * n * d;
    return x;
}

int main() {
    for (int s = 0; s <= 5; ++s) EXPECT(attn_status_str((attn_status)s) != nullptr);
    // workspace sizes: valid shapes on every path, every tiling, and invalid ones
    for (int d : {8, 40, 64, 96, 128, 256, 512, 1024})
        for (int n : {0, 1, 127, 4096})
            for (int dtype : {ATTN_F32, ATTN_BF16})
                for (int tiling = 0; tiling <= 3; ++tiling) {
                    attn_desc x = make_desc(2, 3, n, d, dtype);
                    x.bwd_tiling = tiling;
                    (void)attn_workspace_bytes(&x, nullptr);
                    (void)attn_wgrad_workspace_bytes(&x);
                }
    EXPECT(attn_workspace_bytes(nullptr, nullptr) == 0);
    attn_desc bad = make_desc(1, 1, 128, 64, ATTN_BF16);
    bad.bwd_tiling = 99;
    EXPECT(attn_workspace_bytes(&bad, nullptr) == 0);
    bad = make_desc(1, 1, 128, 64, ATTN_BF16);
    bad.stride_n = 63;
    EXPECT(attn_workspace_bytes(&bad, nullptr) == 0);

    // block-mask validation on host arrays: a good mask, then malformed ones
    {
        const int nblk = 4;
        std::vector<int32_t> rp = {0, 1, 3, 5, 8}, ci = {0, 0, 1, 1, 2, 0, 2, 3};
        std::vector<int32_t> cp = {0, 3, 5, 7, 8}, ri = {0, 1, 3, 1, 2, 2, 3, 3};
        EXPECT(attn_blockmask_validate(128, nblk, 500, 1, rp.data(), ci.data(), cp.data(), ri.data()) == ATTN_OK);
        std::vector<int32_t> ci2 = ci;
        ci2[7] = 9;  // out of range
        EXPECT(attn_blockmask_validate(128, nblk, 500, 1, rp.data(), ci2.data(), cp.data(), ri.data()) != ATTN_OK);
        ci2 = ci;
        ci2[6] = -1;
        EXPECT(attn_blockmask_validate(128, nblk, 500, 1, rp.data(), ci2.data(), cp.data(), ri.data()) != ATTN_OK);
        std::vector<int32_t> rp2 = rp;
        rp2[2] = 0;  // not monotone
        EXPECT(attn_blockmask_validate(128, nblk, 500, 1, rp2.data(), ci.data(), cp.data(), ri.data()) != ATTN_OK);
        rp2 = rp;
        rp2[4] = 1 << 30;  // a list longer than the matrix is wide
        EXPECT(attn_blockmask_validate(128, nblk, 500, 1, rp2.data(), ci.data(), cp.data(), ri.data()) != ATTN_OK);
        std::vector<int32_t> ri2 = ri;
        ri2[0] = 2;  // orientations disagree
        EXPECT(attn_blockmask_validate(128, nblk, 500, 1, rp.data(), ci.data(), cp.data(), ri2.data()) != ATTN_OK);
        EXPECT(attn_blockmask_validate(128, nblk, 700, 1, rp.data(), ci.data(), cp.data(), ri.data()) != ATTN_OK);
        EXPECT(attn_blockmask_validate(128, nblk, 500, 1, nullptr, ci.data(), cp.data(), ri.data()) != ATTN_OK);
        EXPECT(attn_blockmask_validate(0, nblk, 500, 1, rp.data(), ci.data(), cp.data(), ri.data()) != ATTN_OK);
        // two masks, concatenated
        std::vector<int32_t> rpp = {0, 1, 2, 2, 4}, cii = {0, 1, 1, 0}, cpp = {0, 1, 2, 3, 4}, rii = {0, 1, 1, 0};
        // mask 0: [[1,0],[0,1]]; mask 1: [[0,1],[1,0]]  (nblk = 2: pointer arrays of 3 entries each)
        std::vector<int32_t> r2 = {0, 1, 2, 2, 3, 4}, c2 = {0, 1, 1, 0}, p2 = {0, 1, 2, 2, 3, 4}, i2 = {0, 1, 1, 0};
        EXPECT(attn_blockmask_validate(64, 2, 128, 2, r2.data(), c2.data(), p2.data(), i2.data()) == ATTN_OK);
        (void)rpp; (void)cii; (void)cpp; (void)rii;
    }
    // calls that must be rejected on the host: null tensors, misaligned pointers, missing workspace,
    // malformed mask descriptors, tilings that do not exist for the shape
    {
        attn_desc x = make_desc(1, 2, 256, 128, ATTN_BF16);
        void* P = reinterpret_cast<void*>(0x1000);
        float* L = reinterpret_cast<float*>(0x2000);
        EXPECT(attn_fwd(&x, nullptr, nullptr, P, P, P, L, nullptr, 0, nullptr) == ATTN_ERR_INVALID_ARG);
        EXPECT(attn_fwd(&x, nullptr, reinterpret_cast<void*>(0x1004), P, P, P, L, nullptr, 0, nullptr) ==
               ATTN_ERR_INVALID_ARG);
        EXPECT(attn_bwd(&x, P, P, P, P, P, L, P, P, P, nullptr, 0, nullptr) == ATTN_ERR_WORKSPACE);
        EXPECT(attn_bwd(&x, P, P, P, P, P, L, P, P, P, P, 16, nullptr) == ATTN_ERR_WORKSPACE);
        EXPECT(attn_bwd_blocksparse(&x, nullptr, P, P, P, P, P, L, P, P, P, P, 1 << 20, nullptr) ==
               ATTN_ERR_INVALID_ARG);
        attn_blockmask m;
        std::memset(&m, 0, sizeof(m));
        m.block = 128; m.nblk = 3;  // wrong for n = 256
        EXPECT(attn_bwd_blocksparse(&x, &m, P, P, P, P, P, L, P, P, P, P, 1 << 20, nullptr) == ATTN_ERR_INVALID_ARG);
        attn_desc y = make_desc(1, 1, 128, 256, ATTN_BF16);
        y.bwd_tiling = ATTN_BWD_ONEPASS_K128;
        EXPECT(attn_bwd(&y, P, P, P, P, P, L, P, P, P, P, 1 << 20, nullptr) == ATTN_ERR_UNSUPPORTED);
        attn_desc z = make_desc(1, 4, 1 << 20, 64, ATTN_BF16);
        EXPECT(attn_bwd_noalloc(&z, P, P, P, P, P, L, P, P, P, nullptr) == ATTN_ERR_WORKSPACE);
        attn_desc e = make_desc(3, 0, 128, 64, ATTN_BF16);
        EXPECT(attn_bwd(&e, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0,
                        nullptr) == ATTN_OK);
        EXPECT(attn_bwd_noalloc(&e, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                nullptr) == ATTN_OK);
        double flops = 0;
        EXPECT(attn_mfma_ceiling(0, 0, L, &flops, nullptr) == ATTN_ERR_INVALID_ARG);
        EXPECT(attn_bwd_wgrad(&y, P, P, P, P, P, P, L, nullptr, 0, nullptr) == ATTN_ERR_WORKSPACE);
    }
    std::printf("host api driver: %d failed\n", fails);
    return fails ? 1 : 0;
}
