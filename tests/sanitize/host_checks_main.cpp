// Driver for a sanitized build of libdsv's HOST side: descriptor checks, workspace layouts, launch tables and
// split plans run for every benchmark shape and for edge shapes; every call below returns before any kernel
// launch (a query, or an argument error), so it runs on a machine without a GPU.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "dsv.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); std::exit(1); } } while (0)

static dsv_problem make(int B, int H, int L, int d, int r, int dtype, const std::vector<int32_t> &k, uint32_t flags)
{
    dsv_problem p{};
    p.B = B; p.H = H; p.L = L; p.d = d; p.r = r; p.dtype = dtype; p.k_per_head = k.data(); p.scale = 0.125f; p.flags = flags;
    return p;
}

static void queries(const dsv_problem &p)
{
    std::vector<int64_t> off((size_t)p.B * p.H + 1);
    CHECK(dsv_idx_offsets(&p, off.data()) == DSV_OK);
    CHECK(off[0] == 0 && off.back() > 0);
    size_t a = dsv_lowrank_topk_workspace(&p), b = dsv_lowrank_topk_t_workspace(&p);
    CHECK(a > 0 && b >= a);
    size_t f = dsv_sparse_attn_fwd_workspace(&p), q = dsv_sparse_attn_bwd_dq_workspace(&p);
    size_t kv = dsv_sparse_attn_bwd_dkdv_workspace(&p), w = dsv_sparse_attn_bwd_workspace(&p);
    size_t wt = dsv_sparse_attn_bwd_t_workspace(&p), tr = dsv_idx_transpose_workspace(&p);
    CHECK(w >= (size_t)off.back() * 4 && wt >= q && wt >= kv && tr >= (size_t)p.B * p.H * p.L * 4);
    CHECK(dsv_idx_validate_workspace(&p) == 256);
    (void)f;
    // workspace one byte short / missing: rejected before anything is launched
    void *one = reinterpret_cast<void *>(256);
    CHECK(dsv_lowrank_topk(&p, one, one, one, one, static_cast<int32_t *>(one), one, a - 1, nullptr) == DSV_EWORKSPACE);
    CHECK(dsv_lowrank_topk_t(&p, one, one, one, one, static_cast<int32_t *>(one), static_cast<int32_t *>(one),
                             static_cast<int64_t *>(one), nullptr, 0, nullptr) == DSV_EWORKSPACE);
    CHECK(dsv_sparse_attn_bwd(&p, one, one, one, static_cast<int32_t *>(one), one, static_cast<float *>(one), one, one, one,
                              one, one, w - 1, nullptr) == DSV_EWORKSPACE);
    if (q) CHECK(dsv_sparse_attn_bwd_dq(&p, one, one, one, static_cast<int32_t *>(one), one, static_cast<float *>(one), one,
                                        one, static_cast<float *>(one), one, q - 1, nullptr) == DSV_EWORKSPACE);
}

int main()
{
    const uint32_t flags[2] = {0u, DSV_FLAG_SORTED_INDEX};
    for (uint32_t fl : flags) {
        queries(make(1, 2, 1024, 64, 16, DSV_F32, {128, 128}, fl));
        queries(make(1, 24, 32768, 128, 16, DSV_BF16, std::vector<int32_t>(24, 2048), fl));
        queries(make(1, 6, 131072, 128, 16, DSV_BF16, std::vector<int32_t>(6, 8192), fl));
        std::vector<int32_t> mixed;
        for (int h = 0; h < 24; ++h) mixed.push_back(512 << (h % 6));
        queries(make(1, 24, 65536, 128, 32, DSV_BF16, mixed, fl));
        queries(make(1, 2, 524288, 128, 32, DSV_BF16, {16384, 16384}, fl));
        queries(make(3, 70, 33, 64, 64, DSV_BF16, std::vector<int32_t>(70, 33), fl));   // more pairs than one launch table
        queries(make(1, 1, 1, 64, 16, DSV_F32, {1}, fl));
    }
    std::vector<int32_t> k2 = {8, 8};
    dsv_problem bad = make(1, 2, 64, 64, 16, DSV_BF16, k2, 0);
    bad.flags = 2u;
    CHECK(dsv_lowrank_topk_workspace(&bad) == 0);
    bad = make(1, 2, 64, 80, 16, DSV_BF16, k2, 0);
    CHECK(dsv_sparse_attn_fwd_workspace(&bad) == 0);
    CHECK(dsv_idx_offsets(nullptr, nullptr) == DSV_EINVAL);
    CHECK(dsv_status_string(DSV_EHIP) != nullptr && dsv_version() != nullptr);
    float ms = 0.f;
    CHECK(dsv_kernel_ms(99, &ms) == DSV_EINVAL && dsv_kernel_ms(0, nullptr) == DSV_EINVAL);
    // threshold search: the choice per head and the sample size are host arithmetic, for any (L, k) and mode
    for (int mode = 0; mode < 3; ++mode) {
        CHECK(dsv_threshold_search(mode) >= 0);
        for (int L : {1, 31, 4095, 4096, 5000, 16384, 131072, 524288, 1 << 24, 0x7FFFFFF0})
            for (int k : {-1, 0, 1, 7, 64, 1000, 4096, L / 16, L / 4, L / 2, L - 1, L, L + 1}) {
                const int n = dsv_threshold_sample_keys(L, k);
                CHECK(n == 0 || (mode != 1 && n % 32 == 0 && n >= 2048 && n <= L / 2 && k >= 1 && k < L));
            }
    }
    CHECK(dsv_threshold_search(7) == -1 && dsv_threshold_search(0) == 2);
    // query grouping: layouts of the group kernels and of the general path, argument checks
    {
        void *one = reinterpret_cast<void *>(256);
        std::vector<int32_t> k6(6, 8192);
        for (uint32_t fl : flags) {
            dsv_problem p = make(1, 6, 131072, 128, 16, DSV_BF16, k6, fl);
            const dsv_grouping g8{32, 64, 64, 2, 2, 2}, g32{32, 64, 64, 4, 4, 4}, g128{32, 64, 64, 8, 4, 4}, bad{32, 64, 64, 3, 2, 2};   // g32: 64 members, the general path
            CHECK(dsv_lowrank_topk_grouped_workspace(&p, &g8) > 0 && dsv_lowrank_topk_grouped_workspace(&p, &bad) == 0);
            CHECK((dsv_sparse_attn_fwd_grouped_workspace(&p, &g8) > 0) == (fl != 0));
            CHECK(dsv_sparse_attn_fwd_grouped_workspace(&p, &g32) > (size_t)6 * 131072 * 8192 * 4);   // holds the expanded index
            CHECK(dsv_sparse_attn_bwd_grouped_workspace(&p, &g32) > dsv_sparse_attn_bwd_grouped_workspace(&p, &g8));
            CHECK(dsv_sparse_attn_fwd_grouped(&p, &g128, one, one, one, static_cast<int32_t *>(one), one, static_cast<float *>(one),
                                              nullptr, 0, nullptr) == DSV_EUNSUPPORTED);
            CHECK(dsv_sparse_attn_fwd_grouped(&p, &bad, one, one, one, static_cast<int32_t *>(one), one, static_cast<float *>(one),
                                              nullptr, 0, nullptr) == DSV_EINVAL);
            CHECK(dsv_sparse_attn_bwd_grouped(&p, &g32, one, one, one, static_cast<int32_t *>(one), static_cast<int32_t *>(one),
                                              static_cast<int64_t *>(one), one, static_cast<float *>(one), one, one, one, one, one,
                                              16, nullptr) == DSV_EWORKSPACE);
            CHECK(dsv_group_overlap_workspace(&p) >= 48 && dsv_choose_grouping_workspace(&p) > dsv_group_overlap_workspace(&p));
            CHECK(dsv_group_overlap(&p, &g8, static_cast<int32_t *>(one), static_cast<float *>(one), nullptr, 0, nullptr) == DSV_EWORKSPACE);
            int32_t chosen = 7;
            const int32_t cubes[6] = {2, 2, 2, 1, 1, 1};
            CHECK(dsv_choose_grouping(&p, 32, 64, 64, nullptr, 2, static_cast<int32_t *>(one), 0.8f, &chosen, nullptr, one, 1 << 20,
                                      nullptr) == DSV_EINVAL);
            CHECK(dsv_choose_grouping(&p, 32, 64, 64, cubes, 0, static_cast<int32_t *>(one), 0.8f, &chosen, nullptr, one, 1 << 20,
                                      nullptr) == DSV_EINVAL);
            CHECK(dsv_choose_grouping(&p, 32, 64, 64, cubes, 2, static_cast<int32_t *>(one), 0.8f, &chosen, nullptr, one, 8,
                                      nullptr) == DSV_EWORKSPACE && chosen == 7);
        }
        std::vector<int32_t> k128 = {128, 128};
        dsv_problem f32p = make(1, 2, 1024, 64, 16, DSV_F32, k128, 0);
        const dsv_grouping g{8, 8, 16, 2, 2, 2};
        CHECK(dsv_sparse_attn_fwd_grouped_workspace(&f32p, &g) > 0);    // fp32 runs the general path
        CHECK(dsv_predictor_loss_workspace(&f32p, 64) > 0 && dsv_predictor_loss_workspace(&f32p, 0) == 0);
        CHECK(dsv_profile_sparsity_workspace(&f32p, 2000) == 0);        // more rows than tokens
    }
    std::printf("host checks sanitizer run ok\n");
    return 0;
}
