// Runs the HOST logic of libflexsp (plan building for ordinary and key-shard plans, plan inspection,
// argument validation of every entry point, the planner's dynamic programmes) under AddressSanitizer
// and UndefinedBehaviorSanitizer.  csrc/flexsp_host.hip and csrc/planner.hip are compiled into this
// program with the sanitizers on; the kernel launchers they reference are replaced by stubs that
// fail, so nothing here needs or touches a GPU (every context is host-only).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "flexsp_internal.h"

namespace flexsp {
hipError_t launch_pack(const void *, void *, int64_t, int, int, int, int, bool, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_pack_many(int, const void *const *, void *const *, int64_t, const int32_t *, int, int, int, bool,
                            hipStream_t) { return hipErrorUnknown; }
hipError_t launch_attn_fwd(const AttnArgs &, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_attn_fwd_kvshard(const AttnArgs &, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_attn_bwd_dkv(const AttnArgs &, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_attn_bwd_dq(const AttnArgs &, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_attn_bwd_dkv_kvshard(const AttnArgs &, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_attn_bwd_dq_kvshard(const AttnArgs &, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_lse_merge(const uint16_t *, const float *, const uint16_t *, const float *, uint16_t *, float *, int64_t,
                            int, int, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_lse_merge_acc(float *, float *, const uint16_t *, const float *, uint16_t *, int64_t, int, int, int32_t,
                                int32_t, int32_t, int32_t, int32_t, int32_t, hipStream_t) { return hipErrorUnknown; }
hipError_t static_scratch_init(int) { return hipErrorUnknown; }
}  // namespace flexsp

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "FAILED: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main()
{
    flexsp_ctx *ctx = nullptr;
    CHECK(flexsp_ctx_create(&ctx, -1) == FLEXSP_OK);
    unsigned seed = 12345;
    auto rnd = [&](int lo, int hi) { seed = seed * 1664525u + 1013904223u; return lo + (int)((seed >> 8) % (unsigned)(hi - lo + 1)); };
    for (int trial = 0; trial < 40; trial++) {
        const int B = rnd(0, 40), Hkv = rnd(1, 3), G = rnd(1, 4), causal = rnd(0, 1);
        std::vector<int32_t> cu(B + 1, 0), cu_k(B + 1, 0), shift(B > 0 ? B : 1, 0);
        for (int b = 0; b < B; b++) {
            const int kind = rnd(0, 9);
            cu[b + 1] = cu[b] + (kind == 0 ? 0 : kind == 1 ? rnd(3000, 20000) : rnd(1, 700));
            cu_k[b + 1] = cu_k[b] + rnd(0, 900);
            shift[b] = rnd(-500, 500);
        }
        flexsp_plan *p = nullptr;
        CHECK(flexsp_plan_create(ctx, cu.data(), B, Hkv * G, Hkv, trial % 2 ? 64 : 128, causal, &p) == FLEXSP_OK);
        for (int pass = 0; pass < 3; pass++) {
            const int64_t n = flexsp_plan_num_items(p, pass);
            CHECK(n >= 0);
            std::vector<flexsp_item> items((size_t)n + 1);
            int64_t offs[16];
            CHECK(flexsp_plan_get_items(p, pass, items.data(), n, offs) == FLEXSP_OK);
            CHECK(offs[0] == 0 && offs[flexsp_ctx_num_xcd(ctx)] == n);
            CHECK(flexsp_plan_tile_rows(p, pass) > 0);
        }
        (void)flexsp_attn_bwd_workspace_bytes(p);
        flexsp_plan_destroy(p);
        CHECK(flexsp_plan_create_kvshard(ctx, cu.data(), cu_k.data(), shift.data(), B, Hkv * G, Hkv, 128, causal, &p) == FLEXSP_OK);
        const int64_t n = flexsp_plan_num_items(p, FLEXSP_PASS_FWD);
        std::vector<flexsp_item> items((size_t)n + 1);
        CHECK(flexsp_plan_get_items(p, FLEXSP_PASS_FWD, items.data(), n, nullptr) == FLEXSP_OK);
        for (int64_t i = 0; i < n; i++) CHECK(items[i].seq_start >= 0 && items[i].seq_start < B);
        for (int pass : {FLEXSP_PASS_BWD_DKV, FLEXSP_PASS_BWD_DQ}) {
            const int64_t m = flexsp_plan_num_items(p, pass);
            CHECK(m >= 0);
            std::vector<flexsp_item> more((size_t)m + 1);
            CHECK(flexsp_plan_get_items(p, pass, more.data(), m, nullptr) == FLEXSP_OK);
            for (int64_t i = 0; i < m; i++) CHECK(more[i].seq_start >= 0 && more[i].seq_start < B);
        }
        flexsp_plan_destroy(p);
    }
    // validation paths of the hot calls (nothing is launched: the context is host-only)
    {
        const int32_t cu[2] = {0, 8};
        flexsp_plan *p = nullptr;
        CHECK(flexsp_plan_create(ctx, cu, 1, 2, 2, 64, 1, &p) == FLEXSP_OK);
        alignas(16) static char buf[4096];
        flexsp_tensor t{buf, 128, 64}, bad{buf + 2, 128, 64};
        float *lse = (float *)(buf + 2048);
        CHECK(flexsp_attn_varlen_fwd(ctx, p, t, t, t, nullptr, 0, 2, 0, 2, 1, 0.f, t, lse, nullptr) == FLEXSP_NO_DEVICE);
        CHECK(flexsp_attn_varlen_fwd(ctx, p, bad, t, t, nullptr, 0, 2, 0, 2, 1, 0.f, t, lse, nullptr) == FLEXSP_INVALID_ARGUMENT);
        CHECK(flexsp_attn_varlen_bwd(ctx, p, t, t, t, t, t, lse, nullptr, 0, 2, 0, 2, 1, 0.f, t, t, t, 7, nullptr) == FLEXSP_UNSUPPORTED);
        CHECK(flexsp_attn_varlen_fwd_kvshard(ctx, p, t, t, t, 0, 2, 0, 2, 1, 0.f, t, lse, nullptr) == FLEXSP_PLAN_MISMATCH);
        CHECK(flexsp_attn_varlen_bwd_kvshard(ctx, p, t, t, t, t, t, lse, 0, 2, 0, 2, 1, 0.f, t, t, t, FLEXSP_F32, 1, nullptr) == FLEXSP_PLAN_MISMATCH);
        {
            const int32_t cq[2] = {0, 8}, ck[2] = {0, 5}, sh[1] = {3};
            flexsp_plan *sp = nullptr;
            CHECK(flexsp_plan_create_kvshard(ctx, cq, ck, sh, 1, 2, 2, 64, 1, &sp) == FLEXSP_OK);
            CHECK(flexsp_attn_varlen_bwd_kvshard(ctx, sp, t, t, t, t, t, lse, 0, 2, 0, 2, 1, 0.f, t, t, t, FLEXSP_BF16, 1, nullptr) == FLEXSP_UNSUPPORTED);
            CHECK(flexsp_attn_varlen_bwd_kvshard(ctx, sp, t, t, t, t, t, lse, 0, 2, 0, 2, 1, 0.f, t, t, t, FLEXSP_F32, 2, nullptr) == FLEXSP_INVALID_ARGUMENT);
            CHECK(flexsp_attn_varlen_bwd_kvshard(ctx, sp, t, bad, t, t, t, lse, 0, 2, 0, 2, 1, 0.f, t, t, t, FLEXSP_F32, 1, nullptr) == FLEXSP_INVALID_ARGUMENT);
            CHECK(flexsp_attn_varlen_bwd_kvshard(ctx, sp, t, t, t, t, t, lse, 0, 2, 0, 2, 1, 0.f, t, t, t, FLEXSP_F32, 1, nullptr) == FLEXSP_NO_DEVICE);
            CHECK(flexsp_attn_varlen_fwd_kvshard_acc(ctx, sp, t, t, t, 0, 2, 0, 2, 1, 0.f, t, lse, flexsp_tensor{nullptr, 0, 0}, nullptr) == FLEXSP_NO_DEVICE);
            CHECK(flexsp_attn_varlen_fwd_kvshard_acc(ctx, sp, t, t, t, 0, 2, 0, 2, 1, 0.f, t, nullptr, t, nullptr) == FLEXSP_INVALID_ARGUMENT);
            CHECK(flexsp_attn_varlen_fwd_kvshard_acc(ctx, sp, t, t, t, 0, 2, 0, 2, 1, 0.f, t, lse, bad, nullptr) == FLEXSP_INVALID_ARGUMENT);
            flexsp_plan_destroy(sp);
        }
        CHECK(flexsp_lse_merge(ctx, t, lse, t, lse, t, lse, 8, 2, 64, nullptr) == FLEXSP_NO_DEVICE);
        CHECK(flexsp_lse_merge(ctx, t, lse, t, lse, t, lse, 8, 2, 40, nullptr) == FLEXSP_UNSUPPORTED);
        CHECK(flexsp_attn_varlen_fwd_kvshard_acc(ctx, p, t, t, t, 0, 2, 0, 2, 1, 0.f, t, lse, flexsp_tensor{nullptr, 0, 0}, nullptr) == FLEXSP_PLAN_MISMATCH);
        CHECK(flexsp_lse_merge_acc(ctx, t, lse, t, lse, flexsp_tensor{nullptr, 0, 0}, 8, 2, 64, nullptr) == FLEXSP_NO_DEVICE);
        CHECK(flexsp_lse_merge_acc(ctx, t, lse, t, lse, bad, 8, 2, 64, nullptr) == FLEXSP_INVALID_ARGUMENT);
        CHECK(flexsp_lse_merge_acc(ctx, t, nullptr, t, lse, t, 8, 2, 64, nullptr) == FLEXSP_INVALID_ARGUMENT);
        CHECK(flexsp_pack(ctx, buf, buf + 2048, 4, 4, 8, 2, 2, nullptr) == FLEXSP_NO_DEVICE);
        CHECK(flexsp_pack(ctx, buf, buf + 100, 4, 4, 8, 2, 2, nullptr) == FLEXSP_INVALID_ARGUMENT);
        flexsp_plan_destroy(p);
        const int32_t dec[3] = {0, 5, 3};
        CHECK(flexsp_plan_create(ctx, dec, 2, 2, 2, 64, 1, &p) == FLEXSP_INVALID_ARGUMENT);
    }
    // the planner's exact pieces
    for (int trial = 0; trial < 30; trial++) {
        const int K = rnd(1, 300), Q = rnd(1, 20), M = rnd(1, K);
        std::vector<int64_t> lens(K), limits(Q), ends(M);
        std::vector<int32_t> bucket(K);
        for (auto &s : lens) s = rnd(0, 5) == 0 ? rnd(10000, 200000) : rnd(1, 4000);
        int32_t nb = 0;
        int64_t err = -1, mx = -1;
        CHECK(flexsp_bucket_dp(lens.data(), K, Q, limits.data(), &nb, bucket.data(), &err) == FLEXSP_OK);
        CHECK(nb >= 1 && nb <= Q && err >= 0);
        for (int i = 0; i < K; i++) CHECK(bucket[i] >= 0 && bucket[i] < nb && lens[i] <= limits[bucket[i]]);
        CHECK(flexsp_chunk_dp(lens.data(), K, M, ends.data(), &mx) == FLEXSP_OK);
        CHECK(ends[M - 1] == K && mx > 0);
    }
    CHECK(flexsp_min_microbatches(1000, 300) == 4);
    CHECK(flexsp_bucket_dp(nullptr, 3, 2, nullptr, nullptr, nullptr, nullptr) == FLEXSP_INVALID_ARGUMENT);
    flexsp_ctx_destroy(ctx);
    std::puts("host logic under sanitizers: ok");
    return 0;
}
