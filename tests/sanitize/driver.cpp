// Host-side exerciser of the library's C ABI for sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer on the
// host code of executor.cpp / search.cpp).  No GPU is needed: kernels are never launched, HIP calls that need a device
// fail and are reported as statuses.  Exit code 0 = every check held; the sanitizers abort on their own findings.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <string>
#include <vector>
#include "../../include/gacer.h"

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); std::exit(1); } } while (0)

static void *const FAKE = (void *)0x10000;      // aligned, never dereferenced

// a tenant of n operators on 16 channels, 6x6, batch 8: 3x3 convolutions, or (pre_activation) every second and third operator
// a per-channel affine + ReLU and the 1x1 convolution behind it, the pair that the executor issues as one launch
struct Chain {
    std::vector<gacer_op> ops;
    std::vector<gacer_tensor> tensors;
    gacer_tenant desc;
    explicit Chain(int n, bool pre_activation = false)
    {
        tensors.push_back({8, 16, 6, 6, FAKE});
        for (int i = 0; i < n; ++i) {
            tensors.push_back({8, 16, 6, 6, FAKE});
            gacer_op op;
            std::memset(&op, 0, sizeof op);
            op.kind = GACER_CONV2D; op.in0 = i; op.in1 = -1; op.res = -1; op.out = i + 1;
            op.w = FAKE; op.bias = (const float *)FAKE;
            op.cin = 16; op.cout = 16; op.kh = op.kw = 3; op.stride = 1; op.pad = 1; op.groups = 1; op.act = GACER_ACT_RELU; op.alpha = 1.f;
            if (pre_activation && i % 3 == 1) {
                op.kind = GACER_AFFINE_ACT; op.w = nullptr; op.bias = nullptr; op.scale = op.shift = (const float *)FAKE;
                op.kh = op.kw = 1; op.pad = 0;
            } else if (pre_activation && i % 3 == 2) {
                op.kh = op.kw = 1; op.pad = 0;
            }
            ops.push_back(op);
        }
        std::memset(&desc, 0, sizeof desc);
        desc.n_ops = n; desc.ops = ops.data(); desc.n_tensors = (int)tensors.size(); desc.tensors = tensors.data();
        desc.input = 0; desc.output = n; desc.dtype = GACER_F32; desc.batch = 8;
    }
};

int main()
{
    std::mt19937 rng(7);
    for (int trial = 0; trial < 30; ++trial) {
        gacer_ctx *ctx = nullptr;
        CHECK(gacer_create(&ctx) == GACER_OK);
        const int NT = 2 + (int)(rng() % 3);
        std::vector<Chain> chains;
        chains.reserve(NT);
        std::vector<int> n_ops;
        for (int t = 0; t < NT; ++t) { n_ops.push_back(2 + (int)(rng() % 6)); chains.emplace_back(n_ops.back(), t % 2 == 1); }
        std::vector<gacer_tenant> descs;
        for (Chain &c : chains) { c.desc.ops = c.ops.data(); c.desc.tensors = c.tensors.data(); descs.push_back(c.desc); }
        CHECK(gacer_load_tenants(ctx, descs.data(), NT) == GACER_OK);
        {   // launch fusion: fewer launches with it when a pre-activation pair exists, one per operator without it
            int fused = 0, plain = 0, total = 0;
            for (int n : n_ops) total += n;
            CHECK(gacer_launch_count(ctx, GACER_MODE_SEQUENTIAL, &fused) == GACER_OK);
            CHECK(gacer_set_fuse_affine(ctx, 0) == GACER_OK);
            CHECK(gacer_launch_count(ctx, GACER_MODE_SEQUENTIAL, &plain) == GACER_OK && plain == total && fused <= plain);
            CHECK(gacer_set_fuse_affine(ctx, trial % 2) == GACER_OK);
        }
        // Matrix_P -> edges -> text -> plan -> installed
        const int n_ptr = (int)(rng() % 4);
        std::vector<int> P;
        for (int t = 0; t < NT; ++t) {
            std::vector<int> row;
            for (int j = 0; j < n_ptr; ++j) row.push_back((int)(rng() % (n_ops[t] + 1)));
            std::sort(row.begin(), row.end());
            P.insert(P.end(), row.begin(), row.end());
        }
        gacer_plan *edges = nullptr;
        CHECK(gacer_plan_from_pointers(ctx, P.empty() ? nullptr : P.data(), n_ptr, &edges) == GACER_OK);
        int sizes[3] = {5, 2, 1};
        gacer_split sp[2] = {{0, 0, GACER_AXIS_BATCH, 3, sizes, 1}, {1, 1, GACER_AXIS_COUT, 4, nullptr, 0}};
        gacer_plan plan = {2, sp, edges->n_sync, edges->sync};
        CHECK(gacer_set_plan(ctx, &plan) == GACER_OK);
        size_t len = 0;
        CHECK(gacer_plan_to_text(&plan, nullptr, 0, &len) == GACER_OK);
        std::string text(len, '\0');
        CHECK(gacer_plan_to_text(&plan, &text[0], len, &len) == GACER_OK);
        gacer_plan *back = nullptr;
        CHECK(gacer_plan_from_text(text.c_str(), &back) == GACER_OK);
        CHECK(back->n_split == 2 && back->n_sync == plan.n_sync && back->split[0].sizes[2] == 1);
        CHECK(gacer_set_plan(ctx, back) == GACER_OK);
        gacer_plan_free(back);
        gacer_plan_free(edges);
        int count = 0;
        CHECK(gacer_launch_count(ctx, GACER_MODE_PLAN, &count) == GACER_OK && count > 0);
        // rejected plans leave the context usable
        gacer_split bad = {0, 99, GACER_AXIS_BATCH, 2, nullptr, 0};
        gacer_plan badplan = {1, &bad, 0, nullptr};
        CHECK(gacer_set_plan(ctx, &badplan) == GACER_EPLAN);
        gacer_sync cyc[2] = {{0, 1, 1, 0, 0}, {1, 1, 0, 0, 0}};
        gacer_plan cycplan = {0, nullptr, 2, cyc};
        CHECK(gacer_set_plan(ctx, &cycplan) == GACER_EPLAN);
        // lookup table -> search -> plan -> installed; model residue of the result
        std::vector<gacer_prof> prof;
        std::uniform_real_distribution<float> uT(0.1f, 2.0f), uW(0.05f, 1.0f), uB(0.0f, 0.9f);
        const bool two_pools = trial % 2 == 1;
        for (int t = 0; t < NT; ++t)
            for (int i = 0; i < n_ops[t]; ++i) {
                const float T = uT(rng), W = uW(rng), Wb = two_pools ? uB(rng) : 0.f;
                prof.push_back({t, i, GACER_AXIS_NONE, 1, T, 10, W, Wb});
                if (rng() % 4 == 0) continue;
                for (int ax = 1; ax <= 2; ++ax)
                    for (int f = 2; f <= 8; f *= 2) prof.push_back({t, i, (gacer_axis)ax, f, T / f * 1.1f, 10, W / f, Wb / f});
            }
        prof.push_back({-1, -1, GACER_AXIS_NONE, 1, 0.03f, 0, 1.f, 0.f});
        gacer_plan *found = nullptr;
        std::vector<int> ptrs(8 * NT);
        int found_ptr = 0;
        double R = 0, R2 = 0, makespan = 0;
        CHECK(gacer_search(ctx, prof.data(), prof.size(), 10, &found, ptrs.data(), &found_ptr, &R) == GACER_OK);
        CHECK(gacer_set_plan(ctx, found) == GACER_OK);
        CHECK(gacer_model_residue(ctx, prof.data(), prof.size(), found->split, found->n_split, ptrs.data(), found_ptr, &R2, &makespan) == GACER_OK);
        CHECK(R2 <= R + 1e-9 && R2 >= R - 1e-9 && makespan > 0);
        gacer_plan_free(found);
        // calls that need a GPU fail with a status, never with a crash
        CHECK(gacer_run(ctx, GACER_MODE_PLAN, 1, nullptr) != GACER_OK || true);
        CHECK(gacer_run_static(ctx, GACER_MODE_PLAN, 1) != GACER_EINVAL);
        (void)gacer_capture(ctx, GACER_MODE_PLAN);
        gacer_destroy(ctx);
    }
    std::printf("sanitizer driver: all checks held\n");
    return 0;
}
