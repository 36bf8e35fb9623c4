// Issue logic of the executor (one host thread per tenant, generation counters on the sync events) under
// ThreadSanitizer, on the host-only HIP runtime of stub_hip.cpp.  Exit code 0 = no wait was ever issued before the
// record it belongs to; data races are ThreadSanitizer's own findings.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>
#include "../../include/gacer.h"

extern "C" {
void stub_learn_begin(); void stub_learn_end(int rounds); void stub_check_begin(); void stub_check_end();
long stub_violations(); long stub_waits_checked();
}
#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "check failed at line %d: %s (%s)\n", __LINE__, #cond, ctx ? gacer_last_error(ctx) : ""); std::exit(1); } } while (0)

static void *const FAKE = (void *)0x10000;

struct Chain {
    std::vector<gacer_op> ops;
    std::vector<gacer_tensor> tensors;
    gacer_tenant desc;
    Chain(int n, int id)
    {
        tensors.push_back({8, 16, 6, 6, FAKE});
        for (int i = 0; i < n; ++i) {
            tensors.push_back({8, 16, 6, 6, FAKE});
            gacer_op op;
            std::memset(&op, 0, sizeof op);
            op.kind = GACER_CONV2D; op.in0 = i; op.in1 = -1; op.res = -1; op.out = i + 1;
            op.w = FAKE; op.bias = (const float *)FAKE;
            op.cin = 16; op.cout = 16; op.kh = op.kw = 3; op.stride = 1; op.pad = 1; op.groups = 1; op.act = GACER_ACT_RELU; op.alpha = 1.f;
            ops.push_back(op);
        }
        std::memset(&desc, 0, sizeof desc);
        desc.n_ops = n; desc.n_tensors = (int)tensors.size(); desc.input = 0; desc.output = n; desc.dtype = GACER_F32; desc.batch = 8;
        desc.stream = (void *)(uintptr_t)(0x1000 * (id + 1));
        desc.sibling_stream = (void *)(uintptr_t)(0x1000 * (id + 1) + 0x800);
    }
};

int main()
{
    std::mt19937 rng(11);
    long checked = 0;
    for (int trial = 0; trial < 12; ++trial) {
        gacer_ctx *ctx = nullptr;
        CHECK(gacer_create(&ctx) == GACER_OK);
        const int NT = 2 + trial % 4;
        std::vector<Chain> chains;
        chains.reserve(NT);
        std::vector<int> n_ops;
        for (int t = 0; t < NT; ++t) { n_ops.push_back(3 + (int)(rng() % 8)); chains.emplace_back(n_ops.back(), t); }
        std::vector<gacer_tenant> descs;
        for (Chain &c : chains) { c.desc.ops = c.ops.data(); c.desc.tensors = c.tensors.data(); descs.push_back(c.desc); }
        CHECK(gacer_load_tenants(ctx, descs.data(), NT) == GACER_OK);
        const int n_ptr = 1 + (int)(rng() % 3);
        std::vector<int> P;
        for (int t = 0; t < NT; ++t) {
            std::vector<int> row;
            for (int j = 0; j < n_ptr; ++j) row.push_back((int)(rng() % (n_ops[t] + 1)));
            std::sort(row.begin(), row.end());
            P.insert(P.end(), row.begin(), row.end());
        }
        gacer_plan *edges = nullptr;
        CHECK(gacer_plan_from_pointers(ctx, P.data(), n_ptr, &edges) == GACER_OK);
        std::vector<gacer_split> sp;
        for (int t = 0; t < NT; ++t)
            for (int i = 0; i < n_ops[t]; i += 2) sp.push_back({t, i, GACER_AXIS_BATCH, 2, nullptr, (t + i) % 4 == 0});
        gacer_plan plan = {(int)sp.size(), sp.data(), edges->n_sync, edges->sync};
        CHECK(gacer_set_plan(ctx, &plan) == GACER_OK);
        gacer_plan_free(edges);
        for (int mode : {GACER_MODE_PLAN, GACER_MODE_STREAM_PARALLEL}) {
            CHECK(gacer_set_issue_threads(ctx, 0) == GACER_OK);
            stub_learn_begin();
            { const gacer_status st = gacer_run(ctx, mode, 2, nullptr); if (st != GACER_OK) std::fprintf(stderr, "status %d mode %d\n", (int)st, mode); CHECK(st == GACER_OK); }
            stub_learn_end(2);
            CHECK(gacer_set_issue_threads(ctx, 1) == GACER_OK);
            stub_check_begin();
            std::vector<float> ms(40);
            for (int call = 0; call < 3; ++call) CHECK(gacer_run(ctx, mode, 40, ms.data()) == GACER_OK);
            stub_check_end();
        }
        CHECK(gacer_set_sync_every_launch(ctx, 1) == GACER_OK);
        CHECK(gacer_run(ctx, GACER_MODE_PLAN, 5, nullptr) == GACER_OK);
        CHECK(gacer_set_sync_every_launch(ctx, 0) == GACER_OK);
        CHECK(gacer_run_static(ctx, GACER_MODE_PLAN, 2) == GACER_OK);
        gacer_destroy(ctx);
        gacer_ctx *none = nullptr; ctx = none;
        checked = stub_waits_checked();
    }
    if (stub_violations() != 0 || checked == 0) {
        std::fprintf(stderr, "%ld of %ld waits were issued before their record\n", stub_violations(), checked);
        return 1;
    }
    std::printf("tsan driver: %ld waits checked, none before its record\n", checked);
    return 0;
}
