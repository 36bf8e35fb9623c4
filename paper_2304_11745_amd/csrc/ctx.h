// Library-internal state behind the opaque gacer_ctx.
#pragma once
#include <hip/hip_runtime_api.h>
#include <string>
#include <vector>
#include "../../include/gacer.h"
#include "kernels.h"

namespace gacer {

enum LaunchKind { LK_IGEMM, LK_DWCONV, LK_MAXPOOL, LK_GAVGPOOL, LK_ELTWISE, LK_LAYERNORM, LK_SOFTMAX, LK_CONCAT };

struct Launch {
    LaunchKind kind;
    GemmArgs g;
    StreamArgs s;
    size_t ws_off = 0;      // floats into the tenant's split-K workspace: chunks of one operator own disjoint parts
};

struct Tenant {
    std::vector<gacer_op> ops;
    std::vector<gacer_tensor> tensors;
    int input = 0, output = 0, batch = 1;
    gacer_dtype dtype = GACER_F32;
    hipStream_t stream = nullptr;
    hipStream_t sibling = nullptr;                  // optional second stream for decompositions marked `sibling`
    // split-K bookkeeping (conv / GEMM operators only): slices and 64-byte K blocks per slice, fixed per
    // operator from its unsplit shape; one library-owned workspace per tenant (its operators never overlap)
    std::vector<int> ksplit, kb_per_slice;
    float *ws = nullptr;
    size_t ws_floats = 0;
};

// One operator after plan expansion: its chunk launches plus the events it waits on / records.
struct OpExec {
    std::vector<Launch> chunks;
    std::vector<int> waits;     // indices into Ctx::sync_events
    int record = -1;            // event recorded after the last chunk, -1 = none
    int pre_record = -1;        // event recorded after the waits and before the first chunk (barrier hub)
    int fork = -1, join = -1;   // sibling decomposition: odd chunks run on the tenant's sibling stream between these events
};

// Event pairs of a traced call: rounds x kernels-per-round x {start, stop}; row_of[tenant][op][chunk] is the row of
// that chunk's first kernel within one round (a split-K chunk owns two consecutive rows).
struct Trace {
    size_t per_round = 0;
    std::vector<hipEvent_t> ev;
    std::vector<std::vector<std::vector<size_t>>> row_of;
};

struct Ctx {
    int device = 0;
    bool has_device = false;
    int n_cu = 256;
    std::vector<Tenant> tenants;
    bool loaded = false;
    bool ws_missing = false;                        // split-K workspace allocation failed at load
    // current plan (copied)
    std::vector<gacer_split> splits;              // installed plan (sizes pointers refer to split_sizes)
    std::vector<std::vector<int>> split_sizes;
    std::vector<gacer_sync> syncs;
    // expansion: [tenant][op]
    std::vector<std::vector<OpExec>> plan_exec;     // decomposed + edges
    std::vector<std::vector<OpExec>> plain_exec;    // unsplit, no edges
    std::vector<std::pair<int, int>> plan_order;    // host issue order (tenant, op), topological
    std::vector<std::pair<int, int>> par_order;     // stream-parallel issue order
    std::vector<hipEvent_t> sync_events;
    size_t n_sync_events = 0;                       // events the current plan needs
    std::vector<hipEvent_t> join_events;            // one per tenant
    std::vector<hipEvent_t> t_start, t_end;         // per round, timing enabled
    hipGraphExec_t graph_exec[3] = {nullptr, nullptr, nullptr};   // captured round per mode (optional)
    bool issue_threads = false;                     // one host thread per tenant enqueues that tenant's stream
    bool fuse_affine = true;                        // a per-channel affine operator + the 1x1 convolution that reads it run as one launch where allowed
    bool sync_every_launch = false;                 // checking mode: wait for, and check, every kernel before the next is issued
    bool capturing = false;                         // a stream capture is open: nothing may synchronise
    std::string launch_detail;                      // checking mode: which launch failed
    std::vector<float *> ws_run;                    // split-K workspace each tenant uses in the call in progress
    Trace *trace = nullptr;                         // set while gacer_trace_run issues its rounds
    double last_issue_ms = 0;                       // host time the last gacer_run spent enqueueing
    int last_issue_launches = 0;
    std::string err;
};

// axis extent and legality of a decomposition
int axis_extent(const Tenant &t, int op, gacer_axis axis);
bool axis_legal(gacer_opkind kind, gacer_axis axis);
void chunk_range(int extent, int factor, int j, int *lo, int *hi);
// builds the launch of operator `op` restricted to batch items [b_lo,b_hi) and channels [c_lo,c_hi)
Launch make_launch(const Tenant &t, int op, int b_lo, int b_hi, int c_lo, int c_hi);
// `ws` is the split-K workspace of the launch's tenant (only read when the operator's K range is cut into slices)
LaunchInfo enqueue(const Launch &l, hipStream_t s, bool dry, int phase = 0, float *ws = nullptr);
void drop_graphs(Ctx *c);
// every plan the library hands out is built here (and released by gacer_plan_free)
gacer_plan *make_plan(const std::vector<gacer_split> &splits, const std::vector<gacer_sync> &syncs);

}  // namespace gacer

struct gacer_ctx : gacer::Ctx {};
