/*
 * gacer.h -- C ABI of the multi-tenant regulated executor for one AMD MI355X (gfx950).
 *
 * Several DNN tenants M_1..M_N, each a flat operator list M_n = [O_n,1 .. O_n,i]
 * (Section 4.1, "Multi-Tenant Runtime Deployment"), run concurrently on one GPU, one HIP
 * stream per tenant.  A *regulation plan* says
 *   - spatially: which operators are decomposed into chunks (the mask list and list_B of
 *     Section 4.2, Eq. 5) -- here along the batch axis or the output-channel axis; and
 *   - temporally: which operators must wait for which (the synchronisation pointers /
 *     Matrix_P of Section 4.3, Eq. 6 and Eq. 7), expressed as event edges between streams.
 * Every valid plan produces bit-identical tenant outputs; a plan only changes when work runs.
 *
 * Conventions
 *   - All `dptr`, weight, bias, scale and shift pointers are DEVICE pointers owned by the
 *     caller.  They must stay valid until gacer_destroy / the next gacer_load_tenants.
 *     The library never allocates, frees or copies tenant memory.  Descriptor structs
 *     (gacer_tenant, gacer_op, ...) are HOST memory and are deep-copied by the call.
 *   - Activations are stored channels-last: element (n,c,h,w) of a tensor with logical shape
 *     (n,c,h,w) lives at index ((n*H + h)*W + w)*C + c.  Token tensors use c = features,
 *     h = sequence position, w = 1.  Element type is float (GACER_F32) or bfloat16
 *     (GACER_BF16) for activations and for CONV2D/DWCONV2D/GEMM weights; bias, scale and
 *     shift vectors are always float.  All device pointers must be 16-byte aligned.
 *   - Weight layouts: CONV2D [cout][kh][kw][cin/groups];  DWCONV2D [kh][kw][c];
 *     GEMM [cout][cin] with the cin index running over the input item in storage order.
 *   - Functions return a gacer_status and never throw or abort; gacer_last_error gives text.
 *     A failing call leaves the context as it was before the call.
 *   - A context is not thread-safe; calls on one context must not overlap.
 */
#ifndef GACER_H
#define GACER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gacer_ctx gacer_ctx; /* opaque, owned by the library */

typedef enum {
    GACER_OK = 0,
    GACER_EINVAL = 1, /* null pointer, bad enum, misaligned device pointer            */
    GACER_ESHAPE = 2, /* operator / tensor shapes inconsistent                        */
    GACER_EPLAN = 3,  /* plan rejected (illegal split, bad or cyclic sync edges, ...) */
    GACER_ESTATE = 4, /* call order violated (e.g. run before load)                   */
    GACER_ENOMEM = 5,
    GACER_EHIP = 6    /* a HIP runtime call failed; text in gacer_last_error          */
} gacer_status;

typedef enum { GACER_F32 = 0, GACER_BF16 = 1 } gacer_dtype;

typedef enum {
    GACER_CONV2D = 0,     /* y = act(conv(x,w) + bias + res)        dense or grouped          */
    GACER_DWCONV2D = 1,   /* depthwise (groups == cin == cout), same epilogue                */
    GACER_GEMM = 2,       /* y[r,o] = act(sum_k x[r,k] w[o,k] + bias[o] + res[r,o])          */
    GACER_BGEMM_QK = 3,   /* attention scores, see below                                     */
    GACER_BGEMM_PV = 4,   /* attention context, see below                                    */
    GACER_MAXPOOL = 5,    /* window max, padding never wins                                  */
    GACER_GAVGPOOL = 6,   /* mean over h*w                                                   */
    GACER_AFFINE_ACT = 7, /* y = act(x*scale[c] + shift[c] + res)   (bias + folded BN + ReLU) */
    GACER_ADD = 8,        /* y = act(in0 + in1)                                              */
    GACER_LAYERNORM = 9,  /* over c, of (in0 + res); scale = gamma, shift = beta, alpha = eps */
    GACER_SOFTMAX = 10,   /* over c                                                          */
    GACER_ACT = 11,       /* y = act(x)                                                      */
    GACER_SCALE = 12,     /* y[n,c,h,w] = act(in0[n,c,h,w] * in1[n,c]): squeeze-and-excitation gate */
    GACER_CONCAT = 13,    /* y[:, :cin] = in0, y[:, cin:] = in1 (channel concatenation)      */
    GACER_AVGPOOL = 14    /* unpadded window mean (kh = kw, stride)                          */
} gacer_opkind;

/* HSWISH(v) = v * HSIGMOID(v), HSIGMOID(v) = min(max(v + 3, 0), 6) / 6 */
typedef enum {
    GACER_ACT_NONE = 0, GACER_ACT_RELU = 1, GACER_ACT_RELU6 = 2, GACER_ACT_GELU = 3, GACER_ACT_HSWISH = 4, GACER_ACT_HSIGMOID = 5
} gacer_act;

/* Decomposition axis of an operator (Eq. 5 decomposes along batch; the output-channel
 * axis is this library's second axis).  Chunk j of `factor` covers a contiguous sub-range;
 * the first (extent % factor) chunks are one element longer, sizes sum to the extent. */
typedef enum { GACER_AXIS_NONE = 0, GACER_AXIS_BATCH = 1, GACER_AXIS_COUT = 2 } gacer_axis;

/*
 * A tensor is stored channels-last: position (n, h, w) holds its c channels contiguously.  With pitch == 0 positions follow
 * each other without gaps (pitch = c) and `base`, `c_off` are ignored.  With pitch != 0 the tensor is a channel window of a
 * wider one: `base` indexes a gap-free tensor of the same n, h, w with c(base) == pitch, the window starts at channel c_off
 * of it (c_off + c <= pitch, dptr == dptr(base) + c_off elements; a window that does not start on a 16-byte boundary is
 * served by the element-wise kernel paths) and neighbouring positions are pitch elements apart.  Windows let a network concatenate along channels without a copy (DenseNet: every layer writes its
 * window of one buffer per block, the next layer reads a prefix of it).  A window may be in0 of CONV2D, of a per-position
 * GEMM, of AFFINE_ACT and of ACT, and out of those and of MAXPOOL / AVGPOOL; a residual input (`res`) of an operator that
 * writes a window is not supported.  Windows written by different operators must not overlap; a window is readable once
 * every channel of it has been written.
 */
typedef struct {
    int64_t n, c, h, w; /* logical shape; n must be a multiple of the tenant's batch */
    void *dptr;         /* device, caller-owned, 16-byte aligned (windows: see above) */
    int64_t pitch;      /* elements between neighbouring positions; 0 = c            */
    int base, c_off;    /* pitch != 0: the wider tensor and the first channel in it  */
} gacer_tensor;

/*
 * One operator O_n,i.  in0/in1/res/out index the tenant's tensor table (-1 = absent).
 *   CONV2D/DWCONV2D: cin,cout,kh,kw,stride,pad,groups as usual; out h = (h+2*pad-kh)/stride+1.
 *   GEMM: cin = features consumed per output row.  If cin == c(in0) every position (n,h,w)
 *         is a row (a 1x1 convolution); if cin == c*h*w(in0) every item n is one row and the
 *         output has h = w = 1.
 *   BGEMM_QK: in0 = qkv tokens (n=B, c=3*D, h=S, w=1), D = groups*cin (groups = heads,
 *         cin = head size); out (n=B*groups, c=S, h=S, w=1):
 *         out[b*heads+hd, key j, query i] = alpha * sum_d q[b,i,hd,d] * k[b,j,hd,d].
 *   BGEMM_PV: in0 = probabilities (n=B*groups, c=S, h=S, w=1), in1 = qkv tokens, cout = head
 *         size; out (n=B, c=D, h=S, w=1): out[b,i,hd*cout+d] = sum_j p[b*heads+hd,j,i] * v[b,j,hd,d].
 *   MAXPOOL: kh (=kw), stride, pad.   LAYERNORM: alpha = epsilon.
 *   SCALE: in1 has shape (n, c, 1, 1) for in0 = (n, c, h, w).   CONCAT: cin = c(in0), cout = c(in0) + c(in1), same n, h, w.
 *   AVGPOOL: kh (=kw), stride, pad must be 0; out h = (h-kh)/stride+1.
 */
typedef struct {
    gacer_opkind kind;
    int in0, in1, res, out;
    const void *w;      /* device: weights (dtype of the tenant)           */
    const float *bias;  /* device: [cout] or NULL                          */
    const float *scale; /* device: [c]   AFFINE_ACT scale / LAYERNORM gamma */
    const float *shift; /* device: [c]   AFFINE_ACT shift / LAYERNORM beta  */
    int cin, cout, kh, kw, stride, pad, groups;
    gacer_act act;
    float alpha;
} gacer_op;

/* One tenant: its operator list in execution order, its tensors, and the stream it runs on. */
typedef struct {
    int n_ops;
    const gacer_op *ops;
    int n_tensors;
    const gacer_tensor *tensors;
    int input, output; /* tensor indices */
    gacer_dtype dtype;
    int batch;
    void *stream; /* hipStream_t created by the caller (default priority); NULL = null stream */
    void *sibling_stream; /* optional second stream of this tenant (created by the caller, default priority) for
                             decompositions marked `sibling`; NULL = such chunks stay on `stream` */
} gacer_tenant;

/* mask + list_B (Section 4.2, Eq. 5): operator (tenant, op) is decomposed into `factor` chunks on `axis`.
 * sizes == NULL: even chunks, factor in {1,2,4,8}, chunk j holds floor(E/factor) + (j < E mod factor) elements of the
 * axis extent E.  sizes != NULL: list_B itself -- `factor` (1..8) positive chunk sizes in launch order whose sum must
 * equal E (e.g. {24, 8} on a batch of 32); the array is copied by gacer_set_plan.  Chunks are contiguous ascending
 * sub-ranges and run in that order on the tenant's stream.
 * sibling != 0 (the decomposition over several streams of Section 5.4, Table 3): the odd-numbered chunks are issued on
 * the tenant's sibling stream, which first waits for everything the operator itself had to wait for, and the
 * operator counts as finished (for the next operator and for sync edges) only when both streams have finished
 * their chunks -- chunks of one operator can then overlap each other.  Ignored without a sibling stream. */
typedef struct { int tenant, op; gacer_axis axis; int factor; const int *sizes; int sibling; } gacer_split;
/* One ordering constraint between streams.  when == 0: (dst_tenant,dst_op) starts only after every chunk of
 * (src_tenant,src_op) has finished.  when == 1: it starts once everything (src_tenant,src_op) itself has to wait
 * for is done (its stream predecessors and its own when-0 edges) -- the source operator then acts as the hub of a
 * barrier: it gathers the other streams and releases them without making them wait for its own execution.
 * Cluster barriers of Matrix_P expand into such edges. */
typedef struct { int src_tenant, src_op, dst_tenant, dst_op, when; } gacer_sync;
typedef struct { int n_split; const gacer_split *split; int n_sync; const gacer_sync *sync; } gacer_plan;

/* One row of the lookup table of Section 4.1: operator (tenant, op) decomposed `factor` ways on
 * `axis` takes `ms` per chunk in isolation, launches `workgroups` workgroups per chunk and
 * occupies `cu_share` (0..1] of the compute units (the analogue of SM occupancy W).  `bw_share`
 * [0..1] is the chunk's share of the second resource pool, memory bandwidth (Section 4.4, claim (2)):
 * the bytes it has to move (inputs, parameters and output once) per unit of its time, over the
 * device's 8 TB/s; 0 in every row switches the second pool off in gacer_search / gacer_model_residue.
 * The row with tenant == -1 carries the synchronisation wait T_SW (Eq. 8) in `ms`. */
typedef struct { int tenant, op; gacer_axis axis; int factor; float ms; int workgroups; float cu_share; float bw_share; } gacer_prof;

/* One kernel launch of a round, as measured by gacer_trace_run: average duration, algorithmic
 * work of the launched sub-range (flops = 2*MACs for conv/GEMM/attention launches, 0 otherwise;
 * bytes = inputs read once + parameters read once + output written once, at the tensor dtype),
 * grid size and the kernel variant that ran.  start_ms / end_ms place the kernel inside the LAST traced
 * round: its begin and end on the device clock, counted from the moment that round was released on
 * tenant 0's stream -- what a test needs to see that one cluster ends before the next begins (Eq. 6). */
typedef struct {
    int tenant, op, chunk;
    float ms;
    double flops, bytes;
    int workgroups;
    char kernel[40];
    float start_ms, end_ms;
} gacer_launch_stat;

typedef enum { GACER_MODE_PLAN = 0, GACER_MODE_SEQUENTIAL = 1, GACER_MODE_STREAM_PARALLEL = 2 } gacer_mode;

/* Creates an empty context bound to the current HIP device.  GACER_ENOMEM / GACER_EHIP. */
gacer_status gacer_create(gacer_ctx **out);
/* Waits for the tenant streams, destroys library-owned events.  NULL is allowed. */
void gacer_destroy(gacer_ctx *ctx);

/*
 * Problem statement, Section 4.1: registers the N tenant operator lists.  Validates every
 * operator against its tensors (GACER_ESHAPE names the first offending tenant/op), checks
 * that operators only read tensors written earlier, deep-copies the descriptors and resets the
 * plan to "no decomposition, no pointers".  1 <= n <= 64.
 */
gacer_status gacer_load_tenants(gacer_ctx *ctx, const gacer_tenant *tenants, int n);

/*
 * Installs a regulation plan (mask/list_B of Section 4.2 + pointer edges of Section 4.3); NULL
 * means unsplit and unsynchronised.  Rejected with GACER_EPLAN and no change when: factor not
 * in {1,2,4,8}; factor larger than the axis extent; axis not legal for the kind (COUT is legal
 * for CONV2D, DWCONV2D, GEMM, MAXPOOL, GAVGPOOL, AFFINE_ACT only; BATCH for all); duplicate
 * entry for one operator; an edge names a missing operator or stays inside one tenant; the
 * union of stream order and sync edges has a cycle.  The plan is copied.
 */
gacer_status gacer_set_plan(gacer_ctx *ctx, const gacer_plan *plan);

/*
 * Matrix_P -> sync edges (Eq. 6 / Eq. 7).  P holds n_tenants rows of n_ptr sorted pointer
 * values; value p cuts after the p-th operator (1-based; 0 and n_ops give empty segments).
 * Same-index segments form a cluster; after the edges, the first operator of every tenant's
 * segment k+1 is ordered behind the last operator of every other tenant's segments <= k.  Each
 * barrier is built around a hub (the lowest-numbered tenant whose next segment is not empty): the hub's next
 * operator waits for the last operators of all other tenants (when = 0 edges) and the other tenants'
 * next operators wait for the hub to be released (when = 1 edges) -- 2(N-1) edges per pointer instead
 * of N(N-1).  The split part of the returned plan is empty.  Free with gacer_plan_free.
 * GACER_EPLAN if a row is unsorted or out of range.
 */
gacer_status gacer_plan_from_pointers(gacer_ctx *ctx, const int *P, int n_ptr, gacer_plan **out);

/*
 * Runs `rounds` rounds; in each round every tenant executes once.  Mode PLAN issues the
 * decomposed operators on the tenants' streams, ordered by the plan's edges (hipEvent
 * record / wait; the host never blocks inside a round).  SEQUENTIAL issues all tenants one
 * after another, unsplit, on tenant 0's stream.  STREAM_PARALLEL uses one stream per tenant,
 * unsplit, no edges.  Rounds are separated by a fork/join over all streams.  ms_per_round
 * (host, `rounds` floats, may be NULL) receives each round's makespan measured with
 * hipEvents.  Returns after all work of all rounds has finished.
 */
gacer_status gacer_run(gacer_ctx *ctx, int mode, int rounds, float *ms_per_round);

/*
 * gacer_run for callers that cannot allocate device memory: code running under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same rounds, same kernels, same results as gacer_run(ctx, mode, rounds, NULL),
 * but the split-K partial tiles go to a fixed 32 MiB workspace inside the library's code object (one copy per GPU, held
 * until the process ends) instead of the buffers gacer_load_tenants allocated, and the call itself allocates nothing:
 * no hipMalloc / hipFree, no event or stream creation (it uses the events gacer_load_tenants and gacer_set_plan
 * created), one issuing thread, no graph replay, no per-round timing.  Every tenant gets a 256-byte aligned part of
 * the workspace; GACER_ENOMEM when the loaded tenants need more than 32 MiB together (the message states the need),
 * GACER_ESTATE when the context was created without a GPU.  Nothing in the workspace has to start at zero (every
 * partial tile is written before it is read), so the contents a previous call left behind do not matter; but all
 * calls on one GPU share the one workspace, and calls that overlap on a GPU (two contexts, two threads) race.
 * Returns after all rounds have finished.
 */
gacer_status gacer_run_static(gacer_ctx *ctx, int mode, int rounds);

/*
 * Measurement aid: like gacer_run (same issue loop, one thread or one per tenant as set), but every kernel
 * is launched together with a start / stop event pair that the runtime stamps with the kernel's own begin
 * and end on the device clock -- the interval a profiler's kernel trace reports for the dispatch -- so that
 * per-launch durations under the chosen mode (including contention from the other tenants' streams) and
 * the position of every launch inside the round can be read back.  out[k].ms is the mean duration over
 * `rounds`; start_ms / end_ms are those of the last round.  Writes up to `cap` rows (issue order of one
 * round; an operator whose K range is cut into slices contributes its slice kernel and its finishing pass
 * as two rows) and the row count to *n; cap = 0 sizes.  Captured graphs are not replayed here.  The
 * events cost host time per launch; throughput must be taken from gacer_run.
 */
gacer_status gacer_trace_run(gacer_ctx *ctx, int mode, int rounds, gacer_launch_stat *out, size_t cap, size_t *n);

/*
 * Builds the lookup table of Section 4.1 by timing, in isolation on the tenant's stream, every
 * operator unsplit and for every legal (axis, factor in {2,4,8}); plus the T_SW row.  Tenant
 * inputs must hold finite data (the call runs each tenant once first).  Writes up to `cap`
 * rows to `out` (host) and the total number of rows to *n; call with cap = 0 to size.
 */
gacer_status gacer_profile(gacer_ctx *ctx, gacer_prof *out, size_t cap, size_t *n);

/*
 * Granularity-aware search (Section 4.4, Algorithm 1, alternated with the spatial regulation of
 * Section 4.2) on the CPU, over the lookup table `prof`: returns the plan (splits + pointer
 * edges) with the smallest modelled residue R (Eq. 8).  The spatial regulation decomposes an
 * operator into a chunk sized to the residue it is to fill plus the remainder, so the plan's splits
 * carry chunk lists (`sizes`, e.g. {5, 3}); costs of chunk sizes between the table's rows are
 * interpolated linearly in the size.  `pointers_out`, if not NULL, receives n_tenants * (*n_ptr_out)
 * pointer values (capacity 8 per tenant).  No GPU work is done.
 */
gacer_status gacer_search(gacer_ctx *ctx, const gacer_prof *prof, size_t n, int max_rounds,
                          gacer_plan **out, int *pointers_out, int *n_ptr_out, double *residue_out);

/* Modelled residue R (Eq. 8) and completion time of an explicit (splits, Matrix_P) on the table; even
 * decompositions need their row in the table, chunk lists are interpolated.  CPU only. */
gacer_status gacer_model_residue(gacer_ctx *ctx, const gacer_prof *prof, size_t n, const gacer_split *split,
                                 int n_split, const int *P, int n_ptr, double *residue_out, double *makespan_out);

/*
 * Offline deployment (Section 4.4, "Search Cost Analysis for Offline/Online Deployment"): a searched plan written
 * out as text, to be stored per deployment scenario and installed later without searching again.
 * gacer_plan_to_text writes a NUL-terminated text of *len bytes (terminator included) into buf; buf == NULL or
 * cap == 0 only sizes; GACER_EINVAL when cap is too small.  gacer_plan_from_text parses such a text into a
 * library-allocated plan (free with gacer_plan_free); GACER_EPLAN on anything it does not recognise.  The text is
 * not validated against tenants here: gacer_set_plan does that when the plan is installed.
 */
gacer_status gacer_plan_to_text(const gacer_plan *plan, char *buf, size_t cap, size_t *len);
gacer_status gacer_plan_from_text(const char *text, gacer_plan **out);

void gacer_plan_free(gacer_plan *plan);
/* Text of the last error on this context ("" if none); valid until the next call. */
const char *gacer_last_error(const gacer_ctx *ctx);
/* Number of kernel launches one round issues in the given mode under the current plan. */
gacer_status gacer_launch_count(gacer_ctx *ctx, int mode, int *count);

/*
 * Captures one round of `mode` under the current plan into a HIP graph (fork from tenant 0's stream, every
 * operator on its tenant's stream with its event edges, join); later gacer_run calls in that mode replay the
 * graph instead of issuing launch by launch, which removes the per-launch host cost (the issuing overhead
 * discussed in Section 4.2 and Section 5.5).  Outputs are identical to the uncaptured run.  The capture is
 * dropped by gacer_set_plan, gacer_load_tenants and gacer_release_graphs.  Tensor pointers are baked in.
 * HIP runtimes older than 7.2 crash inside hipStreamEndCapture when three or more captured streams wait on
 * each other's events mutually; on such a runtime the call refuses (GACER_EPLAN) a plan whose edges, taken
 * tenant by tenant, close a ring of three or more tenants (a waits on b, b on c, c on a).  Barriers from
 * gacer_plan_from_pointers that all share one hub tenant only pair the hub with each member and are accepted.
 */
gacer_status gacer_capture(gacer_ctx *ctx, int mode);
gacer_status gacer_release_graphs(gacer_ctx *ctx);

/*
 * Multi-tenant deployment model of Section 2.1: with enable != 0, gacer_run in the plan and stream-parallel
 * modes enqueues every tenant's stream from its own host thread (the caller's thread takes tenant 0), which
 * multiplies the launch rate when many small-kernel tenants make the issue loop the bottleneck.  Results and
 * ordering guarantees are unchanged.  Needs a distinct stream per tenant (otherwise the call runs single-threaded).
 */
gacer_status gacer_set_issue_threads(gacer_ctx *ctx, int enable);

/*
 * Checking mode for finding a missing dependency or a failing launch (the regulation of Section 4.3 is only correct if
 * the sync pointers order everything that needs ordering): with enable != 0, gacer_run and gacer_run_static wait
 * for every kernel and read the device's status before issuing the next one, so the launches of all tenants run one
 * at a time in issue order, captured graphs are not replayed, and a failure is reported as
 * GACER_EHIP with the tenant, operator, chunk, kernel name and workgroup count of the launch that caused it.  Outputs
 * must be bit-identical to those of the ordinary mode; if they are not, the plan lacks an edge.  Not for timing.
 */
gacer_status gacer_set_sync_every_launch(gacer_ctx *ctx, int enable);

/*
 * Launch fusion (on by default).  A tenant of very short kernels spends as much time between kernels as inside them -- the
 * issuing overhead that the granularity discussion of Section 5.4 attributes to having more operators -- so where the plan
 * allows, an AFFINE_ACT operator (no residual; activation none, ReLU or ReLU6) and the 1x1 stride-1 convolution that
 * consumes it are issued as ONE kernel: the product applies the affine operator's arithmetic while it loads its A tile and
 * also writes the affine operator's output tensor, which then exists as if its own kernel had run.  Outputs and every
 * intermediate tensor keep the bits of the unfused kernels.  A pair is left alone when the plan decomposes either operator,
 * when the affine operator's completion is the source of a sync edge, and when its tensors or parameter vectors are not
 * 16-byte aligned or its channel count is not a multiple of a 16-byte vector.  In traces and launch counts the affine
 * operator of a fused pair has no launch of its own; the fused kernel's name starts with "igemm_affine_".  enable = 0 issues
 * every operator on its own (the lookup table of gacer_profile always describes the unfused operators).  Re-installs the
 * current plan.
 */
gacer_status gacer_set_fuse_affine(gacer_ctx *ctx, int enable);

/*
 * Stream placement aid.  The device runs the streams of a process on a small number of hardware queues, and kernels of
 * two streams that landed on the same queue never overlap: tenants on such streams run one after the other however
 * the plan orders them (Section 2.1's concurrent streams silently turn sequential).  This call finds out, by
 * measurement, which of the caller's `n` streams (hipStream_t, n <= 64) share a queue: it starts a short spinning
 * kernel (one wavefront, 100 us) on a pair of streams at the same time and checks whether the pair took one or two
 * kernel times.  group[i] receives a small integer, equal for streams that serialise.  A caller with more candidate
 * streams than tenants can then give every tenant a queue of its own, or balance tenants over the queues.  Uses only
 * the given streams; returns after they are idle again.
 */
gacer_status gacer_probe_stream_queues(void *const *streams, int n, int *group);

/*
 * Stream placement proper (the per-tenant streams of Section 2.1, spread over the hardware queues found by
 * gacer_probe_stream_queues).  `tenants` are the n descriptors about to be loaded (their `stream` fields are ignored),
 * `candidates` are n_cand streams created by the caller (n_cand <= 64; about 4 per expected queue is plenty).  The call
 * probes the candidates, estimates every tenant's cost from its operator list (matrix-core work plus a per-launch
 * cost) and places tenants longest first on the least loaded queue.  chosen[i] receives the index of the candidate
 * stream for tenant i, queue_of[i] (may be NULL) its queue, *n_queues (may be NULL) the number of queues found.  Up
 * to n_queues tenants get queues of their own; further tenants share, and once a queue has no unused candidate left
 * its tenants share one stream.  sibling[i] (may be NULL) receives the index of a further, unused candidate on
 * another queue for tenant i's sibling stream (see gacer_split.sibling), or -1 when no such candidate is left.
 */
gacer_status gacer_place_streams(const gacer_tenant *tenants, int n, void *const *candidates, int n_cand, int *chosen,
                                 int *queue_of, int *n_queues, int *sibling);

/*
 * Measured refinement of the installed plan: the greedy spatial step of Section 4.2 ("Overall Spatial Regulation")
 * with the GPU instead of the residue model as the judge.  Tenants are visited in order of their profiled time
 * (`prof`: the table of gacer_profile); for each, the heaviest quarter of its not yet decomposed operators is
 * decomposed -- batch x2, batch x4, output channels x2, or the chunk list {3/4, 1/4} of the batch -- and the first
 * option that lowers the median makespan of `trial_rounds` rounds by more than the fraction `min_gain` is kept.
 * The plan's edges are left as they are.  The refined plan stays installed and is also returned in *out (free with
 * gacer_plan_free); *ms_out (may be NULL) receives its measured makespan.  Outputs stay bit-identical: every
 * candidate is a valid plan.  Runs 3 + trial_rounds rounds per candidate.
 */
gacer_status gacer_refine(gacer_ctx *ctx, const gacer_prof *prof, size_t n, int trial_rounds, float min_gain,
                          gacer_plan **out, float *ms_out);

/* Host cost of the issue loop (the spatial-granularity discussion of Section 5.4, Table 3: decomposition adds
 * operators, and every operator costs the host an issue): wall time the last gacer_run spent enqueueing its
 * rounds, before it started to wait, and the number of operator launches it enqueued. */
gacer_status gacer_issue_stats(gacer_ctx *ctx, double *host_ms, int *launches);

#ifdef __cplusplus
}
#endif
#endif /* GACER_H */
