// Tenant registration, plan validation / expansion, the multi-stream issue loop and the
// per-operator profiler.  Host code only; kernels are reached through kernels.h.
//
// Temporal regulation (Section 4.3) is realised with hipEvents: a synchronisation pointer becomes
// "record on the producer stream, wait on the consumer streams".  The host never blocks inside a
// round, so the GPU does not idle while the CPU synchronises (the overhead analysed around Eq. 8
// shrinks to the device-side wait).
#include <hip/hip_runtime.h>
#include <algorithm>
#include <atomic>
#include <chrono>
#include <memory>
#include <mutex>
#include <thread>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <new>
#include <set>
#include <tuple>
#include "ctx.h"

using namespace gacer;

#define HIPCHK(ctx, call)                                                                                   \
    do {                                                                                                    \
        hipError_t e_ = (call);                                                                             \
        if (e_ != hipSuccess) return fail(ctx, GACER_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));  \
    } while (0)

// issue_op under the checking mode names the launch that failed
#define ISSUE(ctx, call)                                                                                    \
    do {                                                                                                    \
        (ctx)->launch_detail.clear();                                                                       \
        hipError_t e_ = (call);                                                                             \
        if (e_ != hipSuccess && !(ctx)->launch_detail.empty()) return fail(ctx, GACER_EHIP, "%s", (ctx)->launch_detail.c_str()); \
        if (e_ != hipSuccess) return fail(ctx, GACER_EHIP, "issuing an operator failed: %s", hipGetErrorString(e_)); \
    } while (0)

// Workspace of gacer_run_static: device memory that belongs to the loaded code object, so that an entry point which
// may not allocate still has somewhere to put split-K partial tiles.  Every GPU the library runs on holds its own copy
// until the process ends.  In host code the array's name is only a stand-in; its device address is taken once per
// device with hipGetSymbolAddress (gacer_create) and kept here.
#define GACER_STATIC_SCRATCH_BYTES (32u << 20)
static __device__ __align__(256) unsigned char scratch[GACER_STATIC_SCRATCH_BYTES];
static constexpr int MAX_DEVICES = 64;
static unsigned char *g_scratch_ptr[MAX_DEVICES];
static hipError_t g_scratch_err[MAX_DEVICES];
static std::mutex g_scratch_mu;

// Device address of `scratch` on the current device `dev` (looked up on first use, with that device current).  The
// function has external linkage on purpose: the compiler keeps a file-local device array, and gives it a name the
// runtime can look up, only when it sees host code with external linkage refer to it.
namespace gacer { hipError_t scratch_address(int dev, unsigned char **out); }
hipError_t gacer::scratch_address(int dev, unsigned char **out)
{
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[dev] && g_scratch_err[dev] == hipSuccess) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) { (void)hipGetLastError(); g_scratch_err[dev] = e; }
        else g_scratch_ptr[dev] = (unsigned char *)p;
    }
    *out = g_scratch_ptr[dev];
    return g_scratch_err[dev];
}

static gacer_status fail(Ctx *c, gacer_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return st;
}

namespace gacer {

bool axis_legal(gacer_opkind kind, gacer_axis axis)
{
    if (axis == GACER_AXIS_BATCH) return true;
    if (axis == GACER_AXIS_COUT)
        return kind == GACER_CONV2D || kind == GACER_DWCONV2D || kind == GACER_GEMM || kind == GACER_MAXPOOL ||
               kind == GACER_GAVGPOOL || kind == GACER_AFFINE_ACT || kind == GACER_SCALE || kind == GACER_CONCAT ||
               kind == GACER_AVGPOOL;
    return false;
}

int axis_extent(const Tenant &t, int op, gacer_axis axis)
{
    if (axis == GACER_AXIS_BATCH) return t.batch;
    if (axis == GACER_AXIS_COUT) return (int)t.tensors[t.ops[op].out].c;
    return 1;
}

void chunk_range(int extent, int factor, int j, int *lo, int *hi)
{
    const int base = extent / factor, rem = extent % factor;
    *lo = j * base + std::min(j, rem);
    *hi = *lo + base + (j < rem ? 1 : 0);
}

static int dt(const Tenant &t) { return t.dtype == GACER_BF16 ? DT_BF16 : DT_F32; }

Launch make_launch(const Tenant &t, int oi, int b_lo, int b_hi, int c_lo, int c_hi)
{
    const gacer_op &op = t.ops[oi];
    const gacer_tensor &in = t.tensors[op.in0];
    const gacer_tensor &out = t.tensors[op.out];
    Launch l;
    std::memset(&l, 0, sizeof l);
    const int q_out = (int)(out.n / t.batch), q_in = (int)(in.n / t.batch);
    const size_t esz = t.dtype == GACER_BF16 ? 2 : 4;
    GemmArgs &g = l.g;
    StreamArgs &s = l.s;
    g.dtype = s.dtype = dt(t);
    g.alpha = 1.f;
    g.zb = g.zh = 1;
    g.ksplit = 1; g.kb_per_slice = 1 << 28;
    g.act = s.act = (int)op.act;
    switch (op.kind) {
    case GACER_CONV2D:
    case GACER_GEMM: {
        l.kind = LK_IGEMM;
        g.x = in.dptr; g.w = op.w; g.bias = op.bias; g.y = out.dptr;
        g.res = op.res >= 0 ? t.tensors[op.res].dptr : nullptr;
        const bool flat = (op.kind == GACER_GEMM) && (op.cin != in.c || in.h * in.w == 1);
        if (flat) {
            g.H = g.W = 1; g.Cin = op.cin; g.Ho = g.Wo = 1;
            g.kh = g.kw = 1; g.stride = 1; g.pad = 0;
            g.x_pix = op.cin; g.x_img = op.cin;
        } else {
            g.H = (int)in.h; g.W = (int)in.w; g.Cin = (int)in.c; g.Ho = (int)out.h; g.Wo = (int)out.w;
            g.kh = op.kind == GACER_GEMM ? 1 : op.kh; g.kw = op.kind == GACER_GEMM ? 1 : op.kw;
            g.stride = op.kind == GACER_GEMM ? 1 : op.stride; g.pad = op.kind == GACER_GEMM ? 0 : op.pad;
            const int64_t pitch = in.pitch ? in.pitch : in.c;
            g.x_pix = pitch; g.x_img = in.h * in.w * pitch;
        }
        g.K = g.kh * g.kw * g.Cin;
        g.x_bytes = (in.n * in.h * in.w * (in.pitch ? in.pitch : in.c) - (in.pitch ? in.c_off : 0)) * (int64_t)esz;   // to the end of the allocation
        g.w_bytes = (int64_t)out.c * g.K * (int64_t)esz;
        g.w_row = g.K;
        g.y_row = out.pitch ? out.pitch : out.c;
        g.m_lo = b_lo * q_out * g.Ho * g.Wo; g.m_hi = b_hi * q_out * g.Ho * g.Wo;
        g.n_lo = c_lo; g.n_hi = c_hi;
        g.ksplit = t.ksplit[oi]; g.kb_per_slice = t.kb_per_slice[oi];
        g.ws = nullptr;                       // the workspace is chosen per call (see enqueue)
        break;
    }
    case GACER_BGEMM_QK: {
        // scores[b*heads+hd][query i][key j] = alpha * sum_d q[b,i,hd,d] * k[b,j,hd,d]
        l.kind = LK_IGEMM;
        const int heads = op.groups, dh = op.cin, S = (int)in.h;
        const int64_t D = (int64_t)heads * dh;
        g.x = in.dptr; g.w = (const char *)in.dptr + D * esz; g.y = out.dptr;
        g.x_bytes = in.n * in.c * in.h * in.w * (int64_t)esz;
        g.w_bytes = g.x_bytes - D * (int64_t)esz;
        g.H = S; g.W = 1; g.Cin = dh; g.Ho = S; g.Wo = 1; g.kh = g.kw = 1; g.stride = 1; g.pad = 0;
        g.K = dh; g.x_pix = 3 * D; g.x_img = 0; g.w_row = 3 * D; g.y_row = S;
        g.m_lo = 0; g.m_hi = S; g.n_lo = 0; g.n_hi = S;
        g.alpha = op.alpha; g.act = ACT_NONE;
        g.zh = heads; g.zb = (b_hi - b_lo) * q_in; g.z_lo = b_lo * q_in;
        g.x_zb = S * 3 * D; g.x_zh = dh; g.w_zb = S * 3 * D; g.w_zh = dh;
        g.y_zb = (int64_t)heads * S * S; g.y_zh = (int64_t)S * S;
        break;
    }
    case GACER_BGEMM_PV: {
        // ctx[b][i][hd*dh+d] = sum_j p[b*heads+hd][i][j] * v[b,j,hd,d]
        l.kind = LK_IGEMM;
        const gacer_tensor &qkv = t.tensors[op.in1];
        const int heads = op.groups, dh = op.cout, S = (int)qkv.h;
        const int64_t D = (int64_t)heads * dh;
        g.x = in.dptr; g.w = (const char *)qkv.dptr + 2 * D * esz; g.y = out.dptr;
        g.x_bytes = in.n * in.c * in.h * in.w * (int64_t)esz;
        g.w_bytes = qkv.n * qkv.c * qkv.h * qkv.w * (int64_t)esz - 2 * D * (int64_t)esz;
        g.H = S; g.W = 1; g.Cin = S; g.Ho = S; g.Wo = 1; g.kh = g.kw = 1; g.stride = 1; g.pad = 0;
        g.K = S; g.x_pix = S; g.x_img = 0; g.w_row = 3 * D; g.y_row = D;
        g.m_lo = 0; g.m_hi = S; g.n_lo = 0; g.n_hi = dh;
        g.act = ACT_NONE; g.b_trans = 1;
        const int qb = (int)(qkv.n / t.batch);
        g.zh = heads; g.zb = (b_hi - b_lo) * qb; g.z_lo = b_lo * qb;
        g.x_zb = (int64_t)heads * S * S; g.x_zh = (int64_t)S * S; g.w_zb = S * 3 * D; g.w_zh = dh;
        g.y_zb = S * D; g.y_zh = dh;
        break;
    }
    default: {
        s.x = in.dptr; s.y = out.dptr;
        s.x2 = op.in1 >= 0 ? t.tensors[op.in1].dptr : nullptr;
        s.res = op.res >= 0 ? t.tensors[op.res].dptr : nullptr;
        s.w = op.w; s.bias = op.bias; s.scale = op.scale; s.shift = op.shift;
        s.N = (int)in.n; s.H = (int)in.h; s.W = (int)in.w; s.C = (int)in.c; s.Ho = (int)out.h; s.Wo = (int)out.w;
        s.k = op.kh; s.stride = op.stride; s.pad = op.pad;
        s.eps = op.alpha;
        s.n_lo = b_lo * q_out; s.n_hi = b_hi * q_out; s.c_lo = c_lo; s.c_hi = c_hi;
        s.rows_per_item = (int64_t)q_out * out.h * out.w;
        s.gate = nullptr; s.c_split = 0; s.pool_avg = 0;
        s.x_pitch = in.pitch ? in.pitch : in.c; s.y_pitch = out.pitch ? out.pitch : out.c;
        switch (op.kind) {
        case GACER_DWCONV2D: l.kind = LK_DWCONV; break;
        case GACER_MAXPOOL: l.kind = LK_MAXPOOL; break;
        case GACER_AVGPOOL: l.kind = LK_MAXPOOL; s.pool_avg = 1; break;
        case GACER_SCALE: l.kind = LK_ELTWISE; s.gate = s.x2; s.x2 = nullptr; s.scale = s.shift = nullptr; break;
        case GACER_CONCAT: l.kind = LK_CONCAT; s.c_split = (int)in.c; s.C = (int)out.c; break;
        case GACER_GAVGPOOL: l.kind = LK_GAVGPOOL; break;
        case GACER_LAYERNORM: l.kind = LK_LAYERNORM; s.n_lo = b_lo; s.n_hi = b_hi; break;
        case GACER_SOFTMAX: l.kind = LK_SOFTMAX; s.n_lo = b_lo; s.n_hi = b_hi; break;
        default: l.kind = LK_ELTWISE; break;
        }
        if (op.kind == GACER_ADD || op.kind == GACER_ACT) { s.scale = s.shift = nullptr; }
        if (op.kind == GACER_ACT) s.x2 = nullptr;
    }
    }
    return l;
}

LaunchInfo enqueue(const Launch &l, hipStream_t s, bool dry, int phase, float *ws)
{
    switch (l.kind) {
    case LK_IGEMM:
        if (l.g.ksplit > 1 && !dry) {
            if (!ws) return launch_igemm(l.g, s, true, phase);     // never launch slices without a workspace
            GemmArgs g = l.g;
            g.ws = ws + l.ws_off;
            return launch_igemm(g, s, dry, phase);
        }
        return launch_igemm(l.g, s, dry, phase);
    case LK_DWCONV: return launch_dwconv(l.s, s, dry);
    case LK_MAXPOOL: return launch_maxpool(l.s, s, dry);
    case LK_CONCAT: return launch_concat(l.s, s, dry);
    case LK_GAVGPOOL: return launch_gavgpool(l.s, s, dry);
    case LK_LAYERNORM: return launch_layernorm(l.s, s, dry);
    case LK_SOFTMAX: return launch_softmax(l.s, s, dry);
    default: return launch_eltwise(l.s, s, dry);
    }
}

// Library-allocated plan.  The split array carries one extra trailing element whose `sizes` owns the pool that the
// chunk lists of the real elements point into; gacer_plan_free releases it.
gacer_plan *make_plan(const std::vector<gacer_split> &splits, const std::vector<gacer_sync> &syncs)
{
    size_t pool_n = 0;
    for (const gacer_split &s : splits)
        if (s.sizes) pool_n += (size_t)s.factor;
    gacer_plan *pl = new (std::nothrow) gacer_plan();
    gacer_split *sp = new (std::nothrow) gacer_split[splits.size() + 1];
    gacer_sync *sy = new (std::nothrow) gacer_sync[syncs.size() + 1];
    int *pool = new (std::nothrow) int[pool_n + 1];
    if (!pl || !sp || !sy || !pool) { delete pl; delete[] sp; delete[] sy; delete[] pool; return nullptr; }
    size_t used = 0;
    for (size_t k = 0; k < splits.size(); ++k) {
        sp[k] = splits[k];
        if (splits[k].sizes) {
            std::copy(splits[k].sizes, splits[k].sizes + splits[k].factor, pool + used);
            sp[k].sizes = pool + used;
            used += (size_t)splits[k].factor;
        }
    }
    sp[splits.size()] = {-1, -1, GACER_AXIS_NONE, 0, pool};
    std::copy(syncs.begin(), syncs.end(), sy);
    pl->n_split = (int)splits.size(); pl->split = sp;
    pl->n_sync = (int)syncs.size(); pl->sync = sy;
    return pl;
}

}  // namespace gacer

// ------------------------------------------------------------------------------------------------
static bool same_shape(const gacer_tensor &a, const gacer_tensor &b) { return a.n == b.n && a.c == b.c && a.h == b.h && a.w == b.w; }

// Which channels of which allocation hold data: a strided tensor is a channel window of its base tensor, every other
// tensor owns its channels.  A tensor is readable when all of its channels are written, writable when none is.
struct Written {
    const gacer_tenant &t;
    std::vector<std::vector<char>> ch;
    explicit Written(const gacer_tenant &tt) : t(tt), ch(tt.n_tensors)
    {
        for (int i = 0; i < t.n_tensors; ++i)
            if (!t.tensors[i].pitch) ch[i].assign((size_t)t.tensors[i].c, 0);
    }
    int owner(int i) const { return t.tensors[i].pitch ? t.tensors[i].base : i; }
    int first(int i) const { return t.tensors[i].pitch ? t.tensors[i].c_off : 0; }
    int count(int i) const
    {
        const std::vector<char> &v = ch[owner(i)];
        int k = 0;
        for (int64_t q = 0; q < t.tensors[i].c; ++q) k += v[first(i) + q];
        return k;
    }
    bool all(int i) const { return count(i) == t.tensors[i].c; }
    bool none(int i) const { return count(i) == 0; }
    void mark(int i)
    {
        std::vector<char> &v = ch[owner(i)];
        for (int64_t q = 0; q < t.tensors[i].c; ++q) v[first(i) + q] = 1;
    }
};

static gacer_status check_op(Ctx *c, int ti, const gacer_tenant &t, int oi, const Written &written)
{
    const gacer_op &op = t.ops[oi];
    auto bad = [&](const char *why) { return fail(c, GACER_ESHAPE, "tenant %d op %d: %s", ti, oi, why); };
    auto idx_ok = [&](int i, bool required) {
        if (i < 0) return !required;
        return i < t.n_tensors && written.all(i);
    };
    if ((int)op.kind < 0 || (int)op.kind > (int)GACER_AVGPOOL) return fail(c, GACER_EINVAL, "tenant %d op %d: unknown kind", ti, oi);
    if ((int)op.act < 0 || (int)op.act > (int)GACER_ACT_HSIGMOID) return fail(c, GACER_EINVAL, "tenant %d op %d: unknown activation", ti, oi);
    if (!idx_ok(op.in0, true)) return bad("in0 missing or not written by an earlier operator");
    if (!idx_ok(op.in1, false) || !idx_ok(op.res, false)) return bad("in1/res not written by an earlier operator");
    if (op.out < 0 || op.out >= t.n_tensors) return bad("out index out of range");
    if (!written.none(op.out)) return bad("out tensor is written twice");
    const gacer_tensor &in = t.tensors[op.in0], &out = t.tensors[op.out];
    {   // channel windows: only where the kernels take a position pitch
        const bool per_position = op.kind == GACER_CONV2D || (op.kind == GACER_GEMM && op.cin == in.c && in.h * in.w > 1);
        const bool in_ok = per_position || op.kind == GACER_AFFINE_ACT || op.kind == GACER_ACT;
        const bool out_ok = in_ok || op.kind == GACER_MAXPOOL || op.kind == GACER_AVGPOOL;
        if (in.pitch && !in_ok) return bad("in0 is a channel window, which this operator kind does not read");
        if (out.pitch && (!out_ok || op.res >= 0)) return bad("out is a channel window, which this operator kind (or an operator with a residual) does not write");
        if ((op.in1 >= 0 && t.tensors[op.in1].pitch) || (op.res >= 0 && t.tensors[op.res].pitch)) return bad("in1 / res must not be channel windows");
    }
    if (op.res >= 0 && !same_shape(t.tensors[op.res], out)) return bad("res shape differs from out");
    const int B = t.batch;
    switch (op.kind) {
    case GACER_CONV2D:
    case GACER_DWCONV2D: {
        if (!op.w) return fail(c, GACER_EINVAL, "tenant %d op %d: null weights", ti, oi);
        if (op.kh < 1 || op.kw < 1 || op.kh > 31 || op.kw > 31 || op.stride < 1 || op.pad < 0) return bad("bad kernel/stride/pad (kernel extent 1..31)");
        if (op.cin != in.c || op.cout != out.c || in.n != out.n) return bad("cin/cout/n do not match the tensors");
        if (out.h != (in.h + 2 * op.pad - op.kh) / op.stride + 1 || out.w != (in.w + 2 * op.pad - op.kw) / op.stride + 1)
            return bad("output extent does not match (h+2*pad-k)/stride+1");
        if (op.kind == GACER_DWCONV2D) {
            if (op.groups != op.cin || op.cin != op.cout || op.kh != op.kw) return bad("depthwise needs groups == cin == cout, square kernel");
        } else if (op.groups != 1) return bad("grouped convolution other than depthwise is not supported");
        break;
    }
    case GACER_GEMM: {
        if (!op.w) return fail(c, GACER_EINVAL, "tenant %d op %d: null weights", ti, oi);
        if (op.cout != out.c || in.n != out.n) return bad("cout/n do not match the tensors");
        if (op.cin == in.c) { if (out.h != in.h || out.w != in.w) return bad("per-position GEMM must keep h,w"); }
        else if (op.cin == in.c * in.h * in.w) { if (out.h != 1 || out.w != 1) return bad("flattening GEMM must produce h = w = 1"); }
        else return bad("cin is neither c nor c*h*w of in0");
        break;
    }
    case GACER_BGEMM_QK: {
        const int64_t D = (int64_t)op.groups * op.cin;
        if (op.groups < 1 || op.cin < 1 || in.c != 3 * D || in.w != 1) return bad("in0 must be (B, 3*heads*dh, S, 1)");
        if (out.n != in.n * op.groups || out.c != in.h || out.h != in.h || out.w != 1) return bad("out must be (B*heads, S, S, 1)");
        break;
    }
    case GACER_BGEMM_PV: {
        if (!idx_ok(op.in1, true)) return bad("in1 (qkv) missing");
        const gacer_tensor &qkv = t.tensors[op.in1];
        const int64_t D = (int64_t)op.groups * op.cout;
        if (op.groups < 1 || op.cout < 1 || qkv.c != 3 * D || qkv.w != 1) return bad("in1 must be (B, 3*heads*dh, S, 1)");
        if (in.n != qkv.n * op.groups || in.c != qkv.h || in.h != qkv.h || in.w != 1) return bad("in0 must be (B*heads, S, S, 1)");
        if (out.n != qkv.n || out.c != D || out.h != qkv.h || out.w != 1) return bad("out must be (B, heads*dh, S, 1)");
        if (qkv.h % 8 || op.cout % 8) return bad("attention context needs S and head size to be multiples of 8");
        break;
    }
    case GACER_MAXPOOL:
        if (op.kh < 1 || op.stride < 1 || op.pad < 0 || 2 * op.pad > op.kh) return bad("bad window");
        if (in.n != out.n || in.c != out.c || out.h != (in.h + 2 * op.pad - op.kh) / op.stride + 1 ||
            out.w != (in.w + 2 * op.pad - op.kh) / op.stride + 1) return bad("output extent mismatch");
        break;
    case GACER_AVGPOOL:
        if (op.kh < 1 || op.stride < 1 || op.pad != 0 || op.kh > in.h || op.kh > in.w) return bad("bad window (mean pooling is unpadded)");
        if (in.n != out.n || in.c != out.c || out.h != (in.h - op.kh) / op.stride + 1 || out.w != (in.w - op.kh) / op.stride + 1)
            return bad("output extent mismatch");
        break;
    case GACER_GAVGPOOL:
        if (in.n != out.n || in.c != out.c || out.h != 1 || out.w != 1) return bad("out must be (n,c,1,1)");
        break;
    case GACER_SCALE: {
        if (!idx_ok(op.in1, true) || !same_shape(in, out)) return bad("scale needs in0 of the output shape and a gate in1");
        const gacer_tensor &g = t.tensors[op.in1];
        if (g.n != in.n || g.c != in.c || g.h != 1 || g.w != 1) return bad("gate must be (n,c,1,1)");
        break;
    }
    case GACER_CONCAT: {
        if (!idx_ok(op.in1, true)) return bad("concat needs two inputs");
        const gacer_tensor &b = t.tensors[op.in1];
        if (in.n != out.n || b.n != out.n || in.h != out.h || b.h != out.h || in.w != out.w || b.w != out.w || in.c + b.c != out.c ||
            op.cin != in.c || op.cout != out.c) return bad("concat: out must be (n, c(in0)+c(in1), h, w) with cin = c(in0)");
        break;
    }
    case GACER_AFFINE_ACT:
        if (!op.scale || !op.shift) return fail(c, GACER_EINVAL, "tenant %d op %d: null scale/shift", ti, oi);
        if (!same_shape(in, out)) return bad("in/out shapes differ");
        break;
    case GACER_ADD:
        if (!idx_ok(op.in1, true) || !same_shape(in, out) || !same_shape(t.tensors[op.in1], out)) return bad("add needs two inputs of the output shape");
        break;
    case GACER_LAYERNORM:
        if (!op.scale || !op.shift) return fail(c, GACER_EINVAL, "tenant %d op %d: null gamma/beta", ti, oi);
        if (!same_shape(in, out)) return bad("in/out shapes differ");
        break;
    case GACER_SOFTMAX:
    case GACER_ACT:
        if (!same_shape(in, out)) return bad("in/out shapes differ");
        break;
    }
    if (in.n % B || out.n % B) return bad("tensor n is not a multiple of the tenant batch");
    return GACER_OK;
}

// Split-K decision, from the operator's UNSPLIT shape only (so every chunk of it adds in the same order):
// when 64x64 tiles alone would leave most compute units idle, cut K into up to 16 slices of at least four
// 64-byte blocks, aiming at about two workgroups per compute unit.
static void decide_split(int64_t M, int64_t N, int K, gacer_dtype dtype, int *S, int *kbps)
{
    const int bk = dtype == GACER_BF16 ? 32 : 16;
    const int nkb = (K + bk - 1) / bk;
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64);
    int64_t s = 1;
    // Measured on whole concurrent rounds: splitting pays only when the unsplit launch would leave more than half of
    // the compute units empty, and only with slices of at least 8 blocks (the finishing pass costs a kernel boundary).
    if (tiles < 128) {
        // all workgroups of such a launch are resident at once, so its duration follows the fullest compute unit:
        // prefer the slice count whose workgroup total sits just below a multiple of the 256 compute units
        const int64_t smax = std::min<int64_t>(16, nkb / 8);
        double best = -1.0;
        for (int64_t q = 1; q <= smax; ++q) {
            const int64_t wgs = tiles * q;
            if (wgs > 1024) break;
            const double fill = (double)wgs / (double)(((wgs + 255) / 256) * 256);
            const double score = (wgs >= 256 ? 1.0 : (double)wgs / 256.0) * fill - 0.01 * (double)q;   // mild bias to fewer slices
            if (score > best) { best = score; s = q; }
        }
    }
    int per = (int)((nkb + s - 1) / s);
    per += per & 1;
    *kbps = s == 1 ? (1 << 28) : per;
    *S = s == 1 ? 1 : (nkb + per - 1) / per;
}

static void release_workspaces(std::vector<Tenant> &ts)
{
    for (Tenant &t : ts) {
        if (t.ws) (void)hipFree(t.ws);
        t.ws = nullptr;
    }
}

// Sizes the per-tenant split-K workspace and tries to allocate it.  Without a usable device the pointers
// stay null and gacer_run reports the failure; descriptor-only use (validation, search) still works.
static void plan_workspaces(Ctx *c, std::vector<Tenant> &ts)
{
    for (Tenant &t : ts) {
        t.ksplit.assign(t.ops.size(), 1);
        t.kb_per_slice.assign(t.ops.size(), 1 << 28);
        t.ws_floats = 0;
        for (size_t i = 0; i < t.ops.size(); ++i) {
            const gacer_op &op = t.ops[i];
            if (op.kind != GACER_CONV2D && op.kind != GACER_GEMM) continue;
            const gacer_tensor &in = t.tensors[op.in0], &out = t.tensors[op.out];
            const int64_t M = out.n * out.h * out.w, N = out.c;
            const int K = op.kind == GACER_GEMM ? op.cin : (int)in.c * op.kh * op.kw;
            decide_split(M, N, K, t.dtype, &t.ksplit[i], &t.kb_per_slice[i]);
            if (t.ksplit[i] > 1) t.ws_floats = std::max<size_t>(t.ws_floats, (size_t)t.ksplit[i] * M * N);
        }
        if (t.ws_floats) {
            if (hipMalloc((void **)&t.ws, t.ws_floats * sizeof(float)) != hipSuccess) {
                (void)hipGetLastError();
                t.ws = nullptr;
                c->ws_missing = true;
            }
        }
    }
}

// ---- per-channel affine + the 1x1 convolution that reads it, as one launch --------------------------------------------------
// A network whose BatchNorms follow concatenations (DenseNet) runs an affine + ReLU kernel over all features in front of
// every bottleneck convolution; in a chain of kernels a few microseconds long that launch costs as much as the work.  Where
// it can, the executor issues operator i (affine, no residual, activation none / ReLU / ReLU6) and operator i + 1 (1x1
// convolution, stride 1, reading i's output) as one launch of the product, whose A loader applies the affine operator's
// arithmetic on the way in and also writes operator i's output tensor; operator i then has no launch of its own.  Both give
// the bits of the two stand-alone kernels.  Not fused: pairs of which either operator is decomposed by the plan, pairs whose
// first operator's completion is a sync pointer's source, operands that are not 16-byte aligned or whose channel count is
// not a multiple of a 16-byte vector.
static bool aligned16p(const void *p) { return ((uintptr_t)p & 15) == 0; }

static bool fusable_pair(const Tenant &T, int i)
{
    if (i + 1 >= (int)T.ops.size()) return false;
    const gacer_op &af = T.ops[i], &pw = T.ops[i + 1];
    if (af.kind != GACER_AFFINE_ACT || pw.kind != GACER_CONV2D) return false;
    if (af.res >= 0 || (af.act != GACER_ACT_NONE && af.act != GACER_ACT_RELU && af.act != GACER_ACT_RELU6)) return false;
    if (pw.kh != 1 || pw.kw != 1 || pw.stride != 1 || pw.pad != 0 || pw.groups != 1 || pw.in0 != af.out || pw.res == af.out) return false;
    const gacer_tensor &in = T.tensors[af.in0], &mid = T.tensors[af.out];
    const int vec = T.dtype == GACER_BF16 ? 8 : 4;
    if (in.c % vec) return false;
    return aligned16p(in.dptr) && aligned16p(mid.dptr) && aligned16p(af.scale) && aligned16p(af.shift) && aligned16p(pw.w);
}

// `pw` is the unsplit launch of operator i + 1; turns it into the fused launch of operators i and i + 1
static void fuse_into(Launch &pw, const Tenant &T, int i)
{
    const gacer_op &af = T.ops[i];
    GemmArgs &g = pw.g;
    const gacer_tensor &in = T.tensors[af.in0];  // same shape as the tensor the product read before, possibly a channel window
    const int64_t pitch = in.pitch ? in.pitch : in.c;
    g.x = in.dptr; g.x_pix = pitch; g.x_img = in.h * in.w * pitch;
    g.x_bytes = (in.n * in.h * in.w * pitch - (in.pitch ? in.c_off : 0)) * (int64_t)(T.dtype == GACER_BF16 ? 2 : 4);
    g.pre_scale = af.scale; g.pre_shift = af.shift; g.pre_y = T.tensors[af.out].dptr; g.pre_act = (int)af.act;
}

template <typename Decomposed, typename Recorded>
static void fuse_affine_pairs(Ctx *c, std::vector<std::vector<OpExec>> &ex, Decomposed decomposed, Recorded recorded)
{
    if (!c->fuse_affine) return;
    for (size_t t = 0; t < c->tenants.size(); ++t) {
        const Tenant &T = c->tenants[t];
        for (int i = 0; i + 1 < (int)T.ops.size(); ++i) {
            if (!fusable_pair(T, i) || decomposed((int)t, i) || decomposed((int)t, i + 1) || recorded((int)t, i)) continue;
            if (ex[t][i].chunks.size() != 1 || ex[t][i + 1].chunks.size() != 1) continue;
            fuse_into(ex[t][i + 1].chunks[0], T, i);
            ex[t][i].chunks.clear();
            ++i;                                 // the product is taken
        }
    }
}

static void expand_plain(Ctx *c)
{
    c->plain_exec.assign(c->tenants.size(), {});
    c->par_order.clear();
    size_t longest = 0;
    for (size_t t = 0; t < c->tenants.size(); ++t) {
        const Tenant &T = c->tenants[t];
        c->plain_exec[t].resize(T.ops.size());
        for (size_t i = 0; i < T.ops.size(); ++i)
            c->plain_exec[t][i].chunks.push_back(make_launch(T, (int)i, 0, T.batch, 0, (int)T.tensors[T.ops[i].out].c));
        longest = std::max(longest, T.ops.size());
    }
    fuse_affine_pairs(c, c->plain_exec, [](int, int) { return false; }, [](int, int) { return false; });
    for (size_t i = 0; i < longest; ++i)
        for (size_t t = 0; t < c->tenants.size(); ++t)
            if (i < c->tenants[t].ops.size()) c->par_order.push_back({(int)t, (int)i});
}

namespace { gacer_status ensure_plan_events(Ctx *c); }

// Validates and expands (splits, syncs) into c->plan_exec / plan_order.  On failure nothing changes.
static gacer_status install_plan(Ctx *c, const std::vector<gacer_split> &splits, const std::vector<gacer_sync> &syncs)
{
    const int NT = (int)c->tenants.size();
    std::map<std::pair<int, int>, gacer_split> smap;
    for (const gacer_split &s : splits) {
        if (s.tenant < 0 || s.tenant >= NT || s.op < 0 || s.op >= (int)c->tenants[s.tenant].ops.size())
            return fail(c, GACER_EPLAN, "split names a missing operator (tenant %d op %d)", s.tenant, s.op);
        if (s.sizes) {
            if (s.factor < 1 || s.factor > 8)
                return fail(c, GACER_EPLAN, "tenant %d op %d: a chunk list holds 1..8 sizes, not %d", s.tenant, s.op, s.factor);
        } else if (s.factor != 1 && s.factor != 2 && s.factor != 4 && s.factor != 8)
            return fail(c, GACER_EPLAN, "tenant %d op %d: factor %d not in {1,2,4,8}", s.tenant, s.op, s.factor);
        if (smap.count({s.tenant, s.op})) return fail(c, GACER_EPLAN, "tenant %d op %d: split listed twice", s.tenant, s.op);
        if (s.factor > 1) {
            const Tenant &T = c->tenants[s.tenant];
            if (s.axis != GACER_AXIS_BATCH && s.axis != GACER_AXIS_COUT)
                return fail(c, GACER_EPLAN, "tenant %d op %d: factor > 1 needs an axis", s.tenant, s.op);
            if (!axis_legal(T.ops[s.op].kind, s.axis))
                return fail(c, GACER_EPLAN, "tenant %d op %d: this operator kind cannot be split on that axis", s.tenant, s.op);
            if (s.factor > axis_extent(T, s.op, s.axis))
                return fail(c, GACER_EPLAN, "tenant %d op %d: factor %d exceeds the axis extent %d", s.tenant, s.op, s.factor,
                            axis_extent(T, s.op, s.axis));
        }
        if (s.sizes) {                       // list_B: positive sizes that sum to the extent (Eq. 5)
            int64_t sum = 0;
            for (int j = 0; j < s.factor; ++j) {
                if (s.sizes[j] < 1) return fail(c, GACER_EPLAN, "tenant %d op %d: chunk %d has size %d", s.tenant, s.op, j, s.sizes[j]);
                sum += s.sizes[j];
            }
            const int ext = s.factor > 1 ? axis_extent(c->tenants[s.tenant], s.op, s.axis) : (int)sum;
            if (sum != ext)
                return fail(c, GACER_EPLAN, "tenant %d op %d: chunk sizes sum to %lld, the axis extent is %d", s.tenant, s.op,
                            (long long)sum, ext);
        }
        smap[{s.tenant, s.op}] = s;
    }
    for (const gacer_sync &e : syncs) {
        if (e.src_tenant < 0 || e.src_tenant >= NT || e.dst_tenant < 0 || e.dst_tenant >= NT ||
            e.src_op < 0 || e.src_op >= (int)c->tenants[e.src_tenant].ops.size() ||
            e.dst_op < 0 || e.dst_op >= (int)c->tenants[e.dst_tenant].ops.size())
            return fail(c, GACER_EPLAN, "sync edge names a missing operator");
        if (e.src_tenant == e.dst_tenant) return fail(c, GACER_EPLAN, "sync edge inside one tenant (stream order already holds)");
        if (e.when != 0 && e.when != 1) return fail(c, GACER_EPLAN, "sync edge: when must be 0 or 1");
    }
    // topological issue order over (stream order U sync edges); round-robin over tenants so that
    // every stream receives work early.  No progress in a sweep means a cycle.
    std::vector<std::vector<std::vector<std::pair<int, int>>>> deps(NT);
    for (int t = 0; t < NT; ++t) deps[t].resize(c->tenants[t].ops.size());
    for (const gacer_sync &e : syncs) deps[e.dst_tenant][e.dst_op].push_back({e.src_tenant, e.src_op});
    std::vector<int> pos(NT, 0);
    std::vector<std::pair<int, int>> order;
    size_t total = 0;
    for (int t = 0; t < NT; ++t) total += c->tenants[t].ops.size();
    while (order.size() < total) {
        bool progress = false;
        for (int t = 0; t < NT; ++t) {
            if (pos[t] >= (int)c->tenants[t].ops.size()) continue;
            bool ready = true;
            for (auto &d : deps[t][pos[t]]) ready = ready && (pos[d.first] > d.second);
            if (!ready) continue;
            order.push_back({t, pos[t]});
            ++pos[t];
            progress = true;
        }
        if (!progress) return fail(c, GACER_EPLAN, "sync edges form a cycle with the stream order (would deadlock)");
    }
    // events: one per distinct (source operator, when)
    std::map<std::tuple<int, int, int>, int> ev_of;
    for (const gacer_sync &e : syncs)
        if (!ev_of.count({e.src_tenant, e.src_op, e.when})) { const int id = (int)ev_of.size(); ev_of[{e.src_tenant, e.src_op, e.when}] = id; }
    std::vector<std::vector<OpExec>> ex(NT);
    int n_events = (int)ev_of.size();            // edge events first, then a fork / join pair per sibling decomposition
    for (int t = 0; t < NT; ++t) {
        const Tenant &T = c->tenants[t];
        ex[t].resize(T.ops.size());
        for (int i = 0; i < (int)T.ops.size(); ++i) {
            const int cout = (int)T.tensors[T.ops[i].out].c;
            auto it = smap.find({t, i});
            const int f = (it == smap.end()) ? 1 : it->second.factor;
            const gacer_axis ax = (it == smap.end() || f == 1) ? GACER_AXIS_NONE : it->second.axis;
            const int *sizes = (it == smap.end() || f == 1) ? nullptr : it->second.sizes;
            const bool sib = it != smap.end() && f > 1 && it->second.sibling != 0 && T.sibling && T.sibling != T.stream;
            if (sib) { ex[t][i].fork = n_events++; ex[t][i].join = n_events++; }
            int next = 0;
            for (int j = 0; j < f; ++j) {
                int lo, hi;
                if (ax == GACER_AXIS_BATCH) {
                    if (sizes) { lo = next; hi = next += sizes[j]; } else chunk_range(T.batch, f, j, &lo, &hi);
                    ex[t][i].chunks.push_back(make_launch(T, i, lo, hi, 0, cout));
                } else if (ax == GACER_AXIS_COUT) {
                    if (sizes) { lo = next; hi = next += sizes[j]; } else chunk_range(cout, f, j, &lo, &hi);
                    ex[t][i].chunks.push_back(make_launch(T, i, 0, T.batch, lo, hi));
                } else {
                    ex[t][i].chunks.push_back(make_launch(T, i, 0, T.batch, 0, cout));
                }
            }
            // chunks of one operator may run at the same time (sibling streams): each gets its own part of the tenant's
            // split-K workspace; the parts add up to what the unsplit operator needs
            size_t off = 0;
            for (Launch &l : ex[t][i].chunks) {
                if (l.kind != LK_IGEMM || l.g.ksplit <= 1) continue;
                l.ws_off = off;
                off += (size_t)l.g.ksplit * (size_t)(l.g.m_hi - l.g.m_lo) * (size_t)(l.g.n_hi - l.g.n_lo);
            }
        }
    }
    for (const gacer_sync &e : syncs) {
        const int id = ev_of[{e.src_tenant, e.src_op, e.when}];
        if (e.when == 0) ex[e.src_tenant][e.src_op].record = id;
        else ex[e.src_tenant][e.src_op].pre_record = id;
        auto &w = ex[e.dst_tenant][e.dst_op].waits;
        if (std::find(w.begin(), w.end(), id) == w.end()) w.push_back(id);
    }
    fuse_affine_pairs(c, ex,
                      [&](int t, int i) { auto it = smap.find({t, i}); return it != smap.end() && it->second.factor > 1; },
                      [&](int t, int i) { return ex[t][i].record >= 0; });
    for (Tenant &t : c->tenants) (void)hipStreamSynchronize(t.stream);
    drop_graphs(c);                      // captured rounds belong to the plan they were captured under
    c->splits = splits;
    c->split_sizes.assign(splits.size(), {});
    for (size_t k = 0; k < splits.size(); ++k)
        if (splits[k].sizes) {
            c->split_sizes[k].assign(splits[k].sizes, splits[k].sizes + splits[k].factor);
            c->splits[k].sizes = c->split_sizes[k].data();
        }
    c->syncs = syncs;
    c->plan_exec.swap(ex);
    c->plan_order.swap(order);
    c->n_sync_events = (size_t)n_events;
    if (c->has_device) return ensure_plan_events(c);    // fork / join / edge events are created at set-up, not by a run
    return GACER_OK;
}

// ------------------------------------------------------------------------------------------------
extern "C" {

gacer_status gacer_create(gacer_ctx **out)
{
    if (!out) return GACER_EINVAL;
    gacer_ctx *c = new (std::nothrow) gacer_ctx();
    if (!c) return GACER_ENOMEM;
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) {
        c->device = dev;
        c->has_device = true;
        unsigned char *unused = nullptr;
        (void)scratch_address(dev, &unused);     // set-up of gacer_run_static's workspace; a failure is reported by that call
        int cu = 0;
        if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cu > 0) c->n_cu = cu;
    } else {
        (void)hipGetLastError();   // no device: descriptor-only use (validation, search) still works
    }
    *out = c;
    return GACER_OK;
}

void gacer_destroy(gacer_ctx *c)
{
    if (!c) return;
    for (Tenant &t : c->tenants) (void)hipStreamSynchronize(t.stream);
    drop_graphs(c);
    release_workspaces(c->tenants);
    for (hipEvent_t e : c->sync_events) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->join_events) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->t_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->t_end) (void)hipEventDestroy(e);
    delete c;
}

const char *gacer_last_error(const gacer_ctx *c) { return c ? c->err.c_str() : "null context"; }

gacer_status gacer_load_tenants(gacer_ctx *c, const gacer_tenant *tenants, int n)
{
    if (!c) return GACER_EINVAL;
    if (!tenants || n < 1 || n > 64) return fail(c, GACER_EINVAL, "need 1..64 tenants");
    std::vector<Tenant> fresh(n);
    for (int ti = 0; ti < n; ++ti) {
        const gacer_tenant &t = tenants[ti];
        if (!t.ops || !t.tensors || t.n_ops < 1 || t.n_tensors < 1) return fail(c, GACER_EINVAL, "tenant %d: empty operator or tensor list", ti);
        if (t.dtype != GACER_F32 && t.dtype != GACER_BF16) return fail(c, GACER_EINVAL, "tenant %d: unknown dtype", ti);
        if (t.batch < 1) return fail(c, GACER_EINVAL, "tenant %d: batch < 1", ti);
        if (t.input < 0 || t.input >= t.n_tensors || t.output < 0 || t.output >= t.n_tensors)
            return fail(c, GACER_EINVAL, "tenant %d: input/output index out of range", ti);
        for (int i = 0; i < t.n_tensors; ++i) {
            const gacer_tensor &x = t.tensors[i];
            if (x.n < 1 || x.c < 1 || x.h < 1 || x.w < 1) return fail(c, GACER_ESHAPE, "tenant %d tensor %d: non-positive extent", ti, i);
            if (!x.dptr) return fail(c, GACER_EINVAL, "tenant %d tensor %d: null device pointer", ti, i);
            if (!x.pitch && ((uintptr_t)x.dptr) % 16) return fail(c, GACER_EINVAL, "tenant %d tensor %d: device pointer not 16-byte aligned", ti, i);
            if (x.n * x.c * x.h * x.w * (t.dtype == GACER_BF16 ? 2 : 4) >= ((int64_t)1 << 31))
                return fail(c, GACER_ESHAPE, "tenant %d tensor %d: 2 GiB or more", ti, i);
            if (x.pitch) {                      // a channel window of a wider, gap-free tensor
                if (x.base < 0 || x.base >= t.n_tensors || x.base == i) return fail(c, GACER_ESHAPE, "tenant %d tensor %d: base index out of range", ti, i);
                const gacer_tensor &b = t.tensors[x.base];
                if (b.pitch || b.c != x.pitch || b.n != x.n || b.h != x.h || b.w != x.w)
                    return fail(c, GACER_ESHAPE, "tenant %d tensor %d: base must be a gap-free tensor (n, pitch, h, w)", ti, i);
                if (x.c_off < 0 || x.c_off + x.c > x.pitch) return fail(c, GACER_ESHAPE, "tenant %d tensor %d: window leaves its base", ti, i);
                if ((const char *)x.dptr != (const char *)b.dptr + (size_t)x.c_off * (t.dtype == GACER_BF16 ? 2 : 4))
                    return fail(c, GACER_EINVAL, "tenant %d tensor %d: pointer is not base + c_off", ti, i);
            }
        }
        Written written(t);
        written.mark(t.input);
        for (int oi = 0; oi < t.n_ops; ++oi) {
            gacer_status st = check_op(c, ti, t, oi, written);
            if (st != GACER_OK) return st;
            const gacer_op &op = t.ops[oi];
            for (const void *p : {(const void *)op.w, (const void *)op.bias, (const void *)op.scale, (const void *)op.shift})
                if (((uintptr_t)p) % 16) return fail(c, GACER_EINVAL, "tenant %d op %d: parameter pointer not 16-byte aligned", ti, oi);
            written.mark(op.out);
        }
        if (!written.all(t.output)) return fail(c, GACER_ESHAPE, "tenant %d: output tensor is never written", ti);
        Tenant &T = fresh[ti];
        T.ops.assign(t.ops, t.ops + t.n_ops);
        T.tensors.assign(t.tensors, t.tensors + t.n_tensors);
        T.input = t.input; T.output = t.output; T.batch = t.batch; T.dtype = t.dtype;
        T.stream = (hipStream_t)t.stream;
        T.sibling = (hipStream_t)t.sibling_stream;
    }
    for (Tenant &t : c->tenants) (void)hipStreamSynchronize(t.stream);
    drop_graphs(c);
    release_workspaces(c->tenants);
    c->ws_missing = false;
    plan_workspaces(c, fresh);
    c->tenants.swap(fresh);
    c->ws_run.assign(c->tenants.size(), nullptr);
    c->loaded = true;
    expand_plain(c);
    c->err.clear();
    return install_plan(c, {}, {});
}

gacer_status gacer_set_plan(gacer_ctx *c, const gacer_plan *plan)
{
    if (!c) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "gacer_set_plan before gacer_load_tenants");
    std::vector<gacer_split> sp;
    std::vector<gacer_sync> sy;
    if (plan) {
        if ((plan->n_split > 0 && !plan->split) || (plan->n_sync > 0 && !plan->sync) || plan->n_split < 0 || plan->n_sync < 0)
            return fail(c, GACER_EINVAL, "plan arrays missing");
        sp.assign(plan->split, plan->split + plan->n_split);
        sy.assign(plan->sync, plan->sync + plan->n_sync);
    }
    return install_plan(c, sp, sy);
}

gacer_status gacer_plan_from_pointers(gacer_ctx *c, const int *P, int n_ptr, gacer_plan **out)
{
    if (!c || !out) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "gacer_plan_from_pointers before gacer_load_tenants");
    if (n_ptr < 0 || (n_ptr > 0 && !P)) return fail(c, GACER_EINVAL, "bad pointer matrix");
    const int NT = (int)c->tenants.size();
    for (int t = 0; t < NT; ++t)
        for (int j = 0; j < n_ptr; ++j) {
            const int p = P[t * n_ptr + j];
            if (p < 0 || p > (int)c->tenants[t].ops.size() || (j > 0 && p < P[t * n_ptr + j - 1]))
                return fail(c, GACER_EPLAN, "tenant %d: pointers must be sorted and lie in [0, n_ops]", t);
        }
    std::vector<gacer_sync> edges;
    for (int j = 0; j < n_ptr; ++j) {
        // Barrier j separates clusters j and j+1.  Only tenants with a non-empty segment j+1 take part on the
        // release side; the hub is the lowest of them, so every barrier has its own hub operator.  An empty
        // cluster j+1 needs no barrier of its own: barrier j+1 orders everything before it.
        auto seg_begin = [&](int t) { return P[t * n_ptr + j]; };
        auto seg_end = [&](int t) { return j + 1 < n_ptr ? P[t * n_ptr + j + 1] : (int)c->tenants[t].ops.size(); };
        int hub = -1;
        for (int t = 0; t < NT && hub < 0; ++t)
            if (seg_begin(t) < seg_end(t)) hub = t;
        if (hub < 0) continue;
        const int hub_first = seg_begin(hub);
        bool gathers = false;
        for (int a = 0; a < NT; ++a) {
            const int last = P[a * n_ptr + j] - 1;               // 0-based last operator of a's segments <= j
            if (a == hub || last < 0) continue;
            edges.push_back({a, last, hub, hub_first, 0});
            gathers = true;
        }
        if (!gathers && hub_first == 0) continue;                // nothing has run before this barrier
        for (int b = 0; b < NT; ++b) {
            if (b == hub || seg_begin(b) >= seg_end(b)) continue;
            edges.push_back({hub, hub_first, b, seg_begin(b), 1});
        }
    }
    gacer_plan *pl = make_plan({}, edges);
    if (!pl) return fail(c, GACER_ENOMEM, "out of memory");
    *out = pl;
    return GACER_OK;
}

// Plan <-> text.  One line per entry:  "split <tenant> <op> <axis> <factor> <sibling> [size ...]"  /  "sync <src_tenant>
// <src_op> <dst_tenant> <dst_op> <when>", after a header line "gacer-plan 1".
gacer_status gacer_plan_to_text(const gacer_plan *plan, char *buf, size_t cap, size_t *len)
{
    if (!plan || !len || plan->n_split < 0 || plan->n_sync < 0 || (plan->n_split > 0 && !plan->split) || (plan->n_sync > 0 && !plan->sync))
        return GACER_EINVAL;
    std::string text = "gacer-plan 1\n";
    char line[160];
    for (int k = 0; k < plan->n_split; ++k) {
        const gacer_split &s = plan->split[k];
        std::snprintf(line, sizeof line, "split %d %d %d %d %d", s.tenant, s.op, (int)s.axis, s.factor, s.sibling ? 1 : 0);
        text += line;
        if (s.sizes) {
            if (s.factor < 1 || s.factor > 8) return GACER_EINVAL;
            for (int j = 0; j < s.factor; ++j) { std::snprintf(line, sizeof line, " %d", s.sizes[j]); text += line; }
        }
        text += "\n";
    }
    for (int k = 0; k < plan->n_sync; ++k) {
        const gacer_sync &e = plan->sync[k];
        std::snprintf(line, sizeof line, "sync %d %d %d %d %d\n", e.src_tenant, e.src_op, e.dst_tenant, e.dst_op, e.when);
        text += line;
    }
    *len = text.size() + 1;
    if (!buf || cap == 0) return GACER_OK;
    if (cap < text.size() + 1) return GACER_EINVAL;
    std::memcpy(buf, text.c_str(), text.size() + 1);
    return GACER_OK;
}

gacer_status gacer_plan_from_text(const char *text, gacer_plan **out)
{
    if (!text || !out) return GACER_EINVAL;
    std::vector<gacer_split> splits;
    std::vector<gacer_sync> syncs;
    std::vector<std::vector<int>> lists;
    std::vector<size_t> list_of;                      // per split: index into lists, or npos
    const char *p = text;
    bool header = false;
    while (*p) {
        const char *eol = std::strchr(p, '\n');
        const std::string line(p, eol ? (size_t)(eol - p) : std::strlen(p));
        p = eol ? eol + 1 : p + line.size();
        if (line.find_first_not_of(" \t\r") == std::string::npos) continue;
        int a[5], used = 0;
        if (!header) {
            int version = 0;
            if (std::sscanf(line.c_str(), "gacer-plan %d", &version) != 1 || version != 1) return GACER_EPLAN;
            header = true;
        } else if (std::sscanf(line.c_str(), "split %d %d %d %d %d%n", &a[0], &a[1], &a[2], &a[3], &a[4], &used) == 5) {
            if (a[2] < 0 || a[2] > 2 || a[3] < 1 || a[3] > 8) return GACER_EPLAN;
            std::vector<int> sizes;
            const char *q = line.c_str() + used;
            int v = 0, adv = 0;
            while (std::sscanf(q, " %d%n", &v, &adv) == 1) { sizes.push_back(v); q += adv; }
            if (q[std::strspn(q, " \t\r")] != 0) return GACER_EPLAN;
            if (!sizes.empty() && (int)sizes.size() != a[3]) return GACER_EPLAN;
            splits.push_back({a[0], a[1], (gacer_axis)a[2], a[3], nullptr, a[4] ? 1 : 0});
            list_of.push_back(sizes.empty() ? (size_t)-1 : lists.size());
            if (!sizes.empty()) lists.push_back(sizes);
        } else if (std::sscanf(line.c_str(), "sync %d %d %d %d %d%n", &a[0], &a[1], &a[2], &a[3], &a[4], &used) == 5 &&
                   line.find_first_not_of(" \t\r", (size_t)used) == std::string::npos) {
            syncs.push_back({a[0], a[1], a[2], a[3], a[4]});
        } else {
            return GACER_EPLAN;
        }
    }
    if (!header) return GACER_EPLAN;
    for (size_t k = 0; k < splits.size(); ++k)
        if (list_of[k] != (size_t)-1) splits[k].sizes = lists[list_of[k]].data();
    gacer_plan *pl = make_plan(splits, syncs);
    if (!pl) return GACER_ENOMEM;
    *out = pl;
    return GACER_OK;
}

void gacer_plan_free(gacer_plan *p)
{
    if (!p) return;
    if (p->split) delete[] p->split[p->n_split].sizes;     // the chunk-list pool (see make_plan)
    delete[] p->split;
    delete[] p->sync;
    delete p;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------------
// Issue loop.  One function enqueues an operator (its waits, its chunk launches, its records); it serves the
// single-threaded loop, the per-tenant host threads and the traced runs alike.
namespace {

// Host-side ordering between issuing threads: an event must have been recorded by its owner thread before another
// thread may enqueue a wait on it (a wait on an event that was never recorded returns at once).  Generation
// counters, one per event, carry that; with one issuing thread the pointer is null.
struct IssueGate {
    std::unique_ptr<std::atomic<long>[]> ev_gen, join_gen;
    std::atomic<long> fork_gen{0};
    std::atomic<int> failed{0};
    bool wait_gen(const std::atomic<long> &g, long need) const
    {
        while (g.load(std::memory_order_acquire) < need) {
            if (failed.load(std::memory_order_relaxed)) return false;
            std::this_thread::yield();
        }
        return true;
    }
};

// Enqueues operator (t, i) of round `round` on stream s.  Returns the first HIP error, or hipErrorUnknown when another
// issuing thread has failed.
hipError_t issue_op(Ctx *c, int t, int i, const OpExec &e, hipStream_t s, bool with_events, int round, IssueGate *gate)
{
    hipError_t err;
    if (with_events) {
        for (int w : e.waits) {
            if (gate && !gate->wait_gen(gate->ev_gen[w], round + 1)) return hipErrorUnknown;
            if ((err = hipStreamWaitEvent(s, c->sync_events[w], 0)) != hipSuccess) return err;
        }
        if (e.pre_record >= 0) {
            if ((err = hipEventRecord(c->sync_events[e.pre_record], s)) != hipSuccess) return err;
            if (gate) gate->ev_gen[e.pre_record].store(round + 1, std::memory_order_release);
        }
    }
    float *ws = c->ws_run[t];
    // sibling decomposition (Section 5.4, Table 3): odd chunks go to the tenant's second stream, released by `fork` (everything
    // this operator waited for is done) and gathered by `join` before the operator counts as finished
    hipStream_t s2 = s;
    if (with_events && e.fork >= 0) {
        s2 = c->tenants[t].sibling;
        if ((err = hipEventRecord(c->sync_events[e.fork], s)) != hipSuccess) return err;
        if ((err = hipStreamWaitEvent(s2, c->sync_events[e.fork], 0)) != hipSuccess) return err;
    }
    if (Trace *tr = c->trace) {
        for (size_t j = 0; j < e.chunks.size(); ++j) {
            const int phases = enqueue(e.chunks[j], s, true).phases;
            for (int ph = 1; ph <= phases; ++ph) {
                const size_t k = 2 * ((size_t)round * tr->per_round + tr->row_of[t][i][j] + (size_t)(ph - 1));
                const LaunchTimer lt = {tr->ev[k], tr->ev[k + 1]};
                launch_timer = &lt;
                enqueue(e.chunks[j], (j & 1) ? s2 : s, false, phases == 1 ? 0 : ph, ws);
                launch_timer = nullptr;
            }
        }
    } else if (c->sync_every_launch && !c->capturing) {
        // checking mode: every kernel is waited for and its status read before anything else is issued, so that a
        // failure is reported with the launch that caused it
        for (size_t j = 0; j < e.chunks.size(); ++j) {
            hipStream_t sj = (j & 1) ? s2 : s;
            const LaunchInfo li = enqueue(e.chunks[j], sj, false, 0, ws);
            if ((err = hipStreamSynchronize(sj)) != hipSuccess || (err = hipGetLastError()) != hipSuccess) {
                char buf[256];
                std::snprintf(buf, sizeof buf, "tenant %d op %d chunk %zu (%s, %d workgroups): %s", t, i, j, li.kernel, li.workgroups,
                              hipGetErrorString(err));
                c->launch_detail = buf;
                return err;
            }
        }
    } else {
        for (size_t j = 0; j < e.chunks.size(); ++j) enqueue(e.chunks[j], (j & 1) ? s2 : s, false, 0, ws);
    }
    if (s2 != s) {
        if ((err = hipEventRecord(c->sync_events[e.join], s2)) != hipSuccess) return err;
        if ((err = hipStreamWaitEvent(s, c->sync_events[e.join], 0)) != hipSuccess) return err;
    }
    if (with_events && e.record >= 0) {
        if ((err = hipEventRecord(c->sync_events[e.record], s)) != hipSuccess) return err;
        if (gate) gate->ev_gen[e.record].store(round + 1, std::memory_order_release);
    }
    return hipSuccess;
}

gacer_status ensure_plan_events(Ctx *c)
{
    const int NT = (int)c->tenants.size();
    while (c->sync_events.size() < c->n_sync_events) {
        hipEvent_t ev;
        HIPCHK(c, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        c->sync_events.push_back(ev);
    }
    while ((int)c->join_events.size() < NT + 1) {          // [NT] is the fork event
        hipEvent_t e;
        HIPCHK(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        c->join_events.push_back(e);
    }
    return GACER_OK;
}

gacer_status ensure_events(Ctx *c, int rounds)
{
    // the per-round timing events are made in blocks of 128 rounds, so that a caller who warms up with a few rounds
    // and then times many does not pay for event creation inside the timed call
    const int want = (rounds + 127) / 128 * 128;
    while ((int)c->t_start.size() < want) {
        hipEvent_t a, b;
        HIPCHK(c, hipEventCreate(&a));
        c->t_start.push_back(a);
        HIPCHK(c, hipEventCreate(&b));
        c->t_end.push_back(b);
    }
    return ensure_plan_events(c);
}

// Enqueues one round from the calling thread: fork from tenant 0's stream, every operator in issue order, join back.
gacer_status issue_round(Ctx *c, int mode, int round)
{
    const int NT = (int)c->tenants.size();
    hipStream_t s0 = c->tenants[0].stream;
    if (mode == GACER_MODE_SEQUENTIAL) {
        for (int t = 0; t < NT; ++t)
            for (int i = 0; i < (int)c->plain_exec[t].size(); ++i)
                ISSUE(c, issue_op(c, t, i, c->plain_exec[t][i], s0, false, round, nullptr));
        return GACER_OK;
    }
    hipEvent_t fork = c->join_events[NT];
    HIPCHK(c, hipEventRecord(fork, s0));
    for (int t = 1; t < NT; ++t)
        if (c->tenants[t].stream != s0) HIPCHK(c, hipStreamWaitEvent(c->tenants[t].stream, fork, 0));
    const bool plan = (mode == GACER_MODE_PLAN);
    const auto &order = plan ? c->plan_order : c->par_order;
    const auto &ex = plan ? c->plan_exec : c->plain_exec;
    for (const auto &to : order)
        ISSUE(c, issue_op(c, to.first, to.second, ex[to.first][to.second], c->tenants[to.first].stream, plan, round, nullptr));
    for (int t = 1; t < NT; ++t)
        if (c->tenants[t].stream != s0) {
            HIPCHK(c, hipEventRecord(c->join_events[t], c->tenants[t].stream));
            HIPCHK(c, hipStreamWaitEvent(s0, c->join_events[t], 0));
        }
    return GACER_OK;
}

// One host thread per tenant (Section 2.1: every tenant's DFG is wrapped into a processing thread that feeds its
// own stream).  The calling thread plays tenant 0 and owns the fork / join of every round.
struct ThreadedIssue {
    Ctx *c;
    int mode, rounds;
    IssueGate gate;
    std::mutex err_mu;
    std::string err;

    void fail_with(const char *what, hipError_t e)
    {
        std::lock_guard<std::mutex> g(err_mu);
        if (!gate.failed.exchange(1)) err = std::string(what) + " failed: " + hipGetErrorString(e);
    }
    bool issue_tenant(int t, int r)
    {
        const bool plan = (mode == GACER_MODE_PLAN);
        const auto &ex = plan ? c->plan_exec[t] : c->plain_exec[t];
        for (int i = 0; i < (int)ex.size(); ++i) {
            const hipError_t e = issue_op(c, t, i, ex[i], c->tenants[t].stream, plan, r, &gate);
            if (e != hipSuccess) { fail_with("enqueueing an operator", e); return false; }
        }
        return true;
    }
    void worker(int t)
    {
        if (hipSetDevice(c->device) != hipSuccess) { fail_with("hipSetDevice", hipGetLastError()); return; }
        const int NT = (int)c->tenants.size();
        for (int r = 0; r < rounds; ++r) {
            if (!gate.wait_gen(gate.fork_gen, r + 1)) return;
            hipError_t e = hipStreamWaitEvent(c->tenants[t].stream, c->join_events[NT], 0);
            if (e != hipSuccess) { fail_with("hipStreamWaitEvent(fork)", e); return; }
            if (!issue_tenant(t, r)) return;
            e = hipEventRecord(c->join_events[t], c->tenants[t].stream);
            if (e != hipSuccess) { fail_with("hipEventRecord(join)", e); return; }
            gate.join_gen[t].store(r + 1, std::memory_order_release);
        }
    }
#define TI_CHK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { fail_with(#call, e_); return false; } } while (0)
    bool lead()
    {
        const int NT = (int)c->tenants.size();
        hipStream_t s0 = c->tenants[0].stream;
        for (int r = 0; r < rounds; ++r) {
            TI_CHK(hipEventRecord(c->t_start[r], s0));
            TI_CHK(hipEventRecord(c->join_events[NT], s0));
            gate.fork_gen.store(r + 1, std::memory_order_release);
            if (!issue_tenant(0, r)) return false;
            for (int t = 1; t < NT; ++t) {
                if (!gate.wait_gen(gate.join_gen[t], r + 1)) return false;
                TI_CHK(hipStreamWaitEvent(s0, c->join_events[t], 0));
            }
            TI_CHK(hipEventRecord(c->t_end[r], s0));
        }
        return true;
    }
#undef TI_CHK
};

gacer_status run_threaded(Ctx *c, int mode, int rounds)
{
    const int NT = (int)c->tenants.size();
    ThreadedIssue ti;
    ti.c = c; ti.mode = mode; ti.rounds = rounds;
    const size_t ne = std::max<size_t>(1, c->sync_events.size());
    ti.gate.ev_gen.reset(new std::atomic<long>[ne]);
    ti.gate.join_gen.reset(new std::atomic<long>[NT]);
    for (size_t i = 0; i < ne; ++i) ti.gate.ev_gen[i].store(0);
    for (int t = 0; t < NT; ++t) ti.gate.join_gen[t].store(0);
    std::vector<std::thread> workers;
    for (int t = 1; t < NT; ++t) workers.emplace_back([&ti, t] { ti.worker(t); });
    const bool ok = ti.lead();
    if (!ok) ti.gate.failed.store(1);
    for (std::thread &w : workers) w.join();
    if (ti.gate.failed.load()) return fail(c, GACER_EHIP, "%s", ti.err.empty() ? "threaded issue failed" : ti.err.c_str());
    return GACER_OK;
}

bool distinct_streams(const Ctx *c)
{
    for (size_t a = 0; a < c->tenants.size(); ++a)
        for (size_t b = a + 1; b < c->tenants.size(); ++b)
            if (c->tenants[a].stream == c->tenants[b].stream) return false;
    return true;
}

// Enqueues `rounds` rounds with per-round timing events and waits for them.  c->ws_run and c->trace are set by the caller.
gacer_status run_rounds(Ctx *c, int mode, int rounds, bool allow_graph)
{
    hipStream_t s0 = c->tenants[0].stream;
    const auto host_t0 = std::chrono::steady_clock::now();
    const bool graph = allow_graph && c->graph_exec[mode] && !c->sync_every_launch;   // the checking mode issues every launch itself
    const bool threaded = c->issue_threads && mode != GACER_MODE_SEQUENTIAL && !graph && c->tenants.size() > 1 && distinct_streams(c);
    gacer_status st = GACER_OK;
    if (threaded) {
        st = run_threaded(c, mode, rounds);
    } else {
        for (int r = 0; r < rounds && st == GACER_OK; ++r) {
            HIPCHK(c, hipEventRecord(c->t_start[r], s0));
            if (graph) HIPCHK(c, hipGraphLaunch(c->graph_exec[mode], s0));
            else st = issue_round(c, mode, r);
            if (st == GACER_OK) HIPCHK(c, hipEventRecord(c->t_end[r], s0));
        }
    }
    if (st != GACER_OK) { (void)hipDeviceSynchronize(); return st; }
    c->last_issue_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - host_t0).count();
    c->last_issue_launches = 0;
    gacer_launch_count(static_cast<gacer_ctx *>(c), mode, &c->last_issue_launches);
    c->last_issue_launches *= rounds;
    HIPCHK(c, hipStreamSynchronize(s0));
    HIPCHK(c, hipGetLastError());
    return GACER_OK;
}

void use_tenant_workspaces(Ctx *c)
{
    c->ws_run.resize(c->tenants.size());
    for (size_t t = 0; t < c->tenants.size(); ++t) c->ws_run[t] = c->tenants[t].ws;
}

// True when three or more tenants wait on each other's events in a ring (tenant a waits on b, b on c, ..., back to a),
// judged on the tenant-level graph of the plan's edges.  Mutual pairs (a <-> b, the shape of a hub barrier) are not rings.
// Simple paths are enumerated depth first; a search that grows beyond its step budget answers "ring" (the safe side).
bool tenants_wait_in_a_ring(const Ctx *c)
{
    const int NT = (int)c->tenants.size();
    std::vector<std::vector<int>> waits_on(NT);
    for (const gacer_sync &e : c->syncs)
        if (std::find(waits_on[e.dst_tenant].begin(), waits_on[e.dst_tenant].end(), e.src_tenant) == waits_on[e.dst_tenant].end())
            waits_on[e.dst_tenant].push_back(e.src_tenant);
    long budget = 200000;
    std::vector<char> on_path(NT, 0);
    std::vector<std::pair<int, size_t>> stack;
    for (int root = 0; root < NT; ++root) {
        stack.assign(1, {root, 0});
        on_path.assign(NT, 0);
        on_path[root] = 1;
        while (!stack.empty()) {
            if (--budget < 0) return true;
            const int node = stack.back().first;
            if (stack.back().second == waits_on[node].size()) { on_path[node] = 0; stack.pop_back(); continue; }
            const int nxt = waits_on[node][stack.back().second++];
            if (nxt == root && stack.size() >= 3) return true;
            if (nxt > root && !on_path[nxt]) { on_path[nxt] = 1; stack.push_back({nxt, 0}); }   // rings are found from their lowest tenant
        }
    }
    return false;
}

}  // namespace

namespace gacer {
void drop_graphs(Ctx *c)
{
    for (int m = 0; m < 3; ++m)
        if (c->graph_exec[m]) { (void)hipGraphExecDestroy(c->graph_exec[m]); c->graph_exec[m] = nullptr; }
}
}  // namespace gacer

extern "C" {

gacer_status gacer_capture(gacer_ctx *c, int mode)
{
    if (!c) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "gacer_capture before gacer_load_tenants");
    if (mode < 0 || mode > 2) return fail(c, GACER_EINVAL, "bad mode");
    if (mode == GACER_MODE_PLAN) {
        // HIP runtimes before 7.2 crash in hipStreamEndCapture when three or more captured streams wait on each other
        // mutually.  Hub barriers only pair the hub with each member and capture fine.
        int rt = 0;
        if ((hipRuntimeGetVersion(&rt) != hipSuccess || rt < 70200000) && tenants_wait_in_a_ring(c))
            return fail(c, GACER_EPLAN, "this HIP runtime (%d) cannot capture a plan in which three or more tenants wait on each "
                                        "other in a ring; use hub barriers with one hub (gacer_plan_from_pointers) or run uncaptured", rt);
    }
    if (c->ws_missing) return fail(c, GACER_EHIP, "split-K workspace could not be allocated when the tenants were loaded");
    gacer_status st = ensure_events(c, 1);
    if (st != GACER_OK) return st;
    if (c->graph_exec[mode]) { (void)hipGraphExecDestroy(c->graph_exec[mode]); c->graph_exec[mode] = nullptr; }
    hipStream_t s0 = c->tenants[0].stream;
    for (Tenant &t : c->tenants) HIPCHK(c, hipStreamSynchronize(t.stream));
    use_tenant_workspaces(c);
    HIPCHK(c, hipStreamBeginCapture(s0, hipStreamCaptureModeRelaxed));
    c->capturing = true;
    st = issue_round(c, mode, 0);
    c->capturing = false;
    hipGraph_t graph = nullptr;
    const hipError_t e_end = hipStreamEndCapture(s0, &graph);
    if (st != GACER_OK || e_end != hipSuccess || !graph) {
        if (graph) (void)hipGraphDestroy(graph);
        (void)hipGetLastError();
        if (st == GACER_OK) return fail(c, GACER_EHIP, "stream capture failed: %s", hipGetErrorString(e_end));
        return st;
    }
    hipGraphExec_t exec = nullptr;
    const hipError_t e_inst = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e_inst != hipSuccess) return fail(c, GACER_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e_inst));
    c->graph_exec[mode] = exec;
    return GACER_OK;
}

gacer_status gacer_release_graphs(gacer_ctx *c)
{
    if (!c) return GACER_EINVAL;
    for (Tenant &t : c->tenants) (void)hipStreamSynchronize(t.stream);
    drop_graphs(c);
    return GACER_OK;
}

gacer_status gacer_set_issue_threads(gacer_ctx *c, int enable)
{
    if (!c) return GACER_EINVAL;
    c->issue_threads = enable != 0;
    return GACER_OK;
}

gacer_status gacer_set_fuse_affine(gacer_ctx *c, int enable)
{
    if (!c) return GACER_EINVAL;
    c->fuse_affine = enable != 0;
    if (!c->loaded) return GACER_OK;
    expand_plain(c);
    const std::vector<gacer_split> sp = c->splits;          // chunk lists stay alive in c->split_sizes while the plan is rebuilt
    const std::vector<std::vector<int>> keep = c->split_sizes;
    std::vector<gacer_split> again = sp;
    for (size_t k = 0; k < again.size(); ++k)
        if (again[k].sizes) again[k].sizes = keep[k].data();
    const std::vector<gacer_sync> sy = c->syncs;
    return install_plan(c, again, sy);
}

gacer_status gacer_set_sync_every_launch(gacer_ctx *c, int enable)
{
    if (!c) return GACER_EINVAL;
    c->sync_every_launch = enable != 0;
    return GACER_OK;
}

gacer_status gacer_run(gacer_ctx *c, int mode, int rounds, float *ms_per_round)
{
    if (!c) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "gacer_run before gacer_load_tenants");
    if (mode < 0 || mode > 2 || rounds < 1) return fail(c, GACER_EINVAL, "bad mode or rounds");
    if (c->ws_missing) return fail(c, GACER_EHIP, "split-K workspace could not be allocated when the tenants were loaded");
    gacer_status st = ensure_events(c, rounds);
    if (st != GACER_OK) return st;
    use_tenant_workspaces(c);
    st = run_rounds(c, mode, rounds, true);
    if (st != GACER_OK) return st;
    if (ms_per_round)
        for (int r = 0; r < rounds; ++r) HIPCHK(c, hipEventElapsedTime(&ms_per_round[r], c->t_start[r], c->t_end[r]));
    return GACER_OK;
}

gacer_status gacer_run_static(gacer_ctx *c, int mode, int rounds)
{
    if (!c) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "gacer_run_static before gacer_load_tenants");
    if (mode < 0 || mode > 2 || rounds < 1) return fail(c, GACER_EINVAL, "bad mode or rounds");
    const int NT = (int)c->tenants.size();
    // every tenant gets its own 256-byte aligned part of the static workspace (tenants run concurrently)
    size_t need = 0;
    for (const Tenant &t : c->tenants) need += (t.ws_floats * sizeof(float) + 255) / 256 * 256;
    if (need > (size_t)GACER_STATIC_SCRATCH_BYTES)
        return fail(c, GACER_ENOMEM, "the loaded tenants need %zu bytes of split-K workspace, the static workspace holds %zu; "
                                     "use gacer_run", need, (size_t)GACER_STATIC_SCRATCH_BYTES);
    if (!c->has_device) return fail(c, GACER_ESTATE, "the context was created without a GPU");
    if ((int)c->join_events.size() < NT + 1 || c->sync_events.size() < c->n_sync_events || (int)c->ws_run.size() != NT)
        return fail(c, GACER_ESTATE, "the plan's events do not exist (they are created by gacer_load_tenants / gacer_set_plan)");
    unsigned char *base = nullptr;
    const hipError_t e_sym = scratch_address(c->device, &base);
    if (e_sym != hipSuccess || !base) return fail(c, GACER_EHIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e_sym));
    size_t off = 0;
    for (int t = 0; t < NT; ++t) {
        c->ws_run[t] = c->tenants[t].ws_floats ? (float *)(base + off) : nullptr;
        off += (c->tenants[t].ws_floats * sizeof(float) + 255) / 256 * 256;
    }
    // one issuing thread, no captured graph (a capture has the allocated workspaces baked in), no timing events
    gacer_status st = GACER_OK;
    for (int r = 0; r < rounds && st == GACER_OK; ++r) st = issue_round(c, mode, r);
    const hipError_t e_sync = hipStreamSynchronize(c->tenants[0].stream);
    if (st != GACER_OK) return st;
    if (e_sync != hipSuccess) return fail(c, GACER_EHIP, "hipStreamSynchronize failed: %s", hipGetErrorString(e_sync));
    HIPCHK(c, hipGetLastError());
    return GACER_OK;
}

// Algorithmic work of one launch (sub-range only).
static void launch_work(const Launch &l, double *flops, double *bytes)
{
    *flops = 0;
    if (l.kind == LK_IGEMM) {
        const GemmArgs &g = l.g;
        const double esz = g.dtype == DT_BF16 ? 2.0 : 4.0;
        const double z = (double)g.zb * g.zh, M = g.m_hi - g.m_lo, N = g.n_hi - g.n_lo;
        *flops = 2.0 * M * N * g.K * z;
        const double rows_in = M / ((double)g.Ho * g.Wo) * g.H * g.W;      // input positions of the launched images
        *bytes = (rows_in * g.Cin + N * g.K + M * N * (g.res ? 2.0 : 1.0)) * esz * z + (g.bias ? N * 4.0 : 0.0);
        if (g.pre_scale) {                      // fused affine: one FMA per A element, its output written once, its two vectors read
            *flops += 2.0 * M * g.Cin;
            *bytes += M * g.Cin * esz + 8.0 * g.Cin;
        }
        return;
    }
    const StreamArgs &s = l.s;
    const double esz = s.dtype == DT_BF16 ? 2.0 : 4.0;
    double items, C;
    if (l.kind == LK_LAYERNORM || l.kind == LK_SOFTMAX) { items = (double)(s.n_hi - s.n_lo) * s.rows_per_item; C = s.C; }
    else { items = (double)(s.n_hi - s.n_lo); C = s.c_hi - s.c_lo; }
    double in_pos = (double)s.H * s.W, out_pos = (double)s.Ho * s.Wo;
    if (l.kind == LK_LAYERNORM || l.kind == LK_SOFTMAX) in_pos = out_pos = 1;
    if (l.kind == LK_GAVGPOOL) out_pos = 1;
    double b = items * C * (in_pos + out_pos) * esz;
    if (s.x2 && l.kind != LK_CONCAT) b += items * C * in_pos * esz;      // a concatenation reads C channels in total from its two inputs
    if (s.gate) b += items * C * esz;
    if (s.res) b += items * C * out_pos * esz;
    if (l.kind == LK_DWCONV) b += C * s.k * s.k * esz;
    *bytes = b;
}

gacer_status gacer_trace_run(gacer_ctx *c, int mode, int rounds, gacer_launch_stat *out, size_t cap, size_t *n_out)
{
    if (!c || !n_out) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "gacer_trace_run before gacer_load_tenants");
    if (mode < 0 || mode > 2 || rounds < 1) return fail(c, GACER_EINVAL, "bad mode or rounds");
    if (c->ws_missing) return fail(c, GACER_EHIP, "split-K workspace could not be allocated when the tenants were loaded");
    const int NT = (int)c->tenants.size();
    const bool plan = (mode == GACER_MODE_PLAN);
    const auto &ex = plan ? c->plan_exec : c->plain_exec;
    std::vector<std::pair<int, int>> order;
    if (mode == GACER_MODE_SEQUENTIAL) {
        for (int t = 0; t < NT; ++t)
            for (int i = 0; i < (int)c->tenants[t].ops.size(); ++i) order.push_back({t, i});
    } else order = plan ? c->plan_order : c->par_order;
    Trace tr;
    tr.row_of.resize(NT);
    for (int t = 0; t < NT; ++t) tr.row_of[t].resize(c->tenants[t].ops.size());
    size_t total = 0;                          // kernels per round (a split-K chunk is two kernels), rows in issue order
    for (const auto &to : order)
        for (const Launch &l : ex[to.first][to.second].chunks) {
            tr.row_of[to.first][to.second].push_back(total);
            total += (size_t)enqueue(l, nullptr, true).phases;
        }
    *n_out = total;
    if (cap == 0 || !out) return GACER_OK;
    if (cap < total) return fail(c, GACER_EINVAL, "trace buffer too small (%zu rows needed)", total);
    gacer_status st = ensure_events(c, rounds);
    if (st != GACER_OK) return st;
    tr.per_round = total;
    tr.ev.resize(2 * total * (size_t)rounds);
    for (hipEvent_t &e : tr.ev) HIPCHK(c, hipEventCreate(&e));
    for (const auto &to : order) {
        const OpExec &e = ex[to.first][to.second];
        for (size_t j = 0; j < e.chunks.size(); ++j) {
            const int phases = enqueue(e.chunks[j], nullptr, true).phases;
            for (int ph = 1; ph <= phases; ++ph) {
                gacer_launch_stat &row = out[tr.row_of[to.first][to.second][j] + (size_t)(ph - 1)];
                const LaunchInfo li = enqueue(e.chunks[j], nullptr, true, phases == 1 ? 0 : ph);
                row.tenant = to.first; row.op = to.second; row.chunk = (int)j;
                row.ms = row.start_ms = row.end_ms = 0.f;
                row.workgroups = li.workgroups;
                row.flops = row.bytes = 0.0;
                if (ph == 1) launch_work(e.chunks[j], &row.flops, &row.bytes);   // the operator's work is booked on its main kernel
                else {                          // the finishing pass moves the partial tiles in and the output out
                    const GemmArgs &g = e.chunks[j].g;
                    const double mn = (double)(g.m_hi - g.m_lo) * (g.n_hi - g.n_lo) * g.zb * g.zh;
                    row.bytes = mn * (4.0 * g.ksplit + (g.dtype == DT_BF16 ? 2.0 : 4.0) * (g.res ? 2.0 : 1.0));
                }
                std::snprintf(row.kernel, sizeof row.kernel, "%s", li.kernel);
            }
        }
    }
    use_tenant_workspaces(c);
    c->trace = &tr;
    st = run_rounds(c, mode, rounds, false);
    c->trace = nullptr;
    if (st == GACER_OK) {
        for (int r = 0; r < rounds && st == GACER_OK; ++r)
            for (size_t row = 0; row < total; ++row) {
                const size_t b = 2 * ((size_t)r * total + row);
                float ms = 0.f, t0 = 0.f, t1 = 0.f;
                if (hipEventElapsedTime(&ms, tr.ev[b], tr.ev[b + 1]) != hipSuccess ||
                    hipEventElapsedTime(&t0, c->t_start[r], tr.ev[b]) != hipSuccess ||
                    hipEventElapsedTime(&t1, c->t_start[r], tr.ev[b + 1]) != hipSuccess) {
                    st = fail(c, GACER_EHIP, "hipEventElapsedTime failed on a kernel's event pair: %s", hipGetErrorString(hipGetLastError()));
                    break;
                }
                out[row].ms += ms / (float)rounds;
                if (r == rounds - 1) { out[row].start_ms = t0; out[row].end_ms = t1; }
            }
    }
    for (hipEvent_t e : tr.ev) (void)hipEventDestroy(e);
    return st;
}

}  // extern "C"

namespace {
// true when a spin on `a` and a spin on `b`, released together, take about two kernel times instead of one
bool streams_serialise(hipStream_t a, hipStream_t b, hipEvent_t ev[3], bool *ok)
{
    const unsigned long long ticks = 10000;    // 100 us
    float worst = 0.f;
    for (int rep = 0; rep < 3; ++rep) {        // the best of three decides (a slow launch can fake a serialisation)
        *ok = hipEventRecord(ev[0], a) == hipSuccess && hipStreamWaitEvent(b, ev[0], 0) == hipSuccess;
        if (!*ok) return false;
        launch_spin(a, ticks);
        launch_spin(b, ticks);
        *ok = hipEventRecord(ev[1], a) == hipSuccess && hipEventRecord(ev[2], b) == hipSuccess &&
              hipStreamSynchronize(a) == hipSuccess && hipStreamSynchronize(b) == hipSuccess;
        if (!*ok) return false;
        float ta = 0.f, tb = 0.f;
        *ok = hipEventElapsedTime(&ta, ev[0], ev[1]) == hipSuccess && hipEventElapsedTime(&tb, ev[0], ev[2]) == hipSuccess;
        if (!*ok) return false;
        const float t = std::max(ta, tb);
        worst = rep == 0 ? t : std::min(worst, t);
    }
    return worst > 0.15f;                      // one kernel: about 0.10 ms; two in a row: about 0.20 ms
}
}  // namespace

extern "C" {

gacer_status gacer_probe_stream_queues(void *const *streams, int n, int *group)
{
    if (!streams || !group || n < 1 || n > 64) return GACER_EINVAL;
    hipEvent_t ev[3];
    for (hipEvent_t &e : ev)
        if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); return GACER_EHIP; }
    std::vector<int> rep;                      // first stream of every group found so far
    bool ok = true;
    for (int i = 0; i < n && ok; ++i) {
        group[i] = -1;
        for (int j = 0; j < i; ++j)
            if (streams[j] == streams[i]) { group[i] = group[j]; break; }
        for (size_t g = 0; g < rep.size() && group[i] < 0 && ok; ++g)
            if (streams_serialise((hipStream_t)streams[rep[g]], (hipStream_t)streams[i], ev, &ok)) group[i] = (int)g;
        if (group[i] < 0) { group[i] = (int)rep.size(); rep.push_back(i); }
    }
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    if (!ok) { (void)hipGetLastError(); return GACER_EHIP; }
    return GACER_OK;
}

gacer_status gacer_issue_stats(gacer_ctx *c, double *host_ms, int *launches)
{
    if (!c || !host_ms || !launches) return GACER_EINVAL;
    *host_ms = c->last_issue_ms;
    *launches = c->last_issue_launches;
    return GACER_OK;
}

gacer_status gacer_launch_count(gacer_ctx *c, int mode, int *count)
{
    if (!c || !count) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "no tenants loaded");
    const auto &ex = (mode == GACER_MODE_PLAN) ? c->plan_exec : c->plain_exec;
    int n = 0;
    for (const auto &t : ex)
        for (const OpExec &e : t) n += (int)e.chunks.size();
    *count = n;
    return GACER_OK;
}

// Lookup table of Section 4.1: isolated time per chunk, workgroups per chunk and CU share.
gacer_status gacer_profile(gacer_ctx *c, gacer_prof *out, size_t cap, size_t *n_out)
{
    if (!c || !n_out) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "gacer_profile before gacer_load_tenants");
    const int NT = (int)c->tenants.size();
    static const int factors[3] = {2, 4, 8};
    struct Variant { int t, op; gacer_axis axis; int f; };
    std::vector<Variant> vars;
    for (int t = 0; t < NT; ++t)
        for (int i = 0; i < (int)c->tenants[t].ops.size(); ++i) {
            vars.push_back({t, i, GACER_AXIS_NONE, 1});
            for (gacer_axis ax : {GACER_AXIS_BATCH, GACER_AXIS_COUT})
                for (int f : factors)
                    if (axis_legal(c->tenants[t].ops[i].kind, ax) && f <= axis_extent(c->tenants[t], i, ax)) vars.push_back({t, i, ax, f});
        }
    *n_out = vars.size() + 1;
    if (cap == 0 || !out) return GACER_OK;
    if (cap < vars.size() + 1) return fail(c, GACER_EINVAL, "profile buffer too small (%zu rows needed)", vars.size() + 1);
    gacer_status st = gacer_run(c, GACER_MODE_SEQUENTIAL, 1, nullptr);   // populate every tensor
    if (st != GACER_OK) return st;
    hipEvent_t e0, e1;
    HIPCHK(c, hipEventCreate(&e0));
    HIPCHK(c, hipEventCreate(&e1));
    const int reps = 5;
    size_t k = 0;
    for (const Variant &v : vars) {
        const Tenant &T = c->tenants[v.t];
        const int cout = (int)T.tensors[T.ops[v.op].out].c;
        std::vector<Launch> ch;
        for (int j = 0; j < v.f; ++j) {
            int lo, hi;
            if (v.axis == GACER_AXIS_BATCH) { chunk_range(T.batch, v.f, j, &lo, &hi); ch.push_back(make_launch(T, v.op, lo, hi, 0, cout)); }
            else if (v.axis == GACER_AXIS_COUT) { chunk_range(cout, v.f, j, &lo, &hi); ch.push_back(make_launch(T, v.op, 0, T.batch, lo, hi)); }
            else ch.push_back(make_launch(T, v.op, 0, T.batch, 0, cout));
        }
        const LaunchInfo li = enqueue(ch[0], T.stream, true);
        for (const Launch &l : ch) enqueue(l, T.stream, false, 0, T.ws);   // warm-up
        HIPCHK(c, hipEventRecord(e0, T.stream));
        for (int r = 0; r < reps; ++r)
            for (const Launch &l : ch) enqueue(l, T.stream, false, 0, T.ws);
        HIPCHK(c, hipEventRecord(e1, T.stream));
        HIPCHK(c, hipEventSynchronize(e1));
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, e0, e1));
        gacer_prof &p = out[k++];
        p.tenant = v.t; p.op = v.op; p.axis = v.axis; p.factor = v.f;
        p.ms = ms / (float)(reps * v.f);
        p.workgroups = li.workgroups;
        const float share = (float)li.workgroups / (float)(c->n_cu * std::max(1, li.wg_per_cu));
        p.cu_share = std::min(1.f, std::max(share, 1.f / (float)(c->n_cu * 8)));
        double flops = 0, bytes = 0;
        launch_work(ch[0], &flops, &bytes);                   // chunks of one decomposition differ by at most one element
        p.bw_share = p.ms > 0.f ? (float)std::min(1.0, bytes / (p.ms * 1e-3) / 8.0e12) : 0.f;
    }
    // T_SW: extra latency of one cross-stream event hop (record on one stream, wait on another),
    // measured as ping-pong between two tenant streams against the same launches on one stream.
    float t_sw = 0.f;
    if (NT >= 2 && c->tenants[0].stream != c->tenants[1].stream) {
        const Tenant &A = c->tenants[0], &B = c->tenants[1];
        Launch la = make_launch(A, 0, 0, 1, 0, 1), lb = make_launch(B, 0, 0, 1, 0, 1);   // tiny: one item, one channel
        hipEvent_t pa, pb;
        HIPCHK(c, hipEventCreateWithFlags(&pa, hipEventDisableTiming));
        HIPCHK(c, hipEventCreateWithFlags(&pb, hipEventDisableTiming));
        const int hops = 50;
        float serial = 0.f, pingpong = 0.f;
        HIPCHK(c, hipStreamSynchronize(B.stream));
        HIPCHK(c, hipEventRecord(e0, A.stream));
        for (int h = 0; h < hops; ++h) { enqueue(la, A.stream, false, 0, A.ws); enqueue(lb, A.stream, false, 0, B.ws); }
        HIPCHK(c, hipEventRecord(e1, A.stream));
        HIPCHK(c, hipEventSynchronize(e1));
        HIPCHK(c, hipEventElapsedTime(&serial, e0, e1));
        HIPCHK(c, hipEventRecord(e0, A.stream));
        for (int h = 0; h < hops; ++h) {
            enqueue(la, A.stream, false, 0, A.ws);
            HIPCHK(c, hipEventRecord(pa, A.stream));
            HIPCHK(c, hipStreamWaitEvent(B.stream, pa, 0));
            enqueue(lb, B.stream, false, 0, B.ws);
            HIPCHK(c, hipEventRecord(pb, B.stream));
            HIPCHK(c, hipStreamWaitEvent(A.stream, pb, 0));
        }
        HIPCHK(c, hipEventRecord(e1, A.stream));
        HIPCHK(c, hipEventSynchronize(e1));
        HIPCHK(c, hipEventElapsedTime(&pingpong, e0, e1));
        t_sw = std::max(0.f, (pingpong - serial) / (float)(2 * hops));
        (void)hipEventDestroy(pa);
        (void)hipEventDestroy(pb);
        st = gacer_run(c, GACER_MODE_SEQUENTIAL, 1, nullptr);   // restore tensors touched by the tiny launches
        if (st != GACER_OK) return st;
    }
    gacer_prof &p = out[k++];
    p.tenant = -1; p.op = -1; p.axis = GACER_AXIS_NONE; p.factor = 1; p.ms = t_sw; p.workgroups = 0; p.cu_share = 1.f; p.bw_share = 0.f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return GACER_OK;
}


// Rough cost of one tenant for stream placement: matrix-core time of its convolutions / GEMMs plus a fixed cost per
// operator launch.  Only the ranking matters.
static double tenant_weight(const gacer_tenant &t)
{
    double macs = 0;
    for (int i = 0; i < t.n_ops; ++i) {
        const gacer_op &op = t.ops[i];
        if (op.out < 0 || op.out >= t.n_tensors) continue;
        const gacer_tensor &y = t.tensors[op.out];
        const double outs = (double)y.n * y.c * y.h * y.w;
        switch (op.kind) {
        case GACER_CONV2D: case GACER_DWCONV2D: macs += outs * (op.cin / std::max(1, op.groups)) * op.kh * op.kw; break;
        case GACER_GEMM: case GACER_BGEMM_QK: case GACER_BGEMM_PV: macs += outs * op.cin; break;
        default: break;
        }
    }
    return 2.0 * macs / (t.dtype == GACER_BF16 ? 4.0e14 : 1.0e14) + 6e-6 * t.n_ops;
}

gacer_status gacer_place_streams(const gacer_tenant *tenants, int n, void *const *candidates, int n_cand, int *chosen, int *queue_of,
                                 int *n_queues, int *sibling)
{
    if (!tenants || !candidates || !chosen || n < 1 || n > 64 || n_cand < 1 || n_cand > 64) return GACER_EINVAL;
    std::vector<int> group(n_cand);
    const gacer_status st = gacer_probe_stream_queues(candidates, n_cand, group.data());
    if (st != GACER_OK) return st;
    const int nq = *std::max_element(group.begin(), group.end()) + 1;
    std::vector<std::vector<int>> by_queue(nq);
    for (int i = 0; i < n_cand; ++i) by_queue[group[i]].push_back(i);
    std::vector<size_t> next(nq, 0);
    std::vector<double> load(nq, 0.0), w(n);
    for (int t = 0; t < n; ++t) w[t] = tenant_weight(tenants[t]);
    std::vector<int> order(n);
    for (int t = 0; t < n; ++t) order[t] = t;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return w[a] > w[b]; });
    std::vector<int> own_queue(n, 0);
    for (int t : order) {                      // longest first, onto the least loaded queue
        int q = 0;
        for (int k = 1; k < nq; ++k)
            if (load[k] < load[q]) q = k;
        // a queue that has run out of candidate streams shares its first one (those tenants serialise anyway)
        chosen[t] = next[q] < by_queue[q].size() ? by_queue[q][next[q]++] : by_queue[q][0];
        own_queue[t] = q;
        if (queue_of) queue_of[t] = q;
        load[q] += w[t];
    }
    if (sibling) {
        // second stream per tenant: an unused candidate on the least loaded queue other than the tenant's own (a chunk on the
        // tenant's own queue could not overlap the tenant's other chunks); heaviest tenants choose first; -1 when none is left
        for (int t : order) {
            int q = -1;
            for (int k = 0; k < nq; ++k)
                if (k != own_queue[t] && next[k] < by_queue[k].size() && (q < 0 || load[k] < load[q])) q = k;
            sibling[t] = q < 0 ? -1 : by_queue[q][next[q]++];
            if (q >= 0) load[q] += 0.5 * w[t];
        }
    }
    if (n_queues) *n_queues = nq;
    return GACER_OK;
}

gacer_status gacer_refine(gacer_ctx *c, const gacer_prof *prof, size_t n, int trial_rounds, float min_gain, gacer_plan **out, float *ms_out)
{
    if (!c || !prof || !out) return GACER_EINVAL;
    if (!c->loaded) return fail(c, GACER_ESTATE, "gacer_refine before gacer_load_tenants");
    if (trial_rounds < 1 || !(min_gain >= 0.f)) return fail(c, GACER_EINVAL, "trial_rounds < 1 or negative min_gain");
    const int NT = (int)c->tenants.size();
    std::vector<std::vector<double>> T(NT);
    for (int t = 0; t < NT; ++t) T[t].assign(c->tenants[t].ops.size(), 0.0);
    for (size_t k = 0; k < n; ++k)
        if (prof[k].tenant >= 0 && prof[k].tenant < NT && prof[k].factor == 1 && prof[k].op >= 0 && prof[k].op < (int)T[prof[k].tenant].size())
            T[prof[k].tenant][prof[k].op] = prof[k].ms;
    // working copy of the installed plan; chunk lists live in `lists` (an inner vector's storage stays put when the outer one grows)
    std::vector<gacer_split> best_sp = c->splits;
    std::vector<std::vector<int>> lists;
    for (gacer_split &sp : best_sp)
        if (sp.sizes) { lists.emplace_back(sp.sizes, sp.sizes + sp.factor); sp.sizes = lists.back().data(); }
    const std::vector<gacer_sync> syncs = c->syncs;
    std::vector<float> buf((size_t)trial_rounds);
    gacer_status st = GACER_OK;
    auto measure = [&](const std::vector<gacer_split> &sp, float *ms) -> gacer_status {
        gacer_status r = install_plan(c, sp, syncs);
        if (r != GACER_OK) return r;
        if ((r = gacer_run(c, GACER_MODE_PLAN, 3, nullptr)) != GACER_OK) return r;
        if ((r = gacer_run(c, GACER_MODE_PLAN, trial_rounds, buf.data())) != GACER_OK) return r;
        std::vector<float> v = buf;
        std::sort(v.begin(), v.end());
        *ms = v[v.size() / 2];
        return GACER_OK;
    };
    float best = 0.f;
    if ((st = measure(best_sp, &best)) != GACER_OK) return st;
    std::vector<int> order(NT);
    std::vector<double> tot(NT, 0.0);
    for (int t = 0; t < NT; ++t) { order[t] = t; for (double v : T[t]) tot[t] += v; }
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return tot[a] > tot[b]; });
    for (int t : order) {
        const Tenant &Tn = c->tenants[t];
        std::vector<double> sorted = T[t];
        std::sort(sorted.begin(), sorted.end());
        const double thr = sorted.empty() ? 0.0 : sorted[(size_t)(sorted.size() * 0.75)];
        auto taken = [&](int op) {
            for (const gacer_split &s : best_sp)
                if (s.tenant == t && s.op == op) return true;
            return false;
        };
        struct Option { gacer_axis axis; int factor; bool uneven; };
        const Option options[4] = {{GACER_AXIS_BATCH, 2, false}, {GACER_AXIS_BATCH, 4, false}, {GACER_AXIS_COUT, 2, false}, {GACER_AXIS_BATCH, 2, true}};
        for (const Option &o : options) {
            if (o.uneven && Tn.batch < 4) continue;
            std::vector<gacer_split> trial = best_sp;
            size_t added = 0;
            for (int i = 0; i < (int)Tn.ops.size(); ++i) {
                if (T[t][i] < thr || taken(i) || !axis_legal(Tn.ops[i].kind, o.axis) || o.factor > axis_extent(Tn, i, o.axis)) continue;
                gacer_split sp = {t, i, o.axis, o.factor, nullptr};
                if (o.uneven) {                  // a chunk list: three quarters, then one quarter (Section 4.2: a chunk sized to a gap)
                    lists.push_back({Tn.batch - Tn.batch / 4, Tn.batch / 4});
                    sp.sizes = lists.back().data();
                }
                trial.push_back(sp);
                ++added;
            }
            if (!added) continue;
            float ms = 0.f;
            if ((st = measure(trial, &ms)) != GACER_OK) return st;
            if (ms < best * (1.f - min_gain)) { best = ms; best_sp.swap(trial); break; }
        }
    }
    if ((st = install_plan(c, best_sp, syncs)) != GACER_OK) return st;
    gacer_plan *pl = make_plan(best_sp, syncs);
    if (!pl) return fail(c, GACER_ENOMEM, "out of memory building the plan");
    *out = pl;
    if (ms_out) *ms_out = best;
    return GACER_OK;
}

}  // extern "C"
