// Host-side regulation model and granularity-aware search (Sections 4.1-4.4).  CPU only.
//
//   table    : the lookup table of Section 4.1, one row per operator and profiled decomposition: time T of a chunk,
//              its share W of the compute-unit pool (S_GPU = 1) and its share Wb of the memory-bandwidth pool.  A row
//              of factor f describes a chunk of extent/f elements; chunk sizes in between are read off the table by
//              linear interpolation in the size.
//   model    : streams issue their chunks in order; a chunk starts when its stream predecessor is done, its cluster is
//              open and its shares fit into what is left of both pools, otherwise it waits for the next completion
//              (Eq. 1).  Pointers cut every tenant into segments; same-index segments form a cluster that starts when
//              the previous cluster has drained, after a wait T_SW (Eq. 6, Eq. 7).
//   residue  : R = integral of the unused share of the pool(s) over the deployment + |P| * S_GPU * T_SW   (Eq. 8; the
//              bandwidth pool is the extension named in Section 4.4, claim (2), and counts only when the table has Wb)
//   search   : Algorithm 1 -- per pointer count, coordinate descent over pointer positions one tenant at a time --
//              alternated with the spatial regulation of Section 4.2: find the largest residue, take the largest
//              operator that follows it inside the cluster, cut off a chunk sized to that residue (list_B = [b, rest]).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include "ctx.h"

using namespace gacer;

namespace {

struct Cost { double T = 0, W = 0, Wb = 0; };

// What the table knows about one operator: the whole operator and, per axis, samples (chunk size -> cost).
struct OpCosts {
    Cost whole;
    bool have_whole = false;
    int extent[3] = {1, 1, 1};                       // elements of the axis (batch, output channels)
    struct Sample { double size; Cost c; int factor; };
    std::vector<Sample> samples[3];                  // ascending size, per axis (1 batch, 2 cout); without the whole operator
    bool axis_ok[3] = {false, false, false};         // the operator may be decomposed on this axis
};

struct Model {
    std::vector<std::vector<OpCosts>> ops;           // [tenant][op]
    double t_sw = 0;
    bool two_pools = false;
    int NT = 0;
};

// mask + list_B of one operator: untouched (one chunk), f even chunks, or explicit sizes
struct Decomp {
    int axis = 0;
    int even = 1;
    std::vector<int> sizes;
    bool whole() const { return even == 1 && sizes.empty(); }
};
typedef std::vector<std::vector<Decomp>> Mask;       // [tenant][op]
typedef std::vector<std::vector<int>> Pointers;      // [tenant][j], sorted, value p = cut after op p (1-based)

// cost of a chunk of `size` elements of `axis` (exact sample, else interpolation between the neighbouring samples; below
// the smallest sample a line through the origin); shares are capped at their pools
Cost chunk_cost(const OpCosts &o, int axis, int size)
{
    const double s = (double)size;
    const std::vector<OpCosts::Sample> &v = o.samples[axis];
    const double E = (double)o.extent[axis];
    if (std::fabs(E - s) < 1e-12) return o.whole;
    const OpCosts::Sample *lo = nullptr, *hi = nullptr;
    for (const OpCosts::Sample &p : v) {
        if (std::fabs(p.size - s) < 1e-12) return p.c;
        if (p.size < s) lo = &p;
        else if (!hi) hi = &p;
    }
    const double x1 = hi ? hi->size : E;
    const Cost &c1 = hi ? hi->c : o.whole;
    Cost r;
    if (lo) {
        const double a = (s - lo->size) / (x1 - lo->size);
        r.T = lo->c.T + a * (c1.T - lo->c.T);
        r.W = lo->c.W + a * (c1.W - lo->c.W);
        r.Wb = lo->c.Wb + a * (c1.Wb - lo->c.Wb);
    } else {
        const double a = s / x1;
        r.T = a * c1.T; r.W = a * c1.W; r.Wb = a * c1.Wb;
    }
    r.W = std::min(r.W, 1.0);
    r.Wb = std::min(r.Wb, 1.0);
    return r;
}

const Cost *even_row(const OpCosts &o, int axis, int f)
{
    for (const OpCosts::Sample &p : o.samples[axis])
        if (p.factor == f) return &p.c;
    return nullptr;
}

// ---- deployment sequence ------------------------------------------------------------------------------------------
struct Piece { int op, chunk; Cost c; };
struct Span { double t0, t1, used, used_b; int cluster; int n_running, n_pending; };

struct Deployment {
    std::vector<Span> spans;
    std::vector<std::vector<double>> first_start;    // [tenant][op]: start of the operator's first chunk
    double end = 0;
};

void chunks_of(const Model &m, const Mask &mask, int t, int i, std::vector<Piece> &out)
{
    const OpCosts &o = m.ops[t][i];
    const Decomp &d = mask[t][i];
    if (d.whole()) { out.push_back({i, 0, o.whole}); return; }
    if (d.sizes.empty()) {                               // even chunks: the table's own row
        const Cost *row = even_row(o, d.axis, d.even);
        for (int j = 0; j < d.even; ++j) out.push_back({i, j, row ? *row : chunk_cost(o, d.axis, o.extent[d.axis] / d.even)});
        return;
    }
    for (size_t j = 0; j < d.sizes.size(); ++j) out.push_back({i, (int)j, chunk_cost(o, d.axis, d.sizes[j])});
}

void deploy(const Model &m, const Mask &mask, const Pointers &P, Deployment &out)
{
    const int NT = m.NT;
    const int n_ptr = P.empty() ? 0 : (int)P[0].size();
    out.spans.clear();
    out.first_start.assign(NT, {});
    for (int t = 0; t < NT; ++t) out.first_start[t].assign(m.ops[t].size(), 0.0);
    std::vector<std::vector<Piece>> queue(NT);
    std::vector<size_t> head(NT);
    std::vector<double> done_at(NT), w(NT), wb(NT);
    std::vector<char> busy(NT);
    double now = 0;
    for (int k = 0; k <= n_ptr; ++k) {
        if (k > 0) now += m.t_sw;
        for (int t = 0; t < NT; ++t) {
            queue[t].clear();
            head[t] = 0;
            busy[t] = 0;
            const int lo = k == 0 ? 0 : P[t][k - 1], hi = k == n_ptr ? (int)m.ops[t].size() : P[t][k];
            for (int i = lo; i < hi; ++i) chunks_of(m, mask, t, i, queue[t]);
        }
        for (;;) {
            double used = 0, used_b = 0;
            int running = 0;
            for (int t = 0; t < NT; ++t)
                if (busy[t]) { used += w[t]; used_b += wb[t]; ++running; }
            for (int t = 0; t < NT; ++t) {                 // lower tenant index is served first
                if (busy[t] || head[t] >= queue[t].size()) continue;
                const Piece &p = queue[t][head[t]];
                const bool fits = used + p.c.W <= 1.0 + 1e-12 && used_b + p.c.Wb <= 1.0 + 1e-12;
                if (!fits && running > 0) continue;
                busy[t] = 1; done_at[t] = now + p.c.T; w[t] = p.c.W; wb[t] = p.c.Wb;
                if (p.chunk == 0) out.first_start[t][p.op] = now;
                used += p.c.W; used_b += p.c.Wb; ++running;
                ++head[t];
            }
            if (!running) break;
            double t1 = 1e300;
            int pending = 0;
            for (int t = 0; t < NT; ++t) {
                if (busy[t]) t1 = std::min(t1, done_at[t]);
                if (busy[t] || head[t] < queue[t].size()) ++pending;
            }
            out.spans.push_back({now, t1, used, used_b, k, running, pending});
            now = t1;
            for (int t = 0; t < NT; ++t)
                if (busy[t] && done_at[t] <= t1) busy[t] = 0;
        }
    }
    out.end = now;
}

double residue_of(const Model &m, const Deployment &d, int n_ptr)
{
    double R = 0;
    for (const Span &s : d.spans) {
        R += (1.0 - s.used) * (s.t1 - s.t0);
        if (m.two_pools) R += (1.0 - s.used_b) * (s.t1 - s.t0);
    }
    return R + n_ptr * 1.0 * m.t_sw;
}

double score(const Model &m, const Mask &mask, const Pointers &P)
{
    Deployment d;
    deploy(m, mask, P, d);
    return residue_of(m, d, P.empty() ? 0 : (int)P[0].size());
}

// ---- spatial regulation (Section 4.2, "Overall Spatial Regulation") -----------------------------------------------
// largest chunk (whole elements, smaller than the operator) whose shares fit the free shares; 0 if none
int chunk_matching(const OpCosts &o, int axis, double free_cu, double free_bw)
{
    int best = 0;
    for (int b = 1; b < o.extent[axis]; ++b) {
        const Cost c = chunk_cost(o, axis, b);
        if (c.W <= free_cu + 1e-12 && c.Wb <= free_bw + 1e-12) best = b;
    }
    return best;
}

void regulate_spatially(const Model &m, Mask &mask, const Pointers &P, int max_moves = 8)
{
    const int NT = m.NT;
    const int n_ptr = P.empty() ? 0 : (int)P[0].size();
    std::vector<std::vector<char>> given_up(NT);
    for (int t = 0; t < NT; ++t) given_up[t].assign(m.ops[t].size(), 0);
    for (int move = 0; move < max_moves; ++move) {
        Deployment d;
        deploy(m, mask, P, d);
        const double R0 = residue_of(m, d, n_ptr);
        // 1. the largest residue; the tail of a cluster (one tenant left with work) does not count; earliest on ties
        int at = -1;
        double largest = -1;
        for (int a = 0; a < (int)d.spans.size(); ++a) {
            const Span &s = d.spans[a];
            if (s.n_pending == 1) continue;
            const double area = (1.0 - s.used) * (s.t1 - s.t0);
            if (area > largest) { largest = area; at = a; }
        }
        if (at < 0) return;
        const Span &gap = d.spans[at];
        // 2. the largest operator that follows it in the same cluster and is still whole
        int bt = -1, bo = -1;
        double bsize = -1;
        for (int t = 0; t < NT; ++t) {
            const int lo = gap.cluster == 0 ? 0 : P[t][gap.cluster - 1];
            const int hi = gap.cluster == n_ptr ? (int)m.ops[t].size() : P[t][gap.cluster];
            for (int i = lo; i < hi; ++i) {
                const OpCosts &o = m.ops[t][i];
                if (given_up[t][i] || !mask[t][i].whole() || !(o.axis_ok[1] || o.axis_ok[2])) continue;
                if (d.first_start[t][i] < gap.t0 + 1e-12) continue;
                const double size = o.whole.W * o.whole.T;
                if (size > bsize) { bsize = size; bt = t; bo = i; }
            }
        }
        if (bt < 0) return;
        // 3. a chunk that matches the residue, on the axis whose two chunks take the least time
        const OpCosts &o = m.ops[bt][bo];
        int axis = 0, b = 0;
        double t_best = 1e300;
        for (int ax = 1; ax <= 2; ++ax) {
            if (!o.axis_ok[ax]) continue;
            const int fit = chunk_matching(o, ax, 1.0 - gap.used, m.two_pools ? 1.0 - gap.used_b : 1.0);
            if (fit < 1) continue;
            const double t2 = chunk_cost(o, ax, fit).T + chunk_cost(o, ax, o.extent[ax] - fit).T;
            if (t2 < t_best) { t_best = t2; axis = ax; b = fit; }
        }
        if (!axis) { given_up[bt][bo] = 1; continue; }
        // 4. keep it if the residue drops
        mask[bt][bo].axis = axis;
        mask[bt][bo].sizes = {b, o.extent[axis] - b};
        if (score(m, mask, P) < R0) continue;
        mask[bt][bo] = Decomp();
        given_up[bt][bo] = 1;
    }
}

// ---- temporal regulation: the inner loops of Algorithm 1 at a fixed pointer count --------------------------------
void descend_pointers(const Model &m, const Mask &mask, Pointers &P, int rounds)
{
    for (int r = 0; r < rounds; ++r) {
        bool moved = false;
        for (int t = 0; t < m.NT; ++t)
            for (size_t j = 0; j < P[t].size(); ++j) {
                const int lo = j > 0 ? P[t][j - 1] : 0;
                const int hi = j + 1 < P[t].size() ? P[t][j + 1] : (int)m.ops[t].size();
                const int was = P[t][j];
                int best_p = was;
                double best_R = 0;
                for (int p = lo; p <= hi; ++p) {
                    P[t][j] = p;
                    const double R = score(m, mask, P);
                    if (p == lo || R < best_R) { best_R = R; best_p = p; }      // earliest position on ties
                }
                P[t][j] = best_p;
                moved = moved || best_p != was;
            }
        if (!moved) break;
    }
}

// a new pointer starts in the middle of the tenant's longest segment (the earliest such segment)
int new_pointer_position(int n_ops, const std::vector<int> &P)
{
    int from = 0, longest = -1, where = 0;
    for (size_t j = 0; j <= P.size(); ++j) {
        const int to = j < P.size() ? P[j] : n_ops;
        if (to - from > longest) { longest = to - from; where = from + (to - from) / 2; }
        from = to;
    }
    return where;
}

// ---- table -> model ------------------------------------------------------------------------------------------------
gacer_status build_model(Ctx *c, const gacer_prof *prof, size_t n, Model &m)
{
    m.NT = (int)c->tenants.size();
    m.ops.resize(m.NT);
    for (int t = 0; t < m.NT; ++t) {
        m.ops[t].assign(c->tenants[t].ops.size(), OpCosts());
        for (size_t i = 0; i < m.ops[t].size(); ++i) {
            m.ops[t][i].extent[1] = axis_extent(c->tenants[t], (int)i, GACER_AXIS_BATCH);
            m.ops[t][i].extent[2] = axis_extent(c->tenants[t], (int)i, GACER_AXIS_COUT);
        }
    }
    for (size_t k = 0; k < n; ++k) {
        const gacer_prof &p = prof[k];
        if (p.tenant == -1) { m.t_sw = p.ms; continue; }
        if (p.tenant < 0 || p.tenant >= m.NT || p.op < 0 || p.op >= (int)m.ops[p.tenant].size() || (int)p.axis < 0 || (int)p.axis > 2 ||
            (p.factor != 1 && p.factor != 2 && p.factor != 4 && p.factor != 8) || (p.factor > 1) != (p.axis != GACER_AXIS_NONE)) {
            c->err = "profile table row names a missing operator or an illegal (axis, factor)";
            return GACER_EINVAL;
        }
        OpCosts &o = m.ops[p.tenant][p.op];
        Cost cost;
        cost.T = p.ms; cost.W = p.cu_share; cost.Wb = p.bw_share;
        if (cost.Wb > 0) m.two_pools = true;
        if (p.factor == 1) { o.whole = cost; o.have_whole = true; continue; }
        const int ax = (int)p.axis;
        o.axis_ok[ax] = true;
        o.samples[ax].push_back({(double)o.extent[ax] / (double)p.factor, cost, p.factor});
    }
    for (int t = 0; t < m.NT; ++t)
        for (OpCosts &o : m.ops[t]) {
            if (!o.have_whole) {
                c->err = "profile table lacks the unsplit row of an operator";
                return GACER_EINVAL;
            }
            for (int ax = 1; ax <= 2; ++ax)
                std::sort(o.samples[ax].begin(), o.samples[ax].end(), [](const OpCosts::Sample &a, const OpCosts::Sample &b) { return a.size < b.size; });
        }
    return GACER_OK;
}

gacer_plan *to_plan(Ctx *c, const Mask &mask, const Pointers &P)
{
    const int NT = (int)c->tenants.size();
    const int n_ptr = P.empty() ? 0 : (int)P[0].size();
    std::vector<int> flat;
    for (int t = 0; t < NT; ++t) flat.insert(flat.end(), P[t].begin(), P[t].end());
    gacer_plan *edges = nullptr;
    if (gacer_plan_from_pointers(static_cast<gacer_ctx *>(c), flat.empty() ? nullptr : flat.data(), n_ptr, &edges) != GACER_OK) return nullptr;
    std::vector<gacer_split> list;
    for (int t = 0; t < NT; ++t)
        for (int i = 0; i < (int)mask[t].size(); ++i) {
            const Decomp &d = mask[t][i];
            if (d.whole()) continue;
            if (d.sizes.empty()) list.push_back({t, i, (gacer_axis)d.axis, d.even, nullptr});
            else list.push_back({t, i, (gacer_axis)d.axis, (int)d.sizes.size(), d.sizes.data()});
        }
    gacer_plan *pl = make_plan(list, std::vector<gacer_sync>(edges->sync, edges->sync + edges->n_sync));
    gacer_plan_free(edges);
    return pl;
}

}  // namespace

extern "C" {

gacer_status gacer_search(gacer_ctx *c, const gacer_prof *prof, size_t n, int max_rounds, gacer_plan **out, int *pointers_out,
                          int *n_ptr_out, double *residue_out)
{
    if (!c || !prof || !out) return GACER_EINVAL;
    if (!c->loaded) { c->err = "gacer_search before gacer_load_tenants"; return GACER_ESTATE; }
    if (max_rounds < 1) { c->err = "max_rounds < 1"; return GACER_EINVAL; }
    Model m;
    gacer_status st = build_model(c, prof, n, m);
    if (st != GACER_OK) return st;
    const int NT = m.NT;
    Mask mask(NT);
    for (int t = 0; t < NT; ++t) mask[t].assign(m.ops[t].size(), Decomp());
    Pointers P(NT);
    // level 0: no pointers; every level ends with one spatial step; a level that scores worse than the one before ends the search
    regulate_spatially(m, mask, P);
    Mask best_mask = mask;
    Pointers best_P = P;
    double best_R = score(m, mask, P);
    size_t shortest = m.ops[0].size();
    for (int t = 1; t < NT; ++t) shortest = std::min(shortest, m.ops[t].size());
    for (int level = 1; level <= 8 && level <= (int)shortest; ++level) {
        for (int t = 0; t < NT; ++t) {
            P[t].push_back(new_pointer_position((int)m.ops[t].size(), P[t]));
            std::sort(P[t].begin(), P[t].end());
        }
        descend_pointers(m, mask, P, max_rounds);
        regulate_spatially(m, mask, P);
        const double R = score(m, mask, P);
        if (R > best_R) break;
        best_R = R; best_mask = mask; best_P = P;
    }
    gacer_plan *pl = to_plan(c, best_mask, best_P);
    if (!pl) { c->err = "out of memory building the plan"; return GACER_ENOMEM; }
    const int n_ptr = (int)best_P[0].size();
    if (pointers_out)
        for (int t = 0; t < NT; ++t)
            for (int j = 0; j < n_ptr; ++j) pointers_out[t * n_ptr + j] = best_P[t][j];
    if (n_ptr_out) *n_ptr_out = n_ptr;
    if (residue_out) *residue_out = best_R;
    *out = pl;
    return GACER_OK;
}

gacer_status gacer_model_residue(gacer_ctx *c, const gacer_prof *prof, size_t n, const gacer_split *split, int n_split, const int *Pm,
                                 int n_ptr, double *residue_out, double *makespan_out)
{
    if (!c || !prof || !residue_out) return GACER_EINVAL;
    if (!c->loaded) { c->err = "gacer_model_residue before gacer_load_tenants"; return GACER_ESTATE; }
    Model m;
    gacer_status st = build_model(c, prof, n, m);
    if (st != GACER_OK) return st;
    const int NT = m.NT;
    Mask mask(NT);
    for (int t = 0; t < NT; ++t) mask[t].assign(m.ops[t].size(), Decomp());
    for (int k = 0; k < n_split; ++k) {
        const gacer_split &s = split[k];
        if (s.tenant < 0 || s.tenant >= NT || s.op < 0 || s.op >= (int)m.ops[s.tenant].size() || (int)s.axis < 0 || (int)s.axis > 2) {
            c->err = "split names a missing operator or axis";
            return GACER_EPLAN;
        }
        if (s.factor <= 1 && !s.sizes) continue;
        const OpCosts &o = m.ops[s.tenant][s.op];
        Decomp &d = mask[s.tenant][s.op];
        if ((int)s.axis == 0) { c->err = "a decomposed operator needs an axis"; return GACER_EPLAN; }
        d.axis = (int)s.axis;
        if (s.sizes) {
            if (s.factor < 1 || s.factor > 8) { c->err = "a chunk list holds 1..8 sizes"; return GACER_EPLAN; }
            long sum = 0;
            for (int j = 0; j < s.factor; ++j) { if (s.sizes[j] < 1) { c->err = "chunk sizes must be positive"; return GACER_EPLAN; } sum += s.sizes[j]; }
            if (sum != o.extent[d.axis]) { c->err = "chunk sizes must sum to the axis extent"; return GACER_EPLAN; }
            d.sizes.assign(s.sizes, s.sizes + s.factor);
        } else {
            if ((s.factor != 2 && s.factor != 4 && s.factor != 8) || !even_row(o, d.axis, s.factor)) {
                c->err = "split not covered by the profile table";
                return GACER_EPLAN;
            }
            d.even = s.factor;
        }
    }
    Pointers P(NT);
    for (int t = 0; t < NT; ++t)
        for (int j = 0; j < n_ptr; ++j) {
            const int p = Pm[t * n_ptr + j];
            if (p < 0 || p > (int)m.ops[t].size() || (j > 0 && p < Pm[t * n_ptr + j - 1])) { c->err = "pointers must be sorted and in range"; return GACER_EPLAN; }
            P[t].push_back(p);
        }
    Deployment d;
    deploy(m, mask, P, d);
    *residue_out = residue_of(m, d, n_ptr);
    if (makespan_out) *makespan_out = d.end;
    return GACER_OK;
}

}  // extern "C"
