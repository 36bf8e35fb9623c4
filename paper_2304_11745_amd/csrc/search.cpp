// Host-side regulation model and granularity-aware search (Sections 4.1-4.4).  CPU only.
//
//   model    : every launch holds a share W of the compute-unit pool (S_GPU = 1) for its profiled time
//              T; streams issue in order; a launch that does not fit waits for the next completion
//              (Eq. 1).  Pointers cut every tenant into segments; same-index segments form a cluster
//              that starts when the previous cluster has drained, after a wait T_SW (Eq. 6, Eq. 7).
//   residue  : R = integral of (S_GPU - sum W) over the deployment + |P| * S_GPU * T_SW   (Eq. 8)
//   search   : Algorithm 1 -- per pointer count, coordinate descent over pointer positions one tenant
//              at a time -- alternated with the greedy spatial step of Section 4.2 (decompose the
//              largest operator that follows the largest residue); stops when one more pointer per
//              tenant no longer lowers R.
#include <algorithm>
#include <cstring>
#include <map>
#include <new>
#include <set>
#include "ctx.h"

using namespace gacer;

namespace {

struct Cell { double T = 0, W = 0; bool have = false; };
struct OpTable { Cell c[3][4]; };                 // [axis][log2 factor]
struct Split { int axis = 0, f = 1; };

struct Model {
    std::vector<std::vector<OpTable>> tab;        // [tenant][op]
    std::vector<int> n_ops;
    double t_sw = 0;
    int NT = 0;
};

int lg(int f) { return f == 1 ? 0 : f == 2 ? 1 : f == 4 ? 2 : 3; }

const Cell &cell(const Model &m, int t, int i, const Split &s) { return m.tab[t][i].c[s.f > 1 ? s.axis : 0][lg(s.f)]; }

struct Interval { double t0, t1, used; int cluster; unsigned long long running; };

struct Sim {
    std::vector<Interval> iv;
    std::vector<std::vector<double>> start;       // start time of the first chunk of [tenant][op]
    double total = 0;
};

typedef std::vector<std::vector<Split>> Splits;   // [tenant][op]
typedef std::vector<std::vector<int>> Pointers;   // [tenant][j], sorted, value p = cut after op p (1-based)

void simulate(const Model &m, const Splits &sp, const Pointers &P, Sim &out)
{
    const int NT = m.NT;
    const int n_ptr = P.empty() ? 0 : (int)P[0].size();
    out.iv.clear();
    out.start.assign(NT, {});
    for (int t = 0; t < NT; ++t) out.start[t].assign(m.n_ops[t], 0.0);
    double now = 0;
    for (int k = 0; k <= n_ptr; ++k) {
        if (k > 0) now += m.t_sw;
        // per tenant: operator range of this cluster and the position inside it
        std::vector<int> op(NT), op_end(NT), chunk(NT, 0);
        std::vector<double> finish(NT, -1.0), share(NT, 0.0);
        std::vector<char> busy(NT, 0);
        for (int t = 0; t < NT; ++t) {
            op[t] = k == 0 ? 0 : P[t][k - 1];
            op_end[t] = k == n_ptr ? m.n_ops[t] : P[t][k];
        }
        for (;;) {
            double used = 0;
            int n_busy = 0;
            for (int t = 0; t < NT; ++t)
                if (busy[t]) { used += share[t]; ++n_busy; }
            for (int t = 0; t < NT; ++t) {
                if (busy[t] || op[t] >= op_end[t]) continue;
                const Cell &c = cell(m, t, op[t], sp[t][op[t]]);
                if (used + c.W <= 1.0 + 1e-12 || n_busy == 0) {
                    busy[t] = 1; finish[t] = now + c.T; share[t] = c.W;
                    if (chunk[t] == 0) out.start[t][op[t]] = now;
                    used += c.W; ++n_busy;
                    if (++chunk[t] >= sp[t][op[t]].f) { chunk[t] = 0; ++op[t]; }
                }
            }
            if (n_busy == 0) break;
            double t1 = 1e300;
            unsigned long long mask = 0;
            for (int t = 0; t < NT; ++t)
                if (busy[t]) { t1 = std::min(t1, finish[t]); mask |= 1ull << t; }
            out.iv.push_back({now, t1, used, k, mask});
            now = t1;
            for (int t = 0; t < NT; ++t)
                if (busy[t] && finish[t] <= t1) busy[t] = 0;
        }
    }
    out.total = now;
}

double residue(const Model &m, const Sim &s, int n_ptr)
{
    double R = 0;
    for (const Interval &i : s.iv) R += (1.0 - i.used) * (i.t1 - i.t0);
    return R + n_ptr * 1.0 * m.t_sw;
}

double evaluate(const Model &m, const Splits &sp, const Pointers &P)
{
    Sim s;
    simulate(m, sp, P, s);
    return residue(m, s, P.empty() ? 0 : (int)P[0].size());
}

int popcount64(unsigned long long v) { int n = 0; while (v) { v &= v - 1; ++n; } return n; }

// Greedy spatial regulation (Section 4.2, "Overall Spatial Regulation").
void spatial_step(const Model &m, Splits &sp, const Pointers &P, int max_moves = 8)
{
    const int NT = m.NT;
    const int n_ptr = P.empty() ? 0 : (int)P[0].size();
    std::set<std::pair<int, int>> banned;
    for (int move = 0; move < max_moves; ++move) {
        Sim s;
        simulate(m, sp, P, s);
        const double R0 = residue(m, s, n_ptr);
        // largest-residue interval, skipping single-tenant tails of a cluster
        int best_iv = -1;
        double best_area = -1;
        for (int a = 0; a < (int)s.iv.size(); ++a) {
            const Interval &I = s.iv[a];
            if (popcount64(I.running) == 1) {
                bool later_multi = false;
                for (int b = a; b < (int)s.iv.size() && s.iv[b].cluster == I.cluster; ++b)
                    if (popcount64(s.iv[b].running) > 1) { later_multi = true; break; }
                if (!later_multi) continue;
            }
            const double area = (1.0 - I.used) * (I.t1 - I.t0);
            if (area > best_area || (area == best_area && best_iv < 0)) { best_area = area; best_iv = a; }
        }
        if (best_iv < 0) break;
        const Interval &I = s.iv[best_iv];
        // the largest not-yet-started operator of the same cluster
        int bt = -1, bo = -1;
        double bsize = -1;
        for (int t = 0; t < NT; ++t) {
            const int lo = I.cluster == 0 ? 0 : P[t][I.cluster - 1];
            const int hi = I.cluster == n_ptr ? m.n_ops[t] : P[t][I.cluster];
            for (int i = lo; i < hi; ++i) {
                if (banned.count({t, i})) continue;
                const Split &cur = sp[t][i];
                if (cur.f >= 8 || s.start[t][i] < I.t0) continue;
                const OpTable &ot = m.tab[t][i];
                const int nl = lg(cur.f) + 1;
                bool can = false;
                for (int ax = 1; ax <= 2; ++ax)
                    if (ot.c[ax][nl].have && (cur.f == 1 || ax == cur.axis)) can = true;
                if (!can && !(ot.c[1][1].have || ot.c[2][1].have)) continue;     // not splittable at all
                const Cell &c = cell(m, t, i, cur);
                const double size = c.W * c.T * cur.f;
                if (size > bsize) { bsize = size; bt = t; bo = i; }
            }
        }
        if (bt < 0) break;
        const Split cur = sp[bt][bo];
        const int nf = cur.f * 2, nl = lg(nf);
        int pick = 0;
        double pick_T = 1e300;
        for (int ax = 1; ax <= 2; ++ax) {
            const Cell &c = m.tab[bt][bo].c[ax][nl];
            if (!c.have || (cur.f > 1 && ax != cur.axis)) continue;
            if (c.T * nf < pick_T) { pick_T = c.T * nf; pick = ax; }
        }
        if (!pick) { banned.insert({bt, bo}); continue; }
        sp[bt][bo].axis = pick; sp[bt][bo].f = nf;
        if (evaluate(m, sp, P) < R0) continue;
        sp[bt][bo] = cur;
        banned.insert({bt, bo});
    }
}

void temporal_level(const Model &m, const Splits &sp, Pointers &P, int rounds)
{
    const int NT = m.NT;
    for (int r = 0; r < rounds; ++r) {
        bool changed = false;
        for (int t = 0; t < NT; ++t)
            for (int j = 0; j < (int)P[t].size(); ++j) {
                const int lo = j > 0 ? P[t][j - 1] : 0;
                const int hi = j + 1 < (int)P[t].size() ? P[t][j + 1] : m.n_ops[t];
                const int keep = P[t][j];
                int best_p = keep;
                double best_R = 0;
                bool first = true;
                for (int p = lo; p <= hi; ++p) {
                    P[t][j] = p;
                    const double R = evaluate(m, sp, P);
                    if (first || R < best_R) { best_R = R; best_p = p; first = false; }
                }
                P[t][j] = best_p;
                if (best_p != keep) changed = true;
            }
        if (!changed) break;
    }
}

int midpoint_of_longest_segment(int n_ops, const std::vector<int> &P)
{
    int prev = 0, best = -1, where = 0;
    for (size_t j = 0; j <= P.size(); ++j) {
        const int cut = j < P.size() ? P[j] : n_ops;
        if (cut - prev > best) { best = cut - prev; where = prev + (cut - prev) / 2; }
        prev = cut;
    }
    return where;
}

gacer_status build_model(Ctx *c, const gacer_prof *prof, size_t n, Model &m)
{
    m.NT = (int)c->tenants.size();
    m.n_ops.resize(m.NT);
    m.tab.resize(m.NT);
    for (int t = 0; t < m.NT; ++t) {
        m.n_ops[t] = (int)c->tenants[t].ops.size();
        m.tab[t].assign(m.n_ops[t], OpTable());
    }
    for (size_t k = 0; k < n; ++k) {
        const gacer_prof &p = prof[k];
        if (p.tenant == -1) { m.t_sw = p.ms; continue; }
        if (p.tenant < 0 || p.tenant >= m.NT || p.op < 0 || p.op >= m.n_ops[p.tenant] || (int)p.axis < 0 || (int)p.axis > 2 ||
            (p.factor != 1 && p.factor != 2 && p.factor != 4 && p.factor != 8) || (p.factor > 1) != (p.axis != GACER_AXIS_NONE)) {
            c->err = "profile table row names a missing operator or an illegal (axis, factor)";
            return GACER_EINVAL;
        }
        Cell &ce = m.tab[p.tenant][p.op].c[(int)p.axis][lg(p.factor)];
        ce.T = p.ms; ce.W = p.cu_share; ce.have = true;
    }
    for (int t = 0; t < m.NT; ++t)
        for (int i = 0; i < m.n_ops[t]; ++i)
            if (!m.tab[t][i].c[0][0].have) {
                c->err = "profile table lacks the unsplit row of an operator";
                return GACER_EINVAL;
            }
    return GACER_OK;
}

gacer_plan *to_plan(Ctx *c, const Splits &sp, const Pointers &P)
{
    const int NT = (int)c->tenants.size();
    const int n_ptr = P.empty() ? 0 : (int)P[0].size();
    std::vector<int> flat;
    for (int t = 0; t < NT; ++t) flat.insert(flat.end(), P[t].begin(), P[t].end());
    gacer_plan *edges = nullptr;
    if (gacer_plan_from_pointers(static_cast<gacer_ctx *>(c), flat.empty() ? nullptr : flat.data(), n_ptr, &edges) != GACER_OK) return nullptr;
    std::vector<gacer_split> list;
    for (int t = 0; t < NT; ++t)
        for (int i = 0; i < (int)sp[t].size(); ++i)
            if (sp[t][i].f > 1) list.push_back({t, i, (gacer_axis)sp[t][i].axis, sp[t][i].f, nullptr});
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
    Splits sp(NT);
    for (int t = 0; t < NT; ++t) sp[t].assign(m.n_ops[t], Split());
    Pointers P(NT);
    spatial_step(m, sp, P);
    Splits best_sp = sp;
    Pointers best_P = P;
    double best_R = evaluate(m, sp, P);
    const int min_ops = *std::min_element(m.n_ops.begin(), m.n_ops.end());
    for (int level = 1; level <= 8 && level <= min_ops; ++level) {
        for (int t = 0; t < NT; ++t) {
            P[t].push_back(midpoint_of_longest_segment(m.n_ops[t], P[t]));
            std::sort(P[t].begin(), P[t].end());
        }
        temporal_level(m, sp, P, max_rounds);
        spatial_step(m, sp, P);
        const double R = evaluate(m, sp, P);
        if (R > best_R) break;
        best_R = R; best_sp = sp; best_P = P;
    }
    gacer_plan *pl = to_plan(c, best_sp, best_P);
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
    Splits sp(NT);
    for (int t = 0; t < NT; ++t) sp[t].assign(m.n_ops[t], Split());
    for (int k = 0; k < n_split; ++k) {
        const gacer_split &s = split[k];
        if (s.sizes) { c->err = "the model covers even decompositions only (the lookup table has no rows for chunk lists)"; return GACER_EPLAN; }
        if (s.tenant < 0 || s.tenant >= NT || s.op < 0 || s.op >= m.n_ops[s.tenant] || (int)s.axis < 0 || (int)s.axis > 2 ||
            (s.factor != 1 && s.factor != 2 && s.factor != 4 && s.factor != 8) ||
            !m.tab[s.tenant][s.op].c[s.factor > 1 ? (int)s.axis : 0][lg(s.factor)].have) {
            c->err = "split not covered by the profile table";
            return GACER_EPLAN;
        }
        sp[s.tenant][s.op].axis = (int)s.axis;
        sp[s.tenant][s.op].f = s.factor;
    }
    Pointers P(NT);
    for (int t = 0; t < NT; ++t)
        for (int j = 0; j < n_ptr; ++j) {
            const int p = Pm[t * n_ptr + j];
            if (p < 0 || p > m.n_ops[t] || (j > 0 && p < Pm[t * n_ptr + j - 1])) { c->err = "pointers must be sorted and in range"; return GACER_EPLAN; }
            P[t].push_back(p);
        }
    Sim s;
    simulate(m, sp, P, s);
    *residue_out = residue(m, s, n_ptr);
    if (makespan_out) *makespan_out = s.total;
    return GACER_OK;
}

}  // extern "C"
