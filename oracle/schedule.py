"""Oracle for the regulation model: segmentation, residue and the search.

TEST INFRASTRUCTURE ONLY; the product's host-side search is separate code.

Everything here follows Sections 4.1-4.4 step by step, in the paper's notation:

* ``segments``        -- Eq. 7: a pointer list P cuts a model's operator list into
                         len(P)+1 segments; same-index segments of all models form a
                         cluster (Eq. 6).
* ``chunk_entry``     -- the lookup table of Section 4.1 read at a chunk size: (T, W) of
                         operator O with part of its batch (or of its output channels).
* ``simulate``        -- the runtime deployment sequence S_T0 -> S_Tt of Eq. 1 for a
                         given (mask/list_B, Matrix_P): which operators are resident at
                         which time, under  sum W <= S_GPU  (and, when the table carries a
                         second resource, under its pool as well: claim (2) of Section 4.4).
* ``residue``         -- Eq. 2/3 summed over the sequence plus the pointer term of Eq. 8.
* ``spatial_step``    -- "Overall Spatial Regulation" of Section 4.2.
* ``search``          -- Algorithm 1 (coordinate descent over pointer positions, one more
                         pointer per level, stop when the best residue gets worse)
                         alternated with the spatial step.

Where the paper leaves a choice open the reading taken is stated at the spot.
"""
from dataclasses import dataclass
from typing import Dict, List, Tuple

S_GPU = 1.0   # the SM/CU pool, "100%" (Section 4.1)
S_BW = 1.0    # the second pool (memory bandwidth), same normalisation
FACTORS = (1, 2, 4, 8)


def segments(n_ops: int, P) -> List[List[int]]:
    """Eq. 7.  A pointer of value p cuts after the p-th operator (1-based), so
    P=(2,8) on 12 operators yields operators 1-2, 3-8, 9-12.  p=0 or repeated
    values give an empty segment (the ``[None]`` entry of Eq. 6)."""
    P = list(P)
    if any(p < 0 or p > n_ops for p in P) or any(a > b for a, b in zip(P, P[1:])):
        raise ValueError("pointers must be sorted and lie in [0, n_ops]")
    cuts = [0] + P + [n_ops]
    return [list(range(a + 1, b + 1)) for a, b in zip(cuts, cuts[1:])]


def clusters(n_ops_per_model, matrix_P) -> List[List[List[int]]]:
    """Eq. 6.  clusters[k][n] = operators (1-based) of model n in cluster k.
    Every P must hold the same number of pointers (Section 4.3)."""
    if len(set(len(P) for P in matrix_P)) > 1:
        raise ValueError("every P must have the same number of pointers")
    segs = [segments(n, P) for n, P in zip(n_ops_per_model, matrix_P)]
    return [[s[k] for s in segs] for k in range(len(segs[0]))]


@dataclass
class Entry:
    """One row of the lookup table (Section 4.1): time T of one chunk, its
    workload W (share of the SM/CU pool) and, optionally, its share Wb of the
    second pool, for operator (model, op) decomposed ``factor`` ways along
    ``axis``."""
    T: float
    W: float
    Wb: float = 0.0


# (model, op0, axis, factor) -> Entry; axis 0 none, 1 batch, 2 cout.  The row of factor f describes a chunk of
# extent/f elements of the axis; factor 1 (axis 0) is the whole operator.
Table = Dict[Tuple[int, int, int, int], Entry]


def chunk_entry(table: Table, n: int, i: int, axis: int, size: int, extent: int) -> Entry:
    """(T, W, Wb) of a chunk holding ``size`` of the ``extent`` elements of ``axis``.

    The table is sampled at the chunk sizes extent/f, f in FACTORS (the paper
    profiles operators "with different batch settings", Section 4.1).  Reading
    for the sizes in between (list_B may hold any sizes, Eq. 5): linear
    interpolation in the chunk size between the two neighbouring samples; below
    the smallest sample, proportional to the size (a line through the origin).
    W and Wb are capped at their pools."""
    pts = [(float(extent), table[(n, i, 0, 1)])]
    for f in FACTORS[1:]:
        if (n, i, axis, f) in table:
            pts.append((extent / f, table[(n, i, axis, f)]))
    pts.sort(key=lambda p: p[0])
    s = float(size)
    for x, e in pts:
        if abs(x - s) < 1e-12:
            return e
    lo = [(x, e) for x, e in pts if x < s]
    hi = [(x, e) for x, e in pts if x > s]
    if not hi:
        raise ValueError("chunk larger than the operator")
    x1, e1 = hi[0]
    if lo:
        x0, e0 = lo[-1]
        a = (s - x0) / (x1 - x0)
        T, W, Wb = e0.T + a * (e1.T - e0.T), e0.W + a * (e1.W - e0.W), e0.Wb + a * (e1.Wb - e0.Wb)
    else:
        a = s / x1
        T, W, Wb = a * e1.T, a * e1.W, a * e1.Wb
    return Entry(T, min(W, S_GPU), min(Wb, S_BW))


def chunk_list(table: Table, n: int, i: int, split, extent_of=None):
    """The chunks of operator (n,i) in issue order, each (T, W, Wb).  An even
    f-way decomposition is the table's own row for (axis, f), f times; a list of
    sizes is read off the table size by size (``chunk_entry``)."""
    axis, f = split.get((n, i), (0, 1))
    if not isinstance(f, (list, tuple)):
        e = table[(n, i, axis if f > 1 else 0, f)]
        return [(e.T, e.W, e.Wb)] * f
    E = extent_of(n, i, axis)
    if sum(f) != E or min(f) < 1:
        raise ValueError("chunk sizes must be positive and sum to the extent (Eq. 5)")
    out = []
    for sz in f:
        e = chunk_entry(table, n, i, axis, sz, E)
        out.append((e.T, e.W, e.Wb))
    return out


def simulate(n_ops_per_model, table: Table, split, matrix_P, T_SW: float, extent_of=None):
    """Deployment sequence under the pool constraint (Eq. 1).

    Reading of the model: time is continuous; each model issues its operators
    (chunks) in order; an operator occupies W of the pool for T; it starts as
    soon as its predecessor in the same model has finished, its cluster is
    open and its demands fit into what is left of every pool (S_GPU, and the
    second pool when the table carries Wb) -- otherwise it waits for the next
    completion (an operator that lacks any required resource "is moved to the
    next cycle", Section 3.1).  When several models wait, the lower model index
    is served first.  A cluster opens when every operator of the previous
    cluster is done; each pointer then costs an idle wait of T_SW (Section 4.3,
    overhead analysis).

    Returns (intervals, starts, total) where intervals is a list of
    (t0, t1, used, cluster, running_models, used_b, pending_models), starts maps
    (n, i, chunk) -> start time and total is the completion time including
    pointer waits.  pending_models = models that still have a chunk of this
    cluster running or waiting during the interval.
    """
    N = len(n_ops_per_model)
    cl = clusters(n_ops_per_model, matrix_P)
    intervals, starts = [], {}
    t = 0.0
    for k, cluster in enumerate(cl):
        if k > 0:
            t += T_SW
        queues = []
        for n in range(N):
            q = []
            for i1 in cluster[n]:
                for c, (T, W, Wb) in enumerate(chunk_list(table, n, i1 - 1, split, extent_of)):
                    q.append((i1 - 1, c, T, W, Wb))
            queues.append(q)
        pos = [0] * N
        running = {}            # model -> (finish_time, W, Wb)
        while True:
            used = sum(w for (_, w, _) in running.values())
            used_b = sum(wb for (_, _, wb) in running.values())
            for n in range(N):  # greedy issue in model order
                if n in running or pos[n] >= len(queues[n]):
                    continue
                i, c, T, W, Wb = queues[n][pos[n]]
                if (used + W <= S_GPU + 1e-12 and used_b + Wb <= S_BW + 1e-12) or not running:
                    running[n] = (t + T, W, Wb)
                    starts[(n, i, c)] = t
                    used += W
                    used_b += Wb
                    pos[n] += 1
            if not running:
                break
            t1 = min(f for (f, _, _) in running.values())
            pending = tuple(n for n in range(N) if n in running or pos[n] < len(queues[n]))
            intervals.append((t, t1, used, k, tuple(sorted(running)), used_b, pending))
            t = t1
            for n in [n for n, (f, _, _) in running.items() if f <= t1]:
                del running[n]
    return intervals, starts, t


def residue(intervals, n_pointers: int, T_SW: float, second_pool: bool = False) -> float:
    """Eq. 8: sum over the sequence of (S_GPU - sum W) plus |P| * S_GPU * T_SW.
    With continuous time the sum over cycles is the integral over intervals.
    With ``second_pool`` the unused part of the second pool is added cycle by
    cycle in the same way (claim (2) of Section 4.4 gives no formula; reading:
    the residue of every pool counts, each in units of its own pool)."""
    R = 0.0
    for iv in intervals:
        t0, t1, used = iv[0], iv[1], iv[2]
        R += (S_GPU - used) * (t1 - t0)
        if second_pool:
            R += (S_BW - iv[5]) * (t1 - t0)
    return R + n_pointers * S_GPU * T_SW


def _second_pool(table) -> bool:
    return any(e.Wb > 0.0 for e in table.values())


def evaluate(n_ops, table, split, matrix_P, T_SW, extent_of=None):
    iv, _, _ = simulate(n_ops, table, split, matrix_P, T_SW, extent_of)
    return residue(iv, len(matrix_P[0]) if matrix_P else 0, T_SW, _second_pool(table))


def _longest_segment_midpoint(n_ops, P):
    """Where a new pointer starts (the paper does not say): the middle of the
    model's longest segment, earliest such segment on ties."""
    cuts = [0] + list(P) + [n_ops]
    best, where = -1, 0
    for a, b in zip(cuts, cuts[1:]):
        if b - a > best:
            best, where = b - a, a + (b - a) // 2
    return where


def matching_chunk(table, n, i, axis, extent, free, free_b):
    """"Decompose a batch that matches the residue size" (Section 4.2): the
    largest chunk size b < extent whose workload fits the free share of the
    residue it is meant for (W(b) <= free, and Wb(b) <= free_b), or 0 when not
    even one element fits.  Chunk sizes are whole elements of the axis."""
    best = 0
    for b in range(1, extent):
        e = chunk_entry(table, n, i, axis, b, extent)
        if e.W <= free + 1e-12 and e.Wb <= free_b + 1e-12:
            best = b
    return best


def spatial_step(n_ops, table, split, matrix_P, T_SW, splittable, extent_of, max_moves=8):
    """Greedy spatial regulation (Section 4.2, "Overall Spatial Regulation"),
    one move at a time, in the order the section gives:

    1. the biggest residue: the interval of the current deployment sequence
       with the largest unused share x length (Eq. 2 per cycle; in continuous
       time a cycle is an interval).  Residues in the tail of a cluster -- the
       intervals in which only one model still has operators of this cluster
       to run, every other model having finished its segment -- are skipped;
    2. the operator with the largest size following this cycle: among the
       operators of the same cluster that have not started when the interval
       begins (dependence check: a chunk can only move inside its cluster)
       and are not decomposed yet, the one with the largest workload W*T;
    3. a chunk that matches the residue: list_B = [b, extent - b] with b the
       largest chunk whose workload fits the interval's unused share (on the
       allowed axis for which the two chunks take the least time);
    4. the mask, list_B and the sequence are updated; the move is kept if the
       residue of Eq. 8 drops, otherwise undone, and the operator is not tried
       again in this step.

    ``splittable`` maps (n,i) -> tuple of allowed axes, ``extent_of(n,i,axis)``
    gives the axis extent.  Returns the new split dictionary
    (n,i) -> (axis, [b, extent - b]).
    """
    split = dict(split)
    n_ptr = len(matrix_P[0]) if matrix_P else 0
    two = _second_pool(table)
    banned = set()
    for _ in range(max_moves):
        iv, starts, _ = simulate(n_ops, table, split, matrix_P, T_SW, extent_of)
        R0 = residue(iv, n_ptr, T_SW, two)
        cand = []
        for idx, (t0, t1, used, k, run, used_b, pending) in enumerate(iv):
            if len(pending) == 1:
                continue                      # tail of the longest segment of this cluster: skipped
            cand.append(((S_GPU - used) * (t1 - t0), -idx))
        if not cand:
            break
        _, negidx = max(cand)                 # largest residue, earliest interval on ties
        t0, t1, used, k, run, used_b, pending = iv[-negidx]
        cl = clusters(n_ops, matrix_P)[k]
        best = None
        for n, ops1 in enumerate(cl):
            for i1 in ops1:
                i = i1 - 1
                if (n, i) in banned or (n, i) not in splittable or (n, i) in split:
                    continue
                if starts[(n, i, 0)] < t0 + 1e-12:
                    continue                  # already running (or done) when this residue begins
                e = table[(n, i, 0, 1)]
                size = e.W * e.T
                if best is None or size > best[0]:
                    best = (size, n, i)
        if best is None:
            break
        _, n, i = best
        options = []
        for a in splittable[(n, i)]:
            E = extent_of(n, i, a)
            b = matching_chunk(table, n, i, a, E, S_GPU - used, S_BW - used_b if two else S_BW)
            if b >= 1:
                T2 = chunk_entry(table, n, i, a, b, E).T + chunk_entry(table, n, i, a, E - b, E).T
                options.append((T2, a, b, E))
        if not options:
            banned.add((n, i))
            continue
        _, a, b, E = min(options)
        trial = dict(split)
        trial[(n, i)] = (a, [b, E - b])
        if evaluate(n_ops, table, trial, matrix_P, T_SW, extent_of) < R0:
            split = trial
        else:
            banned.add((n, i))
    return split


def temporal_level(n_ops, table, split, matrix_P, T_SW, rounds, D, extent_of=None):
    """The inner loops of Algorithm 1 for a fixed number of pointers: for each
    round, for each model, for each of its pointers, try every position
    between the neighbouring pointers (all other pointers fixed), record
    {R: Matrix_P} in D and move the pointer to the position of smallest R
    (earliest on ties).  Stops early once a full round changes nothing."""
    matrix_P = [list(P) for P in matrix_P]
    N = len(n_ops)
    for _ in range(rounds):
        changed = False
        for n in range(N):
            for j in range(len(matrix_P[n])):
                lo = matrix_P[n][j - 1] if j > 0 else 0
                hi = matrix_P[n][j + 1] if j + 1 < len(matrix_P[n]) else n_ops[n]
                best_R, best_p = None, matrix_P[n][j]
                for p in range(lo, hi + 1):
                    trial = [list(P) for P in matrix_P]
                    trial[n][j] = p
                    R = evaluate(n_ops, table, split, trial, T_SW, extent_of)
                    D.append((R, [tuple(P) for P in trial]))
                    if best_R is None or R < best_R:
                        best_R, best_p = R, p
                if best_p != matrix_P[n][j]:
                    matrix_P[n][j] = best_p
                    changed = True
        if not changed:
            break
    return matrix_P


def search(n_ops, table, T_SW, splittable, extent_of, rounds=100, max_pointers=8):
    """Granularity-aware search (Algorithm 1 alternated with the spatial step).

    Level |P| = 0,1,2,...: (temporal search at this pointer count) then (one
    spatial step); the level's score is the residue of Eq. 8 afterwards.  If a
    level scores worse than the previous one, the previous level's solution is
    returned; otherwise one pointer is added to every P and the search goes on.
    Returns (split, Matrix_P, R, D).
    """
    N = len(n_ops)
    D = []
    split, matrix_P = {}, [[] for _ in range(N)]
    split = spatial_step(n_ops, table, split, matrix_P, T_SW, splittable, extent_of)
    best = (dict(split), [list(P) for P in matrix_P], evaluate(n_ops, table, split, matrix_P, T_SW, extent_of))
    D.append((best[2], [tuple(P) for P in matrix_P]))
    for level in range(1, max_pointers + 1):
        if level > min(n_ops):
            break
        matrix_P = [sorted(P + [_longest_segment_midpoint(n, P)]) for n, P in zip(n_ops, matrix_P)]
        matrix_P = temporal_level(n_ops, table, split, matrix_P, T_SW, rounds, D, extent_of)
        split = spatial_step(n_ops, table, split, matrix_P, T_SW, splittable, extent_of)
        R = evaluate(n_ops, table, split, matrix_P, T_SW, extent_of)
        if R > best[2]:
            break
        best = (dict(split), [list(P) for P in matrix_P], R)
    return best[0], best[1], best[2], D
