"""Oracle for the regulation model: segmentation, residue and the search.

TEST INFRASTRUCTURE ONLY; the product's host-side search is separate code.

Everything here follows Sections 4.1-4.4 step by step, in the paper's notation:

* ``segments``        -- Eq. 7: a pointer list P cuts a model's operator list into
                         len(P)+1 segments; same-index segments of all models form a
                         cluster (Eq. 6).
* ``simulate``        -- the runtime deployment sequence S_T0 -> S_Tt of Eq. 1 for a
                         given (mask/list_B, Matrix_P): which operators are resident at
                         which time, under  sum W <= S_GPU.
* ``residue``         -- Eq. 2/3 summed over the sequence plus the pointer term of Eq. 8.
* ``search``          -- Algorithm 1 (coordinate descent over pointer positions, one more
                         pointer per level, stop when the best residue gets worse)
                         alternated with the greedy spatial step of Section 4.2.

Where the paper leaves a choice open the reading taken is stated at the spot.
"""
from dataclasses import dataclass
from typing import Dict, List, Tuple

S_GPU = 1.0   # the SM/CU pool, "100%" (Section 4.1)
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
    """One row of the lookup table (Section 4.1): time T of one chunk and its
    workload W (share of the pool) for operator (model, op) decomposed
    ``factor`` ways along ``axis``."""
    T: float
    W: float


Table = Dict[Tuple[int, int, int, int], Entry]   # (model, op0, axis, factor) -> Entry; axis 0 none,1 batch,2 cout


def chunk_list(table: Table, n: int, i: int, split):
    """list_B of operator (n,i): ``factor`` equal chunks, each (T, W)."""
    axis, f = split.get((n, i), (0, 1))
    e = table[(n, i, axis if f > 1 else 0, f)]
    return [(e.T, e.W)] * f


def simulate(n_ops_per_model, table: Table, split, matrix_P, T_SW: float):
    """Deployment sequence under the pool constraint (Eq. 1).

    Reading of the model: time is continuous; each model issues its operators
    (chunks) in order; an operator occupies W of the pool for T; it starts as
    soon as its predecessor in the same model has finished, its cluster is
    open and W fits into what is left of S_GPU -- otherwise it waits for the
    next completion ("moved to the next cycle", Section 3.1).  When several
    models wait, the lower model index is served first.  A cluster opens when
    every operator of the previous cluster is done; each pointer then costs an
    idle wait of T_SW (Section 4.3, overhead analysis).

    Returns (intervals, starts, total) where intervals is a list of
    (t0, t1, used, cluster, running_models), starts maps (n, i, chunk) -> start
    time and total is the completion time including pointer waits.
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
                for c, (T, W) in enumerate(chunk_list(table, n, i1 - 1, split)):
                    q.append((i1 - 1, c, T, W))
            queues.append(q)
        pos = [0] * N
        running = {}            # model -> (finish_time, W)
        while True:
            used = sum(w for (_, w) in running.values())
            for n in range(N):  # greedy issue in model order
                if n in running or pos[n] >= len(queues[n]):
                    continue
                i, c, T, W = queues[n][pos[n]]
                if used + W <= S_GPU + 1e-12 or not running:
                    running[n] = (t + T, W)
                    starts[(n, i, c)] = t
                    used += W
                    pos[n] += 1
            if not running:
                break
            t1 = min(f for (f, _) in running.values())
            intervals.append((t, t1, used, k, tuple(sorted(running))))
            t = t1
            for n in [n for n, (f, _) in running.items() if f <= t1]:
                del running[n]
    return intervals, starts, t


def residue(intervals, n_pointers: int, T_SW: float) -> float:
    """Eq. 8: sum over the sequence of (S_GPU - sum W) plus |P| * S_GPU * T_SW.
    With continuous time the sum over cycles is the integral over intervals."""
    R = 0.0
    for (t0, t1, used, _, _) in intervals:
        R += (S_GPU - used) * (t1 - t0)
    return R + n_pointers * S_GPU * T_SW


def evaluate(n_ops, table, split, matrix_P, T_SW):
    iv, _, _ = simulate(n_ops, table, split, matrix_P, T_SW)
    return residue(iv, len(matrix_P[0]) if matrix_P else 0, T_SW)


def _longest_segment_midpoint(n_ops, P):
    """Where a new pointer starts (the paper does not say): the middle of the
    model's longest segment, earliest such segment on ties."""
    cuts = [0] + list(P) + [n_ops]
    best, where = -1, 0
    for a, b in zip(cuts, cuts[1:]):
        if b - a > best:
            best, where = b - a, a + (b - a) // 2
    return where


def spatial_step(n_ops, table, split, matrix_P, T_SW, splittable, max_moves=8):
    """Greedy spatial regulation (Section 4.2, "Overall Spatial Regulation").

    Repeat: find the interval with the largest residue (S_GPU - used) * length,
    ignoring intervals in which a single model runs the tail of its segment
    after every other model of the cluster has finished (those residues are
    skipped); among the not-yet-started operators of the same cluster (the
    dependence check: a chunk can only move inside its cluster) take the one
    with the largest W*T; decompose it one step further (factor 1->2->4->8) on
    the allowed axis whose table time is lowest; keep the change if the
    residue of Eq. 8 drops, otherwise undo it and never try that operator
    again in this step.  ``splittable`` maps (n,i) -> tuple of allowed axes.
    """
    split = dict(split)
    n_ptr = len(matrix_P[0]) if matrix_P else 0
    banned = set()
    for _ in range(max_moves):
        iv, starts, _ = simulate(n_ops, table, split, matrix_P, T_SW)
        R0 = residue(iv, n_ptr, T_SW)
        # last interval index per cluster in which more than one model still has work
        cand_iv = []
        for idx, (t0, t1, used, k, run) in enumerate(iv):
            later_multi = any(k2 == k and len(r2) > 1 for (_, _, _, k2, r2) in iv[idx:])
            if len(run) == 1 and not later_multi:
                continue                      # tail of the longest segment: skipped
            cand_iv.append(((S_GPU - used) * (t1 - t0), -idx))
        if not cand_iv:
            break
        _, negidx = max(cand_iv)
        t0, t1, used, k, run = iv[-negidx]
        cl = clusters(n_ops, matrix_P)[k]
        best = None
        for n, ops1 in enumerate(cl):
            for i1 in ops1:
                i = i1 - 1
                if (n, i) in banned or (n, i) not in splittable:
                    continue
                axis, f = split.get((n, i), (0, 1))
                if f >= FACTORS[-1] or starts[(n, i, 0)] < t0:
                    continue
                e = table[(n, i, axis if f > 1 else 0, f)]
                size = e.W * e.T * f
                if best is None or size > best[0]:
                    best = (size, n, i)
        if best is None:
            break
        _, n, i = best
        axis, f = split.get((n, i), (0, 1))
        nf = FACTORS[FACTORS.index(f) + 1]
        options = [(table[(n, i, a, nf)].T * nf, a) for a in splittable[(n, i)]
                   if (n, i, a, nf) in table and (f == 1 or a == axis)]
        if not options:
            banned.add((n, i))
            continue
        _, a = min(options)
        trial = dict(split)
        trial[(n, i)] = (a, nf)
        if evaluate(n_ops, table, trial, matrix_P, T_SW) < R0:
            split = trial
        else:
            banned.add((n, i))
    return split


def temporal_level(n_ops, table, split, matrix_P, T_SW, rounds, D):
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
                    R = evaluate(n_ops, table, split, trial, T_SW)
                    D.append((R, [tuple(P) for P in trial]))
                    if best_R is None or R < best_R:
                        best_R, best_p = R, p
                if best_p != matrix_P[n][j]:
                    matrix_P[n][j] = best_p
                    changed = True
        if not changed:
            break
    return matrix_P


def search(n_ops, table, T_SW, splittable, rounds=100, max_pointers=8):
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
    split = spatial_step(n_ops, table, split, matrix_P, T_SW, splittable)
    best = (dict(split), [list(P) for P in matrix_P], evaluate(n_ops, table, split, matrix_P, T_SW))
    D.append((best[2], [tuple(P) for P in matrix_P]))
    for level in range(1, max_pointers + 1):
        if level > min(n_ops):
            break
        matrix_P = [sorted(P + [_longest_segment_midpoint(n, P)]) for n, P in zip(n_ops, matrix_P)]
        matrix_P = temporal_level(n_ops, table, split, matrix_P, T_SW, rounds, D)
        split = spatial_step(n_ops, table, split, matrix_P, T_SW, splittable)
        R = evaluate(n_ops, table, split, matrix_P, T_SW)
        if R > best[2]:
            break
        best = (dict(split), [list(P) for P in matrix_P], R)
    return best[0], best[1], best[2], D
