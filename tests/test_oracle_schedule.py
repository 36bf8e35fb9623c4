"""Pins for the regulation-model oracle (segmentation, residue, search)."""
import itertools
import os

import numpy as np
import pytest

import synth
from oracle import schedule as S


def _golden(golden_dir):
    rows = []
    for line in open(os.path.join(golden_dir, "segmentation_eq6_eq7.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, ptr, segs = [s.strip() for s in line.split("|")]
        n_ops = int(head.split()[1])
        P = [int(v) for v in ptr.split()]
        seg = [[] if s.strip() == "-" else [int(v) for v in s.split()] for s in segs.split(";")]
        rows.append((n_ops, P, seg))
    return rows


def test_segmentation_worked_example(golden_dir):
    rows = _golden(golden_dir)
    for n_ops, P, seg in rows:
        assert S.segments(n_ops, P) == seg
    cl = S.clusters([r[0] for r in rows], [r[1] for r in rows])
    assert cl[0] == [[1, 2], []] and cl[1][1] == [1, 2, 3, 4] and cl[2][0] == [9, 10, 11, 12]
    assert [len(s) for s in S.segments(12, (2, 8))] == [2, 6, 4]


def test_pointer_validation():
    with pytest.raises(ValueError):
        S.clusters([4, 4], [[1], [1, 2]])          # unequal pointer counts
    with pytest.raises(ValueError):
        S.segments(4, [3, 2])
    with pytest.raises(ValueError):
        S.segments(4, [5])


def _random_table(rng, n_ops, wmax=1.0):
    table, splittable = {}, {}
    for n, k in enumerate(n_ops):
        for i in range(k):
            T = float(rng.uniform(0.1, 2.0))
            W = float(rng.uniform(0.05, wmax))
            table[(n, i, 0, 1)] = S.Entry(T, W)
            axes = (1, 2) if rng.random() < 0.7 else ((1,) if rng.random() < 0.5 else ())
            if axes:
                splittable[(n, i)] = axes
            for a in axes:
                for f in (2, 4, 8):
                    table[(n, i, a, f)] = S.Entry(T / f * float(rng.uniform(1.0, 1.3)), max(0.02, W / f))
    return table, splittable


def test_residue_closed_form():
    """Eq. 8 with constant S_GPU rearranges to R = S_GPU*T_busy - sum W*T + |P|*S_GPU*T_SW,
    where T_busy is the completion time without the pointer waits."""
    rng = np.random.default_rng(1)
    for trial in range(40):
        n_ops = [int(rng.integers(1, 7)) for _ in range(int(rng.integers(1, 4)))]
        table, splittable = _random_table(rng, n_ops)
        npnt = int(rng.integers(0, 3))
        P = [sorted(int(rng.integers(0, k + 1)) for _ in range(npnt)) for k in n_ops]
        split = {}
        for key, axes in splittable.items():
            if rng.random() < 0.4:
                split[key] = (axes[0], int(rng.choice([2, 4, 8])))
        T_SW = 0.07
        iv, starts, total = S.simulate(n_ops, table, split, P, T_SW)
        work = sum(T * W for n, k in enumerate(n_ops) for i in range(k) for (T, W, _) in S.chunk_list(table, n, i, split))
        closed = S.S_GPU * (total - npnt * T_SW) - work + npnt * S.S_GPU * T_SW
        assert abs(S.residue(iv, npnt, T_SW) - closed) < 1e-9
        assert all(iv_[2] <= S.S_GPU + 1e-9 or len(iv_[4]) == 1 for iv_ in iv)   # Eq. 1 constraint
        assert len(starts) == sum(len(S.chunk_list(table, n, i, split)) for n, k in enumerate(n_ops) for i in range(k))


def test_simulator_special_cases():
    e = lambda T, W: S.Entry(T, W)
    # one stream: completion time is the sum of the operator times
    table = {(0, 0, 0, 1): e(1.0, 0.3), (0, 1, 0, 1): e(2.0, 1.0), (0, 2, 0, 1): e(0.5, 0.6)}
    _, _, total = S.simulate([3], table, {}, [[]], 0.1)
    assert abs(total - 3.5) < 1e-12
    # two identical streams with W <= 0.5 overlap completely
    table = {(n, i, 0, 1): e(1.0 + i, 0.5) for n in range(2) for i in range(3)}
    iv, _, total = S.simulate([3, 3], table, {}, [[], []], 0.1)
    assert abs(total - 6.0) < 1e-12 and abs(S.residue(iv, 0, 0.1)) < 1e-12
    # two streams with W > 0.5 cannot share a cycle: fully serialised
    table = {(n, i, 0, 1): e(1.0, 0.6) for n in range(2) for i in range(2)}
    iv, _, total = S.simulate([2, 2], table, {}, [[], []], 0.1)
    assert abs(total - 4.0) < 1e-12 and abs(S.residue(iv, 0, 0.1) - 4 * 0.4) < 1e-12
    # a pointer after op 1 in both models: two clusters, one T_SW wait
    _, starts, total = S.simulate([2, 2], table, {}, [[1], [1]], 0.1)
    assert abs(total - 4.1) < 1e-12 and abs(starts[(0, 1, 0)] - 2.1) < 1e-12


def test_pointer_reordering_example():
    """Fig. 5 in words: stream 1 = [C, B], stream 2 = [C]; C is too wide to share the pool with C but fits
    beside B.  A pointer that holds stream 2's C back to the second cluster lets it overlap B."""
    e = lambda T, W: S.Entry(T, W)
    table = {(0, 0, 0, 1): e(1.0, 0.7), (0, 1, 0, 1): e(1.0, 0.3), (1, 0, 0, 1): e(1.0, 0.7)}
    R_none = S.evaluate([2, 1], table, {}, [[], []], 0.0)
    R_ptr = S.evaluate([2, 1], table, {}, [[1], [0]], 0.0)
    assert R_ptr < R_none + 1e-12
    iv, _, total = S.simulate([2, 1], table, {}, [[1], [0]], 0.0)
    assert abs(total - 2.0) < 1e-12


def _EXT8(n, i, axis):
    return 8


def _brute_force(n_ops, table, splittable, T_SW, max_ptr=1):
    """every list_B = [b, 8 - b] on every allowed axis of every operator, every pointer matrix of up to max_ptr pointers"""
    best = None
    keys = sorted(splittable)
    choices = []
    for k in keys:
        c = [(0, 1)]
        for a in splittable[k]:
            c += [(a, [b, 8 - b]) for b in range(1, 8)]
        choices.append(c)
    for combo in itertools.product(*choices):
        split = {k: v for k, v in zip(keys, combo) if v[1] != 1}
        for npnt in range(max_ptr + 1):
            for Ps in itertools.product(*[itertools.combinations_with_replacement(range(k + 1), npnt) for k in n_ops]):
                R = S.evaluate(n_ops, table, split, [list(P) for P in Ps], T_SW, _EXT8)
                if best is None or R < best:
                    best = R
    return best


def test_search_against_brute_force():
    rng = np.random.default_rng(3)
    for trial in range(6):
        n_ops = [int(rng.integers(2, 4)), int(rng.integers(2, 4))]
        table, splittable = _random_table(rng, n_ops)
        splittable = {k: v[:1] for k, v in list(splittable.items())[:3]}      # keeps the enumeration small
        T_SW = 0.05
        R_none = S.evaluate(n_ops, table, {}, [[], []], T_SW)
        split, P, R, D = S.search(n_ops, table, T_SW, splittable, _EXT8, rounds=10, max_pointers=1)
        opt = _brute_force(n_ops, table, splittable, T_SW, 1)
        assert opt - 1e-9 <= R <= R_none + 1e-9
        assert abs(S.evaluate(n_ops, table, split, P, T_SW, _EXT8) - R) < 1e-12
        assert len(set(len(p) for p in P)) == 1
        assert all(r >= opt - 1e-9 for r, _ in D)


def test_search_stops_adding_pointers_when_sync_is_expensive():
    rng = np.random.default_rng(5)
    n_ops = [6, 5, 4]
    table, splittable = _random_table(rng, n_ops)
    _, P_cheap, _, _ = S.search(n_ops, table, 0.0, splittable, _EXT8, rounds=5, max_pointers=4)
    _, P_dear, R_dear, _ = S.search(n_ops, table, 100.0, splittable, _EXT8, rounds=5, max_pointers=4)
    assert len(P_dear[0]) == 0 and len(P_cheap[0]) >= len(P_dear[0])


# ---- pins for the choices the search makes (hand-built tables; expected values follow from the rules of Section 4.2 and
# ---- Algorithm 1 as restated in the docstrings, worked out by hand in the comments) --------------------------------------
def _linear_rows(n, i, T, W, axes=(1,), Wb=0.0):
    """table rows of an operator whose time and workload are proportional to the chunk size (batch 8)"""
    rows = {(n, i, 0, 1): S.Entry(T, W, Wb)}
    for a in axes:
        for f in (2, 4, 8):
            rows[(n, i, a, f)] = S.Entry(T / f, W / f, Wb / f)
    return rows


def test_chunk_entry_reads_the_table_between_its_samples():
    table = {(0, 0, 0, 1): S.Entry(1.0, 0.8), (0, 0, 1, 2): S.Entry(0.6, 0.5), (0, 0, 1, 4): S.Entry(0.4, 0.3), (0, 0, 1, 8): S.Entry(0.3, 0.2)}
    assert S.chunk_entry(table, 0, 0, 1, 8, 8) == S.Entry(1.0, 0.8)
    assert S.chunk_entry(table, 0, 0, 1, 4, 8) == S.Entry(0.6, 0.5)               # a sample: the row itself
    e = S.chunk_entry(table, 0, 0, 1, 6, 8)                                       # half way between 4 and 8
    assert abs(e.T - 0.8) < 1e-12 and abs(e.W - 0.65) < 1e-12
    e = S.chunk_entry(table, 0, 0, 1, 3, 8)                                       # half way between 2 and 4
    assert abs(e.T - 0.5) < 1e-12 and abs(e.W - 0.4) < 1e-12
    e = S.chunk_entry(table, 0, 0, 1, 1, 8)                                       # the smallest sample
    assert e == S.Entry(0.3, 0.2)
    # an operator without rows for that axis: the line from the origin to the whole operator
    e = S.chunk_entry({(0, 0, 0, 1): S.Entry(2.0, 0.6)}, 0, 0, 1, 2, 8)
    assert abs(e.T - 0.5) < 1e-12 and abs(e.W - 0.15) < 1e-12
    # chunks of a list are read one by one, and the sizes must sum to the extent (Eq. 5)
    got = S.chunk_list(table, 0, 0, {(0, 0): (1, [6, 2])}, _EXT8)
    assert abs(got[0][0] - 0.8) < 1e-12 and got[1][:2] == (0.4, 0.3)
    with pytest.raises(ValueError):
        S.chunk_list(table, 0, 0, {(0, 0): (1, [6, 3])}, _EXT8)


def test_new_pointer_starts_mid_way_through_the_longest_segment():
    assert S._longest_segment_midpoint(12, [2, 8]) == 5      # segments 2 / 6 / 4 (the example of Eq. 7): middle of [2, 8)
    assert S._longest_segment_midpoint(8, []) == 4
    assert S._longest_segment_midpoint(8, [4]) == 2          # two segments of four: the earlier one
    assert S._longest_segment_midpoint(6, [0]) == 3          # an empty first segment
    assert S._longest_segment_midpoint(7, [1, 2]) == 4       # [2, 7) has five operators: 2 + 5 // 2


def _spatial_case():
    """Model 0 = [a0 (T 1, W .6), a1 (T 2, W .5)], model 1 = [b0 (T 1, W .4), b1 (T 1, W .8), b2 (T .5, W .3), b3 (T 3, W .2)],
    no pointers.  Deployment: [0,1] a0+b0 (pool full); [1,3] a1 alone at .5 while b1 (.8) does not fit -> residue .5 x 2 = 1.0;
    from t = 3 model 1 runs b1, b2, b3 on its own (the tail: residues .2, .35 and 2.4, which must be skipped)."""
    table = {}
    table.update(_linear_rows(0, 0, 1.0, 0.6))
    table.update(_linear_rows(0, 1, 2.0, 0.5))
    table.update(_linear_rows(1, 0, 1.0, 0.4))
    table.update(_linear_rows(1, 1, 1.0, 0.8))
    table[(1, 2, 0, 1)] = S.Entry(0.5, 0.3)
    table.update(_linear_rows(1, 3, 3.0, 0.2))
    splittable = {(0, 0): (1,), (0, 1): (1,), (1, 0): (1,), (1, 1): (1,), (1, 3): (1,)}
    return [2, 4], table, splittable


def test_spatial_step_picks_the_largest_operator_after_the_largest_residue_and_a_matching_chunk():
    n_ops, table, splittable = _spatial_case()
    iv, starts, total = S.simulate(n_ops, table, {}, [[], []], 0.0)
    assert [(a, b) for (a, b, *_r) in iv] == [(0.0, 1.0), (1.0, 3.0), (3.0, 4.0), (4.0, 4.5), (4.5, 7.5)]
    assert [len(r[6]) for r in iv] == [2, 2, 1, 1, 1]                    # from t = 3 only model 1 has work: the tail
    split = S.spatial_step(n_ops, table, {}, [[], []], 0.0, splittable, _EXT8, max_moves=1)
    # largest residue outside the tail: [1,3], unused share .5.  Not started at t = 1: b1 (W*T .8), b2 (.15), b3 (.6); a1
    # (W*T 1.0, the largest of all) starts with the interval and is out.  b1's workload is .1 per batch element, so the
    # largest chunk that fits .5 holds 5 elements: list_B = [5, 3].
    assert split == {(1, 1): (1, [5, 3])}
    iv2, starts2, total2 = S.simulate(n_ops, table, split, [[], []], 0.0, _EXT8)
    assert abs(starts2[(1, 1, 0)] - 1.0) < 1e-12                         # the matching chunk is deployed in that residue
    assert total2 < total
    # further moves never raise the residue
    full = S.spatial_step(n_ops, table, {}, [[], []], 0.0, splittable, _EXT8)
    assert S.evaluate(n_ops, table, full, [[], []], 0.0, _EXT8) <= S.evaluate(n_ops, table, split, [[], []], 0.0, _EXT8) + 1e-12


def test_spatial_step_stays_inside_the_cluster():
    """Model 0 = [a0 (T 2, W .5)], model 1 = [b0 (T 1, W .8), b1 (T 1, W .9)], one pointer after the first operator of each:
    cluster 0 = {a0, b0}, cluster 1 = {b1}.  In cluster 0 b0 does not fit beside a0: residue .5 x 2 on [0,2].  b1 is the
    largest operator that follows, but it belongs to the next cluster and cannot be deployed here; b0 is decomposed, again
    with a chunk of 5 (workload .1 per element against an unused share of .5)."""
    table = {}
    table.update(_linear_rows(0, 0, 2.0, 0.5))
    table.update(_linear_rows(1, 0, 1.0, 0.8))
    table.update(_linear_rows(1, 1, 1.0, 0.9))
    splittable = {(0, 0): (1,), (1, 0): (1,), (1, 1): (1,)}
    split = S.spatial_step([1, 2], table, {}, [[1], [1]], 0.0, splittable, _EXT8, max_moves=1)
    assert split == {(1, 0): (1, [5, 3])}


def test_spatial_step_takes_the_axis_with_the_shorter_chunks():
    """Same as above with two axes for b0: along axis 2 its chunks take 1.5x as long, so axis 1 is taken; when axis 1 is
    the slow one, axis 2 is."""
    base = {}
    base.update(_linear_rows(0, 0, 2.0, 0.5))
    base.update(_linear_rows(1, 0, 1.0, 0.8, axes=(1, 2)))
    for slow, fast in ((2, 1), (1, 2)):
        table = dict(base)
        for f in (2, 4, 8):
            e = table[(1, 0, slow, f)]
            table[(1, 0, slow, f)] = S.Entry(e.T * 1.5, e.W)
        split = S.spatial_step([1, 1], table, {}, [[], []], 0.0, {(1, 0): (1, 2)}, _EXT8, max_moves=1)
        assert split == {(1, 0): (fast, [5, 3])}


def test_temporal_level_moves_a_pointer_to_the_smallest_residue_earliest_on_ties():
    """Model 0 = three operators (T 1, W .25), model 1 = one operator (T 1, W .25) held in the second cluster (P_1 = [0]),
    T_SW = 0.  Model 0's pointer at 0, 1 or 2 gives R = 2.0 each time (model 1's operator always overlaps one of model 0's),
    at 3 it gives 3.0: the tie goes to the earliest position, 0 -- not to the starting position 2."""
    table = {(0, i, 0, 1): S.Entry(1.0, 0.25) for i in range(3)}
    table[(1, 0, 0, 1)] = S.Entry(1.0, 0.25)
    R = [S.evaluate([3, 1], table, {}, [[p], [0]], 0.0) for p in range(4)]
    assert R == [2.0, 2.0, 2.0, 3.0]
    D = []
    P = S.temporal_level([3, 1], table, {}, [[2], [0]], 0.0, 1, D)
    assert P[0] == [0]
    assert len(D) == 4 + 2 and all(len(m) == 2 for _, m in D)             # every tried matrix is recorded with its residue


def test_temporal_level_finds_the_aligning_pointer():
    """Two models of two operators (T 1, W .25).  With model 1 cut after its first operator, model 0's pointer at 1 aligns
    the clusters (R = 1.0); at 0 or 2 one operator runs alone in its cluster (R = 2.0)."""
    table = {(n, i, 0, 1): S.Entry(1.0, 0.25) for n in range(2) for i in range(2)}
    assert [S.evaluate([2, 2], table, {}, [[p], [1]], 0.0) for p in range(3)] == [2.0, 1.0, 2.0]
    assert S.temporal_level([2, 2], table, {}, [[0], [1]], 0.0, 3, [])[0] == [1]


def test_second_pool_keeps_two_bandwidth_bound_operators_apart():
    """claim (2) of Section 4.4: two operators that fit the SM pool together (W .3 each) but each need .7 of the second
    pool cannot share a cycle; with .3 of it each they can.  The residue then counts both pools."""
    heavy = {(0, 0, 0, 1): S.Entry(1.0, 0.3, 0.7), (1, 0, 0, 1): S.Entry(1.0, 0.3, 0.7)}
    iv, _, total = S.simulate([1, 1], heavy, {}, [[], []], 0.0)
    assert total == 2.0 and [r[4] for r in iv] == [(0,), (1,)]
    assert abs(S.evaluate([1, 1], heavy, {}, [[], []], 0.0) - (2 * 0.7 + 2 * 0.3)) < 1e-12     # both pools, two cycles
    light = {(0, 0, 0, 1): S.Entry(1.0, 0.3, 0.3), (1, 0, 0, 1): S.Entry(1.0, 0.3, 0.3)}
    iv, _, total = S.simulate([1, 1], light, {}, [[], []], 0.0)
    assert total == 1.0 and iv[0][4] == (0, 1) and abs(iv[0][5] - 0.6) < 1e-12
    assert abs(S.evaluate([1, 1], light, {}, [[], []], 0.0) - (0.4 + 0.4)) < 1e-12
    # without second-pool shares in the table the residue is Eq. 8 on the SM pool alone
    plain = {k: S.Entry(e.T, e.W) for k, e in light.items()}
    assert abs(S.evaluate([1, 1], plain, {}, [[], []], 0.0) - 0.4) < 1e-12
    # a compute-bound and a bandwidth-bound operator pair up where two bandwidth-bound ones could not
    mixed = {(0, 0, 0, 1): S.Entry(1.0, 0.6, 0.1), (1, 0, 0, 1): S.Entry(1.0, 0.3, 0.8)}
    assert S.simulate([1, 1], mixed, {}, [[], []], 0.0)[2] == 1.0


def test_residue_closed_form_with_second_pool():
    rng = np.random.default_rng(7)
    for trial in range(20):
        n_ops = [int(rng.integers(1, 6)) for _ in range(int(rng.integers(1, 4)))]
        table, _ = _random_table(rng, n_ops)
        table = {k: S.Entry(e.T, e.W, float(rng.uniform(0.05, 0.9))) for k, e in table.items()}
        npnt = int(rng.integers(0, 3))
        P = [sorted(int(rng.integers(0, k + 1)) for _ in range(npnt)) for k in n_ops]
        iv, _, total = S.simulate(n_ops, table, {}, P, 0.07)
        work = sum(e.T * (e.W + e.Wb) for (n, i, a, f), e in table.items() if f == 1)
        closed = (S.S_GPU + S.S_BW) * (total - npnt * 0.07) - work + npnt * S.S_GPU * 0.07
        assert abs(S.residue(iv, npnt, 0.07, True) - closed) < 1e-9
        assert all((r[2] <= 1 + 1e-9 and r[5] <= 1 + 1e-9) or len(r[4]) == 1 for r in iv)
