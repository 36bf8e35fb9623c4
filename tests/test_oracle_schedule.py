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
        work = sum(T * W for n, k in enumerate(n_ops) for i in range(k) for (T, W) in S.chunk_list(table, n, i, split))
        closed = S.S_GPU * (total - npnt * T_SW) - work + npnt * S.S_GPU * T_SW
        assert abs(S.residue(iv, npnt, T_SW) - closed) < 1e-9
        assert all(u <= S.S_GPU + 1e-9 or len(r) == 1 for (_, _, u, _, r) in iv)   # Eq. 1 constraint
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


def _brute_force(n_ops, table, splittable, T_SW, max_ptr=1):
    best = None
    keys = sorted(splittable)
    choices = []
    for k in keys:
        c = [(0, 1)]
        for a in splittable[k]:
            c.append((a, 2))
        choices.append(c)
    for combo in itertools.product(*choices):
        split = {k: v for k, v in zip(keys, combo) if v[1] > 1}
        for npnt in range(max_ptr + 1):
            for Ps in itertools.product(*[itertools.combinations_with_replacement(range(k + 1), npnt) for k in n_ops]):
                R = S.evaluate(n_ops, table, split, [list(P) for P in Ps], T_SW)
                if best is None or R < best:
                    best = R
    return best


def test_search_against_brute_force():
    rng = np.random.default_rng(3)
    for trial in range(12):
        n_ops = [int(rng.integers(2, 5)), int(rng.integers(2, 5))]
        table, splittable = _random_table(rng, n_ops)
        T_SW = 0.05
        # restrict to factor 2 so brute force enumerates the same space
        table = {k: v for k, v in table.items() if k[3] <= 2}
        R_none = S.evaluate(n_ops, table, {}, [[], []], T_SW)
        split, P, R, D = S.search(n_ops, table, T_SW, splittable, rounds=10, max_pointers=1)
        opt = _brute_force(n_ops, table, splittable, T_SW, 1)
        assert opt - 1e-9 <= R <= R_none + 1e-9
        assert abs(S.evaluate(n_ops, table, split, P, T_SW) - R) < 1e-12
        assert len(set(len(p) for p in P)) == 1
        assert all(r >= opt - 1e-9 for r, _ in D)


def test_search_stops_adding_pointers_when_sync_is_expensive():
    rng = np.random.default_rng(5)
    n_ops = [6, 5, 4]
    table, splittable = _random_table(rng, n_ops)
    _, P_cheap, _, _ = S.search(n_ops, table, 0.0, splittable, rounds=5, max_pointers=4)
    _, P_dear, R_dear, _ = S.search(n_ops, table, 100.0, splittable, rounds=5, max_pointers=4)
    assert len(P_dear[0]) == 0 and len(P_cheap[0]) >= len(P_dear[0])
