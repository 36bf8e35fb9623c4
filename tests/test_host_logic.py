"""Host-side logic of the library through the C ABI, no GPU needed: exported symbols, descriptor
validation, plan validation, Matrix_P -> edges, and the host search against the oracle's search."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synth
from oracle import schedule as S
from paper_2304_11745_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KIND = {"conv": B.GACER_CONV2D, "dwconv": B.GACER_DWCONV2D, "gemm": B.GACER_GEMM, "bgemm_qk": B.GACER_BGEMM_QK,
        "bgemm_pv": B.GACER_BGEMM_PV, "maxpool": B.GACER_MAXPOOL, "gavgpool": B.GACER_GAVGPOOL,
        "affine": B.GACER_AFFINE_ACT, "add": B.GACER_ADD, "layernorm": B.GACER_LAYERNORM,
        "softmax": B.GACER_SOFTMAX, "act": B.GACER_ACT, "scale": B.GACER_SCALE, "concat": B.GACER_CONCAT,
        "avgpool": B.GACER_AVGPOOL}
ACT = {"none": 0, "relu": 1, "relu6": 2, "gelu": 3, "hswish": 4, "hsigmoid": 5}
FAKE = 0x10000      # 16-byte aligned, never dereferenced: nothing is launched in these tests


def descriptors(tenants, mutate=None):
    keep = []
    descs = (B.gacer_tenant * len(tenants))()
    for ti, t in enumerate(tenants):
        esz = 2 if t.dtype == "bf16" else 4
        views = getattr(t, "views", {})
        tens = (B.gacer_tensor * len(t.tensors))(*[
            B.gacer_tensor(n, c, h, w, FAKE + views[i][1] * esz, t.tensors[views[i][0]][1], views[i][0], views[i][1]) if i in views
            else B.gacer_tensor(n, c, h, w, FAKE) for i, (n, c, h, w) in enumerate(t.tensors)])
        ops = (B.gacer_op * len(t.ops))()
        for i, op in enumerate(t.ops):
            p = lambda idx: FAKE if idx >= 0 else None
            ops[i] = B.gacer_op(KIND[op.kind], op.in0, op.in1, op.res, op.out, p(op.w), p(op.bias), p(op.scale), p(op.shift),
                                op.cin, op.cout, op.kh, op.kw, op.stride, op.pad, op.groups, ACT[op.act],
                                op.eps if op.kind == "layernorm" else op.alpha)
        descs[ti] = B.gacer_tenant(len(t.ops), ops, len(t.tensors), tens, t.input, t.output,
                                   1 if t.dtype == "bf16" else 0, t.batch, None)
        keep += [tens, ops]
    if mutate:
        mutate(descs)
    return descs, keep


@pytest.fixture()
def ctx():
    c = C.c_void_p()
    assert B.gacer_create(C.byref(c)) == B.GACER_OK
    yield c
    B.gacer_destroy(c)


def load(ctx, tenants, mutate=None):
    d, keep = descriptors(tenants, mutate)
    return B.gacer_load_tenants(ctx, d, len(tenants)), keep


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "gacer.h")).read()
    declared = set(re.findall(r"\b(gacer_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name


def test_state_and_argument_errors(ctx):
    assert B.gacer_run(ctx, 0, 1, None) == B.GACER_ESTATE
    assert B.gacer_set_plan(ctx, None) == B.GACER_ESTATE
    assert b"before" in B.gacer_last_error(ctx)
    assert B.gacer_load_tenants(ctx, None, 1) == B.GACER_EINVAL
    assert B.gacer_create(None) == B.GACER_EINVAL
    B.gacer_destroy(None)


@pytest.mark.parametrize("config", sorted(synth.CONFIG_NAMES))
def test_all_configs_load_and_count_launches(ctx, config):
    tenants, _ = synth.build_config(config, "full", with_data=False)
    st, keep = load(ctx, tenants)
    assert st == B.GACER_OK, B.gacer_last_error(ctx)
    n = C.c_int()
    assert B.gacer_set_fuse_affine(ctx, 0) == B.GACER_OK
    assert B.gacer_launch_count(ctx, B.GACER_MODE_SEQUENTIAL, C.byref(n)) == B.GACER_OK
    assert n.value == sum(len(t.ops) for t in tenants)
    # launch fusion: a per-channel affine followed by the 1x1 convolution that reads it is one launch, unless its channel
    # count is not a multiple of a 16-byte vector
    def fused_pairs(t):
        vec, k = (8 if t.dtype == "bf16" else 4), 0
        for a, b in zip(t.ops, t.ops[1:]):
            if (a.kind == "affine" and a.res < 0 and a.act in ("none", "relu", "relu6") and b.kind == "conv" and b.kh == 1 and
                    b.stride == 1 and b.pad == 0 and b.in0 == a.out and t.tensors[a.out][1] % vec == 0):
                k += 1
        return k
    assert B.gacer_set_fuse_affine(ctx, 1) == B.GACER_OK
    assert B.gacer_launch_count(ctx, B.GACER_MODE_SEQUENTIAL, C.byref(n)) == B.GACER_OK
    assert n.value == sum(len(t.ops) - fused_pairs(t) for t in tenants)
    if config == 8:
        assert sum(fused_pairs(t) for t in tenants) == 61           # DenseNet-121: 58 dense layers and 3 transitions


def test_shape_validation(ctx):
    tenants = [synth.small_resnet("f32", 2)]

    def bad_cout(d):
        d[0].ops[0].cout += 1
    st, _ = load(ctx, tenants, bad_cout)
    assert st == B.GACER_ESHAPE and b"tenant 0 op 0" in B.gacer_last_error(ctx)

    def bad_order(d):
        d[0].ops[1].in0 = d[0].ops[3].out          # reads a tensor that is written later
    st, _ = load(ctx, tenants, bad_order)
    assert st == B.GACER_ESHAPE

    def misaligned(d):
        d[0].tensors[1].dptr = FAKE + 4
    st, _ = load(ctx, tenants, misaligned)
    assert st == B.GACER_EINVAL

    def null_w(d):
        d[0].ops[0].w = None
    st, _ = load(ctx, tenants, null_w)
    assert st == B.GACER_EINVAL
    st, _ = load(ctx, tenants)
    assert st == B.GACER_OK


def test_shape_validation_of_gate_concat_and_mean_pool(ctx):
    """Squeeze-and-excitation gate, channel concatenation, unpadded mean pooling: each shape rule rejects its violation."""
    from synth import graphs as G
    copying_densenet = lambda dtype, batch: G._densenet("copies", dtype, batch, 40, 8, [2, 3], 12, 2, 10, in_place=False)
    for maker, kind in ((synth.small_mbv3, "scale"), (copying_densenet, "concat"), (synth.small_densenet, "avgpool")):
        tenants = [maker("f32", 2)]
        k = next(i for i, op in enumerate(tenants[0].ops) if op.kind == kind)
        st, _ = load(ctx, tenants)
        assert st == B.GACER_OK, B.gacer_last_error(ctx)

        def wrong_second_input(d):
            d[0].ops[k].in1 = d[0].ops[k].in0     # a gate must be (n,c,1,1); a concatenation's channels must add up
        def no_second_input(d):
            d[0].ops[k].in1 = -1
        def padded(d):
            d[0].ops[k].pad = 1
        def wrong_cin(d):
            d[0].ops[k].cin += 1
        for bad in {"scale": (wrong_second_input, no_second_input), "concat": (wrong_second_input, no_second_input, wrong_cin),
                    "avgpool": (padded,)}[kind]:
            st, _ = load(ctx, tenants, bad)
            assert st == B.GACER_ESHAPE and b"tenant 0 op %d" % k in B.gacer_last_error(ctx), (kind, bad.__name__)

    def unknown_act(d):
        d[0].ops[0].act = 6
    st, _ = load(ctx, [synth.small_mbv3("f32", 2)], unknown_act)
    assert st == B.GACER_EINVAL


def test_channel_window_validation(ctx):
    """Tensors that are channel windows of a wider tensor: every rule of the declaration rejects its violation."""
    t = synth.small_densenet("f32", 2)
    assert t.views
    st, _ = load(ctx, [t])
    assert st == B.GACER_OK, B.gacer_last_error(ctx)
    first_slot = next(i for i, (base, off) in sorted(t.views.items()) if off > 0)        # a layer's output window
    prefix = next(i for i, (base, off) in sorted(t.views.items()) if off == 0 and i > first_slot)
    base = t.views[first_slot][0]
    reader = next(k for k, op in enumerate(t.ops) if op.in0 == prefix)
    writer = next(k for k, op in enumerate(t.ops) if op.out == first_slot)

    def leaves_base(d):
        d[0].tensors[first_slot].c_off = t.tensors[base][1] - 1
    def wrong_pointer(d):
        d[0].tensors[first_slot].dptr = FAKE
    def wrong_pitch(d):
        d[0].tensors[first_slot].pitch += 4
    def window_of_a_window(d):
        d[0].tensors[first_slot].base = prefix
    def overlapping(d):                               # the layer's window moved onto channels the pool has already written
        d[0].tensors[first_slot].c_off = 0
        d[0].tensors[first_slot].dptr = FAKE
    def read_too_early(d):                            # the prefix reader moved in front of the layer that completes the prefix
        d[0].ops[writer - 1].in0 = prefix
    def unsupported_reader(d):                        # global pooling takes no position pitch
        d[0].ops[reader].kind = B.GACER_GAVGPOOL
    def residual_into_window(d):
        d[0].ops[writer].res = d[0].ops[writer].in0
    for bad, status in ((leaves_base, B.GACER_ESHAPE), (wrong_pointer, B.GACER_EINVAL), (wrong_pitch, B.GACER_ESHAPE),
                        (window_of_a_window, B.GACER_ESHAPE), (overlapping, B.GACER_ESHAPE), (read_too_early, B.GACER_ESHAPE),
                        (unsupported_reader, B.GACER_ESHAPE), (residual_into_window, B.GACER_ESHAPE)):
        st, _ = load(ctx, [t], bad)
        assert st == status, (bad.__name__, st, B.gacer_last_error(ctx))


def _plan(splits=(), syncs=()):
    sp = (B.gacer_split * max(1, len(splits)))(*[B.gacer_split(*s) for s in splits])
    sy = (B.gacer_sync * max(1, len(syncs)))(*[B.gacer_sync(*s) for s in syncs])
    return B.gacer_plan(len(splits), sp, len(syncs), sy), (sp, sy)


def test_plan_validation(ctx):
    tenants = [synth.small_resnet("f32", 3), synth.small_bert("f32", 3)]
    st, keep = load(ctx, tenants)
    assert st == B.GACER_OK
    ln = next(i for i, op in enumerate(tenants[1].ops) if op.kind == "layernorm")
    bad = [
        [(0, 0, B.GACER_AXIS_COUT, 3)],                                   # factor not in {1,2,4,8}
        [(0, 0, B.GACER_AXIS_BATCH, 4)],                                  # factor > batch (3)
        [(1, ln, B.GACER_AXIS_COUT, 2)],                                  # layernorm cannot split on channels
        [(0, 0, B.GACER_AXIS_COUT, 2), (0, 0, B.GACER_AXIS_BATCH, 2)],    # listed twice
        [(0, 99, B.GACER_AXIS_BATCH, 2)],                                 # missing operator
        [(0, 0, B.GACER_AXIS_NONE, 2)],                                   # factor > 1 without an axis
    ]
    for sp in bad:
        plan, k = _plan(sp)
        assert B.gacer_set_plan(ctx, C.byref(plan)) == B.GACER_EPLAN, sp
    for sy in ([(0, 1, 0, 3)], [(0, 99, 1, 0)], [(0, 3, 1, 1), (1, 2, 0, 2)]):   # same tenant; missing; cycle
        plan, k = _plan((), sy)
        assert B.gacer_set_plan(ctx, C.byref(plan)) == B.GACER_EPLAN, sy
    assert b"cycle" in B.gacer_last_error(ctx)
    plan, k = _plan([(0, 0, B.GACER_AXIS_COUT, 2), (0, 1, B.GACER_AXIS_BATCH, 2)], [(0, 3, 1, 1), (1, 0, 0, 2)])
    assert B.gacer_set_plan(ctx, C.byref(plan)) == B.GACER_OK
    n = C.c_int()
    B.gacer_launch_count(ctx, B.GACER_MODE_PLAN, C.byref(n))
    assert n.value == sum(len(t.ops) for t in tenants) + 2          # two operators became two chunks each
    assert B.gacer_set_plan(ctx, None) == B.GACER_OK


def test_chunk_list_validation(ctx):
    """list_B of Section 4.2: explicit chunk sizes must be positive, at most 8, and sum to the axis extent (Eq. 5)."""
    tenants = [synth.small_resnet("f32", 6), synth.small_bert("f32", 3)]
    st, keep = load(ctx, tenants)
    assert st == B.GACER_OK
    cout0 = tenants[0].ops[0].cout

    def split(t, o, axis, sizes):
        arr = (C.c_int * len(sizes))(*sizes)
        return B.gacer_split(t, o, axis, len(sizes), arr), arr

    def set_plan(rows):
        sp = (B.gacer_split * len(rows))(*[r[0] for r in rows])
        plan = B.gacer_plan(len(rows), sp, 0, None)
        return B.gacer_set_plan(ctx, C.byref(plan))

    bad = [
        [split(0, 0, B.GACER_AXIS_BATCH, [4, 1])],                        # sums to 5, batch is 6
        [split(0, 0, B.GACER_AXIS_BATCH, [6, 0])],                        # empty chunk
        [split(0, 0, B.GACER_AXIS_BATCH, [7, -1])],                       # negative size
        [split(0, 0, B.GACER_AXIS_COUT, [1] * 9)],                        # more than 8 chunks
        [split(0, 0, B.GACER_AXIS_COUT, [cout0 - 1, 2])],                 # sums past the extent
        [split(0, 0, B.GACER_AXIS_NONE, [5, 1])],                         # chunks need an axis
    ]
    for rows in bad:
        assert set_plan(rows) == B.GACER_EPLAN, [list(r[1]) for r in rows]
    good = [split(0, 0, B.GACER_AXIS_BATCH, [5, 1]), split(0, 1, B.GACER_AXIS_COUT, [cout0 - 3, 2, 1]),
            split(1, 0, B.GACER_AXIS_BATCH, [3])]                        # a single chunk is the unsplit operator
    assert set_plan(good) == B.GACER_OK
    n = C.c_int()
    B.gacer_launch_count(ctx, B.GACER_MODE_PLAN, C.byref(n))
    assert n.value == sum(len(t.ops) for t in tenants) + 1 + 2
    for r in good:                                                        # the library copied the lists
        for j in range(len(r[1])):
            r[1][j] = 0
    B.gacer_launch_count(ctx, B.GACER_MODE_PLAN, C.byref(n))
    assert n.value == sum(len(t.ops) for t in tenants) + 3
    assert B.gacer_set_plan(ctx, None) == B.GACER_OK


def test_probe_stream_queues_rejects_bad_arguments():
    grp = (C.c_int * 4)()
    arr = (C.c_void_p * 4)()
    assert B.gacer_probe_stream_queues(None, 4, grp) == B.GACER_EINVAL
    assert B.gacer_probe_stream_queues(arr, 4, None) == B.GACER_EINVAL
    assert B.gacer_probe_stream_queues(arr, 0, grp) == B.GACER_EINVAL
    assert B.gacer_probe_stream_queues(arr, 65, grp) == B.GACER_EINVAL


def _edges(ctx, matrix_P):
    n_ptr = len(matrix_P[0])
    flat = (C.c_int * max(1, len(matrix_P) * n_ptr))(*[p for P in matrix_P for p in P])
    out = C.POINTER(B.gacer_plan)()
    st = B.gacer_plan_from_pointers(ctx, flat, n_ptr, C.byref(out))
    if st != B.GACER_OK:
        return st, None
    e = [(out.contents.sync[i].src_tenant, out.contents.sync[i].src_op, out.contents.sync[i].dst_tenant,
          out.contents.sync[i].dst_op, out.contents.sync[i].when) for i in range(out.contents.n_sync)]
    B.gacer_plan_free(out)
    return st, e


def _check_cluster_order(n_ops, matrix_P, edges):
    """The edges must order the first operator of every model's cluster k+1 behind the last operator of every
    other model's clusters <= k (Eq. 6: clusters run one after another).  Checked by reachability over
    (model, op, start|end) nodes: stream order, when-0 edges end->start, when-1 edges start->start."""
    succ = {}

    def add(a, b):
        succ.setdefault(a, set()).add(b)
    for n, k in enumerate(n_ops):
        for i in range(k):
            add((n, i, "s"), (n, i, "e"))
            if i + 1 < k:
                add((n, i, "e"), (n, i + 1, "s"))
    for (st_, so, dt_, do, when) in edges:
        add((st_, so, "e" if when == 0 else "s"), (dt_, do, "s"))
        if when == 1:                      # the hub's release also carries everything the hub waited for
            pass

    def reach(a, b):
        seen, todo = {a}, [a]
        while todo:
            x = todo.pop()
            if x == b:
                return True
            for y in succ.get(x, ()):
                if y not in seen:
                    seen.add(y)
                    todo.append(y)
        return False
    # a when-1 edge releases dst once src's predecessors are done: model it by linking src's predecessors' ends
    for (st_, so, dt_, do, when) in edges:
        if when == 1:
            if so > 0:
                add((st_, so - 1, "e"), (dt_, do, "s"))
            for (a, ao, b, bo, w2) in edges:
                if w2 == 0 and b == st_ and bo == so:
                    add((a, ao, "e"), (dt_, do, "s"))
    cl = S.clusters(n_ops, matrix_P)
    N = len(n_ops)
    for k in range(len(cl) - 1):
        for src in range(N):
            done = [o for kk in range(k + 1) for o in cl[kk][src]]
            for dst in range(N):
                nxt = [o for kk in range(k + 1, len(cl)) for o in cl[kk][dst]]
                if src != dst and done and nxt:
                    assert reach((src, done[-1] - 1, "e"), (dst, nxt[0] - 1, "s")), (k, src, dst, edges)


def test_pointers_to_edges_follow_the_worked_example(ctx):
    """Eq. 6 / Eq. 7: M_1 with 12 operators and P_1=(2,8); M_2 with 8 operators and an empty first segment."""
    a, b = synth.graphs._B("m1", "f32", 1), synth.graphs._B("m2", "f32", 1)
    for bld, n in ((a, 12), (b, 8)):
        x = y = bld.tensor(1, 8, 4, 4)
        for _ in range(n):
            y = bld.act(y, "relu")
        bld.done(x, y)
    st, keep = load(ctx, [a.t, b.t])
    assert st == B.GACER_OK
    st, edges = _edges(ctx, [[2, 8], [0, 4]])
    assert st == B.GACER_OK
    _check_cluster_order([12, 8], [[2, 8], [0, 4]], edges)
    assert len(edges) <= 2 * 2 * (2 - 1)                       # hub barriers: at most 2(N-1) edges per pointer
    plan, k = _plan((), edges)
    assert B.gacer_set_plan(ctx, C.byref(plan)) == B.GACER_OK
    assert _edges(ctx, [[8, 2], [0, 4]])[0] == B.GACER_EPLAN
    assert _edges(ctx, [[2, 13], [0, 4]])[0] == B.GACER_EPLAN


def test_hub_barriers_order_every_cluster(ctx):
    rng = np.random.default_rng(4)
    for trial in range(20):
        n_ops = [int(rng.integers(1, 9)) for _ in range(int(rng.integers(2, 6)))]
        st, keep = load(ctx, _chain_tenants(n_ops))
        assert st == B.GACER_OK
        npnt = int(rng.integers(1, 4))
        P = [sorted(int(rng.integers(0, k + 1)) for _ in range(npnt)) for k in n_ops]
        st, edges = _edges(ctx, P)
        assert st == B.GACER_OK
        _check_cluster_order(n_ops, P, edges)
        assert len(edges) <= 2 * npnt * (len(n_ops) - 1)
        plan, k = _plan((), edges)
        assert B.gacer_set_plan(ctx, C.byref(plan)) == B.GACER_OK, B.gacer_last_error(ctx)


def _chain_tenants(n_ops):
    out = []
    for k, n in enumerate(n_ops):
        b = synth.graphs._B(f"m{k}", "f32", 8)
        x = y = b.tensor(8, 16, 6, 6)
        for _ in range(n):
            y = b.conv(y, 16, 3, 1, 1, "relu")
        out.append(b.done(x, y))
    return out


def _table_rows(rng, n_ops, wmax=1.0, second_pool=False):
    """random lookup table (float32 values, as the C struct holds them); chain tenants: batch 8, 16 output channels"""
    rows, table, splittable = [], {}, {}
    for n, k in enumerate(n_ops):
        for i in range(k):
            T, W = float(np.float32(rng.uniform(0.1, 2.0))), float(np.float32(rng.uniform(0.05, wmax)))
            Wb = float(np.float32(rng.uniform(0.05, 0.9))) if second_pool else 0.0
            rows.append((n, i, 0, 1, T, W, Wb))
            axes = (1, 2) if rng.random() < 0.7 else ((1,) if rng.random() < 0.5 else ())
            if axes:
                splittable[(n, i)] = axes
            for a in axes:
                for f in (2, 4, 8):
                    rows.append((n, i, a, f, float(np.float32(T / f * rng.uniform(1.0, 1.3))), float(np.float32(max(0.02, W / f))),
                                 float(np.float32(Wb * rng.uniform(0.7, 1.0)))))
    for (n, i, a, f, T, W, Wb) in rows:
        table[(n, i, a, f)] = S.Entry(T, W, Wb)
    return rows, table, splittable


def _chain_extent(n, i, axis):
    return 8 if axis == 1 else 16


def _prof(rows, t_sw):
    arr = (B.gacer_prof * (len(rows) + 1))()
    for k, (n, i, a, f, T, W, Wb) in enumerate(rows):
        arr[k] = B.gacer_prof(n, i, a, f, T, 0, W, Wb)
    arr[len(rows)] = B.gacer_prof(-1, -1, 0, 1, t_sw, 0, 1.0, 0.0)
    return arr


@pytest.mark.parametrize("second_pool", [False, True], ids=["one-pool", "two-pools"])
def test_model_residue_and_search_match_the_oracle(ctx, second_pool):
    rng = np.random.default_rng(12 if second_pool else 11)
    for trial in range(8):
        n_ops = [int(rng.integers(2, 7)) for _ in range(int(rng.integers(2, 4)))]
        st, keep = load(ctx, _chain_tenants(n_ops))
        assert st == B.GACER_OK, B.gacer_last_error(ctx)
        rows, table, splittable = _table_rows(rng, n_ops, second_pool=second_pool)
        t_sw = float(np.float32(0.03))
        prof = _prof(rows, t_sw)
        # (1) residue model on an explicit plan: even decompositions and chunk lists
        npnt = int(rng.integers(0, 3))
        P = [sorted(int(rng.integers(0, k + 1)) for _ in range(npnt)) for k in n_ops]
        split, keep_sizes, sp_rows = {}, [], []
        for key, axes in splittable.items():
            r = rng.random()
            if r < 0.35:
                split[key] = (axes[0], 2)
                sp_rows.append(B.gacer_split(key[0], key[1], axes[0], 2, None))
            elif r < 0.7:
                E = _chain_extent(key[0], key[1], axes[-1])
                b = int(rng.integers(1, E))
                split[key] = (axes[-1], [b, E - b])
                arr = (C.c_int * 2)(b, E - b)
                keep_sizes.append(arr)
                sp_rows.append(B.gacer_split(key[0], key[1], axes[-1], 2, arr))
        sp = (B.gacer_split * max(1, len(sp_rows)))(*sp_rows)
        flat = (C.c_int * max(1, len(n_ops) * npnt))(*[p for row in P for p in row])
        R, mk = C.c_double(), C.c_double()
        assert B.gacer_model_residue(ctx, prof, len(prof), sp, len(sp_rows), flat, npnt, C.byref(R), C.byref(mk)) == B.GACER_OK, \
            B.gacer_last_error(ctx)
        iv, _, total = S.simulate(n_ops, table, split, P, t_sw, _chain_extent)
        assert abs(R.value - S.residue(iv, npnt, t_sw, second_pool)) < 1e-9 and abs(mk.value - total) < 1e-9
        # (2) the search itself: same decisions as the step-by-step oracle
        o_split, o_P, o_R, _ = S.search(n_ops, table, t_sw, splittable, _chain_extent, rounds=20, max_pointers=8)
        out = C.POINTER(B.gacer_plan)()
        ptrs = (C.c_int * (8 * len(n_ops)))()
        n_ptr, Rs = C.c_int(), C.c_double()
        assert B.gacer_search(ctx, prof, len(prof), 20, C.byref(out), ptrs, C.byref(n_ptr), C.byref(Rs)) == B.GACER_OK
        assert abs(Rs.value - o_R) < 1e-9
        got_P = [[ptrs[t * n_ptr.value + j] for j in range(n_ptr.value)] for t in range(len(n_ops))]
        assert got_P == [list(p) for p in o_P]
        got_split = {}
        for k in range(out.contents.n_split):
            s_ = out.contents.split[k]
            got_split[(s_.tenant, s_.op)] = (s_.axis, [s_.sizes[j] for j in range(s_.factor)])
        assert got_split == {k: (a, list(f)) for k, (a, f) in o_split.items()}
        # the returned plan is installable
        assert B.gacer_set_plan(ctx, out) == B.GACER_OK, B.gacer_last_error(ctx)
        B.gacer_plan_free(out)


def test_capture_refuses_a_ring_of_three_tenants(ctx):
    """On a HIP runtime older than 7.2, capturing a plan whose edges close a ring of three or more tenants must be refused
    before anything is enqueued; hub-shaped barriers (mutual pairs with one hub) pass that check (and then fail later here
    for lack of a GPU, with a different status)."""
    tenants = [synth.toy_mlp("f32", 4), synth.toy_mlp("f32", 4), synth.toy_mlp("f32", 4)]
    st, keep = load(ctx, tenants)
    assert st == B.GACER_OK
    ring, k1 = _plan([], [(0, 0, 1, 1, 0), (1, 0, 2, 1, 0), (2, 0, 0, 1, 0)])       # 1 waits on 0, 2 on 1, 0 on 2: single waits only
    assert B.gacer_set_plan(ctx, C.byref(ring)) == B.GACER_OK
    st = B.gacer_capture(ctx, B.GACER_MODE_PLAN)
    import torch
    old_runtime = torch.version.hip is not None and tuple(int(v) for v in torch.version.hip.split(".")[:2]) < (7, 2)
    if old_runtime:
        assert st == B.GACER_EPLAN and b"ring" in B.gacer_last_error(ctx)
    flat = (C.c_int * 3)(1, 1, 1)
    out = C.POINTER(B.gacer_plan)()
    assert B.gacer_plan_from_pointers(ctx, flat, 1, C.byref(out)) == B.GACER_OK
    assert B.gacer_set_plan(ctx, out) == B.GACER_OK
    B.gacer_plan_free(out)
    assert B.gacer_capture(ctx, B.GACER_MODE_PLAN) != B.GACER_EPLAN                 # a star around tenant 0 is no ring


def test_run_static_rejects_more_workspace_than_it_holds(ctx):
    """The allocation-free entry point has a fixed 32 MiB workspace: tenants that need more are refused with the need in
    the message, before anything touches the GPU; tenants that fit get past that check (and stop here for lack of a GPU)."""
    from synth import graphs as G

    def sliced(batch):
        b = G._B("sliced", "f32", batch)
        x = b.tensor(batch, 512, 7, 7)
        return b.done(x, b.conv(x, 512, 3, 1, 1, "relu"))            # 7x7 rows, K = 4608: cut into many slices
    st, keep = load(ctx, [sliced(8)] * 12)
    assert st == B.GACER_OK
    assert B.gacer_run_static(ctx, B.GACER_MODE_STREAM_PARALLEL, 1) == B.GACER_ENOMEM
    msg = B.gacer_last_error(ctx).decode()
    assert "static workspace holds 33554432" in msg and "need" in msg
    st, keep = load(ctx, [sliced(8)])
    assert st == B.GACER_OK
    assert B.gacer_run_static(ctx, B.GACER_MODE_STREAM_PARALLEL, 1) in (B.GACER_ESTATE, B.GACER_EHIP)
    assert B.gacer_run_static(ctx, 7, 1) == B.GACER_EINVAL and B.gacer_run_static(None, 0, 1) == B.GACER_EINVAL


def test_sibling_flag_in_plans(ctx):
    """gacer_split.sibling is accepted on any decomposition and changes neither the launch count nor validation."""
    tenants = [synth.small_resnet("f32", 4), synth.small_mbv2("f32", 4)]
    st, keep = load(ctx, tenants)
    assert st == B.GACER_OK
    arr = (C.c_int * 2)(3, 1)
    sp = (B.gacer_split * 2)(B.gacer_split(0, 0, B.GACER_AXIS_BATCH, 2, arr, 1), B.gacer_split(1, 2, B.GACER_AXIS_COUT, 2, None, 1))
    plan = B.gacer_plan(2, sp, 0, None)
    assert B.gacer_set_plan(ctx, C.byref(plan)) == B.GACER_OK, B.gacer_last_error(ctx)
    n = C.c_int()
    B.gacer_launch_count(ctx, B.GACER_MODE_PLAN, C.byref(n))
    assert n.value == sum(len(t.ops) for t in tenants) + 2
    bad = (B.gacer_split * 1)(B.gacer_split(0, 0, B.GACER_AXIS_BATCH, 8, None, 1))              # factor > batch, sibling or not
    plan = B.gacer_plan(1, bad, 0, None)
    assert B.gacer_set_plan(ctx, C.byref(plan)) == B.GACER_EPLAN


def test_plan_text_round_trip(ctx):
    """Offline deployment (Section 4.4): a plan survives being written out and read back, chunk lists, sibling flags and
    hub edges included, and the parsed plan installs; malformed text is refused."""
    tenants = [synth.small_resnet("f32", 6), synth.small_mbv2("f32", 4)]
    st, keep = load(ctx, tenants)
    assert st == B.GACER_OK
    flat = (C.c_int * 4)(2, 5, 3, 9)
    edges = C.POINTER(B.gacer_plan)()
    assert B.gacer_plan_from_pointers(ctx, flat, 2, C.byref(edges)) == B.GACER_OK
    sizes = (C.c_int * 3)(3, 2, 1)
    sp = (B.gacer_split * 3)(B.gacer_split(0, 0, B.GACER_AXIS_BATCH, 3, sizes, 1), B.gacer_split(0, 2, B.GACER_AXIS_COUT, 2, None, 0),
                             B.gacer_split(1, 1, B.GACER_AXIS_BATCH, 4, None, 1))
    plan = B.gacer_plan(3, sp, edges.contents.n_sync, edges.contents.sync)
    n = C.c_size_t()
    assert B.gacer_plan_to_text(C.byref(plan), None, 0, C.byref(n)) == B.GACER_OK and n.value > 20
    buf = C.create_string_buffer(n.value)
    assert B.gacer_plan_to_text(C.byref(plan), buf, n.value - 1, C.byref(n)) == B.GACER_EINVAL        # too small
    assert B.gacer_plan_to_text(C.byref(plan), buf, n.value, C.byref(n)) == B.GACER_OK
    text = buf.value.decode()
    assert text.splitlines()[0] == "gacer-plan 1" and "split 0 0 1 3 1 3 2 1" in text.splitlines()
    back = C.POINTER(B.gacer_plan)()
    assert B.gacer_plan_from_text(buf.value, C.byref(back)) == B.GACER_OK
    b = back.contents
    assert b.n_split == 3 and b.n_sync == plan.n_sync
    assert [b.split[0].sizes[j] for j in range(3)] == [3, 2, 1] and b.split[0].sibling == 1 and not b.split[1].sizes
    assert [(b.split[k].tenant, b.split[k].op, b.split[k].axis, b.split[k].factor, b.split[k].sibling) for k in range(3)] == \
        [(0, 0, 1, 3, 1), (0, 2, 2, 2, 0), (1, 1, 1, 4, 1)]
    for k in range(plan.n_sync):
        assert tuple(getattr(b.sync[k], f) for f in ("src_tenant", "src_op", "dst_tenant", "dst_op", "when")) == \
            tuple(getattr(plan.sync[k], f) for f in ("src_tenant", "src_op", "dst_tenant", "dst_op", "when"))
    assert B.gacer_set_plan(ctx, back) == B.GACER_OK, B.gacer_last_error(ctx)
    buf2 = C.create_string_buffer(n.value)
    assert B.gacer_plan_to_text(back, buf2, n.value, C.byref(n)) == B.GACER_OK and buf2.value == buf.value
    B.gacer_plan_free(back)
    B.gacer_plan_free(edges)
    for bad in (b"", b"split 0 0 1 2 0\n", b"gacer-plan 2\n", b"gacer-plan 1\nsplit 0 0 1 2\n", b"gacer-plan 1\nsplit 0 0 1 3 0 2 1\n",
                b"gacer-plan 1\nsync 0 1 1 0\n", b"gacer-plan 1\nsplit 0 0 7 2 0\n", b"gacer-plan 1\nhello\n", b"gacer-plan 1\nsplit 0 0 1 2 0 4 x\n"):
        out = C.POINTER(B.gacer_plan)()
        assert B.gacer_plan_from_text(bad, C.byref(out)) == B.GACER_EPLAN, bad
    empty = C.POINTER(B.gacer_plan)()
    assert B.gacer_plan_from_text(b"gacer-plan 1\n", C.byref(empty)) == B.GACER_OK and empty.contents.n_split == 0
    B.gacer_plan_free(empty)
