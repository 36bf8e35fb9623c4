"""GPU checks of the regulation machinery itself, through the C ABI: temporal ordering of clusters (Section 4.3, Eq. 6)
observed on the device clock, the lookup table of Section 4.1 (gacer_profile), and a searched plan (Section 4.4,
Algorithm 1) installed and run end to end."""
import ctypes as C

import numpy as np
import pytest

import synth
from parity import TOL, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2304_11745_amd import harness
    return harness


def _cluster_of(n_ops, P):
    """cluster index of every operator of a tenant with pointer list P (value p cuts after the p-th operator)."""
    out, k = [], 0
    for i in range(n_ops):
        while k < len(P) and i >= P[k]:
            k += 1
        out.append(k)
    return out


def _cluster_windows(rows, clusters):
    """per cluster: (earliest kernel begin, latest kernel end) over all tenants, from a trace of one round."""
    win = {}
    for r in rows:
        k = clusters[r["tenant"]][r["op"]]
        lo, hi = win.get(k, (float("inf"), float("-inf")))
        win[k] = (min(lo, r["start_ms"]), max(hi, r["end_ms"]))
    return win


@pytest.mark.parametrize("config", [3, 4])
@pytest.mark.parametrize("threads", [False, True], ids=["one-thread", "thread-per-tenant"])
def test_clusters_run_one_after_another(gpu, config, threads):
    """Eq. 6: with pointers installed, every kernel of cluster k+1 (of any tenant) begins only after every kernel of
    cluster k (of every tenant) has ended.  Kernel begin / end are read on the device clock.  The same windows taken
    without edges overlap, which shows that the measurement would see a missing barrier."""
    from paper_2304_11745_amd import binding as B
    tenants, data = synth.build_config(config, "small")
    sess = gpu.Session(tenants, data)
    n_ops = [len(t.ops) for t in tenants]
    P = [[n // 3, (2 * n) // 3] for n in n_ops]
    P[-1] = [0, n_ops[-1] // 2]                      # one tenant with an empty first segment (the [None] entry of Eq. 6)
    clusters = [_cluster_of(n, p) for n, p in zip(n_ops, P)]
    sess.set_issue_threads(threads)
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    base = [sess.output_bytes(i) for i in range(len(tenants))]
    for splits in ([], sess.uniform_splits("cout", 2)):
        sess.set_plan(splits, sess.edges_from_pointers(P))
        sess.poison_outputs()
        rows = sess.trace(B.GACER_MODE_PLAN, 2)
        assert all(r["end_ms"] > r["start_ms"] >= 0.0 for r in rows)
        win = _cluster_windows(rows, clusters)
        assert sorted(win) == [0, 1, 2]
        for k in (0, 1):
            assert win[k + 1][0] >= win[k][1], f"cluster {k + 1} began at {win[k + 1][0]:.4f} ms, cluster {k} ended at {win[k][1]:.4f} ms"
        # inside a cluster the streams run freely: a tenant's chunks stay in stream order
        last_end = {}
        for r in rows:
            assert r["start_ms"] >= last_end.get(r["tenant"], 0.0) - 1e-6
            last_end[r["tenant"]] = r["end_ms"]
        for i in range(len(tenants)):
            assert sess.output_bytes(i) == base[i]
    # control: the same cluster windows without edges do overlap
    sess.clear_plan()
    rows = sess.trace(B.GACER_MODE_STREAM_PARALLEL, 2)
    win = _cluster_windows(rows, clusters)
    assert any(win[k + 1][0] < win[k][1] for k in (0, 1)), "free-running streams never overlapped two clusters"
    sess.set_issue_threads(False)
    sess.close()


def test_trace_rows_cover_every_kernel_once(gpu):
    from paper_2304_11745_amd import binding as B
    tenants, data = synth.build_config(2, "small")
    sess = gpu.Session(tenants, data)
    sess.set_plan(sess.uniform_splits("batch", 2), [])
    for mode in (B.GACER_MODE_PLAN, B.GACER_MODE_SEQUENTIAL, B.GACER_MODE_STREAM_PARALLEL):
        rows = sess.trace(mode, 3)
        launches = sess.launch_count(mode)
        assert len(rows) >= launches                                   # a K-sliced operator contributes two kernels
        assert len({(r["tenant"], r["op"], r["chunk"]) for r in rows}) == launches
        assert all(0.0 < r["ms"] < 5.0 and r["workgroups"] > 0 for r in rows)
        assert all(abs((r["end_ms"] - r["start_ms"]) - r["ms"]) < 0.5 for r in rows)
        if mode == B.GACER_MODE_SEQUENTIAL:                            # one stream: kernels never overlap
            ordered = sorted(rows, key=lambda r: r["start_ms"])
            assert all(b["start_ms"] >= a["end_ms"] - 1e-6 for a, b in zip(ordered, ordered[1:]))
    sess.close()


def _legal_variants(tenants):
    cout_ok = ("conv", "dwconv", "gemm", "maxpool", "gavgpool", "affine")
    out = []
    for ti, t in enumerate(tenants):
        for oi, op in enumerate(t.ops):
            out.append((ti, oi, 0, 1))
            for axis, ext in ((1, t.batch), (2, t.tensors[op.out][1] if op.kind in cout_ok else 0)):
                for f in (2, 4, 8):
                    if f <= ext:
                        out.append((ti, oi, axis, f))
    return out


def test_profile_table(gpu):
    """Lookup table of Section 4.1: one row per operator and legal (axis, factor), then the T_SW row; W follows from the
    launch geometry; profiling leaves every tensor as a plain run leaves it."""
    import torch
    from paper_2304_11745_amd import binding as B
    tenants, data = synth.build_config(3, "small")
    sess = gpu.Session(tenants, data)
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    before = [[a.clone() for a in acts] for acts in sess.acts]
    rows = sess.profile()
    got = [(r.tenant, r.op, r.axis, r.factor) for r in rows]
    assert got[:-1] == _legal_variants(tenants)
    last = rows[len(rows) - 1]
    assert (last.tenant, last.op, last.factor) == (-1, -1, 1) and 0.0 <= last.ms < 0.1       # T_SW: below 100 us per pointer
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for r in list(rows)[:-1]:
        assert 0.0 < r.ms < 10.0 and r.workgroups >= 1 and 0.0 < r.bw_share <= 1.0
        # W = min(1, workgroups / (compute units x resident workgroups per unit)), 1..8 resident workgroups per unit
        cands = [min(1.0, max(r.workgroups / (cus * w), 1.0 / (cus * 8))) for w in range(1, 9)]
        assert any(abs(r.cu_share - c) <= 1e-6 for c in cands), (r.workgroups, r.cu_share)
    torch.cuda.synchronize()
    for acts0, acts1 in zip(before, sess.acts):
        for a0, a1 in zip(acts0, acts1):
            assert torch.equal(a0.view(torch.uint8), a1.view(torch.uint8))
    sess.close()


@pytest.mark.parametrize("config", [c for c in sorted(synth.CONFIG_NAMES) if c > 1])
def test_searched_plan_end_to_end(gpu, config):
    """profile -> gacer_search -> gacer_set_plan -> run: bit-identical to the sequential unsplit run and within tolerance
    of the oracle; then the measured refinement (gacer_refine) on top, same checks."""
    from oracle import forward as F
    from paper_2304_11745_amd import binding as B
    tenants, data = synth.build_config(config, "small")
    sess = gpu.Session(tenants, data)
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    base = [sess.output_bytes(i) for i in range(len(tenants))]
    rows = sess.profile()
    splits, syncs, P, R = sess.search(rows, 20)
    assert len(P) == len(tenants) and len({len(p) for p in P}) == 1 and R >= 0.0
    assert sorted(syncs) == sorted(sess.edges_from_pointers(P)) if P[0] else syncs == []

    def check(tag):
        sess.poison_outputs()
        sess.run(B.GACER_MODE_PLAN, 2)
        for i, (t, (x, p)) in enumerate(zip(tenants, data)):
            assert sess.output_bytes(i) == base[i], f"{tag}: tenant {i} differs from the unsplit run"
            e = rel_err(sess.output(i), F.run_tenant(t, x, p))
            assert e <= TOL[t.dtype], f"{tag}: {t.name} rel err {e}"
    sess.set_plan(splits, syncs)
    check("searched")
    sp2, sy2, ms = sess.refine_plan(rows, rounds=3, min_gain=0.0)
    assert ms > 0.0 and sorted(sy2) == sorted(syncs) and len(sp2) >= len(splits)
    check("refined")
    sess.set_plan(sp2, sy2)                       # the returned plan is itself installable
    check("refined, reinstalled")
    sess.close()


def test_sibling_stream_decomposition(gpu):
    """Chunks of one operator on two streams of the same tenant (Section 5.4, Table 3: a model's batch decomposed over
    streams): bit-identical outputs with pointers, decomposition of the other tenant and per-tenant issue threads mixed
    in, K-sliced operators included (their chunks own disjoint parts of the workspace); and the two chunks of an
    operator really do overlap in time."""
    from paper_2304_11745_amd import binding as B
    tenants, data = synth.build_config(2)                      # ResNet-18(8) + MobileNetV2(8), full size
    sess = gpu.Session(tenants, data)
    assert sess.sibling_streams[0] is not None and sess.sibling_streams[0].cuda_stream != sess.streams[0].cuda_stream
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    base = [sess.output_bytes(i) for i in range(2)]
    n_ops = [len(t.ops) for t in tenants]
    halves = [(0, i, "batch", [4, 4], True) for i in range(n_ops[0])]
    plans = {"r18 halves on two streams": (halves, []),
             "+ pointers and mobilenet cout x2": (halves + sess.uniform_splits("cout", 2, tenants=[1]),
                                                  sess.edges_from_pointers([[n // 3, 2 * n // 3] for n in n_ops])),
             "quarters alternating, uneven": ([(0, i, "batch", [3, 2, 2, 1], True) for i in range(n_ops[0])] +
                                              [(1, i, "batch", [5, 3], True) for i in range(n_ops[1])], [])}
    for threads in (False, True):
        sess.set_issue_threads(threads)
        for name, (splits, syncs) in plans.items():
            sess.set_plan(splits, syncs)
            sess.poison_outputs()
            sess.run(B.GACER_MODE_PLAN, 3)
            for i in range(2):
                assert sess.output_bytes(i) == base[i], f"{name} (threads={threads}): tenant {i} differs"
            sess.poison_outputs()
            sess.run_static(B.GACER_MODE_PLAN, 1)
            for i in range(2):
                assert sess.output_bytes(i) == base[i], f"{name}: tenant {i} differs with the static workspace"
    sess.set_issue_threads(False)
    sess.set_plan(halves, [])
    rows = [r for r in sess.trace(B.GACER_MODE_PLAN, 2) if r["tenant"] == 0 and r["kernel"] != "splitk_finish"]
    by_op = {}
    for r in rows:
        by_op.setdefault(r["op"], {})[r["chunk"]] = r
    overlapping = [op for op, ch in by_op.items() if len(ch) == 2 and ch[1]["start_ms"] < ch[0]["end_ms"] and ch[0]["start_ms"] < ch[1]["end_ms"]]
    # how many overlap depends on how fast the host issues the traced launches (each carries an event pair); the long
    # convolutions always do
    assert len(overlapping) >= 2, f"only {len(overlapping)} of {len(by_op)} operators had their two chunks overlap"
    # and the next operator starts only after both chunks of the previous one have ended
    ends = {op: max(c["end_ms"] for c in ch.values()) for op, ch in by_op.items()}
    starts = {op: min(c["start_ms"] for c in ch.values()) for op, ch in by_op.items()}
    assert all(starts[op + 1] >= ends[op] - 1e-6 for op in by_op if op + 1 in by_op)
    sess.close()


def test_sync_every_launch_gives_the_same_bits(gpu):
    """The checking mode (every kernel waited for and checked before the next is issued) serialises all launches in
    issue order.  A plan whose sync pointers, fork/join events and workspace parts order everything that needs ordering
    gives the same bits either way; a captured graph is bypassed while the mode is on."""
    from paper_2304_11745_amd import binding as B
    tenants, data = synth.build_config(2, "small")
    sess = gpu.Session(tenants, data)
    n_ops = [len(t.ops) for t in tenants]
    batch = tenants[0].batch
    splits = [(0, i, "batch", [batch - batch // 2, batch // 2], True) for i in range(0, n_ops[0], 2)] + sess.uniform_splits("cout", 2, tenants=[1])
    sess.set_plan(splits, sess.edges_from_pointers([[n // 3, 2 * n // 3] for n in n_ops]))
    sess.poison_outputs()
    sess.run(B.GACER_MODE_PLAN, 2)
    base = [sess.output_bytes(i) for i in range(len(tenants))]
    sess.capture(B.GACER_MODE_PLAN)
    for threads in (False, True):
        sess.set_issue_threads(threads)
        sess.set_sync_every_launch(True)
        for mode in (B.GACER_MODE_PLAN, B.GACER_MODE_STREAM_PARALLEL, B.GACER_MODE_SEQUENTIAL):
            sess.poison_outputs()
            sess.run(mode, 2)
            assert [sess.output_bytes(i) for i in range(len(tenants))] == base, f"mode {mode}, threads={threads}: checking mode changed the bits"
        sess.poison_outputs()
        sess.run_static(B.GACER_MODE_PLAN, 1)
        assert [sess.output_bytes(i) for i in range(len(tenants))] == base
        sess.set_sync_every_launch(False)
        sess.poison_outputs()
        sess.run(B.GACER_MODE_PLAN, 2)
        assert [sess.output_bytes(i) for i in range(len(tenants))] == base
    sess.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fused_affine_launch_keeps_every_bit(gpu, dtype):
    """Launch fusion: a per-channel affine + ReLU and the 1x1 convolution that reads it run as one kernel.  Every tensor of
    every tenant (the affine outputs included, which the fused kernel writes on the side) must hold the bits of the unfused
    run, in every mode; the trace shows the fused kernel and no launch for the absorbed operator; a plan that decomposes
    one operator of a pair issues that pair unfused."""
    from paper_2304_11745_amd import binding as B
    from synth import graphs as G
    tenants = [G._densenet("dense_a", dtype, 3, 40, 8, [2, 3], 16, 2, 10), G._densenet("dense_b", dtype, 2, 33, 16, [3, 2], 24, 4, 7),
               G.small_resnet(dtype, 2)]
    data = [G.materialise(t, 31, i << 20) for i, t in enumerate(tenants)]
    sess = gpu.Session(tenants, data)

    def snapshot():
        return [[sess.tensor_bytes(t, i) for i in range(len(tn.tensors))] for t, tn in enumerate(tenants)]
    sess.set_fuse_affine(False)
    sess.poison_outputs()
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    want = snapshot()
    rows = sess.trace(B.GACER_MODE_STREAM_PARALLEL, 1)
    assert not any(r["kernel"].startswith("igemm_affine_") for r in rows)
    n_unfused = len(rows)
    sess.set_fuse_affine(True)
    rows = sess.trace(B.GACER_MODE_STREAM_PARALLEL, 1)
    fused = [r for r in rows if r["kernel"].startswith("igemm_affine_")]
    pairs = sorted({(r["tenant"], r["op"]) for r in fused})
    vec = 8 if dtype == "bf16" else 4
    expect = sorted((ti, k + 1) for ti, t in enumerate(tenants) for k, (a, b) in enumerate(zip(t.ops, t.ops[1:]))
                    if a.kind == "affine" and b.kind == "conv" and b.kh == 1 and b.in0 == a.out and t.tensors[a.out][1] % vec == 0)
    assert pairs == expect and len(pairs) >= 10, "every dense layer and transition with a vector-multiple channel count is fused"
    assert len(rows) == n_unfused - len(pairs)
    for t, op in pairs:
        assert tenants[t].ops[op].kind == "conv" and tenants[t].ops[op - 1].kind == "affine"
        assert not any(r["tenant"] == t and r["op"] == op - 1 for r in rows), "the absorbed affine operator still has a launch"
    for mode in (B.GACER_MODE_SEQUENTIAL, B.GACER_MODE_STREAM_PARALLEL, B.GACER_MODE_PLAN):
        sess.poison_outputs()
        sess.run(mode, 2)
        assert snapshot() == want, f"mode {mode}: fused launches changed some tensor"
    # decomposing the product of one pair un-fuses exactly that pair; pointers and other decompositions leave the rest fused
    t, op = pairs[0]
    sess.set_plan([(t, op, "cout", 2), (2, 1, "batch", 2)], sess.edges_from_pointers([[5, 9], [4, 12], [3, 6]]))
    rows = sess.trace(B.GACER_MODE_PLAN, 1)
    assert any(r["tenant"] == t and r["op"] == op - 1 for r in rows)
    still = {(r["tenant"], r["op"]) for r in rows if r["kernel"].startswith("igemm_affine_")}
    assert (t, op) not in still and len(still) >= len(pairs) - 1 - 4      # a pointer that lands on an affine operator un-fuses it too
    sess.poison_outputs()
    sess.run(B.GACER_MODE_PLAN, 2)
    assert snapshot() == want
    sess.close()
