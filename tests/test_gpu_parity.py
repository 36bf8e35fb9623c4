"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, and bit-exactness of
every regulation plan against the unsplit run."""
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


def _oracle_outputs(tenants, data):
    from oracle import forward as F
    return [F.run_tenant(t, x, p) for t, (x, p) in zip(tenants, data)]


def _check_all_modes_and_plans(gpu, tenants, data, plans, check_intermediate=False):
    from paper_2304_11745_amd import binding as B
    from oracle import forward as F
    sess = gpu.Session(tenants, data)
    ref = _oracle_outputs(tenants, data)
    sess.poison_outputs()
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    base = [sess.output_bytes(i) for i in range(len(tenants))]
    for i, t in enumerate(tenants):
        out = sess.output(i)
        assert np.isfinite(out).all(), f"{t.name}: non-finite output"
        e = rel_err(out, ref[i])
        print(f"{t.name}[{t.dtype}] sequential rel_err={e:.3e}")
        assert e <= TOL[t.dtype], f"{t.name}: rel err {e} > {TOL[t.dtype]}"
    if check_intermediate:
        for i, (t, (x, p)) in enumerate(zip(tenants, data)):
            allref = F.run_tenant(t, x, p, keep_all=True)
            for k, op in enumerate(t.ops):
                e = rel_err(sess.tensor(i, op.out), allref[op.out])
                assert e <= TOL[t.dtype], f"{t.name} op {k} ({op.kind}): rel err {e}"
    for mode in (B.GACER_MODE_STREAM_PARALLEL, B.GACER_MODE_PLAN):
        sess.poison_outputs()
        sess.run(mode, 2)
        for i in range(len(tenants)):
            assert sess.output_bytes(i) == base[i], f"mode {mode}: tenant {i} differs from sequential"
    for name, (splits, ptrs) in plans(sess).items():
        syncs = sess.edges_from_pointers(ptrs) if ptrs else []
        sess.set_plan(splits, syncs)
        sess.poison_outputs()
        sess.run(B.GACER_MODE_PLAN, 2)
        for i in range(len(tenants)):
            assert sess.output_bytes(i) == base[i], f"plan {name}: tenant {i} not bit-identical to the unsplit run"
        print(f"plan {name}: {sess.launch_count()} launches, bit-exact")
    sess.close()


def _sweep_plans(sess):
    plans = {}
    for axis in ("batch", "cout"):
        for f in (2, 4, 8):
            sp = sess.uniform_splits(axis, f)
            if sp:
                plans[f"{axis}x{f}"] = (sp, None)
    # explicit chunk lists (list_B, Section 4.2): uneven sizes, channel chunks that start at unaligned offsets
    uneven = []
    for ti, t in enumerate(sess.tenants):
        for oi, op in enumerate(t.ops):
            cout = t.tensors[op.out][1]
            if op.kind in ("conv", "dwconv", "gemm") and cout >= 6 and oi % 2 == 0:
                uneven.append((ti, oi, "cout", [cout - 5, 3, 2]))
            elif t.batch >= 3:
                uneven.append((ti, oi, "batch", [t.batch - 2, 2] if oi % 3 else [1, t.batch - 1]))
    plans["uneven-lists"] = (uneven, None)
    n_ops = [len(t.ops) for t in sess.tenants]
    plans["pointers1"] = ([], [[n // 2] for n in n_ops])
    plans["pointers3+cout2"] = (sess.uniform_splits("cout", 2), [[0, n // 3, n] for n in n_ops])
    plans["pointers2+batch2-tenant0"] = (sess.uniform_splits("batch", 2, tenants=[0]) if sess.tenants[0].batch >= 2 else [],
                                         [[1, n - 1] for n in n_ops])
    return plans


def test_config1_toy_pair(gpu):
    tenants, data = synth.build_config(1)

    def plans(sess):
        return {"unsplit": ([], None),
                "convs-2way-cout": ([(0, 0, "cout", 2), (0, 1, "cout", 2)], None),
                **_sweep_plans(sess)}
    _check_all_modes_and_plans(gpu, tenants, data, plans, check_intermediate=True)


@pytest.mark.parametrize("config", [c for c in sorted(synth.CONFIG_NAMES) if c > 1])
def test_small_families(gpu, config):
    tenants, data = synth.build_config(config, "small")
    _check_all_modes_and_plans(gpu, tenants, data, _sweep_plans, check_intermediate=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_families_all_kinds(gpu, dtype):
    """Every operator kind, including the transformer tenant and standalone affine/add/act operators, in both dtypes."""
    from synth import graphs as G
    b = G._B("eltwise_mix", dtype, 3)
    x = b.tensor(3, 20, 9, 7)
    y = b.conv(x, 24, 3, 1, 1, "none")
    y = b.affine(y, "relu")
    z = b.conv(y, 24, 1, 1, 0, "none")
    z = b.affine(z, "none", res=y)
    y = b.add(z, y, "relu6")
    y = b.act(y, "gelu")
    y = b.maxpool(y, 3, 2, 1)
    y = b.gavgpool(y)
    y = b.gemm(y, 13, flatten=True)
    t = b.done(x, y)
    tenants = [t, G.small_bert(dtype, 3), G.small_mbv2(dtype, 2)]
    data = [G.materialise(tt, 77, i << 20) for i, tt in enumerate(tenants)]
    _check_all_modes_and_plans(gpu, tenants, data, _sweep_plans, check_intermediate=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gate_concat_mean_pool_ragged(gpu, dtype):
    """Channel gate, concatenation and mean pooling at extents that leave the vector paths: a seam that is not a multiple
    of a 16-byte vector, odd channel counts, 3x3 stride-1 and stride-2 mean windows, hard-swish / hard-sigmoid after
    convolutions, depthwise convolutions, FCs, a K-sliced product and standalone operators; every intermediate tensor
    against the oracle, every decomposition bit-exact."""
    from synth import graphs as G
    tenants = []
    for ti, (cin, c1, c2, hw) in enumerate([(5, 13, 6, 11), (8, 24, 16, 14), (3, 40, 7, 9)]):
        b = G._B(f"ragged{ti}", dtype, 3)
        x = b.tensor(3, cin, hw, hw)
        a = b.conv(x, c1, 3, 1, 1, "hswish")
        z = b.conv(a, c2, 1, 1, 0, "hsigmoid")
        y = b.concat(a, z)                                   # seam at c1: 13 and 40 are no vector multiples in bf16, 13 in neither
        g = b.gavgpool(y)
        g = b.gemm(g, 10, "relu", flatten=True)
        g = b.gemm(g, c1 + c2, "hsigmoid", flatten=True, fold=0.25)
        y = b.scale(y, g, "none" if ti else "hswish")
        y = b.conv(y, c1 + c2, 5, 1, 2, "hswish", groups=c1 + c2)
        y = b.avgpool(y, 3, 1 + ti % 2)
        y = b.concat(y, b.act(y, "hswish"))
        y = b.avgpool(y, 2, 2)
        y = b.gemm(y, 9, "hswish", flatten=True)
        tenants.append(b.done(x, y))
    b = G._B("long_k_hswish", dtype, 2)                      # few tiles and a long K: the K-sliced path and its finishing pass
    x = b.tensor(2, 256, 6, 6)
    y = b.conv(x, 72, 3, 1, 1, "hswish")
    y = b.conv(y, 40, 3, 1, 1, "hsigmoid")
    tenants.append(b.done(x, y))
    data = [G.materialise(t, 99, i << 20) for i, t in enumerate(tenants)]
    _check_all_modes_and_plans(gpu, tenants, data, _sweep_plans, check_intermediate=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_conv_shapes(gpu, dtype):
    """Seeded random convolution / depthwise / FC shapes (ragged M, N and K tails, odd channel counts, strides, paddings,
    residuals, every activation): parity with the oracle on every intermediate tensor, bit-exactness under uniform and
    uneven decompositions."""
    import random
    from synth import graphs as G
    rng = random.Random(20230411 if dtype == "f32" else 20230412)
    tenants = []
    for ti in range(6):
        batch = rng.choice([1, 2, 3, 5])
        hw = rng.choice([5, 8, 11, 14, 23])
        cin = rng.choice([1, 3, 5, 8, 16, 24, 40])
        b = G._B(f"rand{ti}", dtype, batch)
        x = b.tensor(batch, cin, hw, hw)
        y = x
        for li in range(rng.choice([3, 4, 5])):
            n, c, h, w = b.shape(y)
            kind = rng.choice(["conv", "conv", "conv", "dw", "pw_res"])
            if kind == "dw" and h >= 3:
                y = b.conv(y, c, 3, rng.choice([1, 2]), 1, rng.choice(["relu6", "none"]), groups=c)
            elif kind == "pw_res":
                y = b.conv(y, c, 1, 1, 0, rng.choice(["relu", "gelu", "none"]), res=y)
            else:
                k = rng.choice([k for k in (1, 3, 5) if k <= h + 2])
                pad = rng.choice([p for p in (0, 1, 2) if h + 2 * p >= k])
                stride = rng.choice([1, 2])
                y = b.conv(y, rng.choice([1, 7, 16, 33, 64, 100, 136]), k, stride, pad, rng.choice(["relu", "relu6", "gelu", "none"]))
        y = b.gemm(b.gavgpool(y), rng.choice([3, 10, 17]), rng.choice(["none", "relu"]), flatten=True)
        tenants.append(b.done(x, y))
    data = [G.materialise(t, 99, i << 20) for i, t in enumerate(tenants)]
    _check_all_modes_and_plans(gpu, tenants, data, _sweep_plans, check_intermediate=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_long_k_conv_shapes(gpu, dtype):
    """Convolutions and GEMMs whose K rows are long enough for the direct-to-LDS pipeline (several stages of K blocks in
    flight): ragged M / N / K tails, taps narrower and wider than a K block, strides, K ranges cut into slices, wide
    outputs that take the larger tiles.  Parity on every tensor, bit-exactness under decomposition."""
    from synth import graphs as G
    specs = [  # (batch, hw, cin, [(cout, k, stride, pad, act, residual)])
        (3, 9, 64, [(100, 5, 1, 2, "relu", False), (136, 3, 2, 1, "none", False), (136, 3, 1, 1, "relu6", True)]),
        (2, 14, 72, [(64, 3, 1, 1, "relu", False), (256, 3, 1, 1, "gelu", False), (24, 1, 1, 0, "none", False)]),
        (5, 7, 40, [(264, 5, 1, 2, "relu", False), (264, 3, 1, 1, "relu", True), (33, 3, 1, 0, "none", False)]),
        (1, 12, 512, [(128, 1, 1, 0, "relu", False), (512, 3, 1, 1, "relu", False), (520, 1, 2, 0, "none", False)]),
        (4, 6, 2048, [(64, 1, 1, 0, "none", False), (96, 3, 1, 1, "relu", False)]),
    ]
    tenants = []
    for ti, (batch, hw, cin, layers) in enumerate(specs):
        b = G._B(f"longk{ti}", dtype, batch)
        x = y = b.tensor(batch, cin, hw, hw)
        for (cout, k, stride, pad, act, res) in layers:
            y = b.conv(y, cout, k, stride, pad, act, res=y if res else -1)
        y = b.gemm(y, 40, "relu", flatten=True)                    # a long flattened K with one row per item
        tenants.append(b.done(x, b.gemm(y, 10, flatten=True)))
    data = [G.materialise(t, 123, i << 20) for i, t in enumerate(tenants)]
    _check_all_modes_and_plans(gpu, tenants, data, _sweep_plans, check_intermediate=True)


def test_stream_placement_over_hardware_queues(gpu):
    """Streams that share a hardware queue serialise: the probe must give the same grouping twice, the harness must put
    up to `queues` tenants on distinct queues, and placement must not change any output."""
    import ctypes as C
    import torch
    from paper_2304_11745_amd import binding as B
    streams = [torch.cuda.Stream() for _ in range(12)]
    arr = (C.c_void_p * len(streams))(*[s.cuda_stream for s in streams])
    g1, g2 = (C.c_int * len(streams))(), (C.c_int * len(streams))()
    assert B.gacer_probe_stream_queues(arr, len(streams), g1) == B.GACER_OK
    assert B.gacer_probe_stream_queues(arr, len(streams), g2) == B.GACER_OK
    assert list(g1) == list(g2)
    queues = len(set(g1))
    assert 1 <= queues <= len(streams) and g1[0] == 0 and max(g1) == queues - 1
    tenants, data = synth.build_config(4, "small")
    outs = []
    for place in (True, False):
        sess = gpu.Session(tenants, data, place_streams=place)
        if place:
            assert sess.queue_groups == queues
            used = [sess.tenant_queue.count(q) for q in range(queues)]
            assert sum(used) == len(tenants) and max(used) - min(used) <= 1          # tenants spread evenly over the queues
            assert len({s.cuda_stream for s in sess.streams}) == len(tenants)      # and still one stream each
        sess.poison_outputs()
        sess.run(B.GACER_MODE_STREAM_PARALLEL, 2)
        outs.append([sess.output_bytes(i) for i in range(len(tenants))])
        sess.close()
    assert outs[0] == outs[1]


@pytest.mark.parametrize("config", [3, 8])
def test_captured_round_replays_bit_exact(gpu, config):
    """A round captured into a HIP graph must reproduce the eager round bit for bit, on every replay, with
    eager rounds and synchronisations in between, for all three modes and a decomposed, pointer-ordered plan
    (config 8: with fused launches, channel-window tensors, gates and mean pools in the graph)."""
    from paper_2304_11745_amd import binding as B
    tenants, data = synth.build_config(config, "small")
    sess = gpu.Session(tenants, data)
    n_ops = [len(t.ops) for t in tenants]
    sess.set_plan(sess.uniform_splits("cout", 2, tenants=[0, 1]) + sess.uniform_splits("batch", 2, tenants=[2]),
                  sess.edges_from_pointers([[n // 3, 2 * n // 3] for n in n_ops]))
    sess.poison_outputs()
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    base = [sess.output_bytes(i) for i in range(len(tenants))]
    for mode in (B.GACER_MODE_PLAN, B.GACER_MODE_STREAM_PARALLEL, B.GACER_MODE_SEQUENTIAL):
        sess.capture(mode)
        for replay in range(4):
            sess.poison_outputs()
            sess.run(mode, 1 + replay)                       # graph replays
            for i in range(len(tenants)):
                assert sess.output_bytes(i) == base[i], f"mode {mode} replay {replay}: tenant {i} differs"
            sess.release_graphs() if replay == 2 else None   # replay 3 runs eagerly again
    # a new plan drops the captures; the eager path must still be right
    sess.clear_plan()
    sess.poison_outputs()
    sess.run(B.GACER_MODE_PLAN, 1)
    for i in range(len(tenants)):
        assert sess.output_bytes(i) == base[i]
    sess.close()


@pytest.mark.parametrize("config", [4, 8])
def test_threaded_issue_bit_exact(gpu, config):
    """One host thread per tenant (config 4: 8 tenants; config 8: fused launches and channel-window tensors), pointers +
    decomposition: same bits as the single-threaded run."""
    from paper_2304_11745_amd import binding as B
    tenants, data = synth.build_config(config, "small")
    sess = gpu.Session(tenants, data)
    n_ops = [len(t.ops) for t in tenants]
    sess.poison_outputs()
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    base = [sess.output_bytes(i) for i in range(len(tenants))]
    sess.set_issue_threads(True)
    for plan in ("unsplit", "regulated"):
        if plan == "regulated":
            sess.set_plan(sess.uniform_splits("cout", 2), sess.edges_from_pointers([[n // 4, n // 2, 3 * n // 4] for n in n_ops]))
        for mode in (B.GACER_MODE_STREAM_PARALLEL, B.GACER_MODE_PLAN):
            for rounds in (1, 5):
                sess.poison_outputs()
                sess.run(mode, rounds)
                for i in range(len(tenants)):
                    assert sess.output_bytes(i) == base[i], f"{plan} mode {mode} rounds {rounds}: tenant {i} differs"
    sess.set_issue_threads(False)
    sess.close()
