"""gacer_run_static (the entry point for callers that cannot allocate) against gacer_run, through the C ABI: same bits,
on two calls in a row, the second with a smaller input; the static workspace keeps whatever the first call left."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def _sliced_tenants(dtype, batch, hw, width):
    """two small networks whose convolutions and classifier have a long K and few output tiles, so that their K ranges
    are cut into slices and the partial tiles go through the workspace"""
    from synth import graphs as G
    out = []
    for name, cin in (("sliced_a", width), (("sliced_b"), width // 2)):
        b = G._B(name, dtype, batch)
        x = b.tensor(batch, cin, hw, hw)
        y = b.conv(x, width, 3, 1, 1, "relu")
        y = b.conv(y, width, 3, 1, 1, "relu", res=-1)
        y = b.conv(y, 2 * width, 3, 2, 1, "relu")
        y = b.gemm(y, 24, "none", flatten=True)
        out.append(b.done(x, y))
    return out


def _all_outputs(sess):
    return [sess.output_bytes(i) for i in range(len(sess.tenants))]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_run_static_matches_run_on_two_calls_in_a_row(dtype):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2304_11745_amd import binding as B
    from paper_2304_11745_amd import harness
    from synth import graphs as G
    for batch, hw, width in ((8, 14, 64), (5, 14, 64)):           # second call: smaller input, smaller workspace need
        tenants = _sliced_tenants(dtype, batch, hw, width)
        data = [G.materialise(t, 31, i << 20) for i, t in enumerate(tenants)]
        sess = harness.Session(tenants, data)
        kernels = {r["kernel"] for r in sess.trace(B.GACER_MODE_SEQUENTIAL, 1)}
        assert "splitk_finish" in kernels, "the test tenants no longer use the split-K workspace"
        n_ops = [len(t.ops) for t in tenants]
        plans = {"unsplit": ([], []),
                 "cout2+pointer": (sess.uniform_splits("cout", 2), sess.edges_from_pointers([[n // 2] for n in n_ops])),
                 "batch-list": ([(0, 1, "batch", [batch - 1, 1])], [])}
        for name, (splits, syncs) in plans.items():
            sess.set_plan(splits, syncs)
            for mode in (B.GACER_MODE_PLAN, B.GACER_MODE_SEQUENTIAL, B.GACER_MODE_STREAM_PARALLEL):
                sess.poison_outputs()
                sess.run(mode, 2)
                want = _all_outputs(sess)
                assert all(np.isfinite(sess.output(i)).all() for i in range(len(tenants)))
                sess.poison_outputs()
                sess.run_static(mode, 2)
                assert _all_outputs(sess) == want, f"{dtype} {name} mode {mode}: gacer_run_static differs from gacer_run"
        sess.close()


def test_run_static_at_full_size_config2():
    """configs[1] at full size (about 11.5 MB of partial tiles per round): static workspace vs allocated workspace."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2304_11745_amd import binding as B
    from paper_2304_11745_amd import harness
    tenants, data = synth.build_config(2)
    sess = harness.Session(tenants, data)
    sess.poison_outputs()
    sess.run(B.GACER_MODE_STREAM_PARALLEL, 1)
    want = _all_outputs(sess)
    sess.poison_outputs()
    sess.run_static(B.GACER_MODE_STREAM_PARALLEL, 3)
    assert _all_outputs(sess) == want
    sess.close()
