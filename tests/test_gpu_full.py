"""Full-size parity in the launch configuration bench.py times: configs[1] (ResNet-18 + MobileNetV2,
fp32, batch 8 each, 224x224) against the oracle, and the split sweep 1/2/4 on batch and Cout
bit-exact against the unsplit run."""
import numpy as np
import pytest

import synth
from parity import TOL, rel_err

pytestmark = pytest.mark.gpu


def test_config2_full_size_vs_oracle_and_split_sweep():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import forward as F
    from paper_2304_11745_amd import binding as B
    from paper_2304_11745_amd import harness
    tenants, data = synth.build_config(2)
    sess = harness.Session(tenants, data)
    sess.poison_outputs()
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    base = [sess.output_bytes(i) for i in range(2)]
    for i, (t, (x, p)) in enumerate(zip(tenants, data)):
        ref = F.run_tenant(t, x, p)
        e = rel_err(sess.output(i), ref)
        print(f"{t.name} full size rel_err={e:.3e}", flush=True)
        assert e <= TOL["f32"]
    for axis in ("batch", "cout"):
        for f in (1, 2, 4):
            sess.set_plan(sess.uniform_splits(axis, f) if f > 1 else [], [])
            sess.poison_outputs()
            sess.run(B.GACER_MODE_PLAN, 1)
            for i in range(2):
                assert sess.output_bytes(i) == base[i], f"{axis} x{f}: tenant {i} not bit-identical"
    # explicit chunk lists (list_B): uneven batch chunks on ResNet-18, an 8-channel tail chunk on MobileNetV2's convolutions
    uneven = [(0, i, "batch", [5, 3]) for i in range(len(tenants[0].ops))]
    uneven += [(1, i, "cout", [op.cout - 8, 8]) for i, op in enumerate(tenants[1].ops) if op.kind in ("conv", "dwconv") and op.cout > 8]
    sess.set_plan(uneven, [])
    sess.poison_outputs()
    sess.run(B.GACER_MODE_PLAN, 1)
    for i in range(2):
        assert sess.output_bytes(i) == base[i], f"uneven chunk lists: tenant {i} not bit-identical"
    # one tenant only, plus pointers
    sess.set_plan(sess.uniform_splits("batch", 2, tenants=[0]), sess.edges_from_pointers([[5, 12], [10, 30]]))
    sess.poison_outputs()
    sess.run(B.GACER_MODE_PLAN, 2)
    for i in range(2):
        assert sess.output_bytes(i) == base[i]
    sess.close()


@pytest.mark.parametrize("config", [3, 4, 5])
def test_bf16_configs_full_size(config):
    """configs[2..4] at full size: every tenant against the oracle (bf16 storage on both sides), and a
    decomposed + pointer-ordered plan bit-exact against the sequential unsplit run."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import forward as F
    from paper_2304_11745_amd import binding as B
    from paper_2304_11745_amd import harness
    tenants, data = synth.build_config(config)
    sess = harness.Session(tenants, data)
    sess.poison_outputs()
    sess.run(B.GACER_MODE_SEQUENTIAL, 1)
    base = [sess.output_bytes(i) for i in range(len(tenants))]
    done = {}
    for i, (t, (x, p)) in enumerate(zip(tenants, data)):
        out = sess.output(i)
        assert np.isfinite(out).all()
        key = (t.name, t.batch)
        if key in done and config != 4:
            continue
        ref = F.run_tenant(t, x, p)
        e = rel_err(out, ref)
        print(f"config {config} {t.name}({t.batch}) rel_err={e:.3e}", flush=True)
        assert e <= TOL["bf16"], f"{t.name}: {e}"
        done[key] = True
    n_ops = [len(t.ops) for t in tenants]
    splits = sess.uniform_splits("cout", 2) if config == 4 else sess.uniform_splits("batch", 2, tenants=[1]) + sess.uniform_splits("cout", 4, tenants=[0])
    sess.set_plan(splits, sess.edges_from_pointers([[n // 3, 2 * n // 3] for n in n_ops]))
    sess.poison_outputs()
    sess.run(B.GACER_MODE_PLAN, 1)
    for i in range(len(tenants)):
        assert sess.output_bytes(i) == base[i], f"tenant {i} not bit-identical under the plan"
    sess.clear_plan()
    sess.poison_outputs()
    sess.run(B.GACER_MODE_STREAM_PARALLEL, 1)
    for i in range(len(tenants)):
        assert sess.output_bytes(i) == base[i]
    sess.close()
