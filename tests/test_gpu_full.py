"""Full-size parity in the launch configuration bench.py times: configs[1] (ResNet-18 + MobileNetV2,
fp32, batch 8 each, 224x224) against the oracle, and the split sweep 1/2/4 on batch and Cout
bit-exact against the unsplit run."""
import numpy as np
import pytest

import synth
from parity import TOL, TOL_ONE_OP, rel_err

pytestmark = pytest.mark.gpu


def _check_every_tensor(sess, i, t, x, p):
    """Tenant i at full size against the oracle: (1) the output, and for fp32 every tensor, of the oracle's own forward
    pass at the end-to-end tolerance; (2) every operator on its own, the oracle evaluating it on the inputs the GPU
    operator read, at the one-operator tolerance -- a wrong tile variant cannot hide behind the depth of the network."""
    from oracle import forward as F
    ref_all = F.run_tenant(t, x, p, keep_all=True)
    gpu_all = [sess.tensor(i, k) for k in range(len(t.tensors))]
    e_out = rel_err(gpu_all[t.output], ref_all[t.output])
    assert e_out <= TOL[t.dtype], f"{t.name}: output rel err {e_out} > {TOL[t.dtype]}"
    drift, forced = (0.0, -1), (0.0, -1)
    for k, op in enumerate(t.ops):
        e = rel_err(gpu_all[op.out], ref_all[op.out])
        drift = max(drift, (e, k))
        if t.dtype == "f32":
            assert e <= TOL["f32"], f"{t.name} op {k} ({op.kind}): rel err {e}"
        e1 = rel_err(gpu_all[op.out], F.run_op(t, k, gpu_all, p))
        forced = max(forced, (e1, k))
        assert e1 <= TOL_ONE_OP[t.dtype], f"{t.name} op {k} ({op.kind}) on the GPU's own inputs: rel err {e1} > {TOL_ONE_OP[t.dtype]}"
    print(f"{t.name}({t.batch}) full size: output {e_out:.3e}; worst tensor of the free-running pass {drift[0]:.3e} (op {drift[1]}); "
          f"worst single operator {forced[0]:.3e} (op {forced[1]})", flush=True)


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
        _check_every_tensor(sess, i, t, x, p)
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


@pytest.mark.parametrize("config", [c for c in sorted(synth.CONFIG_NAMES) if c > 2])
def test_further_configs_full_size(config):
    """Every configuration after the headline one at full size: every tenant against the oracle (storage in the
    tenant's dtype on both sides), and a decomposed + pointer-ordered plan bit-exact against the sequential unsplit run."""
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
        _check_every_tensor(sess, i, t, x, p)
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
    if config in (3, 6):       # the plan the configuration asks for: from the CPU search over the profiled table
        splits, syncs, P, R = sess.search(sess.profile(), 20)
        sess.set_plan(splits, syncs)
        sess.poison_outputs()
        sess.run(B.GACER_MODE_PLAN, 1)
        for i in range(len(tenants)):
            assert sess.output_bytes(i) == base[i], f"tenant {i} not bit-identical under the searched plan"
        print(f"config {config} searched plan: {len(splits)} decomposed operators, pointers {P}, modelled residue {R:.4f}", flush=True)
    sess.close()
