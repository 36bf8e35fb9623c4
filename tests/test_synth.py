"""Seeded generators and tenant graph builders (CPU only)."""
import os
import numpy as np
import pytest

import synth
from synth.rng import _draws


def test_splitmix64_published_vector(golden_dir):
    exp = [int(l) for l in open(os.path.join(golden_dir, "splitmix64_vector.txt")) if not l.startswith("#")]
    got = _draws(0, 1234567, 5)           # state = 0 * 2^32 + 1234567
    assert [int(v) for v in got] == exp


def test_uniform_range_and_determinism():
    a = synth.splitmix64_uniform(7, 3, (1000,))
    b = synth.splitmix64_uniform(7, 3, (1000,))
    assert np.array_equal(a, b) and a.min() >= -1.0 and a.max() < 1.0
    assert abs(a.mean()) < 0.1 and abs(a.var() - 1.0 / 3.0) < 0.05
    assert not np.array_equal(a, synth.splitmix64_uniform(7, 4, (1000,)))


def test_normal_moments():
    a = synth.splitmix64_normal(11, 0, (20001,), 0.02)
    assert abs(a.mean()) < 1e-3 and abs(a.std() - 0.02) < 1e-3


def test_bf16_round_ties_to_even():
    one = np.float32(1.0)
    cases = [(1.0 + 2.0 ** -8, 1.0),                 # exactly half way, even mantissa below -> down
             (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6),  # half way, odd below -> up to even
             (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7),
             (1.0 + 2.0 ** -9, 1.0), (-1.0 - 3 * 2.0 ** -8, -1.0 - 2.0 ** -6), (0.0, 0.0)]
    x = np.array([c[0] for c in cases], np.float32)
    assert np.array_equal(synth.bf16_round(x), np.array([c[1] for c in cases], np.float32))
    r = synth.bf16_round(synth.splitmix64_uniform(1, 1, (4096,)).astype(np.float32))
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert one == synth.bf16_round(np.array([1.0], np.float32))[0]


def test_published_model_totals(golden_dir):
    build = {"resnet18": synth.resnet18, "resnet34": synth.resnet34, "resnet50": synth.resnet50, "resnet101": synth.resnet101,
             "vgg16": synth.vgg16, "alexnet": synth.alexnet, "mobilenetv2": synth.mobilenetv2, "bert_base": synth.bert_base,
             "mobilenetv3_large": synth.mobilenetv3_large, "densenet121": synth.densenet121}
    for line in open(os.path.join(golden_dir, "model_totals.txt")):
        if line.startswith("#"):
            continue
        name, ops, params_m, gmac = line.split()
        t = build[name]("bf16", 1)
        assert len(t.ops) == int(ops)
        assert round(synth.tenant_params(t) / 1e6, 2) == float(params_m)
        assert round(synth.gemm_macs(t) / 1e9, 3) == float(gmac)


def test_final_feature_maps():
    for f, c, hw in [(synth.resnet18, 512, 7), (synth.resnet34, 512, 7), (synth.resnet50, 2048, 7), (synth.resnet101, 2048, 7),
                     (synth.vgg16, 512, 7), (synth.mobilenetv2, 1280, 7), (synth.alexnet, 256, 6),
                     (synth.mobilenetv3_large, 960, 7), (synth.densenet121, 1024, 7)]:
        t = f("f32", 1)
        last_spatial = [op for op in t.ops if t.tensors[op.in0][2] > 1][-1]          # the pool (or flattening FC) in front of the classifier
        assert last_spatial.kind in ("gavgpool", "gemm") and t.tensors[last_spatial.in0] == (1, c, hw, hw)


def test_graphs_are_topologically_ordered():
    for cfg in sorted(synth.CONFIG_NAMES):
        tenants, _ = synth.build_config(cfg, "full", with_data=False)
        for t in tenants:
            # channels written so far, per tensor that owns storage (a channel window writes / reads channels of its base)
            have = {i: set() for i in range(len(t.tensors)) if i not in t.views}

            def channels(i):
                base, off = t.views.get(i, (i, 0))
                return base, set(range(off, off + t.tensors[i][1]))

            def write(i):
                base, ch = channels(i)
                assert not (have[base] & ch), "written twice"
                have[base] |= ch

            def readable(i):
                base, ch = channels(i)
                return ch <= have[base]
            write(t.input)
            for op in t.ops:
                for i in (op.in0, op.in1, op.res):
                    assert i < 0 or readable(i)
                write(op.out)
            assert readable(t.output)
            for i, (base, off) in t.views.items():
                assert base not in t.views and t.tensors[base][0] == t.tensors[i][0] and t.tensors[base][2:] == t.tensors[i][2:]
            assert all(s[0] % t.batch == 0 for s in t.tensors)


def test_config_data_is_seeded_and_bf16_clean():
    t1, d1 = synth.build_config(3, "small")
    t2, d2 = synth.build_config(3, "small")
    for (x1, p1), (x2, p2) in zip(d1, d2):
        assert np.array_equal(x1, x2) and all(np.array_equal(a, b) for a, b in zip(p1, p2))
    x, p = d1[0]
    assert np.all((x.view(np.uint32) & 0xFFFF) == 0)
    w = p[t1[0].ops[0].w]
    assert np.all((w.view(np.uint32) & 0xFFFF) == 0)
    fan_in = t1[0].params[t1[0].ops[0].w].fan_in
    assert np.abs(w).max() <= np.sqrt(6.0 / fan_in) / np.sqrt(1 + 1e-5) * (1 + 2 ** -8)
