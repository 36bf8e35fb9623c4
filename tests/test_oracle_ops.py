"""Pins for the CPU oracle's operators: hand-computed cases, algebraic
identities, and agreement with PyTorch's CPU routines in fp64 (PyTorch is a
referee here only; the oracle contains no PyTorch calls)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as tF

import synth
from oracle import forward as F


def rnd(shape, tid, lo=-1.0, hi=1.0):
    return synth.splitmix64_uniform(99, tid, shape, lo, hi).astype(np.float32)


# ---- hand cases -------------------------------------------------------------------------------
@pytest.mark.parametrize("cin", [1, 3])
def test_conv_all_ones_counts_taps(cin):
    x = np.ones((1, cin, 5, 6), np.float32)
    w = np.ones((2, cin, 3, 3), np.float32)
    y = F.conv2d(x, w, None, None, 1, 1, 1, "none")
    assert y.shape == (1, 2, 5, 6)
    assert np.all(y[0, :, 1:-1, 1:-1] == 9 * cin)
    assert np.all(y[0, :, 0, 1:-1] == 6 * cin) and np.all(y[0, :, 1:-1, 0] == 6 * cin)
    assert y[0, 0, 0, 0] == 4 * cin and y[0, 1, -1, -1] == 4 * cin


def test_conv_is_cross_correlation_not_flipped():
    x = np.zeros((1, 1, 3, 3), np.float32)
    x[0, 0, 0, 1] = 1.0                       # impulse at (0,1)
    w = np.arange(9, dtype=np.float32).reshape(1, 1, 3, 3)
    y = F.conv2d(x, w, None, None, 1, 1, 1, "none")
    # y[oh,ow] = w[ih-oh+1, iw-ow+1] for the impulse at (ih,iw)=(0,1)
    assert y[0, 0, 1, 1] == w[0, 0, 0, 1] and y[0, 0, 0, 0] == w[0, 0, 1, 2] and y[0, 0, 1, 2] == w[0, 0, 0, 0]


def test_conv_centre_tap_identity_and_stride2():
    x = rnd((2, 3, 7, 7), 1)
    w = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        w[c, c, 1, 1] = 1.0
    assert np.array_equal(F.conv2d(x, w, None, None, 1, 1, 1, "none"), x)
    assert np.array_equal(F.conv2d(x, w, None, None, 2, 1, 1, "none"), x[:, :, ::2, ::2])


def test_conv_bias_residual_act_hand():
    x = np.full((1, 1, 2, 2), 2.0, np.float32)
    w = np.full((1, 1, 1, 1), -3.0, np.float32)
    b = np.array([1.0], np.float32)
    res = np.array([[[[10.0, 0.0], [4.0, 20.0]]]], np.float32)
    y = F.conv2d(x, w, b, res, 1, 0, 1, "relu6")      # -6 + 1 + res, clipped to [0,6]
    assert np.array_equal(y, np.array([[[[5.0, 0.0], [0.0, 6.0]]]], np.float32))


def test_conv1x1_equals_fc_over_pixels_and_full_kernel_equals_fc():
    x = rnd((2, 5, 4, 3), 2)
    w = rnd((7, 5, 1, 1), 3)
    b = rnd((7,), 4)
    y = F.conv2d(x, w, b, None, 1, 0, 1, "none")
    rows = np.ascontiguousarray(x.transpose(0, 2, 3, 1)).reshape(-1, 5)
    yf = F.gemm(rows, w.reshape(7, 5), b, None, "none").reshape(2, 4, 3, 7).transpose(0, 3, 1, 2)
    assert np.array_equal(y, yf)
    wk = rnd((6, 5, 4, 3), 5)
    y2 = F.conv2d(x, wk, None, None, 1, 0, 1, "none")
    assert np.array_equal(y2.reshape(2, 6), F.gemm(x.reshape(2, -1), wk.reshape(6, -1), None, None, "none"))


def test_depthwise_equals_independent_single_channel_convs():
    x = rnd((2, 4, 6, 6), 6)
    w = rnd((4, 1, 3, 3), 7)
    y = F.conv2d(x, w, None, None, 2, 1, 4, "none")
    for c in range(4):
        yc = F.conv2d(np.ascontiguousarray(x[:, c:c + 1]), np.ascontiguousarray(w[c:c + 1]), None, None, 2, 1, 1, "none")
        assert np.array_equal(y[:, c:c + 1], yc)


def test_conv_linearity_power_of_two_scale():
    x = rnd((1, 3, 6, 6), 8)
    w = rnd((4, 3, 3, 3), 9)
    assert np.array_equal(F.conv2d(4 * x, w, None, None, 1, 1, 1, "none"), 4 * F.conv2d(x, w, None, None, 1, 1, 1, "none"))


def test_maxpool_ramp_and_negative_border():
    x = np.arange(36, dtype=np.float32).reshape(1, 1, 6, 6)
    y = F.maxpool(x, 2, 2, 0)
    assert np.array_equal(y[0, 0], x[0, 0, 1::2, 1::2])
    xn = -np.ones((1, 1, 5, 5), np.float32) - np.arange(25, dtype=np.float32).reshape(1, 1, 5, 5)
    yn = F.maxpool(xn, 3, 2, 1)               # padding must never win even though all data < 0
    assert yn.shape == (1, 1, 3, 3) and yn.max() <= -1.0 and yn[0, 0, 0, 0] == -1.0
    assert yn[0, 0, 2, 2] == xn[0, 0, 3, 3]


def test_gavgpool_constant_and_hand():
    assert np.all(F.gavgpool(np.full((2, 3, 4, 5), 2.5, np.float32)) == 2.5)
    x = np.arange(8, dtype=np.float32).reshape(1, 2, 2, 2)
    assert np.array_equal(F.gavgpool(x).ravel(), np.array([1.5, 5.5], np.float32))


def test_affine_act_hand_distinct_scale_shift_residual():
    """y = act(x*scale[c] + shift[c] + res): scale, shift and the residual get different values per channel so that
    swapping scale and shift, indexing them by position instead of channel, or dropping the residual changes a result."""
    x = np.array([[[[1.0, -2.0]], [[3.0, 0.5]]]], np.float32)            # (1, 2, 1, 2): channel 0 = [1,-2], channel 1 = [3,0.5]
    scale = np.array([2.0, -4.0], np.float32)
    shift = np.array([0.5, 8.0], np.float32)
    res = np.array([[[[10.0, 1.0]], [[-1.0, 4.0]]]], np.float32)
    # by hand: c0: 1*2+0.5 = 2.5, -2*2+0.5 = -3.5 ; c1: 3*-4+8 = -4, 0.5*-4+8 = 6
    assert np.array_equal(F.affine_act(x, scale, shift, None, "none").ravel(), [2.5, -3.5, -4.0, 6.0])
    # + residual: 12.5, -2.5, -5, 10
    assert np.array_equal(F.affine_act(x, scale, shift, res, "none").ravel(), [12.5, -2.5, -5.0, 10.0])
    assert np.array_equal(F.affine_act(x, scale, shift, res, "relu").ravel(), [12.5, 0.0, 0.0, 10.0])
    assert np.array_equal(F.affine_act(x, scale, shift, res, "relu6").ravel(), [6.0, 0.0, 0.0, 6.0])
    g = F.affine_act(x, scale, shift, None, "gelu").ravel()               # gelu(2.5), gelu(-3.5), gelu(-4), gelu(6)
    from math import erf, sqrt
    for got, v in zip(g, [2.5, -3.5, -4.0, 6.0]):
        assert abs(got - 0.5 * v * (1.0 + erf(v / sqrt(2.0)))) < 1e-6
    # the activation is applied after the residual, not before: relu(-3.5) + 1 would be 1, relu(-3.5 + 1) is 0
    assert F.affine_act(x, scale, shift, res, "relu")[0, 0, 0, 1] == 0.0
    # sub-ranges write only the named images / channels
    y = np.full_like(x, 77.0)
    F.affine_act(x, scale, shift, res, "none", None, (1, 2), y)
    assert np.array_equal(y.ravel(), [77.0, 77.0, -5.0, 10.0])


def test_add_hand():
    a = np.array([[[[1.0, -5.0]], [[7.0, 2.5]]]], np.float32)
    b = np.array([[[[0.25, 2.0]], [[-0.5, 4.0]]]], np.float32)
    assert np.array_equal(F.add(a, b, "none").ravel(), [1.25, -3.0, 6.5, 6.5])
    assert np.array_equal(F.add(a, b, "relu").ravel(), [1.25, 0.0, 6.5, 6.5])
    assert np.array_equal(F.add(a, b, "relu6").ravel(), [1.25, 0.0, 6.0, 6.0])
    two = np.concatenate([a, 2 * a])                                       # batch of 2: only image 1 is written
    y = np.full_like(two, -9.0)
    F.add(two, np.concatenate([b, b]), "none", (1, 2), y)
    assert np.array_equal(y[0].ravel(), [-9.0] * 4) and np.array_equal(y[1].ravel(), [2.25, -8.0, 13.5, 9.0])


@pytest.mark.parametrize("act", ["none", "relu", "relu6", "gelu"])
def test_affine_add_act_vs_torch(act):
    x, res, x2 = rnd((3, 5, 4, 6), 50, -4, 4), rnd((3, 5, 4, 6), 51, -4, 4), rnd((3, 5, 4, 6), 52, -4, 4)
    scale, shift = rnd((5,), 53, -2, 2), rnd((5,), 54, -3, 3)
    actf = {"none": lambda v: v, "relu": torch.relu, "relu6": lambda v: torch.clamp(v, 0, 6), "gelu": tF.gelu}[act]
    tx, tr, t2 = [torch.from_numpy(v).double() for v in (x, res, x2)]
    ts, th = torch.from_numpy(scale).double().view(1, 5, 1, 1), torch.from_numpy(shift).double().view(1, 5, 1, 1)
    assert np.abs(F.affine_act(x, scale, shift, res, act) - actf(tx * ts + th + tr).numpy()).max() < 2e-6
    assert np.abs(F.affine_act(x, scale, shift, None, act) - actf(tx * ts + th).numpy()).max() < 2e-6
    assert np.abs(F.add(x, x2, act) - actf(tx + t2).numpy()).max() < 2e-6
    assert np.abs(F.act(x, act) - actf(tx).numpy()).max() < 2e-6


def test_gelu_relu_values():
    x = np.array([[[[-1.0, 0.0, 1.0, 7.0]]]], np.float32)
    assert np.array_equal(F.act(x, "relu").ravel(), [0, 0, 1, 7])
    assert np.array_equal(F.act(x, "relu6").ravel(), [0, 0, 1, 6])
    g = F.act(x, "gelu").ravel()
    assert abs(g[2] - 0.8413447460685429) < 1e-7 and abs(g[0] + 0.15865525393145707) < 1e-7 and g[1] == 0


def test_layernorm_softmax_invariants():
    x = rnd((3, 16, 5, 1), 10, -3, 3)
    g, b = np.ones(16, np.float32), np.zeros(16, np.float32)
    y = F.layernorm(x, None, g, b, 1e-12).astype(np.float64)
    assert np.abs(y.mean(axis=1)).max() < 1e-6 and np.abs(y.var(axis=1) - 1).max() < 1e-5
    s = F.softmax(x)
    assert np.abs(s.astype(np.float64).sum(axis=1) - 1).max() < 1e-6
    assert np.abs(F.softmax(x + np.float32(2.0)) - s).max() < 1e-6
    hand = F.softmax(np.array([0.0, np.log(3.0)], np.float32).reshape(1, 2, 1, 1)).ravel()
    assert np.allclose(hand, [0.25, 0.75], atol=1e-7)


def test_bf16_rounding_hand_table():
    cases = [(1.0 + 2.0 ** -8, 1.0), (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6), (1.0 + 2.0 ** -8 + 2.0 ** -16, 1.0 + 2.0 ** -7),
             (3.0e38, 3.0e38), (-2.0 ** -9 - 1.0, -1.0)]
    x = np.array([c[0] for c in cases], np.float32)
    y = F.round_bf16(x)
    for got, (_, exp) in zip(y[:3], cases[:3]):
        assert got == np.float32(exp)
    assert y[4] == -1.0
    r = rnd((1000,), 11)
    assert np.array_equal(F.round_bf16(r), torch.from_numpy(r).to(torch.bfloat16).to(torch.float32).numpy())
    assert np.array_equal(F.round_bf16(r), synth.bf16_round(r))


def test_hard_swish_sigmoid_values():
    """ReLU6(v + 3) / 6 and v times that: the break points, the linear part and both saturated ends by hand."""
    x = np.array([[-4.0, -3.0, -1.5, 0.0, 1.0, 3.0, 5.0]], np.float32).reshape(1, 7, 1, 1)
    assert np.allclose(F.act(x, "hsigmoid").ravel(), [0.0, 0.0, 0.25, 0.5, 4.0 / 6.0, 1.0, 1.0], rtol=0, atol=1e-7)
    assert np.allclose(F.act(x, "hswish").ravel(), [0.0, 0.0, -0.375, 0.0, 4.0 / 6.0, 3.0, 5.0], rtol=0, atol=1e-7)


def test_scale_concat_avgpool_hand():
    x = np.arange(2 * 2 * 2 * 2, dtype=np.float32).reshape(2, 2, 2, 2)
    g = np.array([[[[2.0]], [[-1.0]]], [[[0.5]], [[0.0]]]], np.float32)          # gate per (image, channel)
    y = F.scale(x, g, "none")
    assert np.array_equal(y[0, 0], 2 * x[0, 0]) and np.array_equal(y[0, 1], -x[0, 1])
    assert np.array_equal(y[1, 0], 0.5 * x[1, 0]) and np.all(y[1, 1] == 0)
    assert np.array_equal(F.scale(x, g, "relu")[0, 1], np.zeros((2, 2), np.float32))
    b = -np.ones((2, 3, 2, 2), np.float32)
    c = F.concat(x, b)
    assert c.shape == (2, 5, 2, 2) and np.array_equal(c[:, :2], x) and np.all(c[:, 2:] == -1)
    # a chunk of channels that straddles the seam writes exactly its own range
    part = np.full((2, 5, 2, 2), 7.0, np.float32)
    F.concat(x, b, None, (1, 3), part)
    assert np.array_equal(part[:, 1], x[:, 1]) and np.all(part[:, 2] == -1) and np.all(part[:, [0, 3, 4]] == 7)
    r = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    assert np.array_equal(F.avgpool(r, 2, 2), np.array([[[[2.5, 4.5], [10.5, 12.5]]]], np.float32))
    assert np.array_equal(F.avgpool(r, 3, 1), np.array([[[[5.0, 6.0], [9.0, 10.0]]]], np.float32))


def test_scale_concat_avgpool_hard_acts_vs_torch():
    x, g, b = rnd((3, 6, 5, 7), 41, -4, 4), rnd((3, 6, 1, 1), 42), rnd((3, 4, 5, 7), 43)
    tx, tg, tb = [torch.from_numpy(v).double() for v in (x, g, b)]
    for act, f in (("none", lambda v: v), ("hswish", tF.hardswish), ("hsigmoid", tF.hardsigmoid)):
        assert np.allclose(F.scale(x, g, act), f(tx * tg).numpy(), rtol=1e-6, atol=1e-7)
        assert np.allclose(F.act(x, act), f(tx).numpy(), rtol=1e-6, atol=1e-7)
    assert np.array_equal(F.concat(x, b), torch.cat([tx, tb], 1).float().numpy())
    for k, s in ((2, 2), (3, 2), (3, 1)):
        assert np.allclose(F.avgpool(x, k, s), tF.avg_pool2d(tx, k, s).numpy(), rtol=1e-6, atol=1e-7)
    w, bias = rnd((5, 6, 1, 1), 44), rnd((5,), 45)
    ref = tF.hardswish(tF.conv2d(tx, torch.from_numpy(w).double(), torch.from_numpy(bias).double())).numpy()
    assert np.allclose(F.conv2d(x, w, bias, None, 1, 0, 1, "hswish"), ref, rtol=1e-6, atol=1e-6)


# ---- library referee (torch CPU, fp64) --------------------------------------------------------
@pytest.mark.parametrize("k,stride,pad,groups,cin,cout", [(3, 1, 1, 1, 5, 7), (3, 2, 1, 1, 4, 6), (7, 2, 3, 1, 3, 8),
                                                           (1, 2, 0, 1, 6, 4), (3, 2, 1, 6, 6, 6), (3, 1, 1, 2, 4, 6)])
def test_conv_vs_torch(k, stride, pad, groups, cin, cout):
    x, w, b = rnd((2, cin, 9, 11), 20), rnd((cout, cin // groups, k, k), 21), rnd((cout,), 22)
    y = F.conv2d(x, w, b, None, stride, pad, groups, "none")
    ref = tF.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double(),
                    stride=stride, padding=pad, groups=groups).numpy()
    assert y.shape == ref.shape and np.abs(y - ref).max() <= 2e-7 * np.abs(ref).max()


def test_gemm_pool_ln_softmax_gelu_vs_torch():
    x, w, b = rnd((5, 37), 30), rnd((11, 37), 31), rnd((11,), 32)
    ref = tF.linear(torch.from_numpy(x).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double()).numpy()
    assert np.abs(F.gemm(x, w, b, None, "none") - ref).max() < 1e-6
    xi = rnd((2, 3, 9, 10), 33)
    for k, s, p in [(3, 2, 1), (2, 2, 0)]:
        ref = tF.max_pool2d(torch.from_numpy(xi), k, s, p).numpy()
        assert np.array_equal(F.maxpool(xi, k, s, p), ref)
    assert np.abs(F.gavgpool(xi).ravel() - xi.astype(np.float64).mean(axis=(2, 3)).ravel()).max() < 1e-7
    xt = rnd((2, 24, 7, 1), 34, -4, 4)
    rows = torch.from_numpy(xt[..., 0].transpose(0, 2, 1).copy()).double()
    g, bt = rnd((24,), 35), rnd((24,), 36)
    ref = tF.layer_norm(rows, (24,), torch.from_numpy(g).double(), torch.from_numpy(bt).double(), 1e-12).numpy()
    got = F.layernorm(xt, None, g, bt, 1e-12)[..., 0].transpose(0, 2, 1)
    assert np.abs(got - ref).max() < 1e-6
    ref = tF.softmax(rows, dim=-1).numpy()
    assert np.abs(F.softmax(xt)[..., 0].transpose(0, 2, 1) - ref).max() < 1e-7
    ref = tF.gelu(torch.from_numpy(xt).double()).numpy()
    assert np.abs(F.act(xt, "gelu") - ref).max() < 1e-6


def test_attention_vs_torch():
    B, H, dh, S = 2, 3, 4, 5
    qkv = rnd((B, 3 * H * dh, S, 1), 40)
    sc = F.bgemm_qk(qkv, H, dh, 0.5)
    p = F.softmax(sc)
    o = F.bgemm_pv(p, qkv, H, dh)
    t = torch.from_numpy(qkv[..., 0]).double()                       # [B, 3D, S]
    q, k, v = [t[:, i * H * dh:(i + 1) * H * dh].reshape(B, H, dh, S) for i in range(3)]
    s_ref = 0.5 * torch.einsum("bhdi,bhdj->bhij", q, k)
    o_ref = torch.einsum("bhij,bhdj->bhdi", torch.softmax(s_ref, -1), v).reshape(B, H * dh, S)
    assert np.abs(sc[..., 0].reshape(B, H, S, S).transpose(0, 1, 3, 2) - s_ref.numpy()).max() < 1e-6
    assert np.abs(o[..., 0] - o_ref.numpy()).max() < 1e-6


# ---- whole graphs -----------------------------------------------------------------------------
def _torch_forward(t, x, params):
    """Independent walk of the same graph with torch CPU fp64 ops."""
    T = {t.input: torch.from_numpy(x).double()}
    P = [torch.from_numpy(p).double() for p in params]
    views = getattr(t, "views", {})
    parts = {}                                       # wider tensor -> {first channel: window}, concatenated when read
    actf = {"none": lambda v: v, "relu": torch.relu, "relu6": lambda v: torch.clamp(v, 0, 6), "gelu": tF.gelu,
            "hswish": tF.hardswish, "hsigmoid": tF.hardsigmoid}
    def read(i):
        if i in views:                               # a prefix of the wider tensor: the windows written so far, in channel order
            base, off = views[i]
            whole = torch.cat([parts[base][k] for k in sorted(parts[base])], dim=1)
            return whole[:, off:off + t.tensors[i][1]]
        if i in parts:
            return torch.cat([parts[i][k] for k in sorted(parts[i])], dim=1)
        return T[i]
    for op in t.ops:
        a = read(op.in0)
        r = read(op.res) if op.res >= 0 else 0
        if op.kind in ("conv", "dwconv"):
            y = actf[op.act](tF.conv2d(a, P[op.w], P[op.bias], stride=op.stride, padding=op.pad, groups=op.groups) + r)
        elif op.kind == "gemm":
            if op.cin == a[0].numel():
                y = tF.linear(a.reshape(a.shape[0], -1), P[op.w], P[op.bias])[:, :, None, None]
            else:
                y = tF.linear(a.permute(0, 2, 3, 1), P[op.w], P[op.bias]).permute(0, 3, 1, 2)
            y = actf[op.act](y + r)
        elif op.kind == "affine":
            y = actf[op.act](a * P[op.scale].view(1, -1, 1, 1) + P[op.shift].view(1, -1, 1, 1) + r)
        elif op.kind == "add":
            y = actf[op.act](a + T[op.in1])
        elif op.kind == "act":
            y = actf[op.act](a)
        elif op.kind == "scale":
            y = actf[op.act](a * T[op.in1])
        elif op.kind == "concat":
            y = torch.cat([a, T[op.in1]], dim=1)
        elif op.kind == "avgpool":
            y = tF.avg_pool2d(a, op.kh, op.stride)
        elif op.kind == "maxpool":
            y = tF.max_pool2d(a, op.kh, op.stride, op.pad)
        elif op.kind == "gavgpool":
            y = a.mean(dim=(2, 3), keepdim=True)
        elif op.kind == "layernorm":
            y = tF.layer_norm((a + r).permute(0, 2, 3, 1), (a.shape[1],), P[op.scale], P[op.shift], op.eps).permute(0, 3, 1, 2)
        elif op.kind == "softmax":
            y = torch.softmax(a, dim=1)
        elif op.kind == "bgemm_qk":
            B, D3, S, _ = a.shape
            H, dh = op.groups, op.cin
            q = a[:, :D3 // 3, :, 0].reshape(B, H, dh, S)
            k = a[:, D3 // 3:2 * D3 // 3, :, 0].reshape(B, H, dh, S)
            y = (op.alpha * torch.einsum("bhdi,bhdj->bhji", q, k)).reshape(B * H, S, S, 1)
        elif op.kind == "bgemm_pv":
            qkv = T[op.in1]
            B, D3, S, _ = qkv.shape
            H, dh = op.groups, op.cout
            v = qkv[:, 2 * D3 // 3:, :, 0].reshape(B, H, dh, S)
            y = torch.einsum("bhji,bhdj->bhdi", a[..., 0].reshape(B, H, S, S), v).reshape(B, H * dh, S, 1)
        else:
            raise ValueError(op.kind)
        T[op.out] = y
        if op.out in views:
            parts.setdefault(views[op.out][0], {})[views[op.out][1]] = y
    return read(t.output).numpy()


def eltwise_mix(dtype="f32", batch=3):
    """A graph with standalone affine (with and without residual), add and act operators."""
    from synth import graphs as G
    b = G._B("eltwise_mix", dtype, batch)
    x = b.tensor(batch, 20, 9, 7)
    y = b.conv(x, 24, 3, 1, 1, "none")
    y = b.affine(y, "relu")
    z = b.conv(y, 24, 1, 1, 0, "none")
    z = b.affine(z, "none", res=y)
    y = b.add(z, y, "relu6")
    y = b.act(y, "gelu")
    y = b.maxpool(y, 3, 2, 1)
    y = b.gavgpool(y)
    y = b.gemm(y, 13, flatten=True)
    return b.done(x, y)


@pytest.mark.parametrize("maker", [synth.toy_cnn, synth.toy_mlp, synth.small_cnn, synth.small_alexnet, synth.small_resnet,
                                   synth.small_mbv2, synth.small_mbv3, synth.small_densenet, synth.small_bert, eltwise_mix])
def test_graph_walk_vs_torch_fp64(maker):
    t = maker("f32")
    x, p = synth.materialise(t, 5)
    y = F.run_tenant(t, x, p)
    ref = _torch_forward(t, x, p)
    # fp32 storage of every intermediate tensor vs an unrounded fp64 pass
    assert np.abs(y - ref).max() <= 2e-5 * np.abs(ref).max()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_channel_windows_are_concatenation(dtype):
    """The same DenseNet-shaped graph written with channel windows of one tensor per block and with a concatenation
    operator per layer: identical outputs, bit for bit, and identical block tensors."""
    from synth import graphs as G
    a = G._densenet("windows", dtype, 2, 40, 8, [2, 3], 12, 2, 10, in_place=True)
    b = G._densenet("copies", dtype, 2, 40, 8, [2, 3], 12, 2, 10, in_place=False)
    assert len(b.ops) - len(a.ops) == 5 and not b.views      # one concatenation per layer fewer
    assert len(a.views) == (1 + 2 + 1) + (1 + 3 + 2)         # per block: the pool's window, one per layer, a prefix for every layer but the first
    xa, pa = synth.materialise(a, 11)
    xb, pb = synth.materialise(b, 11)
    assert np.array_equal(xa, xb) and all(np.array_equal(u, v) for u, v in zip(pa, pb))
    Ta, Tb = F.run_tenant(a, xa, pa, keep_all=True), F.run_tenant(b, xb, pb, keep_all=True)
    assert np.array_equal(Ta[a.output], Tb[b.output])
    blocks_a = [Ta[i] for i in range(len(a.tensors)) if i in {v[0] for v in a.views.values()}]
    last_cat = [Tb[op.out] for op in b.ops if op.kind == "concat"]
    assert np.array_equal(blocks_a[0], last_cat[1]) and np.array_equal(blocks_a[1], last_cat[4])


@pytest.mark.parametrize("maker", [synth.small_cnn, synth.small_resnet, synth.small_mbv2, synth.small_mbv3, synth.small_densenet,
                                   synth.small_bert, eltwise_mix])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_oracle_split_invariance(maker, dtype):
    """Decomposition (Eq. 5) must not change the oracle's own result, bit for bit."""
    t = maker(dtype)
    x, p = synth.materialise(t, 6)
    base = F.run_tenant(t, x, p)
    for axis in ("batch", "cout"):
        for f in (2, 3):
            splits = {}
            for i, op in enumerate(t.ops):
                ok_c = op.kind in ("conv", "dwconv", "gemm", "maxpool", "gavgpool", "affine")
                if axis == "batch" or ok_c:
                    ext = t.batch if axis == "batch" else op.cout
                    if ext >= f:
                        splits[i] = (axis, f)
            assert np.array_equal(F.run_tenant(t, x, p, splits), base)


def test_oracle_chunk_list_invariance():
    """Uneven chunk lists (list_B such as [24, 8], Section 4.2) leave the oracle's result unchanged, bit for bit."""
    for dtype in ("f32", "bf16"):
        t = synth.small_mbv2(dtype, 5)
        x, p = synth.materialise(t, 8)
        base = F.run_tenant(t, x, p)
        splits = {}
        for i, op in enumerate(t.ops):
            if op.kind in ("conv", "dwconv", "gemm") and op.cout >= 4:
                splits[i] = ("cout", [op.cout - 3, 1, 2]) if i % 2 else ("batch", [1, 4])
        assert len(splits) > 4
        assert np.array_equal(F.run_tenant(t, x, p, splits), base)


def test_chunk_ranges():
    assert F.chunk_ranges(32, [24, 8]) == [(0, 24), (24, 32)]        # the paper's list_B example sizes
    assert F.chunk_ranges(7, [1, 1, 5]) == [(0, 1), (1, 2), (2, 7)]
    assert F.chunk_ranges(10, 4) == [(0, 3), (3, 6), (6, 8), (8, 10)]
    assert F.chunk_ranges(8, 2) == [(0, 4), (4, 8)]
    assert sum(b - a for a, b in F.chunk_ranges(1000, 8)) == 1000


@pytest.mark.parametrize("maker", [synth.small_resnet, synth.small_bert, synth.small_mbv2, eltwise_mix])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_run_op_reproduces_the_graph_walk(maker, dtype):
    """run_op on the walk's own tensors returns the walk's tensors, bit for bit."""
    t = maker(dtype)
    x, p = synth.materialise(t, 3)
    T = F.run_tenant(t, x, p, keep_all=True)
    for i, op in enumerate(t.ops):
        assert np.array_equal(F.run_op(t, i, T, p), T[op.out])
