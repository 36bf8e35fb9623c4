"""Plain CPU forward pass of a tenant graph -- TEST INFRASTRUCTURE ONLY.

The regulated execution (operator chunks, Eq. 5; segments and clusters,
Section 4.3) must give each tenant exactly the result of its ordinary
forward pass, so the oracle is that forward pass: walk the operator list
M_n = [O_n,1 ...] (Section 4.1) in order and evaluate each operator's
textbook definition (``oracle_ops.c``: direct loops, one fp64 accumulator per
output element).  Tensors are float32 numpy arrays in logical NCHW order.  In
bf16 tenants every tensor an operator writes is rounded to bfloat16 (nearest
even) after the operator, which models bfloat16 storage of graph tensors.

``splits`` lets a test evaluate an operator chunk by chunk (batch or
output-channel sub-ranges) to show that decomposition leaves the oracle's
own result unchanged.
"""
import ctypes
import numpy as np

from .build import build

_ACT = {"none": 0, "relu": 1, "relu6": 2, "gelu": 3, "hswish": 4, "hsigmoid": 5}
_lib = None
_fp = ctypes.POINTER(ctypes.c_float)


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_bgemm_qk.argtypes = [_fp, _fp] + [ctypes.c_int] * 4 + [ctypes.c_double] + [ctypes.c_int] * 2
        _lib.orc_layernorm.argtypes = [_fp] * 5 + [ctypes.c_int] * 3 + [ctypes.c_double] + [ctypes.c_int] * 2
        _lib.orc_round_bf16.argtypes = [_fp, ctypes.c_size_t]
        _lib.orc_add.argtypes = [_fp, _fp, _fp, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t]
        _lib.orc_act.argtypes = [_fp, _fp, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t]
    return _lib


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_fp)


def round_bf16(a):
    a = np.ascontiguousarray(a, dtype=np.float32).copy()
    lib().orc_round_bf16(_p(a), a.size)
    return a


def chunk_ranges(extent, factor):
    """Decomposition of an extent into contiguous chunks whose sizes sum to the
    extent (Eq. 5).  ``factor`` is a chunk count (even chunks; the first
    ``extent % factor`` are one element longer) or the list of chunk sizes
    itself (list_B of Section 4.2)."""
    if isinstance(factor, (list, tuple)):
        assert sum(factor) == extent and all(sz >= 1 for sz in factor)
        out, lo = [], 0
        for sz in factor:
            out.append((lo, lo + sz))
            lo += sz
        return out
    out, lo = [], 0
    for i in range(factor):
        sz = extent // factor + (1 if i < extent % factor else 0)
        out.append((lo, lo + sz))
        lo += sz
    return out


# ---- single operators on numpy arrays --------------------------------------------------------
def conv2d(x, w, b, res, stride, pad, groups, act, n_rng=None, c_rng=None, out=None):
    N, C, H, W = x.shape
    Co, _, kh, kw = w.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    y = np.zeros((N, Co, Ho, Wo), np.float32) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    c_lo, c_hi = c_rng or (0, Co)
    lib().orc_conv2d(_p(x), _p(w), _p(b), _p(res), _p(y), N, C, H, W, Co, kh, kw, stride, pad, groups,
                     _ACT[act], n_lo, n_hi, c_lo, c_hi)
    return y


def gemm(x, w, b, res, act, r_rng=None, o_rng=None, out=None):
    rows, K = x.shape
    No = w.shape[0]
    y = np.zeros((rows, No), np.float32) if out is None else out
    r_lo, r_hi = r_rng or (0, rows)
    o_lo, o_hi = o_rng or (0, No)
    lib().orc_gemm(_p(x), _p(w), _p(b), _p(res), _p(y), rows, K, No, _ACT[act], r_lo, r_hi, o_lo, o_hi)
    return y


def maxpool(x, k, stride, pad, n_rng=None, c_rng=None, out=None):
    N, C, H, W = x.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    y = np.zeros((N, C, Ho, Wo), np.float32) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    c_lo, c_hi = c_rng or (0, C)
    lib().orc_maxpool(_p(x), _p(y), N, C, H, W, k, stride, pad, n_lo, n_hi, c_lo, c_hi)
    return y


def gavgpool(x, n_rng=None, c_rng=None, out=None):
    N, C, H, W = x.shape
    y = np.zeros((N, C, 1, 1), np.float32) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    c_lo, c_hi = c_rng or (0, C)
    lib().orc_gavgpool(_p(x), _p(y), N, C, H, W, n_lo, n_hi, c_lo, c_hi)
    return y


def affine_act(x, scale, shift, res, act, n_rng=None, c_rng=None, out=None):
    N, C, H, W = x.shape
    y = np.zeros_like(x) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    c_lo, c_hi = c_rng or (0, C)
    lib().orc_affine_act(_p(x), _p(scale), _p(shift), _p(res), _p(y), N, C, H * W, _ACT[act],
                         n_lo, n_hi, c_lo, c_hi)
    return y


def scale(x, gate, act, n_rng=None, c_rng=None, out=None):
    N, C, H, W = x.shape
    y = np.zeros_like(x) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    c_lo, c_hi = c_rng or (0, C)
    lib().orc_scale(_p(x), _p(gate), _p(y), N, C, H * W, _ACT[act], n_lo, n_hi, c_lo, c_hi)
    return y


def concat(a, b, n_rng=None, c_rng=None, out=None):
    N, Ca, H, W = a.shape
    Cb = b.shape[1]
    y = np.zeros((N, Ca + Cb, H, W), np.float32) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    c_lo, c_hi = c_rng or (0, Ca + Cb)
    lib().orc_concat(_p(a), _p(b), _p(y), N, Ca, Cb, H * W, n_lo, n_hi, c_lo, c_hi)
    return y


def avgpool(x, k, stride, n_rng=None, c_rng=None, out=None):
    N, C, H, W = x.shape
    y = np.zeros((N, C, (H - k) // stride + 1, (W - k) // stride + 1), np.float32) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    c_lo, c_hi = c_rng or (0, C)
    lib().orc_avgpool(_p(x), _p(y), N, C, H, W, k, stride, n_lo, n_hi, c_lo, c_hi)
    return y


def add(a, b, act, n_rng=None, out=None):
    y = np.zeros_like(a) if out is None else out
    per = a[0].size
    n_lo, n_hi = n_rng or (0, a.shape[0])
    lib().orc_add(_p(a), _p(b), _p(y), _ACT[act], n_lo * per, n_hi * per)
    return y


def act(x, kind, n_rng=None, out=None):
    y = np.zeros_like(x) if out is None else out
    per = x[0].size
    n_lo, n_hi = n_rng or (0, x.shape[0])
    lib().orc_act(_p(x), _p(y), _ACT[kind], n_lo * per, n_hi * per)
    return y


def layernorm(x, res, gamma, beta, eps, n_rng=None, out=None):
    N, C, H, W = x.shape
    y = np.zeros_like(x) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    lib().orc_layernorm(_p(x), _p(res), _p(gamma), _p(beta), _p(y), N, C, H * W, float(eps), n_lo, n_hi)
    return y


def softmax(x, n_rng=None, out=None):
    N, C, H, W = x.shape
    y = np.zeros_like(x) if out is None else out
    n_lo, n_hi = n_rng or (0, N)
    lib().orc_softmax(_p(x), _p(y), N, C, H * W, n_lo, n_hi)
    return y


def bgemm_qk(qkv, heads, dh, alpha, b_rng=None, out=None):
    B, _, S, _ = qkv.shape
    y = np.zeros((B * heads, S, S, 1), np.float32) if out is None else out
    b_lo, b_hi = b_rng or (0, B)
    lib().orc_bgemm_qk(_p(qkv), _p(y), B, heads, dh, S, float(alpha), b_lo, b_hi)
    return y


def bgemm_pv(p, qkv, heads, dh, b_rng=None, out=None):
    B, _, S, _ = qkv.shape
    y = np.zeros((B, heads * dh, S, 1), np.float32) if out is None else out
    b_lo, b_hi = b_rng or (0, B)
    lib().orc_bgemm_pv(_p(p), _p(qkv), _p(y), B, heads, dh, S, b_lo, b_hi)
    return y


# ---- graph walker ------------------------------------------------------------------------------
def _eval_op(t, op, T, P, y, n_rng, c_rng):
    """Evaluate operator ``op`` on batch items n_rng and output channels c_rng, writing into y."""
    x = T[op.in0]
    res = T[op.res] if op.res >= 0 else None
    B = t.batch
    k = op.kind
    if k in ("conv", "dwconv"):
        conv2d(x, P[op.w], P[op.bias], res, op.stride, op.pad, op.groups, op.act, n_rng, c_rng, y)
    elif k == "gemm":
        n, c, h, w = x.shape
        if op.cin == c * h * w and h * w > 1:          # flatten in (c,h,w) order, one row per item
            rows, rr = x.reshape(n, -1), n_rng
            gemm(rows, P[op.w], P[op.bias], None if res is None else res.reshape(n, -1), op.act,
                 rr, c_rng, y.reshape(n, -1))
        else:                                            # per position: rows are (n,h,w), features c
            rows = np.ascontiguousarray(x.transpose(0, 2, 3, 1)).reshape(-1, c)
            r2 = None if res is None else np.ascontiguousarray(res.transpose(0, 2, 3, 1)).reshape(-1, op.cout)
            per = h * w
            rr = None if n_rng is None else (n_rng[0] * per, n_rng[1] * per)
            o_lo, o_hi = c_rng or (0, op.cout)
            r_lo, r_hi = rr or (0, rows.shape[0])
            tmp = gemm(rows, P[op.w], P[op.bias], r2, op.act, rr, c_rng)
            tmp = tmp.reshape(n, h, w, op.cout).transpose(0, 3, 1, 2)
            nl, nh = n_rng or (0, n)
            y[nl:nh, o_lo:o_hi] = tmp[nl:nh, o_lo:o_hi]
    elif k == "maxpool":
        maxpool(x, op.kh, op.stride, op.pad, n_rng, c_rng, y)
    elif k == "gavgpool":
        gavgpool(x, n_rng, c_rng, y)
    elif k == "affine":
        affine_act(x, P[op.scale], P[op.shift], res, op.act, n_rng, c_rng, y)
    elif k == "scale":
        scale(x, T[op.in1], op.act, n_rng, c_rng, y)
    elif k == "concat":
        concat(x, T[op.in1], n_rng, c_rng, y)
    elif k == "avgpool":
        avgpool(x, op.kh, op.stride, n_rng, c_rng, y)
    elif k == "add":
        add(x, T[op.in1], op.act, n_rng, y)
    elif k == "act":
        act(x, op.act, n_rng, y)
    elif k == "layernorm":
        layernorm(x, res, P[op.scale], P[op.shift], op.eps, n_rng, y)
    elif k == "softmax":
        per = x.shape[0] // B
        rr = None if n_rng is None else (n_rng[0] * per, n_rng[1] * per)
        softmax(x, rr, y)
    elif k == "bgemm_qk":
        bgemm_qk(x, op.groups, op.cin, op.alpha, n_rng, y)
    elif k == "bgemm_pv":
        bgemm_pv(x, T[op.in1], op.groups, op.cout, n_rng, y)
    else:
        raise ValueError(k)


def run_op(t, i, tensors, params):
    """Operator i of the tenant evaluated on the given tensor list (float32 NCHW arrays; only the operator's own
    inputs are read), with bfloat16 storage of the result in bf16 tenants.  Lets a test check one operator on inputs
    that did not come from the oracle's own earlier operators."""
    op = t.ops[i]
    P = [np.ascontiguousarray(p, dtype=np.float32) for p in params]
    T = [None if a is None else np.ascontiguousarray(a, dtype=np.float32) for a in tensors]
    y = np.zeros(t.tensors[op.out], np.float32)
    _eval_op(t, op, T, P, y, None, None)
    if t.dtype == "bf16":
        lib().orc_round_bf16(_p(y), y.size)
    return y


def run_tenant(t, x, params, splits=None, keep_all=False):
    """Forward pass.  ``splits`` maps op index -> (axis, factor), axis in {'batch','cout'}.
    Returns the output tensor (or the list of all tensors with keep_all).

    A tensor listed in ``t.views`` is a channel window of a wider tensor: writing it writes those channels of the wider
    tensor, reading it reads them (that is all a concatenation along channels is)."""
    views = getattr(t, "views", {})
    T = [None] * len(t.tensors)
    T[t.input] = np.ascontiguousarray(x, dtype=np.float32)
    P = [np.ascontiguousarray(p, dtype=np.float32) for p in params]

    def window(i):
        base, off = views[i]
        if T[base] is None:
            T[base] = np.zeros(t.tensors[base], np.float32)
        return T[base][:, off:off + t.tensors[i][1]]
    for i, op in enumerate(t.ops):
        for src in (op.in0, op.in1, op.res):
            if src in views:
                T[src] = np.ascontiguousarray(window(src))
        y = np.zeros(t.tensors[op.out], np.float32)
        axis, f = (splits or {}).get(i, ("none", 1))
        if axis == "batch":
            for r in chunk_ranges(t.batch, f):
                _eval_op(t, op, T, P, y, r, None)
        elif axis == "cout":
            for r in chunk_ranges(op.cout, f):
                _eval_op(t, op, T, P, y, None, r)
        else:
            _eval_op(t, op, T, P, y, None, None)
        if t.dtype == "bf16":
            lib().orc_round_bf16(_p(y), y.size)
        T[op.out] = y
        if op.out in views:
            window(op.out)[...] = y
    if keep_all:
        for i in views:
            T[i] = np.ascontiguousarray(window(i))
    return T if keep_all else T[t.output]
