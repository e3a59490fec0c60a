"""ctypes loader and numpy marshalling for the CPU oracle (oracle/vqo.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  No arithmetic of the method lives here; every
function forwards numpy arrays to the C routine of the same name.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

_i64 = C.c_int64
_f32 = C.c_float
_int = C.c_int
_p = C.c_void_p


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        _LIB = C.CDLL(path)
        _LIB.vqo_alpha.restype = _f32
        _LIB.vqo_alpha.argtypes = [_f32, _f32, _f32]
        _LIB.vqo_gelu.restype = _f32
        _LIB.vqo_gelu.argtypes = [_f32]
        _LIB.vqo_x_gelu_erf.restype = C.c_double
        _LIB.vqo_x_gelu_erf.argtypes = [C.c_double]
        _LIB.vqo_shift_exp.restype = C.c_uint32
        _LIB.vqo_shift_exp.argtypes = [C.c_int32, _f32]
        for name in ("vqo_matmul_nt", "vqo_matmul_nn_u8", "vqo_linear", "vqo_linear_absorbed", "vqo_matmul_qk",
                     "vqo_matmul_pv", "vqo_attention_block"):
            getattr(_LIB, name).restype = _i64
    return _LIB


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def qrange(bits, is_unsigned=False):
    lo, hi = _int(), _int()
    rc = lib().vqo_qrange(_int(bits), _int(int(is_unsigned)), C.byref(lo), C.byref(hi))
    if rc:
        raise ValueError("bits out of range")
    return lo.value, hi.value


def quantize(x, step, bits, per_row=False):
    x = _c(x, np.float32)
    rows, cols = x.shape
    step = _c(np.atleast_1d(step), np.float32)
    q = np.empty((rows, cols), np.int8)
    rc = lib().vqo_quantize(_ptr(x), _i64(rows), _i64(cols), _i64(cols), _ptr(step),
                            _int(int(per_row)), _int(bits), _ptr(q))
    assert rc == 0
    return q


def weight_steps(w, bits):
    w = _c(w, np.float32)
    rows, cols = w.shape
    s = np.empty(rows, np.float32)
    rc = lib().vqo_weight_steps(_ptr(w), _i64(rows), _i64(cols), _i64(cols), _int(bits), _ptr(s))
    assert rc == 0
    return s


def dequantize(q, step, per_row=False):
    q = _c(q, np.int8)
    rows, cols = q.shape
    step = _c(np.atleast_1d(step), np.float32)
    x = np.empty((rows, cols), np.float32)
    lib().vqo_dequantize(_ptr(q), _i64(rows), _i64(cols), _ptr(step), _int(int(per_row)), _ptr(x))
    return x


def row_stride_for(cols, storage_bits):
    nbytes = (cols * storage_bits + 7) // 8
    return (nbytes + 15) // 16 * 16


def pack(q, storage_bits, row_stride=None):
    """Pack int8 (signed) or uint8 (unsigned) levels; returns uint8 [rows, row_stride]."""
    q = np.ascontiguousarray(q)
    rows, cols = q.shape
    if row_stride is None:
        row_stride = row_stride_for(cols, storage_bits)
    out = np.empty((rows, row_stride), np.uint8)
    if q.dtype == np.uint8:
        rc = lib().vqo_pack_u8(_ptr(q), _i64(rows), _i64(cols), _int(storage_bits), _ptr(out),
                               _i64(row_stride))
    else:
        q = _c(q, np.int8)
        rc = lib().vqo_pack(_ptr(q), _i64(rows), _i64(cols), _int(storage_bits), _ptr(out),
                            _i64(row_stride))
    if rc:
        raise ValueError("vqo_pack failed: %d" % rc)
    return out


def unpack(packed, cols, storage_bits, unsigned=False):
    packed = _c(packed, np.uint8)
    rows, row_stride = packed.shape
    out = np.empty((rows, cols), np.uint8 if unsigned else np.int8)
    fn = lib().vqo_unpack_u8 if unsigned else lib().vqo_unpack
    rc = fn(_ptr(packed), _i64(rows), _i64(cols), _int(storage_bits), _i64(row_stride), _ptr(out))
    if rc:
        raise ValueError("vqo_unpack failed: %d" % rc)
    return out


def matmul_nt(a, b):
    a = _c(a, np.int8)
    b = _c(b, np.int8)
    M, K = a.shape
    N, K2 = b.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    bad = lib().vqo_matmul_nt(_ptr(a), _ptr(b), _i64(M), _i64(N), _i64(K), _ptr(acc))
    return acc, bad


def matmul_nn_u8(p, v):
    p = _c(p, np.uint8)
    v = _c(v, np.int8)
    M, K = p.shape
    K2, N = v.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    bad = lib().vqo_matmul_nn_u8(_ptr(p), _ptr(v), _i64(M), _i64(N), _i64(K), _ptr(acc))
    return acc, bad


def gelu(y):
    y = _c(np.atleast_1d(y), np.float32)
    g = np.empty_like(y)
    lib().vqo_gelu_array(_ptr(y), _i64(y.size), _ptr(g))
    return g


def gelu_erf(y):
    return np.array([lib().vqo_x_gelu_erf(float(v)) for v in np.atleast_1d(y)], np.float64)


def linear(xq, s_x, wq, s_w, bias=None, act=0, s_y=None, bits_y=4, want_acc=True, want_y=True):
    """Returns dict(acc, y, yq, overflow)."""
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    M, K = xq.shape
    Nout, K2 = wq.shape
    assert K == K2
    s_w = _c(np.atleast_1d(s_w), np.float32)
    per_channel = int(s_w.size > 1)
    if per_channel:
        assert s_w.size == Nout
    if bias is not None:
        bias = _c(bias, np.float32)
        assert bias.size == Nout
    acc = np.empty((M, Nout), np.int32) if want_acc else None
    y = np.empty((M, Nout), np.float32) if want_y else None
    yq = np.empty((M, Nout), np.int8) if s_y is not None else None
    bad = lib().vqo_linear(_ptr(xq), _i64(M), _i64(K), _f32(s_x), _ptr(wq), _i64(Nout), _ptr(s_w),
                           _int(per_channel), _ptr(bias), _int(act), _ptr(acc), _ptr(y),
                           _f32(0.0 if s_y is None else s_y), _int(bits_y), _ptr(yq))
    assert bad >= 0
    return dict(acc=acc, y=y, yq=yq, overflow=bad)


def absorb(s_x, s_w, bias, s_y, bits, Nout=None):
    """Equivalent integer bias and integer thresholds of the absorbed mode.  Returns (b_int [Nout], thr [Nout, 2^bits-1])."""
    s_w = _c(np.atleast_1d(s_w), np.float32)
    s_y = _c(np.atleast_1d(s_y), np.float32)
    if Nout is None:
        Nout = max(s_w.size, s_y.size, 1 if bias is None else np.size(bias))
    if bias is not None:
        bias = _c(bias, np.float32)
        assert bias.size == Nout
    assert s_w.size in (1, Nout) and s_y.size in (1, Nout)
    lo, hi = qrange(bits)
    b_int = np.empty(Nout, np.int32)
    thr = np.empty((Nout, hi - lo), np.int32)
    rc = lib().vqo_absorb(_f32(s_x), _ptr(s_w), _int(int(s_w.size > 1)), _ptr(bias), _i64(Nout), _ptr(s_y),
                          _int(int(s_y.size > 1)), _int(bits), _ptr(b_int), _ptr(thr))
    assert rc == 0
    return b_int, thr


def linear_absorbed(xq, wq, b_int, thr, bits, want_acc=True):
    """Integer-only linear + quantizer.  Returns dict(acc, yq, overflow)."""
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    M, K = xq.shape
    Nout, K2 = wq.shape
    assert K == K2
    lo, hi = qrange(bits)
    thr = _c(thr, np.int32)
    assert thr.shape == (Nout, hi - lo)
    if b_int is not None:
        b_int = _c(b_int, np.int32)
        assert b_int.size == Nout
    acc = np.empty((M, Nout), np.int32) if want_acc else None
    yq = np.empty((M, Nout), np.int8)
    bad = lib().vqo_linear_absorbed(_ptr(xq), _i64(M), _i64(K), _ptr(wq), _i64(Nout), _ptr(b_int), _ptr(thr),
                                    _int(bits), _ptr(acc), _ptr(yq))
    assert bad >= 0
    return dict(acc=acc, yq=yq, overflow=bad)


def alpha(s_q, s_k, scale):
    return np.float32(lib().vqo_alpha(_f32(s_q), _f32(s_k), _f32(scale)))


def shift_exp(d, alpha_):
    return int(lib().vqo_shift_exp(C.c_int32(int(d)), _f32(alpha_)))


def softmax_row(s, alpha_, pmax):
    """Returns (p levels uint8 [n], e uint32 [n], sum int)."""
    s = _c(s, np.int32)
    n = s.size
    p = np.empty(n, np.uint8)
    e = np.empty(n, np.uint32)
    tot = C.c_uint64()
    lib().vqo_softmax_row(_ptr(s), _i64(n), _f32(alpha_), _int(pmax), _ptr(p), _ptr(e), C.byref(tot))
    return p, e, tot.value


def softmax_true(s, a, pmax):
    s = _c(s, np.int32)
    n = s.size
    p = np.empty(n, np.uint8)
    prob = np.empty(n, np.float64)
    lib().vqo_x_softmax_true(_ptr(s), _i64(n), C.c_double(a), _int(pmax), _ptr(p), _ptr(prob))
    return p, prob


def matmul_qk(q, k, s_q, s_k, scale, bits_p, want_s=True, want_p=True):
    """q, k: int8 [B, H, N, dh].  Returns dict(s_acc [B,H,N,N] int32, p [B,H,N,N] uint8)."""
    q = _c(q, np.int8)
    k = _c(k, np.int8)
    B, H, N, dh = q.shape
    assert k.shape == q.shape
    s_acc = np.empty((B, H, N, N), np.int32) if want_s else None
    p = np.empty((B, H, N, N), np.uint8) if want_p else None
    bad = lib().vqo_matmul_qk(_ptr(q), _ptr(k), _i64(B), _i64(H), _i64(N), _i64(dh), _f32(s_q),
                              _f32(s_k), _f32(scale), _int(bits_p), _ptr(s_acc), _ptr(p))
    assert bad == 0
    return dict(s_acc=s_acc, p=p)


def matmul_pv(p, v, s_p, s_v, s_o=None, bits_o=4):
    """p: uint8 [B,H,N,N]; v: int8 [B,H,N,dh].  Returns dict(o_acc [B,H,N,dh], o [B*N,H*dh], oq)."""
    p = _c(p, np.uint8)
    v = _c(v, np.int8)
    B, H, N, dh = v.shape
    assert p.shape == (B, H, N, N)
    o_acc = np.empty((B, H, N, dh), np.int32)
    o = np.empty((B * N, H * dh), np.float32)
    oq = np.empty((B * N, H * dh), np.int8) if s_o is not None else None
    bad = lib().vqo_matmul_pv(_ptr(p), _ptr(v), _i64(B), _i64(H), _i64(N), _i64(dh), _f32(s_p),
                              _f32(s_v), _ptr(o_acc), _ptr(o), _f32(0.0 if s_o is None else s_o),
                              _int(bits_o), _ptr(oq))
    assert bad == 0
    return dict(o_acc=o_acc, o=o, oq=oq)


class _Block(C.Structure):
    _fields_ = [("D", _i64), ("H", _i64), ("N", _i64), ("hidden", _i64),
                ("bits_a", C.c_int32), ("bits_p", C.c_int32),
                ("w_qkv", _p), ("sw_qkv", _p), ("b_qkv", _p),
                ("w_proj", _p), ("sw_proj", _p), ("b_proj", _p),
                ("w_fc1", _p), ("sw_fc1", _p), ("b_fc1", _p),
                ("w_fc2", _p), ("sw_fc2", _p), ("b_fc2", _p),
                ("s_x", _f32), ("s_q", _f32), ("s_k", _f32), ("s_v", _f32), ("s_o", _f32),
                ("s_x2", _f32), ("s_h", _f32), ("scale", _f32)]


class _Dumps(C.Structure):
    _fields_ = [("q", _p), ("k", _p), ("v", _p), ("p", _p), ("o", _p), ("y_attn", _p),
                ("x2", _p), ("h", _p)]


def _make_block(dims, weights, steps, bits_a, bits_p):
    """The C descriptor of a block; `keep` holds the arrays it points to."""
    D, H, N, hidden = dims["D"], dims["H"], dims["N"], dims.get("hidden", 0)
    keep = {}

    def w(name, shape):
        a = _c(weights[name], np.int8)
        assert a.shape == shape, (name, a.shape, shape)
        keep[name] = a
        return _ptr(a)

    def f(name, n):
        a = _c(weights[name], np.float32)
        assert a.size == n, (name, a.size, n)
        keep[name] = a
        return _ptr(a)

    blk = _Block()
    blk.D, blk.H, blk.N, blk.hidden = D, H, N, hidden
    blk.bits_a, blk.bits_p = bits_a, bits_p
    blk.w_qkv, blk.sw_qkv, blk.b_qkv = w("w_qkv", (3 * D, D)), f("sw_qkv", 3 * D), f("b_qkv", 3 * D)
    blk.w_proj, blk.sw_proj, blk.b_proj = w("w_proj", (D, D)), f("sw_proj", D), f("b_proj", D)
    if hidden:
        blk.w_fc1, blk.sw_fc1, blk.b_fc1 = w("w_fc1", (hidden, D)), f("sw_fc1", hidden), f("b_fc1", hidden)
        blk.w_fc2, blk.sw_fc2, blk.b_fc2 = w("w_fc2", (D, hidden)), f("sw_fc2", D), f("b_fc2", D)
    for name in ("s_x", "s_q", "s_k", "s_v", "s_o", "scale"):
        setattr(blk, name, float(steps[name]))
    blk.s_x2 = float(steps.get("s_x2", 0.0))
    blk.s_h = float(steps.get("s_h", 0.0))
    return blk, keep


class _QkLn(C.Structure):
    _fields_ = [("gamma", _p), ("beta", _p), ("eps", _f32)]


def attention_block(xq, B, dims, weights, steps, bits_a=4, bits_p=4, dumps=True, dump_p=False,
                    threads=None, qkln=None):
    """Run the whole chain on the CPU.

    xq: int8 [B*N, D].  dims: dict(D, H, N, hidden).  weights: dict of int8 level matrices
    w_qkv/w_proj[/w_fc1/w_fc2], fp32 step vectors sw_* and fp32 biases b_*.
    steps: dict(s_x, s_q, s_k, s_v, s_o, s_x2, s_h, scale).
    qkln: None, or dict(gamma [2D], beta [2D], eps): Q and K go through a per-head LayerNorm
    quantizer (steps s_q, s_k) instead of the plain requantization.
    Returns dict with y [B*N, D] fp32 and (if dumps) the intermediates.
    """
    D, H, N, hidden = dims["D"], dims["H"], dims["N"], dims.get("hidden", 0)
    dh = D // H
    xq = _c(xq, np.int8)
    assert xq.shape == (B * N, D)
    blk, keep = _make_block(dims, weights, steps, bits_a, bits_p)

    y = np.empty((B * N, D), np.float32)
    out = dict(y=y)
    dmp = None
    if dumps:
        dmp = _Dumps()
        out["q"] = np.empty((B, H, N, dh), np.int8)
        out["k"] = np.empty((B, H, N, dh), np.int8)
        out["v"] = np.empty((B, H, N, dh), np.int8)
        out["o"] = np.empty((B * N, D), np.int8)
        out["y_attn"] = np.empty((B * N, D), np.float32)
        dmp.q, dmp.k, dmp.v = _ptr(out["q"]), _ptr(out["k"]), _ptr(out["v"])
        dmp.o, dmp.y_attn = _ptr(out["o"]), _ptr(out["y_attn"])
        if dump_p:
            out["p"] = np.empty((B, H, N, N), np.uint8)
            dmp.p = _ptr(out["p"])
        if hidden:
            out["x2"] = np.empty((B * N, D), np.int8)
            out["h"] = np.empty((B * N, hidden), np.int8)
            dmp.x2, dmp.h = _ptr(out["x2"]), _ptr(out["h"])
    L = lib()
    old = L.vqo_num_threads()
    if threads is not None:
        L.vqo_set_num_threads(_int(threads))
    try:
        if qkln is None:
            bad = L.vqo_attention_block(C.byref(blk), _ptr(xq), _i64(B), _ptr(y),
                                        C.byref(dmp) if dmp is not None else None)
        else:
            ql = _QkLn()
            keep["qk_gamma"], keep["qk_beta"] = _c(qkln["gamma"], np.float32), _c(qkln["beta"], np.float32)
            assert keep["qk_gamma"].size == 2 * D and keep["qk_beta"].size == 2 * D
            ql.gamma, ql.beta, ql.eps = _ptr(keep["qk_gamma"]), _ptr(keep["qk_beta"]), float(qkln["eps"])
            L.vqo_attention_block_qkln.restype = _i64
            bad = L.vqo_attention_block_qkln(C.byref(blk), C.byref(ql), _ptr(xq), _i64(B), _ptr(y),
                                             C.byref(dmp) if dmp is not None else None)
    finally:
        if threads is not None:
            L.vqo_set_num_threads(_int(old))
    assert bad == 0, "int32 overflow or bad shape in oracle chain: %d" % bad
    out["threads"] = threads if threads is not None else old
    return out


def linear_dequant_first(xq, s_x, wq, s_w, bias=None):
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    M, K = xq.shape
    Nout = wq.shape[0]
    s_w = _c(np.atleast_1d(s_w), np.float32)
    if bias is not None:
        bias = _c(bias, np.float32)
    y = np.empty((M, Nout), np.float64)
    lib().vqo_x_linear_dequant_first(_ptr(xq), _i64(M), _i64(K), _f32(s_x), _ptr(wq), _i64(Nout),
                                     _ptr(s_w), _int(int(s_w.size > 1)), _ptr(bias), _ptr(y))
    return y


def num_threads():
    return lib().vqo_num_threads()


def layernorm_quantize(x, gamma, beta, eps, step, bits, res=None, want_sum=False):
    """Returns dict(q int8 [rows, cols], mu, m2 [rows], sum (x + res) if asked)."""
    x = _c(x, np.float32)
    rows, cols = x.shape
    gamma, beta = _c(gamma, np.float32), _c(beta, np.float32)
    res = None if res is None else _c(res, np.float32)
    q = np.empty((rows, cols), np.int8)
    mu, m2 = np.empty(rows, np.float32), np.empty(rows, np.float32)
    total = np.empty((rows, cols), np.float32) if want_sum else None
    rc = lib().vqo_layernorm_quantize(_ptr(x), _ptr(res), _ptr(total), _i64(rows), _i64(cols), _i64(cols),
                                      _ptr(gamma), _ptr(beta), _f32(eps), _f32(step), _int(bits), _ptr(q),
                                      _ptr(mu), _ptr(m2))
    assert rc == 0
    return dict(q=q, mu=mu, m2=m2, sum=total)


def x_layernorm(x, gamma, beta, eps):
    """Cross-check: direct two-pass LayerNorm in double."""
    x = _c(x, np.float32)
    rows, cols = x.shape
    y = np.empty((rows, cols), np.float64)
    lib().vqo_x_layernorm(_ptr(x), _i64(rows), _i64(cols), _i64(cols), _ptr(_c(gamma, np.float32)),
                          _ptr(_c(beta, np.float32)), C.c_double(eps), _ptr(y))
    return y


class _LnParams(C.Structure):
    _fields_ = [("g1", _p), ("b1", _p), ("g2", _p), ("b2", _p), ("eps", _f32)]


def vit_block_preln(x, B, dims, weights, steps, ln, bits_a=4, bits_p=4, threads=None):
    """Pre-LayerNorm block on the fp32 residual stream.  x: fp32 [B*N, D]; ln: dict(g1, b1, g2, b2, eps).
    Returns dict(y, x1 fp32; xq, x2, h, o levels)."""
    D, H, N, hidden = dims["D"], dims["H"], dims["N"], dims["hidden"]
    x = _c(x, np.float32)
    assert x.shape == (B * N, D)
    blk, keep = _make_block(dims, weights, steps, bits_a, bits_p)
    lp = _LnParams()
    for k in ("g1", "b1", "g2", "b2"):
        keep[k] = _c(ln[k], np.float32)
        assert keep[k].size == D
        setattr(lp, k, _ptr(keep[k]))
    lp.eps = float(ln["eps"])
    out = dict(y=np.empty((B * N, D), np.float32), x1=np.empty((B * N, D), np.float32),
               xq=np.empty((B * N, D), np.int8), x2=np.empty((B * N, D), np.int8),
               h=np.empty((B * N, hidden), np.int8), o=np.empty((B * N, D), np.int8))
    dmp = _Dumps()
    dmp.o = _ptr(out["o"])
    L = lib()
    L.vqo_vit_block_preln.restype = _i64
    old = L.vqo_num_threads()
    if threads is not None:
        L.vqo_set_num_threads(_int(threads))
    try:
        bad = L.vqo_vit_block_preln(C.byref(blk), C.byref(lp), _ptr(x), _i64(B), _ptr(out["y"]), _ptr(out["x1"]),
                                    _ptr(out["xq"]), _ptr(out["x2"]), _ptr(out["h"]), C.byref(dmp))
    finally:
        if threads is not None:
            L.vqo_set_num_threads(_int(old))
    assert bad == 0, "int32 overflow or bad shape in oracle chain: %d" % bad
    return out
