"""Thin Python binding of libvitq.so (see include/vitq.h): argument marshalling only.

Every function has the name and the argument order of its C entry point; torch tensors supply
device memory and the current torch stream supplies the HIP stream.  Nothing is computed here,
and there is no fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvitq.so")

STATUS_NAMES = ["VQ_OK", "VQ_ERR_NULL", "VQ_ERR_SHAPE", "VQ_ERR_BITS", "VQ_ERR_STRIDE", "VQ_ERR_STEP",
                "VQ_ERR_UNSUPPORTED", "VQ_ERR_WORKSPACE", "VQ_ERR_HIP"]

EXPORTS = ["vq_status_string", "vq_weight_steps", "vq_quantize", "vq_linear", "vq_matmul_qk",
           "vq_matmul_pv", "vq_attention_block_workspace", "vq_attention_block",
           "vq_prepack_weight_bytes", "vq_prepack_weight", "vq_linear_prepacked", "vq_layernorm_quantize",
           "vq_vit_block_workspace", "vq_vit_block", "vq_qkv_headnorm", "vq_absorb_thresholds",
           "vq_linear_absorbed", "vq_recode_e3m2_bytes", "vq_recode_e3m2", "vq_linear_e3m2", "vq_vit_encoder_workspace", "vq_vit_encoder", "vq_attention_block_static", "vq_probe_mfma_i8",
           "vq_probe_gelu_distance"]


class VitqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__("%s failed: %s (%s)" % (where, name, status_string(status)))


class vq_qmat(C.Structure):
    _fields_ = [("data", C.c_void_p), ("bits", C.c_int32), ("storage_bits", C.c_int32),
                ("is_unsigned", C.c_int32), ("reserved", C.c_int32),
                ("rows", C.c_int64), ("cols", C.c_int64), ("row_stride", C.c_int64)]


class vq_block_desc(C.Structure):
    _fields_ = [("D", C.c_int32), ("H", C.c_int32), ("N", C.c_int32), ("hidden", C.c_int32),
                ("bits_a", C.c_int32), ("bits_p", C.c_int32), ("storage_a", C.c_int32),
                ("reserved", C.c_int32),
                ("w_qkv", vq_qmat), ("w_proj", vq_qmat), ("w_fc1", vq_qmat), ("w_fc2", vq_qmat),
                ("sw_qkv", C.c_void_p), ("b_qkv", C.c_void_p),
                ("sw_proj", C.c_void_p), ("b_proj", C.c_void_p),
                ("sw_fc1", C.c_void_p), ("b_fc1", C.c_void_p),
                ("sw_fc2", C.c_void_p), ("b_fc2", C.c_void_p),
                ("s_x", C.c_float), ("s_q", C.c_float), ("s_k", C.c_float), ("s_v", C.c_float),
                ("s_o", C.c_float), ("s_x2", C.c_float), ("s_h", C.c_float), ("scale", C.c_float),
                ("dump_qkv", C.c_void_p), ("dump_o", C.c_void_p), ("dump_x2", C.c_void_p),
                ("dump_h", C.c_void_p), ("stage_events", C.POINTER(C.c_void_p)),
                ("wp_qkv", C.c_void_p), ("wp_proj", C.c_void_p), ("wp_fc1", C.c_void_p),
                ("wp_fc2", C.c_void_p), ("qk_gamma", C.c_void_p), ("qk_beta", C.c_void_p),
                ("qk_eps", C.c_float), ("reserved2", C.c_int32)]


class vq_preln_desc(C.Structure):
    _fields_ = [("block", vq_block_desc), ("ln1_gamma", C.c_void_p), ("ln1_beta", C.c_void_p),
                ("ln2_gamma", C.c_void_p), ("ln2_beta", C.c_void_p), ("ln_eps", C.c_float),
                ("reserved", C.c_int32), ("dump_xq", C.c_void_p), ("dump_x1", C.c_void_p)]


_lib = None


def lib():
    """Load libvitq.so; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libvitq.so is not built: run `python -c 'import __graft_entry__ as g; "
                              "g.build()'` (or paper_2504_18547_amd/build.py) first")
        _lib = C.CDLL(LIB_PATH)
        _lib.vq_status_string.restype = C.c_char_p
        _lib.vq_status_string.argtypes = [C.c_int]
        qp = C.POINTER(vq_qmat)
        vp = C.c_void_p
        _lib.vq_weight_steps.argtypes = [vp, C.c_int64, C.c_int64, C.c_int64, C.c_int32, vp, vp]
        _lib.vq_quantize.argtypes = [vp, C.c_int64, C.c_int64, C.c_int64, C.c_float, vp, qp, vp]
        _lib.vq_linear.argtypes = [qp, C.c_float, qp, vp, C.c_int32, vp, C.c_int32, vp, vp, C.c_float, qp, vp]
        _lib.vq_matmul_qk.argtypes = [qp, qp, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_float,
                                      C.c_float, vp, qp, vp]
        _lib.vq_matmul_pv.argtypes = [qp, qp, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_float, vp, vp,
                                      C.c_float, qp, vp]
        _lib.vq_attention_block_workspace.argtypes = [C.POINTER(vq_block_desc), C.c_int64,
                                                      C.POINTER(C.c_size_t)]
        _lib.vq_attention_block.argtypes = [C.POINTER(vq_block_desc), qp, C.c_int64, vp, vp, C.c_size_t, vp]
        _lib.vq_attention_block_static.argtypes = [C.POINTER(vq_block_desc), qp, C.c_int64, vp, vp]
        _lib.vq_probe_mfma_i8.argtypes = [C.c_int32, vp, C.POINTER(C.c_double), vp]
        _lib.vq_probe_gelu_distance.argtypes = [vp, vp]
        _lib.vq_prepack_weight_bytes.argtypes = [qp, C.POINTER(C.c_size_t)]
        _lib.vq_prepack_weight.argtypes = [qp, vp, C.c_size_t, vp]
        _lib.vq_linear_prepacked.argtypes = [qp, C.c_float, qp, vp, vp, C.c_int32, vp, C.c_int32, vp, vp,
                                             C.c_float, qp, vp]
        _lib.vq_absorb_thresholds.argtypes = [C.c_float, vp, C.c_int32, vp, C.c_int64, vp, C.c_int32, C.c_int32, vp, vp]
        _lib.vq_linear_absorbed.argtypes = [qp, qp, vp, vp, vp, qp, vp]
        _lib.vq_recode_e3m2_bytes.argtypes = [qp, C.POINTER(C.c_size_t)]
        _lib.vq_recode_e3m2.argtypes = [qp, vp, C.c_size_t, vp]
        _lib.vq_linear_e3m2.argtypes = [vp, C.c_int64, vp, C.c_int64, C.c_int64, C.c_float, vp, C.c_int32, vp, vp, vp]
        _lib.vq_layernorm_quantize.argtypes = [vp, vp, vp, C.c_int64, C.c_int64, C.c_int64, vp, vp, C.c_float,
                                               C.c_float, qp, vp]
        _lib.vq_qkv_headnorm.argtypes = [vp, C.c_int64, C.c_int32, C.c_int32, C.c_int32, vp, vp, C.c_float,
                                         C.c_float, C.c_float, C.c_float, C.c_int32, C.c_int32, vp, vp]
        _lib.vq_vit_block_workspace.argtypes = [C.POINTER(vq_preln_desc), C.c_int64, C.POINTER(C.c_size_t)]
        _lib.vq_vit_block.argtypes = [C.POINTER(vq_preln_desc), vp, C.c_int64, vp, vp, C.c_size_t, vp]
        _lib.vq_vit_encoder_workspace.argtypes = [C.POINTER(vq_preln_desc), C.c_int32, C.c_int64, C.POINTER(C.c_size_t)]
        _lib.vq_vit_encoder.argtypes = [C.POINTER(vq_preln_desc), C.c_int32, vp, C.c_int64, vp, vp, C.c_size_t, vp]
        for n in EXPORTS[1:]:
            getattr(_lib, n).restype = C.c_int
    return _lib


def status_string(status):
    return lib().vq_status_string(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise VitqError(status, where)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def row_stride_for(cols, storage_bits):
    return ((cols * storage_bits + 7) // 8 + 15) // 16 * 16


def default_storage(bits):
    """Smallest storage field (2, 4 or 8 bits) that holds b-bit levels."""
    return 2 if bits <= 2 else (4 if bits <= 4 else 8)


class QMat:
    """A packed quantized matrix: a uint8 tensor [rows, row_stride] plus its description."""

    def __init__(self, data, cols, bits, storage_bits=None, unsigned=False):
        assert data.dtype == torch.uint8 and data.dim() == 2 and data.is_contiguous()
        self.data = data
        self.rows, self.row_stride = data.shape
        self.cols = int(cols)
        self.bits = int(bits)
        self.storage_bits = int(storage_bits if storage_bits is not None else default_storage(bits))
        self.unsigned = bool(unsigned)

    @staticmethod
    def empty(rows, cols, bits, storage_bits=None, unsigned=False, device="cuda", row_stride=None):
        sb = storage_bits if storage_bits is not None else default_storage(bits)
        stride = row_stride if row_stride is not None else row_stride_for(cols, sb)
        return QMat(torch.zeros((rows, stride), dtype=torch.uint8, device=device), cols, bits, sb, unsigned)

    def c(self):
        m = vq_qmat()
        m.data = self.data.data_ptr() if self.data.numel() else None
        m.bits, m.storage_bits, m.is_unsigned = self.bits, self.storage_bits, int(self.unsigned)
        m.rows, m.cols, m.row_stride = self.rows, self.cols, self.row_stride
        return m


def _q(m):
    return None if m is None else C.byref(m.c())


def vq_weight_steps(w, bits, step_out=None):
    rows, cols = w.shape
    if step_out is None:
        step_out = torch.empty(rows, dtype=torch.float32, device=w.device)
    _check(lib().vq_weight_steps(_ptr(w), rows, cols, w.stride(0), bits, _ptr(step_out), _stream()),
           "vq_weight_steps")
    return step_out


def vq_quantize(x, step, step_per_row, out):
    rows, cols = x.shape
    _check(lib().vq_quantize(_ptr(x), rows, cols, x.stride(0), float(step), _ptr(step_per_row), _q(out),
                             _stream()), "vq_quantize")
    return out


def vq_linear(xq, s_x, wq, s_w, s_w_per_channel, bias, act, acc_out, y_out, s_y, yq_out):
    _check(lib().vq_linear(_q(xq), float(s_x), _q(wq), _ptr(s_w), int(s_w_per_channel), _ptr(bias), int(act),
                           _ptr(acc_out), _ptr(y_out), float(s_y), _q(yq_out), _stream()), "vq_linear")


def vq_layernorm_quantize(x, residual, sum_out, gamma, beta, eps, step, out):
    rows, cols = x.shape
    _check(lib().vq_layernorm_quantize(_ptr(x), _ptr(residual), _ptr(sum_out), rows, cols, x.stride(0),
                                       _ptr(gamma), _ptr(beta), float(eps), float(step), _q(out), _stream()),
           "vq_layernorm_quantize")
    return out


def vq_prepack_weight(wq):
    """Expanded int8 copy of a packed 2-/4-bit weight matrix (a new uint8 device tensor)."""
    import torch
    n = C.c_size_t()
    _check(lib().vq_prepack_weight_bytes(_q(wq), C.byref(n)), "vq_prepack_weight_bytes")
    out = torch.empty(max(n.value, 16), dtype=torch.uint8, device=wq.data.device)
    _check(lib().vq_prepack_weight(_q(wq), _ptr(out), n.value, _stream()), "vq_prepack_weight")
    return out


def vq_linear_prepacked(xq, s_x, wq, wp, s_w, s_w_per_channel, bias, act, acc_out, y_out, s_y, yq_out):
    _check(lib().vq_linear_prepacked(_q(xq), float(s_x), _q(wq), _ptr(wp), _ptr(s_w), int(s_w_per_channel),
                                     _ptr(bias), int(act), _ptr(acc_out), _ptr(y_out), float(s_y), _q(yq_out),
                                     _stream()), "vq_linear_prepacked")


def vq_absorb_thresholds(s_x, s_w, bias, s_y, bits):
    """Host arrays in, host arrays out: s_w, s_y float32 numpy arrays of one value or one per channel
    (their larger size, or the bias', is the channel count); returns (b_int [Nout], thr [Nout, 2^bits-1]) int32."""
    import numpy as np
    s_w = np.ascontiguousarray(np.atleast_1d(s_w), np.float32)
    s_y = np.ascontiguousarray(np.atleast_1d(s_y), np.float32)
    n = max(s_w.size, s_y.size, 1 if bias is None else int(np.size(bias)))
    if bias is not None:
        bias = np.ascontiguousarray(bias, np.float32)
        if bias.size != n:
            raise ValueError("bias must hold one value per output channel")
    if s_w.size not in (1, n) or s_y.size not in (1, n):
        raise ValueError("steps must hold one value or one per output channel")
    nthr = (1 << int(bits)) - 1 if 2 <= int(bits) <= 8 else 1
    b_int = np.zeros(n, np.int32)
    thr = np.zeros((n, nthr), np.int32)
    hp = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
    _check(lib().vq_absorb_thresholds(float(s_x), hp(s_w), int(s_w.size > 1), hp(bias), n, hp(s_y), int(s_y.size > 1),
                                      int(bits), hp(b_int), hp(thr)), "vq_absorb_thresholds")
    return b_int, thr


def vq_linear_absorbed(xq, wq, b_int, thr, acc_out, yq_out):
    _check(lib().vq_linear_absorbed(_q(xq), _q(wq), _ptr(b_int), _ptr(thr), _ptr(acc_out), _q(yq_out), _stream()),
           "vq_linear_absorbed")


def vq_recode_e3m2(m):
    """E3M2-coded copy of a packed matrix with 4-bit storage: a uint8 tensor [rows, ceil(cols/128)*96]."""
    n = C.c_size_t(0)
    _check(lib().vq_recode_e3m2_bytes(_q(m), C.byref(n)), "vq_recode_e3m2_bytes")
    out = torch.empty(max(n.value, 16), dtype=torch.uint8, device=m.data.device)
    _check(lib().vq_recode_e3m2(_q(m), _ptr(out), n.value, _stream()), "vq_recode_e3m2")
    return out[:n.value].view(m.rows, -1) if m.rows else out[:0]


def vq_linear_e3m2(x6, rows, w6, out_features, cols, s_x, s_w, s_w_per_channel, bias, y_out):
    _check(lib().vq_linear_e3m2(_ptr(x6), rows, _ptr(w6), out_features, cols, float(s_x), _ptr(s_w),
                                int(s_w_per_channel), _ptr(bias), _ptr(y_out), _stream()), "vq_linear_e3m2")


def vq_matmul_qk(q, k, B, H, N, s_q, s_k, scale, s_acc_out, p_out):
    _check(lib().vq_matmul_qk(_q(q), _q(k), B, H, N, float(s_q), float(s_k), float(scale), _ptr(s_acc_out),
                              _q(p_out), _stream()), "vq_matmul_qk")


def vq_matmul_pv(p, v, B, H, N, s_p, s_v, o_acc_out, o_out, s_o, oq_out):
    _check(lib().vq_matmul_pv(_q(p), _q(v), B, H, N, float(s_p), float(s_v), _ptr(o_acc_out), _ptr(o_out),
                              float(s_o), _q(oq_out), _stream()), "vq_matmul_pv")


def vq_qkv_headnorm(y, B, H, N, gamma, beta, eps, s_q, s_k, s_v, bits, storage_bits, out):
    _check(lib().vq_qkv_headnorm(_ptr(y), y.stride(0), B, H, N, _ptr(gamma), _ptr(beta), float(eps), float(s_q),
                                 float(s_k), float(s_v), bits, storage_bits, _ptr(out), _stream()),
           "vq_qkv_headnorm")


def make_block_desc(dims, bits_a, bits_p, storage_a, weights, steps, dumps=None, qkln=None):
    """weights: dict name -> QMat (w_*) / fp32 tensors (sw_*, b_*); steps: dict of floats;
    qkln: None or dict(gamma, beta device tensors [2D], eps) for the per-head LayerNorm of Q and K."""
    d = vq_block_desc()
    d.D, d.H, d.N, d.hidden = dims["D"], dims["H"], dims["N"], dims.get("hidden", 0)
    d.bits_a, d.bits_p, d.storage_a = bits_a, bits_p, storage_a
    for name in ("qkv", "proj", "fc1", "fc2"):
        if "w_" + name in weights:
            setattr(d, "w_" + name, weights["w_" + name].c())
            setattr(d, "sw_" + name, weights["sw_" + name].data_ptr())
            b = weights.get("b_" + name)
            setattr(d, "b_" + name, b.data_ptr() if b is not None else None)
    for name in ("s_x", "s_q", "s_k", "s_v", "s_o", "s_x2", "s_h", "scale"):
        if name in steps:
            setattr(d, name, float(steps[name]))
    for name, t in (dumps or {}).items():
        setattr(d, "dump_" + name, t.data_ptr())
    for name in ("qkv", "proj", "fc1", "fc2"):
        t = weights.get("wp_" + name)
        if t is not None:
            setattr(d, "wp_" + name, t.data_ptr())
    if qkln is not None:
        d.qk_gamma, d.qk_beta, d.qk_eps = qkln["gamma"].data_ptr(), qkln["beta"].data_ptr(), float(qkln["eps"])
    return d


def vq_attention_block_workspace(desc, B):
    n = C.c_size_t()
    _check(lib().vq_attention_block_workspace(C.byref(desc), int(B), C.byref(n)), "vq_attention_block_workspace")
    return n.value


def vq_attention_block(desc, xq, B, y_out, workspace):
    _check(lib().vq_attention_block(C.byref(desc), _q(xq), int(B), _ptr(y_out), _ptr(workspace),
                                    workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                    _stream()), "vq_attention_block")


def vq_attention_block_static(desc, xq, B, y_out):
    _check(lib().vq_attention_block_static(C.byref(desc), _q(xq), int(B), _ptr(y_out), _stream()),
           "vq_attention_block_static")


def vq_probe_gelu_distance():
    """max over every finite nonzero fp32 y of |fast GELU - definition| / |y| (a device tensor of one float)."""
    import torch
    out = torch.empty(1, dtype=torch.float32, device="cuda")
    _check(lib().vq_probe_gelu_distance(_ptr(out), _stream()), "vq_probe_gelu_distance")
    return out


def vq_probe_mfma_i8(iters, sink=None):
    """Enqueues the matrix-core probe; returns the integer operations it performs."""
    ops = C.c_double()
    _check(lib().vq_probe_mfma_i8(int(iters), _ptr(sink), C.byref(ops), _stream()), "vq_probe_mfma_i8")
    return ops.value


def make_preln_desc(block_desc, ln, dump_xq=None, dump_x1=None):
    """block_desc: a vq_block_desc (hidden > 0); ln: dict of device tensors g1, b1, g2, b2 and eps."""
    d = vq_preln_desc()
    d.block = block_desc
    d.ln1_gamma, d.ln1_beta = ln["g1"].data_ptr(), ln["b1"].data_ptr()
    d.ln2_gamma, d.ln2_beta = ln["g2"].data_ptr(), ln["b2"].data_ptr()
    d.ln_eps = float(ln["eps"])
    d.dump_xq = dump_xq.data_ptr() if dump_xq is not None else None
    d.dump_x1 = dump_x1.data_ptr() if dump_x1 is not None else None
    return d


def vq_vit_block_workspace(desc, B):
    n = C.c_size_t()
    _check(lib().vq_vit_block_workspace(C.byref(desc), int(B), C.byref(n)), "vq_vit_block_workspace")
    return n.value


def vq_vit_block(desc, x, B, y_out, workspace):
    _check(lib().vq_vit_block(C.byref(desc), _ptr(x), int(B), _ptr(y_out), _ptr(workspace),
                              workspace.numel() * workspace.element_size() if workspace is not None else 0,
                              _stream()), "vq_vit_block")


def _layer_array(descs):
    arr = (vq_preln_desc * len(descs))()
    for i, d in enumerate(descs):
        C.memmove(C.byref(arr[i]), C.byref(d), C.sizeof(vq_preln_desc))
    return arr


def vq_vit_encoder_workspace(descs, B):
    n = C.c_size_t()
    _check(lib().vq_vit_encoder_workspace(_layer_array(descs), len(descs), int(B), C.byref(n)), "vq_vit_encoder_workspace")
    return n.value


def vq_vit_encoder(descs, x, B, y_out, workspace):
    """descs: list of vq_preln_desc, one per layer (the tensors they point to must stay alive)."""
    _check(lib().vq_vit_encoder(_layer_array(descs), len(descs), _ptr(x), int(B), _ptr(y_out), _ptr(workspace),
                                workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                _stream()), "vq_vit_encoder")
