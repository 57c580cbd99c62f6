"""ctypes loader for the MOSS CPU oracle (test infrastructure, not product code).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this module.  It marshals numpy arrays into oracle/moss_oracle.c and does no
arithmetic of its own.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moss_oracle.c")
_LIB = os.path.join(_HERE, "libmoss_oracle.so")
_lib = None

EXP_NEAREST = 0
EXP_CEIL = 1


def build(force=False):
    """Compile the oracle with gcc (no HIP, no fast-math, no FMA contraction)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


class WState(C.Structure):
    _fields_ = [("s_base", C.c_float), ("s_cur", C.c_float), ("cum_lr", C.c_double),
                ("step", C.c_int64), ("last_rebase", C.c_int64),
                ("amax_seen", C.c_float), ("overflow_count", C.c_uint32),
                ("clipped_count", C.c_uint32), ("reserved", C.c_uint32)]


class AdamWArgs(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float),
                ("one_minus_beta1", C.c_float), ("one_minus_beta2", C.c_float),
                ("bias_corr1", C.c_float), ("bias_corr2", C.c_float),
                ("margin", C.c_float), ("interval", C.c_int32)]


def adamw_args(lr, beta1, beta2, eps, weight_decay, one_minus_beta1, one_minus_beta2,
               bias_corr1, bias_corr2, margin=1.0, interval=500):
    """Pack optimizer arguments; every derived term is supplied by the caller."""
    return AdamWArgs(lr, beta1, beta2, eps, weight_decay, one_minus_beta1, one_minus_beta2,
                     bias_corr1, bias_corr2, margin, interval)


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.moss_oracle_e4m3_decode.restype = C.c_double
        L.moss_oracle_e4m3_decode.argtypes = [C.c_uint8]
        L.moss_oracle_e4m3_encode.restype = C.c_uint8
        L.moss_oracle_e4m3_encode.argtypes = [C.c_double]
        L.moss_oracle_snr_db.restype = C.c_double
        L.moss_oracle_snr_db.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.moss_oracle_quant_act_2level.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                                   C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.moss_oracle_quant_act_2level_given_max.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int,
                                                             C.c_uint16, C.c_void_p, C.c_void_p, C.c_void_p]
        L.moss_oracle_swiglu.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.moss_oracle_swiglu_backward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.moss_oracle_dequant.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int64, C.c_int64, C.c_void_p]
        L.moss_oracle_weight_init.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.moss_oracle_weight_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                              C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p]
        L.moss_oracle_gemm.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_float,
                                       C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]
        L.moss_oracle_gemm_sampled.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_float,
                                               C.c_void_p, C.c_void_p, C.c_float,
                                               C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.moss_oracle_row_norms.argtypes = [C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]
        L.moss_oracle_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_double, C.c_int64, C.c_int64, C.c_void_p]
        L.moss_oracle_rmsnorm_backward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_int64, C.c_int64,
                                                   C.c_void_p]
        L.moss_oracle_groupwise_fp8.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.moss_oracle_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def _u8(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a if shape is None else a.reshape(shape)


def e4m3_decode(code):
    return lib().moss_oracle_e4m3_decode(int(code))


def e4m3_encode(y):
    return lib().moss_oracle_e4m3_encode(float(y))


def quant_act_2level(x_bf16_bits, axis=0, exp_mode=EXP_NEAREST):
    """x_bf16_bits: uint16 [rows, cols] (C-contiguous).  Returns (q, e, s):
    axis 0 -> q [rows, cols], e [rows, cols/32]; axis 1 -> q [cols, rows],
    e [cols, rows/32]; s is the FP32 global scale."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    rows, cols = x.shape
    outer, inner = (rows, cols) if axis == 0 else (cols, rows)
    q = np.empty((outer, inner), np.uint8)
    e = np.empty((outer, inner // 32), np.uint8)
    s = np.zeros(1, np.float32)
    _check(lib().moss_oracle_quant_act_2level(_p(x), rows, cols, cols, axis, exp_mode, _p(q), _p(e), _p(s)),
           "quant_act_2level")
    return q, e, np.float32(s[0])


def quant_act_2level_given_max(x_bf16_bits, max_bf16_bits, axis=0, exp_mode=EXP_NEAREST):
    """quant_act_2level with the tensor maximum of Eq. 2 handed in (BF16 magnitude bits, at least max|x|)."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    rows, cols = x.shape
    outer, inner = (rows, cols) if axis == 0 else (cols, rows)
    q = np.empty((outer, inner), np.uint8)
    e = np.empty((outer, inner // 32), np.uint8)
    s = np.zeros(1, np.float32)
    _check(lib().moss_oracle_quant_act_2level_given_max(_p(x), rows, cols, cols, axis, exp_mode, int(max_bf16_bits) & 0x7FFF,
                                                        _p(q), _p(e), _p(s)), "quant_act_2level_given_max")
    return q, e, np.float32(s[0])


def swiglu(gate_bits, up_bits):
    """h = silu(gate) * up in double from BF16 bit arrays of equal shape."""
    g = np.ascontiguousarray(gate_bits, dtype=np.uint16); u = np.ascontiguousarray(up_bits, dtype=np.uint16)
    assert g.shape == u.shape
    h = np.empty(g.shape, np.float64)
    _check(lib().moss_oracle_swiglu(_p(g), _p(u), g.size, _p(h)), "swiglu")
    return h


def swiglu_backward(gate_bits, up_bits, dh_bits):
    """(d_gate, d_up) in double for the upstream gradient dh of h = silu(gate) * up."""
    g = np.ascontiguousarray(gate_bits, dtype=np.uint16); u = np.ascontiguousarray(up_bits, dtype=np.uint16)
    d = np.ascontiguousarray(dh_bits, dtype=np.uint16)
    assert g.shape == u.shape == d.shape
    dg = np.empty(g.shape, np.float64); du = np.empty(g.shape, np.float64)
    _check(lib().moss_oracle_swiglu_backward(_p(g), _p(u), _p(d), g.size, _p(dg), _p(du)), "swiglu_backward")
    return dg, du


def dequant(q, e, s):
    q = _u8(q)
    outer, inner = q.shape
    e = None if e is None else _u8(e)
    out = np.empty((outer, inner), np.float64)
    _check(lib().moss_oracle_dequant(_p(q), _p(e), float(s), outer, inner, _p(out)), "dequant")
    return out


def weight_init(w, want_transpose=False):
    w = np.ascontiguousarray(w, dtype=np.float32)
    rows, cols = w.shape
    st = WState()
    wq = np.empty((rows, cols), np.uint8)
    wq_t = np.empty((cols, rows), np.uint8) if want_transpose else None
    _check(lib().moss_oracle_weight_init(_p(w), rows, cols, C.byref(st), _p(wq), _p(wq_t)), "weight_init")
    return st, wq, wq_t


def weight_step(w, m, v, g, args, st, want_transpose=False):
    """In-place AdamW step on float32 arrays w, m, v; g float32 or uint16 (BF16 bits)."""
    for a in (w, m, v):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    g = np.ascontiguousarray(g)
    assert g.dtype in (np.float32, np.uint16)
    rows, cols = w.shape
    wq = np.empty((rows, cols), np.uint8)
    wq_t = np.empty((cols, rows), np.uint8) if want_transpose else None
    _check(lib().moss_oracle_weight_step(_p(w), _p(m), _p(v), _p(g), int(g.dtype == np.uint16), rows, cols,
                                         C.byref(args), C.byref(st), _p(wq), _p(wq_t)), "weight_step")
    return wq, wq_t


def gemm(a_q, a_e, a_s, b_q, b_e, b_s):
    a_q, b_q = _u8(a_q), _u8(b_q)
    M, K = a_q.shape
    N = b_q.shape[0]
    a_e = None if a_e is None else _u8(a_e)
    b_e = None if b_e is None else _u8(b_e)
    out = np.empty((M, N), np.float64)
    _check(lib().moss_oracle_gemm(M, N, K, _p(a_q), _p(a_e), float(a_s), _p(b_q), _p(b_e), float(b_s), _p(out)),
           "gemm")
    return out


def gemm_sampled(a_q, a_e, a_s, b_q, b_e, b_s, ms, ns):
    a_q, b_q = _u8(a_q), _u8(b_q)
    M, K = a_q.shape
    N = b_q.shape[0]
    a_e = None if a_e is None else _u8(a_e)
    b_e = None if b_e is None else _u8(b_e)
    ms = np.ascontiguousarray(ms, dtype=np.int64)
    ns = np.ascontiguousarray(ns, dtype=np.int64)
    out = np.empty(ms.shape[0], np.float64)
    _check(lib().moss_oracle_gemm_sampled(M, N, K, _p(a_q), _p(a_e), float(a_s), _p(b_q), _p(b_e), float(b_s),
                                          _p(ms), _p(ns), ms.shape[0], _p(out)), "gemm_sampled")
    return out


def row_norms(q, e, s):
    q = _u8(q)
    R, K = q.shape
    e = None if e is None else _u8(e)
    out = np.empty(R, np.float64)
    _check(lib().moss_oracle_row_norms(R, K, _p(q), _p(e), float(s), _p(out)), "row_norms")
    return out


def rmsnorm(h_bits, gamma_bits, eps):
    """y = h / sqrt(mean(h^2) + eps) * gamma over each row, in double, from BF16 bit arrays h [rows, cols], gamma [cols]."""
    h = np.ascontiguousarray(h_bits, dtype=np.uint16); g = np.ascontiguousarray(gamma_bits, dtype=np.uint16)
    rows, cols = h.shape
    assert g.shape == (cols,)
    y = np.empty((rows, cols), np.float64)
    _check(lib().moss_oracle_rmsnorm(_p(h), _p(g), float(eps), rows, cols, _p(y)), "rmsnorm")
    return y


def rmsnorm_backward(h_bits, gamma_bits, dy_bits, d_res_bits, eps):
    """d_h for the upstream gradient dy of rmsnorm(h), plus the residual-path gradient d_res (or None), in double."""
    h = np.ascontiguousarray(h_bits, dtype=np.uint16); g = np.ascontiguousarray(gamma_bits, dtype=np.uint16)
    dy = np.ascontiguousarray(dy_bits, dtype=np.uint16)
    dr = None if d_res_bits is None else np.ascontiguousarray(d_res_bits, dtype=np.uint16)
    rows, cols = h.shape
    assert g.shape == (cols,) and dy.shape == h.shape and (dr is None or dr.shape == h.shape)
    out = np.empty((rows, cols), np.float64)
    _check(lib().moss_oracle_rmsnorm_backward(_p(h), _p(g), _p(dy), _p(dr), float(eps), rows, cols, _p(out)), "rmsnorm_backward")
    return out


def groupwise_fp8(x_bf16_bits, group):
    """The comparison schemes of Sec. 3.1 / 4.5.2: one FP32 scale per `group` consecutive elements of a row
    (0: per tensor).  Returns (codes, scales, dequantized values in double)."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    rows, cols = x.shape
    q = np.empty((rows, cols), np.uint8)
    scales = np.empty(1 if group == 0 else rows * cols // group, np.float32)
    dq = np.empty((rows, cols), np.float64)
    _check(lib().moss_oracle_groupwise_fp8(_p(x), rows, cols, group, _p(q), _p(scales), _p(dq)), "groupwise_fp8")
    return q, scales, dq


def snr_db(x, dq):
    x = np.ascontiguousarray(x, dtype=np.float64).ravel()
    dq = np.ascontiguousarray(dq, dtype=np.float64).ravel()
    return lib().moss_oracle_snr_db(_p(x), _p(dq), x.size)


def num_threads():
    return lib().moss_oracle_num_threads()
