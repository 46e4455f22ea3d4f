"""ctypes front end of the CPU oracle (``oracle/dqo.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``; the GPU library never touches it.

All arrays are numpy arrays in host memory.  The functions mirror the C entry points one to one;
the arithmetic lives in the C file, nothing is computed here beyond shapes and buffer sizes.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dqo.c")
_LIB = os.path.join(_HERE, "libdqo.so")

GRANULE = 128


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every float operation a single
    IEEE rounding (the rounding decision of Eq. (6) depends on it); no fast-math."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i64p, f32p, u8p, u32p = (C.POINTER(C.c_int64), C.POINTER(C.c_float),
                                 C.POINTER(C.c_uint8), C.POINTER(C.c_uint32))
        L.dqo_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.dqo_philox4x32_10.restype = None
        L.dqo_padded_elems.argtypes = [i64p, C.c_int32]
        L.dqo_padded_elems.restype = C.c_int64
        L.dqo_seg_start.argtypes = [i64p, C.c_int32, C.c_int32]
        L.dqo_seg_start.restype = C.c_int64
        L.dqo_packed_bytes.argtypes = [i64p, C.c_int32, C.c_int]
        L.dqo_packed_bytes.restype = C.c_int64
        L.dqo_norm.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p]
        L.dqo_norm_linf.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p]
        L.dqo_select_bits_linf.argtypes = [f32p, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_double,
                                           C.c_double, C.c_int, C.c_int, C.POINTER(C.c_int),
                                           C.POINTER(C.c_double)]
        L.dqo_select_bits.argtypes = [f32p, C.c_int32, C.c_int32, C.c_int64, C.c_int64,
                                      C.c_double, C.c_double, C.c_int, C.c_int,
                                      C.POINTER(C.c_int), C.POINTER(C.c_double)]
        L.dqo_quantize.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p, C.c_int,
                                   C.c_uint64, C.c_uint32, C.c_uint32, u8p, u8p]
        L.dqo_quantize_range.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p, C.c_int,
                                         C.c_uint64, C.c_uint32, C.c_uint32, C.c_int64, C.c_int64,
                                         u8p, u8p]
        L.dqo_dequant_reduce_range.argtypes = [i64p, C.c_int32, u8p, u8p, C.c_int32, f32p, C.c_int,
                                               C.c_int64, C.c_int64, f32p]
        L.dqo_pack.argtypes = [u8p, u8p, C.c_int64, C.c_int, u8p]
        L.dqo_unpack.argtypes = [u8p, C.c_int64, C.c_int, u8p, u8p]
        L.dqo_dequant_reduce.argtypes = [i64p, C.c_int32, u8p, u8p, C.c_int32, f32p, C.c_int, f32p]
        L.dqo_quantize_pack.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p,
                                        C.c_int, C.c_uint64, C.c_uint32, C.c_uint32, u8p,
                                        C.c_int64, u8p]
        L.dqo_unpack_dequant_reduce.argtypes = [i64p, C.c_int32, u8p, C.c_int64, C.c_int32, f32p,
                                                C.c_int, f32p, u8p]
        i32p = C.POINTER(C.c_int32)
        L.dqo_select_bits_per_tensor.argtypes = [f32p, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_double,
                                                 C.c_double, C.c_int, C.c_int, i32p, C.POINTER(C.c_double)]
        L.dqo_packed_bytes_v.argtypes = [i64p, C.c_int32, i32p]
        L.dqo_packed_bytes_v.restype = C.c_int64
        L.dqo_quantize_v.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p, i32p, C.c_uint64,
                                     C.c_uint32, C.c_uint32, u8p, u8p]
        L.dqo_quantize_v_range.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p, i32p, C.c_uint64,
                                           C.c_uint32, C.c_uint32, C.c_int64, C.c_int64, u8p, u8p]
        L.dqo_pack_v.argtypes = [u8p, u8p, i64p, C.c_int32, i32p, u8p]
        L.dqo_unpack_v.argtypes = [u8p, i64p, C.c_int32, i32p, u8p, u8p]
        L.dqo_dequant_reduce_v.argtypes = [i64p, C.c_int32, u8p, u8p, C.c_int32, f32p, i32p, f32p]
        L.dqo_dequant_reduce_v_range.argtypes = [i64p, C.c_int32, u8p, u8p, C.c_int32, f32p, i32p, C.c_int64,
                                                 C.c_int64, f32p]
        L.dqo_quantize_pack_v.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p, i32p, C.c_uint64,
                                          C.c_uint32, C.c_uint32, u8p, C.c_int64, u8p]
        L.dqo_unpack_dequant_reduce_v.argtypes = [i64p, C.c_int32, u8p, C.c_int64, C.c_int32, f32p, i32p,
                                                  f32p, u8p]
        L.dqo_comm_cost_bits_per_tensor.argtypes = [C.c_int, i64p, i32p, C.c_int32, C.c_int]
        L.dqo_comm_cost_bits_per_tensor.restype = C.c_int64
        L.dqo_select_bits_per_worker.argtypes = [f32p, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_double,
                                                 C.c_double, C.c_int, C.c_int, C.c_int, i32p]
        L.dqo_quantize_pack_w.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, f32p, i32p, C.c_uint64,
                                          C.c_uint32, C.c_uint32, u8p, C.c_int64, u8p]
        L.dqo_unpack_dequant_reduce_w.argtypes = [i64p, C.c_int32, u8p, C.c_int64, C.c_int32, f32p, i32p, f32p, u8p]
        L.dqo_sign_pack.argtypes = [i64p, C.c_int32, f32p, C.c_int64, C.c_int32, u8p, C.c_int64]
        L.dqo_sign_reduce.argtypes = [i64p, C.c_int32, u8p, C.c_int64, C.c_int32, f32p, C.c_int, f32p]
        L.dqo_update.argtypes = [f32p, f32p, C.c_int64, C.c_float]
        L.dqo_alpha_est.argtypes = [C.c_double, C.c_double, C.c_int64]
        L.dqo_alpha_est.restype = C.c_double
        L.dqo_comm_cost_bits.argtypes = [C.c_int, C.c_int64, C.c_int, C.c_int32, C.c_int]
        L.dqo_comm_cost_bits.restype = C.c_int64
        L.dqo_num_threads.restype = C.c_int
        L.dqo_set_num_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _segs(seg_len):
    a = np.ascontiguousarray(np.asarray(seg_len, dtype=np.int64).reshape(-1))
    if a.size < 1:
        raise ValueError("need at least one segment")
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: oracle returned {rc}")


def num_threads() -> int:
    return int(lib().dqo_num_threads())


def set_num_threads(n: int) -> None:
    lib().dqo_set_num_threads(int(n))


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().dqo_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def padded_elems(seg_len) -> int:
    s = _segs(seg_len)
    return int(lib().dqo_padded_elems(_p(s, C.c_int64), s.size))


def seg_starts(seg_len):
    s = _segs(seg_len)
    return np.array([lib().dqo_seg_start(_p(s, C.c_int64), s.size, l) for l in range(s.size)],
                    dtype=np.int64)


def packed_bytes(seg_len, b: int) -> int:
    s = _segs(seg_len)
    return int(lib().dqo_packed_bytes(_p(s, C.c_int64), s.size, b))


def _grads2d(grads, dp):
    g = np.asarray(grads)
    if g.dtype != np.float32 or g.ndim != 2 or not g.flags.c_contiguous or g.shape[1] < dp:
        raise ValueError("grads must be a C-contiguous float32 [M][>=D'] array")
    return g


def norm(seg_len, grads):
    s = _segs(seg_len)
    g = _grads2d(grads, padded_elems(s))
    M = g.shape[0]
    out = np.zeros((M, s.size), dtype=np.float32)
    _check(lib().dqo_norm(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M,
                          _p(out, C.c_float)), "norm")
    return out


def select_bits(norms, t, T, eps_hat_q, alpha, b_min, b_max):
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32))
    if n.ndim != 2:
        raise ValueError("norms must be [M][n_seg]")
    b = C.c_int(0)
    gbar = C.c_double(0.0)
    _check(lib().dqo_select_bits(_p(n, C.c_float), n.shape[0], n.shape[1], t, T, eps_hat_q,
                                 alpha, b_min, b_max, C.byref(b), C.byref(gbar)), "select_bits")
    return int(b.value), float(gbar.value)


def norm_linf(seg_len, grads):
    s = _segs(seg_len)
    g = _grads2d(grads, padded_elems(s))
    M = g.shape[0]
    out = np.zeros((M, s.size), dtype=np.float32)
    _check(lib().dqo_norm_linf(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M,
                               _p(out, C.c_float)), "norm_linf")
    return out


def select_bits_linf(norms, t, T, eps_hat_q, alpha, b_min, b_max):
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32))
    if n.ndim != 2:
        raise ValueError("norms must be [M][n_seg]")
    b = C.c_int(0)
    gbar = C.c_double(0.0)
    _check(lib().dqo_select_bits_linf(_p(n, C.c_float), n.shape[0], n.shape[1], t, T, eps_hat_q,
                                      alpha, b_min, b_max, C.byref(b), C.byref(gbar)), "select_bits_linf")
    return int(b.value), float(gbar.value)


def quantize(seg_len, grads, norms, b, seed, step, worker_base=0):
    """-> (sign[M][D'], level[M][D']) uint8 codes."""
    s = _segs(seg_len)
    dp = padded_elems(s)
    g = _grads2d(grads, dp)
    M = g.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    sign = np.zeros((M, dp), dtype=np.uint8)
    level = np.zeros((M, dp), dtype=np.uint8)
    _check(lib().dqo_quantize(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M,
                              _p(n, C.c_float), b, seed, step, worker_base,
                              _p(sign, C.c_uint8), _p(level, C.c_uint8)), "quantize")
    return sign, level


def quantize_range(seg_len, grads_slice, norms, b, seed, step, p_begin, p_end, worker_base=0):
    """Codes of padded indices [p_begin, p_end) only; grads_slice is [M][>= p_end - p_begin] and
    holds exactly those elements.  -> (sign, level) uint8 [M][p_end - p_begin]."""
    s = _segs(seg_len)
    span = int(p_end - p_begin)
    g = _grads2d(grads_slice, span)
    M = g.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    sign = np.zeros((M, span), dtype=np.uint8)
    level = np.zeros((M, span), dtype=np.uint8)
    _check(lib().dqo_quantize_range(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M,
                                    _p(n, C.c_float), b, seed, step, worker_base, p_begin, p_end,
                                    _p(sign, C.c_uint8), _p(level, C.c_uint8)), "quantize_range")
    return sign, level


def dequant_reduce_range(seg_len, sign, level, norms, b, p_begin, p_end):
    s = _segs(seg_len)
    span = int(p_end - p_begin)
    sg = np.ascontiguousarray(np.asarray(sign, dtype=np.uint8))
    lv = np.ascontiguousarray(np.asarray(level, dtype=np.uint8))
    M = sg.shape[0]
    if sg.shape != (M, span) or lv.shape != (M, span):
        raise ValueError("codes must be [M][p_end - p_begin]")
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    out = np.zeros(span, dtype=np.float32)
    _check(lib().dqo_dequant_reduce_range(_p(s, C.c_int64), s.size, _p(sg, C.c_uint8),
                                          _p(lv, C.c_uint8), M, _p(n, C.c_float), b, p_begin, p_end,
                                          _p(out, C.c_float)), "dequant_reduce_range")
    return out


def pack(sign, level, b):
    """one worker: codes -> message bytes."""
    sg = np.ascontiguousarray(np.asarray(sign, dtype=np.uint8).reshape(-1))
    lv = np.ascontiguousarray(np.asarray(level, dtype=np.uint8).reshape(-1))
    dp = sg.size
    out = np.zeros(dp // 8 + dp * b // 8, dtype=np.uint8)
    _check(lib().dqo_pack(_p(sg, C.c_uint8), _p(lv, C.c_uint8), dp, b, _p(out, C.c_uint8)), "pack")
    return out


def unpack(packed, dp, b):
    pk = np.ascontiguousarray(np.asarray(packed, dtype=np.uint8).reshape(-1))
    if pk.size < dp // 8 + dp * b // 8:
        raise ValueError("message too short")
    sign = np.zeros(dp, dtype=np.uint8)
    level = np.zeros(dp, dtype=np.uint8)
    _check(lib().dqo_unpack(_p(pk, C.c_uint8), dp, b, _p(sign, C.c_uint8), _p(level, C.c_uint8)),
           "unpack")
    return sign, level


def dequant_reduce(seg_len, sign, level, norms, b):
    s = _segs(seg_len)
    dp = padded_elems(s)
    sg = np.ascontiguousarray(np.asarray(sign, dtype=np.uint8))
    lv = np.ascontiguousarray(np.asarray(level, dtype=np.uint8))
    M = sg.shape[0]
    if sg.shape != (M, dp) or lv.shape != (M, dp):
        raise ValueError("codes must be [M][D']")
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    out = np.zeros(dp, dtype=np.float32)
    _check(lib().dqo_dequant_reduce(_p(s, C.c_int64), s.size, _p(sg, C.c_uint8),
                                    _p(lv, C.c_uint8), M, _p(n, C.c_float), b,
                                    _p(out, C.c_float)), "dequant_reduce")
    return out


def quantize_pack(seg_len, grads, norms, b, seed, step, worker_base=0, packed_stride=None):
    """-> packed[M][stride] uint8: every worker's message."""
    s = _segs(seg_len)
    dp = padded_elems(s)
    g = _grads2d(grads, dp)
    M = g.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    nbytes = packed_bytes(s, b)
    stride = nbytes if packed_stride is None else int(packed_stride)
    packed = np.zeros((M, stride), dtype=np.uint8)
    scratch = np.zeros(2 * M * dp, dtype=np.uint8)
    _check(lib().dqo_quantize_pack(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M,
                                   _p(n, C.c_float), b, seed, step, worker_base,
                                   _p(packed, C.c_uint8), stride, _p(scratch, C.c_uint8)),
           "quantize_pack")
    return packed


def unpack_dequant_reduce(seg_len, packed, norms, b):
    s = _segs(seg_len)
    dp = padded_elems(s)
    pk = np.asarray(packed)
    if pk.dtype != np.uint8 or pk.ndim != 2 or not pk.flags.c_contiguous:
        raise ValueError("packed must be a C-contiguous uint8 [M][stride] array")
    M = pk.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    out = np.zeros(dp, dtype=np.float32)
    scratch = np.zeros(2 * M * dp, dtype=np.uint8)
    _check(lib().dqo_unpack_dequant_reduce(_p(s, C.c_int64), s.size, _p(pk, C.c_uint8),
                                           pk.shape[1], M, _p(n, C.c_float), b,
                                           _p(out, C.c_float), _p(scratch, C.c_uint8)),
           "unpack_dequant_reduce")
    return out


def update(x, ghat, eta):
    """in place: x <- x - eta * ghat (numpy float32 arrays of equal length)."""
    if x.dtype != np.float32 or ghat.dtype != np.float32 or x.shape != ghat.shape or not x.flags.c_contiguous:
        raise ValueError("x and ghat must be equal-shape C-contiguous float32 arrays")
    g = np.ascontiguousarray(ghat)
    _check(lib().dqo_update(_p(x, C.c_float), _p(g, C.c_float), x.size, eta), "update")
    return x


def alpha_est(F_t, F_0, t):
    v = float(lib().dqo_alpha_est(F_t, F_0, t))
    if v < 0:
        raise ValueError("alpha_est undefined")
    return v


def comm_cost_bits(W, d, b, n_norms=1, B_pre=32):
    v = int(lib().dqo_comm_cost_bits(W, d, b, n_norms, B_pre))
    if v < 0:
        raise ValueError("bad argument")
    return v


# ------------------------------------------------------------------ one bit-width per tensor
def _widths(b_seg, n_seg):
    b = np.ascontiguousarray(np.asarray(b_seg, dtype=np.int32).reshape(-1))
    if b.size != n_seg:
        raise ValueError("one width per tensor")
    return b


def select_bits_per_tensor(norms, t, T, eps_hat_q, alpha, b_min, b_max):
    """-> (b[n_seg] int32, Nbar[n_seg] float64)."""
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32))
    if n.ndim != 2:
        raise ValueError("norms must be [M][n_seg]")
    b = np.zeros(n.shape[1], dtype=np.int32)
    nbar = np.zeros(n.shape[1], dtype=np.float64)
    _check(lib().dqo_select_bits_per_tensor(_p(n, C.c_float), n.shape[0], n.shape[1], t, T, eps_hat_q, alpha,
                                            b_min, b_max, _p(b, C.c_int32), _p(nbar, C.c_double)),
           "select_bits_per_tensor")
    return b, nbar


def packed_bytes_v(seg_len, b_seg) -> int:
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    return int(lib().dqo_packed_bytes_v(_p(s, C.c_int64), s.size, _p(b, C.c_int32)))


def quantize_v(seg_len, grads, norms, b_seg, seed, step, worker_base=0):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    dp = padded_elems(s)
    g = _grads2d(grads, dp)
    M = g.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    sign = np.zeros((M, dp), dtype=np.uint8)
    level = np.zeros((M, dp), dtype=np.uint8)
    _check(lib().dqo_quantize_v(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M, _p(n, C.c_float),
                                _p(b, C.c_int32), seed, step, worker_base, _p(sign, C.c_uint8),
                                _p(level, C.c_uint8)), "quantize_v")
    return sign, level


def quantize_v_range(seg_len, grads_slice, norms, b_seg, seed, step, p_begin, p_end, worker_base=0):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    span = int(p_end - p_begin)
    g = _grads2d(grads_slice, span)
    M = g.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    sign = np.zeros((M, span), dtype=np.uint8)
    level = np.zeros((M, span), dtype=np.uint8)
    _check(lib().dqo_quantize_v_range(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M,
                                      _p(n, C.c_float), _p(b, C.c_int32), seed, step, worker_base, p_begin,
                                      p_end, _p(sign, C.c_uint8), _p(level, C.c_uint8)), "quantize_v_range")
    return sign, level


def pack_v(sign, level, seg_len, b_seg):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    sg = np.ascontiguousarray(np.asarray(sign, dtype=np.uint8).reshape(-1))
    lv = np.ascontiguousarray(np.asarray(level, dtype=np.uint8).reshape(-1))
    if sg.size != padded_elems(s) or lv.size != sg.size:
        raise ValueError("codes must have D' entries")
    out = np.zeros(packed_bytes_v(s, b), dtype=np.uint8)
    _check(lib().dqo_pack_v(_p(sg, C.c_uint8), _p(lv, C.c_uint8), _p(s, C.c_int64), s.size, _p(b, C.c_int32),
                            _p(out, C.c_uint8)), "pack_v")
    return out


def unpack_v(packed, seg_len, b_seg):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    pk = np.ascontiguousarray(np.asarray(packed, dtype=np.uint8).reshape(-1))
    if pk.size < packed_bytes_v(s, b):
        raise ValueError("message too short")
    dp = padded_elems(s)
    sign = np.zeros(dp, dtype=np.uint8)
    level = np.zeros(dp, dtype=np.uint8)
    _check(lib().dqo_unpack_v(_p(pk, C.c_uint8), _p(s, C.c_int64), s.size, _p(b, C.c_int32),
                              _p(sign, C.c_uint8), _p(level, C.c_uint8)), "unpack_v")
    return sign, level


def dequant_reduce_v(seg_len, sign, level, norms, b_seg):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    dp = padded_elems(s)
    sg = np.ascontiguousarray(np.asarray(sign, dtype=np.uint8))
    lv = np.ascontiguousarray(np.asarray(level, dtype=np.uint8))
    M = sg.shape[0]
    if sg.shape != (M, dp) or lv.shape != (M, dp):
        raise ValueError("codes must be [M][D']")
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    out = np.zeros(dp, dtype=np.float32)
    _check(lib().dqo_dequant_reduce_v(_p(s, C.c_int64), s.size, _p(sg, C.c_uint8), _p(lv, C.c_uint8), M,
                                      _p(n, C.c_float), _p(b, C.c_int32), _p(out, C.c_float)),
           "dequant_reduce_v")
    return out


def dequant_reduce_v_range(seg_len, sign, level, norms, b_seg, p_begin, p_end):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    span = int(p_end - p_begin)
    sg = np.ascontiguousarray(np.asarray(sign, dtype=np.uint8))
    lv = np.ascontiguousarray(np.asarray(level, dtype=np.uint8))
    M = sg.shape[0]
    if sg.shape != (M, span) or lv.shape != (M, span):
        raise ValueError("codes must be [M][p_end - p_begin]")
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    out = np.zeros(span, dtype=np.float32)
    _check(lib().dqo_dequant_reduce_v_range(_p(s, C.c_int64), s.size, _p(sg, C.c_uint8), _p(lv, C.c_uint8), M,
                                            _p(n, C.c_float), _p(b, C.c_int32), p_begin, p_end,
                                            _p(out, C.c_float)), "dequant_reduce_v_range")
    return out


def quantize_pack_v(seg_len, grads, norms, b_seg, seed, step, worker_base=0):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    dp = padded_elems(s)
    g = _grads2d(grads, dp)
    M = g.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    stride = packed_bytes_v(s, b)
    packed = np.zeros((M, stride), dtype=np.uint8)
    scratch = np.zeros(2 * M * dp, dtype=np.uint8)
    _check(lib().dqo_quantize_pack_v(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M,
                                     _p(n, C.c_float), _p(b, C.c_int32), seed, step, worker_base,
                                     _p(packed, C.c_uint8), stride, _p(scratch, C.c_uint8)), "quantize_pack_v")
    return packed


def unpack_dequant_reduce_v(seg_len, packed, norms, b_seg):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    dp = padded_elems(s)
    pk = np.asarray(packed)
    if pk.dtype != np.uint8 or pk.ndim != 2 or not pk.flags.c_contiguous:
        raise ValueError("packed must be a C-contiguous uint8 [M][stride] array")
    M = pk.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    out = np.zeros(dp, dtype=np.float32)
    scratch = np.zeros(2 * M * dp, dtype=np.uint8)
    _check(lib().dqo_unpack_dequant_reduce_v(_p(s, C.c_int64), s.size, _p(pk, C.c_uint8), pk.shape[1], M,
                                             _p(n, C.c_float), _p(b, C.c_int32), _p(out, C.c_float),
                                             _p(scratch, C.c_uint8)), "unpack_dequant_reduce_v")
    return out


def comm_cost_bits_per_tensor(W, seg_len, b_seg, B_pre=32):
    s = _segs(seg_len)
    b = _widths(b_seg, s.size)
    v = int(lib().dqo_comm_cost_bits_per_tensor(W, _p(s, C.c_int64), _p(b, C.c_int32), s.size, B_pre))
    if v < 0:
        raise ValueError("bad argument")
    return v


# ------------------------------------------------------------------------- sign-only messages
def sign_pack(seg_len, grads):
    """-> packed[M][D'/8] uint8: every worker's sign plane."""
    s = _segs(seg_len)
    dp = padded_elems(s)
    g = _grads2d(grads, dp)
    M = g.shape[0]
    packed = np.zeros((M, dp // 8), dtype=np.uint8)
    _check(lib().dqo_sign_pack(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M,
                               _p(packed, C.c_uint8), dp // 8), "sign_pack")
    return packed


def sign_reduce(seg_len, packed, scales=None, majority=False):
    s = _segs(seg_len)
    dp = padded_elems(s)
    pk = np.asarray(packed)
    if pk.dtype != np.uint8 or pk.ndim != 2 or not pk.flags.c_contiguous:
        raise ValueError("packed must be a C-contiguous uint8 [M][stride] array")
    M = pk.shape[0]
    sc = None
    if scales is not None:
        sc = np.ascontiguousarray(np.asarray(scales, dtype=np.float32)).reshape(M, s.size)
    out = np.zeros(dp, dtype=np.float32)
    _check(lib().dqo_sign_reduce(_p(s, C.c_int64), s.size, _p(pk, C.c_uint8), pk.shape[1], M,
                                 _p(sc, C.c_float) if sc is not None else None, 1 if majority else 0,
                                 _p(out, C.c_float)), "sign_reduce")
    return out


# --------------------------------------------------------- one bit-width per worker and tensor
def _widths2d(b, M, n_seg):
    a = np.ascontiguousarray(np.asarray(b, dtype=np.int32))
    if a.shape != (M, n_seg):
        raise ValueError("widths must be [M][n_seg]")
    return a


def select_bits_per_worker(norms, t, T, eps_hat_q, alpha, b_min, b_max, per_tensor=False):
    """-> b[M][n_seg] int32."""
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32))
    if n.ndim != 2:
        raise ValueError("norms must be [M][n_seg]")
    b = np.zeros(n.shape, dtype=np.int32)
    _check(lib().dqo_select_bits_per_worker(_p(n, C.c_float), n.shape[0], n.shape[1], t, T, eps_hat_q, alpha,
                                            b_min, b_max, 1 if per_tensor else 0, _p(b, C.c_int32)),
           "select_bits_per_worker")
    return b


def quantize_pack_w(seg_len, grads, norms, b, seed, step, worker_base=0):
    """-> packed[M][stride], stride = the longest worker message; shorter messages are zero padded."""
    s = _segs(seg_len)
    dp = padded_elems(s)
    g = _grads2d(grads, dp)
    M = g.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    w = _widths2d(b, M, s.size)
    stride = max(packed_bytes_v(s, w[i]) for i in range(M))
    packed = np.zeros((M, stride), dtype=np.uint8)
    scratch = np.zeros(2 * dp, dtype=np.uint8)
    _check(lib().dqo_quantize_pack_w(_p(s, C.c_int64), s.size, _p(g, C.c_float), g.shape[1], M, _p(n, C.c_float),
                                     _p(w, C.c_int32), seed, step, worker_base, _p(packed, C.c_uint8), stride,
                                     _p(scratch, C.c_uint8)), "quantize_pack_w")
    return packed


def unpack_dequant_reduce_w(seg_len, packed, norms, b):
    s = _segs(seg_len)
    dp = padded_elems(s)
    pk = np.asarray(packed)
    if pk.dtype != np.uint8 or pk.ndim != 2 or not pk.flags.c_contiguous:
        raise ValueError("packed must be a C-contiguous uint8 [M][stride] array")
    M = pk.shape[0]
    n = np.ascontiguousarray(np.asarray(norms, dtype=np.float32)).reshape(M, s.size)
    w = _widths2d(b, M, s.size)
    out = np.zeros(dp, dtype=np.float32)
    scratch = np.zeros(2 * M * dp, dtype=np.uint8)
    _check(lib().dqo_unpack_dequant_reduce_w(_p(s, C.c_int64), s.size, _p(pk, C.c_uint8), pk.shape[1], M,
                                             _p(n, C.c_float), _p(w, C.c_int32), _p(out, C.c_float),
                                             _p(scratch, C.c_uint8)), "unpack_dequant_reduce_w")
    return out
