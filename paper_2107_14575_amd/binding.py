"""Thin ctypes binding of libdq.so.  Argument marshalling only: pointers, sizes and the current
torch stream go straight to the C ABI (``include/dq.h``); no arithmetic of the method happens here
and there is no fallback -- without the built library every call raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libdq.so")

DQ_OK = 0
GRANULE = 128
MAX_WORKERS = 64

EXPORTS = (
    # plan and sizes
    "dq_plan_create", "dq_plan_destroy", "dq_plan_num_segments", "dq_plan_padded_elems", "dq_plan_segment_start",
    "dq_plan_has_device", "dq_plan_is_chunk_local", "dq_packed_bytes", "dq_packed_bytes_v", "dq_workspace_bytes",
    # the path
    "dq_norm", "dq_norm_linf", "dq_norm_static_scratch", "dq_norm_static_scratch_max_bytes", "dq_select_bits", "dq_select_bits_linf", "dq_quantize_pack",
    "dq_unpack_dequant_reduce", "dq_unpack_dequant_reduce_update", "dq_norm_quantize_pack",
    # widths per tensor / per worker, rules on the GPU
    "dq_select_bits_per_tensor", "dq_select_bits_per_worker", "dq_select_bits_device", "dq_widths_create",
    "dq_widths_create_per_worker", "dq_widths_destroy", "dq_widths_set", "dq_widths_packed_bytes",
    "dq_widths_worker_packed_bytes", "dq_quantize_pack_v", "dq_norm_quantize_pack_v", "dq_unpack_dequant_reduce_v",
    "dq_bracketed_workspace_bytes", "dq_norm_quantize_pack_bracketed", "dq_norm_quantize_pack_bracketed_v",
    "dq_norm_bracket",
    "dq_unpack_dequant_reduce_update_v",
    # sign-only baseline
    "dq_sign_pack", "dq_sign_reduce", "dq_sign_majority",
    # accounting and aids
    "dq_alpha_est", "dq_comm_cost_bits", "dq_comm_cost_bits_per_tensor", "dq_status_string",
)


class DQError(RuntimeError):
    def __init__(self, what: str, status: int, text: str):
        super().__init__(f"{what}: {text} (status {status})")
        self.status = status


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen the in-tree libdq.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2107_14575_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(_LIB_PATH)
    vp, i64, i32, f32p = C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_float)
    L.dq_plan_create.argtypes = [C.POINTER(i64), i32, C.POINTER(vp)]
    L.dq_plan_create.restype = C.c_int
    L.dq_plan_destroy.argtypes = [vp]
    L.dq_plan_destroy.restype = None
    L.dq_plan_num_segments.argtypes = [vp]
    L.dq_plan_num_segments.restype = i32
    L.dq_plan_padded_elems.argtypes = [vp]
    L.dq_plan_padded_elems.restype = i64
    L.dq_plan_segment_start.argtypes = [vp, i32]
    L.dq_plan_segment_start.restype = i64
    L.dq_packed_bytes.argtypes = [vp, C.c_int]
    L.dq_packed_bytes.restype = i64
    L.dq_workspace_bytes.argtypes = [vp, C.c_int]
    L.dq_workspace_bytes.restype = i64
    L.dq_plan_has_device.argtypes = [vp]
    L.dq_plan_has_device.restype = C.c_int
    L.dq_plan_is_chunk_local.argtypes = [vp]
    L.dq_plan_is_chunk_local.restype = C.c_int
    L.dq_norm_quantize_pack.argtypes = [vp, vp, i64, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_uint32, C.c_uint32,
                                        vp, vp, i64, vp]
    L.dq_norm_quantize_pack.restype = C.c_int
    L.dq_norm.argtypes = [vp, vp, i64, C.c_int, vp, vp, vp]
    L.dq_norm.restype = C.c_int
    L.dq_norm_linf.argtypes = [vp, vp, i64, C.c_int, vp, vp, vp]
    L.dq_norm_linf.restype = C.c_int
    L.dq_norm_static_scratch.argtypes = [vp, vp, i64, C.c_int, C.c_int, vp, vp]
    L.dq_norm_static_scratch.restype = C.c_int
    L.dq_norm_static_scratch_max_bytes.argtypes = []
    L.dq_norm_static_scratch_max_bytes.restype = i64
    L.dq_select_bits.argtypes = [f32p, C.c_int, C.c_int, i64, i64, C.c_double, C.c_double,
                                 C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_double)]
    L.dq_select_bits.restype = C.c_int
    L.dq_select_bits_linf.argtypes = L.dq_select_bits.argtypes
    L.dq_select_bits_linf.restype = C.c_int
    L.dq_quantize_pack.argtypes = [vp, vp, i64, C.c_int, vp, C.c_int, C.c_uint64, C.c_uint32,
                                   C.c_uint32, vp, i64, vp]
    L.dq_quantize_pack.restype = C.c_int
    L.dq_unpack_dequant_reduce.argtypes = [vp, vp, i64, C.c_int, vp, C.c_int, vp, vp]
    L.dq_unpack_dequant_reduce.restype = C.c_int
    L.dq_unpack_dequant_reduce_update.argtypes = [vp, vp, i64, C.c_int, vp, C.c_int, C.c_float, vp, vp, vp]
    L.dq_unpack_dequant_reduce_update.restype = C.c_int
    i32p = C.POINTER(C.c_int32)
    L.dq_select_bits_per_tensor.argtypes = [f32p, C.c_int, C.c_int, i64, i64, C.c_double, C.c_double,
                                            C.c_int, C.c_int, i32p, C.POINTER(C.c_double)]
    L.dq_select_bits_per_tensor.restype = C.c_int
    L.dq_packed_bytes_v.argtypes = [vp, i32p]
    L.dq_packed_bytes_v.restype = i64
    L.dq_comm_cost_bits_per_tensor.argtypes = [C.c_int, C.POINTER(C.c_int64), i32p, i32, C.c_int]
    L.dq_comm_cost_bits_per_tensor.restype = i64
    L.dq_widths_create.argtypes = [vp, C.POINTER(vp)]
    L.dq_widths_create.restype = C.c_int
    L.dq_widths_destroy.argtypes = [vp]
    L.dq_widths_destroy.restype = None
    L.dq_widths_set.argtypes = [vp, i32p, vp]
    L.dq_widths_set.restype = C.c_int
    L.dq_widths_packed_bytes.argtypes = [vp]
    L.dq_widths_packed_bytes.restype = i64
    L.dq_widths_create_per_worker.argtypes = [vp, C.c_int, C.POINTER(vp)]
    L.dq_widths_create_per_worker.restype = C.c_int
    L.dq_widths_worker_packed_bytes.argtypes = [vp, C.c_int]
    L.dq_widths_worker_packed_bytes.restype = i64
    L.dq_select_bits_per_worker.argtypes = [f32p, C.c_int, C.c_int, i64, i64, C.c_double, C.c_double,
                                            C.c_int, C.c_int, C.c_int, i32p]
    L.dq_select_bits_per_worker.restype = C.c_int
    L.dq_select_bits_device.argtypes = [vp, vp, vp, C.c_int, i64, i64, C.c_double, C.c_double, C.c_int, C.c_int,
                                        C.c_int, vp, vp, vp, vp]
    L.dq_select_bits_device.restype = C.c_int
    L.dq_quantize_pack_v.argtypes = [vp, vp, vp, i64, C.c_int, vp, C.c_uint64, C.c_uint32, C.c_uint32, vp, i64, vp]
    L.dq_quantize_pack_v.restype = C.c_int
    L.dq_norm_quantize_pack_v.argtypes = [vp, vp, vp, i64, C.c_int, C.c_int, C.c_uint64, C.c_uint32, C.c_uint32,
                                          vp, vp, i64, vp]
    L.dq_norm_quantize_pack_v.restype = C.c_int
    L.dq_norm_quantize_pack_bracketed_v.argtypes = [vp, vp, vp, i64, C.c_int, C.c_int, vp, vp, C.c_uint64, C.c_uint32,
                                                    C.c_uint32, vp, vp, i64, vp, vp, vp]
    L.dq_norm_quantize_pack_bracketed_v.restype = C.c_int
    L.dq_norm_bracket.argtypes = [vp, i64, C.c_float, vp, vp, vp]
    L.dq_norm_bracket.restype = C.c_int
    L.dq_bracketed_workspace_bytes.argtypes = [vp, C.c_int]
    L.dq_bracketed_workspace_bytes.restype = i64
    L.dq_norm_quantize_pack_bracketed.argtypes = [vp, vp, i64, C.c_int, C.c_int, vp, vp, C.c_int, C.c_uint64, C.c_uint32,
                                                  C.c_uint32, vp, vp, i64, vp, vp, vp]
    L.dq_norm_quantize_pack_bracketed.restype = C.c_int
    L.dq_unpack_dequant_reduce_v.argtypes = [vp, vp, vp, i64, C.c_int, vp, vp, vp]
    L.dq_unpack_dequant_reduce_v.restype = C.c_int
    L.dq_unpack_dequant_reduce_update_v.argtypes = [vp, vp, vp, i64, C.c_int, vp, C.c_float, vp, vp, vp]
    L.dq_unpack_dequant_reduce_update_v.restype = C.c_int
    L.dq_sign_pack.argtypes = [vp, vp, i64, C.c_int, vp, i64, vp]
    L.dq_sign_pack.restype = C.c_int
    L.dq_sign_reduce.argtypes = [vp, vp, i64, C.c_int, vp, vp, vp]
    L.dq_sign_reduce.restype = C.c_int
    L.dq_sign_majority.argtypes = [vp, vp, i64, C.c_int, vp, vp]
    L.dq_sign_majority.restype = C.c_int
    L.dq_alpha_est.argtypes = [C.c_double, C.c_double, i64]
    L.dq_alpha_est.restype = C.c_double
    L.dq_comm_cost_bits.argtypes = [C.c_int, i64, C.c_int, i32, C.c_int]
    L.dq_comm_cost_bits.restype = i64
    L.dq_status_string.argtypes = [C.c_int]
    L.dq_status_string.restype = C.c_char_p
    _lib = L
    return L


def _check(what: str, status: int) -> None:
    if status != DQ_OK:
        raise DQError(what, status, load_library().dq_status_string(status).decode())


def _stream_handle(stream) -> int:
    """hipStream_t of a torch stream (default: torch's current stream), as an integer."""
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


class Plan:
    """Layout of a list of tensors in the padded flat index space (see ``include/dq.h``)."""

    def __init__(self, seg_len):
        lens = np.ascontiguousarray(np.asarray(seg_len, dtype=np.int64).reshape(-1))
        L = load_library()
        handle = C.c_void_p()
        _check("dq_plan_create",
               L.dq_plan_create(lens.ctypes.data_as(C.POINTER(C.c_int64)), lens.size, C.byref(handle)))
        self._h = handle
        self.seg_len = lens

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            load_library().dq_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("plan is closed")
        return self._h

    @property
    def n_seg(self) -> int:
        return int(load_library().dq_plan_num_segments(self.handle))

    @property
    def padded_elems(self) -> int:
        return int(load_library().dq_plan_padded_elems(self.handle))

    @property
    def has_device(self) -> bool:
        return bool(load_library().dq_plan_has_device(self.handle))

    @property
    def chunk_local(self) -> bool:
        return bool(load_library().dq_plan_is_chunk_local(self.handle))

    def segment_start(self, l: int) -> int:
        return int(load_library().dq_plan_segment_start(self.handle, l))

    def packed_bytes(self, b: int) -> int:
        return int(load_library().dq_packed_bytes(self.handle, b))

    def workspace_bytes(self, M: int) -> int:
        return int(load_library().dq_workspace_bytes(self.handle, M))


def norm(plan: Plan, grads, norms_out, workspace, stream=None) -> None:
    """grads: float32 CUDA tensor [M][stride]; norms_out: float32 CUDA [M][n_seg];
    workspace: CUDA byte tensor of plan.workspace_bytes(M)."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    _check("dq_norm", load_library().dq_norm(plan.handle, grads.data_ptr(), stride, M,
                                             norms_out.data_ptr(), workspace.data_ptr(),
                                             _stream_handle(stream)))


def norm_linf(plan: Plan, grads, norms_out, workspace, stream=None) -> None:
    """As norm, with the max norm (p = infinity)."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    _check("dq_norm_linf", load_library().dq_norm_linf(plan.handle, grads.data_ptr(), stride, M,
                                                       norms_out.data_ptr(), workspace.data_ptr(),
                                                       _stream_handle(stream)))


def norm_static_scratch(plan: Plan, grads, norms_out, linf: bool = False, stream=None) -> None:
    """norm / norm_linf without a workspace: the partial sums live in a fixed array inside the library
    (plan.workspace_bytes(M) must not exceed norm_static_scratch_max_bytes()); allocates nothing."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    _check("dq_norm_static_scratch",
           load_library().dq_norm_static_scratch(plan.handle, grads.data_ptr(), stride, M, 1 if linf else 0,
                                                 norms_out.data_ptr(), _stream_handle(stream)))


def norm_static_scratch_max_bytes() -> int:
    return int(load_library().dq_norm_static_scratch_max_bytes())


def _select_bits(name, norms_host, t, T, eps_hat_q, alpha, b_min, b_max):
    n = np.ascontiguousarray(np.asarray(norms_host, dtype=np.float32))
    if n.ndim != 2:
        raise ValueError("norms must be [M][n_seg]")
    b = C.c_int(0)
    gbar = C.c_double(0.0)
    fn = getattr(load_library(), name)
    _check(name, fn(n.ctypes.data_as(C.POINTER(C.c_float)), n.shape[0], n.shape[1],
                    t, T, eps_hat_q, alpha, b_min, b_max, C.byref(b), C.byref(gbar)))
    return int(b.value), float(gbar.value)


def select_bits(norms_host, t: int, T: int, eps_hat_q: float, alpha: float, b_min: int, b_max: int):
    """norms_host: host float32 array [M][n_seg] -> (b, Gbar)."""
    return _select_bits("dq_select_bits", norms_host, t, T, eps_hat_q, alpha, b_min, b_max)


def select_bits_linf(norms_host, t: int, T: int, eps_hat_q: float, alpha: float, b_min: int, b_max: int):
    """select_bits for norms from norm_linf."""
    return _select_bits("dq_select_bits_linf", norms_host, t, T, eps_hat_q, alpha, b_min, b_max)


def norm_quantize_pack(plan: Plan, grads, b: int, seed: int, step: int, norms_out, packed_out,
                       worker_base: int = 0, linf: bool = False, stream=None) -> None:
    """One pass over the gradient for chunk-local plans: norms (written to norms_out) and messages."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    _check("dq_norm_quantize_pack",
           load_library().dq_norm_quantize_pack(plan.handle, grads.data_ptr(), stride, M, 1 if linf else 0, b, seed,
                                                step, worker_base, norms_out.data_ptr(), packed_out.data_ptr(),
                                                int(packed_out.stride(0)), _stream_handle(stream)))


def norm_bracket(norms, margin: float, lo_out, hi_out, stream=None) -> None:
    """lo_out = norms * (1 - margin), hi_out = norms * (1 + margin): CUDA float32 tensors of one shape."""
    if not (norms.is_contiguous() and lo_out.is_contiguous() and hi_out.is_contiguous()):
        raise ValueError("contiguous tensors")
    if lo_out.numel() != norms.numel() or hi_out.numel() != norms.numel():
        raise ValueError("one bracket per norm")
    _check("dq_norm_bracket", load_library().dq_norm_bracket(norms.data_ptr(), norms.numel(), margin, lo_out.data_ptr(),
                                                             hi_out.data_ptr(), _stream_handle(stream)))


def bracketed_workspace_bytes(plan: Plan, M: int) -> int:
    return int(load_library().dq_bracketed_workspace_bytes(plan.handle, M))


def norm_quantize_pack_bracketed(plan: Plan, grads, norm_lo, norm_hi, b: int, seed: int, step: int, norms_out,
                                 packed_out, workspace, worker_base: int = 0, stats=None, linf: bool = False,
                                 stream=None) -> None:
    """One pass over the gradient for any plan, given a bracket [norm_lo, norm_hi] (CUDA float32
    [M][n_seg]) for every norm: norms (written to norms_out) and the messages of quantize_pack for
    them.  workspace: uint8 CUDA tensor of bracketed_workspace_bytes(plan, M); stats: optional CUDA
    int64 [2] (elements settled afterwards, chunks quantized again)."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    if workspace.numel() * workspace.element_size() < bracketed_workspace_bytes(plan, M):
        raise ValueError("workspace too small: see bracketed_workspace_bytes")
    _check("dq_norm_quantize_pack_bracketed",
           load_library().dq_norm_quantize_pack_bracketed(
               plan.handle, grads.data_ptr(), stride, M, 1 if linf else 0, norm_lo.data_ptr(), norm_hi.data_ptr(), b,
               seed, step,
               worker_base, norms_out.data_ptr(), packed_out.data_ptr(), int(packed_out.stride(0)),
               workspace.data_ptr(), stats.data_ptr() if stats is not None else None, _stream_handle(stream)))


def quantize_pack(plan: Plan, grads, norms, b: int, seed: int, step: int, packed_out,
                  worker_base: int = 0, stream=None) -> None:
    """packed_out: uint8 CUDA tensor [M][stride_bytes], written in full per message."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    _check("dq_quantize_pack",
           load_library().dq_quantize_pack(plan.handle, grads.data_ptr(), stride, M, norms.data_ptr(), b,
                                           seed, step, worker_base, packed_out.data_ptr(),
                                           int(packed_out.stride(0)), _stream_handle(stream)))


def unpack_dequant_reduce(plan: Plan, packed, norms, b: int, out, stream=None) -> None:
    """packed: uint8 CUDA [M][stride_bytes]; out: float32 CUDA [D']."""
    M = int(packed.shape[0])
    _check("dq_unpack_dequant_reduce",
           load_library().dq_unpack_dequant_reduce(plan.handle, packed.data_ptr(), int(packed.stride(0)), M,
                                                   norms.data_ptr(), b, out.data_ptr(),
                                                   _stream_handle(stream)))


def unpack_dequant_reduce_update(plan: Plan, packed, norms, b: int, eta: float, x, ghat=None, stream=None) -> None:
    """x: float32 CUDA [D'], updated in place to x - eta * g_hat; ghat (optional) receives g_hat."""
    M = int(packed.shape[0])
    _check("dq_unpack_dequant_reduce_update",
           load_library().dq_unpack_dequant_reduce_update(
               plan.handle, packed.data_ptr(), int(packed.stride(0)), M, norms.data_ptr(), b, eta,
               x.data_ptr(), None if ghat is None else ghat.data_ptr(), _stream_handle(stream)))


def alpha_est(F_t: float, F_0: float, t: int) -> float:
    v = float(load_library().dq_alpha_est(F_t, F_0, t))
    if v < 0:
        raise DQError("dq_alpha_est", -1, "invalid argument")
    return v


def comm_cost_bits(W: int, d: int, b: int, n_norms: int = 1, B_pre: int = 32) -> int:
    v = int(load_library().dq_comm_cost_bits(W, d, b, n_norms, B_pre))
    if v < 0:
        raise DQError("dq_comm_cost_bits", -1, "invalid argument")
    return v


# ------------------------------------------------------------------ one bit-width per tensor
def _widths_array(b_seg, n_seg):
    b = np.ascontiguousarray(np.asarray(b_seg, dtype=np.int32).reshape(-1))
    if b.size != n_seg:
        raise ValueError("one width per tensor")
    return b


def select_bits_per_tensor(norms_host, t: int, T: int, eps_hat_q: float, alpha: float, b_min: int, b_max: int):
    """norms_host [M][n_seg] -> (b[n_seg] int32, Nbar[n_seg] float64)."""
    n = np.ascontiguousarray(np.asarray(norms_host, dtype=np.float32))
    if n.ndim != 2:
        raise ValueError("norms must be [M][n_seg]")
    b = np.zeros(n.shape[1], dtype=np.int32)
    nbar = np.zeros(n.shape[1], dtype=np.float64)
    _check("dq_select_bits_per_tensor",
           load_library().dq_select_bits_per_tensor(n.ctypes.data_as(C.POINTER(C.c_float)), n.shape[0], n.shape[1],
                                                    t, T, eps_hat_q, alpha, b_min, b_max,
                                                    b.ctypes.data_as(C.POINTER(C.c_int32)),
                                                    nbar.ctypes.data_as(C.POINTER(C.c_double))))
    return b, nbar


def packed_bytes_v(plan: Plan, b_seg) -> int:
    b = _widths_array(b_seg, plan.n_seg)
    return int(load_library().dq_packed_bytes_v(plan.handle, b.ctypes.data_as(C.POINTER(C.c_int32))))


def comm_cost_bits_per_tensor(W: int, seg_len, b_seg, B_pre: int = 32) -> int:
    lens = np.ascontiguousarray(np.asarray(seg_len, dtype=np.int64).reshape(-1))
    b = _widths_array(b_seg, lens.size)
    v = int(load_library().dq_comm_cost_bits_per_tensor(W, lens.ctypes.data_as(C.POINTER(C.c_int64)),
                                                        b.ctypes.data_as(C.POINTER(C.c_int32)), lens.size, B_pre))
    if v < 0:
        raise ValueError("comm_cost_bits_per_tensor: bad argument")
    return v


class Widths:
    """Level bit-widths of a plan's tensors as a table on the plan's GPU: one row shared by the
    workers (workers=None), or one row per worker (workers=M; b_seg is then [M][n_seg])."""

    def __init__(self, plan: Plan, b_seg=None, stream=None, workers=None):
        handle = C.c_void_p()
        if workers is None:
            _check("dq_widths_create", load_library().dq_widths_create(plan.handle, C.byref(handle)))
        else:
            _check("dq_widths_create_per_worker",
                   load_library().dq_widths_create_per_worker(plan.handle, int(workers), C.byref(handle)))
        self._h = handle
        self.plan = plan
        self.workers = workers
        if b_seg is not None:
            self.set(b_seg, stream)

    def set(self, b_seg, stream=None) -> None:
        rows = 1 if self.workers is None else int(self.workers)
        b = np.ascontiguousarray(np.asarray(b_seg, dtype=np.int32).reshape(-1))
        if b.size != rows * self.plan.n_seg:
            raise ValueError("one width per tensor" if rows == 1 else "one width per worker and tensor")
        _check("dq_widths_set", load_library().dq_widths_set(self.handle, b.ctypes.data_as(C.POINTER(C.c_int32)),
                                                             _stream_handle(stream)))

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("widths are closed")
        return self._h

    @property
    def packed_bytes(self) -> int:
        return int(load_library().dq_widths_packed_bytes(self.handle))

    def worker_packed_bytes(self, worker: int) -> int:
        return int(load_library().dq_widths_worker_packed_bytes(self.handle, worker))

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            load_library().dq_widths_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def select_bits_per_worker(norms_host, t: int, T: int, eps_hat_q: float, alpha: float, b_min: int, b_max: int,
                           per_tensor: bool = False):
    """norms_host [M][n_seg] -> b[M][n_seg] int32: Eq. (17) with each worker's own norm."""
    n = np.ascontiguousarray(np.asarray(norms_host, dtype=np.float32))
    if n.ndim != 2:
        raise ValueError("norms must be [M][n_seg]")
    b = np.zeros(n.shape, dtype=np.int32)
    _check("dq_select_bits_per_worker",
           load_library().dq_select_bits_per_worker(n.ctypes.data_as(C.POINTER(C.c_float)), n.shape[0], n.shape[1],
                                                    t, T, eps_hat_q, alpha, b_min, b_max, 1 if per_tensor else 0,
                                                    b.ctypes.data_as(C.POINTER(C.c_int32))))
    return b


RULES = {"single": 0, "single_linf": 1, "per_tensor": 2}


def select_bits_device(plan: Plan, widths: Widths, norms, t: int, T: int, eps_hat_q: float, alpha: float,
                       b_min: int, b_max: int, rule: str = "single", b_out=None, gbar_out=None,
                       packed_bytes_out=None, stream=None) -> None:
    """The bit rule on the GPU: fills `widths` from norms (CUDA float32 [M][n_seg]) without a host
    round trip.  b_out: CUDA int32 [n_seg]; gbar_out: CUDA float64 [1] or [n_seg] (per_tensor);
    packed_bytes_out: CUDA int64 [1]; all optional."""
    ptr = lambda x: x.data_ptr() if x is not None else None
    _check("dq_select_bits_device",
           load_library().dq_select_bits_device(plan.handle, widths.handle, norms.data_ptr(), int(norms.shape[0]),
                                                t, T, eps_hat_q, alpha, b_min, b_max, RULES[rule], ptr(b_out),
                                                ptr(gbar_out), ptr(packed_bytes_out), _stream_handle(stream)))


def norm_quantize_pack_bracketed_v(plan: Plan, widths: Widths, grads, norm_lo, norm_hi, seed: int, step: int, norms_out,
                                   packed_out, workspace, worker_base: int = 0, stats=None, linf: bool = False,
                                   stream=None) -> None:
    """norm_quantize_pack_bracketed with the widths of `widths` (per tensor, shared or one row per worker)."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    if workspace.numel() * workspace.element_size() < bracketed_workspace_bytes(plan, M):
        raise ValueError("workspace too small: see bracketed_workspace_bytes")
    _check("dq_norm_quantize_pack_bracketed_v",
           load_library().dq_norm_quantize_pack_bracketed_v(
               plan.handle, widths.handle, grads.data_ptr(), stride, M, 1 if linf else 0, norm_lo.data_ptr(),
               norm_hi.data_ptr(), seed, step, worker_base, norms_out.data_ptr(), packed_out.data_ptr(),
               int(packed_out.stride(0)), workspace.data_ptr(), stats.data_ptr() if stats is not None else None,
               _stream_handle(stream)))


def quantize_pack_v(plan: Plan, widths: Widths, grads, norms, seed: int, step: int, packed_out,
                    worker_base: int = 0, stream=None) -> None:
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    _check("dq_quantize_pack_v",
           load_library().dq_quantize_pack_v(plan.handle, widths.handle, grads.data_ptr(), stride, M,
                                             norms.data_ptr(), seed, step, worker_base, packed_out.data_ptr(),
                                             int(packed_out.stride(0)), _stream_handle(stream)))


def norm_quantize_pack_v(plan: Plan, widths: Widths, grads, seed: int, step: int, norms_out, packed_out,
                         worker_base: int = 0, linf: bool = False, stream=None) -> None:
    """norm_quantize_pack with per-tensor widths (chunk-local plans)."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    _check("dq_norm_quantize_pack_v",
           load_library().dq_norm_quantize_pack_v(plan.handle, widths.handle, grads.data_ptr(), stride, M,
                                                  1 if linf else 0, seed, step, worker_base, norms_out.data_ptr(),
                                                  packed_out.data_ptr(), int(packed_out.stride(0)),
                                                  _stream_handle(stream)))


def unpack_dequant_reduce_v(plan: Plan, widths: Widths, packed, norms, out, stream=None) -> None:
    M = int(packed.shape[0])
    _check("dq_unpack_dequant_reduce_v",
           load_library().dq_unpack_dequant_reduce_v(plan.handle, widths.handle, packed.data_ptr(),
                                                     int(packed.stride(0)), M, norms.data_ptr(), out.data_ptr(),
                                                     _stream_handle(stream)))


def unpack_dequant_reduce_update_v(plan: Plan, widths: Widths, packed, norms, eta: float, x, ghat=None,
                                   stream=None) -> None:
    M = int(packed.shape[0])
    _check("dq_unpack_dequant_reduce_update_v",
           load_library().dq_unpack_dequant_reduce_update_v(plan.handle, widths.handle, packed.data_ptr(),
                                                            int(packed.stride(0)), M, norms.data_ptr(), eta,
                                                            x.data_ptr(), ghat.data_ptr() if ghat is not None else None,
                                                            _stream_handle(stream)))


# ------------------------------------------------------------------------- sign-only messages
def sign_pack(plan: Plan, grads, packed_out, stream=None) -> None:
    """packed_out: uint8 CUDA [M][>= D'/8]: every worker's sign plane."""
    M, stride = int(grads.shape[0]), int(grads.stride(0))
    _check("dq_sign_pack", load_library().dq_sign_pack(plan.handle, grads.data_ptr(), stride, M,
                                                       packed_out.data_ptr(), int(packed_out.stride(0)),
                                                       _stream_handle(stream)))


def sign_reduce(plan: Plan, packed, out, scales=None, stream=None) -> None:
    M = int(packed.shape[0])
    _check("dq_sign_reduce", load_library().dq_sign_reduce(plan.handle, packed.data_ptr(), int(packed.stride(0)), M,
                                                           scales.data_ptr() if scales is not None else None,
                                                           out.data_ptr(), _stream_handle(stream)))


def sign_majority(plan: Plan, packed, out, stream=None) -> None:
    M = int(packed.shape[0])
    _check("dq_sign_majority", load_library().dq_sign_majority(plan.handle, packed.data_ptr(),
                                                               int(packed.stride(0)), M, out.data_ptr(),
                                                               _stream_handle(stream)))
