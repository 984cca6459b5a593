"""ctypes binding of libnq_binlr.so -- argument marshalling only.

Every function has the name of the C entry point it calls (see
``include/nq_binlr.h``).  Device buffers are passed as ``torch`` CUDA tensors
(or raw integer addresses); the stream defaults to torch's current stream.
Nothing is computed here, and there is no fallback: if the shared library has
not been built, importing symbols from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

NQ_OK = 0
NQ_E_INVALID_ARG, NQ_E_SHAPE, NQ_E_ALIGN, NQ_E_NULL, NQ_E_UNSUPPORTED, NQ_E_HIP, NQ_E_TIMEOUT = -1, -2, -3, -4, -5, -6, -7
NQ_I8, NQ_F32, NQ_F16, NQ_BF16, NQ_F64 = 0, 1, 2, 3, 4
NQ_FLAG_DEFAULT, NQ_FLAG_DECODE_VALU, NQ_FLAG_NO_PREFILL = 0, 1, 2
NQ_MAX_DIM = 65536
NQ_DECODE_MAX_BATCH = 8
NQ_PREFILL_MIN_BATCH = 9
NQ_STATIC_SCRATCH_BYTES = 2 << 20

DTYPE_BY_NAME = {"f32": NQ_F32, "f16": NQ_F16, "bf16": NQ_BF16, "i8": NQ_I8}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libnq_binlr.so")
_lib = None


class NQError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"nq status {status}: {message}")
        self.status = status


def lib() -> ctypes.CDLL:
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_06694_amd.build` "
                              "(there is no CPU fallback)")
        # torch first: it brings its own copy of the HIP runtime, and a process must hold one.  Loaded the other way
        # round (this library, then torch) the system's copy comes in first and torch then finds no GPU.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32
        L.nq_packed_words.argtypes = [i64, i64]; L.nq_packed_words.restype = ctypes.c_size_t
        L.nq_pack_signs.argtypes = [vp, ci, i64, i64, vp]; L.nq_pack_signs.restype = ci
        L.nq_unpack_signs.argtypes = [vp, i64, i64, vp]; L.nq_unpack_signs.restype = ci
        L.nq_binlr_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, vp, vp, vp, vp, ci, ci, u32]
        L.nq_binlr_create.restype = ci
        L.nq_pack_signs_device.argtypes = [vp, ci, i64, i64, vp, vp, vp]; L.nq_pack_signs_device.restype = ci
        L.nq_binlr_create_from_device.argtypes = [ctypes.POINTER(vp), i64, i64, i64, vp, vp, vp, vp, ci, ci, u32]
        L.nq_binlr_create_from_device.restype = ci
        L.nq_binlr_reserve.argtypes = [vp, ci]; L.nq_binlr_reserve.restype = ci
        L.nq_binlr_reserved.argtypes = [vp, ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_size_t)]; L.nq_binlr_reserved.restype = ci
        L.nq_binlr_forward.argtypes = [vp, vp, vp, ci, vp]; L.nq_binlr_forward.restype = ci
        L.nq_binlr_forward_static.argtypes = [vp, vp, vp, ci, vp]; L.nq_binlr_forward_static.restype = ci
        L.nq_binlr_forward_exact.argtypes = [vp, vp, vp, ci, vp]; L.nq_binlr_forward_exact.restype = ci
        L.nq_set_option.argtypes = [ctypes.c_char_p, ci]; L.nq_set_option.restype = ci
        L.nq_get_option.argtypes = [ctypes.c_char_p, ctypes.POINTER(ci)]; L.nq_get_option.restype = ci
        L.nq_binlr_forward_many.argtypes = [vp, vp, vp, ci, ci, vp]; L.nq_binlr_forward_many.restype = ci
        L.nq_plan_create.argtypes = [ctypes.POINTER(vp), vp, vp, vp, ci, ci]; L.nq_plan_create.restype = ci
        L.nq_plan_forward.argtypes = [vp, vp]; L.nq_plan_forward.restype = ci
        L.nq_plan_forward_timed.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_float)]; L.nq_plan_forward_timed.restype = ci
        L.nq_binlr_forward_unscaled.argtypes = [vp, vp, vp, ci, vp]; L.nq_binlr_forward_unscaled.restype = ci
        L.nq_binlr_forward_transposed_unscaled.argtypes = [vp, vp, vp, ci, vp]; L.nq_binlr_forward_transposed_unscaled.restype = ci
        L.nq_binlr_backward_input.argtypes = [vp, vp, vp, ci, vp]; L.nq_binlr_backward_input.restype = ci
        L.nq_scale_grad.argtypes = [vp, ci, vp, ci, ci, ctypes.c_int64, vp, vp]; L.nq_scale_grad.restype = ci
        L.nq_binlr_set_mid_scale.argtypes = [vp, vp]; L.nq_binlr_set_mid_scale.restype = ci
        L.nq_probe_hbm_read.argtypes = [ctypes.c_size_t, ci, ci, ctypes.POINTER(ctypes.c_double)]; L.nq_probe_hbm_read.restype = ci
        L.nq_probe_mfma.argtypes = [ci, ctypes.POINTER(ctypes.c_double)]; L.nq_probe_mfma.restype = ci
        L.nq_plan_schedules.argtypes = [vp, ctypes.POINTER(ctypes.c_int)]; L.nq_plan_schedules.restype = ci
        L.nq_plan_destroy.argtypes = [vp]; L.nq_plan_destroy.restype = ci
        L.nq_binlr_destroy.argtypes = [vp]; L.nq_binlr_destroy.restype = ci
        L.nq_binlr_weight_bytes.argtypes = [vp]; L.nq_binlr_weight_bytes.restype = ctypes.c_size_t
        L.nq_binlr_export_words.argtypes = [vp, vp, vp]; L.nq_binlr_export_words.restype = ci
        L.nq_binlr_read_intermediate.argtypes = [vp, vp, ci]; L.nq_binlr_read_intermediate.restype = ci
        L.nq_exec_create.argtypes = [ctypes.POINTER(vp), vp, vp, vp, vp, ci]; L.nq_exec_create.restype = ci
        L.nq_exec_forward.argtypes = [vp, vp]; L.nq_exec_forward.restype = ci
        L.nq_exec_status.argtypes = [vp, vp]; L.nq_exec_status.restype = ci
        L.nq_exec_info.argtypes = [vp, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_size_t)]; L.nq_exec_info.restype = ci
        L.nq_exec_destroy.argtypes = [vp]; L.nq_exec_destroy.restype = ci
        L.nq_exec_plan_tasks.argtypes = [vp, vp, vp, vp, ci, ci, vp, ci, ctypes.POINTER(ci)]; L.nq_exec_plan_tasks.restype = ci
        L.nq_debug_slab_count.argtypes = []; L.nq_debug_slab_count.restype = ci
        dbl, szp = ctypes.c_double, ctypes.POINTER(ctypes.c_size_t)
        L.nq_lb_admm_workspace_bytes.argtypes = [i64, i64, i64, szp]; L.nq_lb_admm_workspace_bytes.restype = ci
        L.nq_lb_admm.argtypes = [vp, i64, i64, i64, vp, vp, ci, dbl, dbl, dbl, ci, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.nq_lb_admm.restype = ci
        L.nq_lb_admm_balance.argtypes = [vp, vp, i64, vp, vp, i64, i64, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.nq_lb_admm_balance.restype = ci
        L.nq_dgemm.argtypes = [ci, ci, i64, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, vp]; L.nq_dgemm.restype = ci
        L.nq_status_string.argtypes = [ci]; L.nq_status_string.restype = ctypes.c_char_p
        L.nq_last_error_string.argtypes = []; L.nq_last_error_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != NQ_OK:
        L = lib()
        raise NQError(status, f"{L.nq_status_string(status).decode()}: {L.nq_last_error_string().decode()}")


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dev_ptr(t) -> Optional[int]:
    """Address of a device buffer: torch tensor, int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("expected a device (cuda) tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def nq_status_string(status: int) -> str:
    return lib().nq_status_string(status).decode()


def nq_last_error_string() -> str:
    return lib().nq_last_error_string().decode()


def nq_packed_words(rows: int, cols: int) -> int:
    return int(lib().nq_packed_words(rows, cols))


def nq_pack_signs(signs: np.ndarray, dtype: Optional[int] = None) -> np.ndarray:
    """signs: host [rows, cols]; int8 (+-1), float32, float16, or uint16 holding bf16 bits
    (then pass dtype=NQ_BF16).  Returns canonical uint32 [rows, ceil(cols/32)]."""
    if signs.ndim != 2:
        raise ValueError("signs must be 2-D")
    if dtype is None:
        dtype = {np.dtype(np.int8): NQ_I8, np.dtype(np.float32): NQ_F32, np.dtype(np.float16): NQ_F16}.get(signs.dtype)
        if dtype is None:
            raise ValueError(f"cannot infer NQ dtype from {signs.dtype}")
    a = np.ascontiguousarray(signs)
    rows, cols = a.shape
    out = np.empty((rows, (cols + 31) // 32), dtype=np.uint32)
    _check(lib().nq_pack_signs(_np_ptr(a), dtype, rows, cols, _np_ptr(out)))
    return out


def nq_unpack_signs(words: np.ndarray, cols: int) -> np.ndarray:
    w = np.ascontiguousarray(words, dtype=np.uint32)
    rows = w.shape[0]
    if w.shape != (rows, (cols + 31) // 32):
        raise ValueError("words has the wrong shape")
    out = np.empty((rows, cols), dtype=np.int8)
    _check(lib().nq_unpack_signs(_np_ptr(w), rows, cols, _np_ptr(out)))
    return out


def nq_binlr_create(d_out: int, d_in: int, r: int, U_words: np.ndarray, V_words: np.ndarray,
                    s_out: np.ndarray, s_in: np.ndarray, x_dtype: int, y_dtype: int = NQ_F32,
                    flags: int = NQ_FLAG_DEFAULT) -> int:
    """Returns the opaque handle (an integer address)."""
    wpr = (r + 31) // 32
    U = np.ascontiguousarray(U_words, dtype=np.uint32)
    V = np.ascontiguousarray(V_words, dtype=np.uint32)
    so = np.ascontiguousarray(s_out, dtype=np.float16)
    si = np.ascontiguousarray(s_in, dtype=np.float16)
    if U.shape != (d_out, wpr) or V.shape != (d_in, wpr) or so.shape != (d_out,) or si.shape != (d_in,):
        raise ValueError("argument shapes do not match d_out, d_in, r")
    h = ctypes.c_void_p()
    _check(lib().nq_binlr_create(ctypes.byref(h), d_out, d_in, r, _np_ptr(U), _np_ptr(V), _np_ptr(so), _np_ptr(si),
                                 x_dtype, y_dtype, flags))
    return h.value


def nq_pack_signs_device(d_signs, dtype: int, rows: int, cols: int, d_words, d_invalid=None, stream=None) -> None:
    """d_signs / d_words / d_invalid: device arrays (anything with data_ptr()) or raw addresses."""
    _check(lib().nq_pack_signs_device(_dev_ptr(d_signs), dtype, rows, cols, _dev_ptr(d_words),
                                      _dev_ptr(d_invalid) if d_invalid is not None else None, _stream(stream)))


def nq_binlr_create_from_device(d_out: int, d_in: int, r: int, d_U_words, d_V_words, d_s_out, d_s_in,
                                x_dtype: int, y_dtype: int = NQ_F32, flags: int = NQ_FLAG_DEFAULT) -> int:
    """All four inputs are device arrays: canonical words (uint32 / int32 storage) and fp16 scales."""
    h = ctypes.c_void_p()
    _check(lib().nq_binlr_create_from_device(ctypes.byref(h), d_out, d_in, r, _dev_ptr(d_U_words), _dev_ptr(d_V_words),
                                             _dev_ptr(d_s_out), _dev_ptr(d_s_in), x_dtype, y_dtype, flags))
    return h.value


def nq_binlr_set_mid_scale(h: int, s_mid: Optional[np.ndarray]) -> None:
    """s_mid: r fp16 values (numpy float16 or their uint16 bits), or None to remove the scale."""
    if s_mid is None:
        _check(lib().nq_binlr_set_mid_scale(h, None))
        return
    a = np.ascontiguousarray(s_mid)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("s_mid must be float16 (or uint16 bits)")
    _check(lib().nq_binlr_set_mid_scale(h, a.ctypes.data_as(ctypes.c_void_p)))


def nq_binlr_reserve(h: int, max_batch: int) -> None:
    _check(lib().nq_binlr_reserve(h, max_batch))


def nq_binlr_reserved(h: int):
    """(largest batch that allocates nothing, bytes of the dense path's workspace)."""
    b, n = ctypes.c_int(), ctypes.c_size_t()
    _check(lib().nq_binlr_reserved(h, ctypes.byref(b), ctypes.byref(n)))
    return int(b.value), int(n.value)


def nq_binlr_forward(h: int, x, y, batch: int, stream=None) -> None:
    _check(lib().nq_binlr_forward(h, _dev_ptr(x), _dev_ptr(y), batch, _stream(stream)))


def nq_binlr_forward_static(h: int, x, y, batch: int, stream=None) -> None:
    _check(lib().nq_binlr_forward_static(h, _dev_ptr(x), _dev_ptr(y), batch, _stream(stream)))


def nq_binlr_forward_exact(h: int, x, y, batch: int, stream=None) -> None:
    _check(lib().nq_binlr_forward_exact(h, _dev_ptr(x), _dev_ptr(y), batch, _stream(stream)))


def nq_set_option(name: str, value: Optional[int]) -> None:
    """value None (or negative) restores the option's default."""
    _check(lib().nq_set_option(name.encode(), -1 if value is None else int(value)))


def nq_get_option(name: str) -> int:
    v = ctypes.c_int()
    _check(lib().nq_get_option(name.encode(), ctypes.byref(v)))
    return int(v.value)


def nq_binlr_forward_unscaled(h: int, x, z, batch: int, stream=None) -> None:
    _check(lib().nq_binlr_forward_unscaled(h, _dev_ptr(x), _dev_ptr(z), batch, _stream(stream)))


def nq_binlr_forward_transposed_unscaled(h: int, g, w, batch: int, stream=None) -> None:
    _check(lib().nq_binlr_forward_transposed_unscaled(h, _dev_ptr(g), _dev_ptr(w), batch, _stream(stream)))


def nq_binlr_backward_input(h: int, g, dx, batch: int, stream=None) -> None:
    _check(lib().nq_binlr_backward_input(h, _dev_ptr(g), _dev_ptr(dx), batch, _stream(stream)))


def nq_scale_grad(a, a_dtype: int, b, b_dtype: int, batch: int, n: int, out, stream=None) -> None:
    _check(lib().nq_scale_grad(_dev_ptr(a), a_dtype, _dev_ptr(b), b_dtype, batch, n, _dev_ptr(out), _stream(stream)))


def _ptr_array(vals: Sequence[Optional[int]]):
    arr = (ctypes.c_void_p * len(vals))(*vals)
    return arr


def nq_binlr_forward_many(hs: Sequence[int], xs: Sequence, ys: Sequence, batch: int, stream=None) -> None:
    n = len(hs)
    if len(xs) != n or len(ys) != n:
        raise ValueError("hs, xs, ys must have the same length")
    _check(lib().nq_binlr_forward_many(_ptr_array(list(hs)), _ptr_array([_dev_ptr(x) for x in xs]),
                                       _ptr_array([_dev_ptr(y) for y in ys]), n, batch, _stream(stream)))


def nq_plan_create(hs: Sequence[int], xs: Sequence, ys: Sequence, batch: int) -> int:
    n = len(hs)
    if len(xs) != n or len(ys) != n:
        raise ValueError("hs, xs, ys must have the same length")
    p = ctypes.c_void_p()
    _check(lib().nq_plan_create(ctypes.byref(p), _ptr_array(list(hs)), _ptr_array([_dev_ptr(x) for x in xs]),
                                _ptr_array([_dev_ptr(y) for y in ys]), n, batch))
    return p.value


def nq_exec_create(hs: Sequence[int], xs: Sequence, ys: Sequence, level_of: Sequence[int]) -> int:
    n = len(hs)
    if len(xs) != n or len(ys) != n or len(level_of) != n:
        raise ValueError("hs, xs, ys, level_of must have the same length")
    e = ctypes.c_void_p()
    lv = (ctypes.c_int * n)(*[int(v) for v in level_of])
    _check(lib().nq_exec_create(ctypes.byref(e), _ptr_array(list(hs)), _ptr_array([_dev_ptr(x) for x in xs]),
                                _ptr_array([_dev_ptr(y) for y in ys]), lv, n))
    return e.value


def nq_exec_forward(e: int, stream=None) -> None:
    _check(lib().nq_exec_forward(e, _stream(stream)))


def nq_exec_status(e: int, stream=None) -> None:
    """Waits for the stream; raises NQError(NQ_E_TIMEOUT) if a wait inside a launch gave up."""
    _check(lib().nq_exec_status(e, _stream(stream)))


def nq_exec_info(e: int):
    """(workgroups, tasks, LDS bytes per workgroup)."""
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_size_t()
    _check(lib().nq_exec_info(e, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return int(a.value), int(b.value), int(c.value)


def nq_exec_destroy(e: Optional[int]) -> None:
    _check(lib().nq_exec_destroy(e))


def nq_exec_plan_tasks(d_out: Sequence[int], d_in: Sequence[int], r: Sequence[int], level_of: Sequence[int],
                       n_workgroups: int) -> np.ndarray:
    """Host only: int32 [n_tasks, 7] = workgroup, phase, layer, stage, first row block, row blocks, waves per row block."""
    n = len(d_out)
    a = [np.ascontiguousarray(v, dtype=np.int64) for v in (d_out, d_in, r)]
    lv = np.ascontiguousarray(level_of, dtype=np.int32)
    cnt = ctypes.c_int()
    _check(lib().nq_exec_plan_tasks(_np_ptr(a[0]), _np_ptr(a[1]), _np_ptr(a[2]), _np_ptr(lv), n, n_workgroups, None, 0,
                                    ctypes.byref(cnt)))
    out = np.zeros((cnt.value, 7), dtype=np.int32)
    _check(lib().nq_exec_plan_tasks(_np_ptr(a[0]), _np_ptr(a[1]), _np_ptr(a[2]), _np_ptr(lv), n, n_workgroups, _np_ptr(out),
                                    cnt.value, ctypes.byref(cnt)))
    return out


def nq_plan_forward(p: int, stream=None) -> None:
    _check(lib().nq_plan_forward(p, _stream(stream)))


def nq_plan_forward_timed(p: int, stream=None) -> List[float]:
    ms = (ctypes.c_float * 4)()
    _check(lib().nq_plan_forward_timed(p, _stream(stream), ms))
    return [float(v) for v in ms]


def nq_plan_schedules(p: int) -> List[int]:
    w = (ctypes.c_int * 2)()
    _check(lib().nq_plan_schedules(p, w))
    return [int(v) for v in w]


def nq_probe_hbm_read(nbytes: int, iters: int = 10, prewarm_ms: int = 50) -> float:
    out = ctypes.c_double()
    _check(lib().nq_probe_hbm_read(nbytes, iters, prewarm_ms, ctypes.byref(out)))
    return float(out.value)


def nq_probe_mfma(dtype: int) -> float:
    out = ctypes.c_double()
    _check(lib().nq_probe_mfma(dtype, ctypes.byref(out)))
    return float(out.value)


def nq_plan_destroy(p: Optional[int]) -> None:
    _check(lib().nq_plan_destroy(p))


def nq_binlr_destroy(h: Optional[int]) -> None:
    _check(lib().nq_binlr_destroy(h))


def nq_debug_slab_count() -> int:
    return int(lib().nq_debug_slab_count())


def nq_binlr_weight_bytes(h: Optional[int]) -> int:
    return int(lib().nq_binlr_weight_bytes(h))


def nq_binlr_export_words(h: int, d_out: int, d_in: int, r: int):
    wpr = (r + 31) // 32
    U = np.empty((d_out, wpr), dtype=np.uint32)
    V = np.empty((d_in, wpr), dtype=np.uint32)
    _check(lib().nq_binlr_export_words(h, _np_ptr(U), _np_ptr(V)))
    return U, V


def nq_binlr_read_intermediate(h: int, r: int, batch: int) -> np.ndarray:
    t = np.empty((batch, r), dtype=np.float32)
    _check(lib().nq_binlr_read_intermediate(h, _np_ptr(t), batch))
    return t


# ---- latent-binary ADMM (include/nq_lb_admm.h) ----

NQ_ADMM_MAX_RANK = 8192
NQ_ADMM_MAX_DIM = 65536


def nq_lb_admm_workspace_bytes(n: int, m: int, r: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().nq_lb_admm_workspace_bytes(n, m, r, ctypes.byref(out)))
    return out.value


def nq_lb_admm(W, n: int, m: int, r: int, U0, V0, n_iters: int, rho_start: float, rho_end: float, lam: float, power_iters: int,
               U, V, Z_U, Z_V, Lambda_U, Lambda_V, workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib().nq_lb_admm(_dev_ptr(W), n, m, r, _dev_ptr(U0), _dev_ptr(V0), n_iters, rho_start, rho_end, lam, power_iters,
                            _dev_ptr(U), _dev_ptr(V), _dev_ptr(Z_U), _dev_ptr(Z_V), _dev_ptr(Lambda_U), _dev_ptr(Lambda_V),
                            _dev_ptr(workspace), workspace_bytes, _stream(stream)))


def nq_lb_admm_balance(U, Lambda_U, n: int, V, Lambda_V, m: int, r: int, U_words, V_words, s1, s2, eta, workspace,
                       workspace_bytes: int, stream=None) -> None:
    _check(lib().nq_lb_admm_balance(_dev_ptr(U), _dev_ptr(Lambda_U), n, _dev_ptr(V), _dev_ptr(Lambda_V), m, r, _dev_ptr(U_words),
                                    _dev_ptr(V_words), _dev_ptr(s1), _dev_ptr(s2), _dev_ptr(eta), _dev_ptr(workspace), workspace_bytes,
                                    _stream(stream)))


def nq_dgemm(trans_a: int, trans_b: int, M: int, N: int, K: int, alpha: float, A, lda: int, B, ldb: int, beta: float, C, ldc: int,
             stream=None) -> None:
    _check(lib().nq_dgemm(trans_a, trans_b, M, N, K, alpha, _dev_ptr(A), lda, _dev_ptr(B), ldb, beta, _dev_ptr(C), ldc, _stream(stream)))
