"""fp64 CPU oracle (test infrastructure only).

Thin ctypes loader around ``nq_oracle.c``.  Only ``tests/``, the smoke entry
and the benchmark's ``cpu_baseline`` leg may import this package; the product
(``paper_2602_06694_amd``) never does, and this package never imports the
product.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nq_oracle.c")
_LIB = os.path.join(_HERE, "libnq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i64, p, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.nqo_pack_f64.argtypes = [p, i64, i64, p]; L.nqo_pack_f64.restype = ci
        L.nqo_pack_i8.argtypes = [p, i64, i64, p]; L.nqo_pack_i8.restype = ci
        L.nqo_unpack.argtypes = [p, i64, i64, p]; L.nqo_unpack.restype = None
        L.nqo_dense_weight.argtypes = [p, p, p, p, i64, i64, i64, p]; L.nqo_dense_weight.restype = None
        L.nqo_forward_dense.argtypes = [p, p, p, p, i64, i64, i64, p, i64, p]; L.nqo_forward_dense.restype = None
        L.nqo_forward_dense_rows.argtypes = [p, p, p, p, i64, i64, i64, p, i64, p, i64, p]
        L.nqo_forward_dense_rows.restype = None
        L.nqo_forward_factored.argtypes = [p, p, p, p, i64, i64, i64, p, i64, p, p, ci]
        L.nqo_forward_factored.restype = ci
        L.nqo_layer_bits.argtypes = [i64, i64, i64]; L.nqo_layer_bits.restype = i64
        L.nqo_forward_dense_rows_mid.argtypes = [p, p, p, p, p, i64, i64, i64, p, i64, p, i64, p]
        L.nqo_forward_dense_rows_mid.restype = None
        L.nqo_forward_factored_mid.argtypes = [p, p, p, p, p, i64, i64, i64, p, i64, p, p, ci]
        L.nqo_forward_factored_mid.restype = ci
        L.nqo_layer_bits_mid.argtypes = [i64, i64, i64]; L.nqo_layer_bits_mid.restype = i64
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _words(a, rows, r):
    a = np.ascontiguousarray(a, dtype=np.uint32)
    assert a.shape == (rows, (r + 31) // 32), (a.shape, rows, r)
    return a


def _f64(a, n):
    a = np.ascontiguousarray(np.asarray(a).astype(np.float64))
    assert a.shape == (n,), (a.shape, n)
    return a


def pack_signs(vals: np.ndarray) -> np.ndarray:
    """Sign-and-pack of a [rows, cols] array (float -> bit = v>=0; int8 must be +-1)."""
    L = _load()
    rows, cols = vals.shape
    out = np.empty((rows, (cols + 31) // 32), dtype=np.uint32)
    if vals.dtype == np.int8:
        v = np.ascontiguousarray(vals)
        rc = L.nqo_pack_i8(_ptr(v), rows, cols, _ptr(out))
    else:
        v = np.ascontiguousarray(vals.astype(np.float64))
        rc = L.nqo_pack_f64(_ptr(v), rows, cols, _ptr(out))
    if rc != 0:
        raise ValueError("pack_signs: NaN or non +-1 int8 input")
    return out


def unpack_signs(words: np.ndarray, cols: int) -> np.ndarray:
    L = _load()
    rows = words.shape[0]
    w = _words(words, rows, cols)
    out = np.empty((rows, cols), dtype=np.int8)
    L.nqo_unpack(_ptr(w), rows, cols, _ptr(out))
    return out


def dense_weight(U_words, V_words, s_out, s_in, d_out, d_in, r) -> np.ndarray:
    L = _load()
    U, V = _words(U_words, d_out, r), _words(V_words, d_in, r)
    so, si = _f64(s_out, d_out), _f64(s_in, d_in)
    W = np.empty((d_out, d_in), dtype=np.float64)
    L.nqo_dense_weight(_ptr(U), _ptr(V), _ptr(so), _ptr(si), d_out, d_in, r, _ptr(W))
    return W


def _x(x, d_in):
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    if x.ndim == 1:
        x = x[None, :]
    assert x.shape[1] == d_in
    return x


def forward_dense(U_words, V_words, s_out, s_in, d_out, d_in, r, x) -> np.ndarray:
    L = _load()
    U, V = _words(U_words, d_out, r), _words(V_words, d_in, r)
    so, si = _f64(s_out, d_out), _f64(s_in, d_in)
    x = _x(x, d_in)
    y = np.empty((x.shape[0], d_out), dtype=np.float64)
    L.nqo_forward_dense(_ptr(U), _ptr(V), _ptr(so), _ptr(si), d_out, d_in, r, _ptr(x), x.shape[0], _ptr(y))
    return y


def forward_dense_rows(U_words, V_words, s_out, s_in, d_out, d_in, r, x, rows) -> np.ndarray:
    L = _load()
    U, V = _words(U_words, d_out, r), _words(V_words, d_in, r)
    so, si = _f64(s_out, d_out), _f64(s_in, d_in)
    x = _x(x, d_in)
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    assert rows.min() >= 0 and rows.max() < d_out
    y = np.empty((x.shape[0], rows.size), dtype=np.float64)
    L.nqo_forward_dense_rows(_ptr(U), _ptr(V), _ptr(so), _ptr(si), d_out, d_in, r, _ptr(x), x.shape[0],
                             _ptr(rows), rows.size, _ptr(y))
    return y


def forward_factored(U_words, V_words, s_out, s_in, d_out, d_in, r, x, threads: int = 0,
                     return_t: bool = False, return_threads: bool = False):
    """Tier B.  threads=0 -> OpenMP default (all cores); 1 -> single thread."""
    L = _load()
    U, V = _words(U_words, d_out, r), _words(V_words, d_in, r)
    so, si = _f64(s_out, d_out), _f64(s_in, d_in)
    x = _x(x, d_in)
    y = np.empty((x.shape[0], d_out), dtype=np.float64)
    t = np.empty((x.shape[0], r), dtype=np.float64) if return_t else None
    used = L.nqo_forward_factored(_ptr(U), _ptr(V), _ptr(so), _ptr(si), d_out, d_in, r, _ptr(x), x.shape[0],
                                  _ptr(y), _ptr(t) if return_t else None, threads)
    out = (y,)
    if return_t:
        out += (t,)
    if return_threads:
        out += (used,)
    return out[0] if len(out) == 1 else out


def layer_bits(d_out: int, d_in: int, r: int) -> int:
    return int(_load().nqo_layer_bits(d_out, d_in, r))


# ---- three-scale variant: W^ = Diag(s_out) (U Diag(s_mid) V^T) Diag(s_in)  (Appendix F.4) ----

def forward_dense_rows_mid(U_words, V_words, s_out, s_mid, s_in, d_out, d_in, r, x, rows) -> np.ndarray:
    """Tier A (the definition) on the chosen output rows."""
    L = _load()
    U, V = _words(U_words, d_out, r), _words(V_words, d_in, r)
    so, sm, si = _f64(s_out, d_out), _f64(s_mid, r), _f64(s_in, d_in)
    x = _x(x, d_in)
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    assert rows.min() >= 0 and rows.max() < d_out
    y = np.empty((x.shape[0], rows.size), dtype=np.float64)
    L.nqo_forward_dense_rows_mid(_ptr(U), _ptr(V), _ptr(so), _ptr(sm), _ptr(si), d_out, d_in, r, _ptr(x), x.shape[0],
                                 _ptr(rows), rows.size, _ptr(y))
    return y


def forward_factored_mid(U_words, V_words, s_out, s_mid, s_in, d_out, d_in, r, x, threads: int = 0,
                         return_t: bool = False):
    """Tier B: t = V^T (s_in . x); y = s_out . (U (s_mid . t)).  return_t gives t (before s_mid)."""
    L = _load()
    U, V = _words(U_words, d_out, r), _words(V_words, d_in, r)
    so, sm, si = _f64(s_out, d_out), _f64(s_mid, r), _f64(s_in, d_in)
    x = _x(x, d_in)
    y = np.empty((x.shape[0], d_out), dtype=np.float64)
    t = np.empty((x.shape[0], r), dtype=np.float64) if return_t else None
    L.nqo_forward_factored_mid(_ptr(U), _ptr(V), _ptr(so), _ptr(sm), _ptr(si), d_out, d_in, r, _ptr(x), x.shape[0],
                               _ptr(y), _ptr(t) if return_t else None, threads)
    return (y, t) if return_t else y


def layer_bits_mid(d_out: int, d_in: int, r: int) -> int:
    return int(_load().nqo_layer_bits_mid(d_out, d_in, r))


def round_output(y: np.ndarray, dtype: str) -> np.ndarray:
    """The values an output of type ``dtype`` ("f32", "f16", "bf16") holds for the fp64 results ``y``:
    rounded to fp32 first (the path's native result type), then, for the 16-bit types, once more to
    nearest even (IEEE conversion: overflow gives infinity).  Returned as fp64.  The paper states no
    output type (Appendix E.2 speaks of fp16 / bf16 activations); this is the reading the tests check."""
    y32 = np.asarray(y, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return y32.astype(np.float64)
    if dtype == "f16":
        with np.errstate(over="ignore"):
            return y32.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        bits = y32.view(np.uint32).astype(np.uint64)
        nan = np.isnan(y32)
        rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
        out = rounded.view(np.float32).astype(np.float64)
        out[nan] = np.nan
        return out
    raise ValueError(f"unknown output type {dtype!r}")



# ---- gradients with respect to the two scale vectors, signs frozen (Section 3.4; Algorithm 1, Phase 3) ----

def scale_grads(U_words, V_words, s_out, s_in, d_out, d_in, r, x, g):
    """For a loss L of the layer output y = W^ x with upstream gradient g = dL/dy ([batch, d_out]):
        dL/ds_out_i = sum_b g_bi * sum_j (U V^T)_ij s_in_j x_bj
        dL/ds_in_j  = sum_b x_bj * sum_i g_bi s_out_i (U V^T)_ij
    (Eq. 1 differentiated; the packed signs are constants).  Plain fp64 numpy on the unpacked
    factors; returns (ds_out [d_out], ds_in [d_in])."""
    U = unpack_signs(_words(U_words, d_out, r), r).astype(np.float64)
    V = unpack_signs(_words(V_words, d_in, r), r).astype(np.float64)
    so, si = _f64(s_out, d_out), _f64(s_in, d_in)
    x = _x(x, d_in)
    g = np.ascontiguousarray(np.asarray(g, dtype=np.float64))
    assert g.shape == (x.shape[0], d_out)
    ds_out = np.zeros(d_out)
    ds_in = np.zeros(d_in)
    for b in range(x.shape[0]):
        z = U @ (V.T @ (si * x[b]))                      # U V^T (s_in . x_b)
        ds_out += g[b] * z
        w = V @ (U.T @ (so * g[b]))                      # V U^T (s_out . g_b)
        ds_in += x[b] * w
    return ds_out, ds_in
