"""Helpers shared by the GPU parity tests (data movement only, no arithmetic)."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth

# The bar set for the path: max |y - y_ref| <= 1e-3 * ||y_ref||_inf against the fp64 oracle.
BAR = 1e-3
# What the streaming kernels actually promise: exact integer accumulation of 23-bit
# fixed-point activations plus fp32 rounding of t and y  ->  a few 1e-7 in practice.
DECODE_TOL = 1e-5


def to_device(x: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def new_output(batch: int, d_out: int, y_dtype: str = "f32"):
    """A NaN-filled device array for y."""
    import torch
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[y_dtype]
    return torch.full((batch, d_out), float("nan"), dtype=tdt, device="cuda")


def output_to_numpy(y) -> np.ndarray:
    """Device output -> numpy (fp32 stays fp32; the 16-bit types are widened exactly to fp64)."""
    import torch
    if y.dtype == torch.float32:
        return y.cpu().numpy()
    return y.cpu().to(torch.float64).numpy()


def check_rounded(y: np.ndarray, ref: np.ndarray, y_dtype: str, tol: float) -> None:
    """A 16-bit output against the fp64 oracle: the path's own tolerance plus one unit in the last
    place of the output type at each element (the result is rounded once more than the fp32 one)."""
    ulp = {"bf16": 2.0 ** -8, "f16": 2.0 ** -10}[y_dtype]
    lim = 65504.0 if y_dtype == "f16" else np.inf
    inside = np.abs(ref) < lim * (1 - 2.0 ** -11)
    assert np.isfinite(y[inside]).all(), "non-finite output"
    bound = tol * np.abs(ref).max() + ulp * np.abs(ref) + (2.0 ** -24 if y_dtype == "f16" else 0.0)
    bad = np.abs(y - ref)[inside] > bound[inside]
    assert not bad.any(), float((np.abs(y - ref)[inside] / bound[inside]).max())
    # beyond the fp16 range the conversion gives infinity of the right sign (or the largest value, within rounding of the edge)
    over = np.abs(ref) > lim * (1 + 2.0 ** -10)
    assert np.all(np.isinf(y[over]) & (np.sign(y[over]) == np.sign(ref[over])))


class Layer:
    """A synthetic layer resident on the GPU plus everything the oracle needs."""

    def __init__(self, d_out, d_in, r, x_dtype="bf16", seed=0, flags=0, data: synth.LayerData | None = None,
                 y_dtype="f32"):
        self.d_out, self.d_in, self.r, self.x_dtype, self.y_dtype = d_out, d_in, r, x_dtype, y_dtype
        if data is None:
            shp = synth.LinearShape("t", d_out, d_in, r)
            data = synth.LayerData(shp, synth.gen_sign_words(d_out, r, seed + 1), synth.gen_sign_words(d_in, r, seed + 2),
                                   synth.gen_scales(d_out, seed + 3), synth.gen_scales(d_in, seed + 4))
        self.data = data
        self.h = nq.nq_binlr_create(d_out, d_in, r, data.U_words, data.V_words, data.s_out, data.s_in,
                                    nq.DTYPE_BY_NAME[x_dtype], nq.DTYPE_BY_NAME[y_dtype], flags)

    def close(self):
        if self.h:
            nq.nq_binlr_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def forward(self, x_np: np.ndarray):
        import torch
        batch = x_np.shape[0]
        x = to_device(x_np, self.x_dtype)
        y = new_output(batch, self.d_out, self.y_dtype)
        nq.nq_binlr_forward(self.h, x, y, batch)
        torch.cuda.synchronize()
        return output_to_numpy(y)

    def oracle(self, x_np: np.ndarray, threads=0, return_t=False):
        d = self.data
        return oracle.forward_factored(d.U_words, d.V_words, d.s_out, d.s_in, self.d_out, self.d_in, self.r,
                                       synth.x_as_f64(x_np, self.x_dtype), threads=threads, return_t=return_t)

    def oracle_rows(self, x_np: np.ndarray, rows):
        d = self.data
        return oracle.forward_dense_rows(d.U_words, d.V_words, d.s_out, d.s_in, self.d_out, self.d_in, self.r,
                                         synth.x_as_f64(x_np, self.x_dtype), rows)


def rel_err(y: np.ndarray, ref: np.ndarray) -> float:
    assert y.shape == ref.shape, (y.shape, ref.shape)
    assert np.isfinite(y).all(), "non-finite output"
    return float(np.abs(y.astype(np.float64) - ref).max() / np.abs(ref).max())
