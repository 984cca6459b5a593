"""Pins for the CPU oracle: it is checked against things other than itself.

Every check here uses either (a) an independent library routine
(numpy.packbits / numpy.unpackbits / numpy.matmul), (b) a closed form that the
mathematics fixes, (c) complete enumeration in plain Python integers, or
(d) a value printed in the paper (tests/golden/).  A dropped term, a wrong
sign, a transposed operand or a wrong bit order in the oracle fails at least
one of them.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_2602_06694_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------- independent helpers (numpy library routines, not the oracle) ----------

def np_unpack(words: np.ndarray, cols: int) -> np.ndarray:
    """+-1 int8 matrix from packed words via numpy.unpackbits (LSB first)."""
    rows = words.shape[0]
    bits = np.unpackbits(words.view(np.uint8).reshape(rows, -1), axis=1, bitorder="little")[:, :cols]
    return (2 * bits.astype(np.int8) - 1).astype(np.int8)


def np_pack(pm1: np.ndarray) -> np.ndarray:
    rows, cols = pm1.shape
    wpr = (cols + 31) // 32
    bits = np.zeros((rows, wpr * 32), dtype=np.uint8)
    bits[:, :cols] = (pm1 > 0)
    return np.packbits(bits, axis=1, bitorder="little").view(np.uint32).reshape(rows, wpr)


def np_dense_forward(U, V, s_out, s_in, x):
    """y = (diag(s_out) U V^T diag(s_in)) x with numpy.matmul in fp64."""
    W = (s_out.astype(np.float64)[:, None] * (U.astype(np.float64) @ V.astype(np.float64).T)
         * s_in.astype(np.float64)[None, :])
    return x @ W.T


def small_case(d_out, d_in, r, batch, seed):
    rng = np.random.default_rng(seed)
    U = synth.gen_signs_pm1(d_out, r, seed + 1)
    V = synth.gen_signs_pm1(d_in, r, seed + 2)
    s_out = synth.gen_scales(d_out, seed + 3)
    s_in = synth.gen_scales(d_in, seed + 4)
    x = rng.standard_normal((batch, d_in))
    return U, V, s_out, s_in, x


# ---------- packing ----------

@pytest.mark.parametrize("cols", [1, 31, 32, 33, 63, 64, 65, 256, 3520])
def test_pack_matches_numpy_packbits(cols):
    pm1 = synth.gen_signs_pm1(7, cols, 100 + cols)
    w = oracle.pack_signs(pm1)
    assert w.dtype == np.uint32 and w.shape == (7, (cols + 31) // 32)
    assert np.array_equal(w, np_pack(pm1))
    assert np.array_equal(oracle.unpack_signs(w, cols), pm1)
    assert np.array_equal(np_unpack(w, cols), pm1)


def test_pack_bit_positions_and_padding():
    # a single +1 at column k sets exactly bit k%32 of word k//32; pad bits stay 0
    cols = 70
    for k in (0, 1, 31, 32, 33, 63, 64, 69):
        v = -np.ones((1, cols), dtype=np.int8)
        v[0, k] = 1
        w = oracle.pack_signs(v)
        expect = np.zeros(3, dtype=np.uint32)
        expect[k // 32] = np.uint32(1) << np.uint32(k % 32)
        assert np.array_equal(w[0], expect), k
    allp = oracle.pack_signs(np.ones((2, cols), dtype=np.int8))
    assert np.array_equal(allp[0], np.array([0xFFFFFFFF, 0xFFFFFFFF, 0x3F], dtype=np.uint32))
    alln = oracle.pack_signs(-np.ones((2, cols), dtype=np.int8))
    assert not alln.any()


def test_pack_sign_rule_for_floats():
    # polarity of Fig. 2(c): -1 -> 0, +1 -> 1; ties: +0.0 and -0.0 -> +1
    v = np.array([[-1.0, 1.0, 0.0, -0.0, -1e-30, 1e-30, -np.inf, np.inf]])
    w = oracle.pack_signs(v)
    assert w[0, 0] == 0b10101110
    with pytest.raises(ValueError):
        oracle.pack_signs(np.array([[1.0, np.nan]]))
    with pytest.raises(ValueError):
        oracle.pack_signs(np.array([[1, 0]], dtype=np.int8))
    with pytest.raises(ValueError):
        oracle.pack_signs(np.array([[1, 2]], dtype=np.int8))


def test_generated_words_have_zero_padding_and_uniform_signs():
    w = synth.gen_sign_words(64, 100, 5)
    assert (w[:, -1] >> 4 == 0).all()
    pm1 = np_unpack(synth.gen_sign_words(512, 512, 6), 512)
    assert abs(pm1.mean()) < 0.01


# ---------- forward: closed forms ----------

def test_all_plus_one_closed_form():
    d_out, d_in, r, batch = 37, 53, 45, 3
    _, _, s_out, s_in, x = small_case(d_out, d_in, r, batch, 11)
    ones_u = oracle.pack_signs(np.ones((d_out, r), dtype=np.int8))
    ones_v = oracle.pack_signs(np.ones((d_in, r), dtype=np.int8))
    neg_u = oracle.pack_signs(-np.ones((d_out, r), dtype=np.int8))
    neg_v = oracle.pack_signs(-np.ones((d_in, r), dtype=np.int8))
    so, si = s_out.astype(np.float64), s_in.astype(np.float64)
    expect = so[None, :] * r * (x * si[None, :]).sum(axis=1, keepdims=True)
    for fwd in (oracle.forward_dense, oracle.forward_factored):
        y = fwd(ones_u, ones_v, s_out, s_in, d_out, d_in, r, x)
        np.testing.assert_allclose(y, expect, rtol=1e-13, atol=0)
        # all(-1) V flips the sign; all(-1) both leaves y unchanged
        np.testing.assert_allclose(fwd(ones_u, neg_v, s_out, s_in, d_out, d_in, r, x), -expect, rtol=1e-13)
        np.testing.assert_allclose(fwd(neg_u, neg_v, s_out, s_in, d_out, d_in, r, x), expect, rtol=1e-13)


def test_rank_one_closed_form():
    d_out, d_in = 19, 23
    U, V, s_out, s_in, x = small_case(d_out, d_in, 1, 2, 21)
    so, si = s_out.astype(np.float64), s_in.astype(np.float64)
    inner = (x * (V[:, 0] * si)[None, :]).sum(axis=1, keepdims=True)
    expect = (so * U[:, 0])[None, :] * inner
    for fwd in (oracle.forward_dense, oracle.forward_factored):
        y = fwd(oracle.pack_signs(U), oracle.pack_signs(V), s_out, s_in, d_out, d_in, 1, x)
        np.testing.assert_allclose(y, expect, rtol=1e-13)


def test_one_hot_extracts_columns_of_dense_weight():
    d_out, d_in, r = 9, 14, 40
    U, V, s_out, s_in, _ = small_case(d_out, d_in, r, 1, 31)
    Uw, Vw = oracle.pack_signs(U), oracle.pack_signs(V)
    W = oracle.dense_weight(Uw, Vw, s_out, s_in, d_out, d_in, r)
    # element-wise definition of Eq. 1 in plain Python integers / floats
    for i in (0, 4, d_out - 1):
        for j in (0, 7, d_in - 1):
            dot = sum(int(U[i, k]) * int(V[j, k]) for k in range(r))
            assert W[i, j] == float(s_out[i]) * dot * float(s_in[j])
    eye = np.eye(d_in)
    for fwd in (oracle.forward_dense, oracle.forward_factored):
        y = fwd(Uw, Vw, s_out, s_in, d_out, d_in, r, eye)      # y[j] = W[:, j]
        np.testing.assert_allclose(y, W.T, rtol=1e-13, atol=1e-13)


# ---------- forward: complete enumeration on tiny shapes ----------

@pytest.mark.parametrize("shape", [(2, 2, 2), (3, 2, 1), (1, 3, 2)])
def test_brute_force_all_sign_patterns_exact_integers(shape):
    d_out, d_in, r = shape
    s_out = np.array([1, 2, 3][:d_out], dtype=np.float16)
    s_in = np.array([2, 1, 4][:d_in], dtype=np.float16)
    x = np.array([[3, -2, 5][:d_in], [-1, 4, 2][:d_in]], dtype=np.float64)
    nU, nV = d_out * r, d_in * r
    for ubits in itertools.product((-1, 1), repeat=nU):
        U = np.array(ubits, dtype=np.int8).reshape(d_out, r)
        Uw = oracle.pack_signs(U)
        for vbits in itertools.product((-1, 1), repeat=nV):
            V = np.array(vbits, dtype=np.int8).reshape(d_in, r)
            Vw = oracle.pack_signs(V)
            expect = [[int(s_out[i]) * sum(sum(int(U[i, k]) * int(V[j, k]) for k in range(r))
                                            * int(s_in[j]) * int(x[b, j]) for j in range(d_in))
                       for i in range(d_out)] for b in range(2)]
            ya = oracle.forward_dense(Uw, Vw, s_out, s_in, d_out, d_in, r, x)
            yb = oracle.forward_factored(Uw, Vw, s_out, s_in, d_out, d_in, r, x)
            assert ya.tolist() == expect and yb.tolist() == expect


# ---------- forward: independent library reduction ----------

@pytest.mark.parametrize("shape", [(33, 65, 31, 2), (128, 96, 64, 3), (70, 257, 100, 1)])
def test_forward_matches_numpy_matmul(shape):
    d_out, d_in, r, batch = shape
    U, V, s_out, s_in, x = small_case(d_out, d_in, r, batch, 41 + d_out)
    Uw, Vw = np_pack(U), np_pack(V)                      # packed by numpy, not by the oracle
    ref = np_dense_forward(U, V, s_out, s_in, x)
    scale = np.abs(ref).max()
    ya = oracle.forward_dense(Uw, Vw, s_out, s_in, d_out, d_in, r, x)
    yb, t = oracle.forward_factored(Uw, Vw, s_out, s_in, d_out, d_in, r, x, return_t=True)
    assert np.abs(ya - ref).max() <= 1e-12 * scale
    assert np.abs(yb - ref).max() <= 1e-12 * scale
    t_ref = (x * s_in.astype(np.float64)[None, :]) @ V.astype(np.float64)
    assert np.abs(t - t_ref).max() <= 1e-12 * np.abs(t_ref).max()
    rows = np.array([0, d_out - 1, d_out // 2])
    yr = oracle.forward_dense_rows(Uw, Vw, s_out, s_in, d_out, d_in, r, x, rows)
    assert np.abs(yr - ref[:, rows]).max() <= 1e-12 * scale


def test_config1_tier_a_equals_tier_b_and_numpy():
    c = synth.CONFIGS[1]
    shp = c.block[0]
    L = synth.gen_layer(1, 0, 0, shp)
    x = synth.x_as_f64(synth.gen_layer_x(1, 0, 0, shp, 1, c.x_dtype), c.x_dtype)
    ya = oracle.forward_dense(L.U_words, L.V_words, L.s_out, L.s_in, shp.d_out, shp.d_in, shp.r, x)
    yb = oracle.forward_factored(L.U_words, L.V_words, L.s_out, L.s_in, shp.d_out, shp.d_in, shp.r, x)
    ref = np_dense_forward(np_unpack(L.U_words, shp.r), np_unpack(L.V_words, shp.r), L.s_out, L.s_in, x)
    scale = np.abs(ref).max()
    assert np.abs(ya - yb).max() <= 1e-12 * scale
    assert np.abs(ya - ref).max() <= 1e-12 * scale


def test_factored_single_thread_equals_multi_thread():
    d_out, d_in, r, batch = 200, 300, 96, 2
    U, V, s_out, s_in, x = small_case(d_out, d_in, r, batch, 77)
    Uw, Vw = oracle.pack_signs(U), oracle.pack_signs(V)
    y1, n1 = oracle.forward_factored(Uw, Vw, s_out, s_in, d_out, d_in, r, x, threads=1, return_threads=True)
    yN, nN = oracle.forward_factored(Uw, Vw, s_out, s_in, d_out, d_in, r, x, threads=0, return_threads=True)
    assert n1 == 1 and nN >= 1
    assert np.array_equal(y1, yN)       # same summation order per output -> identical bits


# ---------- metamorphic properties of the factorization ----------

def test_metamorphic_properties():
    d_out, d_in, r, batch = 40, 72, 50, 2
    U, V, s_out, s_in, x = small_case(d_out, d_in, r, batch, 51)
    args = (d_out, d_in, r)
    Uw, Vw = oracle.pack_signs(U), oracle.pack_signs(V)
    y = oracle.forward_factored(Uw, Vw, s_out, s_in, *args, x)
    scale = np.abs(y).max()
    # linearity in x
    x2 = np.random.default_rng(1).standard_normal(x.shape)
    y2 = oracle.forward_factored(Uw, Vw, s_out, s_in, *args, x2)
    y12 = oracle.forward_factored(Uw, Vw, s_out, s_in, *args, 3.0 * x - 0.5 * x2)
    assert np.abs(y12 - (3.0 * y - 0.5 * y2)).max() <= 1e-12 * scale
    # scale invariance of the factorization (Appendix A: (eta U)(V / eta)^T): power of two -> exact
    yq = oracle.forward_factored(Uw, Vw, (s_out * np.float16(2)), (s_in / np.float16(2)), *args, x)
    assert np.array_equal(yq, y)
    # flipping column k of both factors leaves U V^T unchanged
    U2, V2 = U.copy(), V.copy()
    U2[:, 7] *= -1
    V2[:, 7] *= -1
    yf = oracle.forward_dense(oracle.pack_signs(U2), oracle.pack_signs(V2), s_out, s_in, *args, x)
    assert np.abs(yf - y).max() <= 1e-12 * scale
    # flipping only U's column changes the result (the test above is not vacuous)
    yg = oracle.forward_dense(oracle.pack_signs(U2), Vw, s_out, s_in, *args, x)
    assert np.abs(yg - y).max() > 1e-6 * scale
    # permuting the rank axis of both factors together leaves y unchanged
    perm = np.random.default_rng(2).permutation(r)
    yp = oracle.forward_factored(oracle.pack_signs(U[:, perm]), oracle.pack_signs(V[:, perm]), s_out, s_in, *args, x)
    assert np.abs(yp - y).max() <= 1e-12 * scale
    # transposition guard: s_in scales columns of the dense weight, s_out its rows
    W = oracle.dense_weight(Uw, Vw, s_out, s_in, *args)
    assert W.shape == (d_out, d_in)
    np.testing.assert_allclose(W[3, 5] / W[3, 6],
                               (float(s_in[5]) * (U[3] @ V[5].astype(np.int64)))
                               / (float(s_in[6]) * (U[3] @ V[6].astype(np.int64))), rtol=1e-12)


# ---------- storage accounting against values the paper prints ----------

def _golden():
    out = {}
    with open(os.path.join(GOLDEN, "model_sizes.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v, tol = line.split()[:3]
                out[k] = (float(v), float(tol))
    return out


def _model_linear_weights(block, n_layers):
    return n_layers * sum(s.d_out * s.d_in for s in block)


def test_storage_formula_and_paper_model_sizes():
    g = _golden()
    # formula r(n+m) + 16(n+m) (Appendix F.5)
    assert oracle.layer_bits(4096, 4096, 1024) == 1024 * 8192 + 16 * 8192
    for s in synth.llama2_70b_block():
        assert oracle.layer_bits(s.d_out, s.d_in, s.r) == s.weight_bits
    emb = {7: 2 * 32000 * 4096 * 2, 70: 2 * 32000 * 8192 * 2}      # bytes: embedding + head, 16-bit
    n7 = _model_linear_weights(synth.llama2_7b_block(), 32)
    n70 = _model_linear_weights(synth.llama2_70b_block(), 80)
    v, tol = g["llama2_7b_bf16_gb"]
    assert abs((2 * n7 + emb[7]) / 1e9 - v) <= tol
    v, tol = g["llama2_70b_bf16_gb"]
    assert abs((2 * n70 + emb[70]) / 1e9 - v) <= tol
    # 1-bit: the largest integer rank with BPW <= 1 in every layer
    bits = 0
    for s in synth.llama2_7b_block():
        r = (s.d_out * s.d_in) // (s.d_out + s.d_in) - 16
        assert oracle.layer_bits(s.d_out, s.d_in, r) <= s.d_out * s.d_in < oracle.layer_bits(s.d_out, s.d_in, r + 1)
        bits += 32 * oracle.layer_bits(s.d_out, s.d_in, r)
    v, tol = g["llama2_7b_1bit_gb"]
    assert abs((bits / 8 + emb[7]) / 1e9 - v) <= tol
    # 0.55 bit on Llama-2-70B
    v, tol = g["llama2_70b_0p55bit_gb"]
    assert abs((0.55 * n70 / 8 + emb[70]) / 1e9 - v) <= tol
    # the synthetic 70B ranks used here land at the same footprint scale (0.55-0.56 bit)
    ours = 80 * sum(oracle.layer_bits(s.d_out, s.d_in, s.r) for s in synth.llama2_70b_block())
    assert 0.55 <= ours / n70 <= 0.565
    v, tol = g["plain_binary_bpw"]
    assert v == 1.0


def test_config_bpw_values():
    expect = {(4096, 4096, 1024): 0.5078, (1024, 1024, 256): 0.5312, (11008, 4096, 1664): 0.5628,
              (8192, 8192, 2240): 0.5508, (28672, 8192, 3520): 0.5550}
    for (n, m, r), bpw in expect.items():
        assert abs(oracle.layer_bits(n, m, r) / (n * m) - bpw) < 5e-5


def test_output_rounding_pins():
    # values fixed by the two 16-bit formats themselves: ties go to the even significand,
    # fp16 overflows to infinity from 65520 on, bf16 keeps the fp32 range
    r = oracle.round_output
    one = 1.0
    assert r(np.array([one + 2.0**-8]), "bf16")[0] == 1.0                       # tie -> even (1.0)
    assert r(np.array([one + 2.0**-8 + 2.0**-20]), "bf16")[0] == one + 2.0**-7   # just above the tie
    assert r(np.array([one + 3 * 2.0**-8]), "bf16")[0] == one + 2.0**-6          # tie -> even (1 + 2^-6)
    assert r(np.array([-(one + 2.0**-7)]), "bf16")[0] == -(one + 2.0**-7)        # representable
    assert np.isfinite(r(np.array([3.0e38]), "bf16")[0])
    assert r(np.array([one + 2.0**-11]), "f16")[0] == 1.0                        # tie -> even
    assert r(np.array([one + 3 * 2.0**-11]), "f16")[0] == one + 2.0**-9
    assert r(np.array([65504.0]), "f16")[0] == 65504.0
    assert r(np.array([65519.0]), "f16")[0] == 65504.0
    assert np.isinf(r(np.array([65520.0]), "f16")[0])                            # tie -> even = infinity
    assert r(np.array([2.0**-24]), "f16")[0] == 2.0**-24                         # smallest subnormal
    assert r(np.array([2.0**-25]), "f16")[0] == 0.0                              # tie -> even (zero)
    assert r(np.array([0.1]), "f32")[0] == float(np.float32(0.1))
    assert np.isnan(r(np.array([np.nan]), "bf16")[0]) and np.isnan(r(np.array([np.nan]), "f16")[0])
    # every bf16 value is a fixed point, and rounding is monotone
    vals = np.random.default_rng(3).standard_normal(1000) * 100
    once = r(vals, "bf16")
    assert np.array_equal(r(once, "bf16"), once)
    order = np.argsort(vals)
    assert np.all(np.diff(once[order]) >= 0)
    assert np.all(np.abs(once - vals) <= np.abs(vals) * 2.0**-8)



# ---------- three-scale variant: W^ = Diag(s_out) (U Diag(s_mid) V^T) Diag(s_in)  (Appendix F.4) ----------

def test_mid_scale_of_ones_is_the_two_scale_layer_bit_for_bit():
    d_out, d_in, r, batch = 70, 130, 45, 2
    U, V, s_out, s_in, x = small_case(d_out, d_in, r, batch, 501)
    Uw, Vw = np_pack(U), np_pack(V)
    ones = np.ones(r, dtype=np.float16)
    y2, t2 = oracle.forward_factored(Uw, Vw, s_out, s_in, d_out, d_in, r, x, return_t=True)
    y3, t3 = oracle.forward_factored_mid(Uw, Vw, s_out, ones, s_in, d_out, d_in, r, x, return_t=True)
    assert np.array_equal(y2, y3) and np.array_equal(t2, t3)
    rows = np.arange(d_out)
    assert np.array_equal(oracle.forward_dense_rows(Uw, Vw, s_out, s_in, d_out, d_in, r, x, rows),
                          oracle.forward_dense_rows_mid(Uw, Vw, s_out, ones, s_in, d_out, d_in, r, x, rows))


@pytest.mark.parametrize("shape", [(33, 65, 31, 2), (128, 96, 64, 3), (70, 257, 100, 1)])
def test_mid_scale_matches_numpy_matmul(shape):
    """Independent library reduction: diag(s_out) (U diag(s_mid) V^T) diag(s_in) built with numpy."""
    d_out, d_in, r, batch = shape
    U, V, s_out, s_in, x = small_case(d_out, d_in, r, batch, 601 + d_out)
    s_mid = synth.gen_scales(r, 777 + r)
    Uw, Vw = np_pack(U), np_pack(V)
    W = (s_out.astype(np.float64)[:, None]
         * ((U.astype(np.float64) * s_mid.astype(np.float64)[None, :]) @ V.astype(np.float64).T)
         * s_in.astype(np.float64)[None, :])
    ref = x @ W.T
    scale = np.abs(ref).max()
    ya = oracle.forward_dense_rows_mid(Uw, Vw, s_out, s_mid, s_in, d_out, d_in, r, x, np.arange(d_out))
    yb, t = oracle.forward_factored_mid(Uw, Vw, s_out, s_mid, s_in, d_out, d_in, r, x, return_t=True)
    assert np.abs(ya - ref).max() <= 1e-12 * scale
    assert np.abs(yb - ref).max() <= 1e-12 * scale
    t_ref = (x * s_in.astype(np.float64)[None, :]) @ V.astype(np.float64)          # t is taken before s_mid
    assert np.abs(t - t_ref).max() <= 1e-12 * np.abs(t_ref).max()


def test_mid_scale_closed_forms():
    d_out, d_in, r, batch = 40, 50, 37, 2
    _, _, s_out, s_in, x = small_case(d_out, d_in, r, batch, 701)
    s_mid = synth.gen_scales(r, 702)
    so, sm, si = (a.astype(np.float64) for a in (s_out, s_mid, s_in))
    # all signs +1:  y_i = s_out_i (sum_k s_mid_k) (sum_j s_in_j x_j)
    ones_u, ones_v = np.ones((d_out, r), np.int8), np.ones((d_in, r), np.int8)
    y = oracle.forward_factored_mid(np_pack(ones_u), np_pack(ones_v), s_out, s_mid, s_in, d_out, d_in, r, x)
    expect = so[None, :] * sm.sum() * (x * si[None, :]).sum(axis=1)[:, None]
    assert np.abs(y - expect).max() <= 1e-12 * np.abs(expect).max()
    # s_mid = e_k selects rank k:  y_i = s_out_i U_ik sum_j V_jk s_in_j x_j
    U = synth.gen_signs_pm1(d_out, r, 703)
    V = synth.gen_signs_pm1(d_in, r, 704)
    for k in (0, 17, r - 1):
        e = np.zeros(r, dtype=np.float16)
        e[k] = 1
        y = oracle.forward_factored_mid(np_pack(U), np_pack(V), s_out, e, s_in, d_out, d_in, r, x)
        expect = so[None, :] * U[:, k].astype(np.float64)[None, :] * ((x * si[None, :]) @ V[:, k].astype(np.float64))[:, None]
        assert np.abs(y - expect).max() <= 1e-12 * np.abs(expect).max()
        ya = oracle.forward_dense_rows_mid(np_pack(U), np_pack(V), s_out, e, s_in, d_out, d_in, r, x, np.arange(d_out))
        assert np.abs(ya - expect).max() <= 1e-12 * np.abs(expect).max()
    # a negative entry of s_mid is a sign flip of that column of U (or of V)
    s_neg = s_mid.copy()
    s_neg[5] = -s_neg[5]
    U2 = U.copy()
    U2[:, 5] = -U2[:, 5]
    assert np.array_equal(oracle.forward_factored_mid(np_pack(U), np_pack(V), s_out, s_neg, s_in, d_out, d_in, r, x),
                          oracle.forward_factored_mid(np_pack(U2), np_pack(V), s_out, s_mid, s_in, d_out, d_in, r, x))


def test_mid_scale_brute_force_exact_integers():
    """Every sign pattern of a (2, 2, 2) layer with small-integer scales: results are exact integers."""
    d_out, d_in, r = 2, 2, 2
    s_out = np.array([1, 3], dtype=np.float16)
    s_mid = np.array([2, 5], dtype=np.float16)
    s_in = np.array([2, 1], dtype=np.float16)
    x = np.array([[3, -2], [-1, 4]], dtype=np.float64)
    for ubits in itertools.product((-1, 1), repeat=d_out * r):
        U = np.array(ubits, dtype=np.int8).reshape(d_out, r)
        for vbits in itertools.product((-1, 1), repeat=d_in * r):
            V = np.array(vbits, dtype=np.int8).reshape(d_in, r)
            expect = [[int(s_out[i]) * sum(sum(int(U[i, k]) * int(s_mid[k]) * int(V[j, k]) for k in range(r))
                                            * int(s_in[j]) * int(x[b, j]) for j in range(d_in))
                       for i in range(d_out)] for b in range(2)]
            Uw, Vw = oracle.pack_signs(U), oracle.pack_signs(V)
            ya = oracle.forward_dense_rows_mid(Uw, Vw, s_out, s_mid, s_in, d_out, d_in, r, x, np.arange(d_out))
            yb = oracle.forward_factored_mid(Uw, Vw, s_out, s_mid, s_in, d_out, d_in, r, x)
            assert ya.tolist() == expect and yb.tolist() == expect


def test_mid_scale_storage_formula():
    """Storage of the three-scale layer (Appendix F.4: r(n+m) + 16(n+r+m) bits), pinned three ways that
    do not retype the oracle's expression: totals worked by hand, a layer counted bit by bit from the
    arrays that would be stored, and the size the paper prints for a 1.00-bit model in this format."""
    # worked by hand: 1024 * 8192 = 8388608 sign bits, 16 * 9216 = 147456 scale bits; 1664 * 15104 = 25133056, 16 * 16768 = 268288
    assert oracle.layer_bits_mid(4096, 4096, 1024) == 8536064
    assert oracle.layer_bits_mid(11008, 4096, 1664) == 25401344
    assert oracle.layer_bits_mid(1, 1, 1) == 50                      # 2 sign bits + three fp16 scales
    # the operands are not interchangeable: a swapped or dropped term changes one of these
    assert oracle.layer_bits_mid(3, 5, 7) == 7 * 8 + 16 * 15 == 296
    assert oracle.layer_bits_mid(5, 7, 3) == 3 * 12 + 16 * 15 == 276
    assert oracle.layer_bits_mid(7, 3, 5) == 5 * 10 + 16 * 15 == 290
    # counted from the arrays a layer of this format stores: one bit per sign, 16 per fp16 scale
    for d_out, d_in, r in [(6, 9, 4), (33, 17, 40), (128, 64, 65)]:
        U = np.ones((d_out, r), np.int8)
        V = np.ones((d_in, r), np.int8)
        scales = [np.ones(d_out, np.float16), np.ones(r, np.float16), np.ones(d_in, np.float16)]
        counted = U.size + V.size + sum(8 * a.nbytes for a in scales)
        assert oracle.layer_bits_mid(d_out, d_in, r) == counted
        assert oracle.layer_bits_mid(d_out, d_in, r) - oracle.layer_bits(d_out, d_in, r) == 8 * scales[1].nbytes
    # Table 1 prints 1.33 GB for Llama-2-7B at 1.00 bit in this format (the DBF row): the largest rank
    # with at most one bit per weight in every layer, plus the 16-bit embedding and output head
    g = _golden()
    bits = 0
    for s in synth.llama2_7b_block():
        r = (s.d_out * s.d_in - 16 * (s.d_out + s.d_in)) // (s.d_out + s.d_in + 16)
        assert oracle.layer_bits_mid(s.d_out, s.d_in, r) <= s.d_out * s.d_in < oracle.layer_bits_mid(s.d_out, s.d_in, r + 1)
        bits += 32 * oracle.layer_bits_mid(s.d_out, s.d_in, r)
    v, tol = g["llama2_7b_1bit_three_scale_gb"]
    assert abs((bits / 8 + 2 * 32000 * 4096 * 2) / 1e9 - v) <= tol


# ---------- gradients of the scale vectors (signs frozen: Section 3.4; Algorithm 1, Phase 3) ----------

def test_scale_gradients_are_exact_differences_of_the_forward():
    """y is linear in each scale entry, so dL/ds_i of L = sum(g * y) equals L(s + e_i) - L(s) exactly
    (up to fp64 rounding): the gradient formulas are pinned to the forward oracle, entry by entry."""
    d_out, d_in, r, batch = 23, 37, 19, 3
    U, V, s_out, s_in, x = small_case(d_out, d_in, r, batch, 901)
    Uw, Vw = np_pack(U), np_pack(V)
    g = np.random.default_rng(902).standard_normal((batch, d_out))
    so, si = s_out.astype(np.float64), s_in.astype(np.float64)

    def loss(so_, si_):
        return float((g * oracle.forward_factored(Uw, Vw, so_, si_, d_out, d_in, r, x)).sum())

    ds_out, ds_in = oracle.scale_grads(Uw, Vw, s_out, s_in, d_out, d_in, r, x, g)
    base = loss(so, si)
    scale = max(np.abs(ds_out).max(), np.abs(ds_in).max())
    for i in range(d_out):
        e = so.copy()
        e[i] += 1.0
        assert abs((loss(e, si) - base) - ds_out[i]) <= 1e-9 * scale, i
    for j in range(d_in):
        e = si.copy()
        e[j] += 1.0
        assert abs((loss(so, e) - base) - ds_in[j]) <= 1e-9 * scale, j


def test_scale_gradients_closed_form_all_plus_one():
    """All signs +1: (U V^T)_ij = r, so ds_out_i = r sum_b g_bi (s_in . x_b) and ds_in_j = r sum_b x_bj (s_out . g_b)."""
    d_out, d_in, r, batch = 12, 9, 7, 2
    _, _, s_out, s_in, x = small_case(d_out, d_in, r, batch, 911)
    g = np.random.default_rng(912).standard_normal((batch, d_out))
    Uw, Vw = np_pack(np.ones((d_out, r), np.int8)), np_pack(np.ones((d_in, r), np.int8))
    ds_out, ds_in = oracle.scale_grads(Uw, Vw, s_out, s_in, d_out, d_in, r, x, g)
    so, si = s_out.astype(np.float64), s_in.astype(np.float64)
    e_out = r * (g * (x @ si)[:, None]).sum(axis=0)
    e_in = r * (x * (g @ so)[:, None]).sum(axis=0)
    assert np.abs(ds_out - e_out).max() <= 1e-12 * np.abs(e_out).max()
    assert np.abs(ds_in - e_in).max() <= 1e-12 * np.abs(e_in).max()
