"""GPU parity of the dense (batch >= 9) path against the fp64 oracle."""
import numpy as np
import pytest

from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth
from gpu_util import BAR, Layer, rel_err, to_device

pytestmark = pytest.mark.gpu

# x' and t pass through fp16 (11-bit significands, per-token power-of-two guards): a few 1e-4
PREFILL_TOL = 7e-4


@pytest.mark.parametrize("shape", [(300, 200, 100), (129, 65, 33), (1024, 1024, 256), (640, 1500, 257), (1, 1, 1),
                                   (2048, 512, 384)])
@pytest.mark.parametrize("x_dtype", ["bf16", "f32"])
def test_prefill_small_shapes(shape, x_dtype):
    d_out, d_in, r = shape
    L = Layer(d_out, d_in, r, x_dtype, seed=3 * d_out + d_in)
    for batch in (9, 40, 64, 130, 256):
        x = synth.gen_x(batch, d_in, 900 + batch, x_dtype, outlier_frac=0.01 if d_in >= 200 else 0.0)
        y = L.forward(x)
        ref = L.oracle(x)
        err = rel_err(y, ref)
        assert err <= PREFILL_TOL and err <= BAR, (shape, x_dtype, batch, err)
    L.close()


@pytest.mark.parametrize("tg,splits,ks", [("2", None, None), ("2", "3", None), ("2", "16", None), (None, "5", None),
                                          (None, "1", "2"), (None, "2", "2")])
def test_prefill_32_token_tiles_and_forced_splits(nqopt, tg, splits, ks):
    # the tiling of the two GEMMs is chosen by a cost model; force the variants it rarely picks on
    # small inputs: 32-token workgroup tiles, with and without a split reduction, 64-token tiles
    # with one, more splits than the reduction has groups of four steps (empty splits), and
    # eight-wave workgroups that halve their part of the reduction through LDS (taken where the
    # reduction is a whole number of groups of eight steps: the second and third shape)
    if ks:
        nqopt.set("pf_ks1", ks)
        nqopt.set("pf_ks2", ks)
    if tg:
        nqopt.set("pf_tg1", tg)
        nqopt.set("pf_tg2", tg)
    if splits:
        nqopt.set("pf_splits1", splits)
        nqopt.set("pf_splits2", splits)
    for shape in [(300, 200, 100), (640, 1500, 257), (1024, 2048, 1024)]:
        L = Layer(*shape, "bf16", seed=61)
        for batch in (9, 64, 100, 200):
            x = synth.gen_x(batch, shape[1], 600 + batch, "bf16", outlier_frac=0.01)
            err = rel_err(L.forward(x), L.oracle(x))
            assert err <= PREFILL_TOL, (shape, batch, err)
        L.close()


def test_prefill_matches_streaming_path():
    d_out, d_in, r = 512, 768, 192
    x = synth.gen_x(96, d_in, 5, "bf16")
    La = Layer(d_out, d_in, r, "bf16", seed=77)
    Lb = Layer(d_out, d_in, r, "bf16", seed=77, flags=nq.NQ_FLAG_NO_PREFILL)
    ya, yb = La.forward(x), Lb.forward(x)
    ref = La.oracle(x)
    assert rel_err(ya, ref) <= PREFILL_TOL
    assert rel_err(yb, ref) <= 1e-5
    La.close()
    Lb.close()


def test_prefill_tokens_of_very_different_magnitude_and_nan():
    d_out, d_in, r = 384, 512, 128
    L = Layer(d_out, d_in, r, "f32", seed=12)
    x = synth.gen_x(128, d_in, 6, "f32")
    x *= (10.0 ** np.random.default_rng(1).integers(-6, 6, 128)).astype(np.float32)[:, None]
    y, ref = L.forward(x), L.oracle(x)
    for b in range(128):
        assert np.abs(y[b] - ref[b]).max() <= PREFILL_TOL * np.abs(ref[b]).max(), b
    x[5, 7] = np.nan
    x[9] = 0.0
    import torch
    from gpu_util import to_device
    xd = to_device(x, "f32")
    yd = torch.zeros((128, d_out), dtype=torch.float32, device="cuda")
    nq.nq_binlr_forward(L.h, xd, yd, 128)
    torch.cuda.synchronize()
    y = yd.cpu().numpy()
    assert np.isnan(y[5]).all()
    assert (y[9] == 0).all()
    keep = [b for b in range(128) if b not in (5, 9)]
    for b in keep:
        assert np.abs(y[b] - ref[b]).max() <= PREFILL_TOL * np.abs(ref[b]).max(), b
    L.close()


def test_prefill_reserve_and_batch_changes():
    d_out, d_in, r = 700, 300, 130
    L = Layer(d_out, d_in, r, "bf16", seed=21)
    nq.nq_binlr_reserve(L.h, 512)
    for batch in (512, 64, 300, 17, 64, 8, 512):
        x = synth.gen_x(batch, d_in, 30 + batch, "bf16")
        tol = PREFILL_TOL if batch >= nq.NQ_PREFILL_MIN_BATCH else 1e-5
        assert rel_err(L.forward(x), L.oracle(x)) <= tol, batch
    L.close()


def test_prefill_activations_with_a_large_mean_and_uniform_sign_columns():
    """The dense kernels accumulate P = the sum of the activations under the +1 weights and form
    the signed sum as 2P - S (S = the plain sum).  That cancels most where the activations share
    a large offset (S far above the signed sums), and it must be exact-ish where a column of V is
    all +1 (P = S) or all -1 (P = 0): long reduction, all-positive inputs, constant inputs, and a V
    whose first columns are uniform.  Same bar as every other dense case."""
    d_out, d_in, r = 640, 8192, 384
    rng = np.random.default_rng(77)
    U = synth.gen_sign_words(d_out, r, 771)
    V = synth.gen_sign_words(d_in, r, 772)
    V[:, 0] |= np.uint32(0x0000FFFF)          # rank columns 0..15 all +1
    V[:, 0] &= np.uint32(0x0000FFFF)          # rank columns 16..31 all -1
    s_out = synth.gen_scales(d_out, 773)
    s_in = np.full(d_in, 1.0, dtype=np.float16)           # keep the offset of x intact in x'
    data = synth.LayerData(synth.LinearShape("m", d_out, d_in, r), U, V, s_out, s_in)
    L = Layer(d_out, d_in, r, "f32", data=data)
    batch = 80
    x = (np.abs(rng.standard_normal((batch, d_in))) + 3.0).astype(np.float32)
    x[1] = 2.5                                  # a constant token
    x[2] = -x[2]                                # an all-negative one
    x[3, ::2] = 0.0                             # half of the inputs zero
    err = rel_err(L.forward(x), L.oracle(x))
    assert err <= PREFILL_TOL, err
    for b in range(4):
        y, ref = L.forward(x)[b], L.oracle(x)[b]
        assert np.abs(y - ref).max() <= PREFILL_TOL * np.abs(ref).max(), b
    L.close()


def test_prefill_eight_wave_workgroups_by_default(nqopt):
    """A first GEMM with a long reduction whose 64-token tiles number no more than the CUs, but too many
    for 32-token tiles to take over (here 7 x 20 tiles of 64 steps) runs eight-wave workgroups that halve the reduction through LDS; NQ_PF_KS1=1
    switches that off.  Both against the oracle on sampled tokens (first, last, tile edges, random),
    and against each other within the dense tolerance."""
    d_out, d_in, r, batch = 256, 4096, 3584, 1280
    L = Layer(d_out, d_in, r, "bf16", seed=4100)
    x = synth.gen_x(batch, d_in, 4101, "bf16", outlier_frac=0.01)
    rng = np.random.default_rng(4102)
    idx = np.unique(np.concatenate([[0, 63, 64, 127, 1215, 1216, batch - 1], rng.integers(0, batch, 40)]))
    ref = L.oracle(x[idx])
    outs = {}
    for ks in (None, "1"):
        if ks:
            nqopt.set("pf_ks1", ks)
        else:
            nqopt.unset("pf_ks1")
        y = L.forward(x)
        outs[ks] = y
        for k, b in enumerate(idx):
            assert np.abs(y[b] - ref[k]).max() <= PREFILL_TOL * np.abs(ref[k]).max(), (ks, int(b))
    assert not np.array_equal(outs[None], outs["1"])       # different summation orders: the two paths did run
    assert rel_err(outs[None], outs["1"]) <= PREFILL_TOL
    L.close()


def test_reserve_covers_every_batch_up_to_the_reserved_one():
    """The dense path's workspace need is not monotone in the batch (small batches split the reduction
    and keep partial sums).  After nq_binlr_reserve(h, 2048) a forward at ANY batch <= 2048 must leave
    the workspace as it is (no reallocation, hence no synchronisation on the stream)."""
    import torch
    for shape in [(2048, 7168, 880), (7168, 2048, 880)]:     # the 70B MLP shapes at a quarter of their size
        L = Layer(*shape, "bf16", seed=5200)
        nq.nq_binlr_reserve(L.h, 2048)
        b0, bytes0 = nq.nq_binlr_reserved(L.h)
        assert b0 == 2048 and bytes0 > 0
        x = torch.zeros((2048, shape[1]), dtype=torch.bfloat16, device="cuda")
        y = torch.empty((2048, shape[0]), dtype=torch.float32, device="cuda")
        for batch in (9, 64, 65, 449, 833, 1473, 1793, 2048):
            nq.nq_binlr_forward(L.h, x, y, batch)
            assert nq.nq_binlr_reserved(L.h) == (b0, bytes0), batch
        torch.cuda.synchronize()
        L.close()


def test_exact_path_above_batch_8_on_request():
    """nq_binlr_forward_exact: any batch through the streaming kernels (their accuracy), bit-identical to
    passes of 8 through nq_binlr_forward."""
    import torch
    d_out, d_in, r, batch = 384, 1000, 200, 21
    L = Layer(d_out, d_in, r, "bf16", seed=5300)
    x_np = synth.gen_x(batch, d_in, 5301, "bf16")
    x = to_device(x_np, "bf16")
    y = torch.full((batch, d_out), float("nan"), dtype=torch.float32, device="cuda")
    nq.nq_binlr_forward_exact(L.h, x, y, batch)
    parts = torch.full((batch, d_out), float("nan"), dtype=torch.float32, device="cuda")
    for b0 in range(0, batch, 8):
        nb = min(8, batch - b0)
        nq.nq_binlr_forward(L.h, x[b0:b0 + nb], parts[b0:b0 + nb], nb)
    torch.cuda.synchronize()
    assert torch.equal(y, parts)
    assert rel_err(y.cpu().numpy(), L.oracle(x_np)) <= 1e-5
    L.close()
