"""GPU parity of the scale gradients with frozen signs (Section 3.4; Algorithm 1, Phase 3) against the
fp64 oracle, through the C ABI: unscaled forwards of the layer and of its transpose, then the reduction
over the batch."""
import numpy as np
import pytest

import oracle
from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth
from gpu_util import Layer, rel_err, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,batch", [((300, 200, 100), 3), ((129, 65, 33), 1), ((512, 1024, 256), 8), ((640, 257, 130), 21)])
def test_scale_gradients_match_oracle(shape, batch):
    import torch
    d_out, d_in, r = shape
    L = Layer(d_out, d_in, r, "f32", seed=4000 + r)
    d = L.data
    # the transposed layer: factors and scale vectors exchanged
    T = nq.nq_binlr_create(d_in, d_out, r, d.V_words, d.U_words, d.s_in, d.s_out, nq.NQ_F32, nq.NQ_F32, 0)
    x_np = synth.gen_x(batch, d_in, 4100 + batch, "f32")
    g_np = synth.gen_x(batch, d_out, 4200 + batch, "f32")
    x, g = to_device(x_np, "f32"), to_device(g_np, "f32")
    z = torch.full((batch, d_out), float("nan"), dtype=torch.float32, device="cuda")
    w = torch.full((batch, d_in), float("nan"), dtype=torch.float32, device="cuda")
    ds_out = torch.zeros(d_out, dtype=torch.float32, device="cuda")
    ds_in = torch.zeros(d_in, dtype=torch.float32, device="cuda")
    nq.nq_binlr_forward_unscaled(L.h, x, z, batch)
    nq.nq_binlr_forward_unscaled(T, g, w, batch)
    nq.nq_scale_grad(g, nq.NQ_F32, z, nq.NQ_F32, batch, d_out, ds_out)
    nq.nq_scale_grad(x, nq.NQ_F32, w, nq.NQ_F32, batch, d_in, ds_in)
    torch.cuda.synchronize()
    # z itself: the forward with unit output scales
    z_ref = oracle.forward_factored(d.U_words, d.V_words, np.ones(d_out, np.float16), d.s_in, d_out, d_in, r,
                                    x_np.astype(np.float64))
    assert rel_err(z.cpu().numpy(), z_ref) <= 1e-5
    ref_out, ref_in = oracle.scale_grads(d.U_words, d.V_words, d.s_out, d.s_in, d_out, d_in, r,
                                         x_np.astype(np.float64), g_np.astype(np.float64))
    assert np.abs(ds_out.cpu().numpy() - ref_out).max() <= 1e-5 * np.abs(ref_out).max(), (shape, batch)
    assert np.abs(ds_in.cpu().numpy() - ref_in).max() <= 1e-5 * np.abs(ref_in).max(), (shape, batch)
    nq.nq_binlr_destroy(T)
    L.close()


def test_batch_reduction_kernel_types_and_checks():
    import torch
    rng = np.random.default_rng(4300)
    a = rng.standard_normal((5, 1000)).astype(np.float32)
    b = rng.standard_normal((5, 1000)).astype(np.float32)
    out = torch.zeros(1000, dtype=torch.float32, device="cuda")
    for dt_name, dt in (("f32", nq.NQ_F32), ("bf16", nq.NQ_BF16), ("f16", nq.NQ_F16)):
        ad = to_device(a if dt_name == "f32" else synth.gen_x(5, 1000, 4301, dt_name), dt_name)
        a64 = synth.x_as_f64(a if dt_name == "f32" else synth.gen_x(5, 1000, 4301, dt_name), dt_name)
        nq.nq_scale_grad(ad, dt, to_device(b, "f32"), nq.NQ_F32, 5, 1000, out)
        torch.cuda.synchronize()
        ref = (a64 * b.astype(np.float64)).sum(axis=0)
        assert np.abs(out.cpu().numpy() - ref).max() <= 1e-6 * np.abs(ref).max(), dt_name
    with pytest.raises(nq.NQError):
        nq.nq_scale_grad(out, nq.NQ_I8, out, nq.NQ_F32, 1, 1000, out)
    with pytest.raises(nq.NQError):
        nq.nq_scale_grad(out, nq.NQ_F32, out, nq.NQ_F32, 0, 1000, out)
