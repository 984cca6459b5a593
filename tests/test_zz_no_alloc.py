"""The entry point that allocates nothing (nq_binlr_forward_static): through the C ABI, against
nq_binlr_forward on the same inputs, bit for bit, on two calls in a row, the second one smaller."""
import numpy as np
import pytest

from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth
from gpu_util import DECODE_TOL, Layer, new_output, rel_err, to_device

pytestmark = pytest.mark.gpu


def both(L, x_np, batch):
    import torch
    x = to_device(x_np, L.x_dtype)
    y_ref = new_output(batch, L.d_out)
    y = new_output(batch, L.d_out)
    nq.nq_binlr_forward(L.h, x, y_ref, batch)
    nq.nq_binlr_forward_static(L.h, x, y, batch)
    torch.cuda.synchronize()
    return y.cpu().numpy(), y_ref.cpu().numpy()


def test_static_scratch_forward_matches_forward_twice_in_a_row_second_call_smaller():
    big = Layer(1536, 4096, 1024, "bf16", seed=7100)         # batch 8: quantisation launches + two-column-group kernels
    small = Layer(300, 1000, 200, "bf16", seed=7200)
    calls = [(big, 8), (small, 3), (big, 1), (small, 1), (big, 5), (small, 8)]
    for i, (L, batch) in enumerate(calls):
        x_np = synth.gen_x(batch, L.d_in, 7300 + i, "bf16")
        y, y_ref = both(L, x_np, batch)
        assert np.array_equal(y, y_ref), (i, batch)
        assert rel_err(y, L.oracle(x_np)) <= DECODE_TOL, (i, batch)
    big.close()
    small.close()


def test_static_scratch_forward_rejects_what_does_not_fit():
    import torch
    # batch 8 needs 8 * 192 * (1024 + 256) bytes of fixed point and 8 * 16384 * 4 of t: 2.5 MB; batch 1 0.3 MB
    L = Layer(128, 65536, 16384, "bf16", seed=7400)
    x = torch.zeros((8, 65536), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((8, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(nq.NQError) as e:
        nq.nq_binlr_forward_static(L.h, x, y, 8)
    assert e.value.status == nq.NQ_E_SHAPE and "static array holds" in str(e.value)
    nq.nq_binlr_forward_static(L.h, x, y, 1)                  # one token of the same layer fits
    torch.cuda.synchronize()
    small = Layer(64, 64, 32, "bf16", seed=7500)
    xs = torch.zeros((9, 64), dtype=torch.bfloat16, device="cuda")
    ys = torch.zeros((9, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(nq.NQError) as e:
        nq.nq_binlr_forward_static(small.h, xs, ys, 9)
    assert e.value.status == nq.NQ_E_UNSUPPORTED
    L.close()
    small.close()
