"""Seeded random shapes, batches and storage types through the forward entry points against the fp64 oracle: single
calls on both paths (streaming up to batch 8, dense above), plans with random tuning options against single calls bit
for bit, and chains of decoder-shaped blocks through the executor.  The fixed-shape tests cover the cases that were
thought of; this one covers ragged combinations nobody listed."""
import numpy as np
import pytest

from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth
from gpu_util import DECODE_TOL, Layer, check_rounded, new_output, to_device
from test_gpu_exec import Chain

pytestmark = pytest.mark.gpu

DENSE_TOL = 7e-4
OPTS = ["schedule_full", "no_selfq", "no_fuse", "no_resident", "no_selfq_c2", "no_quant_wave"]


def close_enough(y, L, x_np, tol):
    """max |y - y_ref| <= tol * scale, scale = the largest |y_ref|, or, where a short output vector happens to cancel,
    what an output of this layer typically is (largest s_out times the norm of t)."""
    ref, t = L.oracle(x_np, return_t=True)
    assert np.isfinite(y).all()
    typical = float(np.abs(L.data.s_out.astype(np.float64)).max()) * float(np.linalg.norm(t, axis=-1).max())
    scale = max(float(np.abs(ref).max()), 0.25 * typical)
    err = float(np.abs(y.astype(np.float64) - ref).max())
    assert err <= tol * scale, (err / scale, tol)
    return ref


def random_shape(g):
    kind = g.integers(0, 4)
    if kind == 0:
        return tuple(int(g.integers(1, 300)) for _ in range(3))
    if kind == 1:
        return int(g.integers(1, 3000)), int(g.integers(1, 3000)), int(g.integers(1, 2100))
    if kind == 2:       # around the tile and block sizes
        return (max(1, int(g.choice([64, 128, 256, 512, 1024])) + int(g.integers(-2, 3))),
                max(1, int(g.choice([64, 128, 1024, 4096])) + int(g.integers(-2, 3))),
                max(1, int(g.choice([32, 64, 128, 1024])) + int(g.integers(-2, 3))))
    return int(g.integers(1, 600)), int(g.integers(3000, 12000)), int(g.integers(1, 600))


def test_single_calls_on_random_shapes():
    g = np.random.default_rng(20260628)
    for c in range(400):
        d_out, d_in, r = random_shape(g)
        batch = int(g.choice([1, 1, 2, 3, 4, 5, 6, 7, 8, 9, 17, 64, 65, 130]))
        x_dtype = str(g.choice(["bf16", "f16", "f32"]))
        y_dtype = str(g.choice(["f32", "f32", "bf16", "f16"]))
        print(f"case {c}: {d_out}x{d_in} r={r} B={batch} x={x_dtype} y={y_dtype}", flush=True)
        L = Layer(d_out, d_in, r, x_dtype, seed=7000 + c, y_dtype=y_dtype)
        x = synth.gen_x(batch, d_in, 9000 + c, x_dtype)
        y = L.forward(x)
        tol = DECODE_TOL if batch <= 8 else DENSE_TOL
        if y_dtype == "f32":
            close_enough(y, L, x, tol)
        else:
            check_rounded(y, L.oracle(x), y_dtype, 4 * tol)
        L.close()


def test_plans_with_random_options_give_the_bits_of_single_calls(nqopt):
    import torch
    g = np.random.default_rng(20260629)
    for c in range(120):
        n = int(g.integers(1, 10))
        batch = int(g.integers(1, 9))
        x_dtype = str(g.choice(["bf16", "f32", "f16"]))
        shapes = []
        for _ in range(n):
            k = g.integers(0, 3)
            if k == 0:
                shapes.append((int(g.integers(1, 400)), int(g.integers(1, 400)), int(g.integers(1, 300))))
            elif k == 1:
                shapes.append((int(g.integers(1, 2000)), int(g.integers(1, 5000)), int(g.integers(1, 2100))))
            else:
                shapes.append((int(g.choice([128, 1024, 4096])), int(g.choice([1024, 4096])), int(g.choice([64, 1024, 1664]))))
        opts = [o for o in OPTS if g.random() < 0.25]
        print(f"case {c}: B={batch} x={x_dtype} options={opts} shapes={shapes}", flush=True)
        layers = [Layer(*s, x_dtype, seed=100 * c + i) for i, s in enumerate(shapes)]
        xs_np = [synth.gen_x(batch, s[1], 100 * c + 50 + i, x_dtype) for i, s in enumerate(shapes)]
        singles = [L.forward(x) for L, x in zip(layers, xs_np)]
        for o in opts:
            nqopt.set(o, 1)
        ys = [new_output(batch, s[0]) for s in shapes]
        plan = nq.nq_plan_create([L.h for L in layers], [to_device(x, x_dtype) for x in xs_np], ys, batch)
        nq.nq_plan_forward(plan)
        nq.nq_plan_forward(plan)
        torch.cuda.synchronize()
        sched = nq.nq_plan_schedules(plan)
        nq.nq_plan_destroy(plan)
        for o in opts:
            nqopt.unset(o)
        for i, L in enumerate(layers):
            assert np.array_equal(ys[i].cpu().numpy(), singles[i]), (shapes[i], sched)
            close_enough(singles[i], L, xs_np[i], DECODE_TOL)
        for L in layers:
            L.close()


def test_executor_on_random_blocks():
    import torch
    g = np.random.default_rng(20260630)
    for c in range(40):
        h, kv, f = int(g.integers(8, 700)), int(g.integers(1, 300)), int(g.integers(8, 1500))
        rr = lambda: int(g.integers(1, 400))
        shapes = [(h, h, rr()), (kv, h, rr()), (kv, h, rr()), (h, h, rr()), (f, h, rr()), (f, h, rr()), (h, f, rr())]
        n_blocks = int(g.integers(1, 3))
        y_dtype = str(g.choice(["f32", "bf16"]))
        print(f"case {c}: blocks={n_blocks} y={y_dtype} shapes={shapes}", flush=True)

        def data(b, li):
            # scales that keep the chain's magnitudes near one (only the data changes)
            d_out, d_in, r = shapes[li]
            s = 1000 * c + 17 * (7 * b + li)
            so = (synth.gen_scales(d_out, s + 3).astype(np.float32) / np.float32(np.sqrt(r))).astype(np.float16)
            si = (synth.gen_scales(d_in, s + 4).astype(np.float32) / np.float32(np.sqrt(d_in))).astype(np.float16)
            return synth.LayerData(synth.LinearShape("t", d_out, d_in, r), synth.gen_sign_words(d_out, r, s + 1),
                                   synth.gen_sign_words(d_in, r, s + 2), so, si)

        ch = Chain(shapes, n_blocks, seed=c, y_dtype=y_dtype, data=data)
        ref = ch.run_as_single_calls()
        e = nq.nq_exec_create([L.h for L in ch.layers], ch.xs, ch.ys, ch.level)
        nq.nq_exec_forward(e)
        nq.nq_exec_status(e)
        for i, (a, b) in enumerate(zip(ref, ch.ys)):
            assert torch.equal(a, b), ("executor differs from single calls", i)
        ch.check_against_oracle(tol=4 * DECODE_TOL)
        nq.nq_exec_destroy(e)
        ch.close()
