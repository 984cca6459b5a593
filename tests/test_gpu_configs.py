"""Parity at the full sizes of the five workload configurations, in the launch
configuration the benchmark times (plans over whole stacks; the dense path for
the prefill shapes).  Where the oracle cannot afford every output, whole layers
and individual rows are sampled."""
import numpy as np
import pytest

import oracle
from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth
from gpu_util import BAR, DECODE_TOL, Layer, rel_err, to_device

pytestmark = pytest.mark.gpu
PREFILL_TOL = 7e-4


def build_stack(cfg, n_layers=None, batch=1):
    import torch
    c = synth.CONFIGS[cfg]
    layers, xs_np, xs, ys = [], [], [], []
    for layer, li, shp in synth.iter_config_layers(cfg, n_layers):
        data = synth.gen_layer(cfg, layer, li, shp)
        layers.append(Layer(shp.d_out, shp.d_in, shp.r, c.x_dtype, data=data))
        x = synth.gen_layer_x(cfg, layer, li, shp, batch, c.x_dtype)
        xs_np.append(x)
        xs.append(to_device(x, c.x_dtype))
        ys.append(torch.full((batch, shp.d_out), float("nan"), dtype=torch.float32, device="cuda"))
    return layers, xs_np, xs, ys


@pytest.mark.parametrize("batch", [1, 8])
def test_config2_pool_as_the_benchmark_runs_it(batch):
    """Config 2's layer as a pool of distinct instances under one plan -- the benchmark's headline
    launch configuration (at batch 8, 320 instances are enough row blocks for the schedules of
    chip-filling launches, the shared-input kernel among them).  Every output of every instance is
    checked against the factored oracle."""
    import torch
    shp = synth.CONFIGS[2].block[0]
    n = 320
    layers, xs_np, xs, ys = [], [], [], []
    for i in range(n):
        layers.append(Layer(shp.d_out, shp.d_in, shp.r, "bf16", data=synth.gen_layer(2, i, 0, shp)))
        x = synth.gen_layer_x(2, i, 0, shp, batch, "bf16")
        xs_np.append(x)
        xs.append(to_device(x, "bf16"))
        ys.append(torch.full((batch, shp.d_out), float("nan"), dtype=torch.float32, device="cuda"))
    plan = nq.nq_plan_create([L.h for L in layers], xs, ys, batch)
    nq.nq_plan_forward(plan)
    nq.nq_plan_forward(plan)
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(y).all()) for y in ys)
    worst = 0.0
    for i in range(n):
        worst = max(worst, rel_err(ys[i].cpu().numpy(), layers[i].oracle(xs_np[i])))
    print(f"config 2 pool, batch {batch}: worst rel err over all {n} instances {worst:.3e}")
    assert worst <= DECODE_TOL and worst <= BAR
    nq.nq_plan_destroy(plan)
    for L in layers:
        L.close()


def test_config3_llama2_7b_stack_every_output():
    import torch
    layers, xs_np, xs, ys = build_stack(3)
    assert len(layers) == 224
    plan = nq.nq_plan_create([L.h for L in layers], xs, ys, 1)
    nq.nq_plan_forward(plan)
    torch.cuda.synchronize()
    worst = 0.0
    for L, x, y in zip(layers, xs_np, ys):
        worst = max(worst, rel_err(y.cpu().numpy(), L.oracle(x)))
    print(f"config 3: worst rel err over 224 layers {worst:.3e}")
    assert worst <= DECODE_TOL and worst <= BAR
    # the same stack through the cached-plan entry point gives identical bits
    y_first = [y.clone() for y in ys]
    nq.nq_binlr_forward_many([L.h for L in layers], xs, ys, 1)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(y_first, ys))
    nq.nq_plan_destroy(plan)
    for L in layers:
        L.close()


def test_config4_llama2_70b_stack_every_output():
    """All 560 layers of the 70B-shaped stack under one plan: every output of every layer against the
    factored oracle (the layers sit at different offsets of ten 512 MiB slabs, which is what varies
    between them), and sampled rows of every eighth decoder layer against the dense definition."""
    import torch
    layers, xs_np, xs, ys = build_stack(4)
    assert len(layers) == 560
    total_bytes = sum(nq.nq_binlr_weight_bytes(L.h) for L in layers)
    assert abs(total_bytes / 1e9 - 4.747) < 0.01            # packed bits + fp16 scales of the whole stack
    plan = nq.nq_plan_create([L.h for L in layers], xs, ys, 1)
    nq.nq_plan_forward(plan)
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    worst_full, worst_rows, at = 0.0, 0.0, -1
    for i, (L, x, y) in enumerate(zip(layers, xs_np, ys)):
        layer = i // 7
        yh = y.cpu().numpy()
        e = rel_err(yh, L.oracle(x))
        if e > worst_full:
            worst_full, at = e, i
        if layer % 8 == 3:                                   # sampled rows against the dense definition
            rows = np.unique(np.concatenate([[0, 127, 128, L.d_out - 1], rng.integers(0, L.d_out, 2)]))
            ref = L.oracle_rows(x, rows)
            scale = np.abs(yh).max()
            worst_rows = max(worst_rows, float(np.abs(yh[:, rows] - ref).max() / scale))
        if i % 70 == 69:
            print(f"config 4: {i + 1} of 560 layers checked, worst so far {worst_full:.3e}", flush=True)
    print(f"config 4: worst rel err over all 560 layers {worst_full:.3e} (op {at}), sampled dense rows {worst_rows:.3e}")
    assert worst_full <= DECODE_TOL and worst_rows <= DECODE_TOL
    nq.nq_plan_destroy(plan)
    for L in layers:
        L.close()


@pytest.mark.parametrize("batch", [512, 2048])
def test_config5_prefill_70b_mlp(batch):
    """The dense path at the prefill sizes: every token at 512; at 2048 one token of every 64-token tile
    (the unit of the workgroup remap and of the eight-wave split) plus 256 random ones -- every output
    of those tokens against the factored oracle, a few rows against the dense definition."""
    import torch
    c = synth.CONFIGS[5]
    rng = np.random.default_rng(5)
    for li, shp in enumerate(c.block):
        data = synth.gen_layer(5, 0, li, shp)
        L = Layer(shp.d_out, shp.d_in, shp.r, c.x_dtype, data=data)
        x = synth.gen_layer_x(5, 0, li, shp, batch, c.x_dtype, c.outlier_frac)
        y = L.forward(x)
        assert np.isfinite(y).all()
        if batch <= 512:
            toks = np.arange(batch)
        else:
            per_tile = np.arange(0, batch, 64) + rng.integers(0, 64, batch // 64)
            toks = np.unique(np.concatenate([[0, 63, 64, batch - 1], per_tile, rng.integers(0, batch, 256)]))
            assert len(set(toks // 64)) == batch // 64
        worst_abs, ref_max, per_token = 0.0, 0.0, 0.0
        for t0 in range(0, len(toks), 64):                   # in pieces, so that the run shows progress
            sel = toks[t0:t0 + 64]
            ref = L.oracle(x[sel])                           # every output of these tokens
            d = np.abs(y[sel] - ref)
            worst_abs, ref_max = max(worst_abs, float(d.max())), max(ref_max, float(np.abs(ref).max()))
            per_token = max(per_token, float((d.max(axis=1) / np.abs(ref).max(axis=1)).max()))
            print(f"config 5 {shp.name} B={batch}: {min(t0 + 64, len(toks))} of {len(toks)} tokens", flush=True)
        err = worst_abs / ref_max                            # the bar's measure: over the whole output of the call
        rows = np.array([0, 127, 128, shp.d_out - 1])
        ra = L.oracle_rows(x[toks[:2]], rows)                # dense definition on a few rows
        err_a = float(np.abs(y[toks[:2]][:, rows] - ra).max() / ref_max)
        print(f"config 5 {shp.name} B={batch}: rel err over {len(toks)} tokens {err:.3e} (worst token relative to "
              f"its own largest output {per_token:.3e}; dense rows {err_a:.3e})")
        assert err <= PREFILL_TOL and err <= BAR and err_a <= PREFILL_TOL and per_token <= BAR
        L.close()


def test_attainable_rate_probes_give_plausible_figures():
    """The measurement aids: a streaming read must land between a third of and the whole nominal HBM
    rate, the matrix-instruction loops between a third of and (with clock tolerance) the nominal peaks."""
    from paper_2602_06694_amd import binding as nq
    gbps = nq.nq_probe_hbm_read(2 << 30, 4, 20)
    assert 2500 < gbps < 8200, gbps
    f16 = nq.nq_probe_mfma(nq.NQ_F16)
    i8 = nq.nq_probe_mfma(nq.NQ_I8)
    assert 800 < f16 < 2800, f16
    assert 1600 < i8 < 5600, i8
    with pytest.raises(nq.NQError):
        nq.nq_probe_mfma(nq.NQ_BF16)
    with pytest.raises(nq.NQError):
        nq.nq_probe_hbm_read(1 << 20, 1, 0)
