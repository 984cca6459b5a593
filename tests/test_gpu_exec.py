"""GPU parity of the dependent-layer executor (one persistent launch for a chain of layers): bit-identical
to the same chain run as single-layer calls, and every level against the fp64 oracle fed with the
GPU's own output of the level before."""
import numpy as np
import pytest

import oracle
from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth
from gpu_util import DECODE_TOL, Layer, rel_err, to_device

pytestmark = pytest.mark.gpu

LEVELS = (0, 0, 0, 1, 2, 2, 3)          # q, k, v | o | gate, up | down
SRC = (-1, -1, -1, 0, 3, 3, 4)          # o reads q's output, gate and up read o's, down reads gate's


class Chain:
    """n_blocks decoder blocks of the given seven shapes; block b + 1 reads block b's down output."""

    def __init__(self, shapes, n_blocks=1, seed=0, y_dtype="f32", first_x="bf16", data=None):
        import torch
        self.layers, self.level, self.src = [], [], []
        for b in range(n_blocks):
            for li, (d_out, d_in, r) in enumerate(shapes):
                src = 7 * b + SRC[li] if SRC[li] >= 0 else (7 * b - 1 if b else -1)
                x_dtype = first_x if src < 0 else y_dtype
                d = data(b, li) if data else None
                self.layers.append(Layer(d_out, d_in, r, x_dtype, seed=seed + 17 * (7 * b + li), y_dtype=y_dtype, data=d))
                self.level.append(4 * b + LEVELS[li])
                self.src.append(src)
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[y_dtype]
        self.first_x = first_x
        self.x0_np = synth.gen_x(1, shapes[0][1], seed + 999, first_x)
        self.x0 = to_device(self.x0_np, first_x)
        self.ys = [torch.full((1, L.d_out), float("nan"), dtype=tdt, device="cuda") for L in self.layers]
        self.xs = [self.x0 if s < 0 else self.ys[s] for s in self.src]

    def set_input(self, seed):
        import torch
        self.x0_np = synth.gen_x(1, self.layers[0].d_in, seed, self.first_x)
        self.x0.copy_(to_device(self.x0_np, self.first_x))

    def executor(self):
        return nq.nq_exec_create([L.h for L in self.layers], self.xs, self.ys, self.level)

    def run_as_single_calls(self):
        """The same chain, layer by layer on the stream; returns copies of the outputs."""
        import torch
        for L, x, y in zip(self.layers, self.xs, self.ys):
            nq.nq_binlr_forward(L.h, x, y, 1)
        torch.cuda.synchronize()
        out = [y.clone() for y in self.ys]
        for y in self.ys:
            y.fill_(float("nan"))
        return out

    def check_against_oracle(self, tol=DECODE_TOL):
        """Every layer against the factored oracle on the input the GPU actually gave it."""
        import torch
        worst = 0.0
        ys = [y.cpu().to(torch.float64).numpy() if y.dtype != torch.float32 else y.cpu().numpy() for y in self.ys]
        for i, L in enumerate(self.layers):
            x = synth.x_as_f64(self.x0_np, self.first_x) if self.src[i] < 0 else ys[self.src[i]].astype(np.float64)
            d = L.data
            ref = oracle.forward_factored(d.U_words, d.V_words, d.s_out, d.s_in, L.d_out, L.d_in, L.r, x)
            if L.y_dtype == "f32":
                worst = max(worst, rel_err(ys[i], ref))
            else:
                ulp = {"bf16": 2.0 ** -8, "f16": 2.0 ** -10}[L.y_dtype]
                assert np.isfinite(ys[i]).all()
                assert (np.abs(ys[i] - ref) <= tol * np.abs(ref).max() + ulp * np.abs(ref)).all(), i
        return worst

    def close(self):
        for L in self.layers:
            L.close()


SMALL = [(512, 384, 160), (192, 384, 96), (192, 384, 96), (384, 512, 128), (1000, 384, 200), (1000, 384, 200), (384, 1000, 200)]
RAGGED = [(300, 131, 33), (65, 131, 1), (1, 131, 70), (131, 300, 129), (257, 131, 64), (257, 131, 64), (131, 257, 31)]
LONG = [(256, 20000, 64), (128, 20000, 32), (128, 20000, 32), (20000, 256, 64), (17000, 20000, 40), (17000, 20000, 40),
        (256, 17000, 48)]


@pytest.mark.parametrize("shapes,n_blocks", [(SMALL, 1), (SMALL, 3), (RAGGED, 2), (LONG, 1)])
def test_executor_matches_single_calls_bit_for_bit_and_the_oracle(shapes, n_blocks):
    import torch
    c = Chain(shapes, n_blocks, seed=8100)
    ref = c.run_as_single_calls()
    e = c.executor()
    n_wg, n_tasks, lds = nq.nq_exec_info(e)
    assert n_wg >= 1 and n_tasks >= 14 * n_blocks and lds <= 160 * 1024
    for rep in range(3):                                     # later launches take a new epoch; inputs change in between
        if rep:
            c.set_input(8200 + rep)
            ref = c.run_as_single_calls()
        nq.nq_exec_forward(e)
        nq.nq_exec_status(e)
        for i, (a, b) in enumerate(zip(c.ys, ref)):
            assert torch.equal(a, b), (rep, i)
        worst = c.check_against_oracle()
        assert worst <= DECODE_TOL, worst
        for y in c.ys:
            y.fill_(float("nan"))
    print(f"executor, {len(c.layers)} layers: worst rel err per layer {worst:.3e}")
    nq.nq_exec_destroy(e)
    c.close()


@pytest.mark.parametrize("y_dtype", ["bf16", "f16"])
def test_executor_hands_over_sixteen_bit_outputs_as_stored(y_dtype):
    """A 16-bit output is handed to the next layer as the stored (rounded) value, as a reader of y would see it."""
    import torch
    c = Chain(SMALL, 1, seed=8300, y_dtype=y_dtype)
    # (keeps the chain inside the fp16 range: scales divided by 64)
    ref = c.run_as_single_calls()
    e = c.executor()
    nq.nq_exec_forward(e)
    nq.nq_exec_status(e)
    for i, (a, b) in enumerate(zip(c.ys, ref)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), i
    nq.nq_exec_destroy(e)
    c.close()


def test_executor_with_rank_wise_scales():
    import torch
    c = Chain(SMALL, 1, seed=8400)
    rng = np.random.default_rng(8401)
    for L in c.layers[::2]:
        nq.nq_binlr_set_mid_scale(L.h, (rng.standard_normal(L.r) * 0.5 + 1.0).astype(np.float16))
    ref = c.run_as_single_calls()
    e = c.executor()
    nq.nq_exec_forward(e)
    nq.nq_exec_status(e)
    for i, (a, b) in enumerate(zip(c.ys, ref)):
        assert torch.equal(a, b), i
    nq.nq_exec_destroy(e)
    c.close()


@pytest.mark.parametrize("cfg", [3, 4])
def test_full_size_decoder_blocks_in_dependency_order(cfg):
    """Two whole decoder blocks of the 7B / 70B shapes, chained q -> o -> gate -> down -> next q: every
    output of every layer against the oracle on the GPU's own previous output."""
    import torch
    block = synth.CONFIGS[cfg].block
    shapes = [(s.d_out, s.d_in, s.r) for s in block]
    c = Chain(shapes, 2, seed=8500, data=lambda b, li: synth.gen_layer(cfg, b, li, block[li]))
    ref = c.run_as_single_calls()
    e = c.executor()
    nq.nq_exec_forward(e)
    nq.nq_exec_status(e)
    for i, (a, b) in enumerate(zip(c.ys, ref)):
        assert torch.equal(a, b), i
    worst = c.check_against_oracle()
    print(f"config {cfg} blocks in dependency order: worst rel err per layer {worst:.3e}")
    assert worst <= DECODE_TOL
    nq.nq_exec_destroy(e)
    c.close()


def test_executor_replays_from_a_hip_graph():
    """A captured launch replayed several times with new inputs and eager work in between: the epoch lives in
    device memory, so every replay hands over fresh data."""
    import torch
    c = Chain(SMALL, 2, seed=8600)
    e = c.executor()
    nq.nq_exec_forward(e)                                    # warm-up outside the capture
    nq.nq_exec_status(e)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        nq.nq_exec_forward(e)
    for rep in range(4):
        c.set_input(8700 + rep)
        ref = c.run_as_single_calls()                        # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(c.ys, ref)):
            assert torch.equal(a, b), (rep, i)
    nq.nq_exec_status(e)
    del graph
    nq.nq_exec_destroy(e)
    c.close()


def test_a_wait_that_cannot_be_met_in_time_gives_up_and_the_grid_drains(nqopt):
    """With a time limit of zero every wait for another workgroup's output gives up at once: the launch must
    still end (all workgroups leave), nq_exec_status reports it once, and the next launch works again."""
    import torch
    c = Chain(SMALL, 2, seed=8800)
    e = c.executor()
    nqopt.set("exec_spin_limit_us", 0)
    nq.nq_exec_forward(e)
    with pytest.raises(nq.NQError) as err:
        nq.nq_exec_status(e)
    assert err.value.status == nq.NQ_E_TIMEOUT
    nqopt.unset("exec_spin_limit_us")
    ref = c.run_as_single_calls()
    nq.nq_exec_forward(e)
    nq.nq_exec_status(e)
    for i, (a, b) in enumerate(zip(c.ys, ref)):
        assert torch.equal(a, b), i
    nq.nq_exec_destroy(e)
    c.close()


def test_executor_argument_checks():
    import torch
    c = Chain(SMALL, 1, seed=8900)
    hs = [L.h for L in c.layers]
    with pytest.raises(nq.NQError):                          # levels out of order
        nq.nq_exec_create(hs, c.xs, c.ys, [0, 0, 0, 2, 1, 1, 3])
    with pytest.raises(nq.NQError):                          # o reads q's output but sits in q's level
        nq.nq_exec_create(hs, c.xs, c.ys, [0, 0, 0, 0, 1, 1, 2])
    with pytest.raises(nq.NQError):                          # two outputs share a buffer
        nq.nq_exec_create(hs, c.xs, [c.ys[0], c.ys[1], c.ys[1]] + c.ys[3:], list(LEVELS))
    with pytest.raises(nq.NQError):                          # a handle twice
        nq.nq_exec_create([hs[0]] + hs[:6], c.xs, c.ys, list(LEVELS))
    wrong = Layer(384, 512, 128, "bf16", seed=8901)          # reads an fp32 output as bf16
    with pytest.raises(nq.NQError):
        nq.nq_exec_create(hs[:3] + [wrong.h] + hs[4:], c.xs, c.ys, list(LEVELS))
    wrong.close()
    c.close()


@pytest.mark.parametrize("shape", [(1024, 1024, 256), (300, 131, 33), (1, 1, 1), (2048, 200, 64), (128, 16000, 8), (129, 65, 4000)])
def test_small_layer_in_one_launch_matches_the_two_launch_path(shape, nqopt):
    """A lone small layer at batch 1 can run both stages in ONE launch by one workgroup, t staying in LDS (an
    option: off by default): same arithmetic, so bit-identical to the two-launch path, t included; also with a
    rank-wise scale, a 16-bit output and without the output scale."""
    import torch
    d_out, d_in, r = shape
    for y_dtype, mid in (("f32", False), ("bf16", True)):
        L = Layer(d_out, d_in, r, "bf16", seed=9100 + d_out, y_dtype=y_dtype)
        if mid:
            nq.nq_binlr_set_mid_scale(L.h, (np.random.default_rng(9101).standard_normal(r) * 0.5 + 1.0).astype(np.float16))
        x_np = synth.gen_x(1, d_in, 9102, "bf16")
        x = to_device(x_np, "bf16")
        outs = {}
        for small in (True, False):
            nqopt.set("small_layer_kb", 4096 if small else 0)
            tdt = torch.float32 if y_dtype == "f32" else torch.bfloat16
            y = torch.full((1, d_out), float("nan"), dtype=tdt, device="cuda")
            z = torch.full((1, d_out), float("nan"), dtype=tdt, device="cuda")
            nq.nq_binlr_forward(L.h, x, y, 1)
            torch.cuda.synchronize()
            t = nq.nq_binlr_read_intermediate(L.h, r, 1)
            nq.nq_binlr_forward_unscaled(L.h, x, z, 1)
            torch.cuda.synchronize()
            outs[small] = (y.view(torch.int16 if y_dtype != "f32" else torch.int32).cpu().numpy(), t.view(np.int32).copy(),
                           z.view(torch.int16 if y_dtype != "f32" else torch.int32).cpu().numpy())
        for a, b in zip(outs[True], outs[False]):
            assert np.array_equal(a, b), (shape, y_dtype)
        if not mid:
            nqopt.set("small_layer_kb", 4096)
            assert rel_err(L.forward(x_np), L.oracle(x_np)) <= DECODE_TOL
        L.close()


def test_small_layer_path_is_an_option_and_changes_no_result(nqopt):
    """The one-launch path is off by default (it measured slower than two launches that spread the row blocks
    over many CUs); the option that sets its size limit switches it on, and results stay the same either way."""
    import torch
    L = Layer(1024, 1024, 256, "bf16", seed=9200)
    x_np = synth.gen_x(1, 1024, 9201, "bf16")
    ref = L.forward(x_np)                                    # default: two launches
    nqopt.set("small_layer_kb", 1)                           # 66 KiB of bits do not fit 1 KiB: still two launches
    assert np.array_equal(L.forward(x_np), ref)
    nqopt.set("small_layer_kb", 128)                         # now one launch by one workgroup
    assert np.array_equal(L.forward(x_np), ref)
    L.close()
