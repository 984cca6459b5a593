"""GPU parity of the binary64 LB-ADMM path (Section 3.2 Step 2-2 / 2-3) against the numpy oracle, through the C ABI:
the dense product, whole runs of the iteration on shapes that span several 64-wide blocks with ragged tails, the
degenerate settings, the balancing step and the failure path of the factorisation."""
import numpy as np
import pytest

from oracle import lb_admm as O
from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth

pytestmark = pytest.mark.gpu

# binary64 on both sides; the two differ in summation order and in forming H^-1 explicitly.  One iteration maps
# an input perturbation e to about cond(H) * e; cond(H) <= 1 + ||V||^2 / (rho + lambda) is below 1e3 for these inputs,
# and the map is a contraction towards the proxies, so 1e-9 relative to the largest entry leaves three orders of
# margin over 2^-53 * 1e3 * (number of iterations).
TOL = 1e-9


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_gpu(w, u0, v0, n_iters, rho0, rho1, lam, power_iters):
    import torch
    n, m = w.shape
    r = u0.shape[1]
    nbytes = nq.nq_lb_admm_workspace_bytes(n, m, r)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dw, du0, dv0 = dev(w), dev(u0), dev(v0)
    outs = {k: torch.full((n if k.endswith("U") else m, r), float("nan"), dtype=torch.float64, device="cuda")
            for k in ("U", "V", "Z_U", "Z_V", "Lambda_U", "Lambda_V")}
    print(f"lb_admm n={n} m={m} r={r} iters={n_iters} power={power_iters}", flush=True)
    nq.nq_lb_admm(dw, n, m, r, du0, dv0, n_iters, rho0, rho1, lam, power_iters, outs["U"], outs["V"], outs["Z_U"], outs["Z_V"],
                  outs["Lambda_U"], outs["Lambda_V"], ws, nbytes)
    torch.cuda.synchronize()
    return outs, ws, nbytes


def compare(outs, ref, tol=TOL):
    worst = 0.0
    # an output that is zero up to rounding (a dual of an exactly reproduced proxy) is measured against the factors' scale
    floor = 1e-3 * max(np.abs(ref["U"]).max(), np.abs(ref["V"]).max())
    for k, t in outs.items():
        got = t.cpu().numpy()
        e = np.abs(got - ref[k]).max() / max(np.abs(ref[k]).max(), floor)
        worst = max(worst, e)
        assert np.isfinite(got).all(), k
        assert e <= tol, (k, e)
    return worst


@pytest.mark.parametrize("ta,tb,M,N,K", [(0, 0, 131, 70, 37), (1, 0, 64, 64, 64), (0, 1, 257, 129, 65), (1, 1, 70, 200, 19),
                                         (0, 0, 1, 1, 1), (1, 0, 300, 300, 1000), (0, 0, 2048, 1536, 260)])
def test_dgemm_against_numpy(ta, tb, M, N, K):
    import torch
    g = np.random.default_rng(M * 7 + N * 3 + K)
    a = g.standard_normal((K, M) if ta else (M, K))
    b = g.standard_normal((N, K) if tb else (K, N))
    c0 = g.standard_normal((M, N + 3))                       # a leading dimension larger than the row
    ref = 1.5 * ((a.T if ta else a) @ (b.T if tb else b)) - 0.25 * c0[:, :N]
    dc = dev(c0)
    nq.nq_dgemm(ta, tb, M, N, K, 1.5, dev(a), a.shape[1], dev(b), b.shape[1], -0.25, dc, N + 3)
    torch.cuda.synchronize()
    got = dc.cpu().numpy()
    assert np.array_equal(got[:, N:], c0[:, N:])             # nothing beyond the N columns is touched
    assert np.abs(got[:, :N] - ref).max() <= 4e-16 * (K + 4) * max(1.0, np.abs(ref).max())
    # beta = 0 never reads C: NaNs there do not spread
    dn = torch.full((M, N), float("nan"), dtype=torch.float64, device="cuda")
    nq.nq_dgemm(ta, tb, M, N, K, 1.0, dev(a), a.shape[1], dev(b), b.shape[1], 0.0, dn, N)
    torch.cuda.synchronize()
    assert np.abs(dn.cpu().numpy() - (a.T if ta else a) @ (b.T if tb else b)).max() <= 4e-16 * (K + 4) * max(1.0, np.abs(ref).max())


SHAPES = [(96, 80, 24), (130, 70, 65), (200, 150, 130), (300, 260, 200), (70, 310, 64), (513, 257, 321), (20, 30, 70), (1100, 40, 33)]


@pytest.mark.parametrize("n,m,r", SHAPES)
def test_iterations_match_the_oracle(n, m, r):
    w, u0, v0 = synth.gen_admm_problem(n, m, r, seed=n + m + r)
    ref = O.lb_admm(w, u0, v0, 6, 0.02, 0.3, 1e-3, 5)
    outs, _, _ = run_gpu(w, u0, v0, 6, 0.02, 0.3, 1e-3, 5)
    print("worst relative error", compare(outs, ref), flush=True)


@pytest.mark.parametrize("option", ["admm_no_overlap", "admm_inline_svid", "admm_no_prio", "admm_product_mode", "admm_no_fused_step"])
def test_every_schedule_of_the_two_streams_gives_the_oracles_result(option, nqopt):
    """Where the SVID and the product with W run (beside the factorisation or on the caller's stream), with how many
    workgroups per CU, at which wave priority, and whether a diagonal block is factorised in the launch of the trailing
    update before it or in one of its own, changes the order of events on the device, not the result: each
    switch on its own, on a shape large enough for the one-workgroup-per-CU product (64 tiles of 128 x 128 or more)."""
    n, m, r = 1100, 1030, 900
    w, u0, v0 = synth.gen_admm_problem(n, m, r, seed=11)
    ref = O.lb_admm(w, u0, v0, 3, 0.5, 2.0, 1e-3, 4)
    outs, _, _ = run_gpu(w, u0, v0, 3, 0.5, 2.0, 1e-3, 4)
    print("default schedule: worst relative error", compare(outs, ref), flush=True)
    nqopt.set(option, 1)
    outs, _, _ = run_gpu(w, u0, v0, 3, 0.5, 2.0, 1e-3, 4)
    print(option, ": worst relative error", compare(outs, ref), flush=True)


def test_random_shapes_and_settings():
    """Seeded random sizes (around one and several 64-wide blocks, ranks above and below both sides), iteration counts,
    power rounds and penalty schedules against the oracle."""
    g = np.random.default_rng(20260701)
    worst = 0.0
    for c in range(80):
        k = g.integers(0, 3)
        if k == 0:
            n, m, r = (int(g.integers(1, 200)) for _ in range(3))
        elif k == 1:
            n, m, r = int(g.integers(1, 900)), int(g.integers(1, 900)), int(g.integers(1, 600))
        else:
            n = int(g.choice([64, 128, 512, 1024])) + int(g.integers(-1, 2))
            m = int(g.choice([64, 256, 1536, 1600])) + int(g.integers(-1, 2))
            r = int(g.choice([63, 64, 65, 128, 256, 320]))
        iters, power = int(g.integers(0, 6)), int(g.integers(0, 7))
        rho0 = float(g.uniform(0.01, 1.0))
        rho1 = float(g.uniform(rho0, 5.0))
        lam = float(g.choice([0.0, 1e-3, 0.1]))
        w, u0, v0 = synth.gen_admm_problem(n, m, r, seed=5000 + c)
        ref = O.lb_admm(w, u0, v0, iters, rho0, rho1, lam, power)
        outs, _, _ = run_gpu(w, u0, v0, iters, rho0, rho1, lam, power)
        worst = max(worst, compare(outs, ref, 1e-8))
    print("worst relative error over the random cases", worst, flush=True)


def test_many_iterations_small():
    w, u0, v0 = synth.gen_admm_problem(96, 80, 40, seed=5)
    ref = O.lb_admm(w, u0, v0, 60, 0.01, 0.5, 1e-3, 8)
    outs, _, _ = run_gpu(w, u0, v0, 60, 0.01, 0.5, 1e-3, 8)
    print("worst relative error", compare(outs, ref, 1e-8), flush=True)


def test_degenerate_settings():
    w, u0, v0 = synth.gen_admm_problem(70, 50, 20, seed=9)
    # no iterations: the start factors, their SVID and zero duals
    ref = O.lb_admm(w, u0, v0, 0, 0.1, 0.1, 0.0, 4)
    outs, _, _ = run_gpu(w, u0, v0, 0, 0.1, 0.1, 0.0, 4)
    compare(outs, ref)
    assert np.array_equal(outs["U"].cpu().numpy(), u0) and not outs["Lambda_V"].cpu().numpy().any()
    # no power rounds: the proxies' magnitudes are the mean magnitude
    ref = O.lb_admm(w, u0, v0, 3, 0.1, 0.2, 1e-2, 0)
    outs, _, _ = run_gpu(w, u0, v0, 3, 0.1, 0.2, 1e-2, 0)
    compare(outs, ref)
    # one iteration, one power round, rank 1, single row / column
    for shape in ((1, 9, 1), (9, 1, 3), (5, 5, 1)):
        w1, a0, b0 = synth.gen_admm_problem(*shape, seed=11)
        ref = O.lb_admm(w1, a0, b0, 1, 0.5, 0.5, 0.0, 1)
        outs, _, _ = run_gpu(w1, a0, b0, 1, 0.5, 0.5, 0.0, 1)
        compare(outs, ref)


def test_outputs_may_alias_the_start_factors():
    import torch
    n, m, r = 130, 90, 70
    w, u0, v0 = synth.gen_admm_problem(n, m, r, seed=3)
    ref = O.lb_admm(w, u0, v0, 3, 0.05, 0.1, 1e-3, 4)
    nbytes = nq.nq_lb_admm_workspace_bytes(n, m, r)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    U, V = dev(u0), dev(v0)
    rest = {k: torch.empty((n if k.endswith("U") else m, r), dtype=torch.float64, device="cuda") for k in ("Z_U", "Z_V", "Lambda_U", "Lambda_V")}
    nq.nq_lb_admm(dev(w), n, m, r, U, V, 3, 0.05, 0.1, 1e-3, 4, U, V, rest["Z_U"], rest["Z_V"], rest["Lambda_U"], rest["Lambda_V"], ws, nbytes)
    compare({"U": U, "V": V, **rest}, ref)


def test_balancing_matches_the_oracle_bit_for_bit_in_the_signs():
    import torch
    n, m, r = 200, 150, 130
    w, u0, v0 = synth.gen_admm_problem(n, m, r, seed=21)
    outs, ws, nbytes = run_gpu(w, u0, v0, 5, 0.02, 0.3, 1e-3, 5)
    state = {k: t.cpu().numpy() for k, t in outs.items()}           # the balancing of the GPU's own state, by the oracle
    su, sv, s1, s2, eta = O.balance(state)
    nw = (r + 31) // 32
    uw = torch.full((n, nw), -1, dtype=torch.int32, device="cuda")
    vw = torch.full((m, nw), -1, dtype=torch.int32, device="cuda")
    d1 = torch.empty(n, dtype=torch.float64, device="cuda")
    d2 = torch.empty(m, dtype=torch.float64, device="cuda")
    de = torch.empty(1, dtype=torch.float64, device="cuda")
    nq.nq_lb_admm_balance(outs["U"], outs["Lambda_U"], n, outs["V"], outs["Lambda_V"], m, r, uw, vw, d1, d2, de, ws, nbytes)
    torch.cuda.synchronize()

    def packed(signs):
        bits = np.zeros((signs.shape[0], nw * 32), dtype=np.uint8)
        bits[:, :r] = signs > 0
        return np.packbits(bits, axis=1, bitorder="little").view("<u4")
    assert np.array_equal(uw.cpu().numpy().view(np.uint32), packed(su))
    assert np.array_equal(vw.cpu().numpy().view(np.uint32), packed(sv))
    assert abs(de.item() - eta) <= 1e-13 * eta
    assert np.abs(d1.cpu().numpy() - s1).max() <= 1e-13 * s1.max()
    assert np.abs(d2.cpu().numpy() - s2).max() <= 1e-13 * s2.max()
    # and the packed words are the library's own canonical format
    assert np.array_equal(nq.nq_pack_signs(su.astype(np.int8)).reshape(-1), uw.cpu().numpy().view(np.uint32).reshape(-1))


def test_factorised_matrix_runs_as_a_layer():
    """From a target matrix to a resident layer without leaving the GPU: LB-ADMM, balancing, the packed signs and the
    scales (rounded to fp16 by the caller) into nq_binlr_create_from_device, one forward; checked against the oracle's
    reconstruction W^ = Diag(s1) sign(P_U) sign(P_V)^T Diag(s2) applied to x, and W^ against the target."""
    import torch
    n, m, r = 256, 192, 96
    w, u0, v0 = synth.gen_admm_problem(n, m, r, seed=33)
    outs, ws, nbytes = run_gpu(w, u0, v0, 30, 0.02, 0.3, 1e-3, 6)
    nw = (r + 31) // 32
    uw = torch.empty((n, nw), dtype=torch.int32, device="cuda")
    vw = torch.empty((m, nw), dtype=torch.int32, device="cuda")
    s1 = torch.empty(n, dtype=torch.float64, device="cuda")
    s2 = torch.empty(m, dtype=torch.float64, device="cuda")
    eta = torch.empty(1, dtype=torch.float64, device="cuda")
    nq.nq_lb_admm_balance(outs["U"], outs["Lambda_U"], n, outs["V"], outs["Lambda_V"], m, r, uw, vw, s1, s2, eta, ws, nbytes)
    s1h, s2h = s1.to(torch.float16).contiguous(), s2.to(torch.float16).contiguous()
    h = nq.nq_binlr_create_from_device(n, m, r, uw, vw, s1h, s2h, nq.NQ_F32, nq.NQ_F32, 0)
    x_np = synth.gen_x(3, m, 3301, "f32")
    y = torch.empty((3, n), dtype=torch.float32, device="cuda")
    nq.nq_binlr_forward(h, dev(x_np), y, 3)
    torch.cuda.synchronize()
    # the oracle's balancing of the oracle's own run, with the scales rounded to fp16 the same way
    ref_state = O.lb_admm(w, u0, v0, 30, 0.02, 0.3, 1e-3, 6)
    su, sv, r1, r2, _ = O.balance(ref_state)
    w_hat = O.reconstruction(su, sv, r1.astype(np.float16).astype(np.float64), r2.astype(np.float16).astype(np.float64))
    y_ref = x_np.astype(np.float64) @ w_hat.T
    assert np.abs(y.cpu().numpy() - y_ref).max() <= 1e-5 * np.abs(y_ref).max()
    # the factorisation is an approximation of the target at about one bit per weight: it must at least beat the
    # sign-only rank-r start by a clear margin
    rel = np.linalg.norm(w - w_hat) / np.linalg.norm(w)
    print("relative reconstruction error of the binary factorisation", rel, flush=True)
    assert rel < 0.9
    nq.nq_binlr_destroy(h)


def test_a_failed_factorisation_is_reported():
    w, u0, v0 = synth.gen_admm_problem(96, 80, 70, seed=2)
    with pytest.raises(nq.NQError) as e:
        run_gpu(w, u0, v0, 1, -50.0, -50.0, 0.0, 2)               # V^T V - 50 I is indefinite
    assert e.value.status == nq.NQ_E_INVALID_ARG and "pivot" in str(e.value)
    # the next call on the same process works
    ref = O.lb_admm(w, u0, v0, 2, 0.1, 0.1, 0.0, 2)
    outs, _, _ = run_gpu(w, u0, v0, 2, 0.1, 0.1, 0.0, 2)
    compare(outs, ref)


def test_argument_checks_on_device():
    import torch
    w, u0, v0 = synth.gen_admm_problem(40, 30, 8, seed=1)
    n, m, r = 40, 30, 8
    nbytes = nq.nq_lb_admm_workspace_bytes(n, m, r)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    t = {k: torch.empty((n if k.endswith("U") else m, r), dtype=torch.float64, device="cuda") for k in ("U", "V", "Z_U", "Z_V", "Lambda_U", "Lambda_V")}
    args = lambda **kw: dict(dict(n_iters=1, rho0=0.1, rho1=0.1, lam=0.0, pw=1, nb=nbytes), **kw)

    def call(n_iters, rho0, rho1, lam, pw, nb):
        nq.nq_lb_admm(dev(w), n, m, r, dev(u0), dev(v0), n_iters, rho0, rho1, lam, pw, t["U"], t["V"], t["Z_U"], t["Z_V"], t["Lambda_U"],
                      t["Lambda_V"], ws, nb)
    for kw, code in ((dict(n_iters=-1), nq.NQ_E_INVALID_ARG), (dict(pw=-1), nq.NQ_E_INVALID_ARG), (dict(rho0=float("nan")), nq.NQ_E_INVALID_ARG),
                     (dict(lam=float("inf")), nq.NQ_E_INVALID_ARG), (dict(nb=nbytes - 256), nq.NQ_E_INVALID_ARG)):
        with pytest.raises(nq.NQError) as e:
            call(**args(**kw))
        assert e.value.status == code, kw
    call(**args())


def test_config2_shape_two_iterations():
    """The headline layer's shape (4096 x 4096, r = 1024): two full iterations against the oracle."""
    n, m, r = 4096, 4096, 1024
    w, u0, v0 = synth.gen_admm_problem(n, m, r, seed=42)
    ref = O.lb_admm(w, u0, v0, 2, 1.0, 20.0, 1e-3, 4)           # a penalty on the scale of this size's Gram diagonal (about 2.6)
    outs, _, _ = run_gpu(w, u0, v0, 2, 1.0, 20.0, 1e-3, 4)
    print("worst relative error", compare(outs, ref), flush=True)
