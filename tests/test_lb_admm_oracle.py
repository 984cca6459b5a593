"""Pins of the LB-ADMM oracle (Section 3.2 Step 2-2 / 2-3; Appendix B) against what the paper and the
mathematics fix: the lemmas of Appendix B, closed forms, library factorizations used as an independent
opinion, and properties a wrong sign, a transposed operand or a dropped term would break."""
import numpy as np
import pytest

from oracle import lb_admm as A


def problem(n, m, r, seed):
    g = np.random.default_rng(seed)
    w = g.standard_normal((n, m)) * 0.05 + (g.standard_normal((n, 3)) @ g.standard_normal((3, m))) * 0.1
    u0 = g.standard_normal((n, r)) * 0.1
    v0 = g.standard_normal((m, r)) * 0.1
    return w, u0, v0


def test_system_matrix_is_spd_with_the_diagonal_shift_as_floor():
    """Appendix B, lemma on positive definiteness: H = V^T V + (rho + lambda) I is symmetric with eigenvalues
    >= rho + lambda, also for a rank-deficient V; its condition number obeys the corollary's bound."""
    g = np.random.default_rng(1)
    v = g.standard_normal((40, 12))
    v[:, 5] = v[:, 2]                                        # rank-deficient on purpose
    for rho, lam in [(0.5, 0.0), (1e-3, 1e-2), (3.0, 1.0)]:
        h = v.T @ v + (rho + lam) * np.eye(12)
        assert np.allclose(h, h.T)
        ev = np.linalg.eigvalsh(h)
        assert ev.min() >= (rho + lam) * (1 - 1e-9)
        assert ev.max() / ev.min() <= (1 + np.linalg.norm(v, 2) ** 2 / (rho + lam)) * (1 + 1e-9)


def test_u_step_solves_the_normal_equation_and_minimises_the_subproblem():
    n, m, r = 17, 23, 6
    w, u0, v0 = problem(n, m, r, 2)
    g = np.random.default_rng(3)
    z, lam_u = g.standard_normal((n, r)), g.standard_normal((n, r)) * 0.3
    rho, lam = 0.7, 0.05
    u = A.u_step(w, v0, z, lam_u, rho, lam)
    # the normal equation of Appendix B, typed as printed: U (V^T V + (rho + lambda) I) = W V + rho (Z - Lambda)
    lhs = u @ (v0.T @ v0 + (rho + lam) * np.eye(r))
    rhs = w @ v0 + rho * (z - lam_u)
    assert np.abs(lhs - rhs).max() <= 1e-12 * np.abs(rhs).max()
    # an independent route: the stacked least-squares problem solved by the library's QR-based solver
    a = np.vstack([v0, np.sqrt(lam) * np.eye(r), np.sqrt(rho) * np.eye(r)])
    for i in (0, n - 1):
        b = np.concatenate([w[i], np.zeros(r), np.sqrt(rho) * (z[i] - lam_u[i])])
        ref = np.linalg.lstsq(a, b, rcond=None)[0]
        assert np.abs(u[i] - ref).max() <= 1e-10 * np.abs(ref).max()

    def obj(uu):
        return (0.5 * np.linalg.norm(w - uu @ v0.T) ** 2 + 0.5 * lam * np.linalg.norm(uu) ** 2
                + 0.5 * rho * np.linalg.norm(uu - z + lam_u) ** 2)
    base = obj(u)
    for _ in range(20):                                      # strongly convex: every perturbation is worse
        assert obj(u + 1e-3 * g.standard_normal((n, r))) > base


def test_u_step_rank_one_closed_form():
    """r = 1: U = (W v + rho (z - Lambda)) / (v^T v + rho + lambda), entry by entry."""
    g = np.random.default_rng(4)
    w, v = g.standard_normal((5, 7)), g.standard_normal((7, 1))
    z, lam_u = g.standard_normal((5, 1)), g.standard_normal((5, 1))
    u = A.u_step(w, v, z, lam_u, 0.3, 0.2)
    expect = (w @ v + 0.3 * (z - lam_u)) / (float((v * v).sum()) + 0.5)
    assert np.abs(u - expect).max() <= 1e-14


def test_svid_keeps_signs_has_rank_one_magnitudes_and_fixes_its_own_family():
    g = np.random.default_rng(5)
    p = g.standard_normal((30, 11))
    p[3, 4] = 0.0
    z = A.svid(p, 60)
    assert np.array_equal(np.sign(z[p != 0]), np.sign(p[p != 0])) and z[3, 4] >= 0          # sign(0) = +1
    assert np.linalg.matrix_rank(np.abs(z), tol=1e-10) == 1
    # the magnitudes are the best rank-one approximation of |P|: the library's SVD as an independent opinion
    uu, ss, vt = np.linalg.svd(np.abs(p))
    best = ss[0] * np.outer(uu[:, 0], vt[0])
    assert np.abs(np.abs(z) - np.abs(best)).max() <= 1e-9 * ss[0]
    assert abs(np.linalg.norm(np.abs(p) - np.abs(z)) - np.sqrt((ss[1:] ** 2).sum())) <= 1e-9 * ss[0]
    # a matrix that already is signs times a positive rank-one matrix is reproduced
    s = A.sign_pm1(g.standard_normal((9, 6)))
    q = s * np.outer(g.random(9) + 0.5, g.random(6) + 0.5)
    assert np.abs(A.svid(q, 40) - q).max() <= 1e-12 * np.abs(q).max()
    # zero rounds of power iteration leave the all-ones start: a b^T is then the mean magnitude everywhere
    z0 = A.svid(p, 0)
    assert np.allclose(np.abs(z0), np.abs(p).mean())


def test_one_iteration_by_hand():
    """One iteration written out step by step with library solves (no Cholesky), in the paper's order; the dual
    update is the printed identity; the V-step sees the new U."""
    n, m, r = 12, 9, 4
    w, u0, v0 = problem(n, m, r, 6)
    rho, lam, pi = 0.4, 0.01, 25
    st = A.lb_admm(w, u0, v0, 1, rho, rho, lam, pi)
    z_u0, z_v0 = A.svid(u0, pi), A.svid(v0, pi)
    u1 = np.linalg.solve(v0.T @ v0 + (rho + lam) * np.eye(r), (w @ v0 + rho * z_u0).T).T
    z_u1 = A.svid(u1, pi)
    l_u1 = u1 - z_u1
    v1 = np.linalg.solve(u1.T @ u1 + (rho + lam) * np.eye(r), (w.T @ u1 + rho * z_v0).T).T
    z_v1 = A.svid(v1, pi)
    for key, ref in (("U", u1), ("Z_U", z_u1), ("Lambda_U", l_u1), ("V", v1), ("Z_V", z_v1), ("Lambda_V", v1 - z_v1)):
        assert np.abs(st[key] - ref).max() <= 1e-11 * max(1.0, np.abs(ref).max()), key


def test_penalty_schedule_is_linear():
    assert A.rho_at(0, 5, 1.0, 3.0) == 1.0 and A.rho_at(4, 5, 1.0, 3.0) == 3.0 and A.rho_at(2, 5, 1.0, 3.0) == 2.0
    assert A.rho_at(0, 1, 1.0, 3.0) == 1.0


def test_consensus_and_reconstruction_improve_over_the_iterations():
    """Sanity of the whole loop on a low-rank-plus-noise target: the consensus gap ||U - Z_U|| shrinks as the
    penalty grows, and the balanced binary reconstruction beats the one from the initial state."""
    n, m, r = 96, 80, 24
    w, u0, v0 = problem(n, m, r, 7)

    def rel(state):
        su, sv, s1, s2, _ = A.balance(state)
        return np.linalg.norm(w - A.reconstruction(su, sv, s1, s2)) / np.linalg.norm(w)
    init = {"U": u0, "V": v0, "Lambda_U": np.zeros_like(u0), "Lambda_V": np.zeros_like(v0)}
    s5 = A.lb_admm(w, u0, v0, 5, 0.05, 0.5, 1e-3, 20)
    s40 = A.lb_admm(w, u0, v0, 40, 0.05, 0.5, 1e-3, 20)
    gap = lambda s: np.linalg.norm(s["U"] - s["Z_U"]) / np.linalg.norm(s["U"])
    assert gap(s40) < gap(s5)
    assert rel(s40) < rel(init) and rel(s40) < 1.0


def test_balancing_equalises_the_norms_and_is_scale_invariant():
    """Step 2-3: eta P_U and P_V / eta have equal Frobenius norms; moving a factor c from U to V (the scale
    ambiguity the step removes) changes neither the signs nor the product of the two scale vectors' entries."""
    g = np.random.default_rng(8)
    st = {"U": g.standard_normal((10, 4)), "V": g.standard_normal((7, 4)) * 30,
          "Lambda_U": g.standard_normal((10, 4)) * 0.1, "Lambda_V": g.standard_normal((7, 4))}
    su, sv, s1, s2, eta = A.balance(st)
    pu, pv = st["U"] + st["Lambda_U"], st["V"] + st["Lambda_V"]
    assert abs(np.linalg.norm(eta * pu) - np.linalg.norm(pv / eta)) <= 1e-12 * np.linalg.norm(pv)
    assert np.allclose(s1, np.abs(eta * pu).mean(axis=1)) and np.allclose(s2, np.abs(pv / eta).mean(axis=1))
    c = 7.5
    st2 = {k: (v * c if k in ("U", "Lambda_U") else v / c) for k, v in st.items()}
    su2, sv2, s1b, s2b, _ = A.balance(st2)
    assert np.array_equal(su, su2) and np.array_equal(sv, sv2)
    assert np.allclose(np.outer(s1, s2), np.outer(s1b, s2b))
    # all signs +1 and constant magnitudes: the reconstruction is the constant it must be
    ones = {"U": np.full((3, 2), 2.0), "V": np.full((5, 2), 8.0), "Lambda_U": np.zeros((3, 2)), "Lambda_V": np.zeros((5, 2))}
    su, sv, s1, s2, eta = A.balance(ones)
    assert np.allclose(A.reconstruction(su, sv, s1, s2), 2 * 2.0 * 8.0)
