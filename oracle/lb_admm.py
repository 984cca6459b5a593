"""CPU oracle for Latent Binary ADMM on one matrix (Section 3.2, Step 2-2 and Step 2-3; Appendix B).

TEST INFRASTRUCTURE ONLY: plain numpy in float64, no blocking, no fusion, the paper's order and
notation.  It shares no code with the HIP library and the product never calls it.

What is computed.  For a target W (n x m) and rank r, the scaled-dual ADMM of

    min  1/2 ||W - U V^T||_F^2 + lambda/2 (||U||_F^2 + ||V||_F^2)   s.t.  U = Z_U, V = Z_V

iterates, for U (and, with the roles of U and V exchanged and W transposed, for V):

    U-step   U (V^T V + (rho + lambda) I) = W V + rho (Z_U - Lambda_U)        (normal equation, Appendix B;
                                                                               solved through a Cholesky factor)
    Z-step   Z_U = SVID(U + Lambda_U)
    dual     Lambda_U = Lambda_U + U - Z_U

Readings taken where the paper is silent:
  * SVID(P) = sign(P) (.) (a b^T): the signs of P times the best rank-one approximation a b^T of |P|
    (Eq. 6 asks for the rank-one approximant whose signs are those of P); sign(0) = +1.  a b^T = sigma u v^T, the leading
    singular triplet of |P|, is found by `power_iters` rounds of power iteration started from the
    all-ones vector (|P| is non-negative, so its leading vectors are too and the start is never orthogonal
    to them); the count is an input, both implementations run exactly that many rounds.
  * order inside one iteration: U-step, Z_U, Lambda_U, then the same for V with the NEW U.
  * the penalty rho follows a linear schedule from rho_start to rho_end over the K iterations (Appendix C
    names the scheduler as linear, over 400 steps, without its end points); K = 1 uses rho_start.
  * initial state: U and V are inputs (random numbers are drawn by the caller), Z = SVID(U), Lambda = 0.
  * magnitude balancing (Step 2-3) with identity preconditioners: P_U = U + Lambda_U, P_V = V + Lambda_V of the
    last iteration, eta = sqrt(||P_V||_F / ||P_U||_F), s1_i = mean_k |eta P_U[i, k]|, s2_j = mean_k |P_V[j, k] / eta|,
    signs = sign(P).
"""
from __future__ import annotations

import numpy as np


def sign_pm1(p: np.ndarray) -> np.ndarray:
    """+1 where p >= 0 (both zeros), -1 where p < 0."""
    return np.where(p >= 0.0, 1.0, -1.0)


def rank_one_of_abs(p: np.ndarray, power_iters: int):
    """Leading singular triplet (sigma, u, v) of |P| by power iteration from the all-ones vector:
    v <- |P|^T u / ||.||, u <- |P| v / ||.||, `power_iters` rounds, sigma = u^T |P| v."""
    a = np.abs(p)
    n, r = a.shape
    u = np.ones(n) / np.sqrt(n)
    v = np.ones(r) / np.sqrt(r)
    for _ in range(power_iters):
        v = a.T @ u
        nv = np.linalg.norm(v)
        v = v / nv if nv > 0 else v
        u = a @ v
        nu = np.linalg.norm(u)
        u = u / nu if nu > 0 else u
    sigma = float(u @ (a @ v))
    return sigma, u, v


def svid(p: np.ndarray, power_iters: int) -> np.ndarray:
    """Sign-value independent decomposition: sign(P) (.) (sigma u v^T) with the rank-one part of |P|."""
    sigma, u, v = rank_one_of_abs(p, power_iters)
    return sign_pm1(p) * (sigma * np.outer(u, v))


def u_step(w: np.ndarray, v: np.ndarray, z_u: np.ndarray, lam_u: np.ndarray, rho: float, lam: float) -> np.ndarray:
    """The unique minimiser of 1/2||W - U V^T||^2 + lam/2||U||^2 + rho/2||U - Z_U + Lambda_U||^2:
    U H = W V + rho (Z_U - Lambda_U) with H = V^T V + (rho + lam) I, through H = L L^T."""
    r = v.shape[1]
    h = v.T @ v + (rho + lam) * np.eye(r)
    rhs = w @ v + rho * (z_u - lam_u)
    l = np.linalg.cholesky(h)
    # U = rhs H^-1  <=>  H U^T = rhs^T : two triangular solves
    y = np.linalg.solve(l, rhs.T)
    return np.linalg.solve(l.T, y).T


def rho_at(k: int, n_iters: int, rho_start: float, rho_end: float) -> float:
    if n_iters <= 1:
        return rho_start
    return rho_start + (rho_end - rho_start) * k / (n_iters - 1)


def lb_admm(w: np.ndarray, u0: np.ndarray, v0: np.ndarray, n_iters: int, rho_start: float, rho_end: float, lam: float,
            power_iters: int):
    """Runs n_iters iterations; returns the final state as a dict (U, V, Z_U, Z_V, Lambda_U, Lambda_V)."""
    u, v = u0.astype(np.float64).copy(), v0.astype(np.float64).copy()
    z_u, z_v = svid(u, power_iters), svid(v, power_iters)
    lam_u, lam_v = np.zeros_like(u), np.zeros_like(v)
    for k in range(n_iters):
        rho = rho_at(k, n_iters, rho_start, rho_end)
        u = u_step(w, v, z_u, lam_u, rho, lam)
        z_u = svid(u + lam_u, power_iters)
        lam_u = lam_u + u - z_u
        v = u_step(w.T, u, z_v, lam_v, rho, lam)
        z_v = svid(v + lam_v, power_iters)
        lam_v = lam_v + v - z_v
    return {"U": u, "V": v, "Z_U": z_u, "Z_V": z_v, "Lambda_U": lam_u, "Lambda_V": lam_v}


def balance(state):
    """Step 2-3 with identity preconditioners: signs of the pre-binary variables P = U + Lambda and the two
    scale vectors.  Returns (sign_U [n, r], sign_V [m, r], s1 [n], s2 [m], eta)."""
    p_u = state["U"] + state["Lambda_U"]
    p_v = state["V"] + state["Lambda_V"]
    eta = float(np.sqrt(np.linalg.norm(p_v) / np.linalg.norm(p_u)))
    s1 = np.abs(eta * p_u).mean(axis=1)
    s2 = np.abs(p_v / eta).mean(axis=1)
    return sign_pm1(p_u), sign_pm1(p_v), s1, s2, eta


def reconstruction(sign_u, sign_v, s1, s2) -> np.ndarray:
    """W^ = Diag(s1) sign_U sign_V^T Diag(s2)  (Section 3.1 Eq. 1)."""
    return (s1[:, None] * (sign_u @ sign_v.T)) * s2[None, :]
