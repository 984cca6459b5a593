/*
 * nq_lb_admm.h -- C ABI of the latent-binary ADMM initialisation of one weight matrix on one
 * MI355X (gfx950): Section 3.2, Step 2-2 (LB-ADMM, the objective of Eq. 4, the linear system of
 * Eq. 5, the SVID proxy update of Eq. 6 and the dual update that follows it) and Step 2-3
 * (latent magnitude balancing); the well-posedness of the linear systems is Appendix B.
 *
 * Everything is IEEE binary64 ("double"), matrices are dense row-major without padding, all
 * matrix pointers are DEVICE pointers of the current HIP device, 8-byte aligned, owned by the
 * caller and never retained.  The functions return the NQ_* codes of nq_binlr.h (NQ_OK = 0); the
 * text of the last failure is nq_last_error_string().  Nothing here allocates device memory: the
 * caller brings the workspace.
 *
 * One iteration k = 0 .. K-1, with rho_k on a straight line from rho_start to rho_end
 * (Appendix C: linear penalty schedule; K = 1 uses rho_start), in this order:
 *     U   <-  (W V + rho_k (Z_U - Lambda_U)) (V^T V + (rho_k + lambda) I)^-1       (Eq. 5, Cholesky)
 *     Z_U <-  SVID(U + Lambda_U)                                                    (Eq. 6)
 *     Lambda_U <- Lambda_U + U - Z_U
 *     then the same for V with W^T and the NEW U.
 * SVID(P) = sign(P) (.) (sigma a b^T): the signs of P (sign(0) = +1) times the leading singular
 * triplet of |P|, found by exactly `power_iters` rounds of power iteration from the all-ones
 * vector (b <- |P|^T a / ||.||, a <- |P| b / ||.||; 0 rounds leave a b^T = mean |P|).
 * Initial state: U0, V0 are inputs, Z = SVID(U0) / SVID(V0), Lambda = 0.
 *
 * How the linear system is solved: H = V^T V + (rho + lambda) I is factorised H = L L^T by a
 * blocked Cholesky (64-wide block columns), L^-1 is formed block-recursively, H^-1 = L^-T L^-1,
 * and U = RHS H^-1 is one dense product.  H is symmetric positive definite with smallest
 * eigenvalue >= rho + lambda (Appendix B), so the inverse exists; a non-positive pivot (NaN or
 * rho + lambda <= 0 in the input) makes the call fail with NQ_E_INVALID_ARG.
 */
#ifndef NQ_LB_ADMM_H
#define NQ_LB_ADMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Largest rank and matrix side the solver accepts. */
#define NQ_ADMM_MAX_RANK 8192
#define NQ_ADMM_MAX_DIM  65536

/* Bytes of device workspace nq_lb_admm / nq_lb_admm_balance need for W [n, m] and rank r.
 * Host only (no GPU needed).  NQ_E_SHAPE for n, m < 1, r < 1 or beyond the limits above. */
int nq_lb_admm_workspace_bytes(int64_t n, int64_t m, int64_t r, size_t* bytes);

/* Runs n_iters >= 0 iterations of LB-ADMM (Section 3.2 Step 2-2; order and SVID as stated above).
 * W: [n, m];  U0: [n, r];  V0: [m, r]  (inputs, not modified; U0 may alias U and V0 may alias V).
 * U, Z_U, Lambda_U: [n, r];  V, Z_V, Lambda_V: [m, r]  (outputs, fully overwritten).
 * workspace: device, at least nq_lb_admm_workspace_bytes(n, m, r) bytes, 256-byte aligned; its
 *            contents before and after the call mean nothing.
 * stream: hipStream_t or NULL.  The call enqueues the factorisations and solves on `stream` and
 * the products with W and the SVIDs on a second stream of the library's own, ordered against
 * `stream` by events; it then waits for both and reports a failed factorisation
 * (NQ_E_INVALID_ARG; the outputs are then unspecified).  That second stream and its events exist
 * once per process: calls from different host threads must not overlap in time, and `stream` must
 * not be under graph capture.
 * NQ_E_NULL / NQ_E_ALIGN / NQ_E_SHAPE / NQ_E_INVALID_ARG (non-finite rho, lambda; power_iters < 0;
 * workspace too small) are returned before anything is launched. */
int nq_lb_admm(const double* W, int64_t n, int64_t m, int64_t r, const double* U0, const double* V0,
               int n_iters, double rho_start, double rho_end, double lambda, int power_iters,
               double* U, double* V, double* Z_U, double* Z_V, double* Lambda_U, double* Lambda_V,
               void* workspace, size_t workspace_bytes, void* stream);

/* Latent magnitude balancing (Section 3.2 Step 2-3, identity preconditioners): with
 * P_U = U + Lambda_U and P_V = V + Lambda_V of the last iteration,
 *     eta = sqrt(||P_V||_F / ||P_U||_F),  s1[i] = mean_k |eta P_U[i, k]|,  s2[j] = mean_k |P_V[j, k] / eta|,
 * and the sign bits of P_U, P_V in the canonical packed format of nq_pack_signs
 * ([rows, ceil(r/32)] words, bit b of word w = column 32 w + b, 1 iff the value is >= 0, pad bits 0).
 * U, Lambda_U: [n, r];  V, Lambda_V: [m, r]  (device, inputs).
 * U_words: device, n * ceil(r/32) words;  V_words: device, m * ceil(r/32) words;  s1: device, n doubles;
 * s2: device, m doubles;  eta: device, 1 double  (all fully overwritten).
 * The scales are left in binary64; rounding them to the layer's fp16 is the caller's step.
 * workspace as for nq_lb_admm.  Asynchronous on `stream`.  A zero P_U or P_V gives non-finite eta
 * and scales (as the formula does). */
int nq_lb_admm_balance(const double* U, const double* Lambda_U, int64_t n,
                       const double* V, const double* Lambda_V, int64_t m, int64_t r,
                       uint32_t* U_words, uint32_t* V_words, double* s1, double* s2, double* eta,
                       void* workspace, size_t workspace_bytes, void* stream);

/* The dense binary64 product behind the solver, exposed for tests and for measuring it:
 *     C = alpha op(A) op(B) + beta C        (C: [M, N] row-major with leading dimension ldc)
 * op(A) is [M, K]: trans_a = 0 -> A is stored [M, K] (lda >= K), 1 -> stored [K, M] (lda >= M);
 * op(B) is [K, N]: trans_b = 0 -> B is stored [K, N] (ldb >= N), 1 -> stored [N, K] (ldb >= K).
 * Device pointers, 8-byte aligned; C must not overlap A or B.  beta = 0 never reads C.
 * Runs on the matrix cores (v_mfma_f64_16x16x4_f64).  Asynchronous on `stream`. */
int nq_dgemm(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K, double alpha,
             const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
             double* C, int64_t ldc, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NQ_LB_ADMM_H */
