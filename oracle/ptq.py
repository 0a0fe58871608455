"""CPU oracle for PTQ-LoRDBA at envelope rank 1: the scaled consensus ADMM that fits a LoRDBA adapter
diag(alpha) B1 diag(beta) B2 diag(gamma) to a given low-rank update Delta W* = A* (B*)^T in the Frobenius norm
(Appendix "Post-training quantisation": Eq. (ptq-problem), Eq. (admm-problem), the ordered updates Eq. (u-step-1),
Eq. (u-step-2), Eq. (scales-step), Eq. (m-y-step); the closed-form scale updates Eq. (alpha-update), Eq. (gamma-update),
Eq. (beta-gram), Eq. (beta-pinv); Alg. PTQ-LoRDBA; the warm start Eq. (svd-init); the hyper-parameters K = 100,
(tau, mu) = (2, 10), rho0 = ||Delta W*||_F^2 / (NR + RM) of the appendix on implementation details).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of
``bench.py``.  The product package never imports this module, and this module never imports the product package.

Everything is numpy fp64 on the dense N x M target; each function is the formula of the passage it cites with library
primitives (matrix product, SVD, linear solve, pseudo-inverse) as steps, and nothing is blocked, fused or factored: the
target is formed densely and every Gram matrix is taken from the dense operands.

Pins (tests/test_oracle_ptq_pins.py): every closed-form update against a generic least-squares solve of the explicitly
vectorised problem and against the vanishing gradient of its objective (torch autograd, fp64); the Tikhonov steps
likewise; rank-one targets are fitted exactly by the warm start; the objective never rises in a scale sweep; the
minimum-norm property of the beta update on a planted singular system; the result never beats the brute-force optimum
over all sign patterns on tiny inputs and reaches it where the optimum is unique and known; the penalty is constant on
the second half of the run and moves only by factors of tau; with the loop's break switched off the sign matrices stop
changing within 50 sweeps, stay so, and the iterates converge on the fixed-penalty tail (the paper's statements on finite
stabilisation); mistakes planted in each update are caught.

Readings of the paper taken here (the product takes the same ones):
  * sign(0) = +1 (the packed format stores a sign bit).
  * The warm start keeps beta = the leading R singular values and takes gamma = 1, then updates alpha, then gamma
    (Alg. PTQ-LoRDBA initialises only alpha and gamma by the sweep; the sweep needs a starting gamma).
  * One scale sweep updates alpha, then gamma, then beta (the order of the appendix on the scale updates), each with the
    newest values of the others, and is taken at the continuous U^(t+1) as Eq. (scales-step) states.
  * Residual balancing (the paper names Boyd's rule only): primal residual r = sqrt(sum_k ||U_k - M_k||_F^2) at the new
    iterates, dual residual s = sqrt(sum_k (rho_k ||M_k^(t+1) - M_k^(t)||_F)^2) with rho_k = rho / n_k; r > mu s multiplies
    rho by tau and divides the scaled duals Y by tau, s > mu r does the opposite; applied after sweeps t < K/2 only.
  * The loop ends after the first sweep whose sign matrices equal those of the sweep before (Alg. PTQ-LoRDBA), and
    the newest iterates are returned.
  * R may not exceed the rank r0 of the target's factors: beyond it the singular vectors of the warm start are not
    defined.
"""
from __future__ import annotations

import numpy as np


def sgn(x):
    """sign with sign(0) = +1."""
    return np.where(np.asarray(x) < 0, -1.0, 1.0)


def adapter_matrix(alpha, B1, beta, B2, gamma):
    """Delta W(theta) of Def. 1 at envelope rank 1: diag(alpha) B1 diag(beta) B2 diag(gamma), N x M."""
    return (alpha[:, None] * B1 * beta[None, :]) @ (B2 * gamma[None, :])


def objective(T, alpha, B1, beta, B2, gamma):
    """f of Eq. (admm-problem): half the squared Frobenius distance to the target."""
    E = T - adapter_matrix(alpha, B1, beta, B2, gamma)
    return 0.5 * float(np.sum(E * E))


def alpha_update(T, B1, beta, B2, gamma):
    """Eq. (alpha-update): per row i, <T_i, D_i> / ||D_i||^2 with D = B1 diag(beta) B2 diag(gamma), Eq. (alpha-D); 0 where D_i = 0."""
    D = (B1 * beta[None, :]) @ (B2 * gamma[None, :])
    num = np.sum(T * D, axis=1)
    den = np.sum(D * D, axis=1)
    out = np.zeros_like(num)
    nz = den > 0
    out[nz] = num[nz] / den[nz]
    return out


def gamma_update(T, alpha, B1, beta, B2):
    """Eq. (gamma-update): per column j, <T_:j, D_:j> / ||D_:j||^2 with D = diag(alpha) B1 diag(beta) B2, Eq. (gamma-D)."""
    D = (alpha[:, None] * B1 * beta[None, :]) @ B2
    num = np.sum(T * D, axis=0)
    den = np.sum(D * D, axis=0)
    out = np.zeros_like(num)
    nz = den > 0
    out[nz] = num[nz] / den[nz]
    return out


def beta_update(T, alpha, B1, B2, gamma):
    """Eq. (beta-gram), Eq. (beta-Schur), Eq. (beta-pinv): G = (P^T P) o (Q Q^T), h_k = <T, P_:k Q_k:>, beta = pinv(G) h."""
    P = alpha[:, None] * B1
    Q = B2 * gamma[None, :]
    G = (P.T @ P) * (Q @ Q.T)
    h = np.sum((P.T @ T) * Q, axis=1)
    return np.linalg.pinv(G, hermitian=True) @ h


def u1_step(T, alpha, beta, U2, gamma, rho1, M1, Y1):
    """Eq. (u-step-1): the Tikhonov least-squares problem in U1; it separates over the rows of U1, row i solving
    (alpha_i^2 C C^T + rho1 I) u = alpha_i C T_i^T + rho1 (M1 - Y1)_i with C = diag(beta) U2 diag(gamma)."""
    C = beta[:, None] * U2 * gamma[None, :]
    G = C @ C.T
    TC = T @ C.T
    R = G.shape[0]
    U1 = np.empty_like(M1)
    for i in range(T.shape[0]):
        H = alpha[i] * alpha[i] * G + rho1 * np.eye(R)
        U1[i] = np.linalg.solve(H, alpha[i] * TC[i] + rho1 * (M1[i] - Y1[i]))
    return U1


def u2_step(T, alpha, U1, beta, gamma, rho2, M2, Y2):
    """Eq. (u-step-2): the same in U2, column j solving (gamma_j^2 C^T C + rho2 I) u = gamma_j C^T T_:j + rho2 (M2 - Y2)_:j
    with C = diag(alpha) U1 diag(beta)."""
    C = alpha[:, None] * U1 * beta[None, :]
    G = C.T @ C
    CT = C.T @ T
    R = G.shape[0]
    U2 = np.empty_like(M2)
    for j in range(T.shape[1]):
        H = gamma[j] * gamma[j] * G + rho2 * np.eye(R)
        U2[:, j] = np.linalg.solve(H, gamma[j] * CT[:, j] + rho2 * (M2[:, j] - Y2[:, j]))
    return U2


def warm_start(T, R):
    """Eq. (svd-init) and the initialisation lines of Alg. PTQ-LoRDBA: carriers = signs of the leading R singular vectors,
    beta = the leading R singular values, then alpha and gamma by their closed forms (from gamma = 1)."""
    Us, S, Vt = np.linalg.svd(T, full_matrices=False)
    U1 = sgn(Us[:, :R])
    U2 = sgn(Vt[:R, :])
    beta = S[:R].copy()
    gamma = np.ones(T.shape[1])
    alpha = alpha_update(T, U1, beta, U2, gamma)
    gamma = gamma_update(T, alpha, U1, beta, U2)
    return U1, U2, alpha, beta, gamma


def ptq(A_star, B_star, R, K=100, tau=2.0, mu=10.0, trace=None, stop_on_freeze=True):
    """Alg. PTQ-LoRDBA.  A_star [N, r0], B_star [M, r0] (any float dtype, taken to fp64); returns a dict with the sign
    matrices B1 [N, R], B2 [R, M] (+-1 as fp64), alpha [N], beta [R], gamma [M], the number of sweeps run, whether the
    loop ended on equal sign matrices, the penalty it ended with, and the objective of Eq. (admm-problem) at the continuous
    U after each sweep's scale update.  `trace`, if a list, receives a copy of the state after every sweep.
    stop_on_freeze=False runs all K sweeps (the algorithm's loop without its break), for looking at the tail."""
    A = np.asarray(A_star, dtype=np.float64)
    B = np.asarray(B_star, dtype=np.float64)
    N, r0 = A.shape
    M_, r0b = B.shape
    if r0 != r0b or R < 1 or R > r0:
        raise ValueError("PTQ needs factors of one rank r0 and 1 <= R <= r0")
    T = A @ B.T
    U1, U2, alpha, beta, gamma = warm_start(T, R)
    M1, M2 = U1.copy(), U2.copy()
    Y1, Y2 = np.zeros_like(U1), np.zeros_like(U2)
    n1, n2 = N * R, R * M_
    rho = float(np.sum(T * T)) / (n1 + n2)
    f_hist = []
    frozen = False
    sweeps = 0
    for t in range(K):
        rho1, rho2 = rho / n1, rho / n2
        U1 = u1_step(T, alpha, beta, U2, gamma, rho1, M1, Y1)
        U2 = u2_step(T, alpha, U1, beta, gamma, rho2, M2, Y2)
        alpha = alpha_update(T, U1, beta, U2, gamma)
        gamma = gamma_update(T, alpha, U1, beta, U2)
        beta = beta_update(T, alpha, U1, U2, gamma)
        f_hist.append(objective(T, alpha, U1, beta, U2, gamma))
        M1n, M2n = sgn(U1 + Y1), sgn(U2 + Y2)
        Y1 = Y1 + U1 - M1n
        Y2 = Y2 + U2 - M2n
        same = bool(np.array_equal(M1n, M1) and np.array_equal(M2n, M2))
        if 2 * t < K:
            r = np.sqrt(np.sum((U1 - M1n) ** 2) + np.sum((U2 - M2n) ** 2))
            s = np.sqrt(rho1 * rho1 * np.sum((M1n - M1) ** 2) + rho2 * rho2 * np.sum((M2n - M2) ** 2))
            if r > mu * s:
                rho *= tau
                Y1 /= tau
                Y2 /= tau
            elif s > mu * r:
                rho /= tau
                Y1 *= tau
                Y2 *= tau
        M1, M2 = M1n, M2n
        sweeps = t + 1
        if trace is not None:
            trace.append(dict(U1=U1.copy(), U2=U2.copy(), M1=M1.copy(), M2=M2.copy(), Y1=Y1.copy(), Y2=Y2.copy(),
                              alpha=alpha.copy(), beta=beta.copy(), gamma=gamma.copy(), rho=rho))
        if same:
            frozen = True
            if stop_on_freeze:
                break
    return dict(B1=M1, B2=M2, alpha=alpha, beta=beta, gamma=gamma, sweeps=sweeps, frozen=frozen, rho=rho,
                objective=np.array(f_hist), U1=U1, U2=U2, Y1=Y1, Y2=Y2)


def canonical_gauge(B1, B2):
    """The pair (B1[:, k], B2[k, :]) is defined up to a common sign (the singular vectors of the warm start are); flip
    each pair so that B1[0, k] = +1.  Returns the flipped copies and the +-1 flips."""
    flip = np.where(B1[0, :] < 0, -1.0, 1.0)
    return B1 * flip[None, :], B2 * flip[:, None], flip
