"""Pins of the post-training quantisation oracle (oracle/ptq.py: the consensus ADMM of the appendix on PTQ-LoRDBA).

No expected value comes from the functions under test.  The closed-form updates are checked against a generic
least-squares solve of the explicitly vectorised problem (the design matrix is built entry by entry from the
definition of the adapter matrix) and against the vanishing gradient of the objective they minimise (torch autograd in
fp64); the whole loop against properties the method fixes (exact fit of rank-one targets, the brute-force optimum on
tiny inputs, the penalty schedule) and against mistakes planted in each update.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import ptq as P
from paper_2605_24058_amd import inputs


def _problem(seed, N, M, R):
    g = np.random.default_rng(seed)
    T = g.standard_normal((N, M))
    U1 = g.standard_normal((N, R))
    U2 = g.standard_normal((R, M))
    alpha = g.standard_normal(N)
    beta = g.standard_normal(R)
    gamma = g.standard_normal(M)
    return T, U1, U2, alpha, beta, gamma


def _dense(alpha, U1, beta, U2, gamma):
    """The adapter matrix entry by entry: sum_k alpha_i U1[i,k] beta_k U2[k,j] gamma_j."""
    N, R = U1.shape
    M = U2.shape[1]
    W = np.zeros((N, M))
    for i in range(N):
        for j in range(M):
            W[i, j] = sum(alpha[i] * U1[i, k] * beta[k] * U2[k, j] * gamma[j] for k in range(R))
    return W


def test_adapter_matrix_and_objective_entrywise():
    T, U1, U2, a, b, c = _problem(0, 5, 4, 3)
    W = _dense(a, U1, b, U2, c)
    assert np.allclose(P.adapter_matrix(a, U1, b, U2, c), W, rtol=1e-13, atol=1e-13)
    assert np.isclose(P.objective(T, a, U1, b, U2, c), 0.5 * sum((T[i, j] - W[i, j]) ** 2 for i in range(5) for j in range(4)),
                      rtol=1e-13)


def _design(which, U1, U2, a, b, c):
    """vec(adapter matrix) = H @ (the scale vector `which`), H built by differentiating the entrywise definition."""
    n = {"alpha": len(a), "beta": len(b), "gamma": len(c)}[which]
    cols = []
    for k in range(n):
        e = np.zeros(n)
        e[k] = 1.0
        args = dict(alpha=a, beta=b, gamma=c)
        args[which] = e
        cols.append(_dense(args["alpha"], U1, args["beta"], U2, args["gamma"]).ravel())
    return np.stack(cols, axis=1)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_scale_updates_solve_their_least_squares_problems(seed):
    T, U1, U2, a, b, c = _problem(seed, 6, 5, 3)
    for which, got in (("alpha", P.alpha_update(T, U1, b, U2, c)), ("gamma", P.gamma_update(T, a, U1, b, U2)),
                       ("beta", P.beta_update(T, a, U1, U2, c))):
        H = _design(which, U1, U2, a, b, c)
        want = np.linalg.lstsq(H, T.ravel(), rcond=None)[0]
        assert np.allclose(got, want, rtol=1e-9, atol=1e-11), which


def _grad(fn, *xs):
    ts = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in xs]
    fn(*ts).backward()
    return [t.grad.numpy() for t in ts]


def _f_torch(T, a, U1, b, U2, c):
    W = (a[:, None] * U1 * b[None, :]) @ (U2 * c[None, :])
    return 0.5 * torch.sum((T - W) ** 2)


@pytest.mark.parametrize("seed", [3, 4])
def test_gradient_vanishes_after_each_scale_update(seed):
    T, U1, U2, a, b, c = _problem(seed, 9, 7, 4)
    Tt, U1t, U2t = (torch.tensor(v) for v in (T, U1, U2))
    a1 = P.alpha_update(T, U1, b, U2, c)
    (ga,) = _grad(lambda x: _f_torch(Tt, x, U1t, torch.tensor(b), U2t, torch.tensor(c)), a1)
    assert np.max(np.abs(ga)) < 1e-10
    c1 = P.gamma_update(T, a1, U1, b, U2)
    (gc,) = _grad(lambda x: _f_torch(Tt, torch.tensor(a1), U1t, torch.tensor(b), U2t, x), c1)
    assert np.max(np.abs(gc)) < 1e-10
    b1 = P.beta_update(T, a1, U1, U2, c1)
    (gb,) = _grad(lambda x: _f_torch(Tt, torch.tensor(a1), U1t, x, U2t, torch.tensor(c1)), b1)
    assert np.max(np.abs(gb)) < 1e-9
    # and the sweep never raises the objective
    f = [P.objective(T, a, U1, b, U2, c), P.objective(T, a1, U1, b, U2, c), P.objective(T, a1, U1, b, U2, c1),
         P.objective(T, a1, U1, b1, U2, c1)]
    assert f[0] >= f[1] >= f[2] >= f[3]


def test_zero_rows_and_columns_get_zero_scale():
    T, U1, U2, a, b, c = _problem(5, 6, 5, 3)
    U1[2, :] = 0.0
    U2[:, 4] = 0.0
    assert P.alpha_update(T, U1, b, U2, c)[2] == 0.0
    assert P.gamma_update(T, a, U1, b, U2)[4] == 0.0


def test_beta_update_is_minimum_norm_on_a_singular_system():
    # two identical rank-one terms: only beta_0 + beta_1 is determined; the minimum-norm solution splits it evenly
    T, U1, U2, a, b, c = _problem(6, 7, 6, 3)
    U1[:, 1] = U1[:, 0]
    U2[1, :] = U2[0, :]
    got = P.beta_update(T, a, U1, U2, c)
    assert np.isclose(got[0], got[1], rtol=1e-9)
    U1m, U2m = np.delete(U1, 1, axis=1), np.delete(U2, 1, axis=0)
    merged = P.beta_update(T, a, U1m, U2m, c)
    assert np.allclose([got[0] + got[1], got[2]], merged, rtol=1e-9)


@pytest.mark.parametrize("seed", [7, 8])
def test_tikhonov_steps_have_vanishing_gradient_and_are_minima(seed):
    T, U1, U2, a, b, c = _problem(seed, 8, 6, 3)
    g = np.random.default_rng(seed + 100)
    M1, Y1 = P.sgn(g.standard_normal(U1.shape)), 0.3 * g.standard_normal(U1.shape)
    M2, Y2 = P.sgn(g.standard_normal(U2.shape)), 0.3 * g.standard_normal(U2.shape)
    rho1, rho2 = 0.37, 0.91
    Tt = torch.tensor(T)
    at, bt, ct = torch.tensor(a), torch.tensor(b), torch.tensor(c)

    def aug1(X):
        return _f_torch(Tt, at, X, bt, torch.tensor(U2), ct) + 0.5 * rho1 * torch.sum((X - torch.tensor(M1) + torch.tensor(Y1)) ** 2)

    X1 = P.u1_step(T, a, b, U2, c, rho1, M1, Y1)
    (g1,) = _grad(aug1, X1)
    assert np.max(np.abs(g1)) < 1e-10
    base = float(aug1(torch.tensor(X1)))
    for _ in range(5):
        assert float(aug1(torch.tensor(X1 + 1e-3 * g.standard_normal(X1.shape)))) > base

    def aug2(X):
        return _f_torch(Tt, at, torch.tensor(X1), bt, X, ct) + 0.5 * rho2 * torch.sum((X - torch.tensor(M2) + torch.tensor(Y2)) ** 2)

    X2 = P.u2_step(T, a, X1, b, c, rho2, M2, Y2)
    (g2,) = _grad(aug2, X2)
    assert np.max(np.abs(g2)) < 1e-10
    base = float(aug2(torch.tensor(X2)))
    for _ in range(5):
        assert float(aug2(torch.tensor(X2 + 1e-3 * g.standard_normal(X2.shape)))) > base


def test_warm_start_fits_rank_one_targets_exactly():
    g = np.random.default_rng(9)
    a, b = g.standard_normal((12, 1)), g.standard_normal((9, 1))
    T = a @ b.T
    U1, U2, alpha, beta, gamma = P.warm_start(T, 1)
    assert P.objective(T, alpha, U1, beta, U2, gamma) < 1e-28 * np.sum(T * T)
    # carriers are the signs of the factors up to the common sign of the pair
    s = np.sign(a[0, 0]) * U1[0, 0]
    assert np.array_equal(U1[:, 0] * s, np.sign(a[:, 0])) and np.array_equal(U2[0, :] * s, np.sign(b[:, 0]))
    assert np.isclose(beta[0], np.linalg.norm(a) * np.linalg.norm(b), rtol=1e-12)
    out = P.ptq(a, b, 1, K=10)
    assert out["frozen"] and out["sweeps"] == 1
    assert 2 * P.objective(T, out["alpha"], out["B1"], out["beta"], out["B2"], out["gamma"]) < 1e-20 * np.sum(T * T)


def test_warm_start_uses_leading_singular_triplets():
    d = inputs.make_ptq_inputs(1, 40, 30, 6)
    T = d["A_star"].astype(np.float64) @ d["B_star"].astype(np.float64).T
    U1, U2, alpha, beta, gamma = P.warm_start(T, 4)
    sv = np.sqrt(np.sort(np.linalg.eigvalsh(T @ T.T))[::-1][:4])      # another route to the singular values
    assert np.allclose(beta, sv, rtol=1e-9)
    for k in range(4):                                                  # sign(u_k): u_k is the eigenvector of T T^T
        w, V = np.linalg.eigh(T @ T.T)
        u = V[:, np.argsort(w)[::-1][k]]
        assert np.array_equal(U1[:, k] * U1[0, k], np.where(u < 0, -1.0, 1.0) * np.where(u[0] < 0, -1.0, 1.0))
    assert np.all(np.abs(U1) == 1) and np.all(np.abs(U2) == 1)


def _brute_force(T, R, sweeps=60):
    """Best objective over every sign pattern of (B1, B2) at R = 1 with the scales fitted by alternating least squares
    (rank-one case: the scaled adapter matrix is (alpha o b1)(gamma o b2)^T beta, whose best fit is the leading singular
    triplet whenever its sign pattern is the one tried)."""
    N, M = T.shape
    best = np.inf
    for s1 in itertools.product([-1.0, 1.0], repeat=N):
        for s2 in itertools.product([-1.0, 1.0], repeat=M):
            B1, B2 = np.array(s1)[:, None], np.array(s2)[None, :]
            a, b, c = np.ones(N), np.ones(1), np.ones(M)
            for _ in range(sweeps):
                a = P.alpha_update(T, B1, b, B2, c)
                c = P.gamma_update(T, a, B1, b, B2)
                b = P.beta_update(T, a, B1, B2, c)
            best = min(best, P.objective(T, a, B1, b, B2, c))
    return best


def test_result_never_beats_and_here_reaches_the_brute_force_optimum():
    g = np.random.default_rng(10)
    A, B = g.standard_normal((3, 2)), g.standard_normal((3, 2))
    T = A @ B.T
    out = P.ptq(A, B, 1, K=40)
    f = P.objective(T, out["alpha"], out["B1"], out["beta"], out["B2"], out["gamma"])
    # at R = 1 signed scales make every sign pattern equivalent, so the optimum is the best rank-one fit:
    sv = np.linalg.svd(T, compute_uv=False)
    assert np.isclose(_brute_force(T, 1), 0.5 * np.sum(sv[1:] ** 2), rtol=1e-6)
    assert f >= 0.5 * np.sum(sv[1:] ** 2) * (1 - 1e-9)


@pytest.mark.parametrize("seed,N,M,R,r0", [(0, 48, 40, 4, 6), (1, 96, 64, 8, 8)])
def test_loop_properties(seed, N, M, R, r0):
    d = inputs.make_ptq_inputs(seed, N, M, r0)
    T = d["A_star"].astype(np.float64) @ d["B_star"].astype(np.float64).T
    K = 30
    tr = []
    out = P.ptq(d["A_star"], d["B_star"], R, K=K, trace=tr)
    rho0 = np.sum(T * T) / (N * R + R * M)
    prev = rho0
    for t, s in enumerate(tr):
        ratio = s["rho"] / prev
        assert ratio in (0.5, 1.0, 2.0)
        if 2 * t >= K:
            assert ratio == 1.0                                          # fixed-penalty tail
        prev = s["rho"]
        assert np.all(np.abs(s["M1"]) == 1) and np.all(np.abs(s["M2"]) == 1)
    # the dual recursion of Eq. (m-y-step), replayed from the trace with the rescaling that follows a penalty change
    Y1 = np.zeros((N, R))
    prev = rho0
    for s in tr:
        Z = s["U1"] + Y1
        assert np.array_equal(s["M1"], np.where(Z < 0, -1.0, 1.0))
        Y1 = (Y1 + s["U1"] - s["M1"]) * (prev / s["rho"])
        assert np.allclose(Y1, s["Y1"], rtol=1e-12, atol=1e-14)
        prev = s["rho"]
    if out["frozen"]:
        assert out["sweeps"] == len(tr) and (len(tr) == 1 or np.array_equal(tr[-1]["M1"], tr[-2]["M1"]))
    # the returned adapter is no worse than a constant fit and its objective matches the dense definition
    f = P.objective(T, out["alpha"], out["B1"], out["beta"], out["B2"], out["gamma"])
    assert f < 0.5 * np.sum(T * T)


def test_planted_mistakes_are_caught():
    T, U1, U2, a, b, c = _problem(11, 7, 6, 3)
    H = _design("beta", U1, U2, a, b, c)
    want = np.linalg.lstsq(H, T.ravel(), rcond=None)[0]
    Pm, Q = a[:, None] * U1, U2 * c[None, :]
    wrong_gram = np.linalg.pinv((Pm.T @ Pm) @ (Q @ Q.T)) @ np.sum((Pm.T @ T) * Q, axis=1)   # matrix, not Hadamard, product
    assert not np.allclose(wrong_gram, want, rtol=1e-3)
    wrong_alpha = np.sum(T * ((U1 * b) @ U2), axis=1) / np.sum(((U1 * b) @ U2) ** 2, axis=1)   # gamma dropped
    assert not np.allclose(wrong_alpha, np.linalg.lstsq(_design("alpha", U1, U2, a, b, c), T.ravel(), rcond=None)[0], rtol=1e-3)
    # a Tikhonov step that forgets the dual no longer zeroes the gradient of the augmented objective
    g = np.random.default_rng(12)
    M1, Y1 = P.sgn(g.standard_normal(U1.shape)), 0.3 * g.standard_normal(U1.shape)
    X = P.u1_step(T, a, b, U2, c, 0.5, M1, np.zeros_like(Y1))
    Tt = torch.tensor(T)

    def aug(Xt):
        return _f_torch(Tt, torch.tensor(a), Xt, torch.tensor(b), torch.tensor(U2), torch.tensor(c)) + 0.25 * torch.sum(
            (Xt - torch.tensor(M1) + torch.tensor(Y1)) ** 2)

    (gr,) = _grad(aug, X)
    assert np.max(np.abs(gr)) > 1e-3


def test_rank_larger_than_the_factors_is_refused():
    d = inputs.make_ptq_inputs(0, 16, 16, 4)
    with pytest.raises(ValueError):
        P.ptq(d["A_star"], d["B_star"], 5)


@pytest.mark.parametrize("seed,N,M,R,r0", [(0, 96, 80, 6, 8), (1, 200, 160, 8, 8), (2, 300, 300, 16, 16)])
def test_signs_stabilise_within_fifty_sweeps_and_the_tail_converges(seed, N, M, R, r0):
    """What the paper states about the run (paragraph on finite stabilisation on a fixed-penalty tail): the sign
    matrices stop changing after finitely many sweeps, at most about 50 in its experiments, and stay so on the
    fixed-penalty tail, where the iterates converge to a single limit.  Checked with the loop's break switched off."""
    d = inputs.make_ptq_inputs(seed, N, M, r0)
    K = 100
    tr = []
    out = P.ptq(d["A_star"], d["B_star"], R, K=K, trace=tr, stop_on_freeze=False)
    assert len(tr) == K and out["frozen"]
    changes = [int((tr[t]["M1"] != tr[t - 1]["M1"]).sum() + (tr[t]["M2"] != tr[t - 1]["M2"]).sum()) for t in range(1, K)]
    first_still = next(t for t, c in enumerate(changes, start=1) if c == 0)
    assert first_still <= 50
    assert all(c == 0 for c in changes[first_still - 1:])                 # once still, still for the rest of the run
    stopped = P.ptq(d["A_star"], d["B_star"], R, K=K)                     # the loop with its break ends exactly there
    assert stopped["sweeps"] == first_still + 1 and np.array_equal(stopped["B1"], tr[first_still]["M1"])
    assert all(tr[t]["rho"] == tr[K // 2]["rho"] for t in range(K // 2, K))
    step = [np.linalg.norm(tr[t]["U1"] - tr[t - 1]["U1"]) + np.linalg.norm(tr[t]["U2"] - tr[t - 1]["U2"]) for t in range(K // 2, K)]
    assert step[-1] <= 1e-10 * np.linalg.norm(tr[-1]["U1"])
    assert abs(out["objective"][-1] - out["objective"][K // 2]) <= 1e-9 * out["objective"][-1]


def test_defaults_are_the_settings_the_paper_prints():
    """K, (tau, mu), the truncation of the penalty schedule and the warm penalty against tests/golden/ptq_settings.txt."""
    import inspect
    import os
    gold = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "ptq_settings.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            gold[k] = float(v)
    sig = inspect.signature(P.ptq).parameters
    assert sig["K"].default == gold["K"] and sig["tau"].default == gold["tau"] and sig["mu"].default == gold["mu"]
    from paper_2605_24058_amd import binding
    bsig = inspect.signature(binding.lordba_ptq).parameters
    assert bsig["K"].default == gold["K"] and bsig["tau"].default == gold["tau"] and bsig["mu"].default == gold["mu"]
    d = inputs.make_ptq_inputs(3, 60, 50, 6)
    T = d["A_star"].astype(np.float64) @ d["B_star"].astype(np.float64).T
    K = 20
    tr = []
    P.ptq(d["A_star"], d["B_star"], 4, K=K, trace=tr, stop_on_freeze=False)
    rho0 = np.sum(T * T) / (60 * 4 + 4 * 50)                                  # the printed warm penalty
    assert tr[0]["rho"] / rho0 in (0.5, 1.0, 2.0)
    last_change = max(t for t in range(1, K) if tr[t]["rho"] != tr[t - 1]["rho"])
    assert last_change < gold["balancing_until_fraction_of_K"] * K             # no change from sweep K / 2 on
