"""Property tests of the oracle over random small shapes (hypothesis): every function against the same map written with
numpy fp64 matrices (dense DeltaW of Eq. (lordba); gradients as contractions of X^T G), none of which shares code with
the C oracle.  The fixed-shape pins live in the other test_oracle_* files; this file widens the shapes."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from paper_2605_24058_amd import inputs

shape = st.tuples(st.integers(1, 6), st.integers(1, 70), st.integers(1, 70), st.integers(1, 9), st.integers(0, 10 ** 6))


def _f64(d):
    return {k: np.asarray(v, dtype=np.float64) for k, v in d.items()}


def _close(a, b, tol=1e-11):
    scale = max(np.max(np.abs(b)), 1e-300)
    return np.max(np.abs(np.asarray(a) - np.asarray(b))) <= tol * scale


@settings(max_examples=40, deadline=None)
@given(shape)
def test_forward_matches_dense_delta_w(s):
    T, d_in, d_out, r, seed = s
    d = inputs.make_inputs(seed, T, d_in, d_out, r)
    f = _f64(d)
    dW = (f["s_in"][:, None] * f["signsA"].T) @ (f["s_rank"][:, None] * f["signsB"].T) * f["s_out"][None, :]
    want = f["y_base"] + f["x"] @ dW
    got = oracle.forward(d["x"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["y_base"])
    assert _close(got, want)
    packed = oracle.forward_packed(d["x"], oracle.pack(d["signsA"]), oracle.pack(d["signsB"]), d["s_in"], d["s_rank"], d["s_out"],
                                   d["y_base"], r)
    assert np.array_equal(packed, got)
    assert _close(oracle.rank_intermediate(d["x"], d["signsA"], d["s_in"]), (f["x"] * f["s_in"]) @ f["signsA"].T)


@settings(max_examples=40, deadline=None)
@given(shape, st.sampled_from([0.5, 7.0, 100.0]))
def test_backward_matches_contractions_of_xt_g(s, kappa):
    T, d_in, d_out, r, seed = s
    d = inputs.make_backward_inputs(seed, T, d_in, d_out, r)
    f = _f64(d)
    al, be, ga, sA, sB = f["s_in"], f["s_rank"], f["s_out"], f["signsA"], f["signsB"]
    M = f["x"].T @ f["g"]                                   # dL/dDeltaW  [d_in, d_out]
    # kappa (1 - tanh^2) written as kappa / cosh^2: at these tiny widths the latents are O(1) and tanh saturates to 1.0
    factor = lambda u: kappa / np.cosh(kappa * u) ** 2
    left = al[:, None] * sA.T                               # D_alpha B1           [d_in, r]
    right = sB.T * ga[None, :]                              # B2 D_gamma           [r, d_out]
    want = {
        "dx": f["dx_base"] + f["g"] @ ((left * be[None, :]) @ right).T,
        "d_s_in": np.sum(M * ((sA.T * be[None, :]) @ right), axis=1),
        "d_s_rank": np.einsum("ik,ij,kj->k", left, M, right),
        "d_s_out": np.sum(M * ((left * be[None, :]) @ sB.T), axis=0),
        "d_latA": ((al[:, None] * (M @ right.T)) * be[None, :]).T * factor(f["latA"]),
        "d_latB": ((left.T @ M) * be[:, None] * ga[None, :]).T * factor(f["latB"]),
    }
    got = oracle.backward(d["x"], d["g"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["latA"], d["latB"], kappa,
                          d["dx_base"])
    for k in want:
        assert _close(got[k], want[k], 1e-9), k


@settings(max_examples=25, deadline=None)
@given(st.integers(1, 40), st.integers(1, 40), st.integers(0, 10 ** 6))
def test_pack_round_trip_and_bit_positions(rows, cols, seed):
    g = np.random.default_rng(seed)
    s = (g.integers(0, 2, size=(rows, cols)) * 2 - 1).astype(np.int8)
    w = oracle.pack(s)
    assert np.array_equal(oracle.unpack(w, rows, cols), s)
    flat = s.reshape(-1)
    n = int(g.integers(0, flat.size))
    assert ((int(w[n // 32]) >> (n % 32)) & 1) == (1 if flat[n] == -1 else 0)       # bit n of the row-major stream, 1 = -1
    assert w.size == (rows * cols + 31) // 32
    if (rows * cols) % 32:
        assert int(w[-1]) >> ((rows * cols) % 32) == 0                               # pad bits are zero


# ---- post-training quantisation (oracle/ptq.py): properties over random small problems ---------------------------------

ptq_shape = st.tuples(st.integers(2, 14), st.integers(2, 14), st.integers(1, 4), st.integers(0, 10 ** 6))


@settings(max_examples=30, deadline=None)
@given(ptq_shape)
def test_ptq_updates_are_coordinate_minimisers(s):
    """Each closed-form update minimises the objective over its block: no random move of that block lowers it, and the
    Tikhonov steps do the same for their augmented objectives."""
    from oracle import ptq as P
    N, M, R, seed = s
    g = np.random.default_rng(seed)
    T = g.standard_normal((N, M))
    U1, U2 = g.standard_normal((N, R)), g.standard_normal((R, M))
    a, b, c = g.standard_normal(N), g.standard_normal(R), g.standard_normal(M)
    f = lambda a_, b_, c_, U1_=U1, U2_=U2: P.objective(T, a_, U1_, b_, U2_, c_)
    a1 = P.alpha_update(T, U1, b, U2, c)
    c1 = P.gamma_update(T, a1, U1, b, U2)
    b1 = P.beta_update(T, a1, U1, U2, c1)
    assert f(a, b, c) >= f(a1, b, c) * (1 - 1e-12) and f(a1, b, c) >= f(a1, b, c1) * (1 - 1e-12) >= 0
    assert f(a1, b, c1) >= f(a1, b1, c1) * (1 - 1e-12)
    slack = 1e-12 * max(np.sum(T * T), 1.0)   # (a flat direction leaves the objective unchanged up to rounding)
    for _ in range(3):
        assert f(a1 + 1e-3 * g.standard_normal(N), b, c) >= f(a1, b, c) - slack
        assert f(a1, b, c1 + 1e-3 * g.standard_normal(M)) >= f(a1, b, c1) - slack
        assert f(a1, b1 + 1e-3 * g.standard_normal(R), c1) >= f(a1, b1, c1) - slack
    M1, Y1 = P.sgn(g.standard_normal((N, R))), 0.2 * g.standard_normal((N, R))
    rho = float(g.uniform(0.05, 2.0))
    X1 = P.u1_step(T, a, b, U2, c, rho, M1, Y1)
    aug = lambda X: f(a, b, c, U1_=X) + 0.5 * rho * np.sum((X - M1 + Y1) ** 2)
    for _ in range(3):
        assert aug(X1 + 1e-3 * g.standard_normal((N, R))) > aug(X1)
    M2, Y2 = P.sgn(g.standard_normal((R, M))), 0.2 * g.standard_normal((R, M))
    X2 = P.u2_step(T, a, X1, b, c, rho, M2, Y2)
    aug2 = lambda X: f(a, b, c, U1_=X1, U2_=X) + 0.5 * rho * np.sum((X - M2 + Y2) ** 2)
    for _ in range(3):
        assert aug2(X2 + 1e-3 * g.standard_normal((R, M))) > aug2(X2)


@settings(max_examples=20, deadline=None)
@given(st.integers(4, 24), st.integers(4, 24), st.integers(1, 4), st.integers(0, 10 ** 6))
def test_ptq_run_invariants(N, M, R, seed):
    """A whole run: +-1 outputs, the recorded objective, and dependence on the factors through their product only
    (negating a column of both factors changes nothing)."""
    from oracle import ptq as P
    r0 = 4
    d = inputs.make_ptq_inputs(seed, N, M, r0)
    A, B = d["A_star"].astype(np.float64), d["B_star"].astype(np.float64)
    tr = []
    out = P.ptq(A, B, R, K=12, trace=tr)
    assert np.all(np.abs(out["B1"]) == 1) and np.all(np.abs(out["B2"]) == 1)
    assert out["sweeps"] == len(tr) == len(out["objective"]) <= 12
    T = A @ B.T
    last = tr[-1]
    assert np.isclose(out["objective"][-1], P.objective(T, last["alpha"], last["U1"], last["beta"], last["U2"], last["gamma"]), rtol=1e-9,
                      atol=1e-14 * np.sum(T * T))
    # the target A B^T does not change when a column of A and the same column of B are both negated: same run
    A2, B2 = A.copy(), B.copy()
    A2[:, 0] *= -1
    B2[:, 0] *= -1
    out2 = P.ptq(A2, B2, R, K=12)
    g1, g2, _ = P.canonical_gauge(out["B1"], out["B2"])
    h1, h2, _ = P.canonical_gauge(out2["B1"], out2["B2"])
    assert out2["sweeps"] == out["sweeps"] and np.array_equal(g1, h1) and np.array_equal(g2, h2)
