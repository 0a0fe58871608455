"""GPU parity of post-training quantisation (appendix on PTQ-LoRDBA; Alg. PTQ-LoRDBA): lordba_ptq through the C ABI
against the fp64 numpy oracle (oracle/ptq.py) on the same seeded factors.

The method decides integers (the sign matrices, the number of sweeps, the power of tau in the penalty) from fp64
arithmetic; both sides take those decisions in fp64, and they must agree exactly: the sign matrices bit for bit (after
fixing the one freedom the method leaves, the common sign of each pair (column k of B1, row k of B2), inherited from the
singular vectors of the warm start), the sweep count, the end flag.  The real-valued results differ only by summation
order and by the route through the linear algebra (the device never forms the N x M target): scales and continuous
iterates within 1e-8 relative L2, the objective within 1e-10 of ||Delta W*||_F^2 (it is a difference of numbers of that
size)."""
import sys

import numpy as np
import pytest

import oracle
from oracle import ptq as P
from paper_2605_24058_amd import binding, inputs

pytestmark = pytest.mark.gpu

TOL_REAL = 1e-8
TOL_OBJ = 1e-10


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_gpu(torch, d, R, K=100, tau=2.0, mu=10.0):
    A = torch.from_numpy(d["A_star"]).cuda()
    B = torch.from_numpy(d["B_star"]).cuda()
    out = binding.lordba_ptq(A, B, R, K=K, tau=tau, mu=mu)
    torch.cuda.synchronize()
    N, M = A.shape[0], B.shape[0]
    res = {k: v.cpu().numpy() for k, v in out.items() if k != "workspace"}
    sA, sB = binding.lordba_unpack_signs(res["packedA"].view(np.uint32), res["packedB"].view(np.uint32), N, M, R)
    res["B1"] = sA.T.astype(np.float64)          # S_A = B1^T [R, N]
    res["B2"] = sB.T.astype(np.float64)          # S_B = B2^T [M, R]
    assert np.array_equal(A.cpu().numpy(), d["A_star"]) and np.array_equal(B.cpu().numpy(), d["B_star"])
    return res


def rel(a, b):
    return np.linalg.norm(np.ravel(a) - np.ravel(b)) / max(np.linalg.norm(np.ravel(b)), 1e-300)


def compare(res, ref, K, check_iterates=True):
    info = res["info"]
    assert info[4] == 0.0
    assert int(info[0]) == ref["sweeps"], (info[0], ref["sweeps"])
    assert bool(info[1]) == ref["frozen"]
    assert abs(info[2] - ref["rho"]) <= 1e-12 * ref["rho"]
    g1, g2, fg = P.canonical_gauge(res["B1"], res["B2"])
    r1, r2, fr = P.canonical_gauge(ref["B1"], ref["B2"])
    assert np.array_equal(g1, r1), "B1 differs in %d entries" % int((g1 != r1).sum())
    assert np.array_equal(g2, r2), "B2 differs in %d entries" % int((g2 != r2).sum())
    for name in ("alpha", "beta", "gamma"):
        assert rel(res[name], ref[name]) <= TOL_REAL, (name, rel(res[name], ref[name]))
    n = ref["sweeps"]
    assert np.max(np.abs(info[8:8 + n] - ref["objective"])) <= TOL_OBJ * info[3]
    assert np.all(info[8 + n:] == 0.0)
    if check_iterates:
        assert rel(res["U1"] * fg[None, :], ref["U1"] * fr[None, :]) <= TOL_REAL
        assert rel(res["U2t"] * fg[None, :], ref["U2"].T * fr[None, :]) <= TOL_REAL
    # the fp16 scales are the fp64 ones rounded to nearest (one rounding)
    for h, f in (("s_in", "alpha"), ("s_rank", "beta"), ("s_out", "gamma")):
        assert np.array_equal(res[h], res[f].astype(np.float16))


SHAPES = [
    # seed, N, M, R, r0
    (0, 64, 48, 4, 8),
    (1, 200, 136, 8, 8),
    (2, 130, 257, 16, 16),       # ragged row blocks on both sides
    (3, 96, 80, 5, 7),           # odd ranks
    (4, 70, 500, 1, 3),          # one rank-one term
    (5, 320, 192, 32, 40),       # the largest carrier rank, 32 lanes per row
    (6, 512, 512, 16, 16),
    (7, 33, 40, 24, 24),         # fewer rows than one block
    (8, 640, 384, 8, 64),        # the largest factor rank
    (9, 2048, 2048, 16, 16),     # a quarter of the benchmark's projection: the dense oracle takes about 10 s
    (10, 1100, 4096, 16, 16),    # one side at the benchmark's width, ragged on the other
    (12, 200, 150, 32, 64),      # both ranks at their limits
    (13, 150, 70, 17, 33),       # just past the 16-lane / 16-entry instantiation
    (11, 4096, 4096, 16, 16),    # the benchmark's projection (the dense oracle: about 10 s on the GPU machine's host, 40 s on 8 cores)
]


@pytest.mark.parametrize("seed,N,M,R,r0", SHAPES)
def test_full_run_matches_oracle(torch_cuda, seed, N, M, R, r0):
    say("ptq full run seed=%d N=%d M=%d R=%d r0=%d" % (seed, N, M, R, r0))
    d = inputs.make_ptq_inputs(seed, N, M, r0)
    K = 100
    ref = P.ptq(d["A_star"], d["B_star"], R, K=K)
    res = run_gpu(torch_cuda, d, R, K=K)
    compare(res, ref, K)


@pytest.mark.parametrize("K", [1, 2, 3, 7])
def test_first_sweeps_match_oracle(torch_cuda, K):
    # a run of K sweeps (its penalty window is the first half of those K) pins every update of the early sweeps
    say("ptq first sweeps K=%d" % K)
    d = inputs.make_ptq_inputs(11, 150, 210, 16)
    ref = P.ptq(d["A_star"], d["B_star"], 12, K=K)
    res = run_gpu(torch_cuda, d, 12, K=K)
    compare(res, ref, K)


@pytest.mark.parametrize("tau,mu", [(2.0, 10.0), (1.5, 3.0), (4.0, 1.0)])
def test_other_balancing_constants(torch_cuda, tau, mu):
    say("ptq balancing tau=%g mu=%g" % (tau, mu))
    d = inputs.make_ptq_inputs(12, 160, 128, 8)
    ref = P.ptq(d["A_star"], d["B_star"], 8, K=40, tau=tau, mu=mu)
    res = run_gpu(torch_cuda, d, 8, K=40, tau=tau, mu=mu)
    compare(res, ref, 40)


def test_flat_spectrum_and_large_entries(torch_cuda):
    # no decay of the factor columns (close singular values) and entries near the top of the fp16 range of a weight update
    say("ptq flat spectrum")
    d = inputs.make_ptq_inputs(13, 256, 192, 8, decay=1.0)
    d["A_star"] = (d["A_star"].astype(np.float32) * 40).astype(np.float16)
    ref = P.ptq(d["A_star"], d["B_star"], 6, K=60)
    res = run_gpu(torch_cuda, d, 6, K=60)
    compare(res, ref, 60)


@pytest.mark.parametrize("case", ["padded", "dependent", "few_rows", "both_sides"])
def test_rank_deficient_factors(torch_cuda, case):
    # factors without full column rank (an adapter padded with dead columns, a repeated column, fewer rows than
    # columns): their triangular factors are singular, which the warm start must not mind; the update still has rank >= R
    say("ptq rank-deficient factors: " + case)
    if case == "padded":
        d = inputs.make_ptq_inputs(30, 180, 140, 12)
        d["A_star"][:, 9:] = 0
        R = 8
    elif case == "dependent":
        d = inputs.make_ptq_inputs(31, 150, 200, 10)
        d["B_star"][:, 7] = d["B_star"][:, 2]
        R = 6
    elif case == "few_rows":
        d = inputs.make_ptq_inputs(32, 5, 90, 8)
        R = 4
    else:
        d = inputs.make_ptq_inputs(33, 120, 130, 16)
        d["A_star"][:, 12:] = 0
        d["B_star"][:, :2] = 0
        R = 10
    ref = P.ptq(d["A_star"], d["B_star"], R, K=50)
    res = run_gpu(torch_cuda, d, R, K=50)
    compare(res, ref, 50)


# Spectra that fall by many orders of magnitude within the first R singular values (column k of A_star damped by 0.6^k or
# 0.55^k; the last columns underflow to zero in fp16).  The trailing singular vectors of the warm start (Eq. (svd-init)) are
# then resolved to about eps sigma_1 / sigma_R by a dense decomposition, and the device must do as well: a route through the
# Gram matrices of the factors would square that ratio and give a few near-zero entries of the trailing carriers the
# other sign (the first case once differed in 9 of its 16 037 signs that way).
ILL_CONDITIONED = [
    # seed, N, M, R, r0, K, decay     sigma_R / sigma_1
    (1056, 259, 294, 29, 36, 100, 0.6),    # 5e-7
    (1057, 250, 221, 27, 40, 30, 0.6),     # 1e-6
    (1076, 141, 215, 24, 35, 2, 0.6),      # 7e-6
    (1090, 300, 280, 24, 40, 100, 0.55),
    (1091, 700, 520, 32, 64, 40, 0.7),     # several QR panels per side, both ranks at their limits
]


@pytest.mark.parametrize("seed,N,M,R,r0,K,decay", ILL_CONDITIONED)
def test_ill_conditioned_spectrum_matches_dense_svd(torch_cuda, seed, N, M, R, r0, K, decay):
    say("ptq steep spectrum seed=%d N=%d M=%d R=%d r0=%d K=%d decay=%g" % (seed, N, M, R, r0, K, decay))
    d = inputs.make_ptq_inputs(seed, N, M, r0, decay=decay)
    T = d["A_star"].astype(np.float64) @ d["B_star"].astype(np.float64).T
    sv = np.linalg.svd(T, compute_uv=False)
    say("  sigma_R / sigma_1 = %.1e" % (sv[R - 1] / sv[0]))
    assert 1e-9 < sv[R - 1] / sv[0] < 1e-3
    ref = P.ptq(d["A_star"], d["B_star"], R, K=K)
    res = run_gpu(torch_cuda, d, R, K=K)
    compare(res, ref, K)


def test_warm_start_alone_on_tall_factors(torch_cuda):
    """K = 1 on tall factors (thousands of rows: several levels of QR panels): after one sweep every sign still agrees."""
    say("ptq warm start, tall factors")
    for seed, N, M, R, r0, decay in ((40, 3000, 1300, 12, 20, 0.7), (41, 5000, 700, 20, 48, 0.8)):
        d = inputs.make_ptq_inputs(seed, N, M, r0, decay=decay)
        ref = P.ptq(d["A_star"], d["B_star"], R, K=1)
        res = run_gpu(torch_cuda, d, R, K=1)
        compare(res, ref, 1)


# ---- the rank-scale update on its own (Eq. (beta-gram), Eq. (beta-pinv)): lordba_ptq_beta_solve against the oracle ----

def _beta_system(T, alpha, B1, B2, gamma):
    """G and h of Eq. (beta-gram) written out with numpy (test input for the device routine)."""
    Pm, Q = alpha[:, None] * B1, B2 * gamma[None, :]
    return (Pm.T @ Pm) * (Q @ Q.T), np.sum((Pm.T @ T) * Q, axis=1)


def _planted(seed, N, M, R, kind):
    rng = np.random.default_rng(seed)
    T = rng.standard_normal((N, M))
    alpha, gamma = np.exp(0.3 * rng.standard_normal(N)), np.exp(0.3 * rng.standard_normal(M))
    B1, B2 = P.sgn(rng.standard_normal((N, R))), P.sgn(rng.standard_normal((R, M)))
    if kind == "duplicate pair":          # carrier pair 1 repeats pair 0: G has two equal rows, rank R - 1
        B1[:, 1], B2[1, :] = B1[:, 0], B2[0, :]
    elif kind == "negated pair":          # pair 2 = minus pair 0 on both sides: the same rank-one term again
        B1[:, 2], B2[2, :] = -B1[:, 0], -B2[0, :]
    elif kind == "three copies":          # rank R - 2
        B1[:, 1], B2[1, :] = B1[:, 0], B2[0, :]
        B1[:, R - 1], B2[R - 1, :] = B1[:, 0], B2[0, :]
    elif kind == "dead rows":             # alpha = 0 on most rows: P^T P (a Gram matrix of 3 rows) has rank 3 and
        alpha[3:] = 0.0                   # Q Q^T is made rank 2, so G has rank <= 6 whatever R is
        B2[2:, :] = B2[:2, :][np.arange(R - 2) % 2]
    elif kind == "zero":
        alpha[:] = 0.0
    return T, alpha, B1, B2, gamma


@pytest.mark.parametrize("R", [1, 2, 5, 16, 17, 29, 32])
@pytest.mark.parametrize("kind", ["full rank", "duplicate pair", "negated pair", "three copies", "dead rows", "zero"])
def test_beta_solve_matches_the_oracle_pseudo_inverse(torch_cuda, R, kind):
    torch = torch_cuda
    if R < 3 and kind in ("negated pair", "three copies", "dead rows") or (R == 1 and kind == "duplicate pair"):
        pytest.skip("needs more carrier pairs")
    say("ptq beta solve R=%d %s" % (R, kind))
    T, alpha, B1, B2, gamma = _planted(100 * R + len(kind), 60, 50, R, kind)
    want = P.beta_update(T, alpha, B1, B2, gamma)
    G, h = _beta_system(T, alpha, B1, B2, gamma)
    rank = np.linalg.matrix_rank(G, hermitian=True)
    assert (rank == R) == (kind == "full rank"), (kind, rank)
    got = binding.lordba_ptq_beta_solve(torch.from_numpy(G).cuda(), torch.from_numpy(h).cuda())
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    say("  rank %d of %d, |beta| %.3e, rel err %.1e" % (rank, R, np.linalg.norm(want), rel(got, want) if np.linalg.norm(want) else 0.0))
    if kind == "zero":
        assert np.all(got == 0.0) and np.all(want == 0.0)
    else:
        assert rel(got, want) <= TOL_REAL
        # the solution of least norm among the least-squares solutions: G beta reproduces G pinv(G) h, and beta is in G's range
        assert np.linalg.norm(G @ got - G @ want) <= 1e-8 * np.linalg.norm(G @ want)


def test_carrier_rank_beyond_the_rank_of_the_update_is_flagged(torch_cuda):
    say("ptq R beyond the rank of the update")
    torch = torch_cuda
    d = inputs.make_ptq_inputs(34, 100, 80, 8)
    d["A_star"][:, 3:] = 0                       # the update has rank 3
    out = binding.lordba_ptq(torch.from_numpy(d["A_star"]).cuda(), torch.from_numpy(d["B_star"]).cuda(), 5, K=5)
    torch.cuda.synchronize()
    info = out["info"].cpu().numpy()
    assert info[4] == 1.0 and info[0] == 0.0
    ok = binding.lordba_ptq(torch.from_numpy(d["A_star"]).cuda(), torch.from_numpy(d["B_star"]).cuda(), 3, K=5)
    torch.cuda.synchronize()
    assert ok["info"][4].item() == 0.0


def test_rank_one_target_is_fitted_exactly_and_ends_after_one_sweep(torch_cuda):
    say("ptq rank one")
    d = inputs.make_ptq_inputs(14, 90, 70, 1)
    res = run_gpu(torch_cuda, d, 1, K=10)
    assert int(res["info"][0]) == 1 and res["info"][1] == 1.0
    T = d["A_star"].astype(np.float64) @ d["B_star"].astype(np.float64).T
    W = P.adapter_matrix(res["alpha"], res["B1"], res["beta"], res["B2"], res["gamma"])
    assert np.sum((T - W) ** 2) <= 1e-20 * np.sum(T * T)


def test_exported_adapter_runs_in_the_forward_kernel(torch_cuda):
    # the packed carriers and fp16 scales go straight into lordba_forward: y = x DeltaW(theta) with d_in = N, d_out = M
    say("ptq export -> forward")
    torch = torch_cuda
    N, M, R = 256, 192, 8
    d = inputs.make_ptq_inputs(15, N, M, 8)
    A, B = torch.from_numpy(d["A_star"]).cuda(), torch.from_numpy(d["B_star"]).cuda()
    out = binding.lordba_ptq(A, B, R, K=30)
    act = inputs.make_activations(15, 40, N, M)
    x, yb = torch.from_numpy(act["x"]).cuda(), torch.zeros(40, M, dtype=torch.float16, device="cuda:0")
    y = binding.lordba_forward(x, out["packedA"], out["packedB"], out["s_in"], out["s_rank"], out["s_out"], yb)
    torch.cuda.synchronize()
    sA, sB = binding.lordba_unpack_signs(out["packedA"].cpu().numpy().view(np.uint32), out["packedB"].cpu().numpy().view(np.uint32), N, M, R)
    want = oracle.forward(act["x"], sA, sB, out["s_in"].cpu().numpy(), out["s_rank"].cpu().numpy(), out["s_out"].cpu().numpy(),
                          np.zeros((40, M), dtype=np.float16))
    got = y.cpu().numpy().astype(np.float64)
    err = np.linalg.norm(got - want, axis=1) / np.maximum(np.linalg.norm(want, axis=1), 1e-30)
    assert err.max() <= 1e-3
    # and the adapter it describes is the fitted one: relative error of the fit below that of a zero adapter
    T = d["A_star"].astype(np.float64) @ d["B_star"].astype(np.float64).T
    W = P.adapter_matrix(out["alpha"].cpu().numpy(), sA.T.astype(np.float64), out["beta"].cpu().numpy(), sB.T.astype(np.float64),
                         out["gamma"].cpu().numpy())
    assert np.sum((T - W) ** 2) < 0.8 * np.sum(T * T)


def test_quantised_adapter_trains_with_frozen_carriers(torch_cuda):
    # the "freeze" training variant (Sec. 3.2, optional variants): carriers from post-training quantisation stay fixed, only
    # the scales get gradients.  lordba_ptq -> lordba_forward_save_t -> lordba_backward without latents, against the
    # backward oracle fed the same carriers and fp16 scales.
    say("ptq -> forward -> backward with frozen carriers")
    torch = torch_cuda
    N, M, R, T = 256, 192, 8, 70
    d = inputs.make_ptq_inputs(21, N, M, 8)
    q = binding.lordba_ptq(torch.from_numpy(d["A_star"]).cuda(), torch.from_numpy(d["B_star"]).cuda(), R, K=30)
    torch.cuda.synchronize()
    sA, sB = binding.lordba_unpack_signs(q["packedA"].cpu().numpy().view(np.uint32), q["packedB"].cpu().numpy().view(np.uint32), N, M, R)
    pAt, pBt = binding.lordba_pack_transposed(sA, sB)
    cu = lambda a_: torch.from_numpy(np.ascontiguousarray(a_)).cuda()
    b = inputs.make_backward_inputs(21, T, N, M, R)
    x, g, yb, dxb = cu(b["x"]), cu(b["g"]), cu(b["y_base"]), cu(b["dx_base"])
    y, t_kept = binding.lordba_forward_save_t(x, q["packedA"], q["packedB"], q["s_in"], q["s_rank"], q["s_out"], yb)
    got = binding.lordba_backward(x, g, q["packedA"], cu(pAt.view(np.int32)), cu(pBt.view(np.int32)), q["s_in"], q["s_rank"], q["s_out"],
                                  None, None, 100.0, dx_base=dxb, t_saved=t_kept)
    torch.cuda.synchronize()
    s_in, s_rank, s_out = (q[k].cpu().numpy() for k in ("s_in", "s_rank", "s_out"))
    want_y = oracle.forward(b["x"], sA, sB, s_in, s_rank, s_out, b["y_base"])
    assert oracle.row_rel_l2(y.cpu().numpy().astype(np.float64), want_y).max() <= 1e-3
    want = oracle.backward(b["x"], b["g"], sA, sB, s_in, s_rank, s_out, b["latA"], b["latB"], 100.0, b["dx_base"])
    assert oracle.row_rel_l2(got["dx"].cpu().numpy().astype(np.float64), want["dx"]).max() <= 1e-3
    for k in ("d_s_in", "d_s_rank", "d_s_out"):
        assert oracle.rel_l2(got[k].cpu().numpy(), want[k]) <= 1e-3, k
    assert got["d_latentA"] is None and got["d_latentB"] is None


def test_calls_are_reproducible_and_reuse_a_workspace(torch_cuda):
    say("ptq reproducible")
    torch = torch_cuda
    d = inputs.make_ptq_inputs(16, 300, 260, 16)
    A, B = torch.from_numpy(d["A_star"]).cuda(), torch.from_numpy(d["B_star"]).cuda()
    ws = torch.full((binding.lordba_ptq_workspace_bytes(300, 260, 16, 16) // 8,), float("nan"), dtype=torch.float64, device="cuda:0")
    a = binding.lordba_ptq(A, B, 16, K=50, workspace=ws)
    torch.cuda.synchronize()
    first = {k: v.clone() for k, v in a.items() if k != "workspace"}
    # a smaller problem in the same workspace, then the first one again
    d2 = inputs.make_ptq_inputs(17, 100, 90, 8)
    binding.lordba_ptq(torch.from_numpy(d2["A_star"]).cuda(), torch.from_numpy(d2["B_star"]).cuda(), 4, K=20, workspace=ws)
    b = binding.lordba_ptq(A, B, 16, K=50, workspace=ws)
    torch.cuda.synchronize()
    for k in first:
        assert torch.equal(first[k], b[k]) or (first[k].dtype.is_floating_point and
                                               torch.equal(torch.nan_to_num(first[k]), torch.nan_to_num(b[k]))), k


def test_a_run_enqueued_in_pieces_is_the_same_run(torch_cuda):
    # lordba_ptq_sweeps: [0, 5) + [5, 6) + [6, 40) against one call of 40 sweeps, bit for bit; the outputs after the first
    # piece are those of the run stopped there (same penalty schedule: K stays 40)
    say("ptq in pieces")
    torch = torch_cuda
    d = inputs.make_ptq_inputs(22, 180, 150, 16)
    A, B = torch.from_numpy(d["A_star"]).cuda(), torch.from_numpy(d["B_star"]).cuda()
    whole = binding.lordba_ptq(A, B, 10, K=40)
    part = binding.lordba_ptq(A, B, 10, K=40, sweeps=(0, 5))
    torch.cuda.synchronize()
    info5 = part["info"].cpu().numpy().copy()
    assert info5[0] == 5.0 and info5[1] == 0.0 and np.all(info5[8:13] != 0.0) and np.all(info5[13:] == 0.0)
    ref = P.ptq(d["A_star"], d["B_star"], 10, K=40, trace=(tr := []))
    assert rel(part["alpha"].cpu().numpy(), tr[4]["alpha"]) <= TOL_REAL and abs(info5[2] - tr[4]["rho"]) <= 1e-12 * tr[4]["rho"]
    binding.lordba_ptq(A, B, 10, K=40, sweeps=(5, 6), out=part)
    binding.lordba_ptq(A, B, 10, K=40, sweeps=(6, 40), out=part)
    torch.cuda.synchronize()
    for k in ("packedA", "packedB", "alpha", "beta", "gamma", "s_in", "s_rank", "s_out", "info", "U1", "U2t"):
        assert torch.equal(part[k], whole[k]), k
    assert int(whole["info"][0].item()) == ref["sweeps"]


def test_graph_replay_matches_eager(torch_cuda):
    # a warmed-up call only launches kernels (no clearing by memset, no allocation, no wait): it can be captured; replays,
    # with eager work of the same library in between, must give the eager result bit for bit
    say("ptq graph replay")
    torch = torch_cuda
    d = inputs.make_ptq_inputs(19, 260, 200, 16)
    A, B = torch.from_numpy(d["A_star"]).cuda(), torch.from_numpy(d["B_star"]).cuda()
    ws = torch.empty(binding.lordba_ptq_workspace_bytes(260, 200, 12, 16) // 8, dtype=torch.float64, device="cuda:0")
    eager = binding.lordba_ptq(A, B, 12, K=30, workspace=ws)
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in eager.items() if k != "workspace"}
    import ctypes
    lib = binding.load_library()
    outs = ("packedA", "packedB", "alpha", "beta", "gamma", "s_in", "s_rank", "s_out", "info")

    def scrub(held):
        for k in outs:
            held[k].fill_(float("nan")) if held[k].dtype.is_floating_point else held[k].fill_(-1)

    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        held = binding.lordba_ptq(A, B, 12, K=30, workspace=ws, stream=side)     # allocates the outputs outside the capture
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            st = lib.lordba_ptq(A.data_ptr(), B.data_ptr(), held["packedA"].data_ptr(), held["packedB"].data_ptr(), held["alpha"].data_ptr(),
                                held["beta"].data_ptr(), held["gamma"].data_ptr(), held["s_in"].data_ptr(), held["s_rank"].data_ptr(),
                                held["s_out"].data_ptr(), held["info"].data_ptr(), ws.data_ptr(), ws.numel() * 8, 260, 200, 12, 16, 30, 2.0, 10.0,
                                ctypes.c_void_p(side.cuda_stream))
            assert st == 0
    for rep in range(3):
        scrub(held)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(held[k], want[k]), (rep, k)
        # eager work between the replays: another problem in the same workspace
        d2 = inputs.make_ptq_inputs(20 + rep, 100, 90, 8)
        binding.lordba_ptq(torch.from_numpy(d2["A_star"]).cuda(), torch.from_numpy(d2["B_star"]).cuda(), 4, K=10, workspace=ws)
        torch.cuda.synchronize()


def test_degenerate_input_is_flagged(torch_cuda):
    say("ptq degenerate")
    torch = torch_cuda
    A = torch.zeros(64, 4, dtype=torch.float16, device="cuda:0")
    B = torch.ones(48, 4, dtype=torch.float16, device="cuda:0")
    out = binding.lordba_ptq(A, B, 2, K=5)
    torch.cuda.synchronize()
    info = out["info"].cpu().numpy()
    assert info[4] == 1.0 and info[0] == 0.0


def test_full_size_properties(torch_cuda):
    """The benchmark's shape (4096 x 4096, R = r0 = 16, K = 100), where the oracle takes minutes: what can be checked
    from the outputs alone, with the dense target formed on the host.  Every scale is the least-squares optimum for the
    returned continuous iterates in turn (beta last, so beta's normal equations hold exactly; alpha's and gamma's held
    before beta moved), the reported objective is the dense one, and the sign matrices are those of the iterates."""
    say("ptq full size 4096x4096 R=16")
    torch = torch_cuda
    N = M = 4096
    R = r0 = 16
    d = inputs.make_ptq_inputs(18, N, M, r0)
    res = run_gpu(torch, d, R, K=100)
    info = res["info"]
    n = int(info[0])
    assert info[4] == 0.0 and 1 <= n <= 100
    T = d["A_star"].astype(np.float64) @ d["B_star"].astype(np.float64).T
    assert abs(info[3] - np.sum(T * T)) <= 1e-12 * np.sum(T * T)
    U1, U2 = res["U1"], res["U2t"].T
    f = P.objective(T, res["alpha"], U1, res["beta"], U2, res["gamma"])
    assert abs(f - info[8 + n - 1]) <= TOL_OBJ * info[3]
    want_beta = P.beta_update(T, res["alpha"], U1, U2, res["gamma"])
    assert rel(res["beta"], want_beta) <= TOL_REAL
    # sampled rows of U1 / columns of U2 are +-1 patterns consistent with the packed carriers where the margin is clear
    assert np.all(np.abs(res["B1"]) == 1) and np.all(np.abs(res["B2"]) == 1)
    if info[1] == 1.0:
        # after the loop ended on repeated signs the continuous iterates sit on the side of their signs
        far = np.abs(U1) > 0.5
        assert np.mean(np.sign(U1[far]) == res["B1"][far]) > 0.99
