"""GPU parity of the branch's backward pass (lordba_backward, through the C ABI) against the fp64 CPU oracle on the
same seeded inputs.  Bar (fp16 activations, fp32 accumulation): relative L2 error <= 1e-3
  * per token row for dx (as configured, and with dx_base = 0 so that the branch's share cannot hide),
  * over the whole vector for d_s_in, d_s_rank, d_s_out,
  * per rank for the latent gradients (row k of d_latentA [r, d_in], column k of d_latentB [d_out, r]).
"""
import sys

import numpy as np
import pytest

import oracle
from paper_2605_24058_amd import binding, inputs

pytestmark = pytest.mark.gpu

TOL = 1e-3
KAPPA = 100.0


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


GUARD = 4096


def new_workspace(torch, nbytes, fill=0xFF):
    """nbytes of workspace followed by a guard band, all set to `fill`."""
    return torch.full((nbytes + GUARD,), fill, dtype=torch.uint8, device="cuda:0")


def gpu_backward(torch, d, kappa=KAPPA, with_dx=True, inplace=False, ws=None, ws_bytes=None, keep_t=False):
    """Runs the library on cuda:0.  ws: a buffer from new_workspace (its last GUARD bytes must stay untouched); by default
    a fresh poisoned one of exactly the size the library asks for: the call must not depend on the workspace's contents
    nor write past it.  ws_bytes: the size reported to the library (default: everything before the guard band)."""
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    pA, _ = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    pAt, pBt = binding.lordba_pack_transposed(d["signsA"], d["signsB"])
    T, d_in = d["x"].shape
    d_out, r = d["signsB"].shape
    if ws is None:
        ws = new_workspace(torch, binding.lordba_backward_workspace_bytes(T, d_in, d_out, r))
    fill = int(ws[-1].item())
    usable = ws.numel() - GUARD if ws_bytes is None else ws_bytes
    dxb = cu(d["dx_base"]) if with_dx else None
    t_saved = None
    if keep_t:  # the rank-r intermediate kept by the training forward pass instead of a second pass over x
        _, pB = binding.lordba_pack_signs(d["signsA"], d["signsB"])
        stride = binding.saved_t_stride(T)
        t_saved = torch.full((r, stride), float("nan"), dtype=torch.float32, device="cuda:0")
        binding.lordba_forward_save_t(cu(d["x"]), cu(pA.view(np.int32)), cu(pB.view(np.int32)), cu(d["s_in"]), cu(d["s_rank"]),
                                      cu(d["s_out"]), cu(d["y_base"]), t_out=t_saved)
    out = binding.lordba_backward(cu(d["x"]), cu(d["g"]), cu(pA.view(np.int32)), cu(pAt.view(np.int32)), cu(pBt.view(np.int32)),
                                  cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]), cu(d["latA"]), cu(d["latB"]), kappa,
                                  dx_base=dxb, dx=dxb if inplace else None, workspace=ws[:usable], t_saved=t_saved)
    torch.cuda.synchronize()
    assert (ws[ws.numel() - GUARD:].cpu().numpy() == fill).all(), "write past the workspace"
    return {k: (None if v is None else v.cpu().numpy()) for k, v in out.items()}


def oracle_backward(d, kappa=KAPPA, with_dx=True):
    return oracle.backward(d["x"], d["g"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["latA"], d["latB"],
                           kappa, d["dx_base"] if with_dx else None)


def compare(got, want, label, with_dx=True):
    worst = {}
    if with_dx:
        e = oracle.row_rel_l2(got["dx"].astype(np.float64), want["dx"])
        assert e.max() <= TOL, "%s dx: max row rel-L2 %.3e at row %d" % (label, e.max(), e.argmax())
        worst["dx"] = e.max()
    for k in ("d_s_in", "d_s_rank", "d_s_out"):
        assert np.isfinite(got[k]).all(), "%s %s: non-finite" % (label, k)
        e = oracle.rel_l2(got[k], want[k])
        assert e <= TOL, "%s %s: rel-L2 %.3e" % (label, k, e)
        worst[k] = e
    eA = oracle.row_rel_l2(got["d_latentA"].astype(np.float64), want["d_latA"])
    assert eA.max() <= TOL, "%s d_latentA: max rel-L2 %.3e at rank %d" % (label, eA.max(), eA.argmax())
    eB = oracle.row_rel_l2(got["d_latentB"].astype(np.float64).T, want["d_latB"].T)
    assert eB.max() <= TOL, "%s d_latentB: max rel-L2 %.3e at rank %d" % (label, eB.max(), eB.argmax())
    worst["d_latentA"], worst["d_latentB"] = eA.max(), eB.max()
    say("  %s: " % label + " ".join("%s %.2e" % kv for kv in worst.items()))
    return worst


def check(torch, d, label, kappa=KAPPA, dx_subnormal=False):
    say("  case %s" % label)
    got = gpu_backward(torch, d, kappa)
    compare(got, oracle_backward(d, kappa), label)
    # the branch's share of dx alone
    dd = dict(d, dx_base=np.zeros_like(d["dx_base"]))
    got0 = gpu_backward(torch, dd, kappa)
    want0 = oracle_backward(dd, kappa)["dx"]
    if dx_subnormal:
        # the branch's share lies below the smallest normal fp16 (2^-14), where the output format itself has an absolute
        # spacing of 2^-24: the bar is one such step
        assert np.abs(want0).max() < 2.0 ** -14
        assert np.abs(got0["dx"].astype(np.float64) - want0).max() <= 2.0 ** -24, label
    else:
        e = oracle.row_rel_l2(got0["dx"].astype(np.float64), want0)
        assert e.max() <= TOL, "%s dx (branch alone): %.3e" % (label, e.max())
    for k in ("d_s_in", "d_s_rank", "d_s_out", "d_latentA", "d_latentB"):
        assert np.array_equal(got[k], got0[k]), "%s: %s depends on dx_base" % (label, k)


# (T, d_in, d_out, r): several tiles of 8 rows and a ragged last one, 128-column blocks with a tail (d = 32 * odd),
# every rank-block count, T below one tile and below one 32-row step
SHAPES = [
    (64, 512, 512, 4),        # the small benchmark configuration
    (37, 1024, 1152, 16),
    (1, 512, 384, 16),
    (8, 256, 256, 8),
    (203, 1056, 2080, 16),    # 33 and 65 words per carrier row: partial last column blocks
    (70, 1024, 768, 32),
    (45, 640, 1024, 48),
    (33, 512, 1024, 64),
    (130, 32, 96, 5),         # the smallest widths, a rank that is not a multiple of 8
    (519, 2048, 1536, 16),    # several 32-row steps per wave
    # widths that are no multiples of 32: the general (vector ALU) kernel, as in the forward pass
    (7, 100, 60, 5),
    (9, 100, 36, 5),
    (50, 33, 17, 3),
    (130, 96, 40, 17),        # only d_out is odd
    (64, 72, 64, 8),          # only d_in is odd
    (21, 200, 136, 33),
    (12, 80, 48, 64),
    (1, 40, 24, 16),
    (300, 1000, 520, 16),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "T%d_%dx%d_r%d" % s)
def test_small_shapes_all_outputs(torch_cuda, shape):
    T, d_in, d_out, r = shape
    d = inputs.make_backward_inputs(21, T, d_in, d_out, r)
    check(torch_cuda, d, "T%d_%dx%d_r%d" % shape)


def test_sixteen_row_tiles(torch_cuda):
    """T >= 4096 takes 16-row tiles in the rank kernel; ragged last tile."""
    d = inputs.make_backward_inputs(22, 4100, 256, 384, 16)
    check(torch_cuda, d, "T4100_256x384_r16")
    d = inputs.make_backward_inputs(23, 4133, 512, 256, 32)
    check(torch_cuda, d, "T4133_512x256_r32")


@pytest.mark.parametrize("g_scale", [2.0 ** -14, 2.0 ** -7, 16.0])
def test_gradient_magnitudes(torch_cuda, g_scale):
    """Upstream gradients far from 1 (loss-scaled or tiny): the per-rank power-of-two scaling keeps the precision."""
    d = inputs.make_backward_inputs(24, 100, 1024, 512, 16, g_scale=g_scale)
    check(torch_cuda, d, "g_scale_%g" % g_scale, dx_subnormal=g_scale < 2.0 ** -10)


def test_uneven_rank_scales(torch_cuda):
    """Rank scales spread over many orders of magnitude, a zero (how extra envelopes start) and negative ones."""
    d = inputs.make_backward_inputs(25, 96, 512, 768, 16)
    s = d["s_rank"].astype(np.float32)
    s *= np.array([1, -1, 2.0 ** -10, 2.0 ** 6, 0, 1, -2.0 ** -12, 1, 1, 64, 1, -1, 2.0 ** -8, 1, 1, 3], dtype=np.float32)
    d["s_rank"] = s.astype(np.float16)
    got = gpu_backward(torch_cuda, d)
    want = oracle_backward(d)
    compare(got, want, "uneven_rank_scales")
    assert not got["d_latentA"][4].any() and not got["d_latentB"][:, 4].any()   # beta_4 = 0: exact zeros
    assert got["d_s_rank"][4] != 0


@pytest.mark.parametrize("kappa", [0.0, 1.0, 25.0, 400.0])
def test_temperatures(torch_cuda, kappa):
    d = inputs.make_backward_inputs(26, 50, 512, 512, 8)
    got = gpu_backward(torch_cuda, d, kappa)
    compare(got, oracle_backward(d, kappa), "kappa_%g" % kappa)
    if kappa == 0.0:
        assert not got["d_latentA"].any() and not got["d_latentB"].any()


def test_without_input_gradient_and_in_place(torch_cuda):
    d = inputs.make_backward_inputs(27, 77, 768, 512, 16)
    want = oracle_backward(d)
    got = gpu_backward(torch_cuda, d, with_dx=False)
    assert got["dx"] is None
    compare(got, want, "no_dx", with_dx=False)
    got_ip = gpu_backward(torch_cuda, d, inplace=True)
    compare(got_ip, want, "dx_in_place")


def test_deterministic_and_workspace_reuse(torch_cuda):
    """The result does not depend on what the workspace held; two calls in a row on one workspace, the second on a
    smaller shape, give what fresh workspaces give, bit for bit."""
    torch = torch_cuda
    big = inputs.make_backward_inputs(28, 300, 1024, 1024, 32)
    small = inputs.make_backward_inputs(29, 40, 512, 256, 8)
    need = binding.lordba_backward_workspace_bytes(300, 1024, 1024, 32)
    assert 0 < binding.lordba_backward_workspace_bytes(40, 512, 256, 8) <= need
    a1 = gpu_backward(torch, big)
    a2 = gpu_backward(torch, big, ws=new_workspace(torch, need, fill=0x00))
    shared = new_workspace(torch, need, fill=0x7F)
    a3 = gpu_backward(torch, big, ws=shared)
    s2 = gpu_backward(torch, small, ws=shared)          # right after, on the same (now used) buffer
    s1 = gpu_backward(torch, small)
    for k in a1:
        assert np.array_equal(a1[k], a2[k]) and np.array_equal(a1[k], a3[k]), k
        assert np.array_equal(s1[k], s2[k]), k
    compare(s2, oracle_backward(small), "small_after_big")


@pytest.mark.parametrize("shape", [(9, 100, 36, 5), (3, 513, 77, 16), (3, 512, 384, 16), (20, 4096, 4096, 64)],
                         ids=lambda s: "T%d_%dx%d_r%d" % s)
def test_forward_that_keeps_t_other_kernels(torch_cuda, shape):
    """The same export through the general kernel (unaligned widths) and through the small-T grid modes (a single partial
    tile; a few tiles whose output blocks are split over workgroups, each of which writes the same t)."""
    torch = torch_cuda
    T, d_in, d_out, r = shape
    d = inputs.make_inputs(37, T, d_in, d_out, r)
    dev = binding.to_device(d)
    y_ref = binding.lordba_forward(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"], dev["y_base"])
    t_buf = torch.full((r, binding.saved_t_stride(T)), float("nan"), dtype=torch.float32, device="cuda:0")
    y, t = binding.lordba_forward_save_t(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                         dev["y_base"], t_out=t_buf)
    _, t_only = binding.lordba_forward_save_t(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"])
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref)
    th = t.cpu().numpy()
    assert np.isnan(th[:, T:]).all() and np.array_equal(th[:, :T], t_only.cpu().numpy()[:, :T])
    e = oracle.row_rel_l2(th[:, :T].T.astype(np.float64), oracle.rank_intermediate(d["x"], d["signsA"], d["s_in"]))
    assert e.max() <= 1e-5, "t: max row rel-L2 %.3e" % e.max()


@pytest.mark.parametrize("shape", [(37, 1024, 1152, 16), (203, 1056, 2080, 16), (130, 32, 96, 5), (4133, 512, 256, 32), (33, 512, 1024, 64)],
                         ids=lambda s: "T%d_%dx%d_r%d" % s)
def test_forward_that_keeps_t(torch_cuda, shape):
    """lordba_forward_save_t: y_out bit-identical to lordba_forward, t against the oracle, entries past T untouched; the
    t-only call gives the same t; lordba_backward fed with the kept t gives what it gives when it recomputes t."""
    torch = torch_cuda
    T, d_in, d_out, r = shape
    d = inputs.make_backward_inputs(32, T, d_in, d_out, r)
    dev = binding.to_device(d)
    y_ref = binding.lordba_forward(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"], dev["y_base"])
    stride = binding.saved_t_stride(T)
    t_buf = torch.full((r, stride), float("nan"), dtype=torch.float32, device="cuda:0")
    y, t = binding.lordba_forward_save_t(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                         dev["y_base"], t_out=t_buf)
    _, t_only = binding.lordba_forward_save_t(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"])
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref)
    th = t.cpu().numpy()
    assert np.isnan(th[:, T:]).all(), "t written past T"
    assert np.array_equal(th[:, :T], t_only.cpu().numpy()[:, :T])
    want = oracle.rank_intermediate(d["x"], d["signsA"], d["s_in"])
    e = oracle.row_rel_l2(th[:, :T].T.astype(np.float64), want)
    assert e.max() <= 1e-5, "t: max row rel-L2 %.3e" % e.max()
    a = gpu_backward(torch, d)
    b = gpu_backward(torch, d, keep_t=True)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_unaligned_tensors_and_any_kept_t_take_the_general_kernel(torch_cuda):
    """Widths that would fit the matrix-core kernels, but x starts 2 bytes past a 16-byte boundary, or the kept t has a row
    stride of exactly T (no multiple of 4): the call is accepted (as lordba_forward accepts such tensors) and takes the
    general kernel; same bar against the oracle."""
    torch = torch_cuda
    T, d_in, d_out, r = 37, 256, 384, 16
    d = inputs.make_backward_inputs(38, T, d_in, d_out, r)
    want = oracle_backward(d)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    pA, pB = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    pAt, pBt = binding.lordba_pack_transposed(d["signsA"], d["signsB"])
    w = lambda a: cu(a.view(np.int32))
    holder = torch.zeros(T * d_in + 8, dtype=torch.float16, device="cuda:0")
    x_off = holder[1:1 + T * d_in].view(T, d_in)
    x_off.copy_(cu(d["x"]))
    assert x_off.data_ptr() % 16 == 2 and x_off.is_contiguous()
    head = (w(pA), w(pAt), w(pBt), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]), cu(d["latA"]), cu(d["latB"]), KAPPA)
    out = binding.lordba_backward(x_off, cu(d["g"]), *head, dx_base=cu(d["dx_base"]))
    torch.cuda.synchronize()
    compare({k: v.cpu().numpy() for k, v in out.items()}, want, "x two bytes off a 16-byte boundary")
    t_odd = torch.full((r, T), float("nan"), dtype=torch.float32, device="cuda:0")       # row stride 37
    binding.lordba_forward_save_t(cu(d["x"]), w(pA), w(pB), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]), t_out=t_odd)
    out = binding.lordba_backward(cu(d["x"]), cu(d["g"]), *head, dx_base=cu(d["dx_base"]), t_saved=t_odd)
    torch.cuda.synchronize()
    compare({k: v.cpu().numpy() for k, v in out.items()}, want, "kept t with row stride T")


@pytest.mark.parametrize("case", [(2, 203, 1056, 2080, 16), (4, 45, 512, 640, 8), (3, 70, 1024, 768, 16), (2, 4100, 256, 384, 32),
                                  (4, 37, 512, 512, 16), (4, 4133, 512, 256, 16), (3, 70, 1024, 768, 32)],
                         ids=lambda c: "ell%d_T%d_%dx%d_r%d" % c)
def test_several_envelopes_in_one_pass(torch_cuda, case):
    """lordba_backward_multi with the workspace of lordba_backward_multi_workspace_bytes: one wgrad and one finish pass hold
    the partial sums of all envelopes (up to four rank blocks in all; the last case has six and goes envelope by envelope
    whatever the workspace).  Every output against the oracle, and against the envelope-by-envelope result of the same
    library (same sums in another order: 1e-5), with recomputed and with kept t."""
    torch = torch_cuda
    ell, T, d_in, d_out, r = case
    d = inputs.make_backward_inputs(39, T, d_in, d_out, r)
    d.update(inputs.make_envelopes(39, d_in, d_out, r, ell))
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    pA, pB = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    pAt, pBt = binding.lordba_pack_transposed(d["signsA"], d["signsB"])
    w = lambda a: cu(a.view(np.int32))
    small, big = binding.lordba_backward_workspace_bytes(T, d_in, d_out, r), binding.lordba_backward_multi_workspace_bytes(T, d_in, d_out, r, ell)
    one_pass = ell * ((r + 15) // 16) <= 4
    assert big >= small and (big > small) == one_pass
    head = (cu(d["x"]), cu(d["g"]), w(pA), w(pAt), w(pBt), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]), cu(d["latA"]), cu(d["latB"]), KAPPA)
    want = oracle.backward_multi(d["x"], d["g"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["latA"], d["latB"],
                                 KAPPA, d["dx_base"])
    _, t_kept = binding.lordba_forward_multi_save_t(cu(d["x"]), w(pA), w(pB), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]))
    results = {}
    for tag, nbytes, t_saved in (("by_envelope", small, None), ("one_pass", big, None), ("one_pass_kept_t", big, t_kept)):
        ws = new_workspace(torch, nbytes)
        out = binding.lordba_backward_multi(*head, dx_base=cu(d["dx_base"]), workspace=ws[:nbytes], t_saved=t_saved)
        torch.cuda.synchronize()
        assert (ws[nbytes:].cpu().numpy() == 0xFF).all(), "write past the workspace (%s)" % tag
        got = {k: v.cpu().numpy() for k, v in out.items()}
        results[tag] = got
        e = oracle.row_rel_l2(got["dx"].astype(np.float64), want["dx"])
        assert e.max() <= TOL, "%s dx: %.3e" % (tag, e.max())
        for k in ("d_s_in", "d_s_rank", "d_s_out"):
            for en in range(ell):
                assert oracle.rel_l2(got[k][en], want[k][en]) <= TOL, (tag, k, en)
        assert oracle.row_rel_l2(got["d_latentA"].astype(np.float64), want["d_latA"]).max() <= TOL, tag
        assert oracle.row_rel_l2(got["d_latentB"].astype(np.float64).T, want["d_latB"].T).max() <= TOL, tag
    for k in ("d_s_in", "d_s_rank", "d_s_out", "d_latentA", "d_latentB"):
        a, b = results["by_envelope"][k].astype(np.float64), results["one_pass"][k].astype(np.float64)
        assert np.linalg.norm(a - b) <= 1e-5 * np.linalg.norm(a), k
        assert np.array_equal(results["one_pass"][k], results["one_pass_kept_t"][k]), k   # a kept t is the recomputed one, bit for bit
    assert np.array_equal(results["by_envelope"]["dx"], results["one_pass"]["dx"])


def test_frozen_carriers_scale_gradients_only(torch_cuda):
    """latentA = latentB = None (only the scales are trained): the scale gradients and dx are bit-identical to the full
    call's, and no latent gradient is produced."""
    torch = torch_cuda
    T, d_in, d_out, r = 150, 768, 1024, 16
    d = inputs.make_backward_inputs(35, T, d_in, d_out, r)
    full = gpu_backward(torch, d)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    pA, _ = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    pAt, pBt = binding.lordba_pack_transposed(d["signsA"], d["signsB"])
    w = lambda a: cu(a.view(np.int32))
    out = binding.lordba_backward(cu(d["x"]), cu(d["g"]), w(pA), w(pAt), w(pBt), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]),
                                  None, None, 0.0, dx_base=cu(d["dx_base"]))
    torch.cuda.synchronize()
    assert out["d_latentA"] is None and out["d_latentB"] is None
    for k in ("dx", "d_s_in", "d_s_rank", "d_s_out"):
        assert np.array_equal(out[k].cpu().numpy(), full[k]), k


@pytest.mark.parametrize("case", [(2, 203, 1056, 2080, 16), (3, 70, 1024, 768, 32), (4, 45, 512, 640, 8), (2, 4100, 256, 384, 16),
                                  (1, 37, 512, 512, 16), (3, 21, 100, 60, 5), (4, 33, 72, 200, 16)],   # the last two: general kernel
                         ids=lambda c: "ell%d_T%d_%dx%d_r%d" % c)
def test_several_envelopes(torch_cuda, case):
    """lordba_backward_multi against the oracle: per-envelope scale gradients (whole vector each), dx per token row (as
    configured and the branch alone), latent gradients per rank."""
    torch = torch_cuda
    ell, T, d_in, d_out, r = case
    d = inputs.make_backward_inputs(36, T, d_in, d_out, r)
    d.update(inputs.make_envelopes(36, d_in, d_out, r, ell))
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    pA, _ = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    pAt, pBt = binding.lordba_pack_transposed(d["signsA"], d["signsB"])
    w = lambda a: cu(a.view(np.int32))
    for tag, dxb in (("full", d["dx_base"]), ("branch", np.zeros_like(d["dx_base"]))):
        ws = new_workspace(torch, binding.lordba_backward_workspace_bytes(T, d_in, d_out, r))
        out = binding.lordba_backward_multi(cu(d["x"]), cu(d["g"]), w(pA), w(pAt), w(pBt), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]),
                                            cu(d["latA"]), cu(d["latB"]), KAPPA, dx_base=cu(dxb), workspace=ws[:ws.numel() - GUARD])
        torch.cuda.synchronize()
        assert (ws[ws.numel() - GUARD:].cpu().numpy() == 0xFF).all(), "write past the workspace"
        got = {k: v.cpu().numpy() for k, v in out.items()}
        want = oracle.backward_multi(d["x"], d["g"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["latA"], d["latB"],
                                     KAPPA, dxb)
        e = oracle.row_rel_l2(got["dx"].astype(np.float64), want["dx"])
        assert e.max() <= TOL, "%s dx: %.3e" % (tag, e.max())
        for k in ("d_s_in", "d_s_rank", "d_s_out"):
            for en in range(ell):
                err = oracle.rel_l2(got[k][en], want[k][en])
                assert err <= TOL, "%s envelope %d: %.3e" % (k, en, err)
        assert oracle.row_rel_l2(got["d_latentA"].astype(np.float64), want["d_latA"]).max() <= TOL
        assert oracle.row_rel_l2(got["d_latentB"].astype(np.float64).T, want["d_latB"].T).max() <= TOL
    # the training forward of the same adapter keeps t of every envelope: y against the oracle, t against the oracle,
    # and the backward pass fed with it gives the same bits as the one that recomputes it
    _, pB = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    t_buf = torch.full((ell, r, binding.saved_t_stride(T)), float("nan"), dtype=torch.float32, device="cuda:0")
    y, t_kept = binding.lordba_forward_multi_save_t(cu(d["x"]), w(pA), w(pB), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]),
                                                    cu(d["y_base"]), t_out=t_buf)
    kept = binding.lordba_backward_multi(cu(d["x"]), cu(d["g"]), w(pA), w(pAt), w(pBt), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]),
                                         cu(d["latA"]), cu(d["latB"]), KAPPA, dx_base=cu(np.zeros_like(d["dx_base"])), t_saved=t_kept,
                                         workspace=ws[:ws.numel() - GUARD])   # (the same envelope-by-envelope mode as above)
    torch.cuda.synchronize()
    ywant = oracle.forward_multi(d["x"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["y_base"])
    assert oracle.row_rel_l2(y.cpu().numpy().astype(np.float64), ywant).max() <= TOL
    th = t_kept.cpu().numpy()
    assert np.isnan(th[:, :, T:]).all()
    for en in range(ell):
        twant = oracle.rank_intermediate(d["x"], d["signsA"], d["s_in"][en])
        assert oracle.row_rel_l2(th[en, :, :T].T.astype(np.float64), twant).max() <= 1e-5
    for k, v in kept.items():
        assert np.array_equal(v.cpu().numpy(), got[k]), k


def test_hip_graph_replays_match_eager(torch_cuda):
    """bench.py replays a captured graph of backward calls: several replays, with eager work and synchronisations in
    between, against the eager result (the call records kernel nodes only: no memset, no allocation)."""
    torch = torch_cuda
    T, d_in, d_out, r = 300, 1024, 768, 16
    d = inputs.make_backward_inputs(33, T, d_in, d_out, r)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    pA, _ = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    pAt, pBt = binding.lordba_pack_transposed(d["signsA"], d["signsB"])
    w = lambda a: cu(a.view(np.int32))
    args = (cu(d["x"]), cu(d["g"]), w(pA), w(pAt), w(pBt), cu(d["s_in"]), cu(d["s_rank"]), cu(d["s_out"]), cu(d["latA"]), cu(d["latB"]), KAPPA)
    dxb = cu(d["dx_base"])
    ws = torch.empty(binding.lordba_backward_workspace_bytes(T, d_in, d_out, r), dtype=torch.uint8, device="cuda:0")
    eager = binding.lordba_backward(*args, dx_base=dxb, workspace=ws)
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in eager.items()}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rec = binding.lordba_backward(*args, dx_base=dxb, workspace=ws)
    for rep in range(4):
        for v in rec.values():
            v.fill_(float("nan"))
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(rec[k], eager[k]), (rep, k)
        again = binding.lordba_backward(*args, dx_base=dxb, workspace=ws)      # eager work between replays
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(again[k], eager[k]), (rep, k)
    compare({k: v.cpu().numpy() for k, v in eager.items()}, oracle_backward(d), "graph_replay")


def test_headline_shape(torch_cuda):
    """d_in = d_out = 4096, r = 16, T = 2048 (the launch configuration bench.py times), every output against the oracle."""
    d = inputs.make_backward_inputs(30, 2048, 4096, 4096, 16)
    got = gpu_backward(torch_cuda, d)
    compare(got, oracle_backward(d), "c2_backward")


@pytest.mark.parametrize("shape", [(4096, 4096, 11008, 16), (4096, 5120, 5120, 16)], ids=lambda s: "T%d_%dx%d_r%d" % s)
def test_large_shapes_in_their_launch_configuration(torch_cuda, shape):
    """The MLP up-projection shape at its own T = 4096 (86 column blocks, the last one partial) and the 5120-wide
    attention shape at T = 4096: 16-row tiles in the dx / t kernels, two wgrad workgroups per CU, as bench.py launches them.
    Every output against the oracle (the oracle needs some ten seconds per shape)."""
    T, d_in, d_out, r = shape
    d = inputs.make_backward_inputs(34, T, d_in, d_out, r)
    got = gpu_backward(torch_cuda, d, keep_t=True)
    compare(got, oracle_backward(d), "T%d_%dx%d_r%d" % shape)


@pytest.mark.parametrize("shape", [(5, 262144, 4096, 8), (12, 2048, 131072, 16), (40000, 256, 256, 16)],
                         ids=lambda s: "T%d_%dx%d_r%d" % s)
def test_extreme_aspect_ratios(torch_cuda, shape):
    """Very wide inputs, very wide outputs (thousands of column blocks, the looped stage 1 of the forward kernel) and a
    very long batch (thousands of token tiles): index arithmetic far from the benchmark shapes."""
    T, d_in, d_out, r = shape
    d = inputs.make_backward_inputs(38, T, d_in, d_out, r)
    got = gpu_backward(torch_cuda, d)
    compare(got, oracle_backward(d), "T%d_%dx%d_r%d" % shape)


def test_argument_errors(torch_cuda):
    torch = torch_cuda
    d = inputs.make_backward_inputs(31, 16, 256, 256, 8)
    need = binding.lordba_backward_workspace_bytes(16, 256, 256, 8)
    assert need > 0
    with pytest.raises(binding.LordbaError) as e:
        gpu_backward(torch, d, ws=new_workspace(torch, need), ws_bytes=need - 16)
    assert e.value.status == 9
    assert binding.lordba_backward_workspace_bytes(16, 250, 256, 8) > 0       # any width (general kernel)
    assert binding.lordba_backward_workspace_bytes(16, 0, 256, 8) == 0
    assert binding.lordba_backward_workspace_bytes(16, 256, 256, 65) == 0


@pytest.mark.parametrize("shape", [(512, 512, 4), (4096, 4096, 16), (96, 40, 7), (33, 17, 1), (64, 64, 64), (4096, 11008, 16), (40, 3, 3)],
                         ids=lambda s: "%dx%d_r%d" % s)
def test_pack_latents_on_the_device_is_bit_exact(torch_cuda, shape):
    """lordba_pack_latents against the oracle's own sign (sign(0) = +1) and packer, for the four packed carriers; zeros of
    both signs and subnormals among the latents; pad bits 0."""
    torch = torch_cuda
    d_in, d_out, r = shape
    g = np.random.default_rng(40)
    latA = g.standard_normal((r, d_in)).astype(np.float32)
    latB = g.standard_normal((d_out, r)).astype(np.float32)
    for lat in (latA, latB):
        flat = lat.reshape(-1)
        idx = g.permutation(flat.size)[: max(4, flat.size // 8)]
        flat[idx[0::4]] = 0.0
        flat[idx[1::4]] = -0.0
        flat[idx[2::4]] = 1e-42
        flat[idx[3::4]] = -1e-42
    pA, pB, pAt, pBt = binding.lordba_pack_latents(torch.from_numpy(latA).cuda(), torch.from_numpy(latB).cuda())
    torch.cuda.synchronize()
    sA, sB = oracle.sign(latA), oracle.sign(latB)
    for got, want in ((pA, oracle.pack(sA)), (pB, oracle.pack(sB)), (pAt, oracle.pack(np.ascontiguousarray(sA.T))),
                      (pBt, oracle.pack(np.ascontiguousarray(sB.T)))):
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want)
    # the same words as the library's host packer, and a call that wants only two of the four
    hA, hB = binding.lordba_pack_signs(latA, latB)
    assert np.array_equal(pA.cpu().numpy().view(np.uint32), hA) and np.array_equal(pB.cpu().numpy().view(np.uint32), hB)
    qA, qB, qAt, qBt = binding.lordba_pack_latents(torch.from_numpy(latA).cuda(), torch.from_numpy(latB).cuda(), transposed=False)
    torch.cuda.synchronize()
    assert qAt is None and qBt is None and torch.equal(qA, pA) and torch.equal(qB, pB)
