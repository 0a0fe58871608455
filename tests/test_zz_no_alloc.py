"""lordba_backward_noalloc (the entry point for callers that cannot allocate: its scratch is a device array inside the
library) against lordba_backward with a caller-owned workspace, through the C ABI.  Both run the same kernels in the same
order on the same plan, so every output must agree bit for bit (which is inside the 1e-3 relative-L2 bar of the backward
parity tests, and those pin lordba_backward to the CPU oracle); the first case is also compared with the oracle directly.
Two calls in a row share the library's array, the second with a smaller input: what the first call left there must not
reach the second call's results."""
import ctypes
import sys

import numpy as np
import pytest

import oracle
from paper_2605_24058_amd import binding, inputs

pytestmark = pytest.mark.gpu

KAPPA = 100.0
KEYS = ("dx", "d_s_in", "d_s_rank", "d_s_out", "d_latentA", "d_latentB")


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def device_args(torch, d):
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    pA, _ = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    pAt, pBt = binding.lordba_pack_transposed(d["signsA"], d["signsB"])
    return dict(x=cu(d["x"]), g=cu(d["g"]), pA=cu(pA.view(np.int32)), pAt=cu(pAt.view(np.int32)), pBt=cu(pBt.view(np.int32)),
                s_in=cu(d["s_in"]), s_rank=cu(d["s_rank"]), s_out=cu(d["s_out"]), latA=cu(d["latA"]), latB=cu(d["latB"]),
                dx_base=cu(d["dx_base"]))


def both(torch, a, label):
    """The same call through lordba_backward (fresh poisoned workspace) and through lordba_backward_noalloc."""
    say("  case %s" % label)
    head = (a["x"], a["g"], a["pA"], a["pAt"], a["pBt"], a["s_in"], a["s_rank"], a["s_out"], a["latA"], a["latB"], KAPPA)
    T, d_in = a["x"].shape
    d_out, r = a["latB"].shape
    ws = torch.full((binding.lordba_backward_workspace_bytes(T, d_in, d_out, r),), 0xFF, dtype=torch.uint8, device="cuda:0")
    want = binding.lordba_backward(*head, dx_base=a["dx_base"], workspace=ws)
    got = binding.lordba_backward_noalloc(*head, dx_base=a["dx_base"])
    torch.cuda.synchronize()
    for k in KEYS:
        g_, w_ = got[k].cpu().numpy(), want[k].cpu().numpy()
        assert np.isfinite(g_.astype(np.float64)).all(), "%s %s: non-finite" % (label, k)
        assert np.array_equal(g_, w_), "%s: %s differs from lordba_backward" % (label, k)
    return got


def test_two_calls_in_a_row_second_one_smaller(torch_cuda):
    torch = torch_cuda
    big = inputs.make_backward_inputs(5, 519, 2048, 1536, 16)
    small = inputs.make_backward_inputs(6, 37, 1024, 1152, 16)
    a_big, a_small = device_args(torch, big), device_args(torch, small)
    got = both(torch, a_big, "T519_2048x1536_r16")
    want = oracle.backward(big["x"], big["g"], big["signsA"], big["signsB"], big["s_in"], big["s_rank"], big["s_out"], big["latA"],
                           big["latB"], KAPPA, big["dx_base"])
    e = oracle.row_rel_l2(got["dx"].cpu().numpy().astype(np.float64), want["dx"]).max()
    assert e <= 1e-3, e
    for k, ko in (("d_s_in", "d_s_in"), ("d_s_rank", "d_s_rank"), ("d_s_out", "d_s_out")):
        assert oracle.rel_l2(got[k].cpu().numpy(), want[ko]) <= 1e-3, k
    assert oracle.row_rel_l2(got["d_latentA"].cpu().numpy().astype(np.float64), want["d_latA"]).max() <= 1e-3
    assert oracle.row_rel_l2(got["d_latentB"].cpu().numpy().astype(np.float64).T, want["d_latB"].T).max() <= 1e-3
    both(torch, a_small, "T37_1024x1152_r16 after the larger call")
    both(torch, a_big, "T519_2048x1536_r16 again")


def test_kept_t_and_frozen_carriers(torch_cuda):
    torch = torch_cuda
    d = inputs.make_backward_inputs(7, 203, 1056, 2080, 16)
    a = device_args(torch, d)
    _, pB = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    pB = torch.from_numpy(pB.view(np.int32)).to("cuda:0")
    _, t_saved = binding.lordba_forward_save_t(a["x"], a["pA"], pB, a["s_in"], a["s_rank"], a["s_out"])
    head = (a["x"], a["g"], a["pA"], a["pAt"], a["pBt"], a["s_in"], a["s_rank"], a["s_out"])
    want = binding.lordba_backward(*head, a["latA"], a["latB"], KAPPA, dx_base=a["dx_base"], t_saved=t_saved)
    got = binding.lordba_backward_noalloc(*head, a["latA"], a["latB"], KAPPA, dx_base=a["dx_base"], t_saved=t_saved)
    torch.cuda.synchronize()
    for k in KEYS:
        assert np.array_equal(got[k].cpu().numpy(), want[k].cpu().numpy()), k
    want = binding.lordba_backward(*head, None, None, KAPPA, dx_base=a["dx_base"])
    got = binding.lordba_backward_noalloc(*head, None, None, KAPPA, dx_base=a["dx_base"])
    torch.cuda.synchronize()
    for k in ("dx", "d_s_in", "d_s_rank", "d_s_out"):
        assert np.array_equal(got[k].cpu().numpy(), want[k].cpu().numpy()), k
    assert got["d_latentA"] is None and got["d_latentB"] is None


def test_allocates_nothing_and_reuses_outputs(torch_cuda):
    """With the outputs of an earlier call handed back, a call leaves torch's allocator untouched (the C call itself never
    allocates; the wrapper's only allocations are the output tensors)."""
    torch = torch_cuda
    d = inputs.make_backward_inputs(8, 64, 512, 512, 4)
    a = device_args(torch, d)
    head = (a["x"], a["g"], a["pA"], a["pAt"], a["pBt"], a["s_in"], a["s_rank"], a["s_out"], a["latA"], a["latB"], KAPPA)
    out = binding.lordba_backward_noalloc(*head, dx_base=a["dx_base"])
    torch.cuda.synchronize()
    first = {k: out[k].clone() for k in KEYS}
    for k in KEYS:
        out[k].fill_(float("nan"))
    torch.cuda.synchronize()
    # the allocator's running count of allocations (bytes in use may fall meanwhile: tensors of earlier tests being collected)
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    again = binding.lordba_backward_noalloc(*head, dx_base=a["dx_base"], out=out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    for k in KEYS:
        assert again[k] is out[k] and torch.equal(out[k], first[k]), k


def test_shape_beyond_the_array_is_refused(torch_cuda):
    """lordba_backward_workspace_bytes above the array's size: LORDBA_ERR_WORKSPACE before anything is enqueued (the
    pointers are never touched, so fake ones serve)."""
    lib = binding.load_library()
    T, d_in, d_out, r = 8192, 13824, 5120, 64
    assert binding.lordba_backward_workspace_bytes(T, d_in, d_out, r) > binding.BACKWARD_NOALLOC_MAX_BYTES
    p = [0x10000000 + i * 0x1000000 for i in range(20)]
    st = lib.lordba_backward_noalloc(p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7], p[8], p[9], ctypes.c_float(KAPPA), None, 0,
                                     p[10], p[11], p[12], p[13], p[14], p[15], p[16], T, d_in, d_out, r, None)
    assert st == 9
    assert "workspace" in binding.lordba_status_string(st)
    # the largest projection of the paper's models at r = 16 fits
    assert binding.lordba_backward_workspace_bytes(8192, 13824, 5120, 16) <= binding.BACKWARD_NOALLOC_MAX_BYTES
    assert binding.lordba_backward_workspace_bytes(8192, 5120, 13824, 16) <= binding.BACKWARD_NOALLOC_MAX_BYTES
