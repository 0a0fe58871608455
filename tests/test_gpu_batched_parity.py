"""GPU parity of the multi-adapter batch forward: lordba_forward_batched through the C ABI against the fp64 oracle on
the same seeded inputs (pool of adapters, one adapter index per token row).  Same bar as the other parity tests."""
import sys

import numpy as np
import pytest

import oracle
from paper_2605_24058_amd import binding, inputs

pytestmark = pytest.mark.gpu

TOL = 1e-3
A_AUTO, A_GEN, A_T8 = 0, 1, 2


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make(seed, T, d_in, d_out, r, n, pattern):
    d = inputs.make_adapter_pool(seed, d_in, d_out, r, n)
    d.update(inputs.make_activations(seed, T, d_in, d_out))
    d["ids"] = inputs.make_adapter_ids(seed, T, n, pattern)
    return d


def gpu_batched(torch, d, algo=A_AUTO, inplace=False):
    pA, pB = binding.lordba_pack_pool(d["signsA"], d["signsB"])
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dev = {k: f(d[k]) for k in ("x", "y_base", "s_in", "s_rank", "s_out", "ids")}
    dev["pA"], dev["pB"] = f(pA.view(np.int32)), f(pB.view(np.int32))
    T, d_out = d["y_base"].shape
    if inplace:
        y = binding.lordba_forward_batched(dev["x"], dev["pA"], dev["pB"], dev["s_in"], dev["s_rank"], dev["s_out"], dev["ids"],
                                           dev["y_base"], y_out=dev["y_base"], algo=algo)
        torch.cuda.synchronize()
        return y.cpu().numpy()
    n, pad = T * d_out, 4096
    big = torch.full((n + 2 * pad,), float("nan"), dtype=torch.float16, device="cuda:0")
    y_out = big[pad:pad + n].view(T, d_out)
    binding.lordba_forward_batched(dev["x"], dev["pA"], dev["pB"], dev["s_in"], dev["s_rank"], dev["s_out"], dev["ids"],
                                   dev["y_base"], y_out=y_out, algo=algo)
    torch.cuda.synchronize()
    host = big.cpu().numpy()
    assert np.isnan(host[:pad]).all() and np.isnan(host[pad + n:]).all(), "write outside y_out"
    assert np.array_equal(dev["x"].cpu().numpy(), d["x"]) and np.array_equal(dev["y_base"].cpu().numpy(), d["y_base"])
    return host[pad:pad + n].reshape(T, d_out)


def want_of(d):
    return oracle.forward_batched(d["x"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["ids"], d["y_base"])


def check(torch, d, algo, label):
    for tag, dd in (("full", d), ("delta", dict(d, y_base=np.zeros_like(d["y_base"])))):
        say("  case %s algo=%d %s" % (label, algo, tag))
        got = gpu_batched(torch, dd, algo)
        assert not np.isnan(got).any(), "unwritten or NaN output (%s, %s)" % (label, tag)
        want = want_of(dd)
        err = oracle.row_rel_l2(got.astype(np.float64), want)
        assert err.max() <= TOL, "%s %s algo %d: max row rel-L2 %.3e at row %d" % (label, tag, algo, err.max(), err.argmax())
        none = (dd["ids"] < 0) | (dd["ids"] >= dd["signsA"].shape[0])
        assert np.array_equal(got[none], dd["y_base"][none]), "rows without an adapter must pass through bit for bit"


CASES = [
    # (T, d_in, d_out, r, n_adapters, pattern)
    (64, 512, 512, 16, 4, "segments"),
    (61, 256, 384, 16, 5, "segments"),          # ragged last tile, boundaries inside tiles
    (40, 256, 256, 16, 40, "decode"),           # every row its own adapter, unsorted
    (100, 384, 640, 16, 7, "mixed"),            # rows without an adapter
    (33, 640, 384, 8, 3, "segments"),           # r = 8 byte-per-column path
    (29, 512, 256, 32, 4, "decode"),            # two rank blocks
    (26, 256, 512, 64, 3, "segments"),          # four rank blocks: 8 waves
    (45, 256, 384, 12, 4, "mixed"),             # generic carrier fetch; 384 * 12 is a multiple of 128
    (30, 160, 136, 16, 3, "segments"),          # pool rows of sign(B) not 16-byte aligned: general kernel
    (9, 33, 17, 3, 2, "decode"),                # nothing aligned: general kernel
    (1, 4096, 4096, 16, 2, "segments"),
    (8, 2048, 1024, 16, 8, "decode"),
    # more than 32 tiles: two 8-wave workgroups per tile share its runs (the second and later runs of a workgroup go through
    # the looped copy of the tile code), tiles dealt to the XCDs in contiguous ranges, tile counts that are no multiple of 8
    (301, 512, 640, 16, 9, "decode"),           # 38 tiles, up to 8 runs each, ragged last tile
    (333, 384, 512, 16, 6, "mixed"),            # runs without an adapter inside the loops
    (290, 640, 384, 8, 5, "decode"),
    (275, 256, 384, 32, 7, "decode"),           # two rank blocks
    (270, 256, 256, 64, 3, "mixed"),            # four rank blocks (one workgroup per compute unit)
    (280, 512, 384, 12, 4, "decode"),           # generic carrier fetch
    (520, 8192, 512, 16, 3, "segments"),        # 64 chunks of x: the looped x pipeline (the batch mode has no 8-deep one)
]


@pytest.mark.parametrize("T,d_in,d_out,r,n,pattern", CASES,
                         ids=["T%d_%dx%d_r%d_n%d_%s" % c for c in CASES])
def test_batched_every_kernel(torch_cuda, T, d_in, d_out, r, n, pattern):
    d = make(3, T, d_in, d_out, r, n, pattern)
    ran = 0
    for algo, may_decline in ((A_AUTO, False), (A_GEN, False), (A_T8, True)):
        try:
            check(torch_cuda, d, algo, "batched")
            ran += 1
        except binding.LordbaError as e:
            assert may_decline and e.status == 8, (algo, e.status)
    assert ran >= 2


def test_headline_shape_eight_requests(torch_cuda):
    sh = inputs.C2
    d = make(0, sh.T, sh.d_in, sh.d_out, sh.r, 8, "segments")
    check(torch_cuda, d, A_AUTO, "c2_8_adapters")


def test_one_adapter_pool_matches_the_plain_call_bit_for_bit(torch_cuda):
    torch = torch_cuda
    d = make(5, 72, 512, 384, 16, 1, "segments")
    got = gpu_batched(torch, d, A_T8)
    one = {k: d[k][0] for k in ("signsA", "signsB", "s_in", "s_rank", "s_out")}
    dev = binding.to_device(dict(one, x=d["x"], y_base=d["y_base"]))
    plain = binding.lordba_forward(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                   dev["y_base"], algo=A_T8)
    torch.cuda.synchronize()
    assert np.array_equal(got, plain.cpu().numpy())


def test_out_of_range_indices_pass_through(torch_cuda):
    d = make(6, 24, 256, 256, 16, 3, "segments")
    d["ids"][[0, 7, 8, 23]] = [-5, 3, 2 ** 30, -1]
    for algo in (A_AUTO, A_GEN):
        check(torch_cuda, d, algo, "out_of_range")


def test_in_place(torch_cuda):
    d = make(7, 50, 384, 256, 16, 6, "mixed")
    got = gpu_batched(torch_cuda, d, inplace=True)
    assert oracle.row_rel_l2(got.astype(np.float64), want_of(d)).max() <= TOL


def test_row_order_does_not_change_a_row(torch_cuda):
    # the same rows sorted by adapter or shuffled: every row's result is the same bits
    d = make(8, 48, 512, 256, 16, 6, "segments")
    perm = np.random.default_rng(1).permutation(48)
    a = gpu_batched(torch_cuda, d)
    b = gpu_batched(torch_cuda, dict(d, x=d["x"][perm], y_base=d["y_base"][perm], ids=d["ids"][perm]))
    assert np.array_equal(a[perm], b)


def test_bad_arguments(torch_cuda):
    torch = torch_cuda
    d = make(9, 8, 64, 64, 4, 2, "segments")
    pA, pB = binding.lordba_pack_pool(d["signsA"], d["signsB"])
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dev = {k: f(d[k]) for k in ("x", "y_base", "s_in", "s_rank", "s_out", "ids")}
    lib = binding.load_library()
    dpA, dpB, y_out = f(pA.view(np.int32)), f(pB.view(np.int32)), torch.empty_like(dev["y_base"])   # kept alive below
    args = [dev["x"].data_ptr(), dpA.data_ptr(), dpB.data_ptr(), dev["s_in"].data_ptr(),
            dev["s_rank"].data_ptr(), dev["s_out"].data_ptr(), dev["ids"].data_ptr(), dev["y_base"].data_ptr(),
            y_out.data_ptr(), 8, 64, 64, 4]
    assert lib.lordba_forward_batched(*args, 0, None) == 2            # empty pool
    a = list(args); a[6] = None
    assert lib.lordba_forward_batched(*a, 2, None) == 1               # no index array
    assert lib.lordba_forward_batched_algo(*args, 2, None, 3) == 8    # 16-row tiles do not exist for batches
    assert lib.lordba_forward_batched(*args, 2, None) == 0
    torch.cuda.synchronize()
    del dpA, dpB, y_out


def test_hip_graph_replays_match_eager(torch_cuda):
    # several replays of a captured batched launch (both grid modes), with eager work in between
    torch = torch_cuda
    for T in (40, 520):                   # a few tiles (a workgroup per run) and many tiles (8-wave workgroups)
        d = make(11, T, 512, 384, 16, 5, "mixed")
        pA, pB = binding.lordba_pack_pool(d["signsA"], d["signsB"])
        f = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        args = (f(d["x"]), f(pA.view(np.int32)), f(pB.view(np.int32)), f(d["s_in"]), f(d["s_rank"]), f(d["s_out"]),
                f(d["ids"]), f(d["y_base"]))
        eager = binding.lordba_forward_batched(*args).clone()
        torch.cuda.synchronize()
        y_g = torch.empty_like(eager)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            binding.lordba_forward_batched(*args, y_out=y_g)
        for rep in range(3):
            y_g.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(y_g, eager), (T, rep)
            again = binding.lordba_forward_batched(*args)
            torch.cuda.synchronize()
            assert torch.equal(again, eager)
        assert oracle.row_rel_l2(eager.cpu().numpy().astype(np.float64), want_of(d)).max() <= TOL


# ---- pools whose adapters have several scale envelopes: lordba_forward_batched_multi ------------------------------------

def make_multi(seed, T, d_in, d_out, r, n, ell, pattern):
    d = inputs.make_adapter_pool_multi(seed, d_in, d_out, r, n, ell)
    d.update(inputs.make_activations(seed, T, d_in, d_out))
    d["ids"] = inputs.make_adapter_ids(seed, T, n, pattern)
    return d


def gpu_batched_multi(torch, d, algo=A_AUTO, inplace=False):
    pA, pB = binding.lordba_pack_pool(d["signsA"], d["signsB"])
    f = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dev = {k: f(d[k]) for k in ("x", "y_base", "s_in", "s_rank", "s_out", "ids")}
    dev["pA"], dev["pB"] = f(pA.view(np.int32)), f(pB.view(np.int32))
    T, d_out = d["y_base"].shape
    args = (dev["x"], dev["pA"], dev["pB"], dev["s_in"], dev["s_rank"], dev["s_out"], dev["ids"], dev["y_base"])
    if inplace:
        y = binding.lordba_forward_batched_multi(*args, y_out=dev["y_base"], algo=algo)
        torch.cuda.synchronize()
        return y.cpu().numpy()
    n, pad = T * d_out, 4096
    big = torch.full((n + 2 * pad,), float("nan"), dtype=torch.float16, device="cuda:0")
    y_out = big[pad:pad + n].view(T, d_out)
    binding.lordba_forward_batched_multi(*args, y_out=y_out, algo=algo)
    torch.cuda.synchronize()
    host = big.cpu().numpy()
    assert np.isnan(host[:pad]).all() and np.isnan(host[pad + n:]).all(), "write outside y_out"
    return host[pad:pad + n].reshape(T, d_out)


def check_multi(torch, d, algo, label):
    for tag, dd in (("full", d), ("delta", dict(d, y_base=np.zeros_like(d["y_base"])))):
        say("  case %s ell=%d algo=%d %s" % (label, d["s_rank"].shape[1], algo, tag))
        got = gpu_batched_multi(torch, dd, algo)
        assert not np.isnan(got).any(), "unwritten or NaN output (%s, %s)" % (label, tag)
        want = oracle.forward_batched_multi(dd["x"], dd["signsA"], dd["signsB"], dd["s_in"], dd["s_rank"], dd["s_out"], dd["ids"],
                                            dd["y_base"])
        err = oracle.row_rel_l2(got.astype(np.float64), want)
        assert err.max() <= TOL, "%s %s algo %d: max row rel-L2 %.3e at row %d" % (label, tag, algo, err.max(), err.argmax())
        none = (dd["ids"] < 0) | (dd["ids"] >= dd["signsA"].shape[0])
        assert np.array_equal(got[none], dd["y_base"][none]), "rows without an adapter must pass through bit for bit"


MULTI_CASES = [
    # (T, d_in, d_out, r, n_adapters, ell, pattern)
    (64, 512, 512, 16, 4, 2, "segments"),
    (61, 256, 384, 16, 5, 3, "mixed"),           # ragged last tile, boundaries inside tiles, rows without an adapter
    (40, 256, 256, 16, 40, 4, "decode"),         # every row its own adapter
    (33, 640, 384, 8, 3, 2, "segments"),         # r = 8
    (29, 512, 256, 32, 4, 3, "decode"),          # two rank blocks
    (27, 512, 256, 32, 4, 4, "decode"),          # two rank blocks with four envelopes: general kernel
    (26, 256, 512, 64, 3, 2, "segments"),        # four rank blocks: general kernel
    (45, 256, 384, 12, 4, 2, "mixed"),           # generic carrier fetch
    (9, 33, 17, 3, 2, 3, "decode"),              # nothing aligned: general kernel
    (301, 512, 640, 16, 9, 2, "decode"),         # more than 32 tiles: two workgroups per tile, looped later runs
    (333, 384, 512, 16, 6, 4, "mixed"),
    (290, 8192, 384, 16, 3, 3, "segments"),      # looped x pipeline
]


@pytest.mark.parametrize("T,d_in,d_out,r,n,ell,pattern", MULTI_CASES,
                         ids=["T%d_%dx%d_r%d_n%d_l%d_%s" % c for c in MULTI_CASES])
def test_batched_multi_every_kernel(torch_cuda, T, d_in, d_out, r, n, ell, pattern):
    d = make_multi(17, T, d_in, d_out, r, n, ell, pattern)
    ran = 0
    for algo, may_decline in ((A_AUTO, False), (A_GEN, False), (A_T8, True)):
        try:
            check_multi(torch_cuda, d, algo, "batched_multi")
            ran += 1
        except binding.LordbaError as e:
            assert may_decline and e.status == 8, (algo, e.status)
            say("  algo %d declines" % algo)
    assert ran >= 2


def test_batched_multi_headline_shape(torch_cuda):
    sh = inputs.C2
    d = make_multi(18, sh.T, sh.d_in, sh.d_out, sh.r, 8, 2, "segments")
    check_multi(torch_cuda, d, A_AUTO, "c2_8_adapters_2_envelopes")


def test_batched_multi_one_envelope_and_one_adapter_reduce_to_the_other_entry_points(torch_cuda):
    torch = torch_cuda
    d1 = make_multi(19, 72, 512, 384, 16, 3, 1, "segments")                 # ell = 1: lordba_forward_batched, bit for bit
    got = gpu_batched_multi(torch, d1)
    plain = gpu_batched(torch, dict(d1, s_in=d1["s_in"][:, 0], s_rank=d1["s_rank"][:, 0], s_out=d1["s_out"][:, 0]))
    assert np.array_equal(got, plain)
    d2 = make_multi(20, 72, 512, 384, 16, 1, 3, "segments")                 # one adapter: lordba_forward_multi within the bar
    got = gpu_batched_multi(torch, d2)
    want = oracle.forward_multi(d2["x"], d2["signsA"][0], d2["signsB"][0], d2["s_in"][0], d2["s_rank"][0], d2["s_out"][0], d2["y_base"])
    assert oracle.row_rel_l2(got.astype(np.float64), want).max() <= TOL


def test_batched_multi_in_place_and_bad_envelope_count(torch_cuda):
    torch = torch_cuda
    d = make_multi(21, 50, 384, 256, 16, 6, 2, "mixed")
    got = gpu_batched_multi(torch, d, inplace=True)
    want = oracle.forward_batched_multi(d["x"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["ids"], d["y_base"])
    assert oracle.row_rel_l2(got.astype(np.float64), want).max() <= TOL
    five = inputs.make_adapter_pool_multi(22, 64, 64, 4, 2, 5)
    five.update(inputs.make_activations(22, 8, 64, 64))
    five["ids"] = inputs.make_adapter_ids(22, 8, 2, "segments")
    with pytest.raises(binding.LordbaError) as e:
        gpu_batched_multi(torch, five)
    assert e.value.status == 2
    torch.cuda.synchronize()
