"""GPU parity of the multi-envelope forward (Eq. (lordba), envelope rank l >= 2): lordba_forward_multi through the C
ABI against the fp64 oracle on the same seeded inputs.  Same bar as the one-envelope tests: per token row
||y_gpu - y||_2 / ||y||_2 <= 1e-3, as configured and with y_base = 0."""
import sys

import numpy as np
import pytest

import oracle
from paper_2605_24058_amd import binding, inputs

pytestmark = pytest.mark.gpu

TOL = 1e-3
NTHREADS = min(16, oracle.available_cores())
A_AUTO, A_GEN, A_T8, A_T16 = 0, 1, 2, 3


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    return torch


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def to_device(torch, d):
    dev = binding.to_device(d)          # packs the carriers, moves x / y_base / (2-D) scale arrays
    return dev


def gpu_multi(torch, d, algo=A_AUTO, inplace=False):
    dev = to_device(torch, d)
    T, d_out = d["y_base"].shape
    n, pad = T * d_out, 4096
    if inplace:
        y = binding.lordba_forward_multi(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                         dev["y_base"], y_out=dev["y_base"], algo=algo)
        torch.cuda.synchronize()
        return y.cpu().numpy()
    big = torch.full((n + 2 * pad,), float("nan"), dtype=torch.float16, device="cuda:0")
    y_out = big[pad:pad + n].view(T, d_out)
    binding.lordba_forward_multi(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                 dev["y_base"], y_out=y_out, algo=algo)
    torch.cuda.synchronize()
    host = big.cpu().numpy()
    assert np.isnan(host[:pad]).all() and np.isnan(host[pad + n:]).all(), "write outside y_out"
    assert np.array_equal(dev["x"].cpu().numpy(), d["x"]) and np.array_equal(dev["y_base"].cpu().numpy(), d["y_base"])
    return host[pad:pad + n].reshape(T, d_out)


def oracle_multi(d, rows=None):
    x, yb = (d["x"], d["y_base"]) if rows is None else (d["x"][rows], d["y_base"][rows])
    return oracle.forward_multi(x, d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], yb, nthreads=NTHREADS)


def check(torch, d, algo, label, rows=None):
    worst = 0.0
    for tag, dd in (("full", d), ("delta", dict(d, y_base=np.zeros_like(d["y_base"])))):
        say("  case %s ell=%d algo=%d %s" % (label, d["s_in"].shape[0], algo, tag))
        got = gpu_multi(torch, dd, algo)
        assert not np.isnan(got).any(), "unwritten or NaN output (%s, %s)" % (label, tag)
        want = oracle_multi(dd, rows)
        g = got if rows is None else got[rows]
        err = oracle.row_rel_l2(g.astype(np.float64), want)
        assert err.max() <= TOL, "%s %s algo %d: max row rel-L2 %.3e at row %d" % (label, tag, algo, err.max(), err.argmax())
        worst = max(worst, err.max())
        if tag == "full":
            assert np.mean(g == want.astype(np.float16)) > 0.97
    return worst


def algos_for(sh, ell):
    """(algo, may_decline): an explicitly requested matrix-core variant may answer LORDBA_ERR_ALGO (8) when the shape
    does not fit its registers or LDS; AUTO and GENERAL must always run."""
    al = [(A_AUTO, False), (A_GEN, False)]
    if sh.d_in % 32 == 0 and sh.d_out % 8 == 0:
        al += [(A_T8, True), (A_T16, True), (6, True), (7, True)]   # 6, 7: the same tile heights on 8 waves
    return al


SMALL = [
    (inputs.C1, 2),
    (inputs.Shape("ragged_T37_160x136_r16", 37, 160, 136, 16), 2),
    (inputs.Shape("ragged_T19_96x200_r4", 19, 96, 200, 4), 3),
    (inputs.Shape("T1_128x128_r16", 1, 128, 128, 16), 4),
    (inputs.Shape("T17_1024x1152_r16", 17, 1024, 1152, 16), 2),
    (inputs.Shape("T33_640x384_r8", 33, 640, 384, 8), 2),
    (inputs.Shape("T9_512x256_r12", 9, 512, 256, 12), 3),
    (inputs.Shape("T40_384x640_r17", 40, 384, 640, 17), 2),
    (inputs.Shape("T16_512x512_r32", 16, 512, 512, 32), 2),
    (inputs.Shape("T23_256x384_r33", 23, 256, 384, 33), 4),
    (inputs.Shape("T8_384x256_r48", 8, 384, 256, 48), 3),
    (inputs.Shape("T31_512x640_r64", 31, 512, 640, 64), 2),
    (inputs.Shape("T12_2048x2048_r7", 12, 2048, 2048, 7), 2),
    (inputs.Shape("T20_4096x1024_r16", 20, 4096, 1024, 16), 4),     # looped stage 1 with four envelopes
    (inputs.Shape("odd_T5_33x17_r3", 5, 33, 17, 3), 2),             # general kernel only
    (inputs.Shape("odd_T4_40x36_r9", 4, 40, 36, 9), 3),
    (inputs.Shape("odd_T3_1x1_r1", 3, 1, 1, 1), 4),
]


@pytest.mark.parametrize("sh,ell", SMALL, ids=["%s_l%d" % (s.name, l) for s, l in SMALL])
def test_small_and_ragged_shapes_every_kernel(torch_cuda, sh, ell):
    d = inputs.make_inputs_multi(7, sh.T, sh.d_in, sh.d_out, sh.r, ell)
    if sh.d_in < 8:                       # keep the outputs out of the fp16 subnormal range
        d["s_out"] = (d["s_out"].astype(np.float32) * 64).astype(np.float16)
    ran = 0
    for algo, may_decline in algos_for(sh, ell):
        try:
            check(torch_cuda, d, algo, sh.name)
            ran += 1
        except binding.LordbaError as e:
            assert may_decline and e.status == 8, (algo, e.status)
            say("  algo %d declines %s with ell=%d" % (algo, sh.name, ell))
    assert ran >= 2


@pytest.mark.parametrize("ell", [2, 3, 4])
def test_headline_shape_all_rows(torch_cuda, ell):
    sh = inputs.C2
    d = inputs.make_inputs_multi(0, sh.T, sh.d_in, sh.d_out, sh.r, ell)
    check(torch_cuda, d, A_AUTO, "c2")


@pytest.mark.parametrize("ell", [2, 3, 4])
def test_tall_shape_sampled_rows(torch_cuda, ell):
    sh = inputs.C3_UP                     # T = 4096: 16-row tiles (four envelopes: the variant with one y block in flight)
    d = inputs.make_inputs_multi(1, sh.T, sh.d_in, sh.d_out, sh.r, ell)
    rows = np.unique(np.concatenate([np.arange(0, sh.T, 97), [0, 15, 16, sh.T - 17, sh.T - 1]]))
    check(torch_cuda, d, A_AUTO, "c3_up", rows=rows)


@pytest.mark.parametrize("sh,ell", [(inputs.Shape("T4100_1024x1152_r16", 4100, 1024, 1152, 16), 3),
                                    (inputs.Shape("T4107_640x896_r16", 4107, 640, 896, 16), 4),
                                    (inputs.Shape("T4099_512x640_r12", 4099, 512, 640, 12), 4),
                                    (inputs.Shape("T4112_384x512_r32", 4112, 384, 512, 32), 3),
                                    (inputs.Shape("T2100_1024x1152_r16", 2100, 1024, 1152, 16), 4),
                                    (inputs.Shape("T300_4096x4096_r16", 300, 4096, 4096, 16), 3)],
                         ids=lambda v: v.name if hasattr(v, "name") else "l%d" % v)
def test_sixteen_row_tiles_and_deep_y_pipeline_every_row(torch_cuda, sh, ell):
    """Three and four envelopes on 16-row tiles (T >= 4096, ragged last tile, a general rank, two rank blocks falling
    back to 8-row tiles) and on 8-row tiles with four y blocks in flight per wave (more blocks than four per wave at
    4096 columns, fewer at 1152), every row against the oracle, every matrix-core selector."""
    d = inputs.make_inputs_multi(13, sh.T, sh.d_in, sh.d_out, sh.r, ell)
    ran = 0
    for algo in (A_AUTO, A_T8, A_T16, 6, 7):
        try:
            check(torch_cuda, d, algo, sh.name)
            ran += 1
        except binding.LordbaError as e:
            assert algo != A_AUTO and e.status == 8, (algo, e.status)
            say("  algo %d declines %s with ell=%d" % (algo, sh.name, ell))
    assert ran >= 2


def test_one_envelope_through_the_multi_entry_point_is_the_single_call(torch_cuda):
    torch = torch_cuda
    d = inputs.make_inputs_multi(3, 50, 256, 384, 16, 1)
    got = gpu_multi(torch, d)
    dev = binding.to_device(dict(d, s_in=d["s_in"][0], s_rank=d["s_rank"][0], s_out=d["s_out"][0]))
    single = binding.lordba_forward(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                    dev["y_base"])
    torch.cuda.synchronize()
    assert np.array_equal(got, single.cpu().numpy())


def test_zero_rank_scale_envelopes_leave_the_first_envelope(torch_cuda):
    # Sec. 3.2: further envelopes start at beta = 0 and the function equals the one-envelope warm start.
    d = inputs.make_inputs_multi(4, 40, 512, 384, 16, 3)
    d["s_rank"][1:] = np.float16(0)
    for algo in (A_AUTO, A_GEN):
        got = gpu_multi(torch_cuda, d, algo)
        want = oracle.forward(d["x"], d["signsA"], d["signsB"], d["s_in"][0], d["s_rank"][0], d["s_out"][0], d["y_base"],
                              nthreads=NTHREADS)
        assert oracle.row_rel_l2(got.astype(np.float64), want).max() <= TOL


def test_cancelling_envelopes_return_y_base_exactly(torch_cuda):
    d = inputs.make_inputs_multi(5, 33, 256, 256, 16, 1)
    two = dict(d, s_in=np.repeat(d["s_in"], 2, 0), s_out=np.repeat(d["s_out"], 2, 0),
               s_rank=np.concatenate([d["s_rank"], -d["s_rank"]]))
    for algo in (A_AUTO, A_GEN):
        got = gpu_multi(torch_cuda, two, algo)
        # each envelope's contribution is computed identically up to sign; their fp32 sum is exactly zero only if
        # both are added to y_base in turn without rounding in between, which fp32 does not promise: within the bar
        assert oracle.row_rel_l2(got.astype(np.float64), d["y_base"].astype(np.float64)).max() <= TOL


def test_envelopes_of_very_different_magnitude(torch_cuda):
    d = inputs.make_inputs_multi(6, 24, 1024, 512, 16, 3)
    d["s_rank"][1] = (d["s_rank"][1].astype(np.float32) * 2.0 ** -8).astype(np.float16)
    d["s_rank"][2] = (d["s_rank"][2].astype(np.float32) * 2.0 ** 6).astype(np.float16)
    for algo in (A_AUTO, A_GEN):
        check(torch_cuda, d, algo, "magnitudes")


def test_in_place(torch_cuda):
    d = inputs.make_inputs_multi(8, 29, 384, 640, 16, 2)
    got = gpu_multi(torch_cuda, d, inplace=True)
    assert oracle.row_rel_l2(got.astype(np.float64), oracle_multi(d)).max() <= TOL


def test_deterministic(torch_cuda):
    d = inputs.make_inputs_multi(9, 64, 1024, 1024, 16, 2)
    a = gpu_multi(torch_cuda, d)
    b = gpu_multi(torch_cuda, d)
    assert np.array_equal(a, b)


def test_envelope_count_out_of_range_is_an_error(torch_cuda):
    torch = torch_cuda
    d = inputs.make_inputs_multi(10, 4, 64, 64, 4, 4)
    big = dict(d, s_in=np.concatenate([d["s_in"], d["s_in"][:1]]), s_rank=np.concatenate([d["s_rank"], d["s_rank"][:1]]),
               s_out=np.concatenate([d["s_out"], d["s_out"][:1]]))
    dev = binding.to_device(big)
    with pytest.raises(binding.LordbaError) as e:
        binding.lordba_forward_multi(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                     dev["y_base"])
    assert e.value.status == 2
    torch.cuda.synchronize()


def test_empty_batch(torch_cuda):
    torch = torch_cuda
    d = inputs.make_inputs_multi(11, 0, 64, 64, 4, 2)
    dev = binding.to_device(d)
    y = binding.lordba_forward_multi(dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"],
                                     dev["y_base"])
    torch.cuda.synchronize()
    assert tuple(y.shape) == (0, 64)


def test_hip_graph_replays_match_eager(torch_cuda):
    # several replays of a captured multi-envelope launch, with eager work in between, against the eager result
    torch = torch_cuda
    d = inputs.make_inputs_multi(12, 70, 1024, 768, 16, 2)
    dev = to_device(torch, d)
    args = (dev["x"], dev["packedA"], dev["packedB"], dev["s_in"], dev["s_rank"], dev["s_out"], dev["y_base"])
    eager = binding.lordba_forward_multi(*args).clone()
    torch.cuda.synchronize()
    y_g = torch.empty_like(eager)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.lordba_forward_multi(*args, y_out=y_g)
    for rep in range(3):
        y_g.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_g, eager), rep
        again = binding.lordba_forward_multi(*args)
        torch.cuda.synchronize()
        assert torch.equal(again, eager)
    assert oracle.row_rel_l2(eager.cpu().numpy().astype(np.float64), oracle_multi(d)).max() <= TOL
