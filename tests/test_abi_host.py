"""Host-side checks of the C-ABI library that need no GPU: the library loads, exports every
symbol the header declares, packs bit-exactly like the oracle's independent packer, and rejects
bad arguments before touching a device.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_24058_amd import binding, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding._LIB_PATH):
        binding.build_library()
    return binding.load_library()


def test_exports_every_declared_symbol(lib):
    text = open(os.path.join(ROOT, "include", "lordba.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(lordba_[a-z0-9_]+)\s*\(", text))
    assert {"lordba_pack_signs", "lordba_forward", "lordba_packed_words", "lordba_status_string"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(lib):
    seen = set()
    for code in range(0, 10):
        s = binding.lordba_status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 10
    assert binding.lordba_status_string(1234) == "unknown status"


@pytest.mark.parametrize("d_in,d_out,r", [(512, 512, 4), (4096, 4096, 16), (96, 40, 7), (33, 17, 1), (64, 64, 64),
                                           (4096, 11008, 16), (5120, 13824, 16)])
def test_pack_is_bit_exact_against_oracle_packer(d_in, d_out, r):
    d = inputs.make_adapter(d_in + d_out + r, d_in, d_out, r)
    pA, pB = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    assert pA.tobytes() == oracle.pack(d["signsA"]).tobytes()
    assert pB.tobytes() == oracle.pack(d["signsB"]).tobytes()
    assert pA.size == binding.lordba_packed_words(r, d_in) == oracle.packed_words(r, d_in)
    A, B = binding.lordba_unpack_signs(pA, pB, d_in, d_out, r)
    assert np.array_equal(A, d["signsA"]) and np.array_equal(B, d["signsB"])


def test_pack_hand_written_words():
    A = np.array([[1, -1, -1, 1, 1, 1, 1, -1]], dtype=np.int8)          # bits 1, 2, 7
    B = np.ones((8, 1), dtype=np.int8)
    B[3, 0] = -1
    pA, pB = binding.lordba_pack_signs(A, B)
    assert pA.tolist() == [0x86] and pB.tolist() == [0x08]


def test_pack_from_latents_uses_sign_zero_plus_one():
    A = np.array([[0.0, -0.0, 1e-30, -1e-30, 2.0, -3.0, np.inf, -np.inf]], dtype=np.float32)
    B = np.zeros((8, 1), dtype=np.float32)
    pA, pB = binding.lordba_pack_signs(A, B)
    assert pA.tolist() == [0b10101000] and pB.tolist() == [0]
    want = oracle.pack(oracle.sign(A.astype(np.float64)))
    assert pA.tobytes() == want.tobytes()
    A[0, 2] = np.nan
    with pytest.raises(binding.LordbaError) as e:
        binding.lordba_pack_signs(A, B)
    assert e.value.status == 3


def test_pack_rejects_bad_values_and_dims(lib):
    A = np.ones((2, 8), dtype=np.int8)
    B = np.ones((8, 2), dtype=np.int8)
    A[1, 5] = 0
    with pytest.raises(binding.LordbaError) as e:
        binding.lordba_pack_signs(A, B)
    assert e.value.status == 3
    buf = (ctypes.c_uint32 * 4)()
    sig = (ctypes.c_int8 * 16)(*([1] * 16))
    p = lambda o: ctypes.cast(o, ctypes.c_void_p)
    assert lib.lordba_pack_signs(None, p(sig), p(buf), p(buf), 8, 8, 2) == 1
    assert lib.lordba_pack_signs(p(sig), p(sig), p(buf), p(buf), 8, 8, 0) == 2
    assert lib.lordba_pack_signs(p(sig), p(sig), p(buf), p(buf), 8, 8, 65) == 2
    assert lib.lordba_pack_signs(p(sig), p(sig), p(buf), p(buf), 0, 8, 2) == 2
    assert lib.lordba_packed_words(-1, 4) == 0 and lib.lordba_packed_words(3, 11) == 2


def test_forward_validation_needs_no_device(lib):
    # Fake, never-dereferenced addresses: every call below must return before any device work.
    base = 0x10000000
    x, pA, pB, si, sr, so, yb, yo = (base + i * 0x1000000 for i in range(8))
    T, d_in, d_out, r = 4, 64, 64, 8
    f = lambda *a: lib.lordba_forward(*a, None)
    ok_args = [x, pA, pB, si, sr, so, yb, yo, T, d_in, d_out, r]
    for i in range(8):                                   # each pointer NULL in turn
        a = list(ok_args); a[i] = None
        assert f(*a) == 1
    empty = list(ok_args); empty[0] = empty[6] = empty[7] = None; empty[8] = 0
    assert f(*empty) == 0                                # T == 0: empty activations may be NULL
    empty[3] = None
    assert f(*empty) == 1
    for bad in [(-1, d_in, d_out, r), (T, 0, d_out, r), (T, d_in, 0, r), (T, d_in, d_out, 0), (T, d_in, d_out, 65),
                (T, 1 << 25, d_out, r), (1 << 31, d_in, d_out, r)]:
        assert f(x, pA, pB, si, sr, so, yb, yo, *bad) == 2
    assert f(x + 1, pA, pB, si, sr, so, yb, yo, T, d_in, d_out, r) == 5      # fp16 pointer at an odd address
    assert f(x, pA + 2, pB, si, sr, so, yb, yo, T, d_in, d_out, r) == 5      # word pointer not 4-aligned
    assert f(x, pA, pB, si, sr, so, yb, x, T, d_in, d_out, r) == 4           # y_out on top of x
    assert f(x, pA, pB, si, sr, so, yb, yb + 16, T, d_in, d_out, r) == 4     # partial overlap with y_base
    assert f(x, pA, pB, si, sr, so, yb, so, T, d_in, d_out, r) == 4
    assert f(x, pA, pB, si, sr, so, yb, yo, 0, d_in, d_out, r) == 0          # T == 0: nothing to do
    assert f(x, pA, pB, si, sr, so, yb, yb, 0, d_in, d_out, r) == 0          # in-place is legal
    assert lib.lordba_forward_algo(x, pA, pB, si, sr, so, yb, yo, T, d_in, d_out, r, None, 99) == 8


def test_backward_validation_needs_no_device(lib):
    """lordba_backward and lordba_forward_save_t reject bad arguments before any device work (fake addresses)."""
    base = 0x10000000
    names = ["x", "g", "pA", "pAt", "pBt", "si", "sr", "so", "lA", "lB", "dxb", "dx", "dsi", "dsr", "dso", "dlA", "dlB", "ws", "ts"]
    p = {n: base + i * 0x1000000 for i, n in enumerate(names)}
    T, d_in, d_out, r = 4, 64, 96, 8
    need = lib.lordba_backward_workspace_bytes(T, d_in, d_out, r)
    assert need > 0 and need % 4 == 0
    assert lib.lordba_backward_workspace_bytes(T, 72, d_out, r) > 0           # any width (the general kernel takes odd ones)
    assert lib.lordba_backward_workspace_bytes(T, 0, d_out, r) == 0 and lib.lordba_backward_workspace_bytes(T, d_in, (1 << 24) + 1, r) == 0
    assert lib.lordba_backward_workspace_bytes(T, d_in, d_out, 0) == 0
    assert lib.lordba_backward_workspace_bytes(0, d_in, d_out, r) > 0

    def call(T=T, d_in=d_in, d_out=d_out, r=r, ws_bytes=need, ts=None, t_stride=0, kappa=100.0, **over):
        q = dict(p); q.update(over)
        return lib.lordba_backward(q["x"], q["g"], q["pA"], q["pAt"], q["pBt"], q["si"], q["sr"], q["so"], q["lA"], q["lB"],
                                   ctypes.c_float(kappa), ts, t_stride, q["dxb"], q["dx"], q["dsi"], q["dsr"], q["dso"], q["dlA"],
                                   q["dlB"], q["ws"], ws_bytes, T, d_in, d_out, r, None)

    for n in ("pA", "pAt", "pBt", "si", "sr", "so", "lA", "lB", "dsi", "dsr", "dso", "dlA", "dlB", "ws", "x", "g"):
        assert call(**{n: None}) == 1, n           # (a single latent pointer missing is an error; all four: frozen carriers)
    assert call(dx=None) == 1 and call(dxb=None) == 1                           # dx and dx_base come or go together
    assert call(d_in=0) == 2 and call(r=65) == 2 and call(T=-1) == 2
    assert call(ws_bytes=need - 4) == 9
    assert call(x=p["x"] + 1) == 5 and call(ws=p["ws"] + 4) == 5 and call(dsi=p["dsi"] + 2) == 5
    assert call(dsi=p["x"]) == 4 and call(dlA=p["lA"]) == 4 and call(ws=p["g"]) == 4 and call(dso=p["dsi"]) == 4   # overlaps
    assert call(dx=p["x"]) == 4
    assert call(ts=p["ts"], t_stride=3) == 2                                    # a kept t must hold T entries per rank
    assert call(ts=p["ts"] + 2, t_stride=128) == 5
    multi = lambda ell: lib.lordba_backward_multi(p["x"], p["g"], p["pA"], p["pAt"], p["pBt"], p["si"], p["sr"], p["so"], p["lA"], p["lB"],
                                                  ctypes.c_float(100.0), None, 0, p["dxb"], p["dx"], p["dsi"], p["dsr"], p["dso"], p["dlA"], p["dlB"],
                                                  p["ws"], need - 4, T, d_in, d_out, r, ell, None)
    assert multi(0) == 2 and multi(5) == 2 and multi(2) == 9                     # envelope count; then the workspace size
    # lordba_forward_save_t: t_out is required, must not overlap the activations, t_stride >= T
    f = lambda *a: lib.lordba_forward_save_t(*a, None)
    yb, yo = p["dxb"], p["dx"]
    ok = [p["x"], p["pA"], p["pBt"], p["si"], p["sr"], p["so"], yb, yo, p["ts"], 128, T, d_in, d_out, r]
    a = list(ok); a[8] = None
    assert f(*a) == 1
    a = list(ok); a[8] = None; a[10] = 0                                        # an empty batch needs no t_out
    assert f(*a) == 0
    a = list(ok); a[9] = T - 1
    assert f(*a) == 2
    a = list(ok); a[8] = p["x"]
    assert f(*a) == 4
    a = list(ok); a[6] = None                                                   # y_base without y_out
    assert f(*a) == 1


def test_ptq_validation_needs_no_device(lib):
    """lordba_ptq rejects bad arguments before any device work (fake addresses)."""
    base = 0x20000000
    names = ["A", "B", "pA", "pB", "al", "be", "ga", "si", "sr", "so", "info", "ws"]
    p = {n: base + i * 0x4000000 for i, n in enumerate(names)}
    N, M, R, r0, K = 300, 200, 8, 16, 100
    need = lib.lordba_ptq_workspace_bytes(N, M, R, r0)
    assert need >= 8 * 3 * (N + M) * R and need % 8 == 0
    assert lib.lordba_ptq_workspace_bytes(N, M, 33, 40) == 0 and lib.lordba_ptq_workspace_bytes(N, M, 8, 65) == 0
    assert lib.lordba_ptq_workspace_bytes(N, M, 8, 4) == 0                     # R may not exceed the factors' rank
    assert lib.lordba_ptq_workspace_bytes(0, M, R, r0) == 0

    def call(N=N, M=M, R=R, r0=r0, K=K, tau=2.0, mu=10.0, ws_bytes=need, **over):
        q = dict(p); q.update(over)
        return lib.lordba_ptq(q["A"], q["B"], q["pA"], q["pB"], q["al"], q["be"], q["ga"], q["si"], q["sr"], q["so"], q["info"],
                              q["ws"], ws_bytes, N, M, R, r0, K, ctypes.c_double(tau), ctypes.c_double(mu), None)

    for n in ("A", "B", "pA", "pB", "al", "be", "ga", "info", "ws"):
        assert call(**{n: None}) == 1, n
    assert call(R=0) == 2 and call(R=33, r0=40) == 2 and call(r0=4) == 2 and call(r0=65) == 2 and call(N=0) == 2
    assert call(K=0) == 2 and call(K=5000) == 2 and call(M=(1 << 22) + 1) == 2
    assert call(tau=1.0) == 3 and call(tau=float("nan")) == 3 and call(mu=0.0) == 3 and call(mu=-1.0) == 3
    assert call(ws_bytes=need - 8) == 9
    assert call(A=p["A"] + 1) == 5 and call(pA=p["pA"] + 2) == 5 and call(al=p["al"] + 4) == 5 and call(ws=p["ws"] + 4) == 5
    assert call(al=p["A"]) == 4 and call(ws=p["B"]) == 4 and call(ga=p["al"]) == 4 and call(info=p["ws"]) == 4
    assert call(si=p["sr"]) == 4
    piece = lambda t0, t1: lib.lordba_ptq_sweeps(p["A"], p["B"], p["pA"], p["pB"], p["al"], p["be"], p["ga"], p["si"], p["sr"], p["so"],
                                                 p["info"], p["ws"], need - 8, N, M, R, r0, K, t0, t1, ctypes.c_double(2.0),
                                                 ctypes.c_double(10.0), None)
    assert piece(-1, 5) == 2 and piece(6, 5) == 2 and piece(0, K + 1) == 2 and piece(3, 7) == 9   # the range, then the workspace size


def test_forward_multi_validation_needs_no_device(lib):
    base = 0x10000000
    x, pA, pB, si, sr, so, yb, yo = (base + i * 0x1000000 for i in range(8))
    T, d_in, d_out, r = 4, 64, 64, 8
    f = lambda *a: lib.lordba_forward_multi(*a, None)
    for ell in (1, 2, 3, 4):
        ok_args = [x, pA, pB, si, sr, so, yb, yo, T, d_in, d_out, r, ell]
        for i in range(8):
            a = list(ok_args); a[i] = None
            assert f(*a) == 1
        assert f(x, pA, pB, si, sr, so, yb, yo, 0, d_in, d_out, r, ell) == 0
        assert f(x, pA, pB, si, sr, so, yb, x, T, d_in, d_out, r, ell) == 4
        assert f(x + 1, pA, pB, si, sr, so, yb, yo, T, d_in, d_out, r, ell) == 5
        assert f(x, pA, pB, si, sr, so, yb, yo, T, d_in, d_out, 65, ell) == 2
    for ell in (0, -1, 5, 1 << 40):
        assert f(x, pA, pB, si, sr, so, yb, yo, T, d_in, d_out, r, ell) == 2
    # y_out overlapping the SECOND row of a scale array is only an overlap when there are two envelopes
    second_row = so + d_out * 2
    assert f(x, pA, pB, si, sr, so, yb, second_row, 1, d_in, d_out, r, 2) == 4
    assert lib.lordba_forward_multi_algo(x, pA, pB, si, sr, so, yb, yo, T, d_in, d_out, r, 2, None, 4) == 8


def test_forward_without_gpu_reports_no_device(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present; the parity tests cover the launch path")
    d = inputs.make_inputs(0, 4, 64, 64, 8)
    pA, pB = binding.lordba_pack_signs(d["signsA"], d["signsB"])
    y = np.zeros_like(d["y_base"])
    ptr = lambda a: ctypes.c_void_p(a.ctypes.data)
    st = lib.lordba_forward(ptr(d["x"]), ptr(pA), ptr(pB), ptr(d["s_in"]), ptr(d["s_rank"]), ptr(d["s_out"]),
                            ptr(d["y_base"]), ptr(y), 4, 64, 64, 8, None)
    assert st == 6


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_24058_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".cpp", ".h")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in src.replace("the CPU oracle", ""), fn
    assert "paper_2605_24058_amd" not in open(os.path.join(ROOT, "oracle", "__init__.py")).read().replace(
        "the product package", "")
