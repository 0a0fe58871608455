"""CPU oracle for the LoRDBA adapter branch: forward (Def. 1, Eq. (lordba) with one or
several scale envelopes, Eq. (adapter-mode-fwd), Eq. (lordba-fwd) of the paper) and the
backward pass of training with the smooth-sign straight-through factor (Eq. (smoothsign)).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and
by the ``cpu_baseline`` leg of ``bench.py``.  The product package never imports
this module, and this module never imports the product package.

The arithmetic lives in ``lordba_oracle.c`` (plain fp64 loops); this file only
compiles it with gcc, marshals numpy arrays through ctypes, and provides the
row-wise error metric the parity tests use.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lordba_oracle.c")
_LIB = os.path.join(_HERE, "liblordba_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared",
             "-Wall", "-Wextra", _SRC, "-o", tmp, "-lm", "-lpthread"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.lordba_oracle_f16_to_f64.restype = ctypes.c_double
        lib.lordba_oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
        lib.lordba_oracle_f16_array_to_f64.restype = None
        lib.lordba_oracle_f16_array_to_f64.argtypes = [vp, vp, i64]
        lib.lordba_oracle_pack.restype = ci
        lib.lordba_oracle_pack.argtypes = [vp, i64, i64, vp]
        lib.lordba_oracle_unpack.restype = None
        lib.lordba_oracle_unpack.argtypes = [vp, i64, i64, vp]
        lib.lordba_oracle_sign_f64.restype = ci
        lib.lordba_oracle_sign_f64.argtypes = [vp, i64, vp]
        lib.lordba_oracle_forward.restype = ci
        lib.lordba_oracle_forward.argtypes = [vp] * 8 + [i64] * 4 + [ci]
        lib.lordba_oracle_forward_packed.restype = ci
        lib.lordba_oracle_forward_packed.argtypes = [vp] * 8 + [i64] * 4 + [ci]
        lib.lordba_oracle_forward_batched.restype = ci
        lib.lordba_oracle_forward_batched.argtypes = [vp] * 9 + [i64] * 5
        lib.lordba_oracle_forward_batched_multi.restype = ci
        lib.lordba_oracle_forward_batched_multi.argtypes = [vp] * 9 + [i64] * 6
        lib.lordba_oracle_forward_multi.restype = ci
        lib.lordba_oracle_forward_multi.argtypes = [vp] * 8 + [i64] * 5 + [ci]
        lib.lordba_oracle_rank_intermediate.restype = ci
        lib.lordba_oracle_rank_intermediate.argtypes = [vp] * 4 + [i64] * 3
        lib.lordba_oracle_smooth_sign_grad.restype = ctypes.c_double
        lib.lordba_oracle_smooth_sign_grad.argtypes = [ctypes.c_double, ctypes.c_double]
        lib.lordba_oracle_backward.restype = ci
        lib.lordba_oracle_backward.argtypes = [vp] * 9 + [ctypes.c_double] + [vp] * 7 + [i64] * 4
        lib.lordba_oracle_backward_multi.restype = ci
        lib.lordba_oracle_backward_multi.argtypes = [vp] * 9 + [ctypes.c_double] + [vp] * 7 + [i64] * 5
        _lib = lib
    return _lib


def _as(a, dtype, shape=None):
    a = np.ascontiguousarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError("expected dtype %s, got %s" % (np.dtype(dtype), a.dtype))
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), tuple(a.shape)))
    return a


def _f16_bits(a, shape=None):
    """fp16 array -> its uint16 bit patterns (a view, no value conversion)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    return _as(a, np.uint16, shape)


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def f16_to_f64(bits) -> np.ndarray:
    """Decode fp16 bit patterns (uint16 or float16 array) with the oracle's own decoder."""
    b = _f16_bits(bits)
    out = np.empty(b.shape, dtype=np.float64)
    _load().lordba_oracle_f16_array_to_f64(_ptr(b), _ptr(out), b.size)
    return out


def packed_words(rows: int, cols: int) -> int:
    return (rows * cols + 31) // 32


def pack(signs) -> np.ndarray:
    """int8 +-1 matrix [rows, cols] -> canonical packed uint32 words (bit = 1 means -1)."""
    s = _as(signs, np.int8)
    if s.ndim != 2:
        raise ValueError("signs must be 2-D")
    rows, cols = s.shape
    words = np.empty(packed_words(rows, cols), dtype=np.uint32)
    st = _load().lordba_oracle_pack(_ptr(s), rows, cols, _ptr(words))
    if st != 0:
        raise ValueError("sign entries must be +1 or -1 (status %d)" % st)
    return words


def unpack(words, rows: int, cols: int) -> np.ndarray:
    w = _as(words, np.uint32, (packed_words(rows, cols),))
    out = np.empty((rows, cols), dtype=np.int8)
    _load().lordba_oracle_unpack(_ptr(w), rows, cols, _ptr(out))
    return out


def sign(u) -> np.ndarray:
    """Entry-wise sign with sign(0) = +1 (Sec. 2, Notation)."""
    u = _as(np.asarray(u, dtype=np.float64), np.float64)
    out = np.empty(u.shape, dtype=np.int8)
    st = _load().lordba_oracle_sign_f64(_ptr(u), u.size, _ptr(out))
    if st != 0:
        raise ValueError("NaN has no sign (status %d)" % st)
    return out


def forward(x, signsA, signsB, s_in, s_rank, s_out, y_base, nthreads: int = 1) -> np.ndarray:
    """fp64 Y = Y_base + X diag(s_in) S_A^T diag(s_rank) S_B^T diag(s_out).

    x[T,d_in], y_base[T,d_out], s_*: float16 (or their uint16 bit patterns);
    signsA[r,d_in], signsB[d_out,r]: int8 +-1.  Returns float64 [T,d_out].
    """
    sA = _as(signsA, np.int8)
    sB = _as(signsB, np.int8)
    r, d_in = sA.shape
    d_out = sB.shape[0]
    if sB.shape != (d_out, r):
        raise ValueError("signsB must be [d_out, r]")
    xb = _f16_bits(x)
    T = xb.shape[0]
    xb = _f16_bits(xb, (T, d_in))
    yb = _f16_bits(y_base, (T, d_out))
    si = _f16_bits(s_in, (d_in,))
    sr = _f16_bits(s_rank, (r,))
    so = _f16_bits(s_out, (d_out,))
    y = np.empty((T, d_out), dtype=np.float64)
    st = _load().lordba_oracle_forward(_ptr(xb), _ptr(sA), _ptr(sB), _ptr(si), _ptr(sr), _ptr(so),
                                       _ptr(yb), _ptr(y), T, d_in, d_out, r, int(nthreads))
    if st != 0:
        raise ValueError("oracle forward failed with status %d" % st)
    return y


def forward_multi(x, signsA, signsB, s_in, s_rank, s_out, y_base, nthreads: int = 1) -> np.ndarray:
    """fp64 Y = Y_base + X sum_e diag(s_in[e]) S_A^T diag(s_rank[e]) S_B^T diag(s_out[e])  (Eq. (lordba), l >= 1).

    s_in[ell,d_in], s_rank[ell,r], s_out[ell,d_out]: float16; the rest as in forward().
    """
    sA = _as(signsA, np.int8)
    sB = _as(signsB, np.int8)
    r, d_in = sA.shape
    d_out = sB.shape[0]
    if sB.shape != (d_out, r):
        raise ValueError("signsB must be [d_out, r]")
    si = _f16_bits(s_in)
    if si.ndim != 2:
        raise ValueError("s_in must be [ell, d_in]")
    ell = si.shape[0]
    si = _f16_bits(si, (ell, d_in))
    sr = _f16_bits(s_rank, (ell, r))
    so = _f16_bits(s_out, (ell, d_out))
    xb = _f16_bits(x)
    T = xb.shape[0]
    xb = _f16_bits(xb, (T, d_in))
    yb = _f16_bits(y_base, (T, d_out))
    y = np.empty((T, d_out), dtype=np.float64)
    st = _load().lordba_oracle_forward_multi(_ptr(xb), _ptr(sA), _ptr(sB), _ptr(si), _ptr(sr), _ptr(so),
                                             _ptr(yb), _ptr(y), T, d_in, d_out, r, ell, int(nthreads))
    if st != 0:
        raise ValueError("oracle forward_multi failed with status %d" % st)
    return y


def forward_batched(x, signsA, signsB, s_in, s_rank, s_out, adapter_of_row, y_base) -> np.ndarray:
    """fp64 Y[t] = Y_base[t] + X[t] DeltaW(adapter adapter_of_row[t]); rows with an id outside [0, n) pass through.

    signsA[n,r,d_in], signsB[n,d_out,r]: int8 +-1; s_in[n,d_in], s_rank[n,r], s_out[n,d_out]: float16;
    adapter_of_row[T]: int32."""
    sA = _as(signsA, np.int8)
    sB = _as(signsB, np.int8)
    if sA.ndim != 3 or sB.ndim != 3:
        raise ValueError("pools must be [n, r, d_in] and [n, d_out, r]")
    n, r, d_in = sA.shape
    d_out = sB.shape[1]
    if sB.shape != (n, d_out, r):
        raise ValueError("signsB must be [n, d_out, r]")
    si = _f16_bits(s_in, (n, d_in))
    sr = _f16_bits(s_rank, (n, r))
    so = _f16_bits(s_out, (n, d_out))
    xb = _f16_bits(x)
    T = xb.shape[0]
    xb = _f16_bits(xb, (T, d_in))
    yb = _f16_bits(y_base, (T, d_out))
    ids = _as(adapter_of_row, np.int32, (T,))
    y = np.empty((T, d_out), dtype=np.float64)
    st = _load().lordba_oracle_forward_batched(_ptr(xb), _ptr(sA), _ptr(sB), _ptr(si), _ptr(sr), _ptr(so), _ptr(ids),
                                               _ptr(yb), _ptr(y), T, d_in, d_out, r, n)
    if st != 0:
        raise ValueError("oracle forward_batched failed with status %d" % st)
    return y


def forward_batched_multi(x, signsA, signsB, s_in, s_rank, s_out, adapter_of_row, y_base) -> np.ndarray:
    """fp64 Y[t] = Y_base[t] + X[t] DeltaW(adapter adapter_of_row[t]) where every adapter of the pool has ell scale envelopes
    over its own carriers (Def. 1 / Eq. (lordba) with l = ell per adapter); rows with an id outside [0, n) pass through.

    signsA[n,r,d_in], signsB[n,d_out,r]: int8 +-1; s_in[n,ell,d_in], s_rank[n,ell,r], s_out[n,ell,d_out]: float16;
    adapter_of_row[T]: int32."""
    sA = _as(signsA, np.int8)
    sB = _as(signsB, np.int8)
    if sA.ndim != 3 or sB.ndim != 3:
        raise ValueError("pools must be [n, r, d_in] and [n, d_out, r]")
    n, r, d_in = sA.shape
    d_out = sB.shape[1]
    if sB.shape != (n, d_out, r):
        raise ValueError("signsB must be [n, d_out, r]")
    sr0 = np.asarray(s_rank)
    if sr0.ndim != 3:
        raise ValueError("s_rank must be [n, ell, r]")
    ell = sr0.shape[1]
    si = _f16_bits(s_in, (n, ell, d_in))
    sr = _f16_bits(s_rank, (n, ell, r))
    so = _f16_bits(s_out, (n, ell, d_out))
    xb = _f16_bits(x)
    T = xb.shape[0]
    xb = _f16_bits(xb, (T, d_in))
    yb = _f16_bits(y_base, (T, d_out))
    ids = _as(adapter_of_row, np.int32, (T,))
    y = np.empty((T, d_out), dtype=np.float64)
    st = _load().lordba_oracle_forward_batched_multi(_ptr(xb), _ptr(sA), _ptr(sB), _ptr(si), _ptr(sr), _ptr(so), _ptr(ids),
                                                     _ptr(yb), _ptr(y), T, d_in, d_out, r, ell, n)
    if st != 0:
        raise ValueError("oracle forward_batched_multi failed with status %d" % st)
    return y


def forward_packed(x, packedA, packedB, s_in, s_rank, s_out, y_base, r: int, nthreads: int = 1) -> np.ndarray:
    """Same map with canonical packed carriers, unpacked by the oracle's own unpacker."""
    xb = _f16_bits(x)
    T, d_in = xb.shape
    yb = _f16_bits(y_base)
    d_out = yb.shape[1]
    pA = _as(packedA, np.uint32, (packed_words(r, d_in),))
    pB = _as(packedB, np.uint32, (packed_words(d_out, r),))
    si = _f16_bits(s_in, (d_in,))
    sr = _f16_bits(s_rank, (r,))
    so = _f16_bits(s_out, (d_out,))
    yb = _f16_bits(yb, (T, d_out))
    y = np.empty((T, d_out), dtype=np.float64)
    st = _load().lordba_oracle_forward_packed(_ptr(xb), _ptr(pA), _ptr(pB), _ptr(si), _ptr(sr), _ptr(so),
                                              _ptr(yb), _ptr(y), T, d_in, d_out, r, int(nthreads))
    if st != 0:
        raise ValueError("oracle forward failed with status %d" % st)
    return y


def rank_intermediate(x, signsA, s_in) -> np.ndarray:
    """fp64 t = (X diag(s_in)) S_A^T [T, r], the inner two factors of Eq. (lordba-fwd)."""
    sA = _as(signsA, np.int8)
    r, d_in = sA.shape
    xb = _f16_bits(x)
    T = xb.shape[0]
    xb = _f16_bits(xb, (T, d_in))
    si = _f16_bits(s_in, (d_in,))
    t = np.empty((T, r), dtype=np.float64)
    st = _load().lordba_oracle_rank_intermediate(_ptr(xb), _ptr(sA), _ptr(si), _ptr(t), T, d_in, r)
    if st != 0:
        raise ValueError("oracle rank_intermediate failed with status %d" % st)
    return t


def smooth_sign_grad(u: float, kappa: float) -> float:
    """kappa (1 - tanh^2(kappa u)), the backward-pass stand-in for d sign(u)/du (Eq. (smoothsign))."""
    return float(_load().lordba_oracle_smooth_sign_grad(float(u), float(kappa)))


def backward(x, g, signsA, signsB, s_in, s_rank, s_out, latA, latB, kappa: float, dx_base=None) -> dict:
    """fp64 gradients of a loss with dL/dY = g through Y = Y_base + X diag(s_in) S_A^T diag(s_rank) S_B^T diag(s_out),
    the carriers' gradients passed through the smooth-sign factor of Eq. (smoothsign) at the latents.

    x[T,d_in], g[T,d_out], dx_base[T,d_in] (optional): float16; signsA[r,d_in], signsB[d_out,r]: int8 +-1;
    s_*: float16; latA[r,d_in], latB[d_out,r]: float32.  Returns a dict of float64 arrays
    dx[T,d_in], d_s_in[d_in], d_s_rank[r], d_s_out[d_out], d_latA[r,d_in], d_latB[d_out,r]."""
    sA = _as(signsA, np.int8)
    sB = _as(signsB, np.int8)
    r, d_in = sA.shape
    d_out = sB.shape[0]
    if sB.shape != (d_out, r):
        raise ValueError("signsB must be [d_out, r]")
    xb = _f16_bits(x)
    T = xb.shape[0]
    xb = _f16_bits(xb, (T, d_in))
    gb = _f16_bits(g, (T, d_out))
    si = _f16_bits(s_in, (d_in,))
    sr = _f16_bits(s_rank, (r,))
    so = _f16_bits(s_out, (d_out,))
    lA = _as(latA, np.float32, (r, d_in))
    lB = _as(latB, np.float32, (d_out, r))
    db = None if dx_base is None else _f16_bits(dx_base, (T, d_in))
    out = {"dx": np.empty((T, d_in)), "d_s_in": np.empty(d_in), "d_s_rank": np.empty(r), "d_s_out": np.empty(d_out),
           "d_latA": np.empty((r, d_in)), "d_latB": np.empty((d_out, r))}
    st = _load().lordba_oracle_backward(
        _ptr(xb), _ptr(gb), _ptr(sA), _ptr(sB), _ptr(si), _ptr(sr), _ptr(so), _ptr(lA), _ptr(lB), float(kappa),
        None if db is None else _ptr(db), _ptr(out["dx"]), _ptr(out["d_s_in"]), _ptr(out["d_s_rank"]),
        _ptr(out["d_s_out"]), _ptr(out["d_latA"]), _ptr(out["d_latB"]), T, d_in, d_out, r)
    if st != 0:
        raise ValueError("oracle backward failed with status %d" % st)
    return out


def backward_multi(x, g, signsA, signsB, s_in, s_rank, s_out, latA, latB, kappa: float, dx_base=None) -> dict:
    """backward() for an adapter with ell envelopes: s_in[ell,d_in], s_rank[ell,r], s_out[ell,d_out] (float16); the scale
    gradients come back with the same leading envelope index."""
    sA = _as(signsA, np.int8)
    sB = _as(signsB, np.int8)
    r, d_in = sA.shape
    d_out = sB.shape[0]
    si = _f16_bits(s_in)
    if si.ndim != 2:
        raise ValueError("s_in must be [ell, d_in]")
    ell = si.shape[0]
    si = _f16_bits(si, (ell, d_in))
    sr = _f16_bits(s_rank, (ell, r))
    so = _f16_bits(s_out, (ell, d_out))
    xb = _f16_bits(x)
    T = xb.shape[0]
    xb = _f16_bits(xb, (T, d_in))
    gb = _f16_bits(g, (T, d_out))
    lA = _as(latA, np.float32, (r, d_in))
    lB = _as(latB, np.float32, (d_out, r))
    db = None if dx_base is None else _f16_bits(dx_base, (T, d_in))
    out = {"dx": np.empty((T, d_in)), "d_s_in": np.empty((ell, d_in)), "d_s_rank": np.empty((ell, r)),
           "d_s_out": np.empty((ell, d_out)), "d_latA": np.empty((r, d_in)), "d_latB": np.empty((d_out, r))}
    st = _load().lordba_oracle_backward_multi(
        _ptr(xb), _ptr(gb), _ptr(sA), _ptr(sB), _ptr(si), _ptr(sr), _ptr(so), _ptr(lA), _ptr(lB), float(kappa),
        None if db is None else _ptr(db), _ptr(out["dx"]), _ptr(out["d_s_in"]), _ptr(out["d_s_rank"]),
        _ptr(out["d_s_out"]), _ptr(out["d_latA"]), _ptr(out["d_latB"]), T, d_in, d_out, r, ell)
    if st != 0:
        raise ValueError("oracle backward_multi failed with status %d" % st)
    return out


def rel_l2(a_test, a_ref) -> float:
    """||a_test - a_ref||_2 / ||a_ref||_2 over a whole array (0 if both are exactly 0, inf if only the reference is)."""
    a = np.asarray(a_test, dtype=np.float64).ravel()
    b = np.asarray(a_ref, dtype=np.float64).ravel()
    num, den = np.sqrt(((a - b) ** 2).sum()), np.sqrt((b ** 2).sum())
    if den > 0:
        return float(num / den)
    return 0.0 if num == 0 else float("inf")


def row_rel_l2(y_test, y_ref) -> np.ndarray:
    """Per token row: ||y_test - y_ref||_2 / ||y_ref||_2 in fp64.

    A row whose reference norm is 0 scores 0 if y_test is exactly 0 there, else inf.
    """
    a = np.asarray(y_test, dtype=np.float64)
    b = np.asarray(y_ref, dtype=np.float64)
    num = np.sqrt(((a - b) ** 2).sum(axis=1))
    den = np.sqrt((b ** 2).sum(axis=1))
    out = np.empty_like(num)
    nz = den > 0
    out[nz] = num[nz] / den[nz]
    out[~nz] = np.where(num[~nz] == 0, 0.0, np.inf)
    return out


def available_cores() -> int:
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        return os.cpu_count() or 1
