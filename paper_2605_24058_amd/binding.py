"""ctypes binding of liblordba.so (argument marshalling only; every step of the path runs in the
library's HIP kernels).  Names and argument order follow include/lordba.h.

torch is used for device memory and streams only: tensors are passed as raw device pointers and
the current torch stream is passed as the hipStream_t.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import sys
from typing import Optional, Tuple

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
_CSRC = os.path.join(_PKG, "csrc")
_LIB_PATH = os.path.join(_PKG, "liblordba.so")
# one translation unit per kernel family and kind (inference / training): they compile side by side
_SOURCES = ("lordba_forward.hip", "lordba_forward_train.hip", "lordba_forward_multi_l2.hip", "lordba_forward_multi_l3.hip",
            "lordba_forward_multi_l4.hip", "lordba_forward_multi_train.hip", "lordba_forward_multi.hip", "lordba_backward.hip",
            "lordba_ptq.hip", "lordba_pack_device.hip", "lordba_pack.cpp")
_lib = None

ALGO_AUTO, ALGO_GENERAL, ALGO_MFMA_T8, ALGO_MFMA_T16 = 0, 1, 2, 3

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument"]


class LordbaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: status %d (%s)" % (where, status, lordba_status_string(status)))


def build_library(verbose: bool = False) -> str:
    """Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU).  The translation units are
    compiled side by side (the kernel templates take most of the time), then linked."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tag = ".tmp.%d" % os.getpid()
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    objs, procs = [], []
    for src in _SOURCES:
        obj = os.path.join(_PKG, src + tag + ".o")
        cmd = [hipcc] + flags + ["-I", os.path.join(_ROOT, "include"), "-c", os.path.join(_CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), file=sys.stderr)
        objs.append(obj)
        procs.append(subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    outs = [p.communicate()[0] for p in procs]
    tmp = _LIB_PATH + tag
    try:
        for p, out in zip(procs, outs):
            out = "\n".join(l for l in out.splitlines() if "not a recognized feature for this target" not in l)
            if p.returncode != 0:
                raise RuntimeError("hipcc failed:\n" + out)
            if verbose and out.strip():
                print(out, file=sys.stderr)
        link = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp],
                              stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if link.returncode != 0:
            raise RuntimeError("link failed:\n" + link.stdout)
        os.replace(tmp, _LIB_PATH)
    finally:
        for f in objs + [tmp]:
            if os.path.exists(f):
                os.remove(f)
    return _LIB_PATH


_BENCH_LIB_PATH = os.path.join(_PKG, "libmembench.so")
_bench_lib = None


def build_bench_library(verbose: bool = False) -> str:
    """Compile the streaming reference kernels that bench.py times next to the adapter kernel."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = _BENCH_LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + [os.path.join(_CSRC, "membench.hip"), "-o", tmp]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    os.replace(tmp, _BENCH_LIB_PATH)
    return _BENCH_LIB_PATH


def load_bench_library():
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(_BENCH_LIB_PATH):
            raise RuntimeError("libmembench.so is not built: run __graft_entry__.build() first")
        lib = ctypes.CDLL(_BENCH_LIB_PATH)
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.lordba_bench_stream.restype = ctypes.c_int
        lib.lordba_bench_stream.argtypes = [vp, vp, vp, i64, i64, vp]
        lib.lordba_bench_copy.restype = ctypes.c_int
        lib.lordba_bench_copy.argtypes = [vp, vp, i64, vp]
        lib.lordba_bench_empty.restype = ctypes.c_int
        lib.lordba_bench_empty.argtypes = [vp]
        _bench_lib = lib
    return _bench_lib


def load_library():
    """Load liblordba.so; there is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("liblordba.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(or paper_2605_24058_amd.build_library()) first; there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.lordba_packed_words.restype = ctypes.c_size_t
    lib.lordba_packed_words.argtypes = [i64, i64]
    for name in ("lordba_pack_signs", "lordba_pack_signs_f32", "lordba_unpack_signs"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [vp, vp, vp, vp, i64, i64, i64]
    lib.lordba_forward.restype = ci
    lib.lordba_forward.argtypes = [vp] * 8 + [i64] * 4 + [vp]
    lib.lordba_forward_algo.restype = ci
    lib.lordba_forward_algo.argtypes = [vp] * 8 + [i64] * 4 + [vp, ci]
    for name, extra in (("lordba_forward_multi", [vp]), ("lordba_forward_multi_algo", [vp, ci])):
        f = getattr(lib, name)      # AttributeError if the library was built from older sources: rebuild it
        f.restype = ci
        f.argtypes = [vp] * 8 + [i64] * 5 + extra
    for name, extra in (("lordba_forward_batched", [vp]), ("lordba_forward_batched_algo", [vp, ci])):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [vp] * 9 + [i64] * 5 + extra
    for name, extra in (("lordba_forward_batched_multi", [vp]), ("lordba_forward_batched_multi_algo", [vp, ci])):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [vp] * 9 + [i64] * 6 + extra
    lib.lordba_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.lordba_backward_workspace_bytes.argtypes = [i64] * 4
    lib.lordba_backward_multi_workspace_bytes.restype = ctypes.c_size_t
    lib.lordba_backward_multi_workspace_bytes.argtypes = [i64] * 5
    lib.lordba_backward.restype = ci
    lib.lordba_backward.argtypes = [vp] * 10 + [ctypes.c_float, vp, i64] + [vp] * 8 + [ctypes.c_size_t] + [i64] * 4 + [vp]
    lib.lordba_backward_noalloc.restype = ci
    lib.lordba_backward_noalloc.argtypes = [vp] * 10 + [ctypes.c_float, vp, i64] + [vp] * 7 + [i64] * 4 + [vp]
    lib.lordba_backward_multi.restype = ci
    lib.lordba_backward_multi.argtypes = [vp] * 10 + [ctypes.c_float, vp, i64] + [vp] * 8 + [ctypes.c_size_t] + [i64] * 5 + [vp]
    lib.lordba_forward_multi_save_t.restype = ci
    lib.lordba_forward_multi_save_t.argtypes = [vp] * 9 + [i64] * 6 + [vp]
    lib.lordba_pack_latents.restype = ci
    lib.lordba_pack_latents.argtypes = [vp] * 6 + [i64] * 3 + [vp]
    lib.lordba_forward_save_t.restype = ci
    lib.lordba_forward_save_t.argtypes = [vp] * 9 + [i64] * 5 + [vp]
    lib.lordba_ptq_workspace_bytes.restype = ctypes.c_size_t
    lib.lordba_ptq_workspace_bytes.argtypes = [i64] * 4
    lib.lordba_ptq.restype = ci
    lib.lordba_ptq.argtypes = [vp] * 12 + [ctypes.c_size_t] + [i64] * 5 + [ctypes.c_double, ctypes.c_double, vp]
    lib.lordba_ptq_sweeps.restype = ci
    lib.lordba_ptq_sweeps.argtypes = [vp] * 12 + [ctypes.c_size_t] + [i64] * 7 + [ctypes.c_double, ctypes.c_double, vp]
    lib.lordba_ptq_beta_solve.restype = ci
    lib.lordba_ptq_beta_solve.argtypes = [vp, vp, vp, i64, vp]
    lib.lordba_status_string.restype = ctypes.c_char_p
    lib.lordba_status_string.argtypes = [ci]
    _lib = lib
    return lib


def lordba_status_string(status: int) -> str:
    return load_library().lordba_status_string(int(status)).decode()


def lordba_packed_words(rows: int, cols: int) -> int:
    return int(load_library().lordba_packed_words(rows, cols))


def _np_ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def lordba_pack_signs(signsA, signsB) -> Tuple[np.ndarray, np.ndarray]:
    """Host packing.  signsA [r, d_in], signsB [d_out, r]: int8 +-1, or float32 latents (sign(0) = +1).
    Returns (packedA, packedB) as uint32 numpy arrays in the canonical format."""
    lib = load_library()
    A = np.ascontiguousarray(signsA)
    B = np.ascontiguousarray(signsB)
    if A.ndim != 2 or B.ndim != 2 or B.shape[1] != A.shape[0]:
        raise ValueError("need signsA [r, d_in] and signsB [d_out, r]")
    if A.dtype != B.dtype or A.dtype not in (np.dtype(np.int8), np.dtype(np.float32)):
        raise TypeError("carriers must both be int8 (+-1) or both float32 (latents)")
    r, d_in = A.shape
    d_out = B.shape[0]
    pA = np.empty(max(lordba_packed_words(r, d_in), 1), dtype=np.uint32)[:lordba_packed_words(r, d_in)]
    pB = np.empty(max(lordba_packed_words(d_out, r), 1), dtype=np.uint32)[:lordba_packed_words(d_out, r)]
    fn = lib.lordba_pack_signs if A.dtype == np.int8 else lib.lordba_pack_signs_f32
    st = fn(_np_ptr(A), _np_ptr(B), _np_ptr(pA), _np_ptr(pB), d_in, d_out, r)
    if st != 0:
        raise LordbaError(st, fn.__name__)
    return pA, pB


def lordba_unpack_signs(packedA, packedB, d_in: int, d_out: int, r: int) -> Tuple[np.ndarray, np.ndarray]:
    lib = load_library()
    pA = np.ascontiguousarray(packedA, dtype=np.uint32)
    pB = np.ascontiguousarray(packedB, dtype=np.uint32)
    if pA.size != lordba_packed_words(r, d_in) or pB.size != lordba_packed_words(d_out, r):
        raise ValueError("packed buffers have the wrong length")
    A = np.empty((r, d_in), dtype=np.int8)
    B = np.empty((d_out, r), dtype=np.int8)
    st = lib.lordba_unpack_signs(_np_ptr(pA), _np_ptr(pB), _np_ptr(A), _np_ptr(B), d_in, d_out, r)
    if st != 0:
        raise LordbaError(st, "lordba_unpack_signs")
    return A, B


def lordba_forward(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out=None, stream=None,
                   algo: int = ALGO_AUTO, check: bool = True):
    """y_out = y_base + adapter branch, on the GPU.  All arguments are torch CUDA tensors:
    x [T, d_in] f16, packedA / packedB int32 (the uint32 words, reinterpreted), s_in [d_in], s_rank [r],
    s_out [d_out], y_base [T, d_out] f16.  y_out defaults to a new tensor; pass y_base itself for in-place.
    Enqueues on `stream` (default: torch's current stream) and returns y_out without synchronising."""
    import torch

    lib = load_library()
    if check:
        for name, t_ in (("x", x), ("s_in", s_in), ("s_rank", s_rank), ("s_out", s_out), ("y_base", y_base)):
            if t_.dtype != torch.float16 or not t_.is_cuda or not t_.is_contiguous():
                raise TypeError("%s must be a contiguous float16 CUDA tensor" % name)
        for name, t_ in (("packedA", packedA), ("packedB", packedB)):
            if t_.dtype != torch.int32 or not t_.is_cuda or not t_.is_contiguous():
                raise TypeError("%s must be a contiguous int32 CUDA tensor holding the packed words" % name)
        if x.dim() != 2 or y_base.dim() != 2 or x.shape[0] != y_base.shape[0]:
            raise ValueError("x must be [T, d_in] and y_base [T, d_out]")
    T, d_in = x.shape
    d_out = y_base.shape[1]
    r = s_rank.numel()
    if check:
        if s_in.numel() != d_in or s_out.numel() != d_out:
            raise ValueError("scale vector lengths do not match x / y_base")
        if packedA.numel() != (r * d_in + 31) // 32 or packedB.numel() != (d_out * r + 31) // 32:
            raise ValueError("packed carrier lengths do not match the shape")
    if y_out is None:
        y_out = torch.empty_like(y_base)
    elif check and (y_out.dtype != torch.float16 or not y_out.is_cuda or not y_out.is_contiguous()
                    or y_out.shape != y_base.shape):
        raise TypeError("y_out must be a contiguous float16 CUDA tensor shaped like y_base")
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    args = (x.data_ptr(), packedA.data_ptr(), packedB.data_ptr(), s_in.data_ptr(), s_rank.data_ptr(), s_out.data_ptr(),
            y_base.data_ptr(), y_out.data_ptr(), T, d_in, d_out, r, ctypes.c_void_p(stream))
    # the library's own choice of kernel goes through the entry point of that name; a selector through its _algo twin
    st = lib.lordba_forward(*args) if int(algo) == ALGO_AUTO else lib.lordba_forward_algo(*args, int(algo))
    if st != 0:
        raise LordbaError(st, "lordba_forward")
    return y_out


def lordba_forward_multi(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out=None, stream=None,
                         algo: int = ALGO_AUTO, check: bool = True):
    """y_out = y_base + the branch of an adapter with ell scale envelopes over the same carriers, on the GPU.
    As lordba_forward, with s_in [ell, d_in], s_rank [ell, r], s_out [ell, d_out] (float16, contiguous)."""
    import torch

    lib = load_library()
    if check:
        for name, t_ in (("x", x), ("s_in", s_in), ("s_rank", s_rank), ("s_out", s_out), ("y_base", y_base)):
            if t_.dtype != torch.float16 or not t_.is_cuda or not t_.is_contiguous():
                raise TypeError("%s must be a contiguous float16 CUDA tensor" % name)
        for name, t_ in (("packedA", packedA), ("packedB", packedB)):
            if t_.dtype != torch.int32 or not t_.is_cuda or not t_.is_contiguous():
                raise TypeError("%s must be a contiguous int32 CUDA tensor holding the packed words" % name)
        if x.dim() != 2 or y_base.dim() != 2 or x.shape[0] != y_base.shape[0]:
            raise ValueError("x must be [T, d_in] and y_base [T, d_out]")
        if s_in.dim() != 2 or s_rank.dim() != 2 or s_out.dim() != 2:
            raise ValueError("s_in, s_rank, s_out must be [ell, d_in], [ell, r], [ell, d_out]")
    T, d_in = x.shape
    d_out = y_base.shape[1]
    ell, r = s_rank.shape
    if check:
        if tuple(s_in.shape) != (ell, d_in) or tuple(s_out.shape) != (ell, d_out):
            raise ValueError("scale array shapes do not match x / y_base / ell")
        if packedA.numel() != (r * d_in + 31) // 32 or packedB.numel() != (d_out * r + 31) // 32:
            raise ValueError("packed carrier lengths do not match the shape")
    if y_out is None:
        y_out = torch.empty_like(y_base)
    elif check and (y_out.dtype != torch.float16 or not y_out.is_cuda or not y_out.is_contiguous()
                    or y_out.shape != y_base.shape):
        raise TypeError("y_out must be a contiguous float16 CUDA tensor shaped like y_base")
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    args = (x.data_ptr(), packedA.data_ptr(), packedB.data_ptr(), s_in.data_ptr(), s_rank.data_ptr(), s_out.data_ptr(),
            y_base.data_ptr(), y_out.data_ptr(), T, d_in, d_out, r, ell, ctypes.c_void_p(stream))
    st = lib.lordba_forward_multi(*args) if int(algo) == ALGO_AUTO else lib.lordba_forward_multi_algo(*args, int(algo))
    if st != 0:
        raise LordbaError(st, "lordba_forward_multi")
    return y_out


def lordba_pack_pool(signsA_pool, signsB_pool) -> Tuple[np.ndarray, np.ndarray]:
    """Packs every adapter of a pool (signsA_pool [n, r, d_in], signsB_pool [n, d_out, r]) with lordba_pack_signs and
    stacks the results: uint32 [n, words_A], [n, words_B]."""
    packed = [lordba_pack_signs(a, b) for a, b in zip(signsA_pool, signsB_pool)]
    return np.stack([p[0] for p in packed]), np.stack([p[1] for p in packed])


def lordba_forward_batched(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, adapter_of_row, y_base,
                           y_out=None, stream=None, algo: int = ALGO_AUTO, check: bool = True):
    """y_out[t] = y_base[t] + the branch of adapter adapter_of_row[t] of a pool, on the GPU.  Pools are torch CUDA tensors
    stacked over the adapter index: packedA_pool / packedB_pool int32 [n, words], s_*_pool float16 [n, .];
    adapter_of_row int32 [T] (an index outside [0, n) = no adapter)."""
    import torch

    lib = load_library()
    if check:
        for name, t_ in (("x", x), ("s_in_pool", s_in_pool), ("s_rank_pool", s_rank_pool), ("s_out_pool", s_out_pool),
                         ("y_base", y_base)):
            if t_.dtype != torch.float16 or not t_.is_cuda or not t_.is_contiguous():
                raise TypeError("%s must be a contiguous float16 CUDA tensor" % name)
        for name, t_ in (("packedA_pool", packedA_pool), ("packedB_pool", packedB_pool), ("adapter_of_row", adapter_of_row)):
            if t_.dtype != torch.int32 or not t_.is_cuda or not t_.is_contiguous():
                raise TypeError("%s must be a contiguous int32 CUDA tensor" % name)
        if x.dim() != 2 or y_base.dim() != 2 or x.shape[0] != y_base.shape[0] or adapter_of_row.numel() != x.shape[0]:
            raise ValueError("x must be [T, d_in], y_base [T, d_out], adapter_of_row [T]")
        if s_rank_pool.dim() != 2 or packedA_pool.dim() != 2 or packedB_pool.dim() != 2:
            raise ValueError("pools must be stacked over the adapter index")
    T, d_in = x.shape
    d_out = y_base.shape[1]
    n, r = s_rank_pool.shape
    if check:
        if tuple(s_in_pool.shape) != (n, d_in) or tuple(s_out_pool.shape) != (n, d_out):
            raise ValueError("scale pool shapes do not match")
        if tuple(packedA_pool.shape) != (n, (r * d_in + 31) // 32) or tuple(packedB_pool.shape) != (n, (d_out * r + 31) // 32):
            raise ValueError("packed pool shapes do not match")
    if y_out is None:
        y_out = torch.empty_like(y_base)
    elif check and (y_out.dtype != torch.float16 or not y_out.is_cuda or not y_out.is_contiguous()
                    or y_out.shape != y_base.shape):
        raise TypeError("y_out must be a contiguous float16 CUDA tensor shaped like y_base")
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    args = (x.data_ptr(), packedA_pool.data_ptr(), packedB_pool.data_ptr(), s_in_pool.data_ptr(), s_rank_pool.data_ptr(),
            s_out_pool.data_ptr(), adapter_of_row.data_ptr(), y_base.data_ptr(), y_out.data_ptr(), T, d_in, d_out, r, n,
            ctypes.c_void_p(stream))
    st = lib.lordba_forward_batched(*args) if int(algo) == ALGO_AUTO else lib.lordba_forward_batched_algo(*args, int(algo))
    if st != 0:
        raise LordbaError(st, "lordba_forward_batched")
    return y_out


def lordba_forward_batched_multi(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, adapter_of_row, y_base,
                                 y_out=None, stream=None, algo: int = ALGO_AUTO):
    """lordba_forward_batched for a pool whose adapters have ell scale envelopes each: s_in_pool [n, ell, d_in],
    s_rank_pool [n, ell, r], s_out_pool [n, ell, d_out] (float16 CUDA tensors); everything else as lordba_forward_batched."""
    import torch

    lib = load_library()
    for name, t_ in (("x", x), ("s_in_pool", s_in_pool), ("s_rank_pool", s_rank_pool), ("s_out_pool", s_out_pool), ("y_base", y_base)):
        if t_.dtype != torch.float16 or not t_.is_cuda or not t_.is_contiguous():
            raise TypeError("%s must be a contiguous float16 CUDA tensor" % name)
    for name, t_ in (("packedA_pool", packedA_pool), ("packedB_pool", packedB_pool), ("adapter_of_row", adapter_of_row)):
        if t_.dtype != torch.int32 or not t_.is_cuda or not t_.is_contiguous():
            raise TypeError("%s must be a contiguous int32 CUDA tensor" % name)
    if x.dim() != 2 or y_base.dim() != 2 or x.shape[0] != y_base.shape[0] or adapter_of_row.numel() != x.shape[0]:
        raise ValueError("x must be [T, d_in], y_base [T, d_out], adapter_of_row [T]")
    if s_rank_pool.dim() != 3:
        raise ValueError("scale pools must be [n, ell, .]")
    T, d_in = x.shape
    d_out = y_base.shape[1]
    n, ell, r = s_rank_pool.shape
    if tuple(s_in_pool.shape) != (n, ell, d_in) or tuple(s_out_pool.shape) != (n, ell, d_out):
        raise ValueError("scale pool shapes do not match")
    if tuple(packedA_pool.shape) != (n, (r * d_in + 31) // 32) or tuple(packedB_pool.shape) != (n, (d_out * r + 31) // 32):
        raise ValueError("packed pool shapes do not match")
    if y_out is None:
        y_out = torch.empty_like(y_base)
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    args = (x.data_ptr(), packedA_pool.data_ptr(), packedB_pool.data_ptr(), s_in_pool.data_ptr(), s_rank_pool.data_ptr(),
            s_out_pool.data_ptr(), adapter_of_row.data_ptr(), y_base.data_ptr(), y_out.data_ptr(), T, d_in, d_out, r, ell, n,
            ctypes.c_void_p(stream))
    st = lib.lordba_forward_batched_multi(*args) if int(algo) == ALGO_AUTO else lib.lordba_forward_batched_multi_algo(*args, int(algo))
    if st != 0:
        raise LordbaError(st, "lordba_forward_batched_multi")
    return y_out


def lordba_backward_workspace_bytes(T: int, d_in: int, d_out: int, r: int) -> int:
    return int(load_library().lordba_backward_workspace_bytes(T, d_in, d_out, r))


def lordba_backward_multi_workspace_bytes(T: int, d_in: int, d_out: int, r: int, ell: int) -> int:
    return int(load_library().lordba_backward_multi_workspace_bytes(T, d_in, d_out, r, ell))


def lordba_pack_transposed(signsA, signsB) -> Tuple[np.ndarray, np.ndarray]:
    """The two extra packed carriers lordba_backward takes: S_A^T as [d_in, r] and S_B^T as [r, d_out], packed by the
    library's host packer in the canonical format.  Returns (packedAt, packedBt)."""
    A = np.ascontiguousarray(np.asarray(signsA).T)   # [d_in, r]
    B = np.ascontiguousarray(np.asarray(signsB).T)   # [r, d_out]
    # lordba_pack_signs(signsA [r', d_in'], signsB [d_out', r']) with r' = r, d_in' = d_out, d_out' = d_in
    pBt, pAt = lordba_pack_signs(B, A)
    return pAt, pBt


def lordba_pack_latents(latentA, latentB, stream=None, transposed: bool = True):
    """Device-side binarisation and packing of the latent carriers (torch CUDA float32 tensors latentA [r, d_in],
    latentB [d_out, r]).  Returns int32 CUDA tensors (packedA, packedB, packedAt, packedBt); the last two are None unless
    `transposed`."""
    import torch

    lib = load_library()
    r, d_in = latentA.shape
    d_out = latentB.shape[0]
    if tuple(latentB.shape) != (d_out, r) or latentA.dtype != torch.float32 or latentB.dtype != torch.float32:
        raise ValueError("need float32 latentA [r, d_in] and latentB [d_out, r]")
    wA, wB = (r * d_in + 31) // 32, (d_out * r + 31) // 32
    new = lambda n: torch.empty(n, dtype=torch.int32, device=latentA.device)
    pA, pB = new(wA), new(wB)
    pAt, pBt = (new(wA), new(wB)) if transposed else (None, None)
    if stream is None:
        stream = torch.cuda.current_stream(latentA.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    ptr = lambda t_: None if t_ is None else t_.data_ptr()
    st = lib.lordba_pack_latents(latentA.contiguous().data_ptr(), latentB.contiguous().data_ptr(), pA.data_ptr(), pB.data_ptr(),
                                 ptr(pAt), ptr(pBt), d_in, d_out, r, ctypes.c_void_p(stream))
    if st != 0:
        raise LordbaError(st, "lordba_pack_latents")
    return pA, pB, pAt, pBt


def saved_t_stride(T: int) -> int:
    """Row stride (in floats) of a kept rank-r intermediate that lordba_backward accepts: T rounded up to a multiple of 128."""
    return (int(T) + 127) // 128 * 128


def lordba_forward_save_t(x, packedA, packedB, s_in, s_rank, s_out, y_base=None, y_out=None, t_out=None, stream=None):
    """The training forward: lordba_forward that also writes the rank-r intermediate t = (x diag(s_in)) S_A^T, fp32,
    rank-major [r, saved_t_stride(T)] (entries past T untouched).  y_base = None: only t is computed.
    Returns (y_out or None, t_out)."""
    import torch

    lib = load_library()
    T, d_in = x.shape
    r = s_rank.numel()
    d_out = s_out.numel()
    stride = saved_t_stride(T) if t_out is None else t_out.shape[1]
    if t_out is None:
        t_out = torch.empty((r, stride), dtype=torch.float32, device=x.device)
    if y_base is not None and y_out is None:
        y_out = torch.empty_like(y_base)
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    ptr = lambda t_: None if t_ is None else t_.data_ptr()
    st = lib.lordba_forward_save_t(x.data_ptr(), packedA.data_ptr(), packedB.data_ptr(), s_in.data_ptr(), s_rank.data_ptr(),
                                   s_out.data_ptr(), ptr(y_base), ptr(y_out), t_out.data_ptr(), stride, T, d_in, d_out, r,
                                   ctypes.c_void_p(stream))
    if st != 0:
        raise LordbaError(st, "lordba_forward_save_t")
    return y_out, t_out


def lordba_backward(x, g, packedA, packedAt, packedBt, s_in, s_rank, s_out, latentA, latentB, kappa: float,
                    dx_base=None, dx=None, workspace=None, stream=None, check: bool = True, t_saved=None,
                    _noalloc: bool = False, out: Optional[dict] = None) -> dict:
    """Gradients of the branch on the GPU (see include/lordba.h).  All tensors are torch CUDA tensors: x [T, d_in],
    g [T, d_out], s_* float16; packed* int32; latentA [r, d_in], latentB [d_out, r] float32; dx_base [T, d_in] float16
    or None (then no input gradient is computed); t_saved: the float32 [r, stride] tensor lordba_forward_save_t returned
    for this x, or None (recomputed).  workspace: a uint8 CUDA tensor of at least
    lordba_backward_workspace_bytes(...) bytes (allocated here if None).  Returns a dict of new tensors dx (or None),
    d_s_in, d_s_rank, d_s_out, d_latentA, d_latentB; enqueues on `stream` without synchronising."""
    import torch

    lib = load_library()
    if check:
        for name, t_ in (("x", x), ("g", g), ("s_in", s_in), ("s_rank", s_rank), ("s_out", s_out)):
            if t_.dtype != torch.float16 or not t_.is_cuda or not t_.is_contiguous():
                raise TypeError("%s must be a contiguous float16 CUDA tensor" % name)
        for name, t_ in (("packedA", packedA), ("packedAt", packedAt), ("packedBt", packedBt)):
            if t_.dtype != torch.int32 or not t_.is_cuda or not t_.is_contiguous():
                raise TypeError("%s must be a contiguous int32 CUDA tensor holding the packed words" % name)
        if (latentA is None) != (latentB is None):
            raise ValueError("latentA and latentB come or go together (both None: frozen carriers, no latent gradients)")
        for name, t_ in (("latentA", latentA), ("latentB", latentB)):
            if t_ is not None and (t_.dtype != torch.float32 or not t_.is_cuda or not t_.is_contiguous()):
                raise TypeError("%s must be a contiguous float32 CUDA tensor" % name)
        if x.dim() != 2 or g.dim() != 2 or x.shape[0] != g.shape[0]:
            raise ValueError("x must be [T, d_in] and g [T, d_out]")
    T, d_in = x.shape
    d_out = g.shape[1]
    r = s_rank.numel()
    if check:
        if s_in.numel() != d_in or s_out.numel() != d_out or (latentA is not None and (
                tuple(latentA.shape) != (r, d_in) or tuple(latentB.shape) != (d_out, r))):
            raise ValueError("scale / latent shapes do not match x / g")
        words = ((r * d_in + 31) // 32, (r * d_out + 31) // 32)
        if packedA.numel() != words[0] or packedAt.numel() != words[0] or packedBt.numel() != words[1]:
            raise ValueError("packed carrier lengths do not match the shape")
        if dx_base is not None and (dx_base.dtype != torch.float16 or not dx_base.is_cuda or not dx_base.is_contiguous()
                                    or dx_base.shape != x.shape):
            raise TypeError("dx_base must be a contiguous float16 CUDA tensor shaped like x")
    if workspace is None and not _noalloc:
        workspace = torch.empty(max(lordba_backward_workspace_bytes(T, d_in, d_out, r), 16), dtype=torch.uint8, device=x.device)
    if out is not None:
        dx = out["dx"]
    elif dx_base is not None and dx is None:
        dx = torch.empty_like(dx_base)
    f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device=x.device)
    if out is None:
        out = {"dx": dx, "d_s_in": f32(d_in), "d_s_rank": f32(r), "d_s_out": f32(d_out),
               "d_latentA": None if latentA is None else f32(r, d_in), "d_latentB": None if latentB is None else f32(d_out, r)}
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    ptr = lambda t_: None if t_ is None else t_.data_ptr()
    head = (x.data_ptr(), g.data_ptr(), packedA.data_ptr(), packedAt.data_ptr(), packedBt.data_ptr(),
            s_in.data_ptr(), s_rank.data_ptr(), s_out.data_ptr(), ptr(latentA), ptr(latentB),
            float(kappa), ptr(t_saved), 0 if t_saved is None else t_saved.shape[1],
            ptr(dx_base), ptr(dx), out["d_s_in"].data_ptr(), out["d_s_rank"].data_ptr(),
            out["d_s_out"].data_ptr(), ptr(out["d_latentA"]), ptr(out["d_latentB"]))
    tail = (T, d_in, d_out, r, ctypes.c_void_p(stream))
    if _noalloc:
        st = lib.lordba_backward_noalloc(*head, *tail)
    else:
        st = lib.lordba_backward(*head, workspace.data_ptr(), workspace.numel(), *tail)
    if st != 0:
        raise LordbaError(st, "lordba_backward_noalloc" if _noalloc else "lordba_backward")
    return out


BACKWARD_NOALLOC_MAX_BYTES = 16 * 1024 * 1024   # LORDBA_BACKWARD_NOALLOC_MAX_BYTES of include/lordba.h


def lordba_backward_noalloc(x, g, packedA, packedAt, packedBt, s_in, s_rank, s_out, latentA, latentB, kappa: float,
                            dx_base=None, stream=None, t_saved=None, out: Optional[dict] = None) -> dict:
    """lordba_backward_noalloc of the C interface: lordba_backward with the scratch in the library's own device array
    instead of a workspace.  The C call allocates nothing; this wrapper allocates the output tensors unless `out` (the
    dict of an earlier call of the same shape) is passed, in which case nothing at all is allocated."""
    return lordba_backward(x, g, packedA, packedAt, packedBt, s_in, s_rank, s_out, latentA, latentB, kappa,
                           dx_base=dx_base, stream=stream, t_saved=t_saved, _noalloc=True, out=out)


def lordba_forward_multi_save_t(x, packedA, packedB, s_in, s_rank, s_out, y_base=None, y_out=None, t_out=None, stream=None):
    """lordba_forward_save_t for ell envelopes (s_in [ell, d_in], s_rank [ell, r], s_out [ell, d_out]): t_out float32
    [ell, r, saved_t_stride(T)].  Returns (y_out or None, t_out)."""
    import torch

    lib = load_library()
    T, d_in = x.shape
    ell, r = s_rank.shape
    d_out = s_out.shape[1]
    if t_out is None:
        t_out = torch.empty((ell, r, saved_t_stride(T)), dtype=torch.float32, device=x.device)
    if y_base is not None and y_out is None:
        y_out = torch.empty_like(y_base)
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    ptr = lambda t_: None if t_ is None else t_.data_ptr()
    st = lib.lordba_forward_multi_save_t(x.data_ptr(), packedA.data_ptr(), packedB.data_ptr(), s_in.data_ptr(), s_rank.data_ptr(),
                                         s_out.data_ptr(), ptr(y_base), ptr(y_out), t_out.data_ptr(), t_out.shape[2], T, d_in, d_out, r,
                                         ell, ctypes.c_void_p(stream))
    if st != 0:
        raise LordbaError(st, "lordba_forward_multi_save_t")
    return y_out, t_out


def lordba_backward_multi(x, g, packedA, packedAt, packedBt, s_in, s_rank, s_out, latentA, latentB, kappa: float,
                          dx_base=None, dx=None, workspace=None, stream=None, t_saved=None) -> dict:
    """lordba_backward for ell envelopes: s_in [ell, d_in], s_rank [ell, r], s_out [ell, d_out] (float16 CUDA tensors); the
    scale gradients come back with the same leading envelope index."""
    import torch

    lib = load_library()
    T, d_in = x.shape
    d_out = g.shape[1]
    ell, r = s_rank.shape
    if tuple(s_in.shape) != (ell, d_in) or tuple(s_out.shape) != (ell, d_out):
        raise ValueError("scale arrays must be [ell, d_in], [ell, r], [ell, d_out]")
    need = lordba_backward_multi_workspace_bytes(T, d_in, d_out, r, ell)   # room for the one-pass form where it applies
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    if dx_base is not None and dx is None:
        dx = torch.empty_like(dx_base)
    f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device=x.device)
    out = {"dx": dx, "d_s_in": f32(ell, d_in), "d_s_rank": f32(ell, r), "d_s_out": f32(ell, d_out),
           "d_latentA": None if latentA is None else f32(r, d_in), "d_latentB": None if latentB is None else f32(d_out, r)}
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    ptr = lambda t_: None if t_ is None else t_.data_ptr()
    st = lib.lordba_backward_multi(x.data_ptr(), g.data_ptr(), packedA.data_ptr(), packedAt.data_ptr(), packedBt.data_ptr(),
                                   s_in.data_ptr(), s_rank.data_ptr(), s_out.data_ptr(), ptr(latentA), ptr(latentB), float(kappa),
                                   ptr(t_saved), 0 if t_saved is None else t_saved.shape[2],
                                   ptr(dx_base), ptr(dx), out["d_s_in"].data_ptr(), out["d_s_rank"].data_ptr(),
                                   out["d_s_out"].data_ptr(), ptr(out["d_latentA"]), ptr(out["d_latentB"]),
                                   workspace.data_ptr(), workspace.numel(), T, d_in, d_out, r, ell, ctypes.c_void_p(stream))
    if st != 0:
        raise LordbaError(st, "lordba_backward_multi")
    return out


def lordba_ptq_workspace_bytes(N: int, M: int, R: int, r0: int) -> int:
    return int(load_library().lordba_ptq_workspace_bytes(N, M, R, r0))


def lordba_ptq(A_star, B_star, R: int, K: int = 100, tau: float = 2.0, mu: float = 10.0, workspace=None, stream=None,
               sweeps=None, out=None):
    """Post-training quantisation of the update A_star B_star^T (torch CUDA float16 tensors [N, r0], [M, r0]) into a LoRDBA
    adapter of carrier rank R: lordba_ptq of the C interface.  Returns a dict of CUDA tensors: packedA, packedB (int32,
    the canonical format, as lordba_forward takes them), alpha [N], beta [R], gamma [M] (float64), s_in, s_rank, s_out
    (float16), info (float64 [8 + K], see include/lordba.h), and U1 [N, R], U2t [M, R] (float64 views into the workspace: the
    last continuous iterates).  sweeps = (t_begin, t_end) enqueues only that piece of the run (lordba_ptq_sweeps); a piece
    with t_begin > 0 continues the run of the dict `out` a previous piece returned (its tensors and workspace are reused)."""
    import torch

    lib = load_library()
    N, r0 = A_star.shape
    M = B_star.shape[0]
    if tuple(B_star.shape) != (M, r0) or A_star.dtype != torch.float16 or B_star.dtype != torch.float16:
        raise ValueError("need float16 A_star [N, r0] and B_star [M, r0]")
    dev = A_star.device
    need = lordba_ptq_workspace_bytes(N, M, R, r0)
    t_begin, t_end = (0, K) if sweeps is None else sweeps
    if out is not None:
        workspace = out["workspace"]
    elif t_begin != 0:
        raise ValueError("a piece that continues a run needs the dict the previous piece returned (out=...)")
    if workspace is None:
        workspace = torch.empty(max(need, 8) // 8, dtype=torch.float64, device=dev)
    out = out if out is not None else {
        "packedA": torch.empty(max((R * N + 31) // 32, 1), dtype=torch.int32, device=dev),
        "packedB": torch.empty(max((M * R + 31) // 32, 1), dtype=torch.int32, device=dev),
        "alpha": torch.empty(max(N, 1), dtype=torch.float64, device=dev),
        "beta": torch.empty(max(R, 1), dtype=torch.float64, device=dev),
        "gamma": torch.empty(max(M, 1), dtype=torch.float64, device=dev),
        "s_in": torch.empty(max(N, 1), dtype=torch.float16, device=dev),
        "s_rank": torch.empty(max(R, 1), dtype=torch.float16, device=dev),
        "s_out": torch.empty(max(M, 1), dtype=torch.float16, device=dev),
        "info": torch.empty(8 + max(K, 0), dtype=torch.float64, device=dev),
    }
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    st = lib.lordba_ptq_sweeps(A_star.contiguous().data_ptr(), B_star.contiguous().data_ptr(), out["packedA"].data_ptr(),
                               out["packedB"].data_ptr(), out["alpha"].data_ptr(), out["beta"].data_ptr(), out["gamma"].data_ptr(),
                               out["s_in"].data_ptr(), out["s_rank"].data_ptr(), out["s_out"].data_ptr(), out["info"].data_ptr(),
                               workspace.data_ptr(), workspace.numel() * workspace.element_size(), N, M, R, r0, K, t_begin, t_end,
                               tau, mu, ctypes.c_void_p(stream))
    if st != 0:
        raise LordbaError(st, "lordba_ptq_sweeps")
    off2 = (N * R + 31) // 32 * 32
    ws = workspace.view(torch.float64) if workspace.dtype != torch.float64 else workspace
    out["U1"] = ws[:N * R].view(N, R)
    out["U2t"] = ws[off2:off2 + M * R].view(M, R)
    out["workspace"] = workspace
    return out


def lordba_ptq_beta_solve(G, h, stream=None):
    """beta = pinv(G) h on the GPU (lordba_ptq_beta_solve of the C interface): G [R, R], h [R] float64 CUDA tensors."""
    import torch

    lib = load_library()
    R = h.numel()
    if tuple(G.shape) != (R, R) or G.dtype != torch.float64 or h.dtype != torch.float64 or not G.is_contiguous() or not h.is_contiguous():
        raise ValueError("need contiguous float64 G [R, R] and h [R]")
    beta = torch.empty(R, dtype=torch.float64, device=G.device)
    if stream is None:
        stream = torch.cuda.current_stream(G.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    st = lib.lordba_ptq_beta_solve(G.data_ptr(), h.data_ptr(), beta.data_ptr(), R, ctypes.c_void_p(stream))
    if st != 0:
        raise LordbaError(st, "lordba_ptq_beta_solve")
    return beta


def to_device(inputs: dict, device="cuda:0") -> dict:
    """Pack the carriers with the library and move one call's tensors to the GPU (plumbing for tests and bench)."""
    import torch

    pA, pB = lordba_pack_signs(inputs["signsA"], inputs["signsB"])
    dev = {k: torch.from_numpy(inputs[k]).to(device) for k in ("x", "y_base", "s_in", "s_rank", "s_out")}
    dev["packedA"] = torch.from_numpy(pA.view(np.int32)).to(device)
    dev["packedB"] = torch.from_numpy(pB.view(np.int32)).to(device)
    return dev
