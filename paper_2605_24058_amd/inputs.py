"""Seeded synthetic inputs for the LoRDBA adapter forward branch.

This module holds no arithmetic of the method: it only draws the tensors that
both the GPU library and the CPU oracle are fed with.  The recipe follows the
benchmark configurations: activations x and y_base ~ N(0,1) rounded to fp16,
carrier signs i.i.d. +-1 with probability 1/2, and the three channel scale
vectors lognormal(mu=-3, sigma=0.5) rounded to fp16.  Everything is a pure
function of (seed, shape); nothing is read from disk.

The shapes stand in for LLaMA-2-7B / LLaMA-2-13B projection shapes; no model
weights, trained adapters or datasets are involved.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Iterator, List, Tuple

import numpy as np


@dataclass(frozen=True)
class Shape:
    name: str
    T: int
    d_in: int
    d_out: int
    r: int

    def activation_bytes(self) -> int:
        return 2 * self.T * (self.d_in + 2 * self.d_out)

    def adapter_bytes(self) -> int:
        bits = self.r * (self.d_in + self.d_out)
        return (bits + 7) // 8 + 2 * (self.d_in + self.r + self.d_out)

    def algorithmic_bytes(self) -> int:
        """x + y_base + y_out + packed carriers + three fp16 scale vectors."""
        return self.activation_bytes() + self.adapter_bytes()

    def adapter_bytes_multi(self, ell: int) -> int:
        """Packed carriers (shared by all envelopes) + ell triples of fp16 scale vectors."""
        bits = self.r * (self.d_in + self.d_out)
        return (bits + 7) // 8 + 2 * ell * (self.d_in + self.r + self.d_out)

    def algorithmic_bytes_multi(self, ell: int) -> int:
        return self.activation_bytes() + self.adapter_bytes_multi(ell)

    def sign_macs(self) -> int:
        return self.T * self.r * (self.d_in + self.d_out)


# The five benchmark configurations (index = position in the configuration list).
C1 = Shape("c1_512x512_r4_T64", 64, 512, 512, 4)
C2 = Shape("c2_llama7b_attn_4096x4096_r16_T2048", 2048, 4096, 4096, 16)
C3_UP = Shape("c3_llama7b_mlp_up_4096x11008_r16_T4096", 4096, 4096, 11008, 16)
C3_DOWN = Shape("c3_llama7b_mlp_down_11008x4096_r16_T4096", 4096, 11008, 4096, 16)
C4: List[Shape] = [Shape("c4_4096x4096_r%d_T%d" % (r, T), T, 4096, 4096, r)
                   for r in (8, 16, 32, 64) for T in (1, 8, 64)]
C5_Q = Shape("c5_llama13b_qkvo_5120x5120_r16_T8192", 8192, 5120, 5120, 16)
C5_UP = Shape("c5_llama13b_gateup_5120x13824_r16_T8192", 8192, 5120, 13824, 16)
C5_DOWN = Shape("c5_llama13b_down_13824x5120_r16_T8192", 8192, 13824, 5120, 16)
C5_LAYERS = 40
C5_PROJECTIONS: Tuple[Tuple[str, Shape], ...] = (
    ("q", C5_Q), ("k", C5_Q), ("v", C5_Q), ("o", C5_Q),
    ("gate", C5_UP), ("up", C5_UP), ("down", C5_DOWN))


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), *map(int, stream)])))


def make_adapter(seed: int, d_in: int, d_out: int, r: int) -> Dict[str, np.ndarray]:
    """Carrier signs (int8 +-1) and fp16 scales of one adapter."""
    g = _rng(seed, 1)
    signsA = (g.integers(0, 2, size=(r, d_in), dtype=np.int8) * 2 - 1).astype(np.int8)
    signsB = (g.integers(0, 2, size=(d_out, r), dtype=np.int8) * 2 - 1).astype(np.int8)

    def lognormal(n):
        return np.exp(-3.0 + 0.5 * g.standard_normal(n)).astype(np.float16)

    return {"signsA": signsA, "signsB": signsB,
            "s_in": lognormal(d_in), "s_rank": lognormal(r), "s_out": lognormal(d_out)}


def make_envelopes(seed: int, d_in: int, d_out: int, r: int, ell: int) -> Dict[str, np.ndarray]:
    """Scale vectors of ell envelopes over the carriers of make_adapter(seed, ...): s_in [ell, d_in], s_rank [ell, r],
    s_out [ell, d_out].  Envelope 0 is the adapter's own triple; each further envelope draws the same lognormal
    magnitudes from its own stream and gives every rank-scale entry a random sign (envelopes are real-valued and
    may cancel one another)."""
    base = make_adapter(seed, d_in, d_out, r)
    s_in, s_rank, s_out = [base["s_in"]], [base["s_rank"]], [base["s_out"]]
    for e in range(1, ell):
        g = _rng(seed, 3, e)
        ln = lambda n: np.exp(-3.0 + 0.5 * g.standard_normal(n))
        flip = g.integers(0, 2, size=r) * 2 - 1
        s_in.append(ln(d_in).astype(np.float16))
        s_rank.append((ln(r) * flip).astype(np.float16))
        s_out.append(ln(d_out).astype(np.float16))
    return {"s_in": np.stack(s_in), "s_rank": np.stack(s_rank), "s_out": np.stack(s_out)}


def make_inputs_multi(seed: int, T: int, d_in: int, d_out: int, r: int, ell: int) -> Dict[str, np.ndarray]:
    """All tensors of one multi-envelope call: carriers and activations as make_inputs, scales as make_envelopes."""
    out = make_inputs(seed, T, d_in, d_out, r)
    out.update(make_envelopes(seed, d_in, d_out, r, ell))
    return out


def make_adapter_pool(seed: int, d_in: int, d_out: int, r: int, n: int) -> Dict[str, np.ndarray]:
    """n independent adapters of one shape, stacked over a leading adapter index (adapter a = make_adapter(seed', ...)
    with a seed derived from (seed, a))."""
    ads = [make_adapter(int(np.random.SeedSequence([int(seed), 4, a]).generate_state(1)[0]), d_in, d_out, r) for a in range(n)]
    return {k: np.stack([ad[k] for ad in ads]) for k in ("signsA", "signsB", "s_in", "s_rank", "s_out")}


def make_adapter_pool_multi(seed: int, d_in: int, d_out: int, r: int, n: int, ell: int) -> Dict[str, np.ndarray]:
    """The pool of make_adapter_pool when every adapter has ell scale envelopes over its carriers (make_envelopes with the
    adapter's derived seed): signsA [n, r, d_in], signsB [n, d_out, r], s_in [n, ell, d_in], s_rank [n, ell, r],
    s_out [n, ell, d_out].  With ell = 1 the scales are those of make_adapter_pool with a unit envelope axis."""
    seeds = [int(np.random.SeedSequence([int(seed), 4, a]).generate_state(1)[0]) for a in range(n)]
    ads = [make_adapter(sd, d_in, d_out, r) for sd in seeds]
    env = [make_envelopes(sd, d_in, d_out, r, ell) for sd in seeds]
    out = {k: np.stack([ad[k] for ad in ads]) for k in ("signsA", "signsB")}
    out.update({k: np.stack([e[k] for e in env]) for k in ("s_in", "s_rank", "s_out")})
    return out


def make_adapter_ids(seed: int, T: int, n: int, pattern: str) -> np.ndarray:
    """int32[T] adapter index per token row.
    "segments": rows sorted by adapter, n contiguous segments of random lengths (prefill of n requests);
    "decode":   every row draws its adapter independently (one token per request, unsorted);
    "mixed":    as "segments", with about one row in eight marked -1 (a request without an adapter)."""
    g = _rng(seed, 5)
    if pattern == "decode":
        return g.integers(0, n, size=T, dtype=np.int64).astype(np.int32)
    cuts = np.sort(g.integers(0, T + 1, size=max(n - 1, 0)))
    bounds = np.concatenate([[0], cuts, [T]]).astype(np.int64)
    ids = np.empty(T, dtype=np.int32)
    for a in range(n):
        ids[bounds[a]:bounds[a + 1]] = a
    if pattern == "mixed":
        ids[g.random(T) < 0.125] = -1
    elif pattern != "segments":
        raise ValueError(pattern)
    return ids


def make_activations(seed: int, T: int, d_in: int, d_out: int) -> Dict[str, np.ndarray]:
    g = _rng(seed, 2)
    x = g.standard_normal((T, d_in), dtype=np.float32).astype(np.float16)
    y_base = g.standard_normal((T, d_out), dtype=np.float32).astype(np.float16)
    return {"x": x, "y_base": y_base}


def make_inputs(seed: int, T: int, d_in: int, d_out: int, r: int) -> Dict[str, np.ndarray]:
    """All tensors of one lordba_forward call, from one seed."""
    out = make_adapter(seed, d_in, d_out, r)
    out.update(make_activations(seed, T, d_in, d_out))
    return out


def make_backward_inputs(seed: int, T: int, d_in: int, d_out: int, r: int, g_scale: float = 1.0) -> Dict[str, np.ndarray]:
    """All tensors of one backward call of the branch in training: the forward tensors of make_inputs, the upstream
    gradient g ~ g_scale * N(0,1) [T, d_out] and the base path's input gradient dx_base ~ g_scale * N(0,1) [T, d_in]
    (fp16), and real-valued latent carriers in the carriers' layouts (float32): each latent entry is the carrier's
    sign times a magnitude |N(0, 1/d)| with d the long side of its matrix, the size of the entries of the orthonormal
    factors of a thin singular value decomposition from which training starts (magnitudes near 1/sqrt(d))."""
    out = make_inputs(seed, T, d_in, d_out, r)
    g = _rng(seed, 6)
    out["g"] = (g_scale * g.standard_normal((T, d_out), dtype=np.float32)).astype(np.float16)
    out["dx_base"] = (g_scale * g.standard_normal((T, d_in), dtype=np.float32)).astype(np.float16)
    magA = np.abs(g.standard_normal((r, d_in), dtype=np.float32)) / np.float32(np.sqrt(d_in))
    magB = np.abs(g.standard_normal((d_out, r), dtype=np.float32)) / np.float32(np.sqrt(d_out))
    out["latA"] = (out["signsA"].astype(np.float32) * magA).astype(np.float32)
    out["latB"] = (out["signsB"].astype(np.float32) * magB).astype(np.float32)
    return out


def make_ptq_inputs(seed: int, N: int, M: int, r0: int, decay: float = 0.85) -> Dict[str, np.ndarray]:
    """The fp16 LoRA factors that post-training quantisation starts from: A_star [N, r0] and B_star [M, r0] with
    Delta W* = A_star B_star^T.  Entries are N(0, 0.05^2); column k of A_star is damped by decay^k, so that the update
    has the decaying singular spectrum of a trained adapter and distinct singular values."""
    g = _rng(seed, 7)
    damp = (np.float32(decay) ** np.arange(r0, dtype=np.float32)).astype(np.float32)
    a = (np.float32(0.05) * g.standard_normal((N, r0), dtype=np.float32) * damp[None, :]).astype(np.float16)
    b = (np.float32(0.05) * g.standard_normal((M, r0), dtype=np.float32)).astype(np.float16)
    return {"A_star": a, "B_star": b}


def make_inputs_for(shape: Shape, seed: int) -> Dict[str, np.ndarray]:
    return make_inputs(seed, shape.T, shape.d_in, shape.d_out, shape.r)


def c5_adapter_seeds(seed: int) -> Iterator[Tuple[int, str, Shape, int]]:
    """(layer, projection name, shape, derived seed) for the 40 x 7 adapter set."""
    for layer in range(C5_LAYERS):
        for p, (name, shape) in enumerate(C5_PROJECTIONS):
            yield layer, name, shape, int(np.random.SeedSequence([int(seed), layer, p]).generate_state(1)[0])
