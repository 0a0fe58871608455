"""Pins of the oracle's multi-adapter batch forward: every token row goes through the adapter its index names.

Expected values come from the one-adapter oracle function (pinned in test_oracle_pins.py) applied to each group of
rows on its own, and from properties of the row-wise definition; none comes from the function under test."""
import numpy as np
import pytest

import oracle
from paper_2605_24058_amd import inputs


def _pool_inputs(seed, T, d_in, d_out, r, n, pattern):
    d = inputs.make_adapter_pool(seed, d_in, d_out, r, n)
    d.update(inputs.make_activations(seed, T, d_in, d_out))
    d["ids"] = inputs.make_adapter_ids(seed, T, n, pattern)
    return d


def _run(d):
    return oracle.forward_batched(d["x"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["ids"], d["y_base"])


def _per_group(d):
    """The definition spelled out with the one-adapter function: gather the rows of each adapter, run them, scatter."""
    y = d["y_base"].astype(np.float64).copy()
    n = d["signsA"].shape[0]
    for a in range(n):
        rows = np.nonzero(d["ids"] == a)[0]
        if rows.size:
            y[rows] = oracle.forward(d["x"][rows], d["signsA"][a], d["signsB"][a], d["s_in"][a], d["s_rank"][a],
                                     d["s_out"][a], d["y_base"][rows])
    return y


@pytest.mark.parametrize("pattern", ["segments", "decode", "mixed"])
@pytest.mark.parametrize("T,d_in,d_out,r,n,seed", [(1, 8, 8, 2, 1, 0), (13, 40, 24, 3, 4, 1), (64, 96, 160, 8, 7, 2),
                                                   (37, 128, 64, 16, 37, 3)])
def test_batched_equals_one_adapter_function_per_group(pattern, T, d_in, d_out, r, n, seed):
    d = _pool_inputs(seed, T, d_in, d_out, r, n, pattern)
    assert np.array_equal(_run(d), _per_group(d))


def test_rows_without_adapter_pass_through():
    d = _pool_inputs(4, 20, 32, 48, 4, 3, "segments")
    d["ids"][[0, 5, 19]] = [-1, 3, 1000]                 # below, just above, far above the pool
    y = _run(d)
    yb = d["y_base"].astype(np.float64)
    assert np.array_equal(y[[0, 5, 19]], yb[[0, 5, 19]])
    assert not np.array_equal(y[1], yb[1])


def test_single_adapter_pool_is_the_plain_forward():
    d = _pool_inputs(5, 9, 64, 40, 5, 1, "segments")
    want = oracle.forward(d["x"], d["signsA"][0], d["signsB"][0], d["s_in"][0], d["s_rank"][0], d["s_out"][0], d["y_base"])
    assert np.array_equal(_run(d), want)


def test_row_permutation_commutes():
    d = _pool_inputs(6, 31, 48, 56, 6, 5, "decode")
    perm = np.random.default_rng(0).permutation(31)
    p = dict(d, x=d["x"][perm], y_base=d["y_base"][perm], ids=d["ids"][perm])
    assert np.array_equal(_run(p), _run(d)[perm])


def test_adapters_are_not_mixed_up():
    # A plausible mistake: index the scale pools with the row number or with a stale id.  Swapping two adapters' ids
    # must change exactly the rows that use them.
    d = _pool_inputs(7, 24, 64, 64, 8, 3, "segments")
    sw = d["ids"].copy()
    sw[d["ids"] == 0], sw[d["ids"] == 1] = 1, 0
    a, b = _run(d), _run(dict(d, ids=sw))
    touched = (d["ids"] == 0) | (d["ids"] == 1)
    assert np.array_equal(a[~touched], b[~touched])
    assert touched.any() and (np.abs(a[touched] - b[touched]).max(axis=1) > 0).all()


def test_id_recipes():
    seg = inputs.make_adapter_ids(1, 100, 6, "segments")
    assert seg.dtype == np.int32 and (np.diff(seg) >= 0).all() and seg.min() >= 0 and seg.max() <= 5
    dec = inputs.make_adapter_ids(1, 200, 6, "decode")
    assert (np.diff(dec) < 0).any() and set(dec) <= set(range(6))
    mix = inputs.make_adapter_ids(1, 400, 6, "mixed")
    assert (mix == -1).any() and (mix >= 0).any()
    pool = inputs.make_adapter_pool(2, 32, 48, 4, 3)
    assert pool["signsA"].shape == (3, 4, 32) and pool["s_out"].shape == (3, 48)
    assert not np.array_equal(pool["signsA"][0], pool["signsA"][1])


# ---- pools whose adapters have several scale envelopes (Def. 1 / Eq. (lordba) with l >= 2 per adapter) ----------------

def _pool_inputs_multi(seed, T, d_in, d_out, r, n, ell, pattern):
    d = inputs.make_adapter_pool_multi(seed, d_in, d_out, r, n, ell)
    d.update(inputs.make_activations(seed, T, d_in, d_out))
    d["ids"] = inputs.make_adapter_ids(seed, T, n, pattern)
    return d


def _run_multi(d):
    return oracle.forward_batched_multi(d["x"], d["signsA"], d["signsB"], d["s_in"], d["s_rank"], d["s_out"], d["ids"], d["y_base"])


def _dense_per_row(d):
    """Eq. (lordba) written out with numpy matrices: DeltaW_a = sum_e diag(alpha_e) S_A^T diag(beta_e) S_B^T diag(gamma_e) for
    every adapter a, then y[t] = y_base[t] + x[t] DeltaW_{id[t]}, in fp64 (no staging, no shared code with the oracle)."""
    n, ell = d["s_rank"].shape[:2]
    f = lambda a: a.astype(np.float64)
    dW = []
    for a in range(n):
        W = 0.0
        for e in range(ell):
            W = W + (f(d["s_in"][a, e])[:, None] * f(d["signsA"][a]).T * f(d["s_rank"][a, e])[None, :]) @ \
                (f(d["signsB"][a]).T * f(d["s_out"][a, e])[None, :])
        dW.append(W)
    y = f(d["y_base"]).copy()
    for t, a in enumerate(d["ids"]):
        if 0 <= a < n:
            y[t] += f(d["x"][t]) @ dW[a]
    return y


@pytest.mark.parametrize("pattern", ["segments", "decode", "mixed"])
@pytest.mark.parametrize("T,d_in,d_out,r,n,ell,seed", [(5, 8, 8, 2, 2, 2, 0), (13, 40, 24, 3, 4, 3, 1), (40, 96, 160, 8, 5, 4, 2),
                                                       (21, 64, 32, 16, 21, 2, 3)])
def test_batched_multi_equals_the_multi_envelope_function_per_group(pattern, T, d_in, d_out, r, n, ell, seed):
    """Per adapter, the rows that use it go through the pinned multi-envelope function: bit-identical."""
    d = _pool_inputs_multi(seed, T, d_in, d_out, r, n, ell, pattern)
    y = d["y_base"].astype(np.float64).copy()
    for a in range(n):
        rows = np.nonzero(d["ids"] == a)[0]
        if rows.size:
            y[rows] = oracle.forward_multi(d["x"][rows], d["signsA"][a], d["signsB"][a], d["s_in"][a], d["s_rank"][a],
                                           d["s_out"][a], d["y_base"][rows])
    assert np.array_equal(_run_multi(d), y)


@pytest.mark.parametrize("T,d_in,d_out,r,n,ell,seed", [(7, 12, 10, 3, 3, 2, 10), (9, 24, 16, 4, 4, 3, 11), (6, 16, 24, 2, 2, 4, 12)])
def test_batched_multi_against_dense_delta_w(T, d_in, d_out, r, n, ell, seed):
    d = _pool_inputs_multi(seed, T, d_in, d_out, r, n, ell, "decode")
    want = _dense_per_row(d)
    got = _run_multi(d)
    assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))


def test_batched_multi_with_one_envelope_is_the_batched_function():
    d = _pool_inputs_multi(13, 19, 48, 40, 5, 4, 1, "mixed")
    one = oracle.forward_batched(d["x"], d["signsA"], d["signsB"], d["s_in"][:, 0], d["s_rank"][:, 0], d["s_out"][:, 0], d["ids"],
                                 d["y_base"])
    assert np.array_equal(_run_multi(d), one)


def test_batched_multi_pass_through_and_permutation():
    d = _pool_inputs_multi(14, 23, 32, 48, 4, 3, 2, "segments")
    d["ids"][[0, 5, 22]] = [-1, 3, 1 << 20]
    y = _run_multi(d)
    yb = d["y_base"].astype(np.float64)
    assert np.array_equal(y[[0, 5, 22]], yb[[0, 5, 22]]) and not np.array_equal(y[1], yb[1])
    perm = np.random.default_rng(1).permutation(23)
    y2 = _run_multi(dict(d, x=d["x"][perm], y_base=d["y_base"][perm], ids=d["ids"][perm]))
    assert np.array_equal(y[perm], y2)


def test_batched_multi_planted_mistakes_are_caught():
    """Mistakes a batched multi-envelope routine can make in its pool indexing: the envelopes of adapter 0 for every row;
    the pool stride of a one-envelope pool (adapter a's scales read at a * d instead of a * ell * d); envelope 0 only."""
    d = _pool_inputs_multi(15, 16, 24, 20, 3, 3, 2, "decode")
    assert len(set(d["ids"].tolist())) >= 2 and (d["ids"] > 0).any()
    want = _dense_per_row(d)
    tol = 1e-9 * np.max(np.abs(want))
    assert np.max(np.abs(_run_multi(d) - want)) <= tol
    n, ell = d["s_rank"].shape[:2]
    shared = dict(d, **{k: np.repeat(d[k][:1], n, axis=0) for k in ("s_in", "s_rank", "s_out")})
    assert np.max(np.abs(_dense_per_row(shared) - want)) > 1e3 * tol
    flat = {k: d[k].reshape(n * ell, -1) for k in ("s_in", "s_rank", "s_out")}
    wrong_stride = dict(d, **{k: np.stack([flat[k][a:a + ell] for a in range(n)]) for k in flat})
    assert np.max(np.abs(_dense_per_row(wrong_stride) - want)) > 1e3 * tol
    first_only = dict(d, **{k: d[k][:, :1] for k in ("s_in", "s_rank", "s_out")})
    assert np.max(np.abs(_dense_per_row(first_only) - want)) > 1e3 * tol
