"""Pins of the rounding model (tests/rounding_model.py) to the C oracle: with every rounding switched off it is the
same function, in plain and in FP8 mode, for every kernel form it distinguishes.  Nothing here touches the HIP path."""
import numpy as np
import pytest

import oracle
from helpers import tiny
from paper_2602_22732_amd import synth
from rounding_model import RoundedModel

SHAPES = [
    dict(T=3, V=[40, 33, 50], d=64, H=2, F=96, L=3, K=1, S=37, B=3, beam=[7, 13, 9], len_min=5),      # dh 32: tiled kernel form
    dict(T=3, V=[17, 30, 9], d=128, H=8, F=64, L=4, K=2, S=70, B=2, beam=[5, 12, 7], len_min=1),      # dh 16: plain form
    dict(T=3, V=[40, 33, 50], d=128, H=2, F=96, L=3, K=2, S=150, B=2, beam=[7, 13, 9], len_min=70),   # dh 64: absorbed lazy layers, 3 key tiles
    dict(T=2, V=[52, 13], d=256, H=2, F=64, L=2, K=0, S=9, B=2, beam=[30, 7]),                        # no lazy layer
    dict(T=3, V=[24, 20, 30], d=512, H=8, F=64, L=2, K=1, S=75, B=2, beam=[5, 8, 6], len_min=1),       # dh 64, width 512: absorbed lazy layers in one pass (tiles of 32 rows)
]


def prefixes_for(w, t, n, seed):
    rng = np.random.default_rng(seed)
    return np.stack([rng.integers(0, w.V[p], n) for p in range(t - 1)], axis=1).astype(np.int32) if t > 1 else np.zeros((1, 0), np.int32)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_without_roundings_the_model_is_the_oracle(shape, fp8, dtype):
    if fp8 and dtype == "f32":
        pytest.skip("FP8 mode exists for bf16 storage only")
    w, W, X = tiny(dtype=dtype, gain_jitter=0.2, **shape)
    w.fp8 = fp8
    lens = synth.make_lengths(w, seed=3)
    o = oracle.Oracle(weights=W, **w.model_kwargs())
    mdl = RoundedModel(w, W, act="none", scale_arith="f64")
    for r in range(w.B):
        rq_o, rq_m = o.request(X[r], int(lens[r])), mdl.request(X[r], int(lens[r]))
        for t in range(1, w.T + 1):
            pre = prefixes_for(w, t, 4, 10 * r + t)
            c0, d0 = rq_o.prefix_dists(t, pre)
            c1, d1 = rq_m.prefix_dists(t, pre)
            np.testing.assert_allclose(c1, c0, atol=1e-9)
            np.testing.assert_allclose(d1, d0, atol=1e-9)


def test_both_lazy_forms_are_the_same_function_without_roundings():
    w, W, X = tiny(dtype="bf16", gain_jitter=0.2, **SHAPES[2])
    a = RoundedModel(w, W, act="none", lazy_form="absorbed").request(X[0], 100)
    b = RoundedModel(w, W, act="none", lazy_form="kv").request(X[0], 100)
    pre = prefixes_for(w, 3, 5, 1)
    np.testing.assert_allclose(a.prefix_dists(3, pre)[1], b.prefix_dists(3, pre)[1], atol=1e-10)


def test_vanilla_input_without_roundings_is_the_oracle():
    w, W, X = tiny(dtype="bf16", gain_jitter=0.2, vanilla=True, T=3, V=[40, 33, 50], d=64, H=2, F=96, L=3, K=0, S=20, B=2, beam=[7, 13, 9])
    o = oracle.Oracle(weights=W, **w.model_kwargs())
    mdl = RoundedModel(w, W, act="none")
    pre = prefixes_for(w, 3, 6, 2)
    c0, d0 = o.request(X[1]).prefix_dists(3, pre)
    c1, d1 = mdl.request(X[1]).prefix_dists(3, pre)
    np.testing.assert_allclose(c1, c0, atol=1e-9)
    np.testing.assert_allclose(d1, d0, atol=1e-9)


@pytest.mark.parametrize("shape", SHAPES[:3])
def test_bf16_storage_moves_log_probabilities_by_a_small_nonzero_amount(shape):
    w, W, X = tiny(dtype="bf16", gain_jitter=0.1, **shape)
    o = oracle.Oracle(weights=W, **w.model_kwargs())
    mdl = RoundedModel(w, W, act="bf16")
    pre = prefixes_for(w, w.T, 6, 5)
    _, d0 = o.request(X[0]).prefix_dists(w.T, pre)
    _, d1 = mdl.request(X[0]).prefix_dists(w.T, pre)
    err = np.abs(d1 - d0).max()
    assert 1e-5 < err < 0.2, err
