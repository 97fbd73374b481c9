"""Pins of the oracle's FP8 mode (appendix A.2, low-precision inference): the E4M3 rounding against PyTorch's
float8_e4m3fn conversion and against the format's definition, the per-row and per-matrix scaling, and the
FP8 forward against a composition of library routines.  Nothing here touches the HIP path."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import MODE_CACHED, MODE_PLAIN
from helpers import tiny

RNG = np.random.default_rng(77)
F8 = torch.float8_e4m3fn


def torch_e4m3(x):
    return torch.tensor(np.asarray(x, np.float64)).to(torch.float32).to(F8).to(torch.float64).numpy()


def test_e4m3_rounding_matches_pytorch_conversion():
    x = np.concatenate([RNG.uniform(-448, 448, 50000), RNG.standard_normal(50000) * 0.02, RNG.standard_normal(20000) * 4,
                        np.ldexp(RNG.uniform(0.5, 1, 20000), RNG.integers(-12, 9, 20000))])
    x = x.astype(np.float32).astype(np.float64)  # float32 inputs: both sides round the same number
    np.testing.assert_array_equal(oracle.prim_e4m3(x), torch_e4m3(x))


def test_e4m3_grid_by_definition():
    # every value s * m * 2^(e-3): m in 8..15 for e in -6..8 (without 15 * 2^5 = 480, the NaN code), subnormals m in 1..7 at e = -6
    grid = sorted({m * 2.0 ** (e - 3) for e in range(-6, 9) for m in range(8, 16)} - {480.0} | {m * 2.0 ** -9 for m in range(1, 8)})
    assert len(grid) == 126 and grid[-1] == 448.0 and grid[0] == 2.0 ** -9
    g = np.array(grid)
    np.testing.assert_array_equal(oracle.prim_e4m3(g), g)            # grid points are fixed points
    np.testing.assert_array_equal(oracle.prim_e4m3(-g), -g)
    dense = np.concatenate([np.linspace(0, 1, 40001), np.linspace(1, 448, 200001)])
    got = oracle.prim_e4m3(dense)
    assert set(np.unique(got)) == set(grid) | {0.0}                   # nothing off the grid, nothing missing
    # nearest: no grid point is closer than the one chosen
    full = np.concatenate([[0.0], g])
    dist = np.abs(dense[:, None] - full[None, :]).min(axis=1)
    np.testing.assert_allclose(np.abs(got - dense), dist, atol=0, rtol=0)
    # ties go to the even mantissa: midway between 1.0 (m = 8) and 1.125 (m = 9) -> 1.0; between 1.125 and 1.25 (m = 10) -> 1.25
    np.testing.assert_array_equal(oracle.prim_e4m3([1.0625, 1.1875, -1.0625, 2.0 ** -10, 3 * 2.0 ** -10]), [1.0, 1.25, -1.0, 0.0, 2 * 2.0 ** -9])
    # saturation
    np.testing.assert_array_equal(oracle.prim_e4m3([448.0, 463.9, 464.0, 1e6, -1e30]), [448, 448, 448, 448, -448])


def test_row_quantisation_scale_error_bound_and_equivariance():
    x = RNG.standard_normal((7, 96)) * np.array([1e-3, 0.1, 1, 10, 300, 1e4, 1])[:, None]
    x[6] = 0.0
    q = oracle.prim_quant_rows(x)
    assert (q[6] == 0).all()
    for r in range(6):
        amax = np.abs(x[r]).max()
        i = np.abs(x[r]).argmax()
        assert abs(q[r, i] - x[r, i]) <= 1e-15 * amax                   # the largest element maps to 448: it survives (up to the scaling's own rounding)
        sc = amax / 448
        assert (np.abs(q[r] - x[r]) <= np.maximum(np.abs(x[r]) * 2.0 ** -4, sc * 2.0 ** -10) * (1 + 1e-12)).all()
        on_grid = q[r] / sc
        np.testing.assert_allclose(oracle.prim_e4m3(on_grid), on_grid, rtol=1e-12)
    np.testing.assert_array_equal(oracle.prim_quant_rows(x * 8.0), q * 8.0)   # powers of two commute with the rounding
    np.testing.assert_allclose(oracle.prim_quant_rows(q), q, rtol=1e-14)      # idempotent
    # rows do not see each other
    np.testing.assert_array_equal(oracle.prim_quant_rows(x[2:3]), q[2:3])


def _qrows(x):
    s = x.abs().amax(dim=1, keepdim=True) / 448
    s = torch.where(s == 0, torch.ones_like(s), s)
    return (x / s).to(torch.float32).to(F8).to(torch.float64) * s


def _qmat(*ws):
    s = max(float(np.abs(w).max()) for w in ws) / 448
    return [torch.tensor(np.asarray(w, np.float64) / s).to(torch.float32).to(F8).to(torch.float64) * s for w in ws]


def _torch_layer_fp8(lw, x, ctx, H, eps, d):
    """Autoregressive layer in FP8 mode from PyTorch routines: every per-row projection takes float8_e4m3fn operands
    (rows scaled per row, matrices per matrix, q/k/v of the self-attention as one matrix); the context keys and
    values keep full precision."""
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    eye = torch.eye(d, dtype=torch.float64)

    def attend(q_in, kv_in, wq, wk, wv, mask):
        out, _ = F.multi_head_attention_forward(
            q_in.unsqueeze(1), kv_in.unsqueeze(1), kv_in.unsqueeze(1), d, H,
            in_proj_weight=None, in_proj_bias=None, bias_k=None, bias_v=None, add_zero_attn=False, dropout_p=0.0,
            out_proj_weight=eye, out_proj_bias=None, training=False, need_weights=False, attn_mask=mask,
            use_separate_proj_weight=True, q_proj_weight=wq, k_proj_weight=wk, v_proj_weight=wv)
        return out.squeeze(1)

    x, ctx = t(x), t(ctx)
    n = x.shape[0]
    (wq_x,), (wo_x,), (wo_s,), (w1,), (w2,) = (_qmat(lw[k]) for k in ("wq_x", "wo_x", "wo_s", "w1", "w2"))
    wq_s, wk_s, wv_s = _qmat(lw["wq_s"], lw["wk_s"], lw["wv_s"])
    a = _qrows(F.rms_norm(x, (d,), t(lw["ln_x"]), eps=eps))
    x = x + F.linear(_qrows(attend(a, ctx, wq_x, t(lw["wk_x"]), t(lw["wv_x"]), None)), wo_x)
    a = _qrows(F.rms_norm(x, (d,), t(lw["ln_s"]), eps=eps))
    causal = torch.triu(torch.ones(n, n, dtype=torch.bool), diagonal=1)
    x = x + F.linear(_qrows(attend(a, a, wq_s, wk_s, wv_s, causal)), wo_s)
    a = _qrows(F.rms_norm(x, (d,), t(lw["ln_f"]), eps=eps))
    x = x + F.linear(_qrows(F.silu(F.linear(a, w1))), w2)
    return x.numpy()


def test_fp8_forward_matches_library_composition():
    from test_oracle_primitives import _torch_layer
    w, W, X = tiny(V=[5, 6, 4, 7], T=4, L=4, K=2, d=24, H=3, F=40, S=6, B=1)
    W["cls_bias"] = [None, np.linspace(-1, 1, 6).astype(np.float32), None, None]
    o = oracle.Oracle(weights=W, fp8=True, **w.model_kwargs())
    length, toks = 4, [3, 1, 2]
    ctx = X[0][:length]
    m = W["pos"].astype(np.float64).copy()
    for l in range(w.K):   # lazy layers: full precision
        m = _torch_layer(W["layers"][l], m, ctx, w.H, w.eps, w.d)
    s = torch.tensor(np.stack([W["bos"]] + [W["emb"][t][toks[t]] for t in range(3)]).astype(np.float64))
    wf = W["w_f"].astype(np.float64)
    (wf1,) = _qmat(wf[:, :w.d])
    gated = _qrows(torch.tensor(m) * (s @ torch.tensor(W["w_g"].T.astype(np.float64))))
    h = (F.linear(gated, wf1) + F.linear(s, torch.tensor(wf[:, w.d:]))).numpy()
    for l in range(w.K, w.L):
        h = _torch_layer_fp8(W["layers"][l], h, ctx, w.H, w.eps, w.d)
    got = o.request(X[0], length).forward_seq(toks)
    full = oracle.Oracle(weights=W, **w.model_kwargs()).request(X[0], length).forward_seq(toks)
    for t in range(w.T):
        (cls,) = _qmat(W["cls"][t])
        z = F.linear(_qrows(F.rms_norm(torch.tensor(h[t:t + 1]), (w.d,), torch.tensor(W["ln_out"].astype(np.float64)), eps=w.eps)), cls)[0]
        if W["cls_bias"][t] is not None:
            z = z + torch.tensor(W["cls_bias"][t].astype(np.float64))
        np.testing.assert_allclose(got[t], F.log_softmax(z, dim=0).numpy(), atol=1e-10)
        # and FP8 is a perturbation of the full-precision model, not something else
        assert 1e-6 < np.abs(got[t] - full[t]).max() < 0.5


@pytest.mark.parametrize("K", [0, 1, 2])
def test_fp8_cached_search_equals_search_by_definition(K):
    w, W, X = tiny(T=3, V=[5, 4, 6], L=3, K=K, S=6, B=2, beam=[3, 5, 4], len_min=2)
    o = oracle.Oracle(weights=W, fp8=True, **w.model_kwargs())
    lens = np.array([6, 3], np.int32)
    a = o.decode_batch(X, lens, w.beam, mode=MODE_CACHED)
    b = o.decode_batch(X, lens, w.beam, mode=MODE_PLAIN)
    assert np.array_equal(a[0], b[0])
    np.testing.assert_allclose(a[1], b[1], atol=1e-12)
    # the K = 0 model in FP8 mode is the plain autoregressive decoder in FP8 mode
    if K == 0:
        rq = o.request(X[0], 6)
        np.testing.assert_allclose(rq.forward_seq([1, 2])[-1], rq.plain_ar_seq([1, 2]), atol=1e-12)


def test_lazy_layers_and_context_projections_stay_full_precision():
    # a model whose only autoregressive layer is the last one: everything before the Fuse is the same numbers in both modes
    w, W, X = tiny(T=2, V=[4, 5], L=3, K=2, S=5, B=1)
    a = oracle.Oracle(weights=W, **w.model_kwargs()).request(X[0])
    b = oracle.Oracle(weights=W, fp8=True, **w.model_kwargs()).request(X[0])
    x = RNG.standard_normal((2, w.d))
    for l in range(w.K):
        np.testing.assert_array_equal(a.layer_seq(l, x), b.layer_seq(l, x))
    assert np.abs(a.layer_seq(2, x) - b.layer_seq(2, x)).max() > 1e-6
