"""Pins of the oracle's primitives against PyTorch CPU library routines and
closed forms.  Nothing here touches the HIP path."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from helpers import tiny

RNG = np.random.default_rng(7)


@pytest.fixture(autouse=True)
def _float64_default_in_this_module_only():
    # the library routines below are compared in double; the setting must not leak into other test modules (pytest imports
    # every module at collection, and a process-wide float64 default silently changes what torch.randn returns elsewhere)
    old = torch.get_default_dtype()
    torch.set_default_dtype(torch.float64)
    yield
    torch.set_default_dtype(old)


def test_linear_matches_library():
    x, W = RNG.standard_normal((5, 7)), RNG.standard_normal((3, 7))
    ref = F.linear(torch.tensor(x), torch.tensor(W)).numpy()
    np.testing.assert_allclose(oracle.prim_linear(x, W), ref, atol=1e-13)


def test_rmsnorm_matches_library():
    x, g = RNG.standard_normal((4, 9)), RNG.standard_normal(9)
    ref = F.rms_norm(torch.tensor(x), (9,), torch.tensor(g), eps=1e-3).numpy()
    np.testing.assert_allclose(oracle.prim_rmsnorm(x, g, 1e-3), ref, atol=1e-13)
    # closed form: a constant row c with unit gain normalises to sign(c) (eps -> 0)
    y = oracle.prim_rmsnorm(np.full((1, 8), -3.0), np.ones(8), 0.0)
    np.testing.assert_allclose(y, -np.ones((1, 8)), atol=1e-15)


def test_silu_matches_library():
    x = RNG.standard_normal(50) * 4
    np.testing.assert_allclose(oracle.prim_silu(x), F.silu(torch.tensor(x)).numpy(), atol=1e-14)
    assert oracle.prim_silu(np.zeros(1))[0] == 0.0


def test_log_softmax_matches_library():
    z = RNG.standard_normal(33) * 5
    np.testing.assert_allclose(oracle.prim_log_softmax(z), F.log_softmax(torch.tensor(z), dim=0).numpy(), atol=1e-13)
    # shift invariance and a huge offset (no overflow)
    np.testing.assert_allclose(oracle.prim_log_softmax(z + 1e4), oracle.prim_log_softmax(z), atol=1e-9)
    # uniform closed form
    np.testing.assert_allclose(oracle.prim_log_softmax(np.zeros(8)), np.full(8, -np.log(8)), atol=1e-15)


@pytest.mark.parametrize("causal", [False, True])
def test_mha_matches_sdpa(causal):
    H, dh, nq, nk = 3, 4, 5, 5 if causal else 7
    d = H * dh
    q, k, v = RNG.standard_normal((nq, d)), RNG.standard_normal((nk, d)), RNG.standard_normal((nk, d))

    def split(a):
        return torch.tensor(a).reshape(a.shape[0], H, dh).transpose(0, 1)

    ref = F.scaled_dot_product_attention(split(q), split(k), split(v), is_causal=causal)
    ref = ref.transpose(0, 1).reshape(nq, d).numpy()
    np.testing.assert_allclose(oracle.prim_mha(q, k, v, H, causal), ref, atol=1e-13)


def test_mha_causal_offset_is_suffix_alignment():
    # nq < nk with causal: query i sees keys 0..(nk-nq)+i (the new positions are the last ones)
    H, dh, nq, nk = 2, 4, 2, 5
    d = H * dh
    q, k, v = RNG.standard_normal((nq, d)), RNG.standard_normal((nk, d)), RNG.standard_normal((nk, d))
    mask = torch.tensor([[j <= (nk - nq) + i for j in range(nk)] for i in range(nq)])

    def split(a):
        return torch.tensor(a).reshape(a.shape[0], H, dh).transpose(0, 1)

    ref = F.scaled_dot_product_attention(split(q), split(k), split(v), attn_mask=mask).transpose(0, 1).reshape(nq, d).numpy()
    np.testing.assert_allclose(oracle.prim_mha(q, k, v, H, True), ref, atol=1e-13)


def test_fuse_closed_forms():
    d = 6
    m, s = RNG.standard_normal(d), RNG.standard_normal(d)
    Wg, Wf = RNG.standard_normal((d, d)), RNG.standard_normal((d, 2 * d))
    # library composition: W_f [ m * (W_g s) ; s ]
    ref = Wf @ np.concatenate([m * (Wg @ s), s])
    np.testing.assert_allclose(oracle.prim_fuse(m, s, Wg, Wf), ref, atol=1e-13)
    I, Z = np.eye(d), np.zeros((d, d))
    # W_f = [0 I] passes the token embedding through untouched
    np.testing.assert_allclose(oracle.prim_fuse(m, s, Wg, np.hstack([Z, I])), s, atol=1e-15)
    # W_f = [I 0] returns the gated trunk state m * (W_g s); with W_g = I that is m*s
    np.testing.assert_allclose(oracle.prim_fuse(m, s, I, np.hstack([I, Z])), m * s, atol=1e-15)
    # W_g = 0 and zero token half: nothing survives
    np.testing.assert_allclose(oracle.prim_fuse(m, s, Z, np.hstack([RNG.standard_normal((d, d)), Z])), 0, atol=1e-15)


@pytest.mark.parametrize("precut", [False, True])
def test_topk_matches_library_sort(precut):
    n, V, k = 5, 11, 9
    score = RNG.standard_normal((n, V))
    flat, ks = oracle.prim_topk(score, k, precut=precut)
    rv, ri = torch.topk(torch.tensor(score).flatten(), k)
    assert np.array_equal(flat, ri.numpy())
    np.testing.assert_array_equal(ks, rv.numpy())


@pytest.mark.parametrize("precut", [False, True])
def test_topk_ties_take_lowest_flat_index(precut):
    # heavy ties: values from a 3-letter alphabet; expected = stable sort of the negated scores
    n, V = 6, 8
    score = RNG.integers(0, 3, size=(n, V)).astype(np.float64)
    for k in (1, 5, 8, 17, n * V if not precut else 8):
        flat, ks = oracle.prim_topk(score, k, precut=precut)
        order = torch.sort(torch.tensor(-score.flatten()), stable=True).indices.numpy()[:k]
        assert np.array_equal(flat, order)
        np.testing.assert_array_equal(ks, score.flatten()[order])


def test_precut_equals_global_selection():
    # appendix A.2: the two-stage selection leaves the result unchanged
    for seed in range(5):
        r = np.random.default_rng(seed)
        n, V = int(r.integers(1, 9)), int(r.integers(2, 40))
        score = np.round(r.standard_normal((n, V)), 1)  # rounding makes ties common
        for k in (1, min(V, 3), V, min(n * V, V + 3)):
            f0, s0 = oracle.prim_topk(score, k, precut=False)
            f1, s1 = oracle.prim_topk(score, k, precut=True)
            assert np.array_equal(f0, f1) and np.array_equal(s0, s1)


def _torch_layer(lw, x, ctx, H, eps, d):
    """Decoder layer composed from PyTorch library routines (MHA is
    F.multi_head_attention_forward, norms F.rms_norm, FFN F.linear/F.silu)."""
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))

    def mha(q_in, kv_in, wq, wk, wv, wo, mask):
        out, _ = F.multi_head_attention_forward(
            q_in.unsqueeze(1), kv_in.unsqueeze(1), kv_in.unsqueeze(1), d, H,
            in_proj_weight=None, in_proj_bias=None, bias_k=None, bias_v=None, add_zero_attn=False, dropout_p=0.0,
            out_proj_weight=t(wo), out_proj_bias=None, training=False, need_weights=False, attn_mask=mask,
            use_separate_proj_weight=True, q_proj_weight=t(wq), k_proj_weight=t(wk), v_proj_weight=t(wv))
        return out.squeeze(1)

    x, ctx = t(x), t(ctx)
    n = x.shape[0]
    a = F.rms_norm(x, (d,), t(lw["ln_x"]), eps=eps)
    # cross-attention: queries from the normed state, keys/values from the RAW context
    q_side = mha(a, ctx, lw["wq_x"], lw["wk_x"], lw["wv_x"], lw["wo_x"], None)
    x = x + q_side
    a = F.rms_norm(x, (d,), t(lw["ln_s"]), eps=eps)
    causal = torch.triu(torch.ones(n, n, dtype=torch.bool), diagonal=1)
    x = x + mha(a, a, lw["wq_s"], lw["wk_s"], lw["wv_s"], lw["wo_s"], causal)
    a = F.rms_norm(x, (d,), t(lw["ln_f"]), eps=eps)
    x = x + F.linear(F.silu(F.linear(a, t(lw["w1"]))), t(lw["w2"]))
    return x.numpy()


def test_layer_matches_library_composition():
    w, W, X = tiny(d=24, H=3, F=40, L=3, K=1, S=7, T=4)
    o = oracle.Oracle(weights=W, **w.model_kwargs())
    for length in (7, 4):
        rq = o.request(X[0], length)
        x = RNG.standard_normal((4, w.d))
        for layer in range(w.L):
            ref = _torch_layer(W["layers"][layer], x, X[0][:length], w.H, w.eps, w.d)
            np.testing.assert_allclose(rq.layer_seq(layer, x), ref, atol=1e-12)


def test_single_context_token_makes_cross_attention_query_free():
    # S = 1: softmax over one key is 1, so the cross-attention output is Wo Wv x_1 whatever the query
    w, W, X = tiny(d=16, H=2, S=1)
    o = oracle.Oracle(weights=W, **w.model_kwargs())
    W2 = dict(W, layers=[dict(lw, wq_x=lw["wq_x"] * -3.0 + 1.0) for lw in W["layers"]])
    o2 = oracle.Oracle(weights=W2, **w.model_kwargs())
    x = RNG.standard_normal((3, w.d))
    np.testing.assert_allclose(o.request(X[0]).layer_seq(0, x), o2.request(X[0]).layer_seq(0, x), atol=1e-13)
