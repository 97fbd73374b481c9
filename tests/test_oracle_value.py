"""Pins of the eCPM-token step (section 3.3, value-aware supervised learning): the value token is one more
prediction step after the SID, i.e. level T+1 of the same decoder with the value vocabulary as its
codebook.  Nothing here touches the HIP path."""
import numpy as np

import oracle
from helpers import tiny
from paper_2602_22732_amd import synth


def models(**kw):
    w, W, X = tiny(**kw)
    kv, Wv = synth.value_model(w, W)
    return w, W, X, oracle.Oracle(weights=W, **w.model_kwargs()), oracle.Oracle(weights=Wv, **kv)


def test_appending_the_value_step_leaves_every_sid_level_unchanged():
    # causal lazy pass and causal head: nothing before position T+1 may depend on it
    w, W, X, base, ext = models(T=3, V=[5, 4, 6], Ve=7, L=3, K=2, S=6, B=2, len_min=2)
    toks = [4, 1, 5]
    for r in range(w.B):
        a = base.request(X[r], 4).forward_seq(toks[:2])
        b = ext.request(X[r], 4).forward_seq(toks)
        assert len(b) == 4 and b[3].shape == (7,)
        for t in range(3):
            np.testing.assert_allclose(a[t], b[t], atol=1e-13)


def test_value_distribution_is_a_distribution_and_all_routes_agree():
    w, W, X, base, ext = models(T=2, V=[4, 5], Ve=9, L=3, K=1, S=5, B=1)
    rq = ext.request(X[0])
    sids = np.array([[0, 0], [3, 4], [1, 2]], np.int32)
    cum, dist = rq.prefix_dists(3, sids)
    assert np.abs(np.exp(dist).sum(axis=1) - 1).max() < 1e-12
    for i, y in enumerate(sids):
        seq = rq.forward_seq(y)
        np.testing.assert_allclose(dist[i], seq[2], atol=1e-12)
        np.testing.assert_allclose(cum[i], seq[0][y[0]] + seq[1][y[1]], atol=1e-12)
    # summed over the value token the joint of (SID, value) gives back the SID probability
    joint = cum[:, None] + dist
    np.testing.assert_allclose(np.log(np.exp(joint).sum(axis=1)), cum, atol=1e-12)


def test_value_distribution_matches_library_composition():
    """Position T+1 with p_{T+1}, Fuse with the embedding of s_T, the autoregressive layers over the
    whole path, final norm and the value classifier (with its bias), wired from PyTorch routines."""
    import torch
    import torch.nn.functional as F
    from test_oracle_primitives import _torch_layer
    w, W, X = tiny(T=3, V=[5, 6, 4], Ve=11, L=4, K=2, d=24, H=3, F=40, S=6, B=1)
    W["value_bias"] = np.linspace(-1.0, 0.5, 11).astype(np.float32)
    kv, Wv = synth.value_model(w, W)
    o = oracle.Oracle(weights=Wv, **kv)
    length, y = 5, [3, 1, 2]
    ctx = X[0][:length]
    m = np.concatenate([W["pos"], W["value_pos"][None]], axis=0).astype(np.float64)
    for l in range(w.K):
        m = _torch_layer(W["layers"][l], m, ctx, w.H, w.eps, w.d)
    s = np.stack([W["bos"], W["emb"][0][y[0]], W["emb"][1][y[1]], W["value_emb"][y[2]]]).astype(np.float64)
    h = np.concatenate([m * (s @ W["w_g"].T.astype(np.float64)), s], axis=1) @ W["w_f"].T.astype(np.float64)
    for l in range(w.K, w.L):
        h = _torch_layer(W["layers"][l], h, ctx, w.H, w.eps, w.d)
    z = F.linear(F.rms_norm(torch.tensor(h[3]), (w.d,), torch.tensor(W["ln_out"].astype(np.float64)), eps=w.eps),
                 torch.tensor(W["value_cls"].astype(np.float64))) + torch.tensor(W["value_bias"].astype(np.float64))
    want = F.log_softmax(z, dim=0).numpy()
    _, dist = o.request(X[0], length).prefix_dists(4, np.array([y], np.int32))
    np.testing.assert_allclose(dist[0], want, atol=1e-12)


def test_dead_value_classifier_gives_equiprobable_buckets():
    # the buckets are built to be equiprobable: a classifier that has learnt nothing predicts exactly that
    w, W, X = tiny(T=2, V=[4, 5], Ve=8, L=2, K=1, S=4, B=1)
    W["value_cls"] = np.zeros_like(W["value_cls"])
    kv, Wv = synth.value_model(w, W)
    _, dist = oracle.Oracle(weights=Wv, **kv).request(X[0]).prefix_dists(3, np.array([[1, 2]], np.int32))
    np.testing.assert_allclose(dist, np.log(1.0 / 8), atol=1e-12)
