"""A model of WHERE the HIP path rounds (test infrastructure; numpy, float64 arithmetic between the roundings).

The oracle computes the decoder exactly (double precision on bf16-representable inputs).  The HIP path computes the
same function but stores every matrix-product operand in bfloat16 (and, in FP8 mode, the per-beam-row operands in
E4M3).  This module evaluates the decoder of paper section 3.2 (eq. trunk, eq. fuse, eq. head, classifier softmax; or
the vanilla decoder's input s_{t-1} + p_t) teacher-forced on given prefixes, in float64, and applies a rounding
function at exactly the places where the library stores a narrower type:

    norm outputs, q, context keys/values, attention probabilities (matrix-core kernel: unnormalised, relative to a
    lazily refreshed maximum; absorbed form: normalised, or like the matrix-core kernel where one kernel forms it) and outputs, self-attention q/k/v and outputs, FFN hidden
    rows, the gated embedding of Fuse; float32 for the residual stream, the Fuse tables and the logits - except the
    logits of large levels, which the persistent GEMM hands to the selection in IEEE half precision.

It shares no code with the library or with the C oracle.  With every rounding switched off it IS the definition,
and is pinned to the C oracle in that mode (tests/test_rounding_model.py); with the roundings on, its distance from
the oracle is the error the storage types alone explain, which is what the GPU parity tests derive their bounds
from, and the GPU is compared with it directly.
"""
import numpy as np
import torch

from paper_2602_22732_amd import synth


def _f32(x):
    return np.asarray(x, np.float64).astype(np.float32).astype(np.float64)


def _bf16(x):
    return synth.round_bf16(np.asarray(x, np.float64).astype(np.float32)).astype(np.float64)


def _f16(x):
    return np.asarray(x, np.float64).astype(np.float32).astype(np.float16).astype(np.float64)


def _ident(x):
    return np.asarray(x, np.float64)


def e4m3(x):
    """Nearest OCP E4M3 value, by PyTorch's float8 type (inputs are scaled into [-448, 448] before)."""
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.float8_e4m3fn).to(torch.float64).numpy()


class RoundedModel:
    """w: synth.Workload (shapes, dtype, fp8, vanilla), W: its weights.
    act: "bf16" rounds where the library stores bfloat16, "none" nowhere.
    fp8: None = follow w.fp8; scale_arith "f32" mirrors the library's float32 scale arithmetic, "f64" the oracle's.
    batch: requests per decode call (decides, with the beam widths, which launches fold the RMSNorm into the
    projections around it: that moves one rounding)."""

    def __init__(self, w, W, act="bf16", fp8=None, scale_arith="f32", batch=None, lazy_form=None):
        self.w, self.W = w, W
        self.rnd = _bf16 if act == "bf16" else _ident
        self.f32 = _f32 if act == "bf16" else _ident
        self.fp8 = bool(w.fp8 if fp8 is None else fp8)
        self.scale_arith = scale_arith
        self.batch = w.B if batch is None else batch
        self.value_level = None  # 0-based level that is an eCPM-token step (its float32 distribution is the output: never half logits)
        d, H = w.d, w.H
        self.dh = d // H
        bf = act == "bf16" and w.dtype == "bf16"
        self.store_bf16 = bf
        # which cross-attention kernel the library runs (float32 storage: the plain kernel everywhere)
        self.flash = bf and self.dh in (32, 64) and d % 64 == 0
        self.absorbed = (w.K > 0 and w.dtype == "bf16" and self.dh % 64 == 0) if lazy_form is None else lazy_form == "absorbed"
        g = lambda a: np.asarray(a, np.float64)
        self.layers = [{k: g(v) for k, v in lw.items()} for lw in W["layers"]]
        self.pos, self.bos, self.ln_out = g(W["pos"]), g(W["bos"]), g(W["ln_out"])
        self.emb = [g(e) for e in W["emb"]]
        self.cls = [g(c) for c in W["cls"]]
        cb = W.get("cls_bias")
        self.bias = [None if cb is None or cb[t] is None else g(cb[t]) for t in range(w.T)]
        self.vanilla = bool(getattr(w, "vanilla", False))
        if not self.vanilla:
            wf = g(W["w_f"])
            self.wf1, wf2, wg = wf[:, :d], wf[:, d:], g(W["w_g"])
            prev = [self.bos[None, :]] + self.emb
            self.G = [self.f32(e @ wg.T) for e in prev[: w.T]]   # per-token tables, float32, built once
            self.P = [self.f32(e @ wf2.T) for e in prev[: w.T]]
        if self.fp8:  # weights of the per-beam-row products on the E4M3 grid, one scale per matrix
            for l in range(w.K, w.L):
                lw = self.layers[l]
                for k in ("wq_x", "wo_x", "wo_s", "w1", "w2"):
                    lw[k] = self.quant_matrix(lw[k])
                stacked = self.quant_matrix(np.concatenate([lw["wq_s"], lw["wk_s"], lw["wv_s"]], axis=0))
                lw["wq_s"], lw["wk_s"], lw["wv_s"] = stacked[:d], stacked[d:2 * d], stacked[2 * d:]
            self.cls = [self.quant_matrix(c) for c in self.cls]
            if not self.vanilla:
                self.wf1 = self.quant_matrix(self.wf1)

    # ---- FP8 operands ---------------------------------------------------------
    def _scale(self, amax):
        if self.scale_arith == "f32":
            amax = np.asarray(amax, np.float32)
            return np.where(amax > 0, amax / np.float32(448), np.float32(1)).astype(np.float64), \
                np.where(amax > 0, np.float32(448) / amax, np.float32(1)).astype(np.float64)
        amax = np.asarray(amax, np.float64)
        sc = np.where(amax > 0, amax / 448.0, 1.0)
        return sc, 1.0 / sc

    def quant_matrix(self, m):
        sc, inv = self._scale(np.abs(m).max())
        if self.scale_arith == "f32":
            return e4m3(m.astype(np.float32) * np.float32(inv)) * sc
        return e4m3(m / sc) * sc

    def quant_rows(self, x):
        sc, inv = self._scale(np.abs(x).max(axis=-1, keepdims=True))
        if self.scale_arith == "f32":
            return e4m3(x.astype(np.float32) * inv.astype(np.float32)) * sc
        return e4m3(x / sc) * sc

    # ---- pieces ---------------------------------------------------------------
    def folds(self, rows, n_cls):
        """True if the launches of a phase with this many rows fold the RMSNorm into the projections around it."""
        w = self.w
        return (self.store_bf16 and not self.fp8 and rows >= 8192 and w.d % 256 == 0 and w.F % 64 == 0 and w.F >= 256 and
                (n_cls == 0 or (n_cls >= 256 and n_cls % 4 == 0)))

    def logits_f16(self, rows, V):
        """True if the classifier of a level with this many rows leaves its logits in half precision (the persistent GEMM runs
        it and the wavefront selection kernel takes the codebook size)."""
        d = self.w.d
        if not self.store_bf16 or V % 8 or not 256 <= V <= 8192:
            return False
        if self.fp8:
            return rows >= 64 and d % 128 == 0 and d >= 384
        return rows >= 8192 and d % 64 == 0 and d >= 192

    def norm_operand(self, x, gain, fold, f8):
        """What the projection after RMSNorm(x) multiplies, and the row factor applied to its product afterwards."""
        inv = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + self.w.eps)
        if f8:
            return self.quant_rows(self.f32(gain * x * inv)), None
        if fold:
            return self.rnd(gain * x), self.f32(inv)
        return self.rnd(gain * x * inv), None

    @staticmethod
    def _proj(a, rowf, W):
        y = a @ W.T
        return y if rowf is None else y * rowf

    def attend_kv(self, q, Kc, Vc):
        """Beam-shared cross-attention of q [..., d] over the context keys/values [len, d]."""
        H, dh = self.w.H, self.dh
        lead = q.shape[:-1]
        qh = q.reshape(-1, H, dh)
        Kh, Vh = Kc.reshape(-1, H, dh), Vc.reshape(-1, H, dh)
        s = np.einsum("nhc,jhc->nhj", qh, Kh)  # raw scores
        if not self.flash:
            sc = s / np.sqrt(dh)
            p = np.exp(sc - sc.max(axis=-1, keepdims=True))
            o = np.einsum("nhj,jhc->nhc", p, Vh) / p.sum(axis=-1, keepdims=True)
            return self.rnd(o.reshape(lead + (H * dh,)))
        # matrix-core kernel: 64-key tiles; probabilities relative to a maximum that is refreshed only when a tile's
        # maximum outgrows it by more than 8 (in the exp2 domain); the probabilities that multiply V are rounded, the
        # normaliser sums the unrounded ones
        c = np.log2(np.e) / np.sqrt(dh)
        n_keys = s.shape[-1]
        m = np.full(s.shape[:2], -np.inf)
        l = np.zeros(s.shape[:2])
        O = np.zeros(s.shape[:2] + (dh,))
        for j0 in range(0, n_keys, 64):
            st = s[:, :, j0:j0 + 64]
            mx = st.max(axis=-1) * c
            upd = mx > m + 8.0
            mnew = np.where(upd, mx, m)
            alpha = np.where(upd, np.exp2(m - mnew), 1.0)
            m = mnew
            l, O = l * alpha, O * alpha[..., None]
            p = np.exp2(st * c - m[..., None])
            l = l + p.sum(axis=-1)
            O = O + np.einsum("nhj,jhc->nhc", self.rnd(p), Vh[j0:j0 + 64])
        return self.rnd((O / l[..., None]).reshape(lead + (H * dh,)))

    def attend_absorbed(self, q, lw, X):
        """Lazy layers (bf16, head width a multiple of 64): q_h . (W_k,h x_s) = (W_k,h^T q_h) . x_s and
        sum_s p_s W_v,h x_s = W_v,h sum_s p_s x_s on the raw context rows X [len, d]."""
        H, dh, d = self.w.H, self.dh, self.w.d
        qh = q.reshape(-1, H, dh)
        Wk, Wv = lw["wk_x"].reshape(H, dh, d), lw["wv_x"].reshape(H, dh, d)
        qp = self.rnd(np.einsum("nhc,hcj->nhj", qh, Wk))           # absorbed queries [n, H, d]
        if d in (512, 1024) and qh.shape[0] * H <= 128:
            # one kernel over 32-row tiles of the context (these widths, at most 128 queries per request): probabilities relative
            # to a maximum that is refreshed when outgrown by more than 8 (exp2 domain), rounded in the product, not in the sum
            s = self.f32(np.einsum("nhj,sj->nhs", qp, X))
            c = np.log2(np.e) / np.sqrt(dh)
            m = np.full(s.shape[:2], -np.inf)
            l = np.zeros(s.shape[:2])
            O = np.zeros(s.shape[:2] + (d,))
            for j0 in range(0, s.shape[-1], 32):
                st = s[:, :, j0:j0 + 32]
                mx = st.max(axis=-1) * c
                upd = mx > m + 8.0
                mnew = np.where(upd, mx, m)
                alpha = np.where(upd, np.exp2(m - mnew), 1.0)
                m = mnew
                l, O = l * alpha, O * alpha[..., None]
                p = np.exp2(st * c - m[..., None])
                l = l + p.sum(axis=-1)
                O = O + np.einsum("nhs,sj->nhj", self.rnd(p), X[j0:j0 + 32])
            z = self.rnd(O / l[..., None])
            o = self.rnd(np.einsum("nhj,hcj->nhc", z, Wv))
            return o.reshape(q.shape)
        s = self.f32(np.einsum("nhj,sj->nhs", qp, X)) / np.sqrt(dh)
        p = np.exp(s - s.max(axis=-1, keepdims=True))
        p = self.rnd(p / p.sum(axis=-1, keepdims=True))
        z = self.rnd(np.einsum("nhs,sj->nhj", p, X))               # weighted context sums [n, H, d]
        o = self.rnd(np.einsum("nhj,hcj->nhc", z, Wv))
        return o.reshape(q.shape)

    def self_attend(self, q, k, v):
        """Attention of q [n, d] (the newest position of each sequence) over k, v [n, u, d] (positions 0..u-1, the newest last)."""
        n, u, d = k.shape
        H, dh = self.w.H, self.dh
        qh, kh, vh = q.reshape(n, H, dh), k.reshape(n, u, H, dh), v.reshape(n, u, H, dh)
        s = np.einsum("nhc,nuhc->nhu", qh, kh) / np.sqrt(dh)
        p = np.exp(s - s.max(axis=-1, keepdims=True))
        p = p / p.sum(axis=-1, keepdims=True)
        return self.rnd(np.einsum("nhu,nuhc->nhc", p, vh).reshape(n, d))

    def layer(self, l, x, ctx, fold, f8, lazy, cache, first_norm_folded=True):
        """One decoder layer for ONE position of n sequences: x [n, d] (float32 residual stream).  cache: list of the (k, v)
        [n, d] pairs this layer produced at the earlier positions (each with the rounding placement of its own level); the
        new pair is appended."""
        lw, rnd, f32 = self.layers[l], self.rnd, self.f32
        q8 = (lambda a: self.quant_rows(a)) if f8 else (lambda a: a)
        a, rf = self.norm_operand(x, lw["ln_x"], fold and first_norm_folded, f8)
        q = rnd(self._proj(a, rf, lw["wq_x"]))
        if lazy and self.absorbed:
            o = self.attend_absorbed(q, lw, ctx["X"])
        else:
            o = self.attend_kv(q, ctx["K"][l], ctx["V"][l])
        x = f32(x + q8(o) @ lw["wo_x"].T)
        a, rf = self.norm_operand(x, lw["ln_s"], fold, f8)
        qs, ks, vs = (rnd(self._proj(a, rf, lw[k])) for k in ("wq_s", "wk_s", "wv_s"))
        cache.append((ks, vs))
        o = self.self_attend(qs, np.stack([c[0] for c in cache], axis=1), np.stack([c[1] for c in cache], axis=1))
        x = f32(x + q8(o) @ lw["wo_s"].T)
        a, rf = self.norm_operand(x, lw["ln_f"], fold, f8)
        hdn = self._proj(a, rf, lw["w1"])
        hdn = rnd(hdn / (1.0 + np.exp(-hdn)))
        return f32(x + q8(hdn) @ lw["w2"].T)

    def request(self, X, length=None):
        return _Request(self, np.asarray(X, np.float64)[: (X.shape[0] if length is None else int(length))])


class _Request:
    def __init__(self, model, X):
        self.m = m = model
        w = m.w
        # context keys/values, once per request; the lazy layers' too unless they run in absorbed form
        self.ctx = {"X": X, "K": {}, "V": {}}
        for l in range(w.L):
            if l >= w.K or not m.absorbed:
                self.ctx["K"][l] = m.rnd(X @ m.layers[l]["wk_x"].T)
                self.ctx["V"][l] = m.rnd(X @ m.layers[l]["wv_x"].T)
        self._trunk = None

    def trunk(self):
        """Lazy pass (eq. trunk): all positions in one set of launches, no beam dimension; [T, d]."""
        if self._trunk is None:
            m, w = self.m, self.m.w
            fold = m.folds(m.batch * w.T, 0)
            caches = [[] for _ in range(w.K)]
            rows = []
            for p in range(w.T):  # causal: position p sees the layer's keys/values of positions 0..p
                x = m.f32(m.pos[p][None, :])
                for l in range(w.K):
                    x = m.layer(l, x, self.ctx, fold, False, True, caches[l], first_norm_folded=l > 0)
                rows.append(x[0])
            self._trunk = np.stack(rows)
        return self._trunk

    def prefix_dists(self, t, prefixes, beam_rows=None):
        """Teacher-forced: for n prefixes of t-1 tokens (level t is 1-based) the cumulative log-probability of each
        prefix and the level-t log-probability distribution after it.  beam_rows[p]: rows per request of the launches that
        computed level p+1 on the GPU (decides whether their norms were folded); default: the workload's schedule."""
        m, w = self.m, self.m.w
        prefixes = np.asarray(prefixes, np.int64).reshape(-1, t - 1) if t > 1 else np.zeros((max(1, len(prefixes)), 0), np.int64)
        n = prefixes.shape[0]
        toks = np.concatenate([np.zeros((n, 1), np.int64), prefixes], axis=1)  # token before each position (column 0: BOS)
        rows = [1] + list(w.beam[: t - 1]) if beam_rows is None else list(beam_rows)
        caches = [[] for _ in range(w.L)]
        cum, lp = np.zeros(n), None
        for p in range(t):  # every position with the rounding placement of the level whose launches computed it
            fold = m.folds(m.batch * rows[p], w.V[p])
            if m.vanilla:
                x = m.f32((np.broadcast_to(m.bos, (n, w.d)) if p == 0 else m.emb[p - 1][toks[:, p]]) + m.pos[p][None, :])
            else:
                gated = m.rnd(self.trunk()[p][None, :] * m.G[p][toks[:, p]])
                if m.fp8:
                    gated = m.quant_rows(gated)
                x = m.f32(gated @ m.wf1.T + m.P[p][toks[:, p]])
            for l in range(w.K, w.L):
                # (the first norm of a level follows Fuse, which folds it; the vanilla input state is not written by a projection)
                x = m.layer(l, x, self.ctx, fold, m.fp8, False, caches[l], first_norm_folded=not (m.vanilla and l == w.K))
            a, rf = m.norm_operand(x, m.ln_out, fold, m.fp8)
            z = m._proj(a, rf, m.cls[p])
            if m.bias[p] is not None:
                z = z + m.bias[p]
            z = _f16(z) if p != m.value_level and m.logits_f16(m.batch * rows[p], w.V[p]) else m.f32(z)
            zmax = z.max(axis=-1, keepdims=True)
            lp = z - (zmax + np.log(np.exp(z - zmax).sum(axis=-1, keepdims=True)))
            if p < t - 1:
                cum += lp[np.arange(n), prefixes[:, p]]
        return cum, lp
