"""Helpers of the GPU parity tests: run the HIP path through the C ABI and judge
it against the CPU oracle."""
import numpy as np
import torch

import oracle
from paper_2602_22732_amd import binding, synth

TOL_LOGPROB = {"f32": 1e-4, "bf16": 2e-2}
# Score gap above which SID indices must agree exactly.  fp32 path: 1e-3.  The bf16 path is
# allowed a log-probability error of 2e-2 per candidate, so two candidates closer than twice
# that can legitimately swap: its indices are held exact beyond 4e-2.  How often the 1e-3 rule
# also holds is reported by judge_decode ("strict_ok").
MARGIN = {"f32": 1e-3, "bf16": 4e-2}
STRICT_MARGIN = 1e-3
# Value step (all V_e log-probabilities of all b_T rows are output and judged): float32 at the stated 1e-4; bf16 runs pass a rounding
# model and take their bounds from it (judge_value); the figures below only apply to a bf16 call without one.
TOL_VALUE = {"f32": 1e-4, "bf16": 2e-2}
TOL_VALUE_TV = {"f32": 1e-4, "bf16": 1e-2}


def gpu_decode(w, W, X, lens, beam=None, trace=True, max_beam=None, value=False):
    """Decode on the GPU.  Returns sid, logprob (numpy) and the per-level trace; with value=True also, fourth, the
    value step's log-probabilities [B, b_T, V_e]."""
    beam = list(w.beam if beam is None else beam)
    dec = binding.decoder_for(w, W, max_beam=max_beam or beam)
    ctx = torch.from_numpy(X).to("cuda", dtype=binding.torch_dtype(w.dtype)).contiguous()
    cl = None if lens is None else torch.from_numpy(np.asarray(lens, np.int32)).cuda()
    tr = dec.enable_trace(ctx.shape[0], beam) if trace else None
    res = dec.decode_batch(ctx, cl, beam, value=value)
    torch.cuda.synchronize()
    out = [t.cpu().numpy() for t in res]
    trace_np = None if tr is None else {k: [t.cpu().numpy() for t in v] for k, v in tr.items()}
    dec.close()
    return (out[0], out[1], trace_np) + ((out[2],) if value else ())


def prefixes_from_trace(trace, r, T):
    """Token prefixes of the survivors of every level of request r: list of [b_t, t+1] arrays."""
    out, prev = [], np.zeros((1, 0), np.int32)
    for t in range(T):
        par, tok = trace["parent"][t][r], trace["tok"][t][r]
        cur = np.concatenate([prev[par], tok[:, None]], axis=1).astype(np.int32)
        out.append(cur)
        prev = cur
    return out


def strict_ok(all_scores, gpu_flat, k, margin=STRICT_MARGIN):
    """True if the survivor set also satisfies the rule at the strict margin."""
    s = np.asarray(all_scores, np.float64).ravel()
    order = np.argsort(-s, kind="stable")
    sig_k1 = s[order[k]] if k < len(s) else -np.inf
    must = set(np.nonzero(s > sig_k1 + margin)[0].tolist())
    return must <= set(gpu_flat.tolist()) and bool((s[gpu_flat] >= s[order[k - 1]] - margin).all())


def judge_selection(all_scores, gpu_flat, gpu_score, k, tol, margin, what=""):
    """all_scores: oracle scores of every candidate (flat).  gpu_flat: the GPU's k survivors in
    its order.  Survivor set and order must agree with the oracle wherever the oracle's gaps
    exceed `margin`; scores must agree within `tol`."""
    s = np.asarray(all_scores, np.float64).ravel()
    order = np.argsort(-s, kind="stable")
    assert len(set(gpu_flat.tolist())) == k, what + ": duplicate survivors"
    sig_k = s[order[k - 1]]
    sig_k1 = s[order[k]] if k < len(s) else -np.inf
    must = set(np.nonzero(s > sig_k1 + margin)[0].tolist())
    got = set(gpu_flat.tolist())
    assert must <= got, what + ": a candidate clearly inside the top-k is missing (%d missing)" % len(must - got)
    assert (s[gpu_flat] >= sig_k - margin).all(), what + ": a survivor lies clearly below the k-th score"
    so = s[gpu_flat]
    assert (so[:-1] >= so[1:] - margin).all(), what + ": survivors not in descending order"
    assert np.abs(so - gpu_score).max() <= tol, what + ": score error %.3g > %.3g" % (np.abs(so - gpu_score).max(), tol)
    exact = sig_k - sig_k1 > margin
    if exact:
        assert got == set(order[:k].tolist()), what + ": survivor set differs although the boundary gap exceeds the margin"
    return exact


# Storage-derived bounds (judge_decode(..., model=RoundedModel)).  The rounding model (tests/rounding_model.py) evaluates the
# same decoder in float64 but rounds wherever the library stores bfloat16 / E4M3, so its distance E from the oracle on a set of
# candidates is the error the storage types alone explain, for THIS model, request and level.  What remains between the GPU and
# the rounding model is float32 accumulation order (the matrix cores add the products of an instruction with limited alignment:
# about 1e-6 of the operand magnitudes for bf16, 7e-5 for FP8), the hardware's exp2/rcp approximations, and the values that, because
# of those, land on the neighbouring bfloat16 or E4M3 code.  Measured: most toy decodes agree with the model to 1e-6 on every
# survivor (no value anywhere on their paths rounded differently); where one did, the row it belongs to moves by up to the size
# of E itself, because a single high-leverage value (an FFN hidden unit, an attention output) one ulp off weighs as much as
# thousands of ordinary half-ulp errors.  So the GPU is another draw of the same rounding noise: it is held to the model within
# MODEL_TOL_ABS + MODEL_TOL_REL * E, hence to the oracle within (1 + MODEL_TOL_REL) * E + MODEL_TOL_ABS, and SID indices must be
# exact wherever the oracle's gaps exceed twice that.  A wrong operand, index or scale shows as an error of the size of the
# logits (several units), orders of magnitude beyond these bounds.
MODEL_TOL_ABS = 2e-3
MODEL_TOL_REL = 1.5


def judge_decode(w, W, X, lens, sid, lp, trace, requests, beam=None, tol=None, margin=None, model=None):
    """Teacher-forced acceptance of a GPU decode on the listed requests: at every level the
    oracle scores all candidates that follow the GPU's own surviving prefixes.
    model: a rounding_model.RoundedModel of the same workload; then the tolerance of every level is derived from it (see
    above) instead of taken from `tol`, and the GPU's scores are also held to the rounding model directly."""
    beam = list(w.beam if beam is None else beam)
    tol = TOL_LOGPROB[w.dtype] if tol is None else tol
    o = oracle.Oracle(weights=W, **w.model_kwargs())
    margin = MARGIN[w.dtype] if margin is None else margin
    stats = {"levels": 0, "exact_boundary": 0, "strict_ok": 0, "max_score_err": 0.0}
    if model is not None:
        stats.update(max_storage_err=0.0, max_gpu_vs_model=0.0, max_bound=0.0)
    for r in requests:
        rq = o.request(X[r], None if lens is None else int(lens[r]))
        rm = None if model is None else model.request(X[r], None if lens is None else int(lens[r]))
        pref = prefixes_from_trace(trace, r, w.T)
        prev = np.zeros((1, 0), np.int32)
        for t in range(w.T):
            cum, dist = rq.prefix_dists(t + 1, prev)
            scores = cum[:, None] + dist
            flat = trace["parent"][t][r].astype(np.int64) * w.V[t] + trace["tok"][t][r]
            if rm is not None:
                mc, md = rm.prefix_dists(t + 1, prev, beam_rows=[1] + beam[:t])
                ms = (mc[:, None] + md).ravel()
                storage = float(np.abs(ms[flat] - scores.ravel()[flat]).max())
                vs_model = float(np.abs(ms[flat] - trace["score"][t][r]).max())
                allowed = MODEL_TOL_ABS + MODEL_TOL_REL * storage
                stats["max_storage_err"] = max(stats["max_storage_err"], storage)
                stats["max_gpu_vs_model"] = max(stats["max_gpu_vs_model"], vs_model)
                assert vs_model <= allowed, "request %d level %d: GPU is %.3g from the rounding model, allowed %.3g (storage error %.3g)" % (
                    r, t + 1, vs_model, allowed, storage)
                tol = storage + allowed
                margin = 2 * tol
                stats["max_bound"] = max(stats["max_bound"], tol)
            ex = judge_selection(scores, flat, trace["score"][t][r], beam[t], tol, margin, what="request %d level %d" % (r, t + 1))
            stats["levels"] += 1
            stats["strict_ok"] += int(strict_ok(scores, flat, beam[t]))
            stats["exact_boundary"] += int(ex)
            stats["max_score_err"] = max(stats["max_score_err"], float(np.abs(scores.ravel()[flat] - trace["score"][t][r]).max()))
            prev = pref[t]
        assert np.array_equal(sid[r], pref[-1]), "returned SIDs differ from the traced paths"
        assert np.array_equal(lp[r], trace["score"][-1][r])
        assert (np.diff(lp[r]) <= 0).all()
    return stats


def judge_decode_rows(w, W, X, lens, sid, lp, trace, requests, rows_per_level=16, beam=None, tol=None, margin=None, seed=0):
    """Cheap form of judge_decode for many requests of a large configuration: per level the oracle scores the candidates of a
    seeded sample of the GPU's live beams only (the best beam always among them), teacher-forced.  Checked for those rows:
    the GPU's scores of the survivors that descend from them; that every one of their candidates the oracle puts clearly
    above the GPU's own k-th score survived; that none of their survivors lies clearly below it.  (Whether the k-th score
    itself is right needs all rows: that is judge_decode's part, on fewer requests.)"""
    beam = list(w.beam if beam is None else beam)
    tol = TOL_LOGPROB[w.dtype] if tol is None else tol
    margin = MARGIN[w.dtype] if margin is None else margin
    o = oracle.Oracle(weights=W, **w.model_kwargs())
    rng = np.random.default_rng(seed)
    stats = {"requests": 0, "rows": 0, "survivors_checked": 0, "max_score_err": 0.0}
    for r in requests:
        rq = o.request(X[r], None if lens is None else int(lens[r]))
        pref = prefixes_from_trace(trace, r, w.T)
        prev = np.zeros((1, 0), np.int32)
        for t in range(w.T):
            n = prev.shape[0]
            rows = np.arange(n) if n <= rows_per_level else np.unique(np.concatenate([[0], rng.choice(n, rows_per_level - 1, replace=False)]))
            cum, dist = rq.prefix_dists(t + 1, prev[rows])
            scores = cum[:, None] + dist                       # [sampled rows, V_t]
            par, tok, gs = trace["parent"][t][r], trace["tok"][t][r], trace["score"][t][r]
            kth = float(gs[-1])
            pos = {int(p): i for i, p in enumerate(rows)}
            kept = np.zeros(scores.shape, bool)
            for j in range(beam[t]):
                i = pos.get(int(par[j]))
                if i is None:
                    continue
                kept[i, tok[j]] = True
                err = abs(scores[i, tok[j]] - gs[j])
                stats["max_score_err"] = max(stats["max_score_err"], float(err))
                assert err <= tol, "request %d level %d: score error %.3g > %.3g" % (r, t + 1, err, tol)
                assert scores[i, tok[j]] >= kth - margin, "request %d level %d: a survivor lies clearly below the k-th score" % (r, t + 1)
                stats["survivors_checked"] += 1
            assert not (~kept & (scores > kth + margin)).any(), "request %d level %d: a candidate clearly above the k-th score is missing" % (r, t + 1)
            stats["rows"] += len(rows)
            prev = pref[t]
        assert np.array_equal(sid[r], pref[-1]) and np.array_equal(lp[r], trace["score"][-1][r])
        stats["requests"] += 1
    return stats


def value_rounding_model(w, W, batch=None):
    """Rounding model of a workload with an eCPM-token step: the same decoder seen as a model of T+1 levels (synth.value_model)."""
    import copy
    from rounding_model import RoundedModel
    kw, Wv = synth.value_model(w, W)
    w2 = copy.copy(w)
    w2.T, w2.V, w2.beam, w2.Ve = kw["T"], list(kw["V"]), list(w.beam) + [w.beam[-1]], 0
    model = RoundedModel(w2, Wv, batch=w.B if batch is None else batch)
    model.value_level = w.T
    return model


def judge_value(w, W, X, lens, sid, lp, val, requests, tol=None, model=None):
    """eCPM-token step: for the listed requests the oracle, teacher-forced on the SIDs the GPU returned, gives
    log p(v | y, X) of every returned SID (the decoder as a model of T+1 levels); the GPU's rows must agree within
    the log-probability tolerance, and so must the SID scores.  model (value_rounding_model): the bounds are derived
    from the rounding model as in judge_decode, and the GPU is held to it directly.  Returns the largest and the mean error seen."""
    tol_sid = TOL_LOGPROB[w.dtype] if tol is None else tol
    tol = TOL_VALUE[w.dtype] if tol is None else 2 * tol
    tol_tv = TOL_VALUE_TV[w.dtype] * (tol_sid / TOL_LOGPROB[w.dtype])
    kw, Wv = synth.value_model(w, W)
    o = oracle.Oracle(weights=Wv, **kw)
    worst, total, count = 0.0, 0.0, 0
    for r in requests:
        rq = o.request(X[r], None if lens is None else int(lens[r]))
        cum, dist = rq.prefix_dists(w.T + 1, sid[r])
        assert val[r].shape == dist.shape
        assert np.abs(np.exp(val[r].astype(np.float64)).sum(axis=1) - 1).max() < 1e-4, "value rows are not distributions"
        err = float(np.abs(val[r] - dist).max())
        if model is not None:
            mc, md = model.request(X[r], None if lens is None else int(lens[r])).prefix_dists(w.T + 1, sid[r], beam_rows=[1] + list(w.beam))
            storage, vs_model = float(np.abs(md - dist).max()), float(np.abs(md - val[r]).max())
            allowed = MODEL_TOL_ABS + MODEL_TOL_REL * storage
            assert vs_model <= allowed, "request %d: value step is %.3g from the rounding model, allowed %.3g (storage error %.3g)" % (
                r, vs_model, allowed, storage)
            tol = storage + allowed
            storage_sid = float(np.abs(mc - cum).max())
            tol_sid = storage_sid + MODEL_TOL_ABS + MODEL_TOL_REL * storage_sid
            tv_model = 0.5 * np.abs(np.exp(md) - np.exp(dist)).sum(axis=1).max()
            tol_tv = tv_model * (1 + MODEL_TOL_REL) + MODEL_TOL_ABS
        assert err <= tol, "request %d: value log-probability error %.3g > %.3g" % (r, err, tol)
        assert np.abs(cum - lp[r]).max() <= tol_sid
        tv = 0.5 * np.abs(np.exp(val[r].astype(np.float64)) - np.exp(dist)).sum(axis=1).max()
        assert tv <= tol_tv, "request %d: total variation %.3g > %.3g" % (r, tv, tol_tv)
        worst = max(worst, err)
        total += float(np.abs(val[r] - dist).sum())
        count += dist.size
    return worst, total / count
