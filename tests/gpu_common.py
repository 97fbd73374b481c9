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
# Value step: all V_e log-probabilities of all b_T rows are output and judged, not only the k survivors of a level, so the
# largest error is taken over some hundred times more values of the same rounding noise (measured at configuration 3 with 256
# buckets: mean 4.5e-3, largest of 262144 values 2.9e-2, against 1.4e-2 for the largest of its 1792 survivor scores).  Every
# value must lie within twice the survivor tolerance, and each row's distribution within 1e-2 of the oracle's in total
# variation (what re-ranking by the predicted value sees).
TOL_VALUE = {"f32": 1e-4, "bf16": 4e-2}
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


def judge_decode(w, W, X, lens, sid, lp, trace, requests, beam=None, tol=None, margin=None):
    """Teacher-forced acceptance of a GPU decode on the listed requests: at every level the
    oracle scores all candidates that follow the GPU's own surviving prefixes."""
    beam = list(w.beam if beam is None else beam)
    tol = TOL_LOGPROB[w.dtype] if tol is None else tol
    o = oracle.Oracle(weights=W, **w.model_kwargs())
    margin = MARGIN[w.dtype] if margin is None else margin
    stats = {"levels": 0, "exact_boundary": 0, "strict_ok": 0, "max_score_err": 0.0}
    for r in requests:
        rq = o.request(X[r], None if lens is None else int(lens[r]))
        pref = prefixes_from_trace(trace, r, w.T)
        prev = np.zeros((1, 0), np.int32)
        for t in range(w.T):
            cum, dist = rq.prefix_dists(t + 1, prev)
            scores = cum[:, None] + dist
            flat = trace["parent"][t][r].astype(np.int64) * w.V[t] + trace["tok"][t][r]
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


def judge_value(w, W, X, lens, sid, lp, val, requests, tol=None):
    """eCPM-token step: for the listed requests the oracle, teacher-forced on the SIDs the GPU returned, gives
    log p(v | y, X) of every returned SID (the decoder as a model of T+1 levels); the GPU's rows must agree within
    the log-probability tolerance, and so must the SID scores.  Returns the largest and the mean error seen."""
    tol_sid = TOL_LOGPROB[w.dtype] if tol is None else tol
    tol = TOL_VALUE[w.dtype] if tol is None else 2 * tol
    kw, Wv = synth.value_model(w, W)
    o = oracle.Oracle(weights=Wv, **kw)
    worst, total, count = 0.0, 0.0, 0
    for r in requests:
        rq = o.request(X[r], None if lens is None else int(lens[r]))
        cum, dist = rq.prefix_dists(w.T + 1, sid[r])
        assert val[r].shape == dist.shape
        assert np.abs(np.exp(val[r].astype(np.float64)).sum(axis=1) - 1).max() < 1e-4, "value rows are not distributions"
        err = float(np.abs(val[r] - dist).max())
        assert err <= tol, "request %d: value log-probability error %.3g > %.3g" % (r, err, tol)
        assert np.abs(cum - lp[r]).max() <= tol_sid
        tv = 0.5 * np.abs(np.exp(val[r].astype(np.float64)) - np.exp(dist)).sum(axis=1).max()
        assert tv <= TOL_VALUE_TV[w.dtype] * (tol_sid / TOL_LOGPROB[w.dtype]), "request %d: total variation %.3g" % (r, tv)
        worst = max(worst, err)
        total += float(np.abs(val[r] - dist).sum())
        count += dist.size
    return worst, total / count
