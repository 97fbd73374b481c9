"""GPU parity at the benchmark configurations (through the C ABI, launch configuration of
bench.py): full batch on the GPU, the oracle judges sampled requests teacher-forced."""
import numpy as np
import pytest

from gpu_common import gpu_decode, judge_decode, judge_decode_rows
from paper_2602_22732_amd import synth
from rounding_model import RoundedModel

pytestmark = pytest.mark.gpu

_weights = {}


def weights_of(w):
    """Weights depend on the configuration's seed and shapes only, not on batch or beam scale."""
    if w.cfg_id not in _weights:
        _weights.clear()  # one large model at a time in host memory
        _weights[w.cfg_id] = synth.make_weights(w)
    return _weights[w.cfg_id]


def run_config(cfg, sample, batch=None, scale=1.0, lazy=None, beam=None, vanilla=False, rows_sample=0, model_sample=()):
    w = synth.workload(cfg, scale=scale, batch=batch, lazy=lazy, vanilla=vanilla)
    if beam is not None:
        w.beam = list(beam)
    W = weights_of(w)
    lens = synth.make_lengths(w)
    X = synth.make_context(w, lens)
    sid, lp, tr = gpu_decode(w, W, X, lens)
    assert sid.shape == (w.B, w.beam[-1], w.T) and (np.diff(lp, axis=1) <= 0).all()
    for t in range(w.T):
        assert sid[..., t].min() >= 0 and sid[..., t].max() < w.V[t]
    # properties that hold for every request of the batch, whatever its size
    assert np.isfinite(lp).all() and (lp <= 0).all()
    for r in range(0, w.B, max(1, w.B // 64)):
        assert len({tuple(p) for p in sid[r]}) == w.beam[-1], "returned SIDs of request %d are not distinct" % r
    stats = judge_decode(w, W, X, lens, sid, lp, tr, sample)
    print("config %d (%s, K=%d): %s" % (cfg, w.name, w.K, stats))
    if model_sample:
        # beside the stated tolerance: the same decode against the rounding model of this configuration
        mstats = judge_decode(w, W, X, lens, sid, lp, tr, model_sample, model=RoundedModel(w, W))
        print("config %d (%s): against the rounding model, requests %s: %s" % (cfg, w.name, list(model_sample), mstats))
        stats["model"] = mstats
    if rows_sample:
        # more requests, judged on a sample of their beams per level: the shortest and the longest context and a seeded spread
        extra = sorted({int(np.argmin(lens)), int(np.argmax(lens))} | set(np.random.default_rng(cfg).choice(w.B, rows_sample, replace=False).tolist()))
        extra = [r for r in extra if r not in set(sample)]
        rstats = judge_decode_rows(w, W, X, lens, sid, lp, tr, extra, seed=cfg)
        print("config %d (%s): sampled beams of requests %s (context lengths %d..%d): %s" % (
            cfg, w.name, extra, min(lens[extra]), max(lens[extra]), rstats))
        stats["row_sampled"] = rstats
    return stats


def test_config2_small_bf16_full_batch():
    run_config(2, sample=range(0, 64, 4), model_sample=[1, 33])


def test_config3_medium_bf16_sampled_requests():
    run_config(3, sample=[0, 101, 255], rows_sample=12, model_sample=[101])


def test_config4_large_bf16_full_batch_sampled_requests():
    # B=1024, ragged context lengths, beams 256/512/512/1024 (bench.py --config 4): two requests judged on all their beams,
    # sixteen more (the shortest and the longest context among them) on a sample of their beams
    run_config(4, sample=[3, 1023], rows_sample=14)


@pytest.mark.parametrize("scale,batch,sample,rows_sample", [
    (0.25, 2048, [2047], 15),   # the full batch of 2048 at every schedule of the sweep
    (0.5, 2048, [5], 15),
    (1.0, 2048, [0, 1095, 1800, 2047], 12),    # the workload bench.py times by default
    (1.0, 96, [95], 0),        # and a slice of the batch: same model, same per-request work, another batch composition
])
def test_config5_load_adaptive_sweep_with_zipf_bias(scale, batch, sample, rows_sample):
    run_config(5, sample=sample, batch=batch, scale=scale, rows_sample=rows_sample)


def test_bf16_indices_are_exact_where_the_gaps_are_wide():
    # The benchmark configurations space their candidates far closer than the bf16 margin near rank b_t, so the rule "identical
    # survivor sets where the boundary gap exceeds the margin" never applies to them.  Here it must: configuration 2's model with a
    # steep popularity bias (-6 ln rank) and narrow beams puts gaps of 0.1 to 1 at every boundary (counted on the CPU: 18 of 18
    # levels of six requests), and judge_selection then demands the oracle's exact survivor set and order.
    w = synth.workload(2)
    w.beam = [16, 16, 16]
    W = dict(weights_of(w))
    W["cls_bias"] = [(-6.0 * np.log(np.random.default_rng(50 + t).permutation(w.V[t]) + 1.0)).astype(np.float32) for t in range(w.T)]
    lens = synth.make_lengths(w)
    X = synth.make_context(w, lens)
    sid, lp, tr = gpu_decode(w, W, X, lens)
    stats = judge_decode(w, W, X, lens, sid, lp, tr, range(0, 64, 8))
    print("config 2 with wide gaps:", stats)
    assert stats["exact_boundary"] >= 0.9 * stats["levels"], "the identical-set branch did not run"
    o_sid, o_lp, _ = __import__("oracle").Oracle(weights=W, **w.model_kwargs()).decode_batch(X[:8], lens[:8], w.beam)
    assert (sid[:8] == o_sid).all(axis=2).mean() > 0.9  # whole decodes agree beam for beam (a few late near-ties aside)


@pytest.mark.parametrize("lazy", [0, 5])
def test_config3_other_lazy_depths(lazy):
    # section 3.2: the same model decoded with no lazy layer (plain autoregressive decoding, every layer per beam and
    # level) and with all but one layer lazy; bench.py --lazy times these against the configuration's own depth
    run_config(3, sample=[7], lazy=lazy)


def test_config3_vanilla_autoregressive_decoder():
    # section 3.2, "Vanilla Autoregressive Decoding": the comparison decoder (s_{t-1} + p_t into L per-beam layers) on the
    # configuration's weights; bench.py --vanilla times it against LazyAR
    run_config(3, sample=[7], vanilla=True)


@pytest.mark.parametrize("beam", [[512, 512, 512], [512, 128, 512]])
def test_config3_other_beam_width_schedules(beam):
    # section 4.2.1 (Dynamic Beam Width): the fixed-width baseline and a schedule that narrows in the middle, which bench.py
    # --beam times against the configuration's own progressively increasing 128/256/512
    run_config(3, sample=[33], beam=beam)
