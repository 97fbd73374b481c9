"""GPU parity at the benchmark configurations (through the C ABI, launch configuration of
bench.py): full batch on the GPU, the oracle judges sampled requests teacher-forced."""
import numpy as np
import pytest

from gpu_common import gpu_decode, judge_decode
from paper_2602_22732_amd import synth

pytestmark = pytest.mark.gpu


def run_config(cfg, sample, batch=None, scale=1.0):
    w = synth.workload(cfg, scale=scale, batch=batch)
    W = synth.make_weights(w)
    lens = synth.make_lengths(w)
    X = synth.make_context(w, lens)
    sid, lp, tr = gpu_decode(w, W, X, lens)
    assert sid.shape == (w.B, w.beam[-1], w.T) and (np.diff(lp, axis=1) <= 0).all()
    for t in range(w.T):
        assert sid[..., t].min() >= 0 and sid[..., t].max() < w.V[t]
    stats = judge_decode(w, W, X, lens, sid, lp, tr, sample)
    print("config %d (%s): %s" % (cfg, w.name, stats))
    return stats


def test_config2_small_bf16_full_batch():
    run_config(2, sample=range(0, 64, 4))


def test_config3_medium_bf16_sampled_requests():
    run_config(3, sample=[0, 101, 255])
