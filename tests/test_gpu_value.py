"""GPU parity of the eCPM-token step (section 3.3): after the SID levels one more prediction step scores the
value buckets of every returned SID; the oracle computes the same distributions teacher-forced on those SIDs."""
import numpy as np
import pytest
import torch

from gpu_common import gpu_decode, judge_decode, judge_value, value_rounding_model
from helpers import tiny
from paper_2602_22732_amd import binding, synth
from rounding_model import RoundedModel

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [
    dict(T=3, V=[40, 33, 50], Ve=21, d=64, H=2, F=96, L=3, K=1, S=37, B=5, beam=[7, 13, 9], len_min=5),       # ragged everywhere
    dict(T=2, V=[520, 130], Ve=300, d=256, H=2, F=64, L=2, K=0, S=9, B=2, beam=[300, 77]),                  # no lazy layer
    dict(T=1, V=[1000], Ve=8, d=64, H=1, F=64, L=2, K=1, S=3, B=4, beam=[10]),                              # one SID level
    dict(T=3, V=[40, 33, 50], Ve=64, d=128, H=2, F=96, L=3, K=2, S=37, B=5, beam=[7, 13, 9], len_min=1),      # absorbed lazy attention in bf16
    dict(T=7, V=[12] * 7, Ve=256, d=640, H=10, F=64, L=2, K=1, S=200, B=2, beam=[4, 6, 5, 6, 4, 6, 5], len_min=90),  # most levels the library takes
    dict(T=2, V=[512, 512], Ve=512, d=256, H=4, F=256, L=3, K=1, S=64, B=96, beam=[64, 96]),                # 9216 rows at the last level and the value step: the persistent GEMM
])
def test_value_step_matches_oracle(dtype, shape):
    w, W, X = tiny(dtype=dtype, gain_jitter=0.3 if dtype == "f32" else 0.1, **shape)
    if shape["Ve"] == 21:
        W["value_bias"] = np.linspace(-2.0, 1.0, 21).astype(np.float32)
    lens = synth.make_lengths(w, seed=11)
    sid, lp, tr, val = gpu_decode(w, W, X, lens, value=True)
    sample = range(w.B) if w.B <= 8 else [0, 17, w.B - 1]
    # float32: the stated 1e-4; bf16: bounds from the rounding model of this shape (gpu_common.judge_decode)
    bf = dtype == "bf16"
    judge_decode(w, W, X, lens, sid, lp, tr, sample, model=RoundedModel(w, W) if bf else None)
    print(dtype, shape["V"], shape["Ve"], "max, mean value error",
          judge_value(w, W, X, lens, sid, lp, val, sample, model=value_rounding_model(w, W) if bf else None))


def test_value_step_switches_on_and_off_per_call_and_leaves_the_sids_alone():
    w, W, X = tiny(T=3, V=[30, 20, 25], Ve=16, d=64, H=2, F=64, L=3, K=1, S=12, B=3, beam=[5, 8, 6])
    dec = binding.decoder_for(w, W)
    ctx = torch.from_numpy(X).cuda().contiguous()
    sid0, lp0 = dec.decode_batch(ctx, None, w.beam)
    sid0, lp0 = sid0.clone(), lp0.clone()
    sid1, lp1, val = dec.decode_batch(ctx, None, w.beam, value=True)
    sid1, lp1 = sid1.clone(), lp1.clone()
    sentinel = torch.full_like(val, 7.0)
    sid2, lp2 = dec.decode_batch(ctx, None, w.beam)  # off again: the old buffer must not be written
    val_copy = val.clone()
    val.copy_(sentinel)
    sid3, lp3 = dec.decode_batch(ctx, None, w.beam)
    torch.cuda.synchronize()
    assert torch.equal(val, sentinel)
    # fp32 model: the lazy pass is causal, so the SID levels are the same numbers with and without position T+1
    for s, l in ((sid1, lp1), (sid2, lp2), (sid3, lp3)):
        assert torch.equal(s, sid0) and torch.allclose(l, lp0, atol=1e-5)
    judge_value(w, W, X, None, sid1.cpu().numpy(), lp1.cpu().numpy(), val_copy.cpu().numpy(), range(w.B))
    dec.close()


def test_value_output_is_rejected_for_a_model_without_the_step():
    w, W, X = tiny(T=2, V=[8, 8], d=64, H=2, F=64, L=2, K=1, S=4, B=1, beam=[2, 2])
    dec = binding.decoder_for(w, W)
    buf = torch.zeros(4, device="cuda")
    assert dec.L_.gr4ad_decode_set_value_output(dec.handle, buf.data_ptr()) == -1
    assert "value step" in dec.L_.gr4ad_last_error(dec.handle).decode()
    dec.close()


def test_config3_with_value_step_sampled_requests():
    # the medium configuration with 256 value buckets; bench.py --value 256 times this step
    w = synth.workload(3, value=256)
    W = synth.make_weights(w)
    lens = synth.make_lengths(w)
    X = synth.make_context(w, lens)
    sid, lp, tr, val = gpu_decode(w, W, X, lens, value=True)
    sample = [0, 201]
    print("config 3 + value:", judge_decode(w, W, X, lens, sid, lp, tr, sample), "max, mean value error",
          judge_value(w, W, X, lens, sid, lp, val, sample, model=value_rounding_model(w, W)))
    assert np.isfinite(val).all() and (val <= 0).all()


def test_config4_with_value_step_full_batch_sampled_request():
    # the workload bench.py --config 4 --value 256 times: 1024 requests, 1024 returned SIDs each
    w = synth.workload(4, value=256)
    W = synth.make_weights(w)
    lens = synth.make_lengths(w)
    X = synth.make_context(w, lens)
    sid, lp, tr, val = gpu_decode(w, W, X, lens, value=True)
    assert val.shape == (w.B, w.beam[-1], 256) and np.isfinite(val).all() and (val <= 0).all()
    assert np.abs(np.exp(val[::97].astype(np.float64)).sum(axis=2) - 1).max() < 1e-4
    print("config 4 + value:", judge_decode(w, W, X, lens, sid, lp, tr, [511]), "max, mean value error", judge_value(w, W, X, lens, sid, lp, val, [511], model=value_rounding_model(w, W)))


@pytest.mark.parametrize("seed", range(6))
def test_value_step_random_shapes_fp32(seed):
    from test_gpu_decode import random_shape
    shape = random_shape(100 + seed)
    rng = np.random.default_rng(seed)
    shape["Ve"] = int(rng.integers(2, 300))
    w, W, X = tiny(dtype="f32", seed=77 + seed, **shape)
    if seed % 2:
        W["value_bias"] = rng.standard_normal(shape["Ve"]).astype(np.float32)
    lens = synth.make_lengths(w, seed=seed)
    sid, lp, tr, val = gpu_decode(w, W, X, lens, value=True)
    judge_decode(w, W, X, lens, sid, lp, tr, range(w.B))
    print(shape, "max, mean value error", judge_value(w, W, X, lens, sid, lp, val, range(w.B)))
