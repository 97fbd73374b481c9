"""Small model factory for the CPU tests (tiny shapes, seeded)."""
import numpy as np

from paper_2602_22732_amd import synth


def tiny(T=3, V=6, d=16, H=2, F=32, L=3, K=1, S=5, B=2, beam=None, seed=1234, dtype="f32", len_min=None, gain_jitter=0.3, Ve=0, vanilla=False):
    V = [V] * T if isinstance(V, int) else list(V)
    beam = [2] * T if beam is None else list(beam)
    w = synth.Workload("tiny-test", dtype, B, S, d, L, K, H, F, T, V, beam, len_min=len_min)
    w.cfg_id = 0
    w.Ve = Ve
    w.vanilla = vanilla
    W = synth.make_weights(w, seed=seed, gain_jitter=gain_jitter)
    X = synth.make_context(w, seed=seed)
    return w, W, X


def all_paths(V):
    grids = np.meshgrid(*[np.arange(v) for v in V], indexing="ij")
    return np.stack([g.ravel() for g in grids], axis=1).astype(np.int32)
