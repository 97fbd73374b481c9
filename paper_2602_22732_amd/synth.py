"""Seeded synthetic workloads (shared by the oracle-side tests and the GPU path).

This module holds none of the method's arithmetic: it only draws random model
weights and context memories with numpy and rounds them to the storage type.
It stands in for the paper's private production traffic; shapes follow the
structure the paper reports (3-4 SID levels, codebooks of 1k-16k entries, beam
widths of 128-1024 that grow with the level, about two thirds of the layers
lazy).
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

BASE_SEED = 260222732
LAYER_FIELDS = ["ln_x", "wq_x", "wk_x", "wv_x", "wo_x", "ln_s", "wq_s", "wk_s", "wv_s", "wo_s", "ln_f", "w1", "w2"]


@dataclass
class Workload:
    name: str
    dtype: str  # "f32" | "bf16"
    B: int
    S: int
    d: int
    L: int
    K: int
    H: int
    F: int
    T: int
    V: List[int]
    beam: List[int]
    len_min: Optional[int] = None  # None: every context has S tokens
    zipf_bias: bool = False
    eps: float = 1e-6
    cfg_id: int = 0
    fp8: bool = False  # low-precision inference (appendix A.2): FP8 operands for the per-beam-row products
    Ve: int = 0  # eCPM-token step (section 3.3): number of value buckets, 0 = the model has no such step
    vanilla: bool = False  # vanilla autoregressive decoder (section 3.2): input s_{t-1} + p_t, no Fuse, K = 0
    extra: dict = field(default_factory=dict)

    @property
    def A(self):
        return self.L - self.K

    @property
    def rows(self):  # live beams entering each level
        return [1] + list(self.beam[:-1])

    def model_kwargs(self):
        kw = dict(d=self.d, H=self.H, F=self.F, L=self.L, K=self.K, T=self.T, V=list(self.V), eps=self.eps)
        if self.fp8:
            kw["fp8"] = True
        if self.vanilla:
            kw["vanilla"] = True
        return kw


def scale_beams(beam, factor):
    """Load-adaptive beam scale: every width times `factor`, rounded, at least 1."""
    return [max(1, int(round(b * factor))) for b in beam]


def workload(cfg, scale=1.0, batch=None, lazy=None, value=None, fp8=False, vanilla=False):
    """The five benchmark configurations (1-based).  lazy: another number of lazy layers K for the same
    model (0 = every layer autoregressive, section 3.2's comparison of LazyAR with plain decoding).
    value: number of eCPM buckets of a value step appended to the model (section 3.3); None or 0 = none.
    vanilla: the vanilla autoregressive decoder of section 3.2 on the same weights (input s_{t-1} + p_t instead of Fuse,
    every layer autoregressive: implies lazy = 0)."""
    if cfg == 1:
        w = Workload("tiny-f32", "f32", 4, 64, 128, 2, 1, 4, 512, 3, [256] * 3, [16] * 3)
    elif cfg == 2:
        w = Workload("small-bf16", "bf16", 64, 256, 256, 4, 2, 8, 1024, 3, [1024] * 3, [64] * 3)
    elif cfg == 3:
        w = Workload("medium-bf16", "bf16", 256, 512, 512, 6, 4, 8, 2048, 3, [4096] * 3, [128, 256, 512])
    elif cfg == 4:
        w = Workload("large-bf16", "bf16", 1024, 1024, 1024, 8, 6, 16, 4096, 4, [8192] * 4, [256, 512, 512, 1024], len_min=256)
    elif cfg == 5:
        w = Workload("sweep-bf16", "bf16", 2048, 1024, 1024, 8, 6, 16, 4096, 4, [8192] * 4,
                     scale_beams([256, 512, 512, 1024], scale), len_min=256, zipf_bias=True)
        w.name += "-x%g" % scale
    else:
        raise ValueError("config must be 1..5")
    w.cfg_id = cfg
    if batch is not None:
        w.B = batch
    if vanilla:
        if lazy not in (None, 0):
            raise ValueError("the vanilla decoder has no lazy layer")
        lazy = 0
        w.vanilla = True
        w.name += "-vanilla"
    if lazy is not None:
        if not 0 <= lazy < w.L:
            raise ValueError("lazy must be in [0, L)")
        w.K = lazy
        w.name += "-K%d" % lazy
    if fp8:
        if w.dtype != "bf16":
            raise ValueError("the FP8 mode needs a bf16 configuration")
        w.fp8 = True
        w.name += "-fp8"
    if value:
        w.Ve = int(value)
        w.name += "-value%d" % w.Ve
    return w


def round_bf16(a):
    """float32 -> nearest bfloat16-representable float32 (ties to even)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(np.shape(a))


def to_bf16_bits(a):
    """float32 (already bf16-representable or not) -> uint16 bfloat16 bit patterns."""
    return (round_bf16(a).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _store(a, dtype):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_bf16(a) if dtype == "bf16" else a


def _xavier(rng, out_f, in_f):
    lim = np.sqrt(6.0 / (in_f + out_f))
    return rng.uniform(-lim, lim, size=(out_f, in_f)).astype(np.float32)


def make_weights(w: Workload, seed=None, gain_jitter=0.1):
    """Random-init weights: Xavier-uniform matrices, N(0,1) embeddings/positions,
    norm gains 1 + gain_jitter*N(0,1).  Values are rounded to the workload's
    storage type, so oracle and GPU start from identical numbers."""
    seed = BASE_SEED + 1000 * w.cfg_id if seed is None else seed
    k = [0]

    def rng():
        k[0] += 1
        return np.random.default_rng(seed + k[0])

    d, F, T = w.d, w.F, w.T

    def gain():
        return (1.0 + gain_jitter * rng().standard_normal(d)).astype(np.float32)

    out = {
        "pos": rng().standard_normal((T, d)).astype(np.float32),
        "bos": rng().standard_normal(d).astype(np.float32),
        "emb": [rng().standard_normal((w.V[t], d)).astype(np.float32) for t in range(T - 1)],
        "w_g": _xavier(rng(), d, d),
        "w_f": _xavier(rng(), d, 2 * d),
        "layers": [],
        "ln_out": gain(),
        "cls": [_xavier(rng(), w.V[t], d) for t in range(T)],
        "cls_bias": None,
    }
    for _ in range(w.L):
        lw = {}
        for n in LAYER_FIELDS:
            if n.startswith("ln_"):
                lw[n] = gain()
            elif n == "w1":
                lw[n] = _xavier(rng(), F, d)
            elif n == "w2":
                lw[n] = _xavier(rng(), d, F)
            else:
                lw[n] = _xavier(rng(), d, d)
        out["layers"].append(lw)
    if w.zipf_bias:
        # Zipf(1.1) popularity: bias = -1.1 ln(rank), rank a seeded permutation of 1..V
        out["cls_bias"] = [(-1.1 * np.log(rng().permutation(w.V[t]) + 1.0)).astype(np.float32) for t in range(T)]
    if w.Ve > 0:
        # eCPM-token step: position T+1, the embedding of s_T, a classifier over the V_e buckets.  Drawn from generators
        # of their own so that the other weights are the same with and without the step.
        vr = [np.random.default_rng(seed + 500 + i) for i in range(3)]
        out["value_pos"] = _store(vr[0].standard_normal(d).astype(np.float32), w.dtype)
        out["value_emb"] = _store(vr[1].standard_normal((w.V[T - 1], d)).astype(np.float32), w.dtype)
        out["value_cls"] = _store(_xavier(vr[2], w.Ve, d), w.dtype)
        out["value_bias"] = None
    # storage rounding (biases stay fp32 on both sides)
    for key in ("pos", "bos", "w_g", "w_f", "ln_out"):
        out[key] = _store(out[key], w.dtype)
    out["emb"] = [_store(a, w.dtype) for a in out["emb"]]
    out["cls"] = [_store(a, w.dtype) for a in out["cls"]]
    out["layers"] = [{n: _store(a, w.dtype) for n, a in lw.items()} for lw in out["layers"]]
    return out


def value_model(w: Workload, W):
    """The eCPM-token step is one more prediction step after s_T: the same decoder seen as a model of T+1 levels whose
    last codebook is the value vocabulary.  Returns (model_kwargs, weights) of that model; no arithmetic, only
    the weights of the step appended to the per-level lists."""
    assert w.Ve > 0
    kw = w.model_kwargs()
    kw["T"], kw["V"] = w.T + 1, list(w.V) + [w.Ve]
    X = dict(W)
    X["pos"] = np.concatenate([W["pos"], W["value_pos"][None, :]], axis=0)
    X["emb"] = list(W["emb"]) + [W["value_emb"]]
    X["cls"] = list(W["cls"]) + [W["value_cls"]]
    cb, vb = W.get("cls_bias"), W.get("value_bias")
    X["cls_bias"] = None if cb is None and vb is None else (list(cb) if cb is not None else [None] * w.T) + [vb]
    return kw, X


def make_lengths(w: Workload, seed=None):
    """Valid context length per request: S, or uniform in [len_min, S]."""
    seed = BASE_SEED + 1000 * w.cfg_id if seed is None else seed
    if w.len_min is None:
        return np.full(w.B, w.S, np.int32)
    return np.random.default_rng([seed, 9001]).integers(w.len_min, w.S + 1, size=w.B).astype(np.int32)


def make_context_request(w: Workload, r, length, seed=None):
    """Context memory of request r: [S,d], N(0,1) on the valid rows and
    10*N(0,1) garbage on the padded rows (a missing mask then fails loudly)."""
    seed = BASE_SEED + 1000 * w.cfg_id if seed is None else seed
    rng = np.random.default_rng([seed, 7, int(r)])
    x = rng.standard_normal((w.S, w.d), dtype=np.float32)
    x[length:] *= 10.0
    return _store(x, w.dtype)


def make_context(w: Workload, lengths=None, seed=None, requests=None):
    """Contexts of the listed requests (default: the whole batch) [n,S,d]."""
    lengths = make_lengths(w, seed) if lengths is None else lengths
    requests = range(w.B) if requests is None else requests
    return np.stack([make_context_request(w, r, int(lengths[r]), seed) for r in requests])
