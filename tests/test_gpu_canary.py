"""Out-of-bounds canaries around everything a decode call may write: the caller's workspace, the outputs, the trace buffers
and the value output sit inside larger allocations whose guard bands hold a byte pattern; after decodes at ragged shapes
(every kernel family: plain, 128x128 tiles, persistent GEMM, both attention kernels, both selection stages, FP8) the guard
bands must be untouched and the context must be unmodified."""
import numpy as np
import pytest
import torch

from helpers import tiny
from paper_2602_22732_amd import binding, synth

pytestmark = pytest.mark.gpu

GUARD = 1 << 16  # bytes on each side
PATTERN = 0xA5


class Guarded:
    """A device buffer of `nbytes` usable bytes (256-byte aligned start) between two guard bands."""

    def __init__(self, nbytes):
        self.n = int(nbytes)
        self.raw = torch.full((GUARD + self.n + GUARD + 256,), PATTERN, dtype=torch.uint8, device="cuda")
        off = (-self.raw.data_ptr() - GUARD) % 256
        self.start = GUARD + off
        self.view = self.raw[self.start:self.start + self.n]
        assert self.view.data_ptr() % 256 == 0

    def typed(self, dtype, shape):
        return self.view.view(dtype).view(*shape)

    def intact(self):
        before, after = self.raw[: self.start], self.raw[self.start + self.n:]
        return bool((before == PATTERN).all().item()) and bool((after == PATTERN).all().item())


SHAPES = [
    dict(dtype="f32", T=3, V=[40, 33, 50], d=64, H=2, F=96, L=3, K=1, S=37, B=5, beam=[7, 13, 9], len_min=5),
    dict(dtype="bf16", T=4, V=[17, 300, 64, 9], d=128, H=8, F=192, L=4, K=2, S=70, B=3, beam=[5, 64, 31, 40], len_min=1),
    dict(dtype="bf16", T=3, V=[40, 33, 50], d=128, H=2, F=96, L=3, K=2, S=37, B=5, beam=[7, 13, 9], len_min=1),       # absorbed lazy layers
    dict(dtype="bf16", T=2, V=[520, 1028], d=256, H=4, F=320, L=3, K=1, S=100, B=37, beam=[250, 300], len_min=3),    # 9250 rows: persistent GEMM, ragged last tile
    dict(dtype="bf16", fp8=True, T=2, V=[520, 516], d=256, H=4, F=384, L=2, K=1, S=64, B=37, beam=[250, 300]),      # FP8 persistent GEMM
    dict(dtype="bf16", Ve=33, T=2, V=[64, 50], d=128, H=2, F=128, L=2, K=1, S=20, B=3, beam=[8, 12]),                 # value step
    dict(dtype="bf16", T=3, V=[24, 20, 30], d=512, H=8, F=64, L=2, K=1, S=75, B=3, beam=[5, 8, 6], len_min=1),          # one-pass absorbed attention
]


@pytest.mark.parametrize("shape", SHAPES)
def test_decode_writes_nothing_outside_its_buffers(shape):
    shape = dict(shape)
    dtype, fp8 = shape.pop("dtype"), shape.pop("fp8", False)
    w, W, X = tiny(dtype=dtype, gain_jitter=0.1, **shape)
    w.fp8 = fp8
    lens = synth.make_lengths(w, seed=5)
    dec = binding.decoder_for(w, W)
    td = binding.torch_dtype(w.dtype)
    esz = 2 if dtype == "bf16" else 4
    g_ctx = Guarded(w.B * w.S * w.d * esz)
    ctx = g_ctx.typed(td, (w.B, w.S, w.d))
    ctx.copy_(torch.from_numpy(X).to("cuda", dtype=td))
    ctx_before = ctx.clone()
    g_len = Guarded(w.B * 4)
    cl = g_len.typed(torch.int32, (w.B,))
    cl.copy_(torch.from_numpy(lens).cuda())
    bT = w.beam[-1]
    g_ws = Guarded(dec.workspace_bytes(w.B, w.S, w.beam))
    g_sid, g_lp = Guarded(w.B * bT * w.T * 4), Guarded(w.B * bT * 4)
    out_sid, out_lp = g_sid.typed(torch.int32, (w.B, bT, w.T)), g_lp.typed(torch.float32, (w.B, bT))
    g_val = Guarded(w.B * bT * w.Ve * 4) if w.Ve else None
    # trace buffers: per level parent, token, score [B, b_t]
    g_tr = {k: [Guarded(w.B * b * 4) for b in w.beam] for k in ("parent", "tok", "score")}
    import ctypes as C
    arrs = [(C.c_void_p * w.T)(*[g.view.data_ptr() for g in g_tr[k]]) for k in ("parent", "tok", "score")]
    assert dec.L_.gr4ad_decode_set_trace(dec.handle, *arrs) == 0
    guards = [g_ctx, g_len, g_ws, g_sid, g_lp] + ([g_val] if g_val else []) + [g for v in g_tr.values() for g in v]
    for _ in range(2):  # twice: the second call starts from the first call's workspace contents
        dec.decode_batch(ctx, cl, w.beam, workspace=g_ws.view, out_sid=out_sid, out_logprob=out_lp, value=bool(w.Ve),
                         out_value=g_val.typed(torch.float32, (w.B, bT, w.Ve)) if g_val else None)
        torch.cuda.synchronize()
        for i, g in enumerate(guards):
            assert g.intact(), "guard band %d was written" % i
        assert torch.equal(ctx, ctx_before), "the context was modified"
    sid, lp = out_sid.cpu().numpy(), out_lp.cpu().numpy()
    assert (np.diff(lp, axis=1) <= 0).all() and np.isfinite(lp).all()
    for t in range(w.T):
        assert sid[..., t].min() >= 0 and sid[..., t].max() < w.V[t]
    dec.close()
