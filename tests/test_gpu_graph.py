"""gr4ad_decode_batch under HIP graph capture: the call only launches kernels on the stream it is given (after one eager
warm-up call, which sets the kernels' attributes), so a serving loop can capture it once and replay it.  Every replay is
checked against an eager call on the same inputs, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from helpers import tiny
from paper_2602_22732_amd import binding, synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,fp8", [("f32", False), ("bf16", False), ("bf16", True)])
def test_captured_decode_replays_match_eager_calls(dtype, fp8):
    w, W, X = tiny(dtype=dtype, gain_jitter=0.1, T=3, V=[300, 256, 280], d=128, H=2, F=256, L=3, K=2, S=40, B=6, beam=[16, 24, 20], len_min=3)
    w.fp8 = fp8
    lens = synth.make_lengths(w, seed=3)
    dec = binding.decoder_for(w, W)
    td = binding.torch_dtype(dtype)
    ctx = torch.from_numpy(X).to("cuda", dtype=td).contiguous()
    cl = torch.from_numpy(lens).cuda()
    ws = torch.empty(dec.workspace_bytes(w.B, w.S, w.beam), dtype=torch.uint8, device="cuda")
    sid = torch.empty(w.B, w.beam[-1], w.T, dtype=torch.int32, device="cuda")
    lp = torch.empty(w.B, w.beam[-1], dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dec.decode_batch(ctx, cl, w.beam, workspace=ws, out_sid=sid, out_logprob=lp)   # eager warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dec.decode_batch(ctx, cl, w.beam, workspace=ws, out_sid=sid, out_logprob=lp)
    rng = np.random.default_rng(8)
    for replay in range(4):
        # new contexts and lengths in the captured buffers
        Xn = synth._store(rng.standard_normal(X.shape).astype(np.float32), dtype)
        ln = rng.integers(1, w.S + 1, w.B).astype(np.int32)
        ctx.copy_(torch.from_numpy(Xn).to("cuda", dtype=td))
        cl.copy_(torch.from_numpy(ln).cuda())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_sid, got_lp = sid.clone(), lp.clone()
        # eager work in between: a decode with its own buffers
        want_sid, want_lp = dec.decode_batch(ctx, cl, w.beam)
        torch.cuda.synchronize()
        assert torch.equal(got_sid, want_sid) and torch.equal(got_lp, want_lp), "replay %d differs from the eager call" % replay
        assert torch.isfinite(got_lp).all()
    dec.close()
