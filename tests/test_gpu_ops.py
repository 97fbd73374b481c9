"""GPU parity tests of the single-operation entry points against the CPU oracle's primitives."""
import zlib

import numpy as np
import pytest
import torch

import oracle
from gpu_common import judge_selection
from paper_2602_22732_amd import binding, synth

pytestmark = pytest.mark.gpu
RNG = np.random.default_rng(2602)


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to("cuda", dtype=binding.torch_dtype(dtype))


@pytest.mark.parametrize("dtype,M,N,K", [
    ("f32", 300, 200, 72), ("f32", 1, 5, 8), ("f32", 129, 64, 256),
    ("bf16", 300, 200, 72),                       # K % 64 != 0: plain kernel
    ("bf16", 300, 200, 192), ("bf16", 1, 8, 64),  # MFMA 128x128 tiles, ragged M and N
    ("bf16", 9000, 520, 256),                     # MFMA 256x256 tiles, ragged M and N
    ("bf16", 8192, 1024, 1024),
])
def test_linear_matches_oracle(dtype, M, N, K):
    A, W = RNG.standard_normal((M, K)).astype(np.float32), RNG.standard_normal((N, K)).astype(np.float32) / np.sqrt(K)
    bias = RNG.standard_normal(N).astype(np.float32)
    if dtype == "bf16":
        A, W = synth.round_bf16(A), synth.round_bf16(W)
    rows = np.unique(np.concatenate([np.arange(min(M, 40)), RNG.integers(0, M, 40), [M - 1]]))
    ref = oracle.prim_linear(A[rows], W) + bias
    out = binding.op_linear(dev(A, dtype), dev(W, dtype), torch.from_numpy(bias).cuda(), out_f32=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy()[rows], ref, atol=2e-5 * np.sqrt(K) if dtype == "f32" else 1e-4 * np.sqrt(K))
    out2 = binding.op_linear(dev(A, dtype), dev(W, dtype), None, out_f32=False)
    torch.cuda.synchronize()
    tol = 1e-4 if dtype == "f32" else 2e-2
    np.testing.assert_allclose(out2.float().cpu().numpy()[rows], ref - bias, atol=tol, rtol=tol)


@pytest.mark.parametrize("B,n,V,k", [
    (3, 1, 256, 16), (2, 16, 256, 16), (2, 7, 1000, 33), (1, 64, 1024, 128), (2, 5, 37, 37), (1, 3, 9, 27),
    (2, 40, 300, 512), (1, 130, 2048, 1024),
])
def test_select_matches_oracle(B, n, V, k):
    logits = (RNG.standard_normal((B, n, V)) * 1.5).astype(np.float32)
    cum = (-RNG.random((B, n)) * 3).astype(np.float32)
    parent, tok, score = binding.op_select(torch.from_numpy(logits).cuda(), torch.from_numpy(cum).cuda(), k)
    torch.cuda.synchronize()
    parent, tok, score = parent.cpu().numpy(), tok.cpu().numpy(), score.cpu().numpy()
    for b in range(B):
        lp = np.stack([oracle.prim_log_softmax(logits[b, i]) for i in range(n)])
        allsc = cum[b].astype(np.float64)[:, None] + lp
        flat = parent[b].astype(np.int64) * V + tok[b]
        judge_selection(allsc, flat, score[b], k, tol=2e-5, margin=1e-5, what="select b=%d" % b)
        # against the oracle's own selection: identical wherever its gaps are wide
        oflat, osc = oracle.prim_topk(allsc, k)
        wide = np.abs(np.diff(osc)).min() > 1e-5 if k > 1 else True
        if wide and (k == n * V or allsc.ravel()[np.argsort(-allsc.ravel())[k]] < osc[-1] - 1e-5):
            assert np.array_equal(flat, oflat)


@pytest.mark.parametrize("profile", ["steep", "flat", "first_row_worst", "first_row_minus_inf"])
@pytest.mark.parametrize("B,n,V,k", [(2, 24, 8192, 1024), (1, 9, 5000, 600), (2, 6, 4096, 4096), (1, 300, 512, 200),
                                     (1, 3, 16384, 4096), (2, 5, 16384, 700)])   # the last two: the largest codebook (and beam) the library takes
def test_select_request_bound_regimes(profile, B, n, V, k):
    # The per-row cut is tightened by a bound taken from each request's first row: rows far below it contribute
    # nothing, rows level with it contribute about k each, and any row may be the first one.
    rng = np.random.default_rng(zlib.crc32(repr((profile, B, n, V, k)).encode()))
    logits = (rng.standard_normal((B, n, V)) * 1.2).astype(np.float32)
    if profile == "steep":
        cum = np.tile(-4.0 * np.arange(n, dtype=np.float32), (B, 1))
    elif profile == "flat":
        cum = np.full((B, n), -7.5, dtype=np.float32)
    elif profile == "first_row_worst":
        cum = np.tile(-3.0 * np.arange(n, dtype=np.float32)[::-1].copy(), (B, 1))
    else:
        cum = (-rng.random((B, n)) * 2).astype(np.float32)
        cum[:, 0] = -np.inf
    parent, tok, score = binding.op_select(torch.from_numpy(logits).cuda(), torch.from_numpy(cum).cuda(), k)
    torch.cuda.synchronize()
    parent, tok, score = parent.cpu().numpy(), tok.cpu().numpy(), score.cpu().numpy()
    for b in range(B):
        lp = np.stack([oracle.prim_log_softmax(logits[b, i]) for i in range(n)])
        allsc = cum[b].astype(np.float64)[:, None] + lp
        flat = parent[b].astype(np.int64) * V + tok[b]
        assert len(set(flat.tolist())) == k
        judge_selection(allsc, flat, score[b], k, tol=2e-5, margin=1e-5, what="%s b=%d" % (profile, b))


@pytest.mark.parametrize("profile", ["random", "steep", "flat", "first_row_worst", "ties"])
@pytest.mark.parametrize("B,n,V,k", [(2, 24, 8192, 1024), (1, 9, 5000, 600), (2, 6, 4096, 4096), (1, 300, 512, 200), (3, 1, 256, 16),
                                     (2, 16, 256, 16), (1, 64, 1024, 128), (1, 130, 2048, 1024), (2, 40, 304, 512), (1, 700, 8, 8),
                                     (5, 37, 1000, 33)])
def test_select_f16_matches_oracle(profile, B, n, V, k):
    # Half-precision logits (what the classifier hands over in bf16 mode).  With several rows per request and k <= V the
    # bounded pass reads the rows packed and lists the rows that need their own cut; "flat" and "ties" put many rows on that
    # list, "steep" almost none.
    rng = np.random.default_rng(zlib.crc32(repr(("f16", profile, B, n, V, k)).encode()))
    logits = (rng.standard_normal((B, n, V)) * 1.2).astype(np.float16)
    cum = (-rng.random((B, n)) * 2).astype(np.float32)
    if profile == "steep":
        cum = np.tile(-4.0 * np.arange(n, dtype=np.float32), (B, 1))
    elif profile == "flat":
        cum = np.full((B, n), -7.5, dtype=np.float32)
    elif profile == "first_row_worst":
        cum = np.tile(-3.0 * np.arange(n, dtype=np.float32)[::-1].copy(), (B, 1))
    elif profile == "ties":  # few distinct values and equal rows: crowded bounds, more than k candidates level with them
        logits = np.round(rng.standard_normal((B, 1, V)) * 2).astype(np.float16).repeat(n, 1)
        cum = np.zeros((B, n), dtype=np.float32)
    parent, tok, score = binding.op_select(torch.from_numpy(logits).cuda(), torch.from_numpy(cum).cuda(), k)
    torch.cuda.synchronize()
    parent, tok, score = parent.cpu().numpy(), tok.cpu().numpy(), score.cpu().numpy()
    assert (parent >= 0).all() and (parent < n).all() and (tok >= 0).all() and (tok < V).all()
    for b in range(B):
        lp = np.stack([oracle.prim_log_softmax(logits[b, i].astype(np.float32)) for i in range(n)])
        allsc = cum[b].astype(np.float64)[:, None] + lp
        flat = parent[b].astype(np.int64) * V + tok[b]
        assert len(set(flat.tolist())) == k
        if profile == "ties":
            # equal rows are bit-identical on the GPU too: equal scores come out in ascending flat index
            sc32 = np.float32(np.tile(np.float32(lp[0]), (n, 1)))
            oflat, _ = oracle.prim_topk(sc32.astype(np.float64), k)
            assert np.array_equal(flat, oflat)
        else:
            judge_selection(allsc, flat, score[b], k, tol=2e-5, margin=1e-5, what="f16 %s b=%d" % (profile, b))


@pytest.mark.parametrize("seed", range(40))
@pytest.mark.parametrize("half", [True, False])
def test_select_random_shapes(seed, half):
    # seeded random shapes through both logit formats: every register width of the wavefront kernels with and without a ragged
    # tail, cuts above and below the codebook size, one to many rows per request, -inf beams, crowded ties
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.choice([8, 16, 24, 64, 200, 256, 264, 1000, 1024, 2048, 2056, 4096, 5000, 8192]))
    n = int(rng.choice([1, 2, 3, 7, 33, 64, 130, 257]))
    B = int(rng.integers(1, 4))
    k = int(min(n * V, rng.choice([1, 2, 7, 16, 33, 128, 512, 1000, 4096])))
    prof = str(rng.choice(["rand", "steep", "flat", "ties", "neginf"]))
    sigma = float(rng.choice([0.3, 1.5, 4.0]))
    logits = (rng.standard_normal((B, n, V)) * sigma).astype(np.float16 if half else np.float32)
    cum = (-rng.random((B, n)) * 3).astype(np.float32)
    if prof == "steep":
        cum = np.tile(-2.5 * np.arange(n, dtype=np.float32), (B, 1))
    elif prof == "flat":
        cum[:] = -1.25
    elif prof == "ties":
        logits = np.round(logits.astype(np.float32)).astype(logits.dtype)
    elif prof == "neginf" and n > 1:
        cum[:, int(rng.integers(0, n))] = -np.inf
    parent, tok, score = binding.op_select(torch.from_numpy(logits).cuda(), torch.from_numpy(cum).cuda(), k)
    torch.cuda.synchronize()
    parent, tok, score = parent.cpu().numpy(), tok.cpu().numpy(), score.cpu().numpy()
    what = "seed %d half=%s B=%d n=%d V=%d k=%d %s" % (seed, half, B, n, V, k, prof)
    assert (parent >= 0).all() and (parent < n).all() and (tok >= 0).all() and (tok < V).all(), what
    for b in range(B):
        lp = np.stack([oracle.prim_log_softmax(logits[b, i].astype(np.float32)) for i in range(n)])
        allsc = cum[b].astype(np.float64)[:, None] + lp
        flat = parent[b].astype(np.int64) * V + tok[b]
        fin = np.isfinite(allsc.ravel()[flat])  # (-inf candidates may fill a cut larger than the finite ones: any of them is right)
        sc = np.where(np.isfinite(allsc), allsc, -1e30)
        judge_selection(sc, flat, np.where(fin, score[b], -1e30), k, tol=3e-5, margin=2e-5, what=what + " b=%d" % b)


def test_select_f16_refuses_shapes_the_packed_rows_cannot_hold():
    z = torch.zeros(1, 2, 12, dtype=torch.float16, device="cuda")
    with pytest.raises(RuntimeError):
        binding.op_select(z, None, 3)          # V not a multiple of 8
    z = torch.zeros(1, 1, 16384, dtype=torch.float16, device="cuda")
    with pytest.raises(RuntimeError):
        binding.op_select(z, None, 3)          # V above 8192


def test_select_exact_ties_and_quantised_scores():
    # equal rows: every candidate of equal score must come out in ascending flat index
    B, n, V, k = 2, 6, 500, 700
    logits = np.round(RNG.standard_normal((1, 1, V)) * 2).astype(np.float32).repeat(B, 0).repeat(n, 1)  # few distinct values, all rows equal
    parent, tok, score = binding.op_select(torch.from_numpy(logits).cuda(), None, k)
    torch.cuda.synchronize()
    flat = parent.cpu().numpy().astype(np.int64) * V + tok.cpu().numpy()
    lp = oracle.prim_log_softmax(logits[0, 0])
    allsc = np.float32(np.tile(lp, (n, 1)))  # compare in the kernel's precision: rows are bit-identical on the GPU too
    oflat, _ = oracle.prim_topk(allsc.astype(np.float64), k)
    for b in range(B):
        assert np.array_equal(flat[b], oflat)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,n,S,d,H", [(2, 5, 37, 64, 2), (1, 70, 130, 128, 2), (3, 1, 1, 64, 4), (2, 33, 200, 256, 2),
                                       (2, 200, 300, 128, 2), (1, 600, 129, 192, 3), (2, 300, 64, 128, 4), (1, 1030, 70, 64, 2)])
def test_cross_attention_matches_oracle(dtype, B, n, S, d, H):
    q = RNG.standard_normal((B, n, d)).astype(np.float32)
    kv = RNG.standard_normal((B, S, 2 * d)).astype(np.float32)
    lens = RNG.integers(1, S + 1, size=B).astype(np.int32)
    if dtype == "bf16":
        q, kv = synth.round_bf16(q), synth.round_bf16(kv)
    for b in range(B):
        kv[b, lens[b]:] = 1e4  # padding must not matter
    out = binding.op_cross_attention(dev(q, dtype), dev(kv, dtype), torch.from_numpy(lens).cuda(), H)
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    for b in range(B):
        ref = oracle.prim_mha(q[b], kv[b, :lens[b], :d], kv[b, :lens[b], d:], H, False)
        np.testing.assert_allclose(out[b], ref, atol=2e-5 if dtype == "f32" else 1.5e-2)


def context_attention_bound(xv):
    """What bf16 storage allows: the kernel rounds every probability that enters the product (8 significand bits: relative
    error up to 2^-8; the normaliser sums the unrounded ones) and the weighted sum itself (2^-8), so an output is off by at
    most 2^-8 (sum_s p_s |x_s| + |z|) <= 2^-7 of the largest value it averages; 1e-3 on top for the fp32 accumulation and the
    hardware's exp2.  (A wrong operand, index or mask shows as an error of the size of the values themselves.)"""
    return 2.0 ** -7 * float(np.abs(xv).max()) + 1e-3


@pytest.mark.parametrize("B,RQ,S,d,gain", [(3, 64, 200, 1024, 1.0), (2, 48, 33, 1024, 4.0), (2, 17, 1, 1024, 1.0), (3, 32, 95, 1024, 2.0),
                                          (2, 24, 130, 512, 1.0), (3, 64, 64, 512, 6.0), (2, 5, 31, 512, 1.0), (4, 40, 257, 512, 3.0),
                                          (2, 80, 150, 1024, 2.0), (3, 128, 70, 512, 1.0), (2, 65, 40, 512, 3.0)])  # more than 64 query rows: two launches
def test_context_attention_matches_oracle(B, RQ, S, d, gain):
    """Attention over the raw context rows as keys and values (the lazy layers' absorbed form) = single-head attention with
    K = V = x in the oracle; `gain` sharpens the softmax so that the running maximum moves between tiles."""
    q = synth.round_bf16((gain * RNG.standard_normal((B, RQ, d))).astype(np.float32))
    x = synth.round_bf16(RNG.standard_normal((B, S, d)).astype(np.float32))
    lens = RNG.integers(1, S + 1, size=B).astype(np.int32)
    lens[0] = S
    for b in range(B):
        x[b, lens[b]:] = 1e4  # padding must not matter
    scale = 1.0 / np.sqrt(d)
    out = binding.op_context_attention(dev(q, "bf16"), dev(x, "bf16"), torch.from_numpy(lens).cuda(), scale)
    full = binding.op_context_attention(dev(q[:1], "bf16"), dev(x[:1], "bf16"), None, scale)
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    for b in range(B):
        ref = oracle.prim_mha(q[b], x[b, :lens[b]], x[b, :lens[b]], 1, False)
        np.testing.assert_allclose(out[b], ref, atol=context_attention_bound(x[b, :lens[b]]))
    assert np.array_equal(full.float().cpu().numpy()[0], out[0])  # no length array = all rows


@pytest.mark.parametrize("seed", range(12))
def test_context_attention_random_shapes(seed):
    rng = np.random.default_rng(900 + seed)
    d = int(rng.choice([512, 1024]))
    B, RQ, S = int(rng.integers(1, 6)), int(rng.integers(1, 129)), int(rng.integers(1, 300))
    gain = float(rng.choice([1.0, 3.0, 8.0]))
    q = synth.round_bf16((gain * rng.standard_normal((B, RQ, d))).astype(np.float32))
    x = synth.round_bf16(rng.standard_normal((B, S, d)).astype(np.float32))
    lens = rng.integers(1, S + 1, size=B).astype(np.int32)
    print("seed", seed, "B RQ S d gain", B, RQ, S, d, gain, "lens", lens.tolist(), flush=True)
    out = binding.op_context_attention(dev(q, "bf16"), dev(x, "bf16"), torch.from_numpy(lens).cuda(), 1.0 / np.sqrt(d))
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    for b in range(B):
        ref = oracle.prim_mha(q[b], x[b, :lens[b]], x[b, :lens[b]], 1, False)
        np.testing.assert_allclose(out[b], ref, atol=context_attention_bound(x[b, :lens[b]]))


def test_context_attention_refuses_what_it_does_not_cover():
    q = torch.zeros((1, 129, 512), dtype=torch.bfloat16, device="cuda")
    x = torch.zeros((1, 8, 512), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(RuntimeError):
        binding.op_context_attention(q, x, None, 1.0)
    with pytest.raises(RuntimeError):
        binding.op_context_attention(q[:, :8, :256].contiguous(), x[:, :, :256].contiguous(), None, 1.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gather_rows_is_an_exact_copy(dtype):
    B, n, k, T, d2 = 3, 9, 14, 4, 64
    src = dev(RNG.standard_normal((B, n, T, d2)), dtype)
    parent = torch.from_numpy(RNG.integers(0, n, size=(B, k)).astype(np.int32)).cuda()
    dst = binding.op_gather_rows(src, parent, row_elems=3 * d2)  # only the first 3 positions are live
    torch.cuda.synchronize()
    ref = torch.stack([src[b][parent[b].long()] for b in range(B)])
    assert torch.equal(dst[:, :, :3], ref[:, :, :3])
    assert (dst[:, :, 3] == 0).all()
