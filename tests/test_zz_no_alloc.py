"""gr4ad_op_select_static (the selection for callers that cannot allocate device memory) against gr4ad_op_select,
through the C ABI: same kernels, so the results must be bit-identical.  Two calls in a row share the static scratch,
the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2602_22732_amd import binding

pytestmark = pytest.mark.gpu


def _case(seed, B, n, V, k):
    g = torch.Generator(device="cpu").manual_seed(seed)
    logits = (torch.randn(B, n, V, generator=g, dtype=torch.float32) * 2.0).cuda().contiguous()
    cum = (-torch.rand(B, n, generator=g, dtype=torch.float32) * 3.0).cuda().contiguous()
    assert logits.dtype == torch.float32 and cum.dtype == torch.float32
    return logits, cum


def _outputs(B, k):
    # allocated by the caller, before the call under test
    return (torch.full((B, k), -1, dtype=torch.int32, device="cuda"), torch.full((B, k), -1, dtype=torch.int32, device="cuda"),
            torch.full((B, k), float("nan"), dtype=torch.float32, device="cuda"))


def test_static_scratch_selection_equals_workspace_selection_on_two_calls_in_a_row():
    # first call: a larger problem (bounded stage A, 2 MiB of candidates); second: a smaller one over the same scratch
    for seed, (B, n, V, k) in enumerate([(16, 128, 2048, 128), (3, 5, 512, 7), (2, 1, 300, 300)]):
        logits, cum = _case(100 + seed, B, n, V, k)
        want = [t.cpu().numpy() for t in binding.op_select(logits, cum, k)]
        outs = _outputs(B, k)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        binding.op_select_static(logits, cum, k, *outs)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        got = [t.cpu().numpy() for t in outs]
        for w, g_, name in zip(want, got, ("parent", "tok", "score")):
            assert np.array_equal(w, g_), "%s differs at case B=%d n=%d V=%d k=%d" % (name, B, n, V, k)
        # and against the definition: the k best of cum + log_softmax(logits), ties by lowest flat index
        sc = (cum[:, :, None].double() + torch.log_softmax(logits.double(), dim=2)).reshape(B, n * V).cpu().numpy()
        order = np.argsort(-sc, axis=1, kind="stable")[:, :k]
        flat = got[0].astype(np.int64) * V + got[1]
        assert np.abs(np.take_along_axis(sc, flat, axis=1) - got[2]).max() < 1e-4
        assert np.abs(np.take_along_axis(sc, order, axis=1) - got[2]).max() < 1e-4


def test_static_scratch_selection_refuses_what_does_not_fit():
    B, n, V, k = 64, 512, 8192, 512  # 128 MiB of candidates
    L = binding.lib()
    assert L.gr4ad_op_select_workspace_bytes(B, n, V, k) > binding.SELECT_STATIC_BYTES
    dummy = torch.zeros(16, dtype=torch.float32, device="cuda")  # never read: the size check comes first
    outs = _outputs(1, 1)
    st = L.gr4ad_op_select_static(dummy.data_ptr(), None, B, n, V, k, outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(), None)
    assert st == -3
    assert b"static scratch" in L.gr4ad_last_error(None)
    assert L.gr4ad_op_select_static(None, None, 1, 1, 8, 1, outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(), None) == -1
