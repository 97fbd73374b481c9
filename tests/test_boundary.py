"""CPU checks of the C-ABI boundary: the library loads, exports every function
include/gr4ad.h declares, and rejects bad arguments before touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2602_22732_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(gr4ad_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_function():
    L = binding.lib()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS) | set(binding.SERVING_EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_strerror_and_null_handling():
    L = binding.lib()
    assert L.gr4ad_strerror(0) == b"ok"
    assert L.gr4ad_strerror(-1) == b"invalid argument"
    assert L.gr4ad_strerror(-3).startswith(b"workspace")
    assert L.gr4ad_strerror(-99) == b"unknown status"
    L.gr4ad_decode_free(None)  # no-op
    beam = (C.c_int32 * 3)(1, 1, 1)
    assert L.gr4ad_decode_workspace_bytes(None, 1, 1, beam) == 0
    assert L.gr4ad_decode_batch(None, None, None, 1, 1, beam, None, 0, None, None, None) == -1
    assert L.gr4ad_decode_set_trace(None, None, None, None) == -1
    assert L.gr4ad_decode_set_value_output(None, None) == -1


def _desc(**over):
    kw = dict(d_model=64, n_heads=2, d_ffn=128, n_layers=3, n_lazy=1, n_levels=3, max_batch=4, max_ctx=16, dtype=0, rms_eps=1e-6)
    kw.update(over)
    V = np.array(kw.pop("codebook", [8, 8, 8]), np.int32)
    mb = np.array(kw.pop("max_beam", [4, 4, 4]), np.int32)
    d = binding.ModelDesc(codebook=V.ctypes.data_as(binding._IP), max_beam=mb.ctypes.data_as(binding._IP), **kw)
    d._keep = (V, mb)
    return d


@pytest.mark.parametrize("over,status,needle", [
    (dict(n_lazy=3), -1, "n_lazy"),
    (dict(n_lazy=-1), -1, "n_lazy"),
    (dict(n_heads=3), -1, "divisible"),
    (dict(n_levels=0), -1, "n_levels"),
    (dict(n_levels=9, codebook=[8] * 9, max_beam=[4] * 9), -1, "n_levels"),
    (dict(d_model=0), -1, "positive"),
    (dict(dtype=7), -1, "dtype"),
    (dict(codebook=[8, 0, 8]), -1, "codebook"),
    (dict(d_model=48, n_heads=2), -2, "head width"),
    (dict(max_beam=[4, 5000, 4]), -2, "max_beam"),
    (dict(codebook=[8, 8, 20000]), -2, "codebook"),
    (dict(n_value_buckets=-1), -1, "n_value_buckets"),
    (dict(vanilla_input=1, n_lazy=1), -1, "vanilla_input"),
    (dict(n_value_buckets=16, n_levels=8, codebook=[8] * 8, max_beam=[4] * 8), -2, "value step"),
])
def test_init_rejects_bad_descriptions_without_a_gpu(over, status, needle):
    L = binding.lib()
    out = C.c_void_p(0xDEAD)
    w = binding.Weights()
    rc = L.gr4ad_decode_init(C.byref(_desc(**over)), C.byref(w), C.byref(out))
    assert rc == status
    assert needle in L.gr4ad_last_error(None).decode()
    assert out.value == 0xDEAD  # untouched on failure


def test_init_rejects_null_pointers():
    L = binding.lib()
    out = C.c_void_p()
    assert L.gr4ad_decode_init(None, None, C.byref(out)) == -1
    assert L.gr4ad_decode_init(C.byref(_desc()), None, C.byref(out)) == -1
    assert L.gr4ad_decode_init(C.byref(_desc()), C.byref(binding.Weights()), C.byref(out)) == -1  # all weight pointers NULL
    assert "NULL" in L.gr4ad_last_error(None).decode()
    assert L.gr4ad_decode_init(C.byref(_desc()), C.byref(binding.Weights()), None) == -1


def test_select_workspace_formula():
    L = binding.lib()
    def expect(B, n, V, k):
        # candidates [B][n*m] 64-bit keys, the first rows' cuts [B][m], request bounds [B] (64-bit), request counts [B] (32-bit),
        # the count of rows listed for their own cut (256 bytes) and the list [B*n] of {row, slot} pairs
        m = min(k, V)
        r = lambda x: (x + 255) // 256 * 256
        return r(B * n * m * 8) + r(B * m * 8) + r(B * 8) + r(B * 4) + 256 + r(B * n * 8)
    assert L.gr4ad_op_select_workspace_bytes(3, 5, 100, 7) == expect(3, 5, 100, 7)
    assert L.gr4ad_op_select_workspace_bytes(3, 5, 4, 7) == expect(3, 5, 4, 7)
    assert L.gr4ad_op_select_workspace_bytes(0, 5, 4, 7) == 0


def test_ops_reject_bad_arguments_without_a_gpu():
    L = binding.lib()
    assert L.gr4ad_op_linear(0, None, None, None, None, 1, 1, 1, 0, None) == -1
    assert L.gr4ad_op_select(None, None, 1, 1, 1, 1, None, 0, None, None, None, None) == -1
    assert L.gr4ad_op_select_f16(None, None, 1, 1, 8, 1, None, 0, None, None, None, None) == -1
    assert L.gr4ad_op_cross_attention(0, None, None, None, None, 1, 1, 1, 8, 1, None, 0, None) == -1
    assert L.gr4ad_op_cross_attention_workspace_bytes(1, 2, 100, 128, 2) == 2 * 128 * 128 * 2   # bf16, dh 64: S padded to 128
    assert L.gr4ad_op_cross_attention_workspace_bytes(0, 2, 100, 128, 2) == 0                   # float32 runs on the plain kernel
    assert L.gr4ad_op_gather_rows(0, None, None, None, 1, 1, 1, 8, 8, None) == -1
    assert L.gr4ad_op_context_attention(1, None, None, None, None, 1, 1, 1, 512, 1.0, None) == -1
    some = C.c_int32(0)  # (shapes are refused on the host, before any pointer is looked at)
    ptr = C.addressof(some)
    for args in ((0, 1, 8, 16, 512), (1, 1, 129, 16, 512), (1, 1, 8, 16, 256)):  # float32; too many query rows; a width without a kernel
        assert L.gr4ad_op_context_attention(args[0], ptr, ptr, None, ptr, args[1], args[2], args[3], args[4], 1.0, None) == -2
    # the selection on static scratch checks its arguments and its size limit on the host, before any device call
    assert L.gr4ad_op_select_static(None, None, 1, 1, 8, 1, None, None, None, None) == -1
    one = C.c_int32(0)
    p = C.addressof(one)  # stands for a device pointer: never dereferenced, the size check comes first
    assert L.gr4ad_op_select_static(p, None, 64, 512, 8192, 512, p, p, p, None) == -3
    assert b"static scratch" in L.gr4ad_last_error(None)
    assert L.gr4ad_op_select_static(p, None, 1, 2, 4, 9, p, p, p, None) == -1  # k > n*V
