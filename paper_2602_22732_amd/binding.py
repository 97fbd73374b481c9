"""Thin Python binding of libgr4ad.so (C ABI in include/gr4ad.h).

Argument marshalling only: torch is used to own device memory and streams, every
step of the decode runs in the library's HIP kernels.  There is no fallback: if
the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgr4ad.so")

F32, BF16 = 0, 1
LAYER_FIELDS = ["ln_x", "wq_x", "wk_x", "wv_x", "wo_x", "ln_s", "wq_s", "wk_s", "wv_s", "wo_s", "ln_f", "w1", "w2"]
EXPORTS = ["gr4ad_decode_init", "gr4ad_decode_workspace_bytes", "gr4ad_decode_batch", "gr4ad_decode_set_trace",
           "gr4ad_decode_set_value_output",
           "gr4ad_decode_free", "gr4ad_strerror", "gr4ad_last_error", "gr4ad_op_linear", "gr4ad_op_select_workspace_bytes",
           "gr4ad_op_quantize_rows", "gr4ad_op_linear_fp8",
           "gr4ad_op_select", "gr4ad_op_select_f16", "gr4ad_op_select_static", "gr4ad_op_cross_attention_workspace_bytes", "gr4ad_op_cross_attention", "gr4ad_op_context_attention", "gr4ad_op_gather_rows",
           "gr4ad_profile_enable",
           "gr4ad_profile_kernel_count", "gr4ad_profile_kernel_name", "gr4ad_profile_read"]

SERVING_EXPORTS = ["gr4ad_tabs_create", "gr4ad_tabs_free", "gr4ad_tabs_observe", "gr4ad_tabs_qps", "gr4ad_tabs_schedule",
                   "gr4ad_cache_create", "gr4ad_cache_free", "gr4ad_cache_insert", "gr4ad_cache_lookup", "gr4ad_cache_lookup_batch",
                   "gr4ad_cache_stats"]

_IP = C.POINTER(C.c_int32)
_VP = C.c_void_p


class ModelDesc(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ffn", C.c_int32), ("n_layers", C.c_int32),
                ("n_lazy", C.c_int32), ("n_levels", C.c_int32), ("codebook", _IP), ("max_beam", _IP),
                ("max_batch", C.c_int32), ("max_ctx", C.c_int32), ("dtype", C.c_int), ("rms_eps", C.c_float),
                ("n_value_buckets", C.c_int32), ("fp8_gemm", C.c_int32), ("vanilla_input", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, _VP) for n in LAYER_FIELDS]


class Weights(C.Structure):
    _fields_ = [("pos_dev", _VP), ("bos_dev", _VP), ("emb_dev", C.POINTER(_VP)), ("w_g_dev", _VP), ("w_f_dev", _VP),
                ("layers", C.POINTER(LayerWeights)), ("ln_out_dev", _VP), ("cls_dev", C.POINTER(_VP)),
                ("cls_bias_dev", C.POINTER(_VP)),
                ("value_pos_dev", _VP), ("value_emb_dev", _VP), ("value_cls_dev", _VP), ("value_bias_dev", _VP)]


class TabsConfig(C.Structure):
    _fields_ = [("n_levels", C.c_int32), ("beam_base", _IP), ("max_beam", _IP), ("codebook", _IP), ("qps_peak", C.c_double),
                ("scale_min", C.c_double), ("scale_max", C.c_double), ("step", C.c_double), ("tau_s", C.c_double)]


class Gr4adError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("gr4ad status %d: %s" % (status, message))
        self.status = status


_lib = None


def lib():
    """Loads libgr4ad.so; raises if it has not been built (python -m paper_2602_22732_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s not built: run `python -m paper_2602_22732_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.gr4ad_decode_init.restype = C.c_int
        L.gr4ad_decode_init.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(_VP)]
        L.gr4ad_decode_workspace_bytes.restype = C.c_size_t
        L.gr4ad_decode_workspace_bytes.argtypes = [_VP, C.c_int32, C.c_int32, _IP]
        L.gr4ad_decode_batch.restype = C.c_int
        L.gr4ad_decode_batch.argtypes = [_VP, _VP, _VP, C.c_int32, C.c_int32, _IP, _VP, C.c_size_t, _VP, _VP, _VP]
        L.gr4ad_decode_set_trace.restype = C.c_int
        L.gr4ad_decode_set_trace.argtypes = [_VP, C.POINTER(_VP), C.POINTER(_VP), C.POINTER(_VP)]
        L.gr4ad_decode_set_value_output.restype = C.c_int
        L.gr4ad_decode_set_value_output.argtypes = [_VP, _VP]
        L.gr4ad_decode_free.restype = None
        L.gr4ad_decode_free.argtypes = [_VP]
        L.gr4ad_strerror.restype = C.c_char_p
        L.gr4ad_strerror.argtypes = [C.c_int]
        L.gr4ad_last_error.restype = C.c_char_p
        L.gr4ad_last_error.argtypes = [_VP]
        L.gr4ad_op_linear.restype = C.c_int
        L.gr4ad_op_linear.argtypes = [C.c_int, _VP, _VP, _VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _VP]
        L.gr4ad_op_quantize_rows.restype = C.c_int
        L.gr4ad_op_quantize_rows.argtypes = [_VP, _VP, _VP, C.c_int32, C.c_int32, _VP]
        L.gr4ad_op_linear_fp8.restype = C.c_int
        L.gr4ad_op_linear_fp8.argtypes = [_VP, _VP, _VP, C.c_float, _VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _VP]
        L.gr4ad_op_select_workspace_bytes.restype = C.c_size_t
        L.gr4ad_op_select_workspace_bytes.argtypes = [C.c_int32] * 4
        L.gr4ad_op_select.restype = C.c_int
        L.gr4ad_op_select.argtypes = [_VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _VP, C.c_size_t, _VP, _VP, _VP, _VP]
        L.gr4ad_op_select_f16.restype = C.c_int
        L.gr4ad_op_select_f16.argtypes = L.gr4ad_op_select.argtypes
        L.gr4ad_op_select_static.restype = C.c_int
        L.gr4ad_op_select_static.argtypes = [_VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _VP, _VP, _VP, _VP]
        L.gr4ad_op_cross_attention.restype = C.c_int
        L.gr4ad_op_cross_attention.argtypes = [C.c_int, _VP, _VP, _VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _VP,
                                               C.c_size_t, _VP]
        L.gr4ad_op_context_attention.restype = C.c_int
        L.gr4ad_op_context_attention.argtypes = [C.c_int, _VP, _VP, _VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float, _VP]
        L.gr4ad_op_cross_attention_workspace_bytes.restype = C.c_size_t
        L.gr4ad_op_cross_attention_workspace_bytes.argtypes = [C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.gr4ad_op_gather_rows.restype = C.c_int
        L.gr4ad_op_gather_rows.argtypes = [C.c_int, _VP, _VP, _VP, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64, _VP]
        L.gr4ad_profile_enable.restype = C.c_int
        L.gr4ad_profile_enable.argtypes = [C.c_int]
        L.gr4ad_profile_kernel_count.restype = C.c_int
        L.gr4ad_profile_kernel_name.restype = C.c_char_p
        L.gr4ad_profile_kernel_name.argtypes = [C.c_int]
        L.gr4ad_profile_read.restype = C.c_int
        L.gr4ad_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int]
        _I64P, _U64P = C.POINTER(C.c_int64), C.POINTER(C.c_uint64)
        L.gr4ad_tabs_create.restype = C.c_int
        L.gr4ad_tabs_create.argtypes = [C.POINTER(TabsConfig), C.POINTER(_VP)]
        L.gr4ad_tabs_free.restype = None
        L.gr4ad_tabs_free.argtypes = [_VP]
        L.gr4ad_tabs_observe.restype = C.c_int
        L.gr4ad_tabs_observe.argtypes = [_VP, C.c_double, C.c_int32]
        L.gr4ad_tabs_qps.restype = C.c_double
        L.gr4ad_tabs_qps.argtypes = [_VP]
        L.gr4ad_tabs_schedule.restype = C.c_int
        L.gr4ad_tabs_schedule.argtypes = [_VP, C.c_double, C.c_double, _IP, C.POINTER(C.c_double)]
        L.gr4ad_cache_create.restype = C.c_int
        L.gr4ad_cache_create.argtypes = [C.c_int64, C.c_double, C.c_int32, C.c_int32, C.POINTER(_VP)]
        L.gr4ad_cache_free.restype = None
        L.gr4ad_cache_free.argtypes = [_VP]
        L.gr4ad_cache_insert.restype = C.c_int
        L.gr4ad_cache_insert.argtypes = [_VP, C.c_uint64, C.c_double, _IP, C.POINTER(C.c_float), C.c_int32]
        L.gr4ad_cache_lookup.restype = C.c_int
        L.gr4ad_cache_lookup.argtypes = [_VP, C.c_uint64, C.c_double, _IP, C.POINTER(C.c_float), _IP]
        L.gr4ad_cache_lookup_batch.restype = C.c_int
        L.gr4ad_cache_lookup_batch.argtypes = [_VP, _U64P, C.c_int32, C.c_double, C.POINTER(C.c_uint8), _IP, _IP]
        L.gr4ad_cache_stats.restype = C.c_int
        L.gr4ad_cache_stats.argtypes = [_VP, _I64P, _I64P, _I64P, _I64P, _I64P]
        _lib = L
    return _lib


def profile_enable(on):
    _check(lib().gr4ad_profile_enable(int(on)))


def profile_read(reset=True):
    """{kernel name: {"ms", "flops", "bytes", "launches"}} of the launches recorded since the last reset."""
    L = lib()
    n = L.gr4ad_profile_kernel_count()
    ms, fl, by, cnt = (C.c_double * n)(), (C.c_double * n)(), (C.c_double * n)(), (C.c_int64 * n)()
    _check(L.gr4ad_profile_read(ms, fl, by, cnt, int(reset)))
    return {L.gr4ad_profile_kernel_name(i).decode(): {"ms": ms[i], "flops": fl[i], "bytes": by[i], "launches": cnt[i]}
            for i in range(n) if cnt[i]}


def _check(status, dec=None):
    if status != 0:
        L = lib()
        msg = L.gr4ad_last_error(dec).decode() or L.gr4ad_strerror(status).decode()
        raise Gr4adError(status, msg)


def _i32arr(values):
    a = np.ascontiguousarray(values, dtype=np.int32)
    return a, a.ctypes.data_as(_IP)


def torch_dtype(dtype):
    return torch.bfloat16 if dtype in (BF16, "bf16") else torch.float32


def dtype_code(dtype):
    return BF16 if dtype in (BF16, "bf16", torch.bfloat16) else F32


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def weights_to_device(weights, dtype, device="cuda"):
    """numpy float32 weight dict (see synth.make_weights) -> same dict of device tensors in the storage dtype."""
    td = torch_dtype(dtype)

    def dev(a, t=td):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=t).contiguous()

    out = {k: dev(weights[k]) for k in ("pos", "bos", "w_g", "w_f", "ln_out")}
    out["emb"] = [dev(a) for a in weights["emb"]]
    out["cls"] = [dev(a) for a in weights["cls"]]
    out["layers"] = [{n: dev(lw[n]) for n in LAYER_FIELDS} for lw in weights["layers"]]
    cb = weights.get("cls_bias")
    out["cls_bias"] = None if cb is None else [None if b is None else dev(b, torch.float32) for b in cb]
    if weights.get("value_cls") is not None:  # eCPM-token step
        for k in ("value_pos", "value_emb", "value_cls"):
            out[k] = dev(weights[k])
        vb = weights.get("value_bias")
        out["value_bias"] = None if vb is None else dev(vb, torch.float32)
    return out


class Decoder:
    """gr4ad_decode_init / gr4ad_decode_batch / gr4ad_decode_free."""

    def __init__(self, d, H, F, L, K, T, V, dev_weights, dtype, max_beam, max_batch, max_ctx, eps=1e-6, Ve=0, fp8=False, vanilla=False):
        self.L_ = lib()
        self.handle = None
        self.T, self.V, self.d, self.dtype, self.Ve = T, list(V), d, dtype_code(dtype), int(Ve)
        V_arr, V_ptr = _i32arr(self.V)
        mb_arr, mb_ptr = _i32arr(max_beam)
        desc = ModelDesc(d, H, F, L, K, T, V_ptr, mb_ptr, max_batch, max_ctx, self.dtype, eps, self.Ve, int(bool(fp8)), int(bool(vanilla)))
        w = dev_weights
        ptr = lambda t: C.c_void_p(t.data_ptr())
        emb = (_VP * max(T - 1, 1))(*[t.data_ptr() for t in w["emb"]])
        cls = (_VP * T)(*[t.data_ptr() for t in w["cls"]])
        bias = None
        if w.get("cls_bias") is not None:
            bias = (_VP * T)(*[(b.data_ptr() if b is not None else None) for b in w["cls_bias"]])
        layers = (LayerWeights * L)(*[LayerWeights(*[lw[n].data_ptr() for n in LAYER_FIELDS]) for lw in w["layers"]])
        ws = Weights(ptr(w["pos"]), ptr(w["bos"]), emb, None if vanilla else ptr(w["w_g"]), None if vanilla else ptr(w["w_f"]), layers,
                     ptr(w["ln_out"]), cls,
                     bias if bias is not None else C.POINTER(_VP)(),
                     *[(w[k].data_ptr() if w.get(k) is not None else None) for k in ("value_pos", "value_emb", "value_cls", "value_bias")])
        h = _VP()
        _check(self.L_.gr4ad_decode_init(C.byref(desc), C.byref(ws), C.byref(h)))
        self.handle = h
        self._trace = None
        self._ws = None

    def close(self):
        if getattr(self, "handle", None):
            self.L_.gr4ad_decode_free(self.handle)
            self.handle = None

    __del__ = close

    def workspace_bytes(self, B, S, beam):
        _, bp = _i32arr(beam)
        return int(self.L_.gr4ad_decode_workspace_bytes(self.handle, B, S, bp))

    def enable_trace(self, B, beam, device="cuda"):
        """Allocates per-level survivor buffers and registers them; returns the dict of tensors."""
        tr = {"parent": [torch.zeros(B, b, dtype=torch.int32, device=device) for b in beam],
              "tok": [torch.zeros(B, b, dtype=torch.int32, device=device) for b in beam],
              "score": [torch.zeros(B, b, dtype=torch.float32, device=device) for b in beam]}
        arrs = [(_VP * self.T)(*[t.data_ptr() for t in tr[k]]) for k in ("parent", "tok", "score")]
        _check(self.L_.gr4ad_decode_set_trace(self.handle, *arrs), self.handle)
        self._trace = tr
        return tr

    def disable_trace(self):
        _check(self.L_.gr4ad_decode_set_trace(self.handle, None, None, None), self.handle)
        self._trace = None

    def decode_batch(self, ctx, ctx_len, beam, workspace=None, out_sid=None, out_logprob=None, stream=None, value=False, out_value=None):
        """ctx [B,S,d] device tensor of the storage dtype; ctx_len [B] int32 device tensor or None.
        Returns (sid [B,b_T,T] int32, logprob [B,b_T] float32) device tensors; asynchronous on the stream.
        value=True (model with an eCPM-token step): also runs that step and returns, third, the
        log-probabilities of the value buckets [B,b_T,V_e] float32 (gr4ad_decode_set_value_output)."""
        B, S, d = ctx.shape
        assert d == self.d and ctx.is_contiguous() and ctx.dtype == torch_dtype(self.dtype)
        beam_arr, beam_ptr = _i32arr(beam)
        need = int(self.L_.gr4ad_decode_workspace_bytes(self.handle, B, S, beam_ptr))
        if workspace is None:
            if self._ws is None or self._ws.numel() < need:
                self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=ctx.device)
            workspace = self._ws
        bT = int(beam_arr[-1])
        if out_sid is None:
            out_sid = torch.empty(B, bT, self.T, dtype=torch.int32, device=ctx.device)
        if out_logprob is None:
            out_logprob = torch.empty(B, bT, dtype=torch.float32, device=ctx.device)
        if value or self.Ve > 0:
            if value and out_value is None:
                out_value = torch.empty(B, bT, self.Ve, dtype=torch.float32, device=ctx.device)
            if value:
                assert out_value.is_contiguous() and out_value.dtype == torch.float32 and out_value.numel() == B * bT * self.Ve
            _check(self.L_.gr4ad_decode_set_value_output(self.handle, C.c_void_p(out_value.data_ptr()) if value else None), self.handle)
        cl = None if ctx_len is None else C.c_void_p(ctx_len.data_ptr())
        st = self.L_.gr4ad_decode_batch(self.handle, C.c_void_p(ctx.data_ptr()), cl, B, S, beam_ptr, C.c_void_p(workspace.data_ptr()),
                                        workspace.numel(), C.c_void_p(out_sid.data_ptr()), C.c_void_p(out_logprob.data_ptr()),
                                        _stream_ptr(stream))
        _check(st, self.handle)
        if value:
            return out_sid, out_logprob, out_value
        return out_sid, out_logprob


def decoder_for(workload, weights, max_beam=None, device="cuda"):
    """Decoder for a synth.Workload and its numpy weight dict."""
    w = workload
    dev_w = weights_to_device(weights, w.dtype, device)
    dec = Decoder(w.d, w.H, w.F, w.L, w.K, w.T, w.V, dev_w, w.dtype, max_beam or list(w.beam), w.B, w.S, eps=w.eps, Ve=w.Ve, fp8=w.fp8, vanilla=w.vanilla)
    dec._keep = dev_w  # init copies the weights; kept only so callers may inspect them
    return dec


# ---- single-operation entry points ----------------------------------------------
def op_linear(A, W, bias=None, out_f32=False, stream=None):
    M, K = A.shape
    N = W.shape[0]
    dt = dtype_code(A.dtype)
    Cout = torch.empty(M, N, dtype=torch.float32 if out_f32 else A.dtype, device=A.device)
    _check(lib().gr4ad_op_linear(dt, A.data_ptr(), W.data_ptr(), None if bias is None else bias.data_ptr(), Cout.data_ptr(), M, N, K,
                                 int(out_f32), _stream_ptr(stream)))
    return Cout


def op_quantize_rows(x, stream=None):
    """x [rows, n] bf16 -> (q [rows, n] uint8 holding E4M3 bytes, scale [rows] float32)."""
    rows, n = x.shape
    q = torch.empty(rows, n, dtype=torch.uint8, device=x.device)
    scale = torch.empty(rows, dtype=torch.float32, device=x.device)
    _check(lib().gr4ad_op_quantize_rows(x.data_ptr(), q.data_ptr(), scale.data_ptr(), rows, n, _stream_ptr(stream)))
    return q, scale


def op_linear_fp8(Aq, a_scale, Wq, w_scale, bias=None, out_f32=False, stream=None):
    M, K = Aq.shape
    N = Wq.shape[0]
    Cout = torch.empty(M, N, dtype=torch.float32 if out_f32 else torch.bfloat16, device=Aq.device)
    _check(lib().gr4ad_op_linear_fp8(Aq.data_ptr(), a_scale.data_ptr(), Wq.data_ptr(), float(w_scale), None if bias is None else bias.data_ptr(),
                                     Cout.data_ptr(), M, N, K, int(out_f32), _stream_ptr(stream)))
    return Cout


def op_select(logits, cum, k, stream=None):
    """gr4ad_op_select (float32 logits) or gr4ad_op_select_f16 (float16 logits), by the tensor's dtype."""
    B, n, V = logits.shape
    L = lib()
    if logits.dtype not in (torch.float32, torch.float16):
        raise TypeError("op_select takes float32 or float16 logits, got %s" % logits.dtype)
    entry = L.gr4ad_op_select_f16 if logits.dtype == torch.float16 else L.gr4ad_op_select
    nbytes = int(L.gr4ad_op_select_workspace_bytes(B, n, V, k))
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=logits.device)
    parent = torch.empty(B, k, dtype=torch.int32, device=logits.device)
    tok = torch.empty_like(parent)
    score = torch.empty(B, k, dtype=torch.float32, device=logits.device)
    _check(entry(logits.data_ptr(), None if cum is None else cum.data_ptr(), B, n, V, k, ws.data_ptr(), ws.numel(),
                             parent.data_ptr(), tok.data_ptr(), score.data_ptr(), _stream_ptr(stream)))
    return parent, tok, score


SELECT_STATIC_BYTES = 32 << 20


def op_select_static(logits, cum, k, parent, tok, score, stream=None):
    """gr4ad_op_select_static: the selection without a workspace (static scratch inside the library).  The caller
    passes the outputs parent, tok [B,k] int32 and score [B,k] float32: the call itself allocates nothing."""
    B, n, V = logits.shape
    _check(lib().gr4ad_op_select_static(logits.data_ptr(), None if cum is None else cum.data_ptr(), B, n, V, k, parent.data_ptr(),
                                        tok.data_ptr(), score.data_ptr(), _stream_ptr(stream)))
    return parent, tok, score


def op_cross_attention(q, kv, ctx_len, H, stream=None):
    B, n, d = q.shape
    S = kv.shape[1]
    out = torch.empty_like(q)
    nbytes = int(lib().gr4ad_op_cross_attention_workspace_bytes(dtype_code(q.dtype), B, S, d, H))
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=q.device)
    _check(lib().gr4ad_op_cross_attention(dtype_code(q.dtype), q.data_ptr(), kv.data_ptr(), None if ctx_len is None else ctx_len.data_ptr(),
                                          out.data_ptr(), B, n, S, d, H, ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return out


def op_context_attention(q, x, ctx_len, scale, stream=None):
    """gr4ad_op_context_attention: q, out [B,RQ,d], x [B,S,d] (bf16): attention over the raw context rows as keys and values."""
    B, RQ, d = q.shape
    out = torch.empty_like(q)
    _check(lib().gr4ad_op_context_attention(dtype_code(q.dtype), q.data_ptr(), x.data_ptr(), None if ctx_len is None else ctx_len.data_ptr(),
                                            out.data_ptr(), B, RQ, x.shape[1], d, float(scale), _stream_ptr(stream)))
    return out


def op_gather_rows(src, parent, k=None, row_elems=None, stream=None):
    B, n = src.shape[0], src.shape[1]
    stride = int(np.prod(src.shape[2:]))
    k = parent.shape[1] if k is None else k
    dst = torch.zeros((B, k) + tuple(src.shape[2:]), dtype=src.dtype, device=src.device)
    _check(lib().gr4ad_op_gather_rows(dtype_code(src.dtype), src.data_ptr(), parent.data_ptr(), dst.data_ptr(), B, n, k,
                                      stride if row_elems is None else row_elems, stride, _stream_ptr(stream)))
    return dst


# ---- host-side serving policies (include/gr4ad_serving.h) ------------------------------
class TabsController:
    """gr4ad_tabs_*: the beam schedule of a call from the traffic (Traffic-Aware Adaptive Beam Search)."""

    def __init__(self, beam_base, max_beam, codebook, qps_peak, scale_min=1.0, scale_max=1.6, step=0.1, tau_s=10.0):
        self.L_ = lib()
        self.T = len(beam_base)
        arrs = [_i32arr(a) for a in (beam_base, max_beam, codebook)]
        cfg = TabsConfig(self.T, arrs[0][1], arrs[1][1], arrs[2][1], qps_peak, scale_min, scale_max, step, tau_s)
        h = _VP()
        _check(self.L_.gr4ad_tabs_create(C.byref(cfg), C.byref(h)))
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            self.L_.gr4ad_tabs_free(self.handle)
            self.handle = None

    __del__ = close

    def observe(self, t_s, n_requests):
        _check(self.L_.gr4ad_tabs_observe(self.handle, t_s, n_requests))

    def qps(self):
        return float(self.L_.gr4ad_tabs_qps(self.handle))

    def schedule(self, t_s, c_avail=1.0):
        beam = (C.c_int32 * self.T)()
        scale = C.c_double()
        _check(self.L_.gr4ad_tabs_schedule(self.handle, t_s, c_avail, beam, C.byref(scale)))
        return list(beam), scale.value


class ResultCache:
    """gr4ad_cache_*: per-user results reused inside a time window (Reco Result Cache)."""

    def __init__(self, capacity, ttl_s, n_levels, max_items):
        self.L_ = lib()
        self.T, self.max_items = n_levels, max_items
        h = _VP()
        _check(self.L_.gr4ad_cache_create(capacity, ttl_s, n_levels, max_items, C.byref(h)))
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            self.L_.gr4ad_cache_free(self.handle)
            self.handle = None

    __del__ = close

    def insert(self, key, now_s, sid, logprob):
        sid = np.ascontiguousarray(sid, dtype=np.int32)
        logprob = np.ascontiguousarray(logprob, dtype=np.float32)
        _check(self.L_.gr4ad_cache_insert(self.handle, key, now_s, sid.ctypes.data_as(_IP), logprob.ctypes.data_as(C.POINTER(C.c_float)),
                                          logprob.shape[0]))

    def lookup(self, key, now_s):
        """(sid [n,T], logprob [n]) or None."""
        sid = np.empty((self.max_items, self.T), np.int32)
        lp = np.empty(self.max_items, np.float32)
        n = C.c_int32()
        r = self.L_.gr4ad_cache_lookup(self.handle, key, now_s, sid.ctypes.data_as(_IP), lp.ctypes.data_as(C.POINTER(C.c_float)), C.byref(n))
        if r < 0:
            _check(r)
        return (sid[:n.value], lp[:n.value]) if r == 1 else None

    def lookup_batch(self, keys, now_s):
        """(hit [B] uint8, indices of the requests to decode)."""
        keys = np.ascontiguousarray(keys, dtype=np.uint64)
        B = keys.shape[0]
        hit = np.empty(B, np.uint8)
        miss = np.empty(B, np.int32)
        n = C.c_int32()
        _check(self.L_.gr4ad_cache_lookup_batch(self.handle, keys.ctypes.data_as(C.POINTER(C.c_uint64)), B, now_s,
                                                hit.ctypes.data_as(C.POINTER(C.c_uint8)), miss.ctypes.data_as(_IP), C.byref(n)))
        return hit, miss[:n.value].copy()

    def stats(self):
        v = [C.c_int64() for _ in range(5)]
        _check(self.L_.gr4ad_cache_stats(self.handle, *[C.byref(x) for x in v]))
        return dict(zip(("lookups", "hits", "entries", "evictions", "expired"), (x.value for x in v)))
