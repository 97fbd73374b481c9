"""ctypes front end of the CPU oracle (test infrastructure, not the product).

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this package.  It imports nothing from the HIP path.  Weights are plain
dicts of float32 numpy arrays:

    pos [T,d], bos [d], emb: list of T-1 arrays [V_t,d], w_g [d,d], w_f [d,2d],
    layers: list of L dicts {ln_x,wq_x,wk_x,wv_x,wo_x,ln_s,wq_s,wk_s,wv_s,wo_s,ln_f,w1,w2},
    ln_out [d], cls: list of T arrays [V_t,d], cls_bias: None or list of (array [V_t] | None)
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LAYER_FIELDS = ["ln_x", "wq_x", "wk_x", "wv_x", "wo_x", "ln_s", "wq_s", "wk_s", "wv_s", "wo_s", "ln_f", "w1", "w2"]
_FP = C.POINTER(C.c_float)
_DP = C.POINTER(C.c_double)
_IP = C.POINTER(C.c_int32)
_LP = C.POINTER(C.c_int64)


class _Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "H", "F", "L", "K", "T")] + [("V", _IP), ("eps", C.c_float), ("fp8", C.c_int32), ("vanilla", C.c_int32)]


class _Layer(C.Structure):
    _fields_ = [(n, _FP) for n in _LAYER_FIELDS]


class _Weights(C.Structure):
    _fields_ = [("pos", _FP), ("bos", _FP), ("emb", C.POINTER(_FP)), ("w_g", _FP), ("w_f", _FP),
                ("layers", C.POINTER(_Layer)), ("ln_out", _FP), ("cls", C.POINTER(_FP)), ("cls_bias", C.POINTER(_FP))]


_libs = {}


def build():
    from . import build_oracle
    build_oracle.build()


def _lib(precision):
    if precision not in _libs:
        path = os.path.join(_HERE, {"f64": "liborc_f64.so", "f32": "liborc_f32.so"}[precision])
        if not os.path.exists(path):
            build()
        lib = C.CDLL(path)
        lib.orc_model_create.restype = C.c_void_p
        lib.orc_model_create.argtypes = [C.POINTER(_Desc), C.POINTER(_Weights)]
        lib.orc_model_free.argtypes = [C.c_void_p]
        lib.orc_req_create.restype = C.c_void_p
        lib.orc_req_create.argtypes = [C.c_void_p, _FP, C.c_int]
        lib.orc_req_free.argtypes = [C.c_void_p]
        lib.orc_forward_seq.argtypes = [C.c_void_p, C.c_void_p, C.c_int, _IP, _DP, _DP]
        lib.orc_plain_ar_seq.argtypes = [C.c_void_p, C.c_void_p, C.c_int, _IP, _DP]
        lib.orc_vanilla_ar_seq.argtypes = [C.c_void_p, C.c_void_p, C.c_int, _IP, _DP]
        lib.orc_decode_batch.restype = C.c_int
        lib.orc_decode_batch.argtypes = [C.c_void_p, _FP, _IP, C.c_int, C.c_int, _IP, _IP, _DP, _IP, _IP, _DP, C.c_int]
        lib.orc_prefix_dists.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, _IP, _DP, _DP]
        lib.orc_prim_linear.argtypes = [_DP, _DP, _DP, C.c_int, C.c_int, C.c_int]
        lib.orc_prim_rmsnorm.argtypes = [_DP, _DP, _DP, C.c_int, C.c_int, C.c_double]
        lib.orc_prim_silu.argtypes = [_DP, _DP, C.c_int]
        lib.orc_prim_log_softmax.argtypes = [_DP, _DP, C.c_int]
        lib.orc_prim_mha.argtypes = [_DP, _DP, _DP, _DP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
        lib.orc_prim_fuse.argtypes = [_DP, _DP, _DP, _DP, _DP, C.c_int]
        lib.orc_prim_topk.argtypes = [_DP, C.c_int, C.c_int, C.c_int, _LP, _DP, C.c_int]
        lib.orc_prim_layer_seq.argtypes = [C.c_void_p, C.c_void_p, C.c_int, _DP, C.c_int]
        lib.orc_prim_e4m3.argtypes = [_DP, _DP, C.c_int]
        lib.orc_prim_quant_rows.argtypes = [_DP, _DP, C.c_int, C.c_int]
        lib.orc_real_bytes.restype = C.c_int
        _libs[precision] = lib
    return _libs[precision]


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a, t):
    return a.ctypes.data_as(t)


MODE_CACHED, MODE_PLAIN, MODE_PLAIN_PRECUT = 0, 1, 2


class Oracle:
    """One model (shapes + weights) loaded into the oracle."""

    def __init__(self, d, H, F, L, K, T, V, weights, eps=1e-6, precision="f64", fp8=False, vanilla=False):
        self.lib = _lib(precision)
        self.d, self.H, self.F, self.L, self.K, self.T, self.V, self.eps = d, H, F, L, K, T, list(V), eps
        keep = []  # keeps the float32 copies alive during orc_model_create

        def fp(a):
            a = _f32(a)
            keep.append(a)
            return _p(a, _FP)

        w = weights
        Varr = _i32(self.V)
        desc = _Desc(d, H, F, L, K, T, _p(Varr, _IP), eps, int(bool(fp8)), int(bool(vanilla)))
        emb = (_FP * max(T - 1, 1))(*[fp(e) for e in w["emb"]]) if T > 1 else (_FP * 1)()
        cls = (_FP * T)(*[fp(c) for c in w["cls"]])
        cb = w.get("cls_bias")
        bias = None
        if cb is not None:
            bias = (_FP * T)(*[(fp(b) if b is not None else _FP()) for b in cb])
        layers = (_Layer * L)(*[_Layer(*[fp(lw[n]) for n in _LAYER_FIELDS]) for lw in w["layers"]])
        ws = _Weights(fp(w["pos"]), fp(w["bos"]), emb, None if vanilla else fp(w["w_g"]), None if vanilla else fp(w["w_f"]), layers,
                      fp(w["ln_out"]), cls,
                      bias if bias is not None else C.POINTER(_FP)())
        self.h = self.lib.orc_model_create(C.byref(desc), C.byref(ws))
        if not self.h:
            raise ValueError("orc_model_create rejected the model description")

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.orc_model_free(self.h)
            self.h = None

    # ---- per-request handle -------------------------------------------------
    def request(self, X, length=None):
        X = _f32(X)
        assert X.ndim == 2 and X.shape[1] == self.d
        return _Request(self, X, X.shape[0] if length is None else int(length))

    # ---- batch decode -------------------------------------------------------
    def decode_batch(self, X, ctx_len, beam, mode=MODE_CACHED):
        """X [B,S,d]; ctx_len [B] or None.  Returns sid [B,bT,T] int32, logprob
        [B,bT] float64 and the per-level trace dict {parent,tok,score}: lists of
        T arrays [B,b_t]."""
        X = _f32(X)
        B, S, d = X.shape
        assert d == self.d
        beam = _i32(beam)
        assert beam.shape == (self.T,)
        bT, tot = int(beam[-1]), int(beam.sum())
        sid = np.zeros((B, bT, self.T), np.int32)
        lp = np.zeros((B, bT), np.float64)
        tp, tt, ts = np.zeros((B, tot), np.int32), np.zeros((B, tot), np.int32), np.zeros((B, tot), np.float64)
        cl = _i32(ctx_len) if ctx_len is not None else None
        rc = self.lib.orc_decode_batch(self.h, _p(X, _FP), _p(cl, _IP) if cl is not None else None, B, S, _p(beam, _IP),
                                       _p(sid, _IP), _p(lp, _DP), _p(tp, _IP), _p(tt, _IP), _p(ts, _DP), mode)
        if rc:
            raise ValueError("oracle rejected the beam schedule")
        off = np.concatenate([[0], np.cumsum(beam)])
        trace = {"parent": [tp[:, off[t]:off[t + 1]] for t in range(self.T)],
                 "tok": [tt[:, off[t]:off[t + 1]] for t in range(self.T)],
                 "score": [ts[:, off[t]:off[t + 1]] for t in range(self.T)]}
        return sid, lp, trace


class _Request:
    def __init__(self, orc, X, length):
        self.orc, self.lib = orc, orc.lib
        self.h = self.lib.orc_req_create(orc.h, _p(X, _FP), length)
        if not self.h:
            raise ValueError("orc_req_create failed")

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.orc_req_free(self.h)
            self.h = None

    def forward_seq(self, tokens):
        """tokens s_1..s_{t-1} -> list of t log-prob distributions (levels 1..t)."""
        o = self.orc
        tokens = _i32(tokens)
        t = len(tokens) + 1
        sizes = o.V[:t]
        last = np.zeros(sizes[-1])
        buf = np.zeros(sum(sizes))
        self.lib.orc_forward_seq(o.h, self.h, t, _p(tokens, _IP), _p(last, _DP), _p(buf, _DP))
        off = np.concatenate([[0], np.cumsum(sizes)])
        out = [buf[off[i]:off[i + 1]].copy() for i in range(t)]
        assert np.array_equal(out[-1], last)
        return out

    def plain_ar_seq(self, tokens):
        o = self.orc
        tokens = _i32(tokens)
        t = len(tokens) + 1
        last = np.zeros(o.V[t - 1])
        self.lib.orc_plain_ar_seq(o.h, self.h, t, _p(tokens, _IP), _p(last, _DP))
        return last

    def vanilla_ar_seq(self, tokens):
        """Level-t distribution of the separately written vanilla decoder (input s_{t-1} + p_t, L layers)."""
        o = self.orc
        tokens = _i32(tokens)
        t = len(tokens) + 1
        last = np.zeros(o.V[t - 1])
        self.lib.orc_vanilla_ar_seq(o.h, self.h, t, _p(tokens, _IP), _p(last, _DP))
        return last

    def prefix_dists(self, t, prefixes):
        """prefixes [n, t-1] -> (cum [n], lp [n, V_t]) for 1-based level t."""
        o = self.orc
        prefixes = _i32(prefixes).reshape(-1, t - 1) if t > 1 else np.zeros((len(prefixes), 0), np.int32)
        n = prefixes.shape[0]
        cum, lp = np.zeros(n), np.zeros((n, o.V[t - 1]))
        self.lib.orc_prefix_dists(o.h, self.h, t, n, _p(prefixes, _IP), _p(cum, _DP), _p(lp, _DP))
        return cum, lp

    def layer_seq(self, layer, x):
        x = _f64(x).copy()
        self.lib.orc_prim_layer_seq(self.orc.h, self.h, layer, _p(x, _DP), x.shape[0])
        return x


# ---- primitives (double in / double out) -------------------------------------
def prim_linear(x, W, precision="f64"):
    x, W = _f64(x), _f64(W)
    y = np.zeros((x.shape[0], W.shape[0]))
    _lib(precision).orc_prim_linear(_p(y, _DP), _p(x, _DP), _p(W, _DP), x.shape[0], x.shape[1], W.shape[0])
    return y


def prim_rmsnorm(x, g, eps, precision="f64"):
    x, g = _f64(x), _f64(g)
    y = np.zeros_like(x)
    _lib(precision).orc_prim_rmsnorm(_p(y, _DP), _p(x, _DP), _p(g, _DP), x.shape[0], x.shape[1], eps)
    return y


def prim_silu(x, precision="f64"):
    x = _f64(x)
    y = np.zeros_like(x)
    _lib(precision).orc_prim_silu(_p(y, _DP), _p(x, _DP), x.size)
    return y


def prim_log_softmax(z, precision="f64"):
    z = _f64(z)
    y = np.zeros_like(z)
    _lib(precision).orc_prim_log_softmax(_p(y, _DP), _p(z, _DP), z.size)
    return y


def prim_mha(q, k, v, H, causal, precision="f64"):
    q, k, v = _f64(q), _f64(k), _f64(v)
    o = np.zeros_like(q)
    _lib(precision).orc_prim_mha(_p(o, _DP), _p(q, _DP), _p(k, _DP), _p(v, _DP), q.shape[0], k.shape[0], q.shape[1], H, int(causal))
    return o


def prim_fuse(m, s, w_g, w_f, precision="f64"):
    m, s, w_g, w_f = _f64(m), _f64(s), _f64(w_g), _f64(w_f)
    o = np.zeros_like(m)
    _lib(precision).orc_prim_fuse(_p(o, _DP), _p(m, _DP), _p(s, _DP), _p(w_g, _DP), _p(w_f, _DP), m.size)
    return o


def prim_topk(score, k, precut=False, precision="f64"):
    score = _f64(score)
    n, V = score.shape
    flat, ks = np.zeros(k, np.int64), np.zeros(k)
    _lib(precision).orc_prim_topk(_p(score, _DP), n, V, k, _p(flat, _LP), _p(ks, _DP), int(precut))
    return flat, ks


def prim_e4m3(x, precision="f64"):
    """Nearest value of the OCP E4M3 grid (saturating at 448), element by element."""
    x = _f64(x)
    y = np.zeros_like(x)
    _lib(precision).orc_prim_e4m3(_p(y, _DP), _p(x, _DP), x.size)
    return y


def prim_quant_rows(x, precision="f64"):
    """Rows as FP8 operands: scale amax(row)/448, E4M3 rounding, scaled back."""
    x = _f64(x)
    y = np.zeros_like(x)
    _lib(precision).orc_prim_quant_rows(_p(y, _DP), _p(x, _DP), x.shape[0], x.shape[1])
    return y
