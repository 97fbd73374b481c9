// Host side of libgr4ad.so: the C ABI, weight packing, workspace plan and the
// per-level decode loop (section 3.2 LazyAR decoder under the beam search of
// section 4.2).  All device work is enqueued on the caller's stream.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "common.h"

namespace {

struct LayerPacked {
    void *ln_x, *wq_x, *wkv_x, *wo_x;   // wkv_x [2d,d]: rows of W_k then W_v (context projection)
    void *ln_s, *wqkv_s, *wo_s;         // wqkv_s [3d,d]
    void *ln_f, *w1, *w2;
    void *wkT_x;  // lazy layers in absorbed form only: [H][d][dh], the key projection transposed per head
    // FP8 mode, autoregressive layers only: E4M3 copies of the per-row projections, one scale per matrix
    void *wq_x8, *wo_x8, *wqkv_s8, *wo_s8, *w1_8, *w2_8;
    float s_wq_x, s_wo_x, s_wqkv_s, s_wo_s, s_w1, s_w2;
};

thread_local char g_init_error[512] = "";

}  // namespace

struct gr4ad_decoder {
    int d, H, F, L, K, T, A;
    int Ve, Tp;  // value step: eCPM buckets (0 = none); Tp = T + (Ve > 0): positions the trunk computes, levels with tables
    float *value_out;  // [B, b_T, Ve] log-probabilities of the value step, NULL = step off
    int V[GR4AD_MAX_LEVELS], max_beam[GR4AD_MAX_LEVELS];
    int max_batch, max_ctx;
    gr4ad_dtype dtype;
    size_t esz;
    float eps;
    int device;
    void *pos, *ln_out, *wf1;
    void *G[GR4AD_MAX_LEVELS], *P[GR4AD_MAX_LEVELS];  // per-level Fuse tables: W_g s and W_f[:,d:] s of the previous token
    bool vanilla;                 // vanilla autoregressive decoder: input state s_{t-1} + p_t, no Fuse, no lazy layer
    void *E[GR4AD_MAX_LEVELS];    // vanilla only: per-level embedding table of the previous token (one BOS row at level 1)
    void *cls[GR4AD_MAX_LEVELS];
    float *cls_bias[GR4AD_MAX_LEVELS];
    std::vector<LayerPacked> layers;
    std::vector<void *> allocs;
    int32_t *tr_parent[GR4AD_MAX_LEVELS], *tr_tok[GR4AD_MAX_LEVELS];
    float *tr_score[GR4AD_MAX_LEVELS];
    bool trace;
    bool absorbed;  // lazy layers' cross-attention runs in absorbed form (see decode_batch)
    bool fp8;       // FP8 mode: the per-beam-row products take E4M3 operands (see decode_batch)
    void *wf1_8, *cls8[GR4AD_MAX_LEVELS];
    float s_wf1, s_cls[GR4AD_MAX_LEVELS];
    char err[512];
};

namespace {

int fail(gr4ad_decoder *dec, int code, const char *fmt, ...) {
    char *buf = dec ? dec->err : g_init_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, 512, fmt, ap);
    va_end(ap);
    return code;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Everything decode_batch carves out of the caller's workspace.
struct Plan {
    size_t aq, ascale;  // FP8 mode: the quantised operand of the next product [rows_max, max(d, F)] bytes and its row scales
    size_t kv_ar, kv_lazy, vt_ar, vt_lazy, vt_bytes, xt, qp, zb, sc, pb, ss, trunk, h, xn, q, o, qkv, f, logits, selws, qkv_lvl[GR4AD_MAX_LEVELS], cum[2], par, tok[2], sid[2], anc[2], total;
    int64_t rows_max, nmax, bmax;
    size_t qkv_lvl_layer_bytes[GR4AD_MAX_LEVELS];  // one layer's [B*n_t, 3d] buffer of level t
};

bool beams_ok(const gr4ad_decoder *dec, const int32_t *beam) {
    int64_t n = 1;
    for (int t = 0; t < dec->T; t++) {
        if (beam[t] < 1 || beam[t] > dec->max_beam[t] || (int64_t)beam[t] > n * dec->V[t]) return false;
        n = beam[t];
    }
    return true;
}

GemmEpilogue plain_epilogue(void *C, int64_t ldc);

// Level t (0-based) with `rows` beam rows: does the classifier leave its logits in half precision for the selection?  It does
// where the persistent GEMM runs the classifier (it alone has that epilogue) and the wavefront selection kernel takes the
// codebook size: the logits then make their round trip through HBM in 2 instead of 4 bytes.  The log-sum-exp, the scores and
// the selection stay float32; the rounding of a logit (at most 2^-11 of its magnitude) is far below what bf16 operands leave
// in it.  float32 storage, small levels and the value step (whose output IS the distribution) keep float32 logits.
bool level_logits_f16(const gr4ad_decoder *dec, int64_t rows, int t) {
    if (dec->dtype != GR4AD_BF16 || t >= dec->T || !select_takes_f16(dec->V[t])) return false;
    GemmEpilogue g = plain_epilogue((void *)4096, dec->V[t]);  // (pointers are only inspected for alignment)
    g.out_f32 = 1;
    g.out_f16 = 1;
    if (dec->fp8) return gemm_f8_on_persistent_kernel(dec->ln_out, dec->d, dec->cls8[t], dec->d, rows, dec->V[t], dec->d, g);
    return gemm_on_persistent_kernel(dec->dtype, dec->ln_out, dec->d, dec->cls[t], dec->d, rows, dec->V[t], dec->d, g);
}

Plan make_plan(const gr4ad_decoder *dec, int64_t B, int64_t S, const int32_t *beam) {
    Plan p;
    memset(&p, 0, sizeof(p));
    const size_t e = dec->esz;
    const int64_t d = dec->d, T = dec->T, Tp = dec->Tp;
    int64_t n = 1, nmax = 1, bmax = 1, logit_max = 0;  // logit_max: bytes per request
    size_t selmax = 0;
    for (int t = 0; t < T; t++) {
        if (n > nmax) nmax = n;
        if (beam[t] > bmax) bmax = beam[t];
        const int64_t lb = n * dec->V[t] * (level_logits_f16(dec, B * n, t) ? 2 : 4);
        if (lb > logit_max) logit_max = lb;
        size_t s = select_workspace_bytes((int)B, (int)n, dec->V[t], beam[t]);
        if (s > selmax) selmax = s;
        n = beam[t];
    }
    if (dec->Ve > 0) {  // the value step: one more level of n = b_T rows, no selection
        if (n > nmax) nmax = n;
        if (n * dec->Ve * 4 > logit_max) logit_max = n * dec->Ve * 4;
    }
    p.nmax = nmax;
    p.bmax = bmax;
    p.rows_max = B * (nmax > Tp ? nmax : Tp);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
    p.kv_ar = take((size_t)dec->A * B * S * 2 * d * e);
    const bool lazy_kv = dec->K > 0 && !dec->absorbed;
    p.kv_lazy = take(lazy_kv ? (size_t)B * S * 2 * d * e : 0);
    p.vt_bytes = cross_attention_workspace_bytes(dec->dtype, (int)B, (int)S, dec->d, dec->H);
    p.vt_ar = take((size_t)dec->A * p.vt_bytes);
    p.vt_lazy = take(lazy_kv ? p.vt_bytes : 0);
    if (dec->absorbed) {  // bf16 only
        const int64_t Spad = (S + 63) / 64 * 64, RQ = Tp * dec->H;
        const bool two_pass = !context_attention_covers(dec->dtype, (int)RQ, dec->d);  // (else one kernel, no transposed copy, scores or probabilities in HBM)
        p.xt = take(two_pass ? (size_t)B * d * Spad * e : 0);
        p.qp = take((size_t)B * RQ * d * e);
        p.zb = take((size_t)B * RQ * d * e);
        p.sc = take(two_pass ? (size_t)B * RQ * Spad * sizeof(float) : 0);
        p.pb = take(two_pass ? (size_t)B * RQ * Spad * e : 0);
    }
    p.ss = take((size_t)p.rows_max * (d / 64 + 1) * sizeof(float));  // partial sums of squares of the folded RMSNorm
    p.trunk = take((size_t)B * Tp * d * sizeof(float));  // residual streams stay float32 whatever the storage dtype
    p.h = take((size_t)p.rows_max * d * sizeof(float));
    p.xn = take((size_t)p.rows_max * d * e);
    p.q = take((size_t)p.rows_max * d * e);
    p.o = take((size_t)p.rows_max * d * e);
    p.qkv = take((size_t)B * Tp * 3 * d * e);  // lazy layers; the autoregressive layers keep one buffer per (level, layer), below
    p.f = take((size_t)p.rows_max * dec->F * e);
    p.logits = take((size_t)B * logit_max);
    p.aq = take(dec->fp8 ? (size_t)p.rows_max * (dec->F > d ? dec->F : d) : 0);
    p.ascale = take(dec->fp8 ? (size_t)p.rows_max * sizeof(float) : 0);
    p.selws = take(selmax);
    // q/k/v of every level stay resident: they are the self-attention cache of the later levels, read through the
    // beams' ancestor table.  No level follows the last one, so its layers share one buffer.
    n = 1;
    for (int t = 0; t < Tp; t++) {
        p.qkv_lvl_layer_bytes[t] = align256((size_t)B * n * 3 * d * e);
        p.qkv_lvl[t] = take((size_t)(t == Tp - 1 ? 1 : dec->A) * p.qkv_lvl_layer_bytes[t]);
        if (t < T) n = beam[t];
    }
    for (int i = 0; i < 2; i++) p.cum[i] = take((size_t)B * bmax * sizeof(float));
    p.par = take((size_t)B * bmax * sizeof(int32_t));
    for (int i = 0; i < 2; i++) p.tok[i] = take((size_t)B * bmax * sizeof(int32_t));
    for (int i = 0; i < 2; i++) p.sid[i] = take((size_t)B * bmax * T * sizeof(int32_t));
    for (int i = 0; i < 2; i++) p.anc[i] = take((size_t)B * bmax * T * sizeof(int32_t));
    p.total = off;
    return p;
}

#define HIP_TRY(dec, call)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) return fail(dec, GR4AD_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define OP_TRY(dec, call, what)                                                  \
    do {                                                                         \
        int s_ = (call);                                                         \
        if (s_ != GR4AD_OK) return fail(dec, s_, "%s failed: %s", what, gr4ad_strerror(s_)); \
    } while (0)

int dev_alloc(gr4ad_decoder *dec, void **out, size_t bytes) {
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, bytes ? bytes : 256);
    if (e != hipSuccess) return fail(dec, e == hipErrorOutOfMemory ? GR4AD_ENOMEM : GR4AD_EHIP, "hipMalloc(%zu): %s", bytes, hipGetErrorString(e));
    dec->allocs.push_back(p);
    *out = p;
    return GR4AD_OK;
}

int dev_clone(gr4ad_decoder *dec, void **out, const void *src, size_t bytes) {
    int s = dev_alloc(dec, out, bytes);
    if (s) return s;
    HIP_TRY(dec, hipMemcpy(*out, src, bytes, hipMemcpyDeviceToDevice));
    return GR4AD_OK;
}

// rows of several [r_i, d] matrices stacked into one [sum r_i, d] matrix
int dev_stack(gr4ad_decoder *dec, void **out, const void *const *srcs, int count, size_t bytes_each) {
    int s = dev_alloc(dec, out, bytes_each * count);
    if (s) return s;
    for (int i = 0; i < count; i++) HIP_TRY(dec, hipMemcpy((char *)*out + i * bytes_each, srcs[i], bytes_each, hipMemcpyDeviceToDevice));
    return GR4AD_OK;
}

GemmEpilogue plain_epilogue(void *C, int64_t ldc);
GemmEpilogue f32_epilogue(void *C, int64_t ldc) {
    GemmEpilogue e = plain_epilogue(C, ldc);
    e.out_f32 = 1;
    return e;
}

GemmEpilogue plain_epilogue(void *C, int64_t ldc) {
    GemmEpilogue e;
    memset(&e, 0, sizeof(e));
    e.C = C;
    e.ldc = ldc;
    return e;
}

int validate_desc(const gr4ad_model_desc *ds) {
    if (!ds) return fail(nullptr, GR4AD_EINVAL, "desc is NULL");
    if (!ds->codebook || !ds->max_beam) return fail(nullptr, GR4AD_EINVAL, "codebook/max_beam is NULL");
    if (ds->d_model <= 0 || ds->n_heads <= 0 || ds->d_ffn <= 0 || ds->n_layers <= 0 || ds->max_batch <= 0 || ds->max_ctx <= 0)
        return fail(nullptr, GR4AD_EINVAL, "sizes must be positive");
    if (ds->d_model % ds->n_heads) return fail(nullptr, GR4AD_EINVAL, "d_model %d not divisible by n_heads %d", ds->d_model, ds->n_heads);
    if (ds->n_lazy < 0 || ds->n_lazy >= ds->n_layers) return fail(nullptr, GR4AD_EINVAL, "n_lazy %d outside [0, n_layers=%d)", ds->n_lazy, ds->n_layers);
    if (ds->vanilla_input && ds->n_lazy != 0) return fail(nullptr, GR4AD_EINVAL, "vanilla_input needs n_lazy = 0 (got %d)", ds->n_lazy);
    if (ds->n_levels < 1 || ds->n_levels > GR4AD_MAX_LEVELS) return fail(nullptr, GR4AD_EINVAL, "n_levels %d outside [1,%d]", ds->n_levels, GR4AD_MAX_LEVELS);
    if (ds->dtype != GR4AD_F32 && ds->dtype != GR4AD_BF16) return fail(nullptr, GR4AD_EINVAL, "unknown dtype %d", (int)ds->dtype);
    if (!(ds->rms_eps >= 0.0f)) return fail(nullptr, GR4AD_EINVAL, "rms_eps must be >= 0");
    if (ds->n_value_buckets < 0 || ds->n_value_buckets > GR4AD_MAX_CODEBOOK)
        return fail(nullptr, GR4AD_EINVAL, "n_value_buckets %d outside [0,%d]", ds->n_value_buckets, GR4AD_MAX_CODEBOOK);
    if (ds->fp8_gemm && ds->dtype != GR4AD_BF16) return fail(nullptr, GR4AD_EUNSUPPORTED, "fp8_gemm needs the bf16 storage dtype");
    if (ds->n_value_buckets > 0 && ds->n_levels + 1 > GR4AD_MAX_LEVELS)
        return fail(nullptr, GR4AD_EUNSUPPORTED, "a value step needs n_levels <= %d", GR4AD_MAX_LEVELS - 1);
    for (int t = 0; t < ds->n_levels; t++) {
        if (ds->codebook[t] < 1 || ds->max_beam[t] < 1) return fail(nullptr, GR4AD_EINVAL, "codebook/max_beam of level %d must be >= 1", t + 1);
        if (ds->codebook[t] > GR4AD_MAX_CODEBOOK) return fail(nullptr, GR4AD_EUNSUPPORTED, "codebook %d of level %d exceeds %d", ds->codebook[t], t + 1, GR4AD_MAX_CODEBOOK);
        if (ds->max_beam[t] > GR4AD_MAX_BEAM) return fail(nullptr, GR4AD_EUNSUPPORTED, "max_beam %d of level %d exceeds %d", ds->max_beam[t], t + 1, GR4AD_MAX_BEAM);
    }
    const int dh = ds->d_model / ds->n_heads;
    if (dh != 16 && dh != 32 && dh != 64 && dh != 128) return fail(nullptr, GR4AD_EUNSUPPORTED, "head width %d not in {16,32,64,128}", dh);
    if (ds->d_model % 8 || ds->d_ffn % 8) return fail(nullptr, GR4AD_EUNSUPPORTED, "d_model and d_ffn must be multiples of 8");
    return GR4AD_OK;
}

int validate_weights(const gr4ad_model_desc *ds, const gr4ad_weights *w) {
    if (!w) return fail(nullptr, GR4AD_EINVAL, "weights is NULL");
    if (!w->pos_dev || !w->bos_dev || !w->layers || !w->ln_out_dev || !w->cls_dev) return fail(nullptr, GR4AD_EINVAL, "a weight pointer is NULL");
    if (!ds->vanilla_input && (!w->w_g_dev || !w->w_f_dev)) return fail(nullptr, GR4AD_EINVAL, "a Fuse weight pointer is NULL");
    if (ds->n_levels > 1 && !w->emb_dev) return fail(nullptr, GR4AD_EINVAL, "emb_dev is NULL");
    for (int t = 0; t + 1 < ds->n_levels; t++)
        if (!w->emb_dev[t]) return fail(nullptr, GR4AD_EINVAL, "emb_dev[%d] is NULL", t);
    for (int t = 0; t < ds->n_levels; t++)
        if (!w->cls_dev[t]) return fail(nullptr, GR4AD_EINVAL, "cls_dev[%d] is NULL", t);
    if (ds->n_value_buckets > 0 && (!w->value_pos_dev || !w->value_emb_dev || !w->value_cls_dev))
        return fail(nullptr, GR4AD_EINVAL, "a value-step weight pointer is NULL");
    for (int l = 0; l < ds->n_layers; l++) {
        const gr4ad_layer_weights *x = &w->layers[l];
        const void *all[] = {x->ln_x, x->wq_x, x->wk_x, x->wv_x, x->wo_x, x->ln_s, x->wq_s, x->wk_s, x->wv_s, x->wo_s, x->ln_f, x->w1, x->w2};
        for (const void *p : all)
            if (!p) return fail(nullptr, GR4AD_EINVAL, "a weight pointer of layer %d is NULL", l);
    }
    return GR4AD_OK;
}

int init_impl(gr4ad_decoder *dec, const gr4ad_model_desc *ds, const gr4ad_weights *w) {
    const size_t e = dec->esz, d = dec->d, F = dec->F;
    HIP_TRY(dec, hipGetDevice(&dec->device));
    int s;
    if ((s = dev_alloc(dec, &dec->pos, dec->Tp * d * e))) return s;  // p_1..p_T, then p_{T+1} of the value step
    HIP_TRY(dec, hipMemcpy(dec->pos, w->pos_dev, dec->T * d * e, hipMemcpyDeviceToDevice));
    if (dec->Ve > 0) HIP_TRY(dec, hipMemcpy((char *)dec->pos + dec->T * d * e, w->value_pos_dev, d * e, hipMemcpyDeviceToDevice));
    if ((s = dev_clone(dec, &dec->ln_out, w->ln_out_dev, d * e))) return s;
    for (int t = 0; t < dec->T; t++) {
        if ((s = dev_clone(dec, &dec->cls[t], w->cls_dev[t], (size_t)dec->V[t] * d * e))) return s;
        dec->cls_bias[t] = nullptr;
        if (w->cls_bias_dev && w->cls_bias_dev[t])
            if ((s = dev_clone(dec, (void **)&dec->cls_bias[t], w->cls_bias_dev[t], (size_t)dec->V[t] * sizeof(float)))) return s;
    }
    if (dec->Ve > 0) {  // the value step is level T+1 with its own classifier
        const int T = dec->T;
        if ((s = dev_clone(dec, &dec->cls[T], w->value_cls_dev, (size_t)dec->Ve * d * e))) return s;
        dec->cls_bias[T] = nullptr;
        if (w->value_bias_dev)
            if ((s = dev_clone(dec, (void **)&dec->cls_bias[T], w->value_bias_dev, (size_t)dec->Ve * sizeof(float)))) return s;
    }
    dec->layers.resize(dec->L);
    for (int l = 0; l < dec->L; l++) {
        const gr4ad_layer_weights *x = &w->layers[l];
        LayerPacked &p = dec->layers[l];
        if ((s = dev_clone(dec, &p.ln_x, x->ln_x, d * e))) return s;
        if ((s = dev_clone(dec, &p.wq_x, x->wq_x, d * d * e))) return s;
        const void *kv[2] = {x->wk_x, x->wv_x};
        if ((s = dev_stack(dec, &p.wkv_x, kv, 2, d * d * e))) return s;
        if ((s = dev_clone(dec, &p.wo_x, x->wo_x, d * d * e))) return s;
        if ((s = dev_clone(dec, &p.ln_s, x->ln_s, d * e))) return s;
        const void *qkv[3] = {x->wq_s, x->wk_s, x->wv_s};
        if ((s = dev_stack(dec, &p.wqkv_s, qkv, 3, d * d * e))) return s;
        if ((s = dev_clone(dec, &p.wo_s, x->wo_s, d * d * e))) return s;
        if ((s = dev_clone(dec, &p.ln_f, x->ln_f, d * e))) return s;
        if ((s = dev_clone(dec, &p.w1, x->w1, F * d * e))) return s;
        if ((s = dev_clone(dec, &p.w2, x->w2, d * F * e))) return s;
        p.wkT_x = nullptr;
        if (dec->absorbed && l < dec->K) {
            if ((s = dev_alloc(dec, &p.wkT_x, d * d * e))) return s;
            OP_TRY(dec, launch_head_transpose(p.wkv_x, p.wkT_x, (int)d, dec->H, 0), "per-head key weight transpose");
        }
    }
    if (dec->vanilla) {  // no Fuse: the level's input is an embedding row plus the position embedding
        for (int t = 0; t < dec->Tp; t++) {
            const void *emb = t == 0 ? w->bos_dev : t == dec->T ? w->value_emb_dev : w->emb_dev[t - 1];
            const int64_t rows = t == 0 ? 1 : dec->V[t - 1];
            if ((s = dev_clone(dec, &dec->E[t], emb, rows * d * e))) return s;
        }
    }
    // Fuse (eq. fuse) is linear in the token embedding s: W_f [m*(W_g s); s] = W_f[:, :d] (m * (W_g s)) + W_f[:, d:] s.
    // Split W_f and tabulate W_g s and W_f[:, d:] s for BOS and for every token of every level.
    void *wf2 = nullptr, *wg = nullptr;
    if (!dec->vanilla) {
    if ((s = dev_alloc(dec, &dec->wf1, d * d * e))) return s;
    if ((s = dev_alloc(dec, &wf2, d * d * e))) return s;
    if ((s = dev_clone(dec, &wg, w->w_g_dev, d * d * e))) return s;
    HIP_TRY(dec, hipMemcpy2D(dec->wf1, d * e, w->w_f_dev, 2 * d * e, d * e, d, hipMemcpyDeviceToDevice));
    HIP_TRY(dec, hipMemcpy2D(wf2, d * e, (const char *)w->w_f_dev + d * e, 2 * d * e, d * e, d, hipMemcpyDeviceToDevice));
    for (int t = 0; t < dec->Tp; t++) {
        const void *emb = t == 0 ? w->bos_dev : t == dec->T ? w->value_emb_dev : w->emb_dev[t - 1];
        const int64_t rows = t == 0 ? 1 : dec->V[t - 1];
        if ((s = dev_alloc(dec, &dec->G[t], rows * d * sizeof(float)))) return s;
        if ((s = dev_alloc(dec, &dec->P[t], rows * d * sizeof(float)))) return s;
        OP_TRY(dec, launch_gemm(dec->dtype, emb, d, wg, d, rows, (int)d, (int)d, f32_epilogue(dec->G[t], d), 0), "Fuse gate table");
        OP_TRY(dec, launch_gemm(dec->dtype, emb, d, wf2, d, rows, (int)d, (int)d, f32_epilogue(dec->P[t], d), 0), "Fuse token table");
    }
    }
    if (dec->fp8) {
        unsigned *amax = nullptr;
        if ((s = dev_alloc(dec, (void **)&amax, 256))) return s;
        auto quant = [&](const void *wsrc, size_t count, void **out, float *scale) -> int {
            int r = dev_alloc(dec, out, count);
            if (r) return r;
            r = launch_quantize_matrix(wsrc, *out, (int64_t)count, amax, scale, 0);
            return r ? fail(dec, r, "FP8 weight quantisation failed: %s", gr4ad_strerror(r)) : GR4AD_OK;
        };
        for (int l = dec->K; l < dec->L; l++) {
            LayerPacked &p = dec->layers[l];
            if ((s = quant(p.wq_x, d * d, &p.wq_x8, &p.s_wq_x))) return s;
            if ((s = quant(p.wo_x, d * d, &p.wo_x8, &p.s_wo_x))) return s;
            if ((s = quant(p.wqkv_s, 3 * d * d, &p.wqkv_s8, &p.s_wqkv_s))) return s;
            if ((s = quant(p.wo_s, d * d, &p.wo_s8, &p.s_wo_s))) return s;
            if ((s = quant(p.w1, F * d, &p.w1_8, &p.s_w1))) return s;
            if ((s = quant(p.w2, d * F, &p.w2_8, &p.s_w2))) return s;
        }
        if (!dec->vanilla && (s = quant(dec->wf1, d * d, &dec->wf1_8, &dec->s_wf1))) return s;
        for (int t = 0; t < dec->Tp; t++)
            if ((s = quant(dec->cls[t], (size_t)dec->V[t] * d, &dec->cls8[t], &dec->s_cls[t]))) return s;
    }
    HIP_TRY(dec, hipDeviceSynchronize());
    return GR4AD_OK;
}

}  // namespace

int gr4ad_set_thread_error(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_init_error, sizeof(g_init_error), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" {

const char *gr4ad_strerror(int status) {
    switch (status) {
        case GR4AD_OK: return "ok";
        case GR4AD_EINVAL: return "invalid argument";
        case GR4AD_EUNSUPPORTED: return "unsupported configuration";
        case GR4AD_EWORKSPACE: return "workspace too small or misaligned";
        case GR4AD_EHIP: return "HIP runtime error";
        case GR4AD_ENOMEM: return "out of memory";
        default: return "unknown status";
    }
}

const char *gr4ad_last_error(const gr4ad_decoder *dec) { return dec ? dec->err : g_init_error; }

int gr4ad_decode_init(const gr4ad_model_desc *ds, const gr4ad_weights *w, gr4ad_decoder **out) {
    g_init_error[0] = 0;
    if (!out) return fail(nullptr, GR4AD_EINVAL, "out is NULL");
    int s = validate_desc(ds);
    if (s) return s;
    if ((s = validate_weights(ds, w))) return s;
    gr4ad_decoder *dec = new (std::nothrow) gr4ad_decoder();
    if (!dec) return fail(nullptr, GR4AD_ENOMEM, "host allocation failed");
    dec->d = ds->d_model; dec->H = ds->n_heads; dec->F = ds->d_ffn; dec->L = ds->n_layers; dec->K = ds->n_lazy;
    dec->T = ds->n_levels; dec->A = dec->L - dec->K; dec->max_batch = ds->max_batch; dec->max_ctx = ds->max_ctx;
    dec->dtype = ds->dtype; dec->esz = ds->dtype == GR4AD_BF16 ? 2 : 4; dec->eps = ds->rms_eps;
    dec->trace = false; dec->err[0] = 0;
    dec->fp8 = ds->fp8_gemm != 0;
    dec->vanilla = ds->vanilla_input != 0;
    dec->Ve = ds->n_value_buckets; dec->Tp = dec->T + (dec->Ve > 0 ? 1 : 0); dec->value_out = nullptr;
    {
        // The lazy layers attend with only T queries per request, so projecting every context row to keys and values
        // would dominate them.  Where the batched matrix-core kernel covers the shapes they use the absorbed form instead.
        const int dh = dec->d / dec->H;
        dec->absorbed = dec->K > 0 && dec->dtype == GR4AD_BF16 && dh % 64 == 0;
    }
    for (int t = 0; t < dec->T; t++) { dec->V[t] = ds->codebook[t]; dec->max_beam[t] = ds->max_beam[t]; }
    if (dec->Ve > 0) dec->V[dec->T] = dec->Ve;
    s = init_impl(dec, ds, w);
    if (s) {
        snprintf(g_init_error, sizeof(g_init_error), "%s", dec->err);
        gr4ad_decode_free(dec);
        return s;
    }
    *out = dec;
    return GR4AD_OK;
}

void gr4ad_decode_free(gr4ad_decoder *dec) {
    if (!dec) return;
    for (void *p : dec->allocs) (void)hipFree(p);
    delete dec;
}

size_t gr4ad_decode_workspace_bytes(const gr4ad_decoder *dec, int32_t B, int32_t S, const int32_t *beam) {
    if (!dec || !beam || B < 1 || S < 1 || B > dec->max_batch || S > dec->max_ctx || !beams_ok(dec, beam)) return 0;
    return make_plan(dec, B, S, beam).total;
}

int gr4ad_decode_set_trace(gr4ad_decoder *dec, int32_t *const *parent_dev, int32_t *const *tok_dev, float *const *score_dev) {
    if (!dec) return GR4AD_EINVAL;
    dec->trace = parent_dev || tok_dev || score_dev;
    for (int t = 0; t < dec->T; t++) {
        dec->tr_parent[t] = parent_dev ? parent_dev[t] : nullptr;
        dec->tr_tok[t] = tok_dev ? tok_dev[t] : nullptr;
        dec->tr_score[t] = score_dev ? score_dev[t] : nullptr;
    }
    return GR4AD_OK;
}

int gr4ad_decode_set_value_output(gr4ad_decoder *dec, float *out_value_logprob_dev) {
    if (!dec) return GR4AD_EINVAL;
    if (dec->Ve <= 0) return fail(dec, GR4AD_EINVAL, "the model has no value step (n_value_buckets = 0)");
    dec->value_out = out_value_logprob_dev;
    return GR4AD_OK;
}

int gr4ad_decode_batch(gr4ad_decoder *dec, const void *ctx, const int32_t *ctx_len, int32_t B, int32_t S, const int32_t *beam,
                       void *workspace, size_t workspace_bytes, int32_t *out_sid, float *out_logprob, void *hip_stream) {
    if (!dec) return GR4AD_EINVAL;
    dec->err[0] = 0;
    if (!ctx || !beam || !out_sid || !out_logprob) return fail(dec, GR4AD_EINVAL, "a required pointer is NULL");
    if (B < 1 || B > dec->max_batch) return fail(dec, GR4AD_EINVAL, "B=%d outside [1, max_batch=%d]", B, dec->max_batch);
    if (S < 1 || S > dec->max_ctx) return fail(dec, GR4AD_EINVAL, "S=%d outside [1, max_ctx=%d]", S, dec->max_ctx);
    if (!beams_ok(dec, beam)) return fail(dec, GR4AD_EINVAL, "beam schedule invalid: need 1 <= b_t <= max_beam[t] and b_t <= b_{t-1}*V_t");
    const Plan p = make_plan(dec, B, S, beam);
    if (!workspace || workspace_bytes < p.total) return fail(dec, GR4AD_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, p.total);
    if ((uintptr_t)workspace % 256) return fail(dec, GR4AD_EWORKSPACE, "workspace must be 256-byte aligned");
    if ((uintptr_t)ctx % 16) return fail(dec, GR4AD_EINVAL, "ctx_dev must be 16-byte aligned");

    hipStream_t st = (hipStream_t)hip_stream;
    const gr4ad_dtype dt = dec->dtype;
    const size_t e = dec->esz;
    const int d = dec->d, F = dec->F, T = dec->T, H = dec->H, A = dec->A, K = dec->K;
    // positions of the lazy pass and steps of the level loop: the value step (section 3.3) is one more level after s_T that
    // ends in a log-softmax instead of a selection.  The lazy pass is causal, so the first T positions do not depend on it.
    const bool value_step = dec->Ve > 0 && dec->value_out;
    const int Tq = value_step ? T + 1 : T;
    char *ws = (char *)workspace;
    void *h = ws + p.h, *xn = ws + p.xn, *q = ws + p.q, *o = ws + p.o, *qkv = ws + p.qkv, *f = ws + p.f, *trunk = ws + p.trunk;
    float *logits = (float *)(ws + p.logits);
    auto kv_ar = [&](int a) { return (void *)(ws + p.kv_ar + (size_t)a * B * S * 2 * d * e); };
    auto qkv_lvl = [&](int t, int a) { return (void *)(ws + p.qkv_lvl[t] + (size_t)(t == dec->Tp - 1 ? 0 : a) * p.qkv_lvl_layer_bytes[t]); };

    auto gemm = [&](const void *Ain, int64_t M, const void *W, int N, int Kdim, const GemmEpilogue &epi) {
        return launch_gemm(dt, Ain, Kdim, W, Kdim, M, N, Kdim, epi, st);
    };
    auto resid_epi = [&](void *x, int64_t ld) { GemmEpilogue g = plain_epilogue(x, ld); g.resid = (const float *)x; g.ldr = ld; g.out_f32 = 1; return g; };
    auto silu_epi = [&](void *x, int64_t ld) { GemmEpilogue g = plain_epilogue(x, ld); g.act = ACT_SILU; return g; };

    // RMSNorm folded into the projections around it.  Every norm sits between a projection that writes the residual
    // stream x (residual update or Fuse) and one that reads norm(x).  On launches that run on the persistent kernel the
    // writer also stores gain * x (storage dtype, into xn) and per-row partial sums of x^2, and the reader scales its
    // product rows by 1/rms(x) - (gain * x / rms) W^T = (1/rms) (gain * x) W^T - so the norm kernel and its pass over
    // the stream disappear.  Elsewhere (small launches, float32, widths the kernel does not cover) the norm kernel runs.
    const int nparts = d / 64;
    float *ss = (float *)(ws + p.ss), *rinv = ss + (size_t)p.rows_max * nparts;  // partial sums of x^2; 1/rms per row
    bool fold = false;             // set per phase: this row count and these widths run on the persistent kernel
    bool scaled = false;           // xn holds gain * x without the 1/rms factor; its reader must apply row_ss
    const void *emitted = nullptr; // gain the last writer of x folded in (xn and ss are current for exactly that norm)
    auto fold_ok = [&](int64_t rows, int n_cls) -> bool {
        if (dt != GR4AD_BF16 || d % 256 || F % 64 || F < 256 || F % 8 || (n_cls && (n_cls < 256 || n_cls % 4))) return false;
        GemmEpilogue g = plain_epilogue(trunk, d);  // representative writer: a d x d residual update
        g.resid = (const float *)trunk; g.ldr = d; g.out_f32 = 1;
        g.norm_gain = dec->ln_out; g.norm_out = xn; g.norm_ld = d; g.norm_ss = ss;
        GemmEpilogue r = plain_epilogue(q, d);      // representative reader
        r.row_inv = rinv;
        return gemm_on_persistent_kernel(dt, o, d, dec->layers[0].wo_x, d, rows, d, d, g) &&
               gemm_on_persistent_kernel(dt, xn, d, dec->layers[0].wq_x, d, rows, d, d, r);
    };
    auto emit_norm = [&](GemmEpilogue g, const void *next_gain) {  // writer side: x is followed by RMSNorm with next_gain
        emitted = nullptr;
        if (fold && next_gain) { g.norm_gain = next_gain; g.norm_out = xn; g.norm_ld = d; g.norm_ss = ss; emitted = next_gain; }
        return g;
    };
    // FP8 mode (autoregressive levels only; f8 is set there): a per-row projection reads its operand from aq, E4M3 bytes with
    // one scale per row.  The norm in front of a projection writes it directly; a bf16 operand (attention output, FFN
    // hidden rows, gated embedding) is quantised by its own pass over the rows.
    bool f8 = false;
    uint8_t *aq = (uint8_t *)(ws + p.aq);
    float *ascale = (float *)(ws + p.ascale);
    auto quant_act = [&](const void *act, int64_t rows, int width) { return launch_quantize_rows(act, aq, ascale, rows, width, st); };
    auto gemm8 = [&](int64_t M, const void *W8, float wscale, int N, int Kdim, const GemmEpilogue &epi) {
        return launch_gemm_f8(aq, Kdim, ascale, W8, Kdim, wscale, M, N, Kdim, epi, st);
    };
    auto norm = [&](void *x, const void *gain, int64_t rows) -> int {
        if (f8) {
            emitted = nullptr;
            scaled = false;
            return launch_rmsnorm_quant(x, gain, aq, ascale, rows, d, dec->eps, st);
        }
        if (emitted && emitted == gain) {
            emitted = nullptr;
            scaled = true;
            return launch_row_inv(ss, rinv, rows, nparts, d, dec->eps, st);
        }
        emitted = nullptr;
        scaled = false;
        return launch_rmsnorm(dt, x, gain, xn, rows, d, dec->eps, st);
    };
    auto reads_norm = [&](GemmEpilogue g) {  // reader side: the A operand is xn
        if (scaled) g.row_inv = rinv;
        return g;
    };

    // cross-attention + its residual; x is the residual stream [rows,d]; next_gain: gain of the norm that follows
    auto cross_block = [&](const LayerPacked &lw, void *x, int64_t rows, int n, const void *kvbuf, const void *vtbuf) -> int {
        int s;
        if ((s = norm(x, lw.ln_x, rows))) return s;
        if (f8) s = gemm8(rows, lw.wq_x8, lw.s_wq_x, d, d, plain_epilogue(q, d));
        else s = gemm(xn, rows, lw.wq_x, d, d, reads_norm(plain_epilogue(q, d)));
        if (s) return s;
        if ((s = launch_cross_attention(dt, q, d, kvbuf, vtbuf, ctx_len, o, d, B, n, S, d, H, st))) return s;
        if (f8) {
            if ((s = quant_act(o, rows, d))) return s;
            return gemm8(rows, lw.wo_x8, lw.s_wo_x, d, d, resid_epi(x, d));
        }
        return gemm(o, rows, lw.wo_x, d, d, emit_norm(resid_epi(x, d), lw.ln_s));
    };
    auto ffn_block = [&](const LayerPacked &lw, void *x, int64_t rows, const void *next_gain) -> int {
        int s;
        if ((s = norm(x, lw.ln_f, rows))) return s;
        if (f8) {
            if ((s = gemm8(rows, lw.w1_8, lw.s_w1, F, d, silu_epi(f, F)))) return s;
            if ((s = quant_act(f, rows, F))) return s;
            return gemm8(rows, lw.w2_8, lw.s_w2, d, F, resid_epi(x, d));
        }
        if ((s = gemm(xn, rows, lw.w1, F, d, reads_norm(silu_epi(f, F))))) return s;
        return gemm(f, rows, lw.w2, d, F, emit_norm(resid_epi(x, d), next_gain));
    };

    // ---- step 0: context keys/values of the autoregressive layers, once per request ----
    auto vt_ar = [&](int a) { return p.vt_bytes ? (void *)(ws + p.vt_ar + (size_t)a * p.vt_bytes) : (void *)nullptr; };
    void *vt_lazy = p.vt_bytes ? (void *)(ws + p.vt_lazy) : (void *)nullptr;
    // Where the attention kernel reads the values from its transposed copy, the value projection writes that copy
    // directly (transposed per request, zero beyond the length) and only the key half of the K/V buffer is filled.
    auto context_kv = [&](const LayerPacked &lw, void *kvbuf, void *vtbuf) -> int {
        const void *wv = (const char *)lw.wkv_x + (size_t)d * d * e;
        if (vtbuf && gemm_vt_supported(dt, ctx, d, wv, d, (int64_t)B * S, d, d, S, vtbuf, S)) {
            // (keys and values of rows past a request's length are never read: whole tiles of them are not computed)
            GemmEpilogue ke = plain_epilogue(kvbuf, 2 * d);
            ke.skip_len = ctx_len;
            ke.skip_S = S;
            int s = gemm(ctx, (int64_t)B * S, lw.wkv_x, d, d, ke);
            if (s) return s;
            return launch_gemm_vt(ctx, d, wv, d, (int64_t)B * S, d, d, S, ctx_len, vtbuf, S, st);
        }
        int s = gemm(ctx, (int64_t)B * S, lw.wkv_x, 2 * d, d, plain_epilogue(kvbuf, 2 * d));
        if (s) return s;
        return launch_cross_attention_prepare(dt, kvbuf, ctx_len, vtbuf, B, S, d, H, st);
    };
    for (int a = 0; a < A; a++) OP_TRY(dec, context_kv(dec->layers[K + a], kv_ar(a), vt_ar(a)), "context K/V projection");

    // Lazy layers, cross-attention in absorbed form.  With k_s = W_k x_s and v_s = W_v x_s (per head h: rows h*dh.. of W_k, W_v),
    //   q_h . k_{s,h} = (W_{k,h}^T q_h) . x_s        and        sum_s p_s v_{s,h} = W_{v,h} (sum_s p_s x_s),
    // so T*H queries per request attend over the raw context rows: no key/value projection of the S context rows
    // (2*S*d*2d flops per request and layer) but two small products per (row, head) and two [T*H, d] x [d, S] products
    // per request.  Same function of the inputs as eq. trunk's cross-attention; the intermediate roundings to bf16
    // fall on q' = W_{k,h}^T q_h and z = sum_s p_s x_s instead of on k_s and v_s.
    auto absorbed_cross_block = [&](const LayerPacked &lw, bool first) -> int {
        const int64_t rows = (int64_t)B * Tq, RQ = (int64_t)Tq * H;
        const int dh = d / H, Spad = (S + 63) / 64 * 64;
        char *xt = ws + p.xt, *qp = ws + p.qp, *zb = ws + p.zb, *pb = ws + p.pb;
        float *sc = (float *)(ws + p.sc);
        const char *wv = (const char *)lw.wkv_x + (size_t)d * d * e;
        int s;
        const bool one_pass = context_attention_covers(dt, (int)RQ, d);
        if (first && !one_pass && (s = launch_context_transpose(ctx, ctx_len, xt, B, S, d, st))) return s;  // once per decode, shared by all lazy layers
        if ((s = norm(trunk, lw.ln_x, rows))) return s;
        if ((s = gemm(xn, rows, lw.wq_x, d, d, reads_norm(plain_epilogue(q, d))))) return s;
        // q'[row][h][:] = W_{k,h}^T q[row][h*dh : (h+1)*dh]      (batch = head)
        if ((s = launch_gemm_batched(q, d, dh, lw.wkT_x, dh, (int64_t)d * dh, qp, (int64_t)H * d, d, 0, rows, d, dh, H, nullptr, 0, st))) return s;
        if (one_pass) {
            // scores, softmax and z in one kernel that reads the request's context rows once (widths and query counts it covers)
            if ((s = launch_context_attention(dt, qp, ctx, ctx_len, zb, B, (int)RQ, S, d, 1.0f / sqrtf((float)dh), st))) return s;
        } else {
            // raw scores[b][(t,h)][s] = q'[b][(t,h)] . x[b][s]         (batch = request; columns beyond the length are not needed)
            if ((s = launch_gemm_batched(qp, d, RQ * d, ctx, d, (int64_t)S * d, sc, Spad, RQ * Spad, 1, RQ, S, d, B, ctx_len, 1, st))) return s;
            if ((s = launch_masked_softmax(sc, pb, ctx_len, (int64_t)B * RQ, (int)RQ, S, Spad, 1.0f / sqrtf((float)dh), st))) return s;
            // z[b][(t,h)][:] = sum_s p[b][(t,h)][s] x[b][s][:]         (batch = request; p and x^T are zero beyond the length)
            if ((s = launch_gemm_batched(pb, Spad, RQ * Spad, xt, Spad, (int64_t)d * Spad, zb, d, RQ * d, 0, RQ, d, Spad, B, ctx_len, 2, st))) return s;
        }
        // o[row][h*dh : (h+1)*dh] = W_{v,h} z[row][h][:]           (batch = head)
        if ((s = launch_gemm_batched(zb, (int64_t)H * d, d, wv, d, (int64_t)dh * d, o, d, dh, 0, rows, dh, d, H, nullptr, 0, st))) return s;
        return gemm(o, rows, lw.wo_x, d, d, emit_norm(resid_epi(trunk, d), lw.ln_s));
    };

    // ---- step 1: lazy pass (eq. trunk): all T levels at once, no beam dimension ----
    if (!dec->vanilla) OP_TRY(dec, launch_broadcast_rows(dt, dec->pos, trunk, B, Tq, d, st), "trunk input");
    fold = K > 0 && fold_ok((int64_t)B * Tq, 0);
    for (int l = 0; l < K; l++) {
        const LayerPacked &lw = dec->layers[l];
        void *kvl = ws + p.kv_lazy;
        const int64_t rows = (int64_t)B * Tq;
        if (dec->absorbed) {
            OP_TRY(dec, absorbed_cross_block(lw, l == 0), "lazy cross-attention (absorbed form)");
        } else {
            OP_TRY(dec, context_kv(lw, kvl, vt_lazy), "lazy context K/V projection");
            OP_TRY(dec, cross_block(lw, trunk, rows, Tq, kvl, vt_lazy), "lazy cross-attention");
        }
        OP_TRY(dec, norm(trunk, lw.ln_s, rows), "lazy norm");
        OP_TRY(dec, gemm(xn, rows, lw.wqkv_s, 3 * d, d, reads_norm(plain_epilogue(qkv, 3 * d))), "lazy qkv");
        OP_TRY(dec, launch_trunk_self_attention(dt, qkv, o, B, Tq, d, H, st), "lazy self-attention");
        OP_TRY(dec, gemm(o, rows, lw.wo_s, d, d, emit_norm(resid_epi(trunk, d), lw.ln_f)), "lazy self-attention output");
        OP_TRY(dec, ffn_block(lw, trunk, rows, l + 1 < K ? dec->layers[l + 1].ln_x : nullptr), "lazy FFN");
    }

    // ---- level loop (eq. fuse, eq. head, classifier, selection, reorder) ----
    int n = 1, cur = 0;
    for (int t = 0; t < Tq; t++) {
        const int64_t rows = (int64_t)B * n;
        const int bt = t < T ? beam[t] : n;  // the value step keeps every beam
        const int32_t *tok_prev = t == 0 ? nullptr : (const int32_t *)(ws + p.tok[cur]);
        f8 = dec->fp8;
        fold = !f8 && fold_ok(rows, dec->V[t]);
        scaled = false;
        emitted = nullptr;
        if (dec->vanilla) {
            // vanilla decoder (section 3.2): h^(0)_t = s_{t-1} + p_t
            OP_TRY(dec, launch_embed_pos(dt, dec->E[t], tok_prev, (const char *)dec->pos + (size_t)t * d * e, h, rows, d, st), "vanilla input state");
        } else {
            // the gated embedding goes through q when the Fuse projection also writes the first norm's input into xn
            void *gated = fold ? q : xn;
            OP_TRY(dec, launch_fuse_gate(dt, (const float *)trunk + (size_t)t * d, (int64_t)Tq * d, dec->G[t], t == 0 ? 1 : dec->V[t - 1], tok_prev, gated, B, n, d, st), "Fuse gate");
            GemmEpilogue g = plain_epilogue(h, d);
            g.out_f32 = 1;
            g.table = (const float *)dec->P[t];
            g.tok = tok_prev;
            if (f8) {
                OP_TRY(dec, quant_act(gated, rows, d), "Fuse operand quantisation");
                OP_TRY(dec, gemm8(rows, dec->wf1_8, dec->s_wf1, d, d, g), "Fuse projection");
            } else {
                OP_TRY(dec, gemm(gated, rows, dec->wf1, d, d, emit_norm(g, dec->layers[K].ln_x)), "Fuse projection");
            }
        }
        for (int a = 0; a < A; a++) {
            const LayerPacked &lw = dec->layers[K + a];
            OP_TRY(dec, cross_block(lw, h, rows, n, kv_ar(a), vt_ar(a)), "cross-attention");
            OP_TRY(dec, norm(h, lw.ln_s, rows), "self-attention norm");
            LevelBuffers prev;
            for (int u = 0; u < GR4AD_MAX_LEVELS; u++) {
                prev.p[u] = u < t ? qkv_lvl(u, a) : nullptr;
                prev.rows[u] = u < t ? (int64_t)B * (u == 0 ? 1 : beam[u - 1]) : 0;
            }
            if (f8) OP_TRY(dec, gemm8(rows, lw.wqkv_s8, lw.s_wqkv_s, 3 * d, d, plain_epilogue(qkv_lvl(t, a), 3 * d)), "self-attention qkv");
            else OP_TRY(dec, gemm(xn, rows, lw.wqkv_s, 3 * d, d, reads_norm(plain_epilogue(qkv_lvl(t, a), 3 * d))), "self-attention qkv");
            OP_TRY(dec, launch_self_attention_step(dt, qkv_lvl(t, a), prev, (const int32_t *)(ws + p.anc[cur]), o, rows, t, T, d, H, st),
                   "self-attention");
            if (f8) {
                OP_TRY(dec, quant_act(o, rows, d), "self-attention output quantisation");
                OP_TRY(dec, gemm8(rows, lw.wo_s8, lw.s_wo_s, d, d, resid_epi(h, d)), "self-attention output");
            } else {
                OP_TRY(dec, gemm(o, rows, lw.wo_s, d, d, emit_norm(resid_epi(h, d), lw.ln_f)), "self-attention output");
            }
            OP_TRY(dec, ffn_block(lw, h, rows, a + 1 < A ? dec->layers[K + a + 1].ln_x : dec->ln_out), "FFN");
        }
        OP_TRY(dec, norm(h, dec->ln_out, rows), "final norm");
        const bool lf16 = level_logits_f16(dec, rows, t);
        {
            GemmEpilogue g = plain_epilogue(logits, dec->V[t]);
            g.out_f32 = 1;
            g.out_f16 = lf16 ? 1 : 0;
            g.bias = dec->cls_bias[t];
            if (f8) OP_TRY(dec, gemm8(rows, dec->cls8[t], dec->s_cls[t], dec->V[t], d, g), "classifier");
            else OP_TRY(dec, gemm(xn, rows, dec->cls[t], dec->V[t], d, reads_norm(g)), "classifier");
        }
        if (t == T) {  // value step: log p(v | y, X) for every surviving beam, in the order of out_sid
            OP_TRY(dec, launch_log_softmax_rows(logits, dec->value_out, rows, dec->Ve, st), "value log-softmax");
            break;
        }
        const bool last = t == T - 1;
        int32_t *par = (int32_t *)(ws + p.par), *tok_new = (int32_t *)(ws + p.tok[cur ^ 1]);
        float *score_new = last ? out_logprob : (float *)(ws + p.cum[cur ^ 1]);
        int32_t *sid_new = last ? out_sid : (int32_t *)(ws + p.sid[cur ^ 1]);
        OP_TRY(dec, launch_select(logits, lf16 ? 1 : 0, t == 0 ? nullptr : (const float *)(ws + p.cum[cur]), B, n, dec->V[t], bt, ws + p.selws,
                                  select_workspace_bytes(B, n, dec->V[t], bt), par, tok_new, score_new, (const int32_t *)(ws + p.sid[cur]),
                                  sid_new, (const int32_t *)(ws + p.anc[cur]), last && !value_step ? nullptr : (int32_t *)(ws + p.anc[cur ^ 1]), T, t, st),
               "selection");
        if (dec->trace) {
            const size_t nb = (size_t)B * bt * 4;
            if (dec->tr_parent[t]) HIP_TRY(dec, hipMemcpyAsync(dec->tr_parent[t], par, nb, hipMemcpyDeviceToDevice, st));
            if (dec->tr_tok[t]) HIP_TRY(dec, hipMemcpyAsync(dec->tr_tok[t], tok_new, nb, hipMemcpyDeviceToDevice, st));
            if (dec->tr_score[t]) HIP_TRY(dec, hipMemcpyAsync(dec->tr_score[t], score_new, nb, hipMemcpyDeviceToDevice, st));
        }
        // beam reorder: the survivors' ancestor rows (written by the selection) are all that moves; keys and values stay where
        // their level wrote them
        cur ^= 1;
        n = bt;
    }
    return GR4AD_OK;
}

// ---- single-operation entry points ------------------------------------------
int gr4ad_op_linear(gr4ad_dtype dtype, const void *A, const void *W, const float *bias, void *C, int32_t M, int32_t N, int32_t K,
                    int32_t out_f32, void *hip_stream) {
    if (!A || !W || !C || M < 1 || N < 1 || K < 1 || (dtype != GR4AD_F32 && dtype != GR4AD_BF16)) return GR4AD_EINVAL;
    GemmEpilogue e = plain_epilogue(C, N);
    e.bias = bias;
    e.out_f32 = out_f32 ? 1 : 0;
    return launch_gemm(dtype, A, K, W, K, M, N, K, e, (hipStream_t)hip_stream);
}

int gr4ad_op_quantize_rows(const void *x, void *q, float *scale, int32_t rows, int32_t n, void *hip_stream) {
    if (!x || !q || !scale || rows < 1 || n < 8 || n % 8) return GR4AD_EINVAL;
    return launch_quantize_rows(x, q, scale, rows, n, (hipStream_t)hip_stream);
}

int gr4ad_op_linear_fp8(const void *Aq, const float *a_scale, const void *Wq, float w_scale, const float *bias, void *C, int32_t M, int32_t N,
                        int32_t K, int32_t out_f32, void *hip_stream) {
    if (!Aq || !a_scale || !Wq || !C || M < 1 || N < 1 || K < 1 || !(w_scale > 0.0f)) return GR4AD_EINVAL;
    GemmEpilogue e = plain_epilogue(C, N);
    e.bias = bias;
    e.out_f32 = out_f32 ? 1 : 0;
    return launch_gemm_f8(Aq, K, a_scale, Wq, K, w_scale, M, N, K, e, (hipStream_t)hip_stream);
}

size_t gr4ad_op_select_workspace_bytes(int32_t B, int32_t n, int32_t V, int32_t k) {
    if (B < 1 || n < 1 || V < 1 || k < 1) return 0;
    return select_workspace_bytes(B, n, V, k);
}

int gr4ad_op_select(const float *logits, const float *cum, int32_t B, int32_t n, int32_t V, int32_t k, void *ws, size_t ws_bytes,
                    int32_t *parent, int32_t *tok, float *score, void *hip_stream) {
    if (!logits || !ws || !parent || !tok || !score) return GR4AD_EINVAL;
    return launch_select(logits, 0, cum, B, n, V, k, ws, ws_bytes, parent, tok, score, nullptr, nullptr, nullptr, nullptr, 0, 0,
                         (hipStream_t)hip_stream);
}

int gr4ad_op_select_f16(const void *logits, const float *cum, int32_t B, int32_t n, int32_t V, int32_t k, void *ws, size_t ws_bytes,
                        int32_t *parent, int32_t *tok, float *score, void *hip_stream) {
    if (!logits || !ws || !parent || !tok || !score) return GR4AD_EINVAL;
    return launch_select(logits, 1, cum, B, n, V, k, ws, ws_bytes, parent, tok, score, nullptr, nullptr, nullptr, nullptr, 0, 0,
                         (hipStream_t)hip_stream);
}

size_t gr4ad_op_cross_attention_workspace_bytes(gr4ad_dtype dtype, int32_t B, int32_t S, int32_t d, int32_t H) {
    if (B < 1 || S < 1 || d < 1 || H < 1 || d % H) return 0;
    return cross_attention_workspace_bytes(dtype, B, S, d, H);
}

int gr4ad_op_cross_attention(gr4ad_dtype dtype, const void *q, const void *kv, const int32_t *ctx_len, void *out, int32_t B, int32_t n,
                             int32_t S, int32_t d, int32_t H, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!q || !kv || !out || (dtype != GR4AD_F32 && dtype != GR4AD_BF16) || B < 1 || n < 1 || S < 1 || d < 1 || H < 1 || d % H) return GR4AD_EINVAL;
    const size_t need = cross_attention_workspace_bytes(dtype, B, S, d, H);
    if (need && (!workspace || workspace_bytes < need)) return GR4AD_EWORKSPACE;
    int s = launch_cross_attention_prepare(dtype, kv, ctx_len, workspace, B, S, d, H, (hipStream_t)hip_stream);
    if (s) return s;
    return launch_cross_attention(dtype, q, d, kv, need ? workspace : nullptr, ctx_len, out, d, B, n, S, d, H, (hipStream_t)hip_stream);
}

int gr4ad_op_context_attention(gr4ad_dtype dtype, const void *q, const void *x, const int32_t *ctx_len, void *out, int32_t B, int32_t RQ,
                               int32_t S, int32_t d, float scale, void *hip_stream) {
    if (!q || !x || !out || B < 1 || RQ < 1 || S < 1 || d < 1 || !(scale > 0.0f)) return GR4AD_EINVAL;
    return launch_context_attention(dtype, q, x, ctx_len, out, B, RQ, S, d, scale, (hipStream_t)hip_stream);
}

int gr4ad_op_gather_rows(gr4ad_dtype dtype, const void *src, const int32_t *parent, void *dst, int32_t B, int32_t n, int32_t k,
                         int64_t row_elems, int64_t row_stride, void *hip_stream) {
    if (!src || !parent || !dst || B < 1 || n < 1 || k < 1 || row_elems < 1 || row_stride < row_elems) return GR4AD_EINVAL;
    return launch_gather_rows(dtype, src, parent, dst, B, n, k, row_elems, row_stride, (hipStream_t)hip_stream);
}

}  // extern "C"
