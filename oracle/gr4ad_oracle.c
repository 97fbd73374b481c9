/*
 * GR4AD LazyAR beam decode -- CPU ORACLE (test infrastructure, not the product).
 *
 * A plain, slow, obviously-correct implementation of what the serving hot path
 * computes: the LazyAR decoder (paper section 3.2, Lazy Autoregressive Decoder:
 * eq. trunk / fuse / head and the classifier softmax) driven by beam search
 * with a per-level beam width (section 4.2, Dynamic Beam Width; appendix A.2).
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP path.
 *
 * Arithmetic type: `real`, double unless compiled with -DORC_REAL_FLOAT.
 * All inputs are float32 arrays; all floating point outputs are double.
 *
 * What is the *definition* and what is an acceleration here:
 *   - orc_forward_seq   teacher-forced forward over a whole prefix.  This is the
 *                       definition of p(s_t | s_<t, X): nothing is cached except
 *                       the per-request cross-attention keys/values.
 *   - orc_decode_plain  beam search by definition: every live prefix is re-run
 *                       through orc_forward_seq, all n_t*V_t candidates are
 *                       fully sorted, the first b_t are kept.
 *   - orc_decode_cached the same search with the lossless accelerations the
 *                       paper names (trunk computed once and shared by beams
 *                       and levels; self-attention K/V kept per beam path).
 *                       Pinned to orc_decode_plain by tests.
 *
 * Readings of the paper where it is silent (decoder layer internals are
 * deferred to OneRec-V2 in section 3.2):
 *   RMSNorm with gain, pre-norm residual sub-layers in the order the paper
 *   lists them (cross-attention over X, causal self-attention over decoder
 *   states, feed-forward W2*SiLU(W1*x)); no linear biases; standard multi-head
 *   attention with per-layer key/value projections of the raw context X;
 *   final RMSNorm before the per-level classifier W_t (+ optional bias);
 *   Fuse weights shared by all levels; beam score = sum of log-probabilities;
 *   equal scores ordered by ascending flat candidate index i*V_t + v.
 *
 * FP8 mode (orc_desc.fp8 != 0; appendix A.2, "Low-Precision Inference": the
 * deployed model computes in FP8).  The paper names neither the format nor the
 * scaling; the reading taken here: the matrix products that run once per beam
 * row - the projections of the autoregressive layers (all but the context
 * key/value projections, which run once per request), the W_f[:, :d] half of
 * Fuse and the level classifiers - take both operands on the OCP E4M3 grid
 * (4 exponent bits, bias 7, 3 mantissa bits, largest value 448, round to
 * nearest even, saturating).  A weight matrix has one scale amax(W)/448 for
 * the whole matrix (the three self-attention input projections count as one
 * matrix); an activation row has its own scale amax(row)/448, taken when the
 * product is formed.  Products and sums are exact in `real`; everything else
 * (norms, attention, residuals, softmax, the lazy layers) is unchanged.
 *
 * Vanilla input (orc_desc.vanilla != 0; section 3.2, "Vanilla Autoregressive
 * Decoding"): the decoder the paper compares LazyAR against.  The input state of
 * level t is h^(0)_t = s_{t-1} + p_t (embedding of the previous token plus the
 * position embedding), every one of the L layers runs autoregressively (K must
 * be 0) and Fuse does not exist (w_g, w_f are ignored and may be NULL).
 *
 * Parity with the authors' trained model: parity unpinned (no weights exist).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifdef ORC_REAL_FLOAT
typedef float real;
#define R_EXP expf
#define R_LOG logf
#define R_SQRT sqrtf
#else
typedef double real;
#define R_EXP exp
#define R_LOG log
#define R_SQRT sqrt
#endif

#define ORC_MAX_LEVELS 8

/* ------------------------------------------------------------------ */
/* public structs (mirrored by ctypes in oracle/__init__.py)           */
/* ------------------------------------------------------------------ */
typedef struct {
    int32_t d, H, F, L, K, T;
    const int32_t *V; /* [T] codebook size per level */
    float eps;
    int32_t fp8;      /* != 0: FP8 mode (see the header comment) */
    int32_t vanilla;  /* != 0: vanilla autoregressive input h^(0)_t = s_{t-1} + p_t, K must be 0 (see the header comment) */
} orc_desc;

typedef struct {
    const float *ln_x, *wq_x, *wk_x, *wv_x, *wo_x; /* cross-attention: [d], 4 x [d,d] */
    const float *ln_s, *wq_s, *wk_s, *wv_s, *wo_s; /* self-attention */
    const float *ln_f, *w1, *w2;                   /* FFN: [d], [F,d], [d,F] */
} orc_layer_w;

typedef struct {
    const float *pos;            /* [T,d]  p_t */
    const float *bos;            /* [d]    s_0 */
    const float *const *emb;     /* [T-1] -> [V_t,d] embedding of s_t, t = 1..T-1 */
    const float *w_g, *w_f;      /* [d,d], [d,2d] */
    const orc_layer_w *layers;   /* [L] */
    const float *ln_out;         /* [d] */
    const float *const *cls;     /* [T] -> [V_t,d] */
    const float *const *cls_bias;/* [T] -> [V_t] or NULL (array itself may be NULL) */
} orc_weights;

/* internal model: weights converted to `real`, all matrices kept [out,in] */
typedef struct {
    real *ln_x, *wq_x, *wk_x, *wv_x, *wo_x, *ln_s, *wq_s, *wk_s, *wv_s, *wo_s, *ln_f, *w1, *w2;
} layer_r;

typedef struct orc_model {
    int d, H, F, L, K, T;
    int V[ORC_MAX_LEVELS];
    real eps;
    int fp8, vanilla;
    real *pos, *bos, *emb[ORC_MAX_LEVELS], *w_g, *w_f, *ln_out, *cls[ORC_MAX_LEVELS], *cls_bias[ORC_MAX_LEVELS];
    layer_r *layers;
} orc_model;

/* per-request state: valid context length and the cross-attention keys and
 * values Kc = X Wk^T, Vc = X Wv^T of every layer (computed once: they depend
 * on neither the beam nor the level). */
typedef struct orc_req {
    int len;
    real **Kc, **Vc; /* [L] -> [len,d] */
    int L;
} orc_req;

/* ------------------------------------------------------------------ */
/* primitives                                                          */
/* ------------------------------------------------------------------ */
static real *ralloc(size_t n) {
    real *p = (real *)calloc(n ? n : 1, sizeof(real));
    if (!p) { fprintf(stderr, "oracle: out of memory (%zu reals)\n", n); abort(); }
    return p;
}
static real *rcopy_f(const float *src, size_t n) {
    real *p = ralloc(n);
    for (size_t i = 0; i < n; i++) p[i] = (real)src[i];
    return p;
}

/* y[r][o] = sum_i W[o][i] * x[r][i]   (y = W x for every row) */
static void linear(real *y, const real *x, const real *W, int rows, int in, int out) {
#pragma omp parallel for schedule(static) if (!omp_in_parallel() && rows >= 8)
    for (int r = 0; r < rows; r++)
        for (int o = 0; o < out; o++) {
            const real *w = W + (size_t)o * in, *xr = x + (size_t)r * in;
            real acc = 0;
#pragma omp simd reduction(+ : acc)
            for (int i = 0; i < in; i++) acc += w[i] * xr[i];
            y[(size_t)r * out + o] = acc;
        }
}

/* N(x) = g * x / sqrt(mean(x^2) + eps), row by row */
static void rmsnorm(real *y, const real *x, const real *g, int rows, int d, real eps) {
    for (int r = 0; r < rows; r++) {
        real ss = 0;
        for (int i = 0; i < d; i++) ss += x[(size_t)r * d + i] * x[(size_t)r * d + i];
        real inv = 1 / R_SQRT(ss / d + eps);
        for (int i = 0; i < d; i++) y[(size_t)r * d + i] = g[i] * x[(size_t)r * d + i] * inv;
    }
}

static real silu(real x) { return x / (1 + R_EXP(-x)); }

/* nearest value of the OCP E4M3 grid: +-m * 2^(e-3), m in 8..15, e in -6..8 (normal) or m in 0..7, e = -6 (subnormal),
 * largest value 448; ties go to the even m; magnitudes beyond the grid saturate at 448 */
static real e4m3_round(real v) {
    double a = fabs((double)v);
    if (a == 0) return 0;
    int e;
    (void)frexp(a, &e); /* a = f * 2^e with f in [0.5, 1): binary exponent e - 1 */
    int ex = e - 1 < -6 ? -6 : e - 1;
    double ulp = ldexp(1.0, ex - 3);
    double q = nearbyint(a / ulp) * ulp; /* default rounding mode: ties to even */
    if (q > 448) q = 448;
    return (real)copysign(q, (double)v);
}

/* per-row FP8 operand: y = s * e4m3(x / s) with s = amax(row) / 448 (a zero row stays zero) */
static void quant_rows(real *y, const real *x, int rows, int n) {
    for (int r = 0; r < rows; r++) {
        const real *xr = x + (size_t)r * n;
        real amax = 0;
        for (int i = 0; i < n; i++) if (fabs((double)xr[i]) > amax) amax = (real)fabs((double)xr[i]);
        real sc = amax > 0 ? amax / 448 : 1;
        for (int i = 0; i < n; i++) y[(size_t)r * n + i] = e4m3_round(xr[i] / sc) * sc;
    }
}

/* per-matrix FP8 operand, in place, one scale for all the listed pieces of one matrix */
static void quant_matrix(real **pieces, const size_t *sizes, int count) {
    real amax = 0;
    for (int c = 0; c < count; c++)
        for (size_t i = 0; i < sizes[c]; i++) if (fabs((double)pieces[c][i]) > amax) amax = (real)fabs((double)pieces[c][i]);
    real sc = amax > 0 ? amax / 448 : 1;
    for (int c = 0; c < count; c++)
        for (size_t i = 0; i < sizes[c]; i++) pieces[c][i] = e4m3_round(pieces[c][i] / sc) * sc;
}

/* operand of a per-beam-row product: the rows themselves, or their FP8 image in FP8 mode (into `tmp`) */
static const real *operand(int fp8, real *tmp, const real *x, int rows, int n) {
    if (!fp8) return x;
    quant_rows(tmp, x, rows, n);
    return tmp;
}

/* out[v] = z[v] - log(sum_u exp(z[u])) */
static void log_softmax(real *out, const real *z, int n) {
    real mx = z[0];
    for (int i = 1; i < n; i++) if (z[i] > mx) mx = z[i];
    real s = 0;
    for (int i = 0; i < n; i++) s += R_EXP(z[i] - mx);
    real lse = mx + R_LOG(s);
    for (int i = 0; i < n; i++) out[i] = z[i] - lse;
}

/* Multi-head attention.  q [nq,d], k,v [nk,d], heads are contiguous slices of
 * width dh = d/H.  Query i sees keys 0..nk-1, or, if causal, keys
 * 0..(nk-nq)+i.  out [nq,d] = heads concatenated. */
static void mha(real *out, const real *q, const real *k, const real *v, int nq, int nk, int d, int H, int causal) {
    int dh = d / H;
    real scale = 1 / R_SQRT((real)dh);
#pragma omp parallel for schedule(static) if (!omp_in_parallel() && nq >= 8)
    for (int i = 0; i < nq; i++) {
        real *p = (real *)malloc(sizeof(real) * (size_t)nk);
        int vis = causal ? (nk - nq) + i + 1 : nk;
        for (int h = 0; h < H; h++) {
            const real *qh = q + (size_t)i * d + h * dh;
            real mx = -INFINITY;
            for (int j = 0; j < vis; j++) {
                const real *kh = k + (size_t)j * d + h * dh;
                real s = 0;
#pragma omp simd reduction(+ : s)
                for (int c = 0; c < dh; c++) s += qh[c] * kh[c];
                p[j] = s * scale;
                if (p[j] > mx) mx = p[j];
            }
            real den = 0;
            for (int j = 0; j < vis; j++) { p[j] = R_EXP(p[j] - mx); den += p[j]; }
            real *oh = out + (size_t)i * d + h * dh;
            for (int c = 0; c < dh; c++) oh[c] = 0;
            for (int j = 0; j < vis; j++) {
                const real *vh = v + (size_t)j * d + h * dh;
                real w = p[j] / den;
                for (int c = 0; c < dh; c++) oh[c] += w * vh[c];
            }
        }
        free(p);
    }
}

/* Fuse(m, s) = W_f [ m * (W_g s) ; s ]   (section 3.2, gated projection) */
static void fuse(real *out, const real *m, const real *s, const real *w_g, const real *w_f, int d, int fp8) {
    real *cat = ralloc(2 * (size_t)d);
    linear(cat, s, w_g, 1, d, d);
    for (int i = 0; i < d; i++) cat[i] *= m[i];
    if (fp8) quant_rows(cat, cat, 1, d); /* the gated half meets the FP8 half of W_f; W_g s and W_f[:, d:] s depend on the token alone */
    for (int i = 0; i < d; i++) cat[d + i] = s[i];
    linear(out, cat, w_f, 1, 2 * d, d);
    free(cat);
}

/* Input state of the first autoregressive layer at one position: Fuse(m, s) with m the trunk output of that position
 * (eq. fuse), or, for the vanilla decoder, s + p with p the position embedding (then m IS p: no lazy layer ran). */
static void input_state(const orc_model *md, real *out, const real *m, const real *s) {
    if (md->vanilla) { for (int i = 0; i < md->d; i++) out[i] = s[i] + m[i]; return; }
    fuse(out, m, s, md->w_g, md->w_f, md->d, md->fp8);
}

/* One decoder layer over a sequence x [n,d] of decoder states (in place):
 * cross-attention over the context, causal self-attention over the n states,
 * feed-forward; each sub-layer is pre-normed and residual. */
static void layer_seq(const orc_model *m, int l, real *x, int n, const real *Kc, const real *Vc, int len) {
    const layer_r *w = &m->layers[l];
    int d = m->d, F = m->F;
    size_t nd = (size_t)n * d;
    real *a = ralloc(nd), *q = ralloc(nd), *k = ralloc(nd), *v = ralloc(nd), *o = ralloc(nd);
    real *f = ralloc((size_t)n * F);
    const int q8 = m->fp8 && l >= m->K; /* FP8 mode: the autoregressive layers' per-row products take FP8 operands */
    real *tq = ralloc((size_t)n * (F > d ? F : d));
    /* cross-attention */
    rmsnorm(a, x, w->ln_x, n, d, m->eps);
    linear(q, operand(q8, tq, a, n, d), w->wq_x, n, d, d);
    mha(o, q, Kc, Vc, n, len, d, m->H, 0);
    linear(a, operand(q8, tq, o, n, d), w->wo_x, n, d, d);
    for (size_t i = 0; i < nd; i++) x[i] += a[i];
    /* causal self-attention over the decoder states */
    rmsnorm(a, x, w->ln_s, n, d, m->eps);
    const real *as = operand(q8, tq, a, n, d);
    linear(q, as, w->wq_s, n, d, d);
    linear(k, as, w->wk_s, n, d, d);
    linear(v, as, w->wv_s, n, d, d);
    mha(o, q, k, v, n, n, d, m->H, 1);
    linear(a, operand(q8, tq, o, n, d), w->wo_s, n, d, d);
    for (size_t i = 0; i < nd; i++) x[i] += a[i];
    /* feed-forward */
    rmsnorm(a, x, w->ln_f, n, d, m->eps);
    linear(f, operand(q8, tq, a, n, d), w->w1, n, d, F);
    for (size_t i = 0; i < (size_t)n * F; i++) f[i] = silu(f[i]);
    linear(a, operand(q8, tq, f, n, F), w->w2, n, F, d);
    for (size_t i = 0; i < nd; i++) x[i] += a[i];
    free(a); free(q); free(k); free(v); free(o); free(f); free(tq);
}

/* classifier of level t (0-based): lp = log_softmax(W_t N_out(h) + bias_t) */
static void classify(const orc_model *m, int t, const real *h, real *lp) {
    int d = m->d, V = m->V[t];
    real *a = ralloc(d);
    rmsnorm(a, h, m->ln_out, 1, d, m->eps);
    if (m->fp8) quant_rows(a, a, 1, d);
    linear(lp, a, m->cls[t], 1, d, V);
    if (m->cls_bias[t]) for (int v = 0; v < V; v++) lp[v] += m->cls_bias[t][v];
    log_softmax(lp, lp, V);
    free(a);
}

/* embedding of the token that precedes 0-based level t: BOS for t = 0 */
static const real *prev_embedding(const orc_model *m, int t, const int32_t *tokens) {
    return t == 0 ? m->bos : m->emb[t - 1] + (size_t)tokens[t - 1] * m->d;
}

/* ------------------------------------------------------------------ */
/* model / request handles                                             */
/* ------------------------------------------------------------------ */
orc_model *orc_model_create(const orc_desc *ds, const orc_weights *w) {
    if (!ds || !w || ds->T < 1 || ds->T > ORC_MAX_LEVELS || ds->K < 0 || ds->K >= ds->L || ds->d % ds->H) return NULL;
    if (ds->vanilla && ds->K != 0) return NULL; /* the vanilla decoder has no lazy layer */
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->d = ds->d; m->H = ds->H; m->F = ds->F; m->L = ds->L; m->K = ds->K; m->T = ds->T; m->eps = (real)ds->eps;
    m->fp8 = ds->fp8 != 0;
    m->vanilla = ds->vanilla != 0;
    size_t d = ds->d, F = ds->F;
    for (int t = 0; t < m->T; t++) m->V[t] = ds->V[t];
    m->pos = rcopy_f(w->pos, m->T * d);
    m->bos = rcopy_f(w->bos, d);
    for (int t = 0; t + 1 < m->T; t++) m->emb[t] = rcopy_f(w->emb[t], (size_t)m->V[t] * d);
    if (!m->vanilla) {
        m->w_g = rcopy_f(w->w_g, d * d);
        m->w_f = rcopy_f(w->w_f, d * 2 * d);
    }
    m->ln_out = rcopy_f(w->ln_out, d);
    for (int t = 0; t < m->T; t++) {
        m->cls[t] = rcopy_f(w->cls[t], (size_t)m->V[t] * d);
        m->cls_bias[t] = (w->cls_bias && w->cls_bias[t]) ? rcopy_f(w->cls_bias[t], m->V[t]) : NULL;
    }
    m->layers = (layer_r *)calloc(m->L, sizeof(layer_r));
    for (int l = 0; l < m->L; l++) {
        const orc_layer_w *s = &w->layers[l];
        layer_r *r = &m->layers[l];
        r->ln_x = rcopy_f(s->ln_x, d); r->wq_x = rcopy_f(s->wq_x, d * d); r->wk_x = rcopy_f(s->wk_x, d * d);
        r->wv_x = rcopy_f(s->wv_x, d * d); r->wo_x = rcopy_f(s->wo_x, d * d);
        r->ln_s = rcopy_f(s->ln_s, d); r->wq_s = rcopy_f(s->wq_s, d * d); r->wk_s = rcopy_f(s->wk_s, d * d);
        r->wv_s = rcopy_f(s->wv_s, d * d); r->wo_s = rcopy_f(s->wo_s, d * d);
        r->ln_f = rcopy_f(s->ln_f, d); r->w1 = rcopy_f(s->w1, F * d); r->w2 = rcopy_f(s->w2, d * F);
    }
    if (m->fp8) { /* the weights of the per-beam-row products move onto the FP8 grid once, here */
        const size_t dd = d * d, dF = d * F;
        for (int l = m->K; l < m->L; l++) {
            layer_r *r = &m->layers[l];
            real *qkv[3] = {r->wq_s, r->wk_s, r->wv_s};
            const size_t qkv_n[3] = {dd, dd, dd};
            quant_matrix(&r->wq_x, &dd, 1); quant_matrix(&r->wo_x, &dd, 1);
            quant_matrix(qkv, qkv_n, 3); quant_matrix(&r->wo_s, &dd, 1);
            quant_matrix(&r->w1, &dF, 1); quant_matrix(&r->w2, &dF, 1);
        }
        for (int t = 0; t < m->T; t++) { const size_t n = (size_t)m->V[t] * d; quant_matrix(&m->cls[t], &n, 1); }
        if (!m->vanilla) { /* W_f[:, :d]: the first d entries of each of its d rows */
            real *half = ralloc(dd);
            for (size_t o = 0; o < d; o++) memcpy(half + o * d, m->w_f + o * 2 * d, d * sizeof(real));
            quant_matrix(&half, &dd, 1);
            for (size_t o = 0; o < d; o++) memcpy(m->w_f + o * 2 * d, half + o * d, d * sizeof(real));
            free(half);
        }
    }
    return m;
}

void orc_model_free(orc_model *m) {
    if (!m) return;
    free(m->pos); free(m->bos); free(m->w_g); free(m->w_f); free(m->ln_out);
    for (int t = 0; t < ORC_MAX_LEVELS; t++) { free(m->emb[t]); free(m->cls[t]); free(m->cls_bias[t]); }
    for (int l = 0; l < m->L; l++) {
        layer_r *r = &m->layers[l];
        free(r->ln_x); free(r->wq_x); free(r->wk_x); free(r->wv_x); free(r->wo_x);
        free(r->ln_s); free(r->wq_s); free(r->wk_s); free(r->wv_s); free(r->wo_s);
        free(r->ln_f); free(r->w1); free(r->w2);
    }
    free(m->layers);
    free(m);
}

/* X [S,d] float; only rows 0..len-1 are read (padding never enters). */
orc_req *orc_req_create(const orc_model *m, const float *X, int len) {
    if (!m || !X || len < 1) return NULL;
    orc_req *rq = (orc_req *)calloc(1, sizeof(orc_req));
    rq->len = len; rq->L = m->L;
    rq->Kc = (real **)calloc(m->L, sizeof(real *));
    rq->Vc = (real **)calloc(m->L, sizeof(real *));
    real *x = rcopy_f(X, (size_t)len * m->d);
    for (int l = 0; l < m->L; l++) {
        rq->Kc[l] = ralloc((size_t)len * m->d);
        rq->Vc[l] = ralloc((size_t)len * m->d);
        linear(rq->Kc[l], x, m->layers[l].wk_x, len, m->d, m->d);
        linear(rq->Vc[l], x, m->layers[l].wv_x, len, m->d, m->d);
    }
    free(x);
    return rq;
}

void orc_req_free(orc_req *rq) {
    if (!rq) return;
    for (int l = 0; l < rq->L; l++) { free(rq->Kc[l]); free(rq->Vc[l]); }
    free(rq->Kc); free(rq->Vc); free(rq);
}

/* ------------------------------------------------------------------ */
/* the definition: teacher-forced forward over a prefix                */
/* ------------------------------------------------------------------ */
/* Levels 1..t (t positions).  tokens[0..t-2] are s_1..s_{t-1}.  Writes the
 * log-probability distribution of level t to lp_last [V_t] and, if lp_all is
 * not NULL, the distributions of levels 1..t back to back. */
void orc_forward_seq(const orc_model *m, const orc_req *rq, int t, const int32_t *tokens, double *lp_last, double *lp_all) {
    int d = m->d;
    real *x = ralloc((size_t)t * d);
    /* trunk (eq. trunk): m^(0)_tau = p_tau, K lazy layers, no token enters */
    memcpy(x, m->pos, sizeof(real) * (size_t)t * d);
    for (int l = 0; l < m->K; l++) layer_seq(m, l, x, t, rq->Kc[l], rq->Vc[l], rq->len);
    /* late injection (eq. fuse); the vanilla decoder adds the token embedding to the position embedding instead */
    real *h = ralloc((size_t)t * d);
    for (int p = 0; p < t; p++) input_state(m, h + (size_t)p * d, x + (size_t)p * d, prev_embedding(m, p, tokens));
    /* autoregressive head (eq. head) */
    for (int l = m->K; l < m->L; l++) layer_seq(m, l, h, t, rq->Kc[l], rq->Vc[l], rq->len);
    size_t off = 0;
    for (int p = 0; p < t; p++) {
        if (!lp_all && p != t - 1) continue;
        int V = m->V[p];
        real *lp = ralloc(V);
        classify(m, p, h + (size_t)p * d, lp);
        if (lp_all) { for (int v = 0; v < V; v++) lp_all[off + v] = (double)lp[v]; off += V; }
        if (p == t - 1 && lp_last) for (int v = 0; v < V; v++) lp_last[v] = (double)lp[v];
        free(lp);
    }
    free(x); free(h);
}

/* A second decoder written without any trunk/head split: the step-tau input
 * is Fuse(p_tau, s_{tau-1}) and all L layers run autoregressively.  This is
 * what lazy depth 0 must reproduce. */
void orc_plain_ar_seq(const orc_model *m, const orc_req *rq, int t, const int32_t *tokens, double *lp_last) {
    int d = m->d;
    real *h = ralloc((size_t)t * d);
    for (int p = 0; p < t; p++) fuse(h + (size_t)p * d, m->pos + (size_t)p * d, prev_embedding(m, p, tokens), m->w_g, m->w_f, d, m->fp8);
    for (int l = 0; l < m->L; l++) layer_seq(m, l, h, t, rq->Kc[l], rq->Vc[l], rq->len);
    real *lp = ralloc(m->V[t - 1]);
    classify(m, t - 1, h + (size_t)(t - 1) * d, lp);
    for (int v = 0; v < m->V[t - 1]; v++) lp_last[v] = (double)lp[v];
    free(lp); free(h);
}

/* The vanilla autoregressive decoder (section 3.2, "Vanilla Autoregressive Decoding"), written on its own: the state that
 * enters the first layer at step tau is s_{tau-1} + p_tau, all L layers are ordinary decoder layers over the tau states,
 * the level's classifier follows.  A model created with vanilla != 0 must reproduce it through orc_forward_seq. */
void orc_vanilla_ar_seq(const orc_model *m, const orc_req *rq, int t, const int32_t *tokens, double *lp_last) {
    int d = m->d;
    real *h = ralloc((size_t)t * d);
    for (int p = 0; p < t; p++) {
        const real *s = prev_embedding(m, p, tokens);
        for (int i = 0; i < d; i++) h[(size_t)p * d + i] = s[i] + m->pos[(size_t)p * d + i];
    }
    for (int l = 0; l < m->L; l++) layer_seq(m, l, h, t, rq->Kc[l], rq->Vc[l], rq->len);
    real *lp = ralloc(m->V[t - 1]);
    classify(m, t - 1, h + (size_t)(t - 1) * d, lp);
    for (int v = 0; v < m->V[t - 1]; v++) lp_last[v] = (double)lp[v];
    free(lp); free(h);
}

/* ------------------------------------------------------------------ */
/* selection                                                           */
/* ------------------------------------------------------------------ */
typedef struct { real score; int64_t flat; } cand;

static int cand_cmp(const void *a, const void *b) {
    const cand *x = (const cand *)a, *y = (const cand *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->flat > y->flat) - (x->flat < y->flat);
}

/* full sort of all n candidates, descending score, ties by ascending flat index */
static void sort_candidates(cand *c, size_t n) { qsort(c, n, sizeof(cand), cand_cmp); }

/* TopK Pre-Cut (appendix A.2): per row keep the min(k,V) best, then the global
 * k best of the survivors.  score [n,V]; writes k (flat index, score). */
static void topk_precut(const real *score, int n, int V, int k, int64_t *out_flat, real *out_score) {
    int m = k < V ? k : V;
    cand *stage = (cand *)malloc(sizeof(cand) * (size_t)n * m);
    cand *row = (cand *)malloc(sizeof(cand) * (size_t)V);
    for (int i = 0; i < n; i++) {
        for (int v = 0; v < V; v++) { row[v].score = score[(size_t)i * V + v]; row[v].flat = (int64_t)i * V + v; }
        sort_candidates(row, V);
        memcpy(stage + (size_t)i * m, row, sizeof(cand) * m);
    }
    sort_candidates(stage, (size_t)n * m);
    for (int j = 0; j < k; j++) { out_flat[j] = stage[j].flat; out_score[j] = stage[j].score; }
    free(stage); free(row);
}

static void topk_global(const real *score, int n, int V, int k, int64_t *out_flat, real *out_score) {
    size_t N = (size_t)n * V;
    cand *c = (cand *)malloc(sizeof(cand) * N);
    for (size_t i = 0; i < N; i++) { c[i].score = score[i]; c[i].flat = (int64_t)i; }
    sort_candidates(c, N);
    for (int j = 0; j < k; j++) { out_flat[j] = c[j].flat; out_score[j] = c[j].score; }
    free(c);
}

/* ------------------------------------------------------------------ */
/* beam search by definition                                           */
/* ------------------------------------------------------------------ */
/* trace arrays (may be NULL): per level t, b_t entries at offset sum_{u<t} b_u */
static int check_beams(const orc_model *m, const int32_t *beam) {
    int64_t n = 1;
    for (int t = 0; t < m->T; t++) {
        if (beam[t] < 1 || (int64_t)beam[t] > n * m->V[t]) return -1;
        n = beam[t];
    }
    return 0;
}

int orc_decode_plain(const orc_model *m, const orc_req *rq, const int32_t *beam, int32_t *out_sid, double *out_logprob,
                     int32_t *tr_parent, int32_t *tr_tok, double *tr_score, int use_precut) {
    if (check_beams(m, beam)) return -1;
    int T = m->T, n = 1;
    int32_t *paths = (int32_t *)calloc((size_t)T, sizeof(int32_t)); /* [n,T] */
    real *cum = ralloc(1);
    size_t tr_off = 0;
    for (int t = 0; t < T; t++) {
        int V = m->V[t], k = beam[t];
        real *score = ralloc((size_t)n * V);
        double *lp = (double *)malloc(sizeof(double) * V);
        for (int i = 0; i < n; i++) {
            orc_forward_seq(m, rq, t + 1, paths + (size_t)i * T, lp, NULL);
            for (int v = 0; v < V; v++) score[(size_t)i * V + v] = cum[i] + (real)lp[v];
        }
        int64_t *flat = (int64_t *)malloc(sizeof(int64_t) * k);
        real *ks = ralloc(k);
        if (use_precut) topk_precut(score, n, V, k, flat, ks); else topk_global(score, n, V, k, flat, ks);
        int32_t *npaths = (int32_t *)calloc((size_t)k * T, sizeof(int32_t));
        for (int j = 0; j < k; j++) {
            int par = (int)(flat[j] / V), tok = (int)(flat[j] % V);
            memcpy(npaths + (size_t)j * T, paths + (size_t)par * T, sizeof(int32_t) * T);
            npaths[(size_t)j * T + t] = tok;
            if (tr_parent) tr_parent[tr_off + j] = par;
            if (tr_tok) tr_tok[tr_off + j] = tok;
            if (tr_score) tr_score[tr_off + j] = (double)ks[j];
        }
        tr_off += k;
        free(paths); free(cum); free(score); free(lp); free(flat);
        paths = npaths; cum = ks; n = k;
    }
    for (int j = 0; j < n; j++) {
        for (int t = 0; t < T; t++) out_sid[(size_t)j * T + t] = paths[(size_t)j * T + t];
        out_logprob[j] = (double)cum[j];
    }
    free(paths); free(cum);
    return 0;
}

/* ------------------------------------------------------------------ */
/* beam search with the lossless accelerations                         */
/* ------------------------------------------------------------------ */
/* One autoregressive layer for a single new position `p` (0-based) of one
 * beam path.  selfK/selfV [T,d] hold this layer's self-attention keys/values
 * of the path's positions 0..p-1; position p is appended. */
static void layer_step(const orc_model *m, int l, real *x, int p, const real *Kc, const real *Vc, int len, real *selfK, real *selfV) {
    const layer_r *w = &m->layers[l];
    int d = m->d, F = m->F;
    real *a = ralloc(d), *q = ralloc(d), *o = ralloc(d), *f = ralloc(F);
    const int q8 = m->fp8 && l >= m->K;
    real *tq = ralloc(F > d ? F : d);
    rmsnorm(a, x, w->ln_x, 1, d, m->eps);
    linear(q, operand(q8, tq, a, 1, d), w->wq_x, 1, d, d);
    mha(o, q, Kc, Vc, 1, len, d, m->H, 0);
    linear(a, operand(q8, tq, o, 1, d), w->wo_x, 1, d, d);
    for (int i = 0; i < d; i++) x[i] += a[i];
    rmsnorm(a, x, w->ln_s, 1, d, m->eps);
    const real *as = operand(q8, tq, a, 1, d);
    linear(q, as, w->wq_s, 1, d, d);
    linear(selfK + (size_t)p * d, as, w->wk_s, 1, d, d);
    linear(selfV + (size_t)p * d, as, w->wv_s, 1, d, d);
    mha(o, q, selfK, selfV, 1, p + 1, d, m->H, 0);
    linear(a, operand(q8, tq, o, 1, d), w->wo_s, 1, d, d);
    for (int i = 0; i < d; i++) x[i] += a[i];
    rmsnorm(a, x, w->ln_f, 1, d, m->eps);
    linear(f, operand(q8, tq, a, 1, d), w->w1, 1, d, F);
    for (int i = 0; i < F; i++) f[i] = silu(f[i]);
    linear(a, operand(q8, tq, f, 1, F), w->w2, 1, F, d);
    for (int i = 0; i < d; i++) x[i] += a[i];
    free(a); free(q); free(o); free(f); free(tq);
}

int orc_decode_cached(const orc_model *m, const orc_req *rq, const int32_t *beam, int32_t *out_sid, double *out_logprob,
                      int32_t *tr_parent, int32_t *tr_tok, double *tr_score) {
    if (check_beams(m, beam)) return -1;
    int T = m->T, d = m->d, A = m->L - m->K, n = 1;
    /* trunk once per request, for all levels at once, shared by every beam */
    real *trunk = ralloc((size_t)T * d);
    memcpy(trunk, m->pos, sizeof(real) * (size_t)T * d);
    for (int l = 0; l < m->K; l++) layer_seq(m, l, trunk, T, rq->Kc[l], rq->Vc[l], rq->len);

    size_t kvsz = (size_t)A * T * d; /* per beam: [A][T][d] keys, same for values */
    int32_t *paths = (int32_t *)calloc((size_t)T, sizeof(int32_t));
    real *cum = ralloc(1), *sK = ralloc(kvsz), *sV = ralloc(kvsz);
    size_t tr_off = 0;
    for (int t = 0; t < T; t++) {
        int V = m->V[t], k = beam[t];
        real *score = ralloc((size_t)n * V);
#pragma omp parallel for schedule(dynamic) if (!omp_in_parallel() && n >= 4)
        for (int i = 0; i < n; i++) {
            real *h = ralloc(d), *lp = ralloc(V);
            input_state(m, h, trunk + (size_t)t * d, prev_embedding(m, t, paths + (size_t)i * T));
            for (int a = 0; a < A; a++) {
                int l = m->K + a;
                layer_step(m, l, h, t, rq->Kc[l], rq->Vc[l], rq->len, sK + i * kvsz + (size_t)a * T * d, sV + i * kvsz + (size_t)a * T * d);
            }
            classify(m, t, h, lp);
            for (int v = 0; v < V; v++) score[(size_t)i * V + v] = cum[i] + lp[v];
            free(h); free(lp);
        }
        int64_t *flat = (int64_t *)malloc(sizeof(int64_t) * k);
        real *ks = ralloc(k);
        topk_global(score, n, V, k, flat, ks);
        int32_t *npaths = (int32_t *)calloc((size_t)k * T, sizeof(int32_t));
        real *nK = ralloc(k * kvsz), *nV = ralloc(k * kvsz);
        for (int j = 0; j < k; j++) {
            int par = (int)(flat[j] / V), tok = (int)(flat[j] % V);
            memcpy(npaths + (size_t)j * T, paths + (size_t)par * T, sizeof(int32_t) * T);
            npaths[(size_t)j * T + t] = tok;
            memcpy(nK + j * kvsz, sK + par * kvsz, sizeof(real) * kvsz);
            memcpy(nV + j * kvsz, sV + par * kvsz, sizeof(real) * kvsz);
            if (tr_parent) tr_parent[tr_off + j] = par;
            if (tr_tok) tr_tok[tr_off + j] = tok;
            if (tr_score) tr_score[tr_off + j] = (double)ks[j];
        }
        tr_off += k;
        free(paths); free(cum); free(sK); free(sV); free(score); free(flat);
        paths = npaths; cum = ks; sK = nK; sV = nV; n = k;
    }
    for (int j = 0; j < n; j++) {
        for (int t = 0; t < T; t++) out_sid[(size_t)j * T + t] = paths[(size_t)j * T + t];
        out_logprob[j] = (double)cum[j];
    }
    free(paths); free(cum); free(sK); free(sV); free(trunk);
    return 0;
}

/* Batch driver: requests are independent; one request per thread when the
 * batch is large enough, otherwise the per-request code parallelises over
 * rows.  X [B,S,d]; ctx_len [B] or NULL (= S).  mode 0 = cached, 1 = plain
 * (global sort), 2 = plain with pre-cut.  Trace arrays are [B, sum_t b_t]. */
int orc_decode_batch(const orc_model *m, const float *X, const int32_t *ctx_len, int B, int S, const int32_t *beam,
                     int32_t *out_sid, double *out_logprob, int32_t *tr_parent, int32_t *tr_tok, double *tr_score, int mode) {
    if (!m || !X || check_beams(m, beam)) return -1;
    int T = m->T, bT = beam[T - 1];
    size_t tr_n = 0;
    for (int t = 0; t < T; t++) tr_n += beam[t];
    int rc = 0, nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic) if (B >= nthreads && nthreads > 1)
    for (int r = 0; r < B; r++) {
        int len = ctx_len ? ctx_len[r] : S;
        if (len < 1) len = 1;
        if (len > S) len = S;
        orc_req *rq = orc_req_create(m, X + (size_t)r * S * m->d, len);
        int32_t *tp = tr_parent ? tr_parent + r * tr_n : NULL, *tt = tr_tok ? tr_tok + r * tr_n : NULL;
        double *ts = tr_score ? tr_score + r * tr_n : NULL;
        int e = (mode == 0) ? orc_decode_cached(m, rq, beam, out_sid + (size_t)r * bT * T, out_logprob + (size_t)r * bT, tp, tt, ts)
                            : orc_decode_plain(m, rq, beam, out_sid + (size_t)r * bT * T, out_logprob + (size_t)r * bT, tp, tt, ts, mode == 2);
        if (e) rc = e;
        orc_req_free(rq);
    }
    return rc;
}

/* Teacher-forced scores of the candidates that follow given prefixes: for n
 * prefixes of t-1 tokens each ([n, t-1], level t is 1-based), writes the
 * cumulative log-probability of each prefix (out_cum [n]) and the level-t
 * log-probability distribution after it (out_lp [n, V_t]). */
void orc_prefix_dists(const orc_model *m, const orc_req *rq, int t, int n, const int32_t *prefixes, double *out_cum, double *out_lp) {
    int V = m->V[t - 1];
    size_t all = 0;
    for (int p = 0; p < t; p++) all += m->V[p];
#pragma omp parallel for schedule(dynamic) if (!omp_in_parallel() && n >= 2)
    for (int i = 0; i < n; i++) {
        const int32_t *tok = prefixes + (size_t)i * (t - 1);
        double *buf = (double *)malloc(sizeof(double) * all);
        orc_forward_seq(m, rq, t, tok, out_lp + (size_t)i * V, buf);
        double c = 0; size_t off = 0;
        for (int p = 0; p + 1 < t; p++) { c += buf[off + tok[p]]; off += m->V[p]; }
        out_cum[i] = c;
        free(buf);
    }
}

/* ------------------------------------------------------------------ */
/* primitive exports, so tests can pin each one against library code   */
/* ------------------------------------------------------------------ */
static real *from_d(const double *x, size_t n) { real *p = ralloc(n); for (size_t i = 0; i < n; i++) p[i] = (real)x[i]; return p; }
static void to_d(double *y, const real *x, size_t n) { for (size_t i = 0; i < n; i++) y[i] = (double)x[i]; }

void orc_prim_linear(double *y, const double *x, const double *W, int rows, int in, int out) {
    real *xr = from_d(x, (size_t)rows * in), *wr = from_d(W, (size_t)in * out), *yr = ralloc((size_t)rows * out);
    linear(yr, xr, wr, rows, in, out); to_d(y, yr, (size_t)rows * out); free(xr); free(wr); free(yr);
}
void orc_prim_rmsnorm(double *y, const double *x, const double *g, int rows, int d, double eps) {
    real *xr = from_d(x, (size_t)rows * d), *gr = from_d(g, d), *yr = ralloc((size_t)rows * d);
    rmsnorm(yr, xr, gr, rows, d, (real)eps); to_d(y, yr, (size_t)rows * d); free(xr); free(gr); free(yr);
}
void orc_prim_silu(double *y, const double *x, int n) { for (int i = 0; i < n; i++) y[i] = (double)silu((real)x[i]); }
void orc_prim_log_softmax(double *y, const double *z, int n) {
    real *zr = from_d(z, n), *yr = ralloc(n); log_softmax(yr, zr, n); to_d(y, yr, n); free(zr); free(yr);
}
void orc_prim_mha(double *out, const double *q, const double *k, const double *v, int nq, int nk, int d, int H, int causal) {
    real *qr = from_d(q, (size_t)nq * d), *kr = from_d(k, (size_t)nk * d), *vr = from_d(v, (size_t)nk * d), *o = ralloc((size_t)nq * d);
    mha(o, qr, kr, vr, nq, nk, d, H, causal); to_d(out, o, (size_t)nq * d); free(qr); free(kr); free(vr); free(o);
}
void orc_prim_fuse(double *out, const double *mvec, const double *s, const double *w_g, const double *w_f, int d) {
    real *mr = from_d(mvec, d), *sr = from_d(s, d), *g = from_d(w_g, (size_t)d * d), *f = from_d(w_f, (size_t)2 * d * d), *o = ralloc(d);
    fuse(o, mr, sr, g, f, d, 0); to_d(out, o, d); free(mr); free(sr); free(g); free(f); free(o);
}
/* mode 0 global full sort, 1 pre-cut */
void orc_prim_topk(const double *score, int n, int V, int k, int64_t *out_flat, double *out_score, int precut) {
    real *s = from_d(score, (size_t)n * V), *ks = ralloc(k);
    if (precut) topk_precut(s, n, V, k, out_flat, ks); else topk_global(s, n, V, k, out_flat, ks);
    to_d(out_score, ks, k); free(s); free(ks);
}
/* one decoder layer of the model over a sequence x [n,d] (in place, double) */
void orc_prim_layer_seq(const orc_model *m, const orc_req *rq, int l, double *x, int n) {
    real *xr = from_d(x, (size_t)n * m->d);
    layer_seq(m, l, xr, n, rq->Kc[l], rq->Vc[l], rq->len); to_d(x, xr, (size_t)n * m->d); free(xr);
}
void orc_prim_e4m3(double *y, const double *x, int n) { for (int i = 0; i < n; i++) y[i] = (double)e4m3_round((real)x[i]); }
void orc_prim_quant_rows(double *y, const double *x, int rows, int n) {
    real *xr = from_d(x, (size_t)rows * n), *yr = ralloc((size_t)rows * n);
    quant_rows(yr, xr, rows, n); to_d(y, yr, (size_t)rows * n); free(xr); free(yr);
}
int orc_real_bytes(void) { return (int)sizeof(real); }
