/*
 * gr4ad.h -- C ABI of the MI355X LazyAR beam-decode library (libgr4ad.so).
 *
 * The library decodes, for a batch of user requests, the top multi-level
 * semantic-ID (UA-SID) candidates y = (s_1..s_T), s_t in V_t (paper section 3.1,
 * UA-SID definition) with the LazyAR decoder (section 3.2: eq. trunk, eq. fuse,
 * eq. head, per-level classifier softmax) under beam search with one beam width
 * per level (section 4.2, Dynamic Beam Width), against a context memory
 * X in R^{S x d} that is already encoded (section 3.2, first paragraph).
 *
 * Conventions
 *   - Pointers named *_dev are device (HBM) pointers; everything else is host memory.
 *   - Matrices are row-major [out, in]: y = W x.  No linear layer has a bias.
 *   - dtype selects the storage type of weights, context and activations
 *     (float32 or bfloat16 bit patterns); accumulation, softmax, log-softmax and
 *     beam scores are always float32.
 *   - Every function returns a gr4ad_status (0 = ok, negative = error) and never
 *     throws or aborts.  gr4ad_last_error gives a readable message.
 *   - Same inputs give bit-identical outputs from run to run.  Candidates with
 *     exactly equal scores are ordered by ascending flat index i*V_t + v
 *     (i = parent beam, v = token).
 */
#ifndef GR4AD_H
#define GR4AD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GR4AD_OK = 0,
    GR4AD_EINVAL = -1,       /* bad argument (shape, range, null pointer) */
    GR4AD_EUNSUPPORTED = -2, /* valid but outside what the kernels cover */
    GR4AD_EWORKSPACE = -3,   /* workspace_dev too small or misaligned */
    GR4AD_EHIP = -4,         /* a HIP runtime call failed */
    GR4AD_ENOMEM = -5        /* device or host allocation failed */
} gr4ad_status;

typedef enum { GR4AD_F32 = 0, GR4AD_BF16 = 1 } gr4ad_dtype;

#define GR4AD_MAX_LEVELS 8     /* T <= 8 */
#define GR4AD_MAX_BEAM 4096    /* b_t <= 4096 */
#define GR4AD_MAX_CODEBOOK 16384 /* V_t <= 16384 */

/* Model shape (section 3.2: L decoder layers, the first K lazy; section 3.1: T levels, |V_t|). */
typedef struct {
    int32_t d_model;         /* d, multiple of 8 */
    int32_t n_heads;         /* H, d % H == 0, head width d/H in {16, 32, 64, 128} */
    int32_t d_ffn;           /* F, multiple of 8 */
    int32_t n_layers;        /* L >= 1 */
    int32_t n_lazy;          /* K, 0 <= K < L; K = 0 makes every layer autoregressive */
    int32_t n_levels;        /* T, 1..GR4AD_MAX_LEVELS */
    const int32_t *codebook; /* host [T]: V_t */
    const int32_t *max_beam; /* host [T]: upper bound of b_t accepted by decode_batch */
    int32_t max_batch;       /* upper bound of B */
    int32_t max_ctx;         /* upper bound of S */
    gr4ad_dtype dtype;
    float rms_eps;           /* epsilon inside every RMSNorm */
    int32_t n_value_buckets; /* V_e: size of the eCPM-token vocabulary of the value step (section 3.3), 0 = no value step;
                              * with a value step T <= GR4AD_MAX_LEVELS - 1 */
    int32_t fp8_gemm;        /* != 0: low-precision inference (appendix A.2).  dtype must be GR4AD_BF16; weights are still
                              * handed over in bf16.  The matrix products that run once per beam row - the projections of the
                              * autoregressive layers except the context key/value projections, the W_f[:, :d] half of Fuse and
                              * the classifiers - take both operands as OCP E4M3 bytes with float32 accumulation: init
                              * quantises those weights with one scale amax/448 per matrix (the three self-attention input
                              * projections count as one matrix), decode quantises every activation row with its own scale
                              * amax(row)/448.  Everything else (lazy layers, attention, norms, softmax, scores) is unchanged. */
    int32_t vanilla_input;   /* != 0: the vanilla autoregressive decoder LazyAR is compared against (section 3.2, "Vanilla
                              * Autoregressive Decoding"): the state entering the first layer at level t is s_{t-1} + p_t (embedding of
                              * the previous token, BOS at t = 1, plus the position embedding), all L layers run per beam and level.
                              * n_lazy must be 0; w_g_dev and w_f_dev are not read and may be NULL. */
} gr4ad_model_desc;

/* One decoder layer (section 3.2: cross-attention over X, self-attention over
 * decoder states, feed-forward, each pre-normed).  All device pointers. */
typedef struct {
    const void *ln_x, *wq_x, *wk_x, *wv_x, *wo_x; /* [d], 4 x [d,d]; wk_x/wv_x act on raw X */
    const void *ln_s, *wq_s, *wk_s, *wv_s, *wo_s; /* [d], 4 x [d,d] */
    const void *ln_f, *w1, *w2;                   /* [d], [F,d], [d,F]; FFN = w2 * SiLU(w1 * x) */
} gr4ad_layer_weights;

/* All parameters.  The struct and the pointer arrays are host memory; the
 * tensors they point to are device memory of the model's dtype (cls_bias: float32). */
typedef struct {
    const void *pos_dev;                /* [T,d]  position embeddings p_t (trunk input, eq. trunk) */
    const void *bos_dev;                /* [d]    s_0 = BOS embedding */
    const void *const *emb_dev;         /* host [T-1] -> [V_t,d]: embedding of s_t, t = 1..T-1 */
    const void *w_g_dev;                /* [d,d]  gate of Fuse (eq. fuse) */
    const void *w_f_dev;                /* [d,2d] projection of Fuse, acting on [m*(W_g s) ; s] */
    const gr4ad_layer_weights *layers;  /* host [L] */
    const void *ln_out_dev;             /* [d]    gain of the final RMSNorm */
    const void *const *cls_dev;         /* host [T] -> [V_t,d]: classifier W_t */
    const float *const *cls_bias_dev;   /* NULL, or host [T] -> (NULL | [V_t] float32 logit bias) */
    /* value step (only read when n_value_buckets > 0): the eCPM token is one more prediction step after s_T */
    const void *value_pos_dev;          /* [d]      position embedding p_{T+1} */
    const void *value_emb_dev;          /* [V_T,d]  embedding of s_T */
    const void *value_cls_dev;          /* [V_e,d]  classifier over the eCPM buckets */
    const float *value_bias_dev;        /* NULL or [V_e] float32 logit bias */
} gr4ad_weights;

typedef struct gr4ad_decoder gr4ad_decoder;

/*
 * gr4ad_decode_init -- validate the description, copy and re-pack the weights
 * into library-owned device memory and precompute the per-token Fuse tables
 * (eq. fuse is linear in the token embedding: W_g s and the token half of
 * W_f s are looked up per token at decode time).
 * The caller may release its weight buffers afterwards.  On failure *out is
 * left untouched.  Uses the current HIP device; synchronises it once.
 * Errors: EINVAL (null pointer, d % H != 0, K outside [0,L), T outside
 * [1,8], non-positive sizes, vanilla_input with K > 0), EUNSUPPORTED (head width, beam or codebook
 * beyond the limits above), ENOMEM, EHIP.
 */
int gr4ad_decode_init(const gr4ad_model_desc *desc, const gr4ad_weights *weights, gr4ad_decoder **out);

/*
 * gr4ad_decode_workspace_bytes -- bytes of device workspace decode_batch needs
 * for B requests of S context tokens with beam widths beam[T] (host array).
 * Returns 0 if the arguments are invalid for this decoder.
 */
size_t gr4ad_decode_workspace_bytes(const gr4ad_decoder *dec, int32_t B, int32_t S, const int32_t *beam);

/*
 * gr4ad_decode_batch -- one pass of the whole hot path for B requests:
 * context K/V projection, lazy pass (once per request, all levels, no beam
 * dimension), then per level: Fuse, the L-K autoregressive layers with
 * beam-shared cross-attention, classifier, log-softmax + cumulative score +
 * top-b_t selection, reorder of the surviving beams' self-attention K/V.
 *
 *   ctx_dev        [B,S,d] dtype; rows >= ctx_len[b] are padding and never influence results
 *   ctx_len_dev    [B] int32 valid lengths, clamped to [1,S] on the device; NULL = all S
 *   beam           host [T]: b_t of THIS call (section 4.2: the schedule may change per call);
 *                  1 <= b_t <= max_beam[t] and b_t <= b_{t-1} * V_t (b_0 = 1)
 *   workspace_dev  caller-owned scratch, 256-byte aligned, >= workspace_bytes(B,S,beam)
 *   out_sid_dev    [B, b_T, T] int32: the b_T surviving SIDs per request, best first
 *   out_logprob_dev[B, b_T] float32: their log-probabilities, non-increasing
 *   hip_stream     hipStream_t (NULL = default stream).  The call only enqueues work:
 *                  outputs are valid once the stream has been synchronised.
 *
 * Calls on one decoder must not overlap (they share the decoder's tables and
 * the caller's workspace).  Errors: EINVAL, EWORKSPACE, EHIP.
 */
int gr4ad_decode_batch(gr4ad_decoder *dec, const void *ctx_dev, const int32_t *ctx_len_dev, int32_t B, int32_t S,
                       const int32_t *beam, void *workspace_dev, size_t workspace_bytes, int32_t *out_sid_dev,
                       float *out_logprob_dev, void *hip_stream);

/*
 * gr4ad_decode_set_trace -- optional per-level survivor record for tests.
 * Each argument is NULL or a host array [T] of device pointers [B, b_t]
 * (parent beam index, token, cumulative score of the survivors of level t);
 * the arrays are copied, the device buffers stay caller-owned and are written
 * by every later decode_batch call.  Pass three NULLs to switch it off.
 */
int gr4ad_decode_set_trace(gr4ad_decoder *dec, int32_t *const *parent_dev, int32_t *const *tok_dev, float *const *score_dev);

/*
 * gr4ad_decode_set_value_output -- eCPM-token step (section 3.3, "ECPM-Aware
 * Token Prediction": one more prediction step after the SID, used to re-rank
 * the generated SIDs).  With a buffer set, every later decode_batch call runs
 * that step for the b_T surviving beams of each request - Fuse with s_T, the
 * autoregressive layers at position T+1, final norm, value classifier - with no
 * beam expansion and writes log p(v | y, X):
 *   out_value_logprob_dev  [B, b_T, V_e] float32, rows in the order of out_sid_dev.
 * NULL switches the step off again (its workspace stays part of
 * workspace_bytes).  EINVAL if the model has no value step.
 */
int gr4ad_decode_set_value_output(gr4ad_decoder *dec, float *out_value_logprob_dev);

/* gr4ad_decode_free -- release everything init allocated.  NULL is a no-op. */
void gr4ad_decode_free(gr4ad_decoder *dec);

/* Static description of a status code. */
const char *gr4ad_strerror(int status);

/* Message of the last failing call on this decoder ("" if none).  With
 * dec == NULL: the last failure on this thread of gr4ad_decode_init or of an
 * entry point that takes no decoder (gr4ad_op_select_static). */
const char *gr4ad_last_error(const gr4ad_decoder *dec);

/*
 * Single-operation entry points (device pointers, enqueue on hip_stream).
 * They run the same kernels decode_batch uses, so each can be checked and
 * timed on its own.  dtype as above.  Return a gr4ad_status.
 */

/* C[M,N] = A[M,K] * W[N,K]^T  (+ bias[N] float32, may be NULL).
 * out_f32 != 0: C is float32, else C has the storage dtype. */
int gr4ad_op_linear(gr4ad_dtype dtype, const void *A_dev, const void *W_dev, const float *bias_dev, void *C_dev, int32_t M,
                    int32_t N, int32_t K, int32_t out_f32, void *hip_stream);

/*
 * gr4ad_op_quantize_rows -- rows of bf16 values as FP8 operands (appendix A.2; the quantiser of fp8_gemm mode):
 *   q[r, :] = nearest OCP E4M3 value (ties to even) of x[r, :] / scale[r],  scale[r] = max|x[r, :]| / 448 (1 for a zero row).
 * x [rows, n] bf16, q [rows, n] bytes, scale [rows] float32, all device; n a multiple of 8, x 16-byte and q 8-byte aligned.
 */
int gr4ad_op_quantize_rows(const void *x_dev, void *q_dev, float *scale_dev, int32_t rows, int32_t n, void *hip_stream);

/*
 * gr4ad_op_linear_fp8 -- C[M,N] = (a_scale[m] * w_scale) * Aq[M,K] Wq[N,K]^T (+ bias[n]) with E4M3 operands and float32
 * accumulation (the product fp8_gemm mode runs).  Aq, Wq device bytes, row-major, K contiguous; a_scale [M] and bias [N] (or
 * NULL) device float32; C device, float32 if out_f32 else bf16.  Shapes with M >= 64, N >= 256, K a multiple of 128 and
 * >= 384 and 16-byte aligned rows run on the matrix cores, the rest on a plain kernel.
 */
int gr4ad_op_linear_fp8(const void *Aq_dev, const float *a_scale_dev, const void *Wq_dev, float w_scale, const float *bias_dev, void *C_dev,
                        int32_t M, int32_t N, int32_t K, int32_t out_f32, void *hip_stream);

/* Log-softmax + cumulative score + top-k (appendix A.2, TopK Pre-Cut):
 * logits [B, n, V] float32, cum [B, n] float32 (NULL = zeros); keeps for each
 * request the k best of the n*V candidates cum[i] + log_softmax(logits[i])[v],
 * best first: parent [B,k], tok [B,k], score [B,k].  workspace_dev must hold
 * gr4ad_op_select_workspace_bytes(B, n, V, k) bytes. */
size_t gr4ad_op_select_workspace_bytes(int32_t B, int32_t n, int32_t V, int32_t k);
int gr4ad_op_select(const float *logits_dev, const float *cum_dev, int32_t B, int32_t n, int32_t V, int32_t k,
                    void *workspace_dev, size_t workspace_bytes, int32_t *parent_dev, int32_t *tok_dev, float *score_dev,
                    void *hip_stream);

/* gr4ad_op_select_f16 -- gr4ad_op_select on half-precision logits (IEEE binary16, [B, n, V] row-major), the form
 * in which decode_batch hands the classifier's output to the selection in bf16 mode: the log-softmax and the scores are
 * computed in float32 from the stored halves.  V must be a multiple of 8 and at most 8192 and logits_dev 16-byte aligned
 * (GR4AD_EUNSUPPORTED otherwise).  Same workspace, outputs and ordering as gr4ad_op_select. */
int gr4ad_op_select_f16(const void *logits_f16_dev, const float *cum_dev, int32_t B, int32_t n, int32_t V, int32_t k,
                        void *workspace_dev, size_t workspace_bytes, int32_t *parent_dev, int32_t *tok_dev, float *score_dev,
                        void *hip_stream);

/*
 * gr4ad_op_select_static -- gr4ad_op_select for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as gr4ad_op_select without the
 * workspace: the candidate lists, bounds and counts live in a fixed device array inside the library
 * (GR4AD_SELECT_STATIC_BYTES per GPU, held until the process ends).  The call allocates nothing (no hipMalloc, hipFree
 * or allocating library routine; per-kernel timing must be off, it creates events) and only enqueues kernels on
 * hip_stream.  Sizes with gr4ad_op_select_workspace_bytes(B, n, V, k) > GR4AD_SELECT_STATIC_BYTES are refused with
 * GR4AD_EWORKSPACE (message through gr4ad_last_error(NULL)).  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU, on whatever streams, race; nothing needs to be cleared between calls.
 */
#define GR4AD_SELECT_STATIC_BYTES (32u << 20)
int gr4ad_op_select_static(const float *logits_dev, const float *cum_dev, int32_t B, int32_t n, int32_t V, int32_t k,
                           int32_t *parent_dev, int32_t *tok_dev, float *score_dev, void *hip_stream);

/* Beam-shared cross-attention (section 4.2, Beam-Shared KV Caching): for each
 * request b and head h, out[b, i, h] = softmax(q[b,i,h] . K[b,:len_b,h] / sqrt(dh)) V[b,:len_b,h]
 * for all n query rows of the request.  q, out [B, n, d]; kv [B, S, 2d]
 * (keys in columns 0..d-1, values in d..2d-1); ctx_len [B] or NULL.
 * workspace_dev (16-byte aligned) must hold gr4ad_op_cross_attention_workspace_bytes
 * bytes: the matrix-core kernel reads the values from a per-head transposed copy
 * it first writes there (0 bytes for shapes that run on the plain kernel). */
size_t gr4ad_op_cross_attention_workspace_bytes(gr4ad_dtype dtype, int32_t B, int32_t S, int32_t d, int32_t H);
int gr4ad_op_cross_attention(gr4ad_dtype dtype, const void *q_dev, const void *kv_dev, const int32_t *ctx_len_dev,
                             void *out_dev, int32_t B, int32_t n, int32_t S, int32_t d, int32_t H, void *workspace_dev,
                             size_t workspace_bytes, void *hip_stream);

/* Attention of query rows over the raw context rows as keys AND values: the core of the lazy layers' cross-attention
 * (section 3.2, eq. trunk) in absorbed form, where q_h . (W_k,h x_s) = (W_k,h^T q_h) . x_s and
 * sum_s p_s W_v,h x_s = W_v,h sum_s p_s x_s leave one query of width d per (position, head).  For each request b and
 * query row i < RQ:  out[b, i, :] = sum_{s < len_b} softmax_s(scale * q[b, i, :] . x[b, s, :]) x[b, s, :].
 * q, out [B, RQ, d]; x [B, S, d]; all bf16, device, row-major, 16-byte aligned; ctx_len [B] int32 or NULL (all S rows,
 * values clamped to [1, S]); rows of x past a request's length are never used.  One kernel that reads the context once.
 * Covers dtype GR4AD_BF16, d = 512 or 1024 and RQ <= 128 (more than 64 query rows: two launches, each reading the
 * context): GR4AD_EUNSUPPORTED otherwise (gr4ad_decode_batch then forms scores, softmax and sums in three launches);
 * GR4AD_EINVAL for null or misaligned pointers.  No workspace. */
int gr4ad_op_context_attention(gr4ad_dtype dtype, const void *q_dev, const void *x_dev, const int32_t *ctx_len_dev, void *out_dev,
                               int32_t B, int32_t RQ, int32_t S, int32_t d, float scale, void *hip_stream);

/* Beam reorder as a row gather: dst[b, j, 0:row_elems] = src[b, parent[b,j],
 * 0:row_elems] for j < k; rows are `row_stride` elements apart in both buffers,
 * src holds n rows per request and dst k.  Element size follows dtype.
 * (gr4ad_decode_batch itself reorders nothing: it addresses a beam's earlier
 * keys and values through an ancestor-row table.  This entry point is for
 * callers that keep a per-beam cache of their own.) */
int gr4ad_op_gather_rows(gr4ad_dtype dtype, const void *src_dev, const int32_t *parent_dev, void *dst_dev, int32_t B, int32_t n,
                         int32_t k, int64_t row_elems, int64_t row_stride, void *hip_stream);

/*
 * Per-kernel timing for measurement (process-wide, off by default).  While on,
 * every kernel the library launches is bracketed by two HIP events recorded on
 * the stream the kernel is launched on.  gr4ad_profile_read waits for the
 * recorded events and sums, per kernel class c < gr4ad_profile_kernel_count():
 * elapsed milliseconds ms[c], algorithmic flops flops[c] (2*M*N*K per GEMM
 * launch; 4*n*S*d per request for cross-attention), algorithmic HBM bytes
 * bytes[c] (what the operation must read and write once: operands, outputs;
 * a table row shared by several beams once) and the number of launches.
 * The valid context lengths live on the device, so launches that depend on
 * them (cross-attention, the context key/value projections) are counted on
 * the padded length S - an upper bound; a caller that knows the lengths
 * rescales by mean(len)/S, as bench.py does.
 * reset != 0 forgets the records afterwards.  Not thread-safe.
 */
int gr4ad_profile_enable(int on);
int gr4ad_profile_kernel_count(void);
const char *gr4ad_profile_kernel_name(int kernel_class);
int gr4ad_profile_read(double *ms, double *flops, double *bytes, int64_t *launches, int reset);

#ifdef __cplusplus
}
#endif
#endif /* GR4AD_H */
