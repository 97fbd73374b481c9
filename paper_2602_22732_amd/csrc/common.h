// Internal declarations shared by the HIP translation units of libgr4ad.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gr4ad.h"

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef int intx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float to_f(float x) { return x; }
__device__ __forceinline__ float to_f(bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f(float x);
template <> __device__ __forceinline__ float from_f<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f<bf16>(float x) { return (bf16)x; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// The same reductions through data-parallel-primitive operands instead of LDS permutes (a few cycles per step instead of an
// LDS round trip); every lane must be active.  Rotations by 8, 4, 2, 1 inside each row of 16 lanes leave the row's result in
// all of its lanes; two row broadcasts (lane 15 into the next row for rows 1 and 3, lane 31 into rows 2 and 3) leave the
// wavefront's result in lane 63, which is read back as a scalar.  The summation tree differs from wave_sum's: kernels that
// must agree to the bit use the same one.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_move(float old, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum_dpp(float v) {
    v += dpp_move<0x128, 0xF>(0.0f, v);  // row_ror:8
    v += dpp_move<0x124, 0xF>(0.0f, v);  // row_ror:4
    v += dpp_move<0x122, 0xF>(0.0f, v);  // row_ror:2
    v += dpp_move<0x121, 0xF>(0.0f, v);  // row_ror:1
    v += dpp_move<0x142, 0xA>(0.0f, v);  // row_bcast:15 into rows 1 and 3 (the other rows add 0)
    v += dpp_move<0x143, 0xC>(0.0f, v);  // row_bcast:31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max_dpp(float v) {
    v = fmaxf(v, dpp_move<0x128, 0xF>(v, v));
    v = fmaxf(v, dpp_move<0x124, 0xF>(v, v));
    v = fmaxf(v, dpp_move<0x122, 0xF>(v, v));
    v = fmaxf(v, dpp_move<0x121, 0xF>(v, v));
    v = fmaxf(v, dpp_move<0x142, 0xA>(v, v));  // (the other rows take the maximum with themselves)
    v = fmaxf(v, dpp_move<0x143, 0xC>(v, v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Records the message gr4ad_last_error(NULL) returns on this thread (entry points that take no decoder); returns `code`.
int gr4ad_set_thread_error(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// ---- GEMM: C[M,N] = A[M,K] * W[N,K]^T with a fused epilogue -----------------
enum { ACT_NONE = 0, ACT_SILU = 1 };
struct GemmEpilogue {
    void *C;             // output, row stride ldc elements
    int64_t ldc;
    int out_f32;         // 1: C is float, 0: C has the storage dtype
    int out_f16;         // with out_f32 = 1 and no residual/table (persistent kernel only): the float32 results (scaled, biased) leave as
                         // IEEE half precision, C is a half array (row stride ldc elements): the classifier's logits for the selection
    const float *resid;  // float32 [M, stride ldr] residual stream, added to the product (may alias C)
    int64_t ldr;
    const float *bias;   // [N] float, added per column
    const float *table;  // float32 [*, N]: row tok[row] (or row 0 if tok == NULL) added per row
    const int32_t *tok;  // [M] row selector of `table`
    const void *rowmul;  // unused by the GEMM (reserved)
    int act;             // ACT_*
    const int32_t *ctx_len;  // launch_gemm_vt only: valid rows per request (NULL = all)
    int vt_S;                // launch_gemm_vt only: rows per request
    // RMSNorm folded into the projections around it (persistent kernel only; launch_gemm fails if it cannot honour them):
    // writer side (out_f32 with resid or table, N % 256 == 0): besides C, write norm_out[row, col] = C[row, col] * norm_gain[col]
    // in the storage dtype (row stride norm_ld) and norm_ss[row * (N / 64) + col / 64] = sum of C^2 over those 64 columns
    // (launch_row_inv turns them into 1/rms per row); reader side: scale row r of the product by row_inv[r] before anything
    // else the epilogue does (activation, bias).
    const void *norm_gain;
    void *norm_out;
    int64_t norm_ld;
    float *norm_ss;
    const float *row_inv;
    // persistent kernel only (ignored elsewhere): the rows of A are requests of skip_S rows each of which only the first
    // skip_len[b] are valid; output tiles whose rows all lie in one request's padding are not computed (their C is not written)
    const int32_t *skip_len;
    int skip_S;
    const float *a_scale;      // launch_gemm_f8 only (set by it): per-row scale of the FP8 A operand
    float w_scale;             // launch_gemm_f8 only (set by it): scale of the FP8 W operand
    const int32_t *batch_len;  // launch_gemm_batched only: valid length per batch (NULL = none)
    int len_bounds;            // 1: the length bounds the columns of C that are needed, 2: it bounds K
};
// A row stride lda, W row stride ldw (elements).  dtype: storage type of A, W (and C unless out_f32).
int launch_gemm(gr4ad_dtype dtype, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K,
                const GemmEpilogue &epi, hipStream_t st);
// true if launch_gemm would run this product on the persistent kernel (the one that supports the folded RMSNorm)
bool gemm_on_persistent_kernel(gr4ad_dtype dtype, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K,
                               const GemmEpilogue &epi);

// FP8 (OCP E4M3) operands: C = (a_scale[row] * w_scale) * Aq Wq^T followed by the same epilogues; lda, ldw in elements (bytes);
// C is bf16 unless epi.out_f32.  Large shapes run on the persistent kernel's FP8 form, the rest on the plain kernel.
int launch_gemm_f8(const void *A, int64_t lda, const float *a_scale, const void *W, int64_t ldw, float w_scale, int64_t M, int N, int K,
                   const GemmEpilogue &epi, hipStream_t st);
bool gemm_f8_on_persistent_kernel(const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K, const GemmEpilogue &epi);

// batched small products (bf16 operands, 128x128 MFMA tiles): see gemm.hip
int launch_gemm_batched(const void *A, int64_t lda, int64_t batch_a, const void *W, int64_t ldw, int64_t batch_w, void *C, int64_t ldc,
                        int64_t batch_c, int out_f32, int64_t M, int N, int K, int batch, const int32_t *batch_len, int len_bounds,
                        hipStream_t st);
// transposed-per-request product (context values for the attention kernel): see gemm.hip
bool gemm_vt_supported(gr4ad_dtype dtype, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K, int S,
                       const void *out, int64_t ld_out);
int launch_gemm_vt(const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K, int S, const int32_t *ctx_len, void *out,
                   int64_t ld_out, hipStream_t st);

// ---- element-wise / norm kernels -------------------------------------------
// y[r,:] = g * x[r,:] / sqrt(mean(x[r,:]^2) + eps); x is the float32 residual stream, g and y have the storage dtype
int launch_rmsnorm(gr4ad_dtype dtype, const void *x, const void *g, void *y, int64_t rows, int d, float eps, hipStream_t st);
// inv[r] = 1 / sqrt(sum(ss[r*parts .. r*parts+parts-1]) / dim + eps): per-row factor of the folded RMSNorm from the partial sums
int launch_row_inv(const float *ss, float *inv, int64_t rows, int parts, int dim, float eps, hipStream_t st);
// a[(b*n+i), :] = m[b*m_stride + :] * G[tok(b,i), :]   (tok == NULL: row 0 of G); m and G float32 (G: table_rows rows), a storage dtype
int launch_fuse_gate(gr4ad_dtype dtype, const void *m, int64_t m_req_stride, const void *G, int64_t table_rows, const int32_t *tok, void *a,
                     int B, int n, int d, hipStream_t st);
// h[row, :] = E[tok[row], :] + p[:]   (tok == NULL: row 0 of E); E and p storage dtype, h float32: the vanilla decoder's input state
int launch_embed_pos(gr4ad_dtype dtype, const void *E, const int32_t *tok, const void *p, void *h, int64_t rows, int d, hipStream_t st);
// dst[b*T + t, :] = pos[t, :]   (pos storage dtype, dst float32)
int launch_broadcast_rows(gr4ad_dtype dtype, const void *pos, void *dst, int B, int T, int d, hipStream_t st);
// dst[b, j, 0:row_elems] = src[b, parent[b,j], 0:row_elems]
int launch_gather_rows(gr4ad_dtype dtype, const void *src, const int32_t *parent, void *dst, int B, int n, int k, int64_t row_elems,
                       int64_t row_stride, hipStream_t st);

// out[r, :] = logits[r, :] - log(sum(exp(logits[r, :])))   (float32 rows of V values)
int launch_log_softmax_rows(const float *logits, float *out, int64_t rows, int V, hipStream_t st);

// FP8 (OCP E4M3) operands.  Rows: yq[r, :] = e4m3(x[r, :] / scale[r]), scale[r] = amax(row) / 448 (1 for a zero row);
// launch_rmsnorm_quant takes the float32 residual stream and quantises g * x / rms(x), launch_quantize_rows a bf16 row as it is.
int launch_rmsnorm_quant(const void *x, const void *g, void *yq, float *scale, int64_t rows, int d, float eps, hipStream_t st);
int launch_quantize_rows(const void *x, void *yq, float *scale, int64_t rows, int n, hipStream_t st);
// init time, synchronises the stream: one scale for the whole bf16 matrix of `count` elements, returned on the host
int launch_quantize_matrix(const void *w, void *wq, int64_t count, unsigned *amax_dev, float *scale_host, hipStream_t st);

// out[h][j][c] = w[h*dh + c][j] for a bf16 [d, d] weight (init-time)
int launch_head_transpose(const void *w, void *out, int d, int H, hipStream_t st);

// ---- attention ---------------------------------------------------------------
// beam-shared cross-attention; q/out row stride ldq/ldo elements, rows (b*n+i)
// vt: per-(request, head) transposed values built by launch_cross_attention_prepare (NULL: plain kernel on kv alone)
int launch_cross_attention(gr4ad_dtype dtype, const void *q, int64_t ldq, const void *kv, const void *vt, const int32_t *ctx_len, void *out,
                           int64_t ldo, int B, int n, int S, int d, int H, hipStream_t st);
// bytes of the transposed-value buffer the MFMA kernel needs for kv [B,S,2d] (0: the shape runs on the plain kernel)
size_t cross_attention_workspace_bytes(gr4ad_dtype dtype, int B, int S, int d, int H);
int launch_cross_attention_prepare(gr4ad_dtype dtype, const void *kv, const int32_t *ctx_len, void *vt, int B, int S, int d, int H,
                                   hipStream_t st);
// lazy layers' cross-attention in absorbed form (see decoder.hip): transposed, length-masked context copy [B, d, Spad]
int launch_context_transpose(const void *x, const int32_t *ctx_len, void *xt, int B, int S, int d, hipStream_t st);
// p[r, :] = softmax(scale * sc[r, :len]) (bf16, zero from len to ld) for float32 score rows; request of row r = r / rows_per_req
int launch_masked_softmax(const float *sc, void *p, const int32_t *ctx_len, int64_t rows, int rows_per_req, int S, int ld, float scale,
                          hipStream_t st);
// Lazy layers in absorbed form, one pass: z [B, RQ, d] = softmax(scale * qp x^T) x per request over its first len rows
// (qp [B, RQ, d], x [B, S, d], bf16; 64 queries of every request per launch).  GR4AD_EUNSUPPORTED for shapes
// context_attention_covers() refuses.
bool context_attention_covers(gr4ad_dtype dtype, int RQ, int d);
int launch_context_attention(gr4ad_dtype dtype, const void *qp, const void *x, const int32_t *ctx_len, void *z, int B, int RQ, int S, int d,
                             float scale, hipStream_t st);
// autoregressive self-attention of position `pos` for rows (b*n+i).  qkv [rows,3d] holds q, k, v of the new position;
// the keys and values of position p < pos are columns d..3d of row anc[row*T + p] of prev.p[p] (the [*,3d] q/k/v buffer
// that level wrote): the beam reorder is the ancestor table, no rows are moved.
struct LevelBuffers { const void *p[GR4AD_MAX_LEVELS]; int64_t rows[GR4AD_MAX_LEVELS]; };  // rows: rows of that level's buffer
int launch_self_attention_step(gr4ad_dtype dtype, const void *qkv, const LevelBuffers &prev, const int32_t *anc, void *out, int64_t rows,
                               int pos, int T, int d, int H, hipStream_t st);
// causal self-attention over the T trunk positions of each request: qkv [B*T,3d] -> out [B*T,d]
int launch_trunk_self_attention(gr4ad_dtype dtype, const void *qkv, void *out, int B, int T, int d, int H, hipStream_t st);

// ---- selection ---------------------------------------------------------------
size_t select_workspace_bytes(int B, int n, int V, int k);
// sid_old [B,n,T] / sid_new [B,k,T] may be NULL (no path bookkeeping); anc_old / anc_new likewise: batch-wide row index of
// each survivor's ancestor at levels 0..level (anc_new[.., level] = b*n + parent); level = 0-based t
// logits_f16 != 0: logits is a half-precision array (what the classifier's persistent GEMM leaves for large levels); needs select_takes_f16(V)
int launch_select(const void *logits, int logits_f16, const float *cum, int B, int n, int V, int k, void *ws, size_t ws_bytes, int32_t *parent,
                  int32_t *tok, float *score, const int32_t *sid_old, int32_t *sid_new, const int32_t *anc_old, int32_t *anc_new, int T,
                  int level, hipStream_t st);
bool select_takes_f16(int V);

// ---- optional per-kernel event timing ----------------------------------------
enum KernelClass { KC_GEMM_256 = 0, KC_GEMM_128, KC_GEMM_SIMPLE, KC_XATTN_FLASH, KC_XATTN_SIMPLE, KC_SELF_STEP, KC_TRUNK_SELF,
                   KC_RMSNORM, KC_FUSE_GATE, KC_SELECT_ROWS, KC_SELECT_REQUEST, KC_GATHER, KC_BROADCAST, KC_V_TRANSPOSE, KC_GEMM_RING, KC_SOFTMAX, KC_GEMM_RING_F8, KC_QUANTIZE, KC_CONTEXT_ATTN, KC_COUNT };
// Declared around a kernel launch: records an event before and (on scope exit) after it when timing is on.
struct ProfScope {
    ProfScope(int cls, hipStream_t st, double flops = 0.0, double bytes = 0.0);  // algorithmic work of the launch
    ~ProfScope();
    int idx_;
    hipStream_t st_;
};

#define GR4AD_LAUNCH_CHECK()                                   \
    do {                                                       \
        hipError_t e_ = hipGetLastError();                     \
        if (e_ != hipSuccess) return GR4AD_EHIP;               \
    } while (0)
