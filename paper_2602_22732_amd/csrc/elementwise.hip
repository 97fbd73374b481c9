// Row-wise HBM-bound kernels: RMSNorm, the gate half of Fuse, trunk input
// broadcast, and the beam reorder (row gather).  All move 16-byte vectors with
// consecutive lanes on consecutive addresses.
#include <string.h>

#include "common.h"

template <typename T> struct Vec16;  // 16 bytes of T
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<bf16> { static constexpr int N = 8; };

template <typename T> __device__ __forceinline__ void load16(const T *p, float *out) {
    uint4 raw = *(const uint4 *)p;
    const T *e = (const T *)&raw;
#pragma unroll
    for (int i = 0; i < Vec16<T>::N; i++) out[i] = to_f(e[i]);
}
template <typename T> __device__ __forceinline__ void store16(T *p, const float *in) {
    uint4 raw;
    T *e = (T *)&raw;
#pragma unroll
    for (int i = 0; i < Vec16<T>::N; i++) e[i] = from_f<T>(in[i]);
    *(uint4 *)p = raw;
}

// ---------------------------------------------------------------------------
// RMSNorm (pre-norm of every sub-layer and the final norm, section 3.2):
// one wavefront per row, the row is read once and kept in registers.
// ---------------------------------------------------------------------------
template <typename T, int MAXV>  // MAXV: 16-byte vectors per lane
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *__restrict__ x, const T *__restrict__ g, T *__restrict__ y,
                                                      int64_t rows, int d, float eps) {
    constexpr int N = Vec16<T>::N;
    const int lane = threadIdx.x % 64;
    const int64_t row = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (row >= rows) return;
    const int nvec = d / N;
    float v[MAXV][N];
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXV; i++) {
        int c = lane + i * 64;
        if (c < nvec) {
#pragma unroll
            for (int e = 0; e < N; e += 4) load16<float>(x + row * d + (int64_t)c * N + e, &v[i][e]);
#pragma unroll
            for (int e = 0; e < N; e++) ss += v[i][e] * v[i][e];
        }
    }
    ss = wave_sum(ss);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int i = 0; i < MAXV; i++) {
        int c = lane + i * 64;
        if (c < nvec) {
            float gg[N];
            load16<T>(g + (int64_t)c * N, gg);
#pragma unroll
            for (int e = 0; e < N; e++) v[i][e] = gg[e] * v[i][e] * inv;
            store16<T>(y + row * d + (int64_t)c * N, v[i]);
        }
    }
}

int launch_rmsnorm(gr4ad_dtype dtype, const void *x, const void *g, void *y, int64_t rows, int d, float eps, hipStream_t st) {
    if (rows <= 0) return GR4AD_OK;
    int64_t grid = ceil_div64(rows, 4);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_RMSNORM, st, 0.0, (double)rows * d * (4 + (dtype == GR4AD_BF16 ? 2 : 4)));
    if (dtype == GR4AD_BF16) {
        int nvec = d / 8;
        if (d % 8) return GR4AD_EUNSUPPORTED;
        if (nvec <= 128)
            hipLaunchKernelGGL((rmsnorm_kernel<bf16, 2>), dim3((unsigned)grid), dim3(256), 0, st, (const float *)x, (const bf16 *)g, (bf16 *)y, rows, d, eps);
        else if (nvec <= 512)
            hipLaunchKernelGGL((rmsnorm_kernel<bf16, 8>), dim3((unsigned)grid), dim3(256), 0, st, (const float *)x, (const bf16 *)g, (bf16 *)y, rows, d, eps);
        else
            return GR4AD_EUNSUPPORTED;
    } else {
        int nvec = d / 4;
        if (d % 4) return GR4AD_EUNSUPPORTED;
        if (nvec <= 128)
            hipLaunchKernelGGL((rmsnorm_kernel<float, 2>), dim3((unsigned)grid), dim3(256), 0, st, (const float *)x, (const float *)g, (float *)y, rows, d, eps);
        else if (nvec <= 1024)
            hipLaunchKernelGGL((rmsnorm_kernel<float, 16>), dim3((unsigned)grid), dim3(256), 0, st, (const float *)x, (const float *)g, (float *)y, rows, d, eps);
        else
            return GR4AD_EUNSUPPORTED;
    }
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// Gate half of Fuse (eq. fuse): a[row,:] = m_t[request,:] * (W_g s)[token,:],
// with W_g s read from the per-token table built at init.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void fuse_gate_kernel(const float *__restrict__ m, int64_t m_req_stride, const float *__restrict__ G,
                                                        const int32_t *__restrict__ tok, T *__restrict__ a, int64_t rows, int n, int d) {
    constexpr int N = Vec16<T>::N;
    const int nvec = d / N;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * nvec) return;
    const int64_t row = idx / nvec;
    const int c = (int)(idx % nvec);
    const int64_t b = row / n;
    const int64_t t = tok ? (int64_t)tok[row] : 0;
    float mv[N], gv[N];
#pragma unroll
    for (int e = 0; e < N; e += 4) load16<float>(m + b * m_req_stride + (int64_t)c * N + e, &mv[e]);
#pragma unroll
    for (int e = 0; e < N; e += 4) load16<float>(G + t * d + (int64_t)c * N + e, &gv[e]);
#pragma unroll
    for (int e = 0; e < N; e++) mv[e] *= gv[e];
    store16<T>(a + row * d + (int64_t)c * N, mv);
}

int launch_fuse_gate(gr4ad_dtype dtype, const void *m, int64_t m_req_stride, const void *G, int64_t table_rows, const int32_t *tok, void *a,
                     int B, int n, int d, hipStream_t st) {
    const int N = dtype == GR4AD_BF16 ? 8 : 4;
    int64_t rows = (int64_t)B * n, total = rows * (d / N);
    int64_t grid = ceil_div64(total, 256);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    // what must move once: the gated rows written, one trunk row per request, and each table row at most once (beams that carry
    // the same token share it; at most min(rows, table rows) distinct ones)
    const double distinct = (double)(rows < table_rows ? rows : table_rows);
    ProfScope ps(KC_FUSE_GATE, st, 0.0, (double)rows * d * (dtype == GR4AD_BF16 ? 2 : 4) + ((double)B + distinct) * d * 4);
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(fuse_gate_kernel<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)m, m_req_stride, (const float *)G, tok, (bf16 *)a, rows, n, d);
    else
        hipLaunchKernelGGL(fuse_gate_kernel<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)m, m_req_stride, (const float *)G, tok, (float *)a, rows, n, d);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// Input state of the vanilla autoregressive decoder (section 3.2): h^(0)_t = s_{t-1} + p_t, the embedding of the
// beam's previous token plus the level's position embedding, written to the float32 residual stream.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_pos_kernel(const T *__restrict__ E, const int32_t *__restrict__ tok, const T *__restrict__ p,
                                                        float *__restrict__ h, int64_t rows, int d) {
    constexpr int N = Vec16<T>::N;
    const int nvec = d / N;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * nvec) return;
    const int64_t row = idx / nvec;
    const int c = (int)(idx % nvec);
    const int64_t t = tok ? (int64_t)tok[row] : 0;
    float ev[N], pv[N];
    load16<T>(E + t * d + (int64_t)c * N, ev);
    load16<T>(p + (int64_t)c * N, pv);
#pragma unroll
    for (int e = 0; e < N; e++) ev[e] += pv[e];
#pragma unroll
    for (int e = 0; e < N; e += 4) store16<float>(h + row * d + (int64_t)c * N + e, &ev[e]);
}

int launch_embed_pos(gr4ad_dtype dtype, const void *E, const int32_t *tok, const void *p, void *h, int64_t rows, int d, hipStream_t st) {
    const int N = dtype == GR4AD_BF16 ? 8 : 4;
    if (!E || !p || !h || rows < 1 || d < N || d % N) return GR4AD_EINVAL;
    if (((uintptr_t)E % 16) || ((uintptr_t)p % 16) || ((uintptr_t)h % 16)) return GR4AD_EUNSUPPORTED;
    const int64_t grid = ceil_div64(rows * (d / N), 256);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    // one embedding row per distinct token is the least that must be read; rows of float32 written
    ProfScope ps(KC_FUSE_GATE, st, 0.0, (double)rows * d * 4);
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(embed_pos_kernel<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)E, tok, (const bf16 *)p, (float *)h, rows, d);
    else
        hipLaunchKernelGGL(embed_pos_kernel<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)E, tok, (const float *)p, (float *)h, rows, d);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// Trunk input (eq. trunk): m^(0)_t = p_t for every request.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void broadcast_rows_kernel(const T *__restrict__ pos, float *__restrict__ dst, int64_t total, int per_req) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    dst[idx] = to_f(pos[idx % per_req]);
}

int launch_broadcast_rows(gr4ad_dtype dtype, const void *pos, void *dst, int B, int T, int d, hipStream_t st) {
    int per_req = T * d;
    int64_t total = (int64_t)B * per_req;
    int64_t grid = ceil_div64(total, 256);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_BROADCAST, st, 0.0, (double)total * 4);
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(broadcast_rows_kernel<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)pos, (float *)dst, total, per_req);
    else
        hipLaunchKernelGGL(broadcast_rows_kernel<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)pos, (float *)dst, total, per_req);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// Beam reorder: survivors inherit their parent's self-attention K/V rows
// (KV caching, appendix A.2).  Pure copy: dst[b,j,:] = src[b,parent[b,j],:].
// One workgroup moves one row with 16-byte lanes; grid = B*k rows.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4 *__restrict__ src, const int32_t *__restrict__ parent,
                                                          uint4 *__restrict__ dst, int n, int k, int64_t row_vec, int64_t stride_vec) {
    const int64_t r = blockIdx.x;  // b*k + j
    const int64_t b = r / k;
    const int64_t p = parent[r];
    const uint4 *s = src + (b * n + p) * stride_vec;
    uint4 *o = dst + r * stride_vec;
    for (int64_t i = threadIdx.x; i < row_vec; i += 256) o[i] = s[i];
}

int launch_gather_rows(gr4ad_dtype dtype, const void *src, const int32_t *parent, void *dst, int B, int n, int k, int64_t row_elems,
                       int64_t row_stride, hipStream_t st) {
    const int N = dtype == GR4AD_BF16 ? 8 : 4;
    if (row_elems % N || row_stride % N || ((uintptr_t)src % 16) || ((uintptr_t)dst % 16)) return GR4AD_EUNSUPPORTED;
    int64_t rows = (int64_t)B * k;
    if (rows <= 0 || row_elems <= 0) return GR4AD_OK;
    if (rows > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_GATHER, st, 0.0, 2.0 * rows * (double)row_elems * (dtype == GR4AD_BF16 ? 2 : 4));
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)rows), dim3(256), 0, st, (const uint4 *)src, parent, (uint4 *)dst, n, k, row_elems / N, row_stride / N);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// Per-head transposed copy of a [d, d] projection weight (rows = output features): out[h][j][c] = w[h*dh + c][j].
// Built once at init for the key projection of the lazy layers, whose cross-attention runs in absorbed form.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void head_transpose_kernel(const bf16 *__restrict__ w, bf16 *__restrict__ out, int d, int dh) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // output element
    if (idx >= (int64_t)d * d) return;
    const int c = (int)(idx % dh);
    const int j = (int)((idx / dh) % d);
    const int h = (int)(idx / ((int64_t)dh * d));
    out[idx] = w[((int64_t)h * dh + c) * d + j];
}

int launch_head_transpose(const void *w, void *out, int d, int H, hipStream_t st) {
    if (!w || !out || d < 1 || H < 1 || d % H) return GR4AD_EINVAL;
    const int64_t grid = ceil_div64((int64_t)d * d, 256);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    hipLaunchKernelGGL(head_transpose_kernel, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)w, (bf16 *)out, d, d / H);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// Folded RMSNorm: per-row factor from the partial sums of squares a projection's epilogue left
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void row_inv_kernel(const float *__restrict__ ss, float *__restrict__ inv, int64_t rows, int parts, int dim,
                                                      float eps) {
    // 16 lanes per row: consecutive lanes read consecutive 16-byte pieces of the row's partial sums
    const int64_t r = ((int64_t)blockIdx.x * 256 + threadIdx.x) / 16;
    const int sub = threadIdx.x % 16;
    float s = 0.0f;
    if (r < rows)
        for (int u = sub * 4; u < parts; u += 64) {  // parts % 4 == 0
            const floatx4 v = *(const floatx4 *)(ss + r * parts + u);
            s += (v[0] + v[1]) + (v[2] + v[3]);
        }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o, 64);
    if (r < rows && sub == 0) inv[r] = 1.0f / sqrtf(s / (float)dim + eps);
}

int launch_row_inv(const float *ss, float *inv, int64_t rows, int parts, int dim, float eps, hipStream_t st) {
    if (!ss || !inv || rows < 1 || parts < 4 || parts % 4 || dim < 1 || ((uintptr_t)ss % 16)) return GR4AD_EINVAL;
    const int64_t grid = ceil_div64(rows * 16, 256);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_RMSNORM, st, 0.0, (double)rows * (parts + 1) * sizeof(float));
    hipLaunchKernelGGL(row_inv_kernel, dim3((unsigned)grid), dim3(256), 0, st, ss, inv, rows, parts, dim, eps);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// row-wise log-softmax of float32 logits (value step: no selection follows, the whole distribution is the output)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void log_softmax_rows_kernel(const float *__restrict__ logits, float *__restrict__ out, int64_t rows, int V) {
    // one wave per row; the row is read three times (maximum, sum, write), the second and third time from cache
    const int lane = threadIdx.x % 64;
    const int64_t r = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (r >= rows) return;
    const float *x = logits + r * V;
    float mx = -INFINITY;
    for (int c = lane; c < V; c += 64) mx = fmaxf(mx, x[c]);
    mx = wave_max(mx);
    float s = 0.0f;
    for (int c = lane; c < V; c += 64) s += __expf(x[c] - mx);
    s = wave_sum(s);
    const float lse = mx + __logf(s);
    float *y = out + r * V;
    for (int c = lane; c < V; c += 64) y[c] = x[c] - lse;
}

int launch_log_softmax_rows(const float *logits, float *out, int64_t rows, int V, hipStream_t st) {
    if (!logits || !out || rows < 1 || V < 1) return GR4AD_EINVAL;
    const int64_t grid = ceil_div64(rows, 4);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_SOFTMAX, st, 0.0, (double)rows * V * 2 * sizeof(float));
    hipLaunchKernelGGL(log_softmax_rows_kernel, dim3((unsigned)grid), dim3(256), 0, st, logits, out, rows, V);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// FP8 operands (low-precision inference, appendix A.2): rows become OCP E4M3 bytes with one scale per row,
// scale = amax(row) / 448, q = round_to_nearest_even(x / scale); a weight matrix gets one scale for the whole matrix.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint2 pack8_e4m3(const float (&v)[8], float qinv) {
    int w0 = 0, w1 = 0;
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(v[0] * qinv, v[1] * qinv, w0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(v[2] * qinv, v[3] * qinv, w0, true);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(v[4] * qinv, v[5] * qinv, w1, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(v[6] * qinv, v[7] * qinv, w1, true);
    return make_uint2((unsigned)w0, (unsigned)w1);
}

// One wavefront per row, the row stays in registers.  NORM: x is the float32 residual stream and the row is
// g * x / rms(x) (the RMSNorm in front of a projection); otherwise x is a bf16 activation row taken as it is.
template <bool NORM, int MAXV>  // MAXV: 8-element vectors per lane
__global__ __launch_bounds__(256) void quantize_rows_kernel(const void *__restrict__ xin, const bf16 *__restrict__ g, uint8_t *__restrict__ yq,
                                                            float *__restrict__ scale, int64_t rows, int n, float eps) {
    const int lane = threadIdx.x % 64;
    const int64_t row = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (row >= rows) return;
    const int nvec = n / 8;
    float v[MAXV][8];
    float ss = 0.0f, amax = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXV; i++) {
        const int c = lane + i * 64;
        if (c < nvec) {
            if (NORM) {
                load16<float>((const float *)xin + row * n + (int64_t)c * 8, &v[i][0]);
                load16<float>((const float *)xin + row * n + (int64_t)c * 8 + 4, &v[i][4]);
#pragma unroll
                for (int e = 0; e < 8; e++) ss += v[i][e] * v[i][e];
            } else {
                load16<bf16>((const bf16 *)xin + row * n + (int64_t)c * 8, v[i]);
#pragma unroll
                for (int e = 0; e < 8; e++) amax = fmaxf(amax, fabsf(v[i][e]));
            }
        }
    }
    if (NORM) {
        ss = wave_sum(ss);
        const float inv = 1.0f / sqrtf(ss / (float)n + eps);
#pragma unroll
        for (int i = 0; i < MAXV; i++) {
            const int c = lane + i * 64;
            if (c < nvec) {
                float gg[8];
                load16<bf16>(g + (int64_t)c * 8, gg);
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    v[i][e] = gg[e] * v[i][e] * inv;
                    amax = fmaxf(amax, fabsf(v[i][e]));
                }
            }
        }
    }
    amax = wave_max(amax);
    const float qinv = amax > 0.0f ? 448.0f / amax : 1.0f;
#pragma unroll
    for (int i = 0; i < MAXV; i++) {
        const int c = lane + i * 64;
        if (c < nvec) *(uint2 *)(yq + row * n + (int64_t)c * 8) = pack8_e4m3(v[i], qinv);
    }
    if (lane == 0) scale[row] = amax > 0.0f ? amax / 448.0f : 1.0f;
}

template <bool NORM>
static int launch_quantize_rows_any(const void *x, const void *g, void *yq, float *scale, int64_t rows, int n, float eps, hipStream_t st) {
    if (!x || !yq || !scale || rows < 1 || n < 8 || n % 8 || (NORM && !g)) return GR4AD_EINVAL;
    if (((uintptr_t)x % 16) || ((uintptr_t)yq % 8)) return GR4AD_EUNSUPPORTED;
    const int64_t grid = ceil_div64(rows, 4);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    const int nvec = n / 8;
    ProfScope ps(KC_QUANTIZE, st, 0.0, (double)rows * n * ((NORM ? 4 : 2) + 1));
    if (nvec <= 128)
        hipLaunchKernelGGL((quantize_rows_kernel<NORM, 2>), dim3((unsigned)grid), dim3(256), 0, st, x, (const bf16 *)g, (uint8_t *)yq, scale, rows, n, eps);
    else if (nvec <= 512)
        hipLaunchKernelGGL((quantize_rows_kernel<NORM, 8>), dim3((unsigned)grid), dim3(256), 0, st, x, (const bf16 *)g, (uint8_t *)yq, scale, rows, n, eps);
    else if (nvec <= 2048)
        hipLaunchKernelGGL((quantize_rows_kernel<NORM, 32>), dim3((unsigned)grid), dim3(256), 0, st, x, (const bf16 *)g, (uint8_t *)yq, scale, rows, n, eps);
    else
        return GR4AD_EUNSUPPORTED;
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

int launch_rmsnorm_quant(const void *x, const void *g, void *yq, float *scale, int64_t rows, int d, float eps, hipStream_t st) {
    return launch_quantize_rows_any<true>(x, g, yq, scale, rows, d, eps, st);
}

int launch_quantize_rows(const void *x, void *yq, float *scale, int64_t rows, int n, hipStream_t st) {
    return launch_quantize_rows_any<false>(x, nullptr, yq, scale, rows, n, 0.0f, st);
}

// whole-matrix scale (init time): largest magnitude through an integer maximum of the bit patterns (non-negative floats order like integers)
__global__ __launch_bounds__(256) void absmax_kernel(const bf16 *__restrict__ x, int64_t count, unsigned *__restrict__ out) {
    float m = 0.0f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) m = fmaxf(m, fabsf((float)x[i]));
    m = wave_max(m);
    if (threadIdx.x % 64 == 0) atomicMax(out, __float_as_uint(m));
}

__global__ __launch_bounds__(256) void quantize_flat_kernel(const bf16 *__restrict__ x, int64_t count, const unsigned *__restrict__ amax_bits,
                                                            uint8_t *__restrict__ out) {
    const float amax = __uint_as_float(*amax_bits);
    const float qinv = amax > 0.0f ? 448.0f / amax : 1.0f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count / 2; i += (int64_t)gridDim.x * 256) {
        const int w = __builtin_amdgcn_cvt_pk_fp8_f32((float)x[2 * i] * qinv, (float)x[2 * i + 1] * qinv, 0, false);
        *(uint16_t *)(out + 2 * i) = (uint16_t)(w & 0xffff);
    }
}

int launch_quantize_matrix(const void *w, void *wq, int64_t count, unsigned *amax_dev, float *scale_host, hipStream_t st) {
    if (!w || !wq || !amax_dev || !scale_host || count < 2 || count % 2 || ((uintptr_t)wq % 2)) return GR4AD_EINVAL;
    if (hipMemsetAsync(amax_dev, 0, sizeof(unsigned), st) != hipSuccess) return GR4AD_EHIP;
    int64_t grid = ceil_div64(count, 256 * 8);
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(absmax_kernel, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)w, count, amax_dev);
    GR4AD_LAUNCH_CHECK();
    hipLaunchKernelGGL(quantize_flat_kernel, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)w, count, amax_dev, (uint8_t *)wq);
    GR4AD_LAUNCH_CHECK();
    unsigned bits = 0;
    if (hipMemcpyAsync(&bits, amax_dev, sizeof(bits), hipMemcpyDeviceToHost, st) != hipSuccess || hipStreamSynchronize(st) != hipSuccess)
        return GR4AD_EHIP;
    float amax;
    memcpy(&amax, &bits, sizeof(amax));
    *scale_host = amax > 0.0f ? amax / 448.0f : 1.0f;
    return GR4AD_OK;
}
