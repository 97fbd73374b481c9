// Attention kernels of the decoder layer (section 3.2: cross-attention between
// decoder states and the context X, self-attention over decoder states).
//
//  * cross_attn_flash_bf16  beam-shared cross-attention (section 4.2, Beam-Shared
//                           KV Caching): one workgroup owns a block of beams of one
//                           (request, head); the context K/V tile is staged in LDS
//                           once and reused by every beam of the block.  MFMA, online
//                           softmax.
//  * cross_attn_simple<T>   one wavefront per (beam row, head), any shape; float32
//                           path and fallback.
//  * self_attn_step<T>      autoregressive self-attention of the new position over
//                           the beam path's cached positions (at most T keys).
//  * trunk_self_attn<T>     causal self-attention over the T trunk positions.
#include "common.h"

// ---------------------------------------------------------------------------
// simple cross-attention: wave per (row, head)
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void cross_attn_simple(const T *__restrict__ q, int64_t ldq, const T *__restrict__ kv,
                                                         const int32_t *__restrict__ ctx_len, T *__restrict__ out, int64_t ldo,
                                                         int64_t rows, int n, int S, int d, int H) {
    __shared__ float sq[4][128];
    __shared__ float sp[4][64];
    const int lane = threadIdx.x % 64, wv = threadIdx.x / 64;
    const int64_t wid = (int64_t)blockIdx.x * 4 + wv;
    if (wid >= rows * H) return;
    const int64_t row = wid / H;
    const int h = (int)(wid % H);
    const int64_t b = row / n;
    const int dh = d / H;
    int len = ctx_len ? ctx_len[b] : S;
    len = len < 1 ? 1 : (len > S ? S : len);
    const float scale = 1.0f / sqrtf((float)dh);
    for (int c = lane; c < dh; c += 64) sq[wv][c] = to_f(q[row * ldq + h * dh + c]) * scale;
    const T *kbase = kv + b * (int64_t)S * 2 * d + h * dh;  // key j at kbase + j*2d, value at + d
    float m = -INFINITY, l = 0.0f, acc[2] = {0.0f, 0.0f};
    for (int j0 = 0; j0 < len; j0 += 64) {
        const int j = j0 + lane;
        float s = -INFINITY;
        if (j < len) {
            const T *kr = kbase + (int64_t)j * 2 * d;
            s = 0.0f;
            for (int c = 0; c < dh; c++) s = fmaf(sq[wv][c], to_f(kr[c]), s);
        }
        const float mnew = fmaxf(m, wave_max(s));
        const float p = (j < len) ? __expf(s - mnew) : 0.0f;
        const float alpha = __expf(m - mnew);  // m = -inf on the first tile gives 0
        l = l * alpha + wave_sum(p);
        m = mnew;
        sp[wv][lane] = p;
        acc[0] *= alpha;
        acc[1] *= alpha;
        const int cnt = (len - j0) < 64 ? (len - j0) : 64;
        for (int jj = 0; jj < cnt; jj++) {
            const float pj = sp[wv][jj];
            const T *vr = kbase + (int64_t)(j0 + jj) * 2 * d + d;
            if (lane < dh) acc[0] = fmaf(pj, to_f(vr[lane]), acc[0]);
            if (lane + 64 < dh) acc[1] = fmaf(pj, to_f(vr[lane + 64]), acc[1]);
        }
    }
    const float inv = 1.0f / l;
    if (lane < dh) out[row * ldo + h * dh + lane] = from_f<T>(acc[0] * inv);
    if (lane + 64 < dh) out[row * ldo + h * dh + lane + 64] = from_f<T>(acc[1] * inv);
}

int launch_cross_attention(gr4ad_dtype dtype, const void *q, int64_t ldq, const void *kv, const int32_t *ctx_len, void *out, int64_t ldo,
                           int B, int n, int S, int d, int H, hipStream_t st) {
    if (B <= 0 || n <= 0 || S <= 0 || d <= 0 || H <= 0 || d % H) return GR4AD_EINVAL;
    const int dh = d / H;
    if (dh > 128) return GR4AD_EUNSUPPORTED;
    const int64_t rows = (int64_t)B * n;
    const int64_t grid = ceil_div64(rows * H, 4);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_XATTN_SIMPLE, st);
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(cross_attn_simple<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)q, ldq, (const bf16 *)kv, ctx_len, (bf16 *)out, ldo, rows, n, S, d, H);
    else
        hipLaunchKernelGGL(cross_attn_simple<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)q, ldq, (const float *)kv, ctx_len, (float *)out, ldo, rows, n, S, d, H);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// self-attention of the new position over the beam path's cache
// ---------------------------------------------------------------------------
// qkv [rows,3d]; cache [rows][T][2d] (keys then values per position); the new
// position's k,v are appended at `pos` and the query attends to 0..pos.
template <typename T>
__global__ __launch_bounds__(256) void self_attn_step(const T *__restrict__ qkv, T *__restrict__ cache, T *__restrict__ out,
                                                      int64_t rows, int pos, int Tlev, int d, int H) {
    const int lane = threadIdx.x % 64, wv = threadIdx.x / 64;
    const int64_t wid = (int64_t)blockIdx.x * 4 + wv;
    if (wid >= rows * H) return;
    const int64_t row = wid / H;
    const int h = (int)(wid % H);
    const int dh = d / H;
    const float scale = 1.0f / sqrtf((float)dh);
    const T *qr = qkv + row * 3 * d + h * dh;
    T *cr = cache + row * (int64_t)Tlev * 2 * d + h * dh;
    float qv[2], kn[2], vn[2];
#pragma unroll
    for (int e = 0; e < 2; e++) {
        const int c = lane + 64 * e;
        const bool ok = c < dh;
        qv[e] = ok ? to_f(qr[c]) : 0.0f;
        T kt = ok ? qr[d + c] : from_f<T>(0.0f), vt = ok ? qr[2 * d + c] : from_f<T>(0.0f);
        kn[e] = to_f(kt);
        vn[e] = to_f(vt);
        if (ok) {
            cr[(int64_t)pos * 2 * d + c] = kt;
            cr[(int64_t)pos * 2 * d + d + c] = vt;
        }
    }
    float s[GR4AD_MAX_LEVELS];
    float mx = -INFINITY;
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++) {
        if (p <= pos) {
            float part = 0.0f;
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const int c = lane + 64 * e;
                float kk = (p == pos) ? kn[e] : (c < dh ? to_f(cr[(int64_t)p * 2 * d + c]) : 0.0f);
                part = fmaf(qv[e], kk, part);
            }
            s[p] = wave_sum(part) * scale;
            mx = fmaxf(mx, s[p]);
        }
    }
    float den = 0.0f;
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++)
        if (p <= pos) { s[p] = __expf(s[p] - mx); den += s[p]; }
    const float inv = 1.0f / den;
    float o[2] = {0.0f, 0.0f};
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++) {
        if (p <= pos) {
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const int c = lane + 64 * e;
                float vv = (p == pos) ? vn[e] : (c < dh ? to_f(cr[(int64_t)p * 2 * d + d + c]) : 0.0f);
                o[e] = fmaf(s[p] * inv, vv, o[e]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 2; e++) {
        const int c = lane + 64 * e;
        if (c < dh) out[row * d + h * dh + c] = from_f<T>(o[e]);
    }
}

int launch_self_attention_step(gr4ad_dtype dtype, const void *qkv, void *cache, void *out, int64_t rows, int pos, int T, int d, int H,
                               hipStream_t st) {
    if (rows <= 0 || pos < 0 || pos >= T || T > GR4AD_MAX_LEVELS || d % H) return GR4AD_EINVAL;
    if (d / H > 128) return GR4AD_EUNSUPPORTED;
    const int64_t grid = ceil_div64(rows * H, 4);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_SELF_STEP, st);
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(self_attn_step<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)qkv, (bf16 *)cache, (bf16 *)out, rows, pos, T, d, H);
    else
        hipLaunchKernelGGL(self_attn_step<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)qkv, (float *)cache, (float *)out, rows, pos, T, d, H);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// causal self-attention over the trunk positions (lazy layers, eq. trunk)
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void trunk_self_attn(const T *__restrict__ qkv, T *__restrict__ out, int64_t rows, int Tlev, int d, int H) {
    const int lane = threadIdx.x % 64, wv = threadIdx.x / 64;
    const int64_t wid = (int64_t)blockIdx.x * 4 + wv;
    if (wid >= rows * H) return;
    const int64_t row = wid / H;  // b*T + tau
    const int h = (int)(wid % H);
    const int tau = (int)(row % Tlev);
    const int64_t first = row - tau;  // row of position 0 of this request
    const int dh = d / H;
    const float scale = 1.0f / sqrtf((float)dh);
    float qv[2];
#pragma unroll
    for (int e = 0; e < 2; e++) {
        const int c = lane + 64 * e;
        qv[e] = c < dh ? to_f(qkv[row * 3 * d + h * dh + c]) : 0.0f;
    }
    float s[GR4AD_MAX_LEVELS];
    float mx = -INFINITY;
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++) {
        if (p <= tau) {
            float part = 0.0f;
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const int c = lane + 64 * e;
                if (c < dh) part = fmaf(qv[e], to_f(qkv[(first + p) * 3 * d + d + h * dh + c]), part);
            }
            s[p] = wave_sum(part) * scale;
            mx = fmaxf(mx, s[p]);
        }
    }
    float den = 0.0f;
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++)
        if (p <= tau) { s[p] = __expf(s[p] - mx); den += s[p]; }
    const float inv = 1.0f / den;
#pragma unroll
    for (int e = 0; e < 2; e++) {
        const int c = lane + 64 * e;
        if (c < dh) {
            float o = 0.0f;
#pragma unroll
            for (int p = 0; p < GR4AD_MAX_LEVELS; p++)
                if (p <= tau) o = fmaf(s[p] * inv, to_f(qkv[(first + p) * 3 * d + 2 * d + h * dh + c]), o);
            out[row * d + h * dh + c] = from_f<T>(o);
        }
    }
}

int launch_trunk_self_attention(gr4ad_dtype dtype, const void *qkv, void *out, int B, int T, int d, int H, hipStream_t st) {
    if (B <= 0 || T <= 0 || T > GR4AD_MAX_LEVELS || d % H) return GR4AD_EINVAL;
    if (d / H > 128) return GR4AD_EUNSUPPORTED;
    const int64_t rows = (int64_t)B * T;
    const int64_t grid = ceil_div64(rows * H, 4);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_TRUNK_SELF, st);
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(trunk_self_attn<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)qkv, (bf16 *)out, rows, T, d, H);
    else
        hipLaunchKernelGGL(trunk_self_attn<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)qkv, (float *)out, rows, T, d, H);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}
