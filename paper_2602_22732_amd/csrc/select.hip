// Fused log-softmax + cumulative score + top-k beam selection.
//
// At level t the search keeps the b_t best of the n_t*V_t candidates
// score(i,v) = c_i + log_softmax(z_i)[v] of a request (section 3.2 beam search,
// section 4.2 Dynamic Beam Width).  The selection is two-stage, as TopK Pre-Cut
// (appendix A.2) describes: every beam row first keeps its own min(b_t, V_t)
// best tokens, then the request keeps the b_t best of those.  Both stages are
// exact radix selections, so the result equals a full sort of all candidates.
//
// Candidates travel between the stages as unique 64-bit keys
//     (order-preserving bits of the fp32 score) << 32 | (0xFFFFFFFF - flat index)
// so "larger key" means "higher score, then lower flat index i*V + v": equal
// scores resolve deterministically and the final order is a plain key sort.
#include "common.h"

__device__ __forceinline__ uint32_t score_key(float f) {
    f += 0.0f;  // -0 -> +0 so equal scores have equal keys
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_score(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

// inclusive scan over a 256-thread block (4 wavefronts)
__device__ __forceinline__ int block_scan_256(int v, int *wave_tot /*[4] LDS*/) {
    const int lane = threadIdx.x % 64, wv = threadIdx.x / 64;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    if (lane == 63) wave_tot[wv] = v;
    __syncthreads();
    int add = 0;
    for (int w = 0; w < wv; w++) add += wave_tot[w];
    __syncthreads();
    return v + add;
}

// ---------------------------------------------------------------------------
// stage A: one workgroup per beam row
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void select_rows(const float *__restrict__ logits, const float *__restrict__ cum, int n, int V, int m,
                                                   unsigned long long *__restrict__ cand) {
    extern __shared__ uint32_t skey[];  // [V] logits, then keys
    __shared__ float red[4];
    __shared__ int hist[256];
    __shared__ int wave_tot[4];
    __shared__ int sel_digit, sel_krem, sel_cnt, out_gt, out_eq;
    const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
    const int64_t row = blockIdx.x;
    const float *z = logits + row * (int64_t)V;
    float *sz = (float *)skey;
    const float c = cum ? cum[row] : 0.0f;

    float mx = -INFINITY;
    for (int v = tid; v < V; v += 256) {
        float x = z[v];
        sz[v] = x;
        mx = fmaxf(mx, x);
    }
    mx = wave_max(mx);
    if (lane == 0) red[wv] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float sum = 0.0f;
    for (int v = tid; v < V; v += 256) sum += __expf(sz[v] - mx);
    sum = wave_sum(sum);
    if (lane == 0) red[wv] = sum;
    __syncthreads();
    const float lse = mx + __logf((red[0] + red[1]) + (red[2] + red[3]));
    for (int v = tid; v < V; v += 256) skey[v] = score_key(c + (sz[v] - lse));  // each thread rewrites only its own slots
    if (tid == 0) { sel_krem = m; out_gt = 0; }
    __syncthreads();

    // radix select of the m-th largest key: 4 passes of 8 bits, most significant first
    uint32_t prefix = 0;
    int krem = m, cnt_eq = V;
    if (m < V) {
        for (int pass = 0; pass < 4; pass++) {
            const int shift = 24 - 8 * pass;
            hist[tid] = 0;
            __syncthreads();
            for (int v = tid; v < V; v += 256) {
                uint32_t k = skey[v];
                if (pass == 0 || (k >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(k >> shift) & 255], 1);
            }
            __syncthreads();
            const int own = hist[255 - tid];  // thread t owns digit 255-t: scan runs from the top digit down
            const int incl = block_scan_256(own, wave_tot);
            if (incl >= krem && incl - own < krem) { sel_digit = 255 - tid; sel_krem = krem - (incl - own); sel_cnt = own; }
            __syncthreads();
            prefix |= (uint32_t)sel_digit << shift;
            krem = sel_krem;
            cnt_eq = sel_cnt;
            __syncthreads();
        }
    }
    // keys > prefix go first (any order), then krem of the cnt_eq keys == prefix, lowest token first
    unsigned long long *dst = cand + row * (int64_t)m;
    const uint32_t flat0 = (uint32_t)((row % n) * (int64_t)V);
    const int n_gt = m - krem;
    if (tid == 0) out_eq = 0;
    __syncthreads();
    if (m >= V || cnt_eq == krem) {
        for (int v = tid; v < V; v += 256) {
            uint32_t k = skey[v];
            if (m >= V || k >= prefix) {
                int p = (m >= V) ? v : ((k > prefix) ? atomicAdd(&out_gt, 1) : n_gt + atomicAdd(&out_eq, 1));
                dst[p] = ((unsigned long long)k << 32) | (0xFFFFFFFFu - (flat0 + (uint32_t)v));
            }
        }
    } else {
        int base = 0;  // equal keys taken so far, in token order
        for (int v0 = 0; v0 < V; v0 += 256) {
            const int v = v0 + tid;
            const uint32_t k = v < V ? skey[v] : 0u;
            const int flag = (v < V && k == prefix) ? 1 : 0;
            const int incl = block_scan_256(flag, wave_tot);
            if (v < V && k > prefix) dst[atomicAdd(&out_gt, 1)] = ((unsigned long long)k << 32) | (0xFFFFFFFFu - (flat0 + (uint32_t)v));
            const int rank = base + incl - flag;
            if (flag && rank < krem) dst[n_gt + rank] = ((unsigned long long)k << 32) | (0xFFFFFFFFu - (flat0 + (uint32_t)v));
            if (tid == 255) sel_cnt = base + incl;
            __syncthreads();
            base = sel_cnt;
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------
// stage B: one workgroup per request
// ---------------------------------------------------------------------------
#define SELB_THREADS 1024
#define SELB_SORT_MAX 4096

__device__ __forceinline__ void bitonic_sort_desc(unsigned long long *s, int n_pow2) {
    for (int k = 2; k <= n_pow2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < n_pow2; i += SELB_THREADS) {
                int ixj = i ^ j;
                if (ixj > i) {
                    unsigned long long a = s[i], b = s[ixj];
                    bool desc = (i & k) == 0;
                    if (desc ? (a < b) : (a > b)) { s[i] = b; s[ixj] = a; }
                }
            }
            __syncthreads();
        }
}

__global__ __launch_bounds__(SELB_THREADS) void select_request(const unsigned long long *__restrict__ cand, int64_t ncand, int V, int k,
                                                               int32_t *__restrict__ parent, int32_t *__restrict__ tok,
                                                               float *__restrict__ score, const int32_t *__restrict__ sid_old,
                                                               int32_t *__restrict__ sid_new, int n, int T, int level) {
    __shared__ unsigned long long skeys[SELB_SORT_MAX];
    __shared__ int hist[2048];
    __shared__ int wave_tot[16];
    __shared__ int sel_digit, sel_krem, sel_cnt, out_cnt;
    const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
    const int64_t b = blockIdx.x;
    const unsigned long long *src = cand + b * ncand;
    int kp = 1;
    while (kp < k) kp <<= 1;

    if (ncand <= SELB_SORT_MAX) {
        int np = 1;
        while (np < ncand) np <<= 1;
        for (int i = tid; i < np; i += SELB_THREADS) skeys[i] = i < ncand ? src[i] : 0ull;
        __syncthreads();
        bitonic_sort_desc(skeys, np);
    } else {
        // radix select on the unique 64-bit keys, 11-bit digits from the top; stops as
        // soon as the chosen bin holds exactly the number of keys still needed
        unsigned long long prefix = 0;  // value of key >> shift
        int krem = k, shift = 64;
        const int widths[6] = {11, 11, 11, 11, 11, 9};
        for (int pass = 0; pass < 6; pass++) {
            const int w = widths[pass];
            const int nshift = shift - w;
            for (int i = tid; i < 2048; i += SELB_THREADS) hist[i] = 0;
            __syncthreads();
            for (int64_t i = tid; i < ncand; i += SELB_THREADS) {
                unsigned long long key = src[i];
                if (pass == 0 || (key >> shift) == prefix) atomicAdd(&hist[(int)((key >> nshift) & ((1u << w) - 1))], 1);
            }
            __syncthreads();
            // thread t owns digits 2047-2t (hi) and 2046-2t (lo); scan from the top digit down
            const int hi = hist[2047 - 2 * tid], lo = hist[2046 - 2 * tid];
            int v = hi + lo;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                int t = __shfl_up(v, o, 64);
                if (lane >= o) v += t;
            }
            if (lane == 63) wave_tot[wv] = v;
            __syncthreads();
            int add = 0;
            for (int q = 0; q < wv; q++) add += wave_tot[q];
            const int incl = v + add, excl = incl - hi - lo;
            if (excl < krem && incl >= krem) {
                if (excl + hi >= krem) { sel_digit = 2047 - 2 * tid; sel_krem = krem - excl; sel_cnt = hi; }
                else { sel_digit = 2046 - 2 * tid; sel_krem = krem - excl - hi; sel_cnt = lo; }
            }
            __syncthreads();
            prefix = (prefix << w) | (unsigned long long)sel_digit;
            krem = sel_krem;
            shift = nshift;
            const int cnt = sel_cnt;
            __syncthreads();
            if (cnt == krem || shift == 0) break;  // uniform: all threads read the same shared values
        }
        if (tid == 0) out_cnt = 0;
        for (int i = tid; i < kp; i += SELB_THREADS) skeys[i] = 0ull;
        __syncthreads();
        for (int64_t i = tid; i < ncand; i += SELB_THREADS) {
            unsigned long long key = src[i];
            if ((key >> shift) >= prefix) {
                int p = atomicAdd(&out_cnt, 1);
                if (p < kp) skeys[p] = key;
            }
        }
        __syncthreads();
        bitonic_sort_desc(skeys, kp);
    }

    for (int j = tid; j < k; j += SELB_THREADS) {
        const unsigned long long key = skeys[j];
        const uint32_t flat = 0xFFFFFFFFu - (uint32_t)(key & 0xFFFFFFFFull);
        const int par = (int)(flat / (uint32_t)V), tk = (int)(flat % (uint32_t)V);
        parent[b * k + j] = par;
        tok[b * k + j] = tk;
        score[b * k + j] = key_score((uint32_t)(key >> 32));
        if (sid_new) {
            for (int t = 0; t < level; t++) sid_new[(b * k + j) * T + t] = sid_old[(b * n + par) * T + t];
            sid_new[(b * k + j) * T + level] = tk;
            for (int t = level + 1; t < T; t++) sid_new[(b * k + j) * T + t] = 0;
        }
    }
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t select_workspace_bytes(int B, int n, int V, int k) {
    int m = k < V ? k : V;
    return align256((size_t)B * n * m * sizeof(unsigned long long));
}

int launch_select(const float *logits, const float *cum, int B, int n, int V, int k, void *ws, size_t ws_bytes, int32_t *parent,
                  int32_t *tok, float *score, const int32_t *sid_old, int32_t *sid_new, int T, int level, hipStream_t st) {
    if (B <= 0 || n <= 0 || V <= 0 || k <= 0 || (int64_t)k > (int64_t)n * V) return GR4AD_EINVAL;
    if (k > GR4AD_MAX_BEAM || V > GR4AD_MAX_CODEBOOK || (int64_t)n * V >= 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    if (ws_bytes < select_workspace_bytes(B, n, V, k) || ((uintptr_t)ws % 8)) return GR4AD_EWORKSPACE;
    const int m = k < V ? k : V;
    const int64_t rows = (int64_t)B * n;
    if (rows > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    static bool attr_done = false;  // rows of up to GR4AD_MAX_CODEBOOK floats exceed the default dynamic LDS limit
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)select_rows, hipFuncAttributeMaxDynamicSharedMemorySize, GR4AD_MAX_CODEBOOK * 4) != hipSuccess) return GR4AD_EHIP;
        attr_done = true;
    }
    {
        ProfScope ps(KC_SELECT_ROWS, st);
        hipLaunchKernelGGL(select_rows, dim3((unsigned)rows), dim3(256), (size_t)V * 4, st, logits, cum, n, V, m, (unsigned long long *)ws);
    }
    GR4AD_LAUNCH_CHECK();
    ProfScope ps(KC_SELECT_REQUEST, st);
    hipLaunchKernelGGL(select_request, dim3((unsigned)B), dim3(SELB_THREADS), 0, st, (const unsigned long long *)ws, (int64_t)n * m, V, k,
                       parent, tok, score, sid_old, sid_new, n, T, level);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}
