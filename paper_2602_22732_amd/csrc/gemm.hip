// GEMM kernels: C[M,N] = A[M,K] * W[N,K]^T with fused epilogue.
//
// Every linear map of the decoder (section 3.2: the projections of the
// cross-/self-attention and feed-forward sub-layers, the Fuse projection
// and the per-level classifier W_t) is this contraction: activations are
// row-major with the reduction index contiguous, and so are the weights
// ([out,in]), so both MFMA operands stream K-contiguous 16-byte chunks.
//
//  * gemm_simple<T>      64x64 tile, plain FMA, any shape; float32 path and fallback.
//  * gemm_bf16_mfma<..>  bf16 operands, fp32 accumulation on the matrix cores with
//                        v_mfma_f32_32x32x16_bf16; LDS double buffering with an
//                        XOR swizzle of 16-byte chunks; XCD-aware tile order.
#include "common.h"

// ---------------------------------------------------------------------------
// epilogue of one element (plain kernel)
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmEpilogue &e, int64_t row, int col, int N, float v) {
    if (e.bias) v += e.bias[col];
    if (e.table) {
        int64_t tr = e.tok ? (int64_t)e.tok[row] : 0;
        v += e.table[tr * N + col];
    }
    if (e.act == ACT_SILU) v = v / (1.0f + __expf(-v));
    if (e.resid) v += e.resid[row * e.ldr + col];
    if (e.out_f32)
        ((float *)e.C)[row * e.ldc + col] = v;
    else
        ((T *)e.C)[row * e.ldc + col] = from_f<T>(v);
}

// ---------------------------------------------------------------------------
// plain FMA kernel
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gemm_simple(const T *__restrict__ A, int64_t lda, const T *__restrict__ W, int64_t ldw,
                                                   int64_t M, int N, int K, GemmEpilogue epi) {
    __shared__ float As[16][65], Ws[16][65];
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int64_t m0 = (int64_t)blockIdx.x * 64;
    const int n0 = blockIdx.y * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            int idx = tid + i * 256, r = idx / 16, kk = idx % 16;
            int64_t gr = m0 + r;
            int gk = k0 + kk;
            As[kk][r] = (gr < M && gk < K) ? to_f(A[gr * lda + gk]) : 0.0f;
            int gn = n0 + r;
            Ws[kk][r] = (gn < N && gk < K) ? to_f(W[(int64_t)gn * ldw + gk]) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; kk++) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; i++) { a[i] = As[kk][ty * 4 + i]; w[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            int64_t row = m0 + ty * 4 + i;
            int col = n0 + tx * 4 + j;
            if (row < M && col < N) epilogue_store<T>(epi, row, col, N, acc[i][j]);
        }
}

// ---------------------------------------------------------------------------
// MFMA kernel (bf16)
// ---------------------------------------------------------------------------
// Block tile BM x BN, wave tile WM x WN, BK = 64 (one 128-byte row of bf16 per
// tile row = 8 chunks of 16 bytes).  LDS holds two stages of (BM + BN) rows.
// Chunk c of row r sits at slot c ^ ((r >> 1) & 7): the LDS serves 16 lanes x 16 bytes
// per cycle from 64 banks, and the 16 rows such a group of lanes reads (or the 2 rows it
// writes) then fall on 16 different 16-byte slots.  The next K tile travels
// global -> registers while the current one is multiplied, then registers -> LDS.
enum { EPI_STORE = 0, EPI_SILU, EPI_F32, EPI_F32_RESID, EPI_F32_TABLE };

template <int BM, int BN, int WM, int WN, int KIND>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_mfma(const bf16 *__restrict__ A, int64_t lda,
                                                                             const bf16 *__restrict__ W, int64_t ldw, int64_t M,
                                                                             int N, int K, int64_t tiles_m, int tiles_n,
                                                                             GemmEpilogue epi) {
    constexpr int WAVES_N = BN / WN;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int RPP = NT / 8;  // tile rows covered by one pass of all threads (8 threads per 128-byte row)
    constexpr int A_PASSES = BM / RPP, W_PASSES = BN / RPP;
    constexpr int STAGE_CHUNKS = (BM + BN) * 8;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile/threads mismatch");
    extern __shared__ bf16x8 smem[];  // native vectors: arrays of them stay in registers

    // XCD-aware order: consecutive workgroup ids land on different XCDs (each with
    // its own L2), so give every XCD a contiguous range of tiles; inside the range
    // the N index runs fastest so neighbouring tiles re-read the same rows of A.
    const int64_t total = tiles_m * tiles_n;
    const int64_t per_xcd = (total + 7) / 8;
    const int64_t logical = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (logical >= total) return;
    const int64_t m0 = (logical / tiles_n) * BM;
    const int n0 = (int)(logical % tiles_n) * BN;

    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int lc = tid % 8, lr = tid / 8;

    // global source of this thread's chunks (rows past the end re-read the last row; never stored)
    const bf16 *a_src[A_PASSES];
    const bf16 *w_src[W_PASSES];
#pragma unroll
    for (int i = 0; i < A_PASSES; i++) {
        int64_t r = m0 + lr + i * RPP;
        a_src[i] = A + (r < M ? r : M - 1) * lda + lc * 8;
    }
#pragma unroll
    for (int i = 0; i < W_PASSES; i++) {
        int64_t r = (int64_t)n0 + lr + i * RPP;
        w_src[i] = W + (r < N ? r : N - 1) * ldw + lc * 8;
    }
    // LDS slot of this thread's chunks (same for every stage): row r, chunk lc ^ ((r >> 1) & 7); RPP is a multiple of 16
    const int st_slot = lr * 8 + (lc ^ ((lr >> 1) & 7));

    bf16x8 a_reg[A_PASSES], w_reg[W_PASSES];
#pragma unroll
    for (int i = 0; i < A_PASSES; i++) a_reg[i] = *(const bf16x8 *)(a_src[i]);
#pragma unroll
    for (int i = 0; i < W_PASSES; i++) w_reg[i] = *(const bf16x8 *)(w_src[i]);

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

    {
        bf16x8 *sa = smem, *sw = smem + BM * 8;
#pragma unroll
        for (int i = 0; i < A_PASSES; i++) sa[st_slot + i * RPP * 8] = a_reg[i];
#pragma unroll
        for (int i = 0; i < W_PASSES; i++) sw[st_slot + i * RPP * 8] = w_reg[i];
    }
    __syncthreads();

    const int frow = lane % 32, fhalf = lane / 32;
    // fragment read slots: row r = base + frow, chunk (2*kk + fhalf) ^ ((r >> 1) & 7); tile bases are multiples of 32
    int a_slot[TM], w_slot[TN];
#pragma unroll
    for (int i = 0; i < TM; i++) a_slot[i] = (wm * WM + i * 32 + frow) * 8;
#pragma unroll
    for (int j = 0; j < TN; j++) w_slot[j] = (BM + wn * WN + j * 32 + frow) * 8;
    const int fx = (frow >> 1) & 7;

    const int KT = K / 64;
    for (int kt = 0; kt < KT; kt++) {
        const bool more = kt + 1 < KT;
        if (more) {
            const int k0 = (kt + 1) * 64;
#pragma unroll
            for (int i = 0; i < A_PASSES; i++) a_reg[i] = *(const bf16x8 *)(a_src[i] + k0);
#pragma unroll
            for (int i = 0; i < W_PASSES; i++) w_reg[i] = *(const bf16x8 *)(w_src[i] + k0);
        }
        const bf16x8 *s = smem + (kt & 1) * STAGE_CHUNKS;
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            const int ch = (2 * kk + fhalf) ^ fx;
            bf16x8 af[TM], wf[TN];
#pragma unroll
            for (int i = 0; i < TM; i++) {
                af[i] = s[a_slot[i] + ch];
            }
#pragma unroll
            for (int j = 0; j < TN; j++) {
                wf[j] = s[w_slot[j] + ch];
            }
#pragma unroll
            for (int i = 0; i < TM; i++)
#pragma unroll
                for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            bf16x8 *sa = smem + ((kt + 1) & 1) * STAGE_CHUNKS, *sw = sa + BM * 8;
#pragma unroll
            for (int i = 0; i < A_PASSES; i++) sa[st_slot + i * RPP * 8] = a_reg[i];
#pragma unroll
            for (int i = 0; i < W_PASSES; i++) sw[st_slot + i * RPP * 8] = w_reg[i];
        }
        __syncthreads();
    }

    // Accumulator layout of the 32x32 MFMA: lane -> column lane%32, register v -> row 8*(v/4) + 4*(lane/32) + v%4.
    // For one register the 32 lanes of a half-wave write 32 consecutive columns of one row.
    const int64_t row_base = m0 + wm * WM + 4 * fhalf;
    const int col_base = n0 + wn * WN + frow;
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++) {
            const int col = col_base + j * 32;
            if (col >= N) continue;
            const float bias = (KIND == EPI_F32 && epi.bias) ? epi.bias[col] : 0.0f;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int64_t row = row_base + i * 32 + 8 * (v / 4) + (v % 4);
                if (row >= M) continue;
                float x = acc[i][j][v];
                if (KIND == EPI_STORE) {
                    ((bf16 *)epi.C)[row * epi.ldc + col] = (bf16)x;
                } else if (KIND == EPI_SILU) {
                    ((bf16 *)epi.C)[row * epi.ldc + col] = (bf16)(x / (1.0f + __expf(-x)));
                } else if (KIND == EPI_F32) {
                    ((float *)epi.C)[row * epi.ldc + col] = x + bias;
                } else if (KIND == EPI_F32_RESID) {
                    ((float *)epi.C)[row * epi.ldc + col] = x + epi.resid[row * epi.ldr + col];
                } else {
                    const int64_t tr = epi.tok ? (int64_t)epi.tok[row] : 0;
                    ((float *)epi.C)[row * epi.ldc + col] = x + epi.table[tr * N + col];
                }
            }
        }
}

// Which fused epilogues the MFMA kernel covers; anything else runs on the plain kernel.
static int epilogue_kind(const GemmEpilogue &e) {
    const bool extra = e.bias || e.table || e.resid || e.act != ACT_NONE;
    if (!e.out_f32 && !extra) return EPI_STORE;
    if (!e.out_f32 && e.act == ACT_SILU && !e.bias && !e.table && !e.resid) return EPI_SILU;
    if (e.out_f32 && !e.table && !e.resid && e.act == ACT_NONE) return EPI_F32;
    if (e.out_f32 && e.resid && !e.bias && !e.table && e.act == ACT_NONE) return EPI_F32_RESID;
    if (e.out_f32 && e.table && !e.bias && !e.resid && e.act == ACT_NONE) return EPI_F32_TABLE;
    return -1;
}

template <int BM, int BN, int WM, int WN, int KIND>
static int launch_mfma_kind(const bf16 *A, int64_t lda, const bf16 *W, int64_t ldw, int64_t M, int N, int K, const GemmEpilogue &epi,
                            hipStream_t st) {
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr size_t smem = 2 * (size_t)(BM + BN) * 128;
    auto kern = gemm_bf16_mfma<BM, BN, WM, WN, KIND>;
    static bool attr_done = false;  // one attribute call per instantiation is enough (value never changes)
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess) return GR4AD_EHIP;
        attr_done = true;
    }
    int64_t tiles_m = ceil_div64(M, BM);
    int tiles_n = (N + BN - 1) / BN;
    int64_t total = tiles_m * tiles_n;
    int64_t grid = ceil_div64(total, 8) * 8;
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    {
        ProfScope ps(BM == 256 ? KC_GEMM_256 : KC_GEMM_128, st, 2.0 * (double)M * N * K);
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), smem, st, A, lda, W, ldw, M, N, K, tiles_m, tiles_n, epi);
    }
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

template <int BM, int BN, int WM, int WN>
static int launch_mfma(const bf16 *A, int64_t lda, const bf16 *W, int64_t ldw, int64_t M, int N, int K, int kind, const GemmEpilogue &epi,
                       hipStream_t st) {
    switch (kind) {
        case EPI_STORE: return launch_mfma_kind<BM, BN, WM, WN, EPI_STORE>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_SILU: return launch_mfma_kind<BM, BN, WM, WN, EPI_SILU>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_F32: return launch_mfma_kind<BM, BN, WM, WN, EPI_F32>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_F32_RESID: return launch_mfma_kind<BM, BN, WM, WN, EPI_F32_RESID>(A, lda, W, ldw, M, N, K, epi, st);
        default: return launch_mfma_kind<BM, BN, WM, WN, EPI_F32_TABLE>(A, lda, W, ldw, M, N, K, epi, st);
    }
}

// 0 auto, 1 plain FMA kernel, 2 128x128 tiles, 3 256x256 tiles with 8 wavefronts, 4 256x256 tiles with 4 wavefronts
static int g_gemm_mode = -1;
static int gemm_mode() {
    if (g_gemm_mode < 0) {
        const char *e = getenv("GR4AD_GEMM_MODE");
        g_gemm_mode = e ? atoi(e) : 0;
    }
    return g_gemm_mode;
}

int launch_gemm(gr4ad_dtype dtype, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K,
                const GemmEpilogue &epi, hipStream_t st) {
    if (M <= 0 || N <= 0 || K <= 0) return GR4AD_EINVAL;
    const int mode = gemm_mode();
    const int kind = epilogue_kind(epi);
    if (dtype == GR4AD_BF16 && mode != 1 && kind >= 0 && K % 64 == 0 && lda % 8 == 0 && ldw % 8 == 0 && ((uintptr_t)A % 16) == 0 &&
        ((uintptr_t)W % 16) == 0) {
        const bf16 *a = (const bf16 *)A, *w = (const bf16 *)W;
        const bool big = (M >= 8192 && N >= 256);
        if (mode == 4) return launch_mfma<256, 256, 128, 128>(a, lda, w, ldw, M, N, K, kind, epi, st);
        if ((mode == 0 && big) || mode == 3) return launch_mfma<256, 256, 128, 64>(a, lda, w, ldw, M, N, K, kind, epi, st);
        return launch_mfma<128, 128, 64, 64>(a, lda, w, ldw, M, N, K, kind, epi, st);
    }
    dim3 grid((unsigned)ceil_div64(M, 64), (unsigned)((N + 63) / 64));
    if (ceil_div64(M, 64) > 0x7fffffffLL || grid.y > 65535) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_GEMM_SIMPLE, st, 2.0 * (double)M * N * K);
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(gemm_simple<bf16>, grid, dim3(256), 0, st, (const bf16 *)A, lda, (const bf16 *)W, ldw, M, N, K, epi);
    else
        hipLaunchKernelGGL(gemm_simple<float>, grid, dim3(256), 0, st, (const float *)A, lda, (const float *)W, ldw, M, N, K, epi);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}
