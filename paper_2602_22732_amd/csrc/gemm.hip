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
// epilogue shared by both kernels (one element)
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmEpilogue &e, int64_t row, int col, int N, float v) {
    if (e.bias) v += e.bias[col];
    if (e.table) {
        int64_t tr = e.tok ? (int64_t)e.tok[row] : 0;
        v += ((const float *)e.table)[tr * N + col];
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
// Chunk c of row r sits at slot c ^ (r & 7), so the 32 rows a wave touches in
// one fragment read are spread over all banks.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_mfma(const bf16 *__restrict__ A, int64_t lda,
                                                                             const bf16 *__restrict__ W, int64_t ldw, int64_t M,
                                                                             int N, int K, int64_t tiles_m, int tiles_n,
                                                                             GemmEpilogue epi) {
    constexpr int WAVES_N = BN / WN;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWS_PER_PASS = NT / 8;
    constexpr int A_PASSES = BM / ROWS_PER_PASS, W_PASSES = BN / ROWS_PER_PASS;
    constexpr int STAGE_CHUNKS = (BM + BN) * 8;
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile/threads mismatch");
    extern __shared__ uint4 smem[];

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

    const bf16 *a_ptr[A_PASSES];
    const bf16 *w_ptr[W_PASSES];
#pragma unroll
    for (int i = 0; i < A_PASSES; i++) {
        int64_t r = m0 + lr + i * ROWS_PER_PASS;
        if (r > M - 1) r = M - 1;
        a_ptr[i] = A + r * lda + lc * 8;
    }
#pragma unroll
    for (int i = 0; i < W_PASSES; i++) {
        int64_t r = (int64_t)n0 + lr + i * ROWS_PER_PASS;
        if (r > N - 1) r = N - 1;
        w_ptr[i] = W + r * ldw + lc * 8;
    }
    uint4 a_reg[A_PASSES], w_reg[W_PASSES];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_PASSES; i++) a_reg[i] = *(const uint4 *)(a_ptr[i] + k0);
#pragma unroll
        for (int i = 0; i < W_PASSES; i++) w_reg[i] = *(const uint4 *)(w_ptr[i] + k0);
    };
    auto store_lds = [&](int stage) {
        uint4 *sa = smem + stage * STAGE_CHUNKS, *sw = sa + BM * 8;
#pragma unroll
        for (int i = 0; i < A_PASSES; i++) {
            int r = lr + i * ROWS_PER_PASS;
            sa[r * 8 + (lc ^ (r & 7))] = a_reg[i];
        }
#pragma unroll
        for (int i = 0; i < W_PASSES; i++) {
            int r = lr + i * ROWS_PER_PASS;
            sw[r * 8 + (lc ^ (r & 7))] = w_reg[i];
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

    const int KT = K / 64;
    load_global(0);
    store_lds(0);
    __syncthreads();
    const int frow = lane % 32, fhalf = lane / 32;
    for (int kt = 0; kt < KT; kt++) {
        if (kt + 1 < KT) load_global((kt + 1) * 64);
        const uint4 *sa = smem + (kt & 1) * STAGE_CHUNKS, *sw = sa + BM * 8;
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            bf16x8 af[TM], wf[TN];
#pragma unroll
            for (int i = 0; i < TM; i++) {
                int r = wm * WM + i * 32 + frow;
                uint4 t = sa[r * 8 + ((2 * kk + fhalf) ^ (r & 7))];
                af[i] = *(bf16x8 *)&t;
            }
#pragma unroll
            for (int j = 0; j < TN; j++) {
                int r = wn * WN + j * 32 + frow;
                uint4 t = sw[r * 8 + ((2 * kk + fhalf) ^ (r & 7))];
                wf[j] = *(bf16x8 *)&t;
            }
#pragma unroll
            for (int i = 0; i < TM; i++)
#pragma unroll
                for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // accumulator layout of the 32x32 MFMA: lane -> column lane%32, register v -> row 8*(v/4) + 4*(lane/32) + v%4
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++) {
            int col = n0 + wn * WN + j * 32 + frow;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                int64_t row = m0 + wm * WM + i * 32 + 8 * (v / 4) + 4 * fhalf + (v % 4);
                if (row < M && col < N) epilogue_store<bf16>(epi, row, col, N, acc[i][j][v]);
            }
        }
}

template <int BM, int BN, int WM, int WN>
static int launch_mfma(const bf16 *A, int64_t lda, const bf16 *W, int64_t ldw, int64_t M, int N, int K, const GemmEpilogue &epi,
                       hipStream_t st) {
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr size_t smem = 2 * (size_t)(BM + BN) * 128;
    auto kern = gemm_bf16_mfma<BM, BN, WM, WN>;
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

static int g_gemm_mode = -1;  // 0 auto, 1 force plain FMA kernel, 2 force 128x128 MFMA tiles, 3 force 256x256 (8 waves)
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
    if (dtype == GR4AD_BF16 && mode != 1 && K % 64 == 0 && lda % 8 == 0 && ldw % 8 == 0 && ((uintptr_t)A % 16) == 0 &&
        ((uintptr_t)W % 16) == 0) {
        const bool big = (M >= 8192 && N >= 256);
        if ((mode == 0 && big) || mode == 3)
            return launch_mfma<256, 256, 128, 64>((const bf16 *)A, lda, (const bf16 *)W, ldw, M, N, K, epi, st);
        return launch_mfma<128, 128, 64, 64>((const bf16 *)A, lda, (const bf16 *)W, ldw, M, N, K, epi, st);
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
