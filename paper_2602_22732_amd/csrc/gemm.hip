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

// bytes a bf16 GEMM must move once: both operands, the output, and the residual it adds
static double gemm_bytes(int64_t M, int N, int K, bool out_f32, bool resid) {
    return 2.0 * ((double)M * K + (double)N * K) + (double)M * N * ((out_f32 ? 4 : 2) + (resid ? 4 : 0));
}

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

// ---------------------------------------------------------------------------
// MFMA kernel with a four-stage LDS pipeline fed by direct global->LDS loads
// ---------------------------------------------------------------------------
// 256x256 block tile, 8 wavefronts (wave tile 128x64), BK = 32: a K tile is 512 rows
// of 64 bytes (4 chunks of 16 bytes; chunk c of row r at slot c ^ ((r >> 2) & 3), which
// keeps fragment reads conflict-free).  Four stages of 32 KB sit in LDS.  A K tile is
// fetched by global_load_lds_dwordx4: every lane moves 16 bytes straight into LDS (no
// staging registers, no ds_write); one wave instruction fills 64 consecutive slots
// = 16 tile rows, and the swizzle is applied on the global side (which chunk a lane
// fetches).  Loads run three tiles ahead of the math; the wave waits on its own loads
// with s_waitcnt vmcnt(n) and the workgroup meets at a bare s_barrier (a full fence
// would wait for every load in flight).  The first fragments of the next tile are read
// before the barrier, so the MFMA stream continues across it.
// After the last tile the stages are reused to transpose the accumulators, so that C
// leaves in 16-byte pieces along rows (128 or 256 contiguous bytes per row).
#define PIPE_STAGES 4
#define PIPE_STAGE_CHUNKS 2048  // 512 rows x 4 chunks
#define PIPE_LDS_BYTES (8 * 64 * 288)  // epilogue staging (8 waves x 64 rows x 288 B) >= 4 stages x 32 KB

__device__ __forceinline__ void dma16(const bf16 *g, bf16x8 *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)g,
                                     (void __attribute__((address_space(3))) *)lds_wave_base, 16, 0, 0);
}

template <int KIND>
__global__ __launch_bounds__(512) void gemm_bf16_pipe(const bf16 *__restrict__ A, int64_t lda, const bf16 *__restrict__ W, int64_t ldw,
                                                      int64_t M, int N, int K, int64_t tiles_m, int tiles_n, GemmEpilogue epi) {
    extern __shared__ bf16x8 smem[];
    const int64_t total = tiles_m * tiles_n;
    const int64_t per_xcd = (total + 7) / 8;
    const int64_t logical = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (logical >= total) return;
    const int64_t m0 = (logical / tiles_n) * 256;
    const int n0 = (int)(logical % tiles_n) * 256;
    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int wm = wave / 4, wn = wave % 4;  // 2 x 4 waves, wave tile 128 x 64
    const int frow = lane % 32, fhalf = lane / 32;

    // DMA sources: load j of this wave covers tile rows (wave*4 + j)*16 .. +15, lane -> row + lane/4, slot lane%4
    const bf16 *src[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const int r = (wave * 4 + j) * 16 + lane / 4;  // 0..255: A rows, 256..511: W rows
        const int c = (lane % 4) ^ ((r >> 2) & 3);     // logical chunk that lives in this slot
        if (r < 256) {
            int64_t gr = m0 + r;
            src[j] = A + (gr < M ? gr : M - 1) * lda + c * 8;
        } else {
            int64_t gr = (int64_t)n0 + (r - 256);
            src[j] = W + (gr < N ? gr : N - 1) * ldw + c * 8;
        }
    }
    const int KT = K / 32;
    auto issue = [&](int kt) {  // tile kt -> stage kt % 4
        bf16x8 *base = smem + (kt & 3) * PIPE_STAGE_CHUNKS + wave * 256;
#pragma unroll
        for (int j = 0; j < 4; j++) dma16(src[j] + (int64_t)kt * 32, base + j * 64);
    };

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

    // fragment slots inside a stage: row r, k-step kk: chunk (2*kk + fhalf) ^ ((r >> 2) & 3)
    int a_slot[4], w_slot[2];
#pragma unroll
    for (int i = 0; i < 4; i++) a_slot[i] = (wm * 128 + i * 32 + frow) * 4;
#pragma unroll
    for (int j = 0; j < 2; j++) w_slot[j] = (256 + wn * 64 + j * 32 + frow) * 4;
    const int fx = (frow >> 2) & 3;
    const int ch0 = fhalf ^ fx, ch1 = (2 + fhalf) ^ fx;

    // prologue: three tiles in flight, the first two landed before the first barrier
    issue(0);
    if (KT > 1) issue(1);
    if (KT > 2) issue(2);
    if (KT > 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    bf16x8 af0[4], wf0[2], af1[4], wf1[2];
#pragma unroll
    for (int i = 0; i < 4; i++) af0[i] = smem[a_slot[i] + ch0];
#pragma unroll
    for (int j = 0; j < 2; j++) wf0[j] = smem[w_slot[j] + ch0];

    for (int kt = 0; kt < KT; kt++) {
        const bf16x8 *s = smem + (kt & 3) * PIPE_STAGE_CHUNKS;
        // first k-step: its fragments were read before the barrier, so the MFMAs start at once
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af0[i], wf0[j], acc[i][j], 0, 0, 0);
        // while they run: fragments of the second k-step, and the loads of tile kt+3
#pragma unroll
        for (int i = 0; i < 4; i++) af1[i] = s[a_slot[i] + ch1];
#pragma unroll
        for (int j = 0; j < 2; j++) wf1[j] = s[w_slot[j] + ch1];
        if (kt + 3 < KT) issue(kt + 3);  // stage of tile kt-1: every wave finished reading it before the last barrier
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af1[i], wf1[j], acc[i][j], 0, 0, 0);
        if (kt + 1 < KT) {  // tile kt+1 has been visible since the previous barrier
            const bf16x8 *sn = smem + ((kt + 1) & 3) * PIPE_STAGE_CHUNKS;
#pragma unroll
            for (int i = 0; i < 4; i++) af0[i] = sn[a_slot[i] + ch0];
#pragma unroll
            for (int j = 0; j < 2; j++) wf0[j] = sn[w_slot[j] + ch0];
        }
        // tiles <= kt+2 must have landed before the barrier; only tile kt+3 (4 loads) may stay in flight
        if (kt + 3 < KT) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }

    // ---- epilogue: accumulators -> this wave's LDS region (row-major, padded) -> 16-byte row pieces ----
    constexpr bool OUT_F32 = KIND >= EPI_F32;
    constexpr int PITCH = OUT_F32 ? 288 : 144;        // bytes per staged row of 64 columns
    constexpr int ROWS_PER_PASS = OUT_F32 ? 64 : 128;  // 18 KB per wave and pass
    constexpr int PASSES = 128 / ROWS_PER_PASS;
    constexpr int LANES_PER_ROW = OUT_F32 ? 16 : 8;    // 16-byte pieces per staged row
    char *stage = (char *)smem + wave * (64 * 288);
    const int64_t wrow0 = m0 + wm * 128;
    const int wcol0 = n0 + wn * 64;
#pragma unroll
    for (int pass = 0; pass < PASSES; pass++) {
        // MFMA layout: lane -> column lane%32 of the 32x32 tile, register v -> row 8*(v/4) + 4*(lane/32) + v%4
#pragma unroll
        for (int ii = 0; ii < ROWS_PER_PASS / 32; ii++) {
            const int i = pass * (ROWS_PER_PASS / 32) + ii;
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    const int r = ii * 32 + 8 * (v / 4) + 4 * fhalf + (v % 4), c = j * 32 + frow;
                    if (OUT_F32) *(float *)(stage + r * PITCH + c * 4) = acc[i][j][v];
                    else *(bf16 *)(stage + r * PITCH + c * 2) = (bf16)(KIND == EPI_SILU ? acc[i][j][v] / (1.0f + __expf(-acc[i][j][v])) : acc[i][j][v]);
                }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // wave-private region: no barrier needed
#pragma unroll
        for (int it = 0; it < ROWS_PER_PASS / (64 / LANES_PER_ROW); it++) {
            const int r = it * (64 / LANES_PER_ROW) + lane / LANES_PER_ROW;
            const int piece = lane % LANES_PER_ROW;
            const int64_t row = wrow0 + pass * ROWS_PER_PASS + r;
            const int col = wcol0 + piece * (OUT_F32 ? 4 : 8);
            if (row >= M || col >= N) continue;
            if (OUT_F32) {
                floatx4 x = *(const floatx4 *)(stage + r * PITCH + piece * 16);
                if (col + 3 < N) {
                    floatx4 add = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (KIND == EPI_F32 && epi.bias) add = *(const floatx4 *)(epi.bias + col);
                    if (KIND == EPI_F32_RESID) add = *(const floatx4 *)(epi.resid + row * epi.ldr + col);
                    if (KIND == EPI_F32_TABLE) add = *(const floatx4 *)(epi.table + (epi.tok ? (int64_t)epi.tok[row] : 0) * N + col);
                    *(floatx4 *)((float *)epi.C + row * epi.ldc + col) = x + add;
                } else {
                    for (int e = 0; e < 4 && col + e < N; e++) {
                        float y = x[e];
                        if (KIND == EPI_F32 && epi.bias) y += epi.bias[col + e];
                        if (KIND == EPI_F32_RESID) y += epi.resid[row * epi.ldr + col + e];
                        if (KIND == EPI_F32_TABLE) y += epi.table[(epi.tok ? (int64_t)epi.tok[row] : 0) * N + col + e];
                        ((float *)epi.C)[row * epi.ldc + col + e] = y;
                    }
                }
            } else {
                bf16x8 x = *(const bf16x8 *)(stage + r * PITCH + piece * 16);
                if (col + 7 < N) {
                    *(bf16x8 *)((bf16 *)epi.C + row * epi.ldc + col) = x;
                } else {
                    for (int e = 0; e < 8 && col + e < N; e++) ((bf16 *)epi.C)[row * epi.ldc + col + e] = x[e];
                }
            }
        }
        if (pass + 1 < PASSES) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
}

template <int KIND>
static int launch_pipe_kind(const bf16 *A, int64_t lda, const bf16 *W, int64_t ldw, int64_t M, int N, int K, const GemmEpilogue &epi,
                            hipStream_t st) {
    auto kern = gemm_bf16_pipe<KIND>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, PIPE_LDS_BYTES) != hipSuccess) return GR4AD_EHIP;
        attr_done = true;
    }
    int64_t tiles_m = ceil_div64(M, 256);
    int tiles_n = (N + 255) / 256;
    int64_t grid = ceil_div64(tiles_m * tiles_n, 8) * 8;
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    {
        ProfScope ps(KC_GEMM_PIPE, st, 2.0 * (double)M * N * K, gemm_bytes(M, N, K, KIND >= EPI_F32, KIND == EPI_F32_RESID));
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), PIPE_LDS_BYTES, st, A, lda, W, ldw, M, N, K, tiles_m, tiles_n, epi);
    }
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// The pipelined kernel stores 16-byte pieces: it needs 16-byte aligned rows of C (and of what the epilogue adds).
static bool pipe_ok(int kind, int N, const GemmEpilogue &e) {
    const bool f32 = kind >= EPI_F32;
    if (e.ldc % (f32 ? 4 : 8) || ((uintptr_t)e.C % 16)) return false;
    if (kind == EPI_F32 && e.bias && ((uintptr_t)e.bias % 16)) return false;
    if (kind == EPI_F32_RESID && (e.ldr % 4 || ((uintptr_t)e.resid % 16))) return false;
    if (kind == EPI_F32_TABLE && (N % 4 || ((uintptr_t)e.table % 16))) return false;
    return true;
}

static int launch_pipe(const bf16 *A, int64_t lda, const bf16 *W, int64_t ldw, int64_t M, int N, int K, int kind, const GemmEpilogue &epi,
                       hipStream_t st) {
    switch (kind) {
        case EPI_STORE: return launch_pipe_kind<EPI_STORE>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_SILU: return launch_pipe_kind<EPI_SILU>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_F32: return launch_pipe_kind<EPI_F32>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_F32_RESID: return launch_pipe_kind<EPI_F32_RESID>(A, lda, W, ldw, M, N, K, epi, st);
        default: return launch_pipe_kind<EPI_F32_TABLE>(A, lda, W, ldw, M, N, K, epi, st);
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
        ProfScope ps(BM == 256 ? KC_GEMM_256 : KC_GEMM_128, st, 2.0 * (double)M * N * K, gemm_bytes(M, N, K, KIND >= EPI_F32, KIND == EPI_F32_RESID));
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

// 0 auto, 1 plain FMA kernel, 2 128x128 tiles, 3 256x256 tiles with 8 wavefronts, 4 256x256 tiles with 4 wavefronts,
// 5 pipelined 256x256 kernel
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
        if ((mode == 5 || (mode == 0 && big)) && pipe_ok(kind, N, epi)) return launch_pipe(a, lda, w, ldw, M, N, K, kind, epi, st);
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
