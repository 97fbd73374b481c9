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
//  * gemm_bf16_ring<..>  the kernel of the large shapes: persistent, 256x256 tiles,
//                        operands stream global -> LDS without passing registers.
#include <string.h>

#include "common.h"

// An FP8 operand byte (OCP E4M3: sign, 4 exponent bits with bias 7, 3 mantissa bits), decoded in software by the plain kernel.
struct fp8e4m3 { uint8_t v; };
__device__ __forceinline__ float to_f(fp8e4m3 x) {
    const int e = (x.v >> 3) & 15, m = x.v & 7;
    const float a = e ? ldexpf((float)(8 + m), e - 10) : ldexpf((float)m, -9);
    return (x.v & 0x80) ? -a : a;
}

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
// T: operand type; TO: type of C when it is not float32.  FP8 operands: the product row is scaled by a_scale[row] * w_scale.
template <typename T, typename TO = T>
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
            if (row < M && col < N) {
                float v = acc[i][j];
                if (epi.a_scale) v *= epi.a_scale[row] * epi.w_scale;
                epilogue_store<TO>(epi, row, col, N, v);
            }
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
enum { EPI_STORE = 0, EPI_SILU, EPI_F32, EPI_F32_RESID, EPI_F32_TABLE, EPI_VT };  // EPI_VT: persistent kernel only

// bytes a bf16 GEMM must move once: both operands, the output, and the residual it adds
static double gemm_bytes(int64_t M, int N, int K, bool out_f32, bool resid) {
    return 2.0 * ((double)M * K + (double)N * K) + (double)M * N * ((out_f32 ? 4 : 2) + (resid ? 4 : 0));
}

template <int BM, int BN, int WM, int WN, int KIND>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_mfma(const bf16 *__restrict__ A, int64_t lda,
                                                                             const bf16 *__restrict__ W, int64_t ldw, int64_t M,
                                                                             int N, int K, int64_t tiles_m, int tiles_n,
                                                                             GemmEpilogue epi, int64_t batch_a, int64_t batch_w,
                                                                             int64_t batch_c) {
    // blockIdx.y: batch index; the operands and the output of batch i start batch_a/w/c elements further on
    A += (int64_t)blockIdx.y * batch_a;
    W += (int64_t)blockIdx.y * batch_w;
    epi.C = (char *)epi.C + (int64_t)blockIdx.y * batch_c * (KIND >= EPI_F32 ? 4 : 2);
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
    // batched launches may carry a valid length per batch: as a bound on N (columns from it on are never read by the
    // consumer, so tiles wholly beyond it are skipped) or on K (the operands are zero from it on)
    if (epi.batch_len) {
        int len = epi.batch_len[blockIdx.y];
        len = len < 1 ? 1 : len;
        if (epi.len_bounds == 1 && n0 >= len) return;
        if (epi.len_bounds == 2 && len < K) K = (len + 63) / 64 * 64;
    }

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
// Persistent MFMA kernel: 256x256 block tile, BK = 64, ring of five 32 KB half-tiles in LDS
// ---------------------------------------------------------------------------
// One workgroup (8 wavefronts, 2 x 4, wave tile 128 x 64) per compute unit walks a list of output tiles.
// A k-tile is two half-tiles of 256 rows x 128 bytes (one full cache line per row): A(g) and W(g).  The ring holds
// five half-tiles, filled by global_load_lds_dwordx4 (every lane moves 16 bytes straight into LDS; one wave
// instruction fills 8 rows; chunk c of row r sits at position c ^ ((r >> 1) & 7), which keeps both the 1 KB
// writes and the fragment reads conflict-free, and the swizzle is applied on the global side).  In item order
// A0 W0 A1 W1 A2 ... item q lives in slot q % 5.  The bf16 loop requests A(g+2) under the first MFMAs of k-tile g (into
// the slot W(g-1) left at the previous barrier) and W(g+2) under the MFMAs that follow the barrier ending k-tile g (into
// the slot A(g) just left), one load after every second MFMA: a burst of eight loads per wave right after the barrier
// holds up the MFMAs queued behind it.  (The FP8 loop requests W(g+2) and A(g+3) under the four MFMAs after the barrier.)
// The item stream runs on into the next tile of the workgroup, so a tile's first operands arrive while the previous
// tile is still being multiplied and stored.
// Per k-tile: four k-steps of 8 MFMAs; the fragments of step s+1 are read while step s multiplies.  Fragment
// reads are inline assembly so that their waits can be exact (lgkmcnt(6): the six reads just issued may still
// be in flight); one bare s_barrier per k-tile separates "every wave has read A(g), W(g)" from "everybody's
// share of A(g+1), W(g+1) has landed" (each wave waits for its own loads with vmcnt first).
// The MFMA operands are swapped (W fragment first), so a lane owns one row of C and, per group of four
// accumulator registers, four consecutive columns: the epilogue writes 8/16-byte pieces into the two slots the
// last k-tile released (8 KB per wave, rows swizzled) and reads them back as full rows, so C leaves in 16-byte
// pieces with whole cache lines per row.
#define RING_SLOTS 5
#define SLOT_CHUNKS 2048  // 256 rows x 8 chunks of 16 bytes
#define RING_LDS_BYTES (RING_SLOTS * SLOT_CHUNKS * 16)

__device__ __forceinline__ void ring_dma16(const char *g, bf16x8 *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)g,
                                     (void __attribute__((address_space(3))) *)lds_wave_base, 16, 0, 0);
}

__device__ __forceinline__ float fast_silu(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x)); }

// F8: the operands are FP8 (E4M3) bytes instead of bf16.  The byte geometry is unchanged - a k-tile is still 128 bytes per
// row, now 128 values of k - so loads, ring and epilogue are shared; the main loop issues v_mfma_f32_32x32x64_f8f6f4, whose
// 32-byte operand per lane is the two 16-byte fragments the bf16 loop reads for two consecutive k-steps.  (Which of the 64
// values of k a lane holds does not matter as long as both operands agree, and they are read the same way.)  lda, ldw and K
// count elements (bytes).  The product row is scaled by a_scale[row] * w_scale before the epilogue.
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx8 __attribute__((ext_vector_type(8)));

template <int KIND, bool F8 = false>
__global__ __launch_bounds__(512) void gemm_bf16_ring(const bf16 *__restrict__ A, int64_t lda, const bf16 *__restrict__ W, int64_t ldw,
                                                      int64_t M, int N, int K, int64_t tiles_m, int tiles_n, int group_m, GemmEpilogue epi) {
    extern __shared__ bf16x8 smem[];
    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int wm = wave / 4, wn = wave % 4;
    const int frow = lane % 32, hf = lane / 32;
    const int KT = F8 ? K / 128 : K / 64;
    static_assert(!(F8 && KIND == EPI_VT), "the transposed epilogue has no FP8 form");

    // ---- tile schedule: every XCD (workgroup id % 8) owns a contiguous range of logical tiles and its workgroups walk it
    // with stride nslots; inside a group of group_m row blocks the row index runs fastest, so the workgroups of an XCD
    // share a few A blocks and a few W blocks through their L2 at any time ----
    const int64_t total = tiles_m * tiles_n;
    const int nslots = gridDim.x / 8;
    const int xcd = blockIdx.x % 8, wslot = blockIdx.x / 8;
    const int64_t per_xcd = (total + 7) / 8;
    const int64_t xcd_end = (xcd + 1) * per_xcd < total ? (xcd + 1) * per_xcd : total;
    const uint32_t gsz = (uint32_t)group_m * (uint32_t)tiles_n;
    auto tile_coords = [&](int64_t l64, int64_t &m0, int &n0) {  // fewer than 2^31 tiles: 32-bit division
        const uint32_t l = (uint32_t)l64;
        const uint32_t grp = l / gsz, in = l - grp * gsz;
        const uint32_t first_m = grp * (uint32_t)group_m;
        const uint32_t left = (uint32_t)tiles_m - first_m;
        const uint32_t gm = left < (uint32_t)group_m ? left : (uint32_t)group_m;
        const uint32_t nn = in / gm;
        m0 = (int64_t)(first_m + (in - nn * gm)) * 256;
        n0 = (int)nn * 256;
    };
    // Rows of A beyond a request's valid length (epi.skip_len[b] of every skip_S rows) are padding nobody reads the product
    // of: a tile whose 256 rows all lie in one request's padding is passed over.
    auto tile_live = [&](int64_t l) -> bool {
        if (!epi.skip_len) return true;
        int64_t tm0;
        int tn0;
        tile_coords(l, tm0, tn0);
        const uint32_t r0 = (uint32_t)tm0, rows_per = (uint32_t)epi.skip_S;
        const uint32_t b0 = r0 / rows_per, b1 = (r0 + 255u) / rows_per;
        if (b0 != b1) return true;  // straddles two requests
        int len = epi.skip_len[b0];
        len = len < 1 ? 1 : len;
        return r0 - b0 * rows_per < (uint32_t)len;
    };
    auto next_live = [&](int64_t l) {
        while (l < xcd_end && !tile_live(l)) l += nslots;
        return l;
    };
    int64_t L = next_live(xcd * per_xcd + wslot);
    if (L >= xcd_end) return;

    // ---- loads: load j of this wave fills rows (wave*4+j)*8 .. +7 of a half-tile, lane -> row lane/8, position lane%8.
    // The chunk that lives at position p of row r is p ^ ((r >> 1) & 7), and (r >> 1) & 7 = 4*(j&1) + (lane/8 >> 1).
    // Per tile: a wave-uniform base pointer (row block; a k-tile adds 128 bytes) and the last valid row of the block (rows
    // past the matrix edge re-read it).  The lane's byte offset - clamped row times the pitch plus the chunk - is computed
    // when the load is issued (three vector instructions that run beside the MFMAs) instead of being kept per tile. ----
    const int dma_row0 = wave * 32 + lane / 8;
    const uint32_t cb0 = (uint32_t)(((lane % 8) ^ ((lane / 8) >> 1)) * 16), cb1 = cb0 ^ 64u;
    const uint32_t lda2 = (uint32_t)lda * (F8 ? 1 : 2), ldw2 = (uint32_t)ldw * (F8 ? 1 : 2);  // row pitches in bytes
    int64_t m0, m0n = 0;
    int n0, n0n = 0;
    tile_coords(L, m0, n0);
    int64_t Lnext = next_live(L + nslots);
    bool has_next = Lnext < xcd_end;
    if (has_next) tile_coords(Lnext, m0n, n0n);
    const char *baseA, *baseW, *baseAn, *baseWn;
    int maxa, maxw, maxan, maxwn;
    auto tile_sources = [&](int64_t tm0, int tn0, const char *&bA, const char *&bW, int &mA, int &mW) {
        bA = (const char *)A + tm0 * lda2;
        bW = (const char *)W + (int64_t)tn0 * ldw2;
        mA = (int)(M - 1 - tm0 < 255 ? M - 1 - tm0 : 255);
        mW = N - 1 - tn0 < 255 ? N - 1 - tn0 : 255;
    };
    tile_sources(m0, n0, baseA, baseW, maxa, maxw);
    // Without a next tile the loads that would fetch its first k-tiles re-read the current tile's instead (valid memory, into
    // slots nobody reads again and the epilogue does not stage in; all of them have landed at the tile's last barrier): the
    // load sequence stays free of branches, which the register allocation of this kernel depends on.
    baseAn = baseA; baseWn = baseW; maxan = maxa; maxwn = maxw;
    if (has_next) tile_sources(m0n, n0n, baseAn, baseWn, maxan, maxwn);
    // piece j (8 rows) of this wave's share of a half-tile
    auto load_piece = [&](const char *base, int mx, uint32_t pitch, bf16x8 *dst, int j) {
        const int r = dma_row0 + j * 8;
        const uint32_t off = (uint32_t)(r < mx ? r : mx) * pitch + ((j & 1) ? cb1 : cb0);
        ring_dma16(base + off, dst + j * 64);
    };
    // k-tile gk of the current tile (gk < KT) or of the workgroup's next tile (gk >= KT)
    auto issue_a = [&](int gk, int slot) {
        const bool cur = gk < KT;
        const char *base = cur ? baseA + gk * 128 : baseAn + (gk - KT) * 128;
        const int mx = cur ? maxa : maxan;
        bf16x8 *dst = smem + slot * SLOT_CHUNKS + wave * 256;
#pragma unroll
        for (int j = 0; j < 4; j++) load_piece(base, mx, lda2, dst, j);
    };
    auto issue_w = [&](int gk, int slot) {
        const bool cur = gk < KT;
        const char *base = cur ? baseW + gk * 128 : baseWn + (gk - KT) * 128;
        const int mx = cur ? maxw : maxwn;
        bf16x8 *dst = smem + slot * SLOT_CHUNKS + wave * 256;
#pragma unroll
        for (int j = 0; j < 4; j++) load_piece(base, mx, ldw2, dst, j);
    };

    // ---- fragments: lane reads row frow of a 32-row block, chunk 2s + hf of k-step s, i.e. position (hf ^ fx) ^ 2s ----
    const int fx = (frow >> 1) & 7;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    const uint32_t a_lane = lds0 + (uint32_t)((wm * 128 + frow) * 8 + (hf ^ fx)) * 16;
    const uint32_t w_lane = lds0 + (uint32_t)((wn * 64 + frow) * 8 + (hf ^ fx)) * 16;
    auto read_frags = [&](bf16x8 (&af)[4], bf16x8 (&wf)[2], int slot_a, int slot_w, int s) {
        const uint32_t pa = (a_lane ^ (uint32_t)(s << 5)) + (uint32_t)slot_a * 32768u;
        const uint32_t pw = (w_lane ^ (uint32_t)(s << 5)) + (uint32_t)slot_w * 32768u;
        asm volatile("ds_read_b128 %0, %1" : "=v"(af[0]) : "v"(pa));
        asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(af[1]) : "v"(pa));
        asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(af[2]) : "v"(pa));
        asm volatile("ds_read_b128 %0, %1 offset:12288" : "=v"(af[3]) : "v"(pa));
        asm volatile("ds_read_b128 %0, %1" : "=v"(wf[0]) : "v"(pw));
        asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(wf[1]) : "v"(pw));
    };
    // the fragments are operands of the wait, so nothing that uses them can move above it
    auto wait_frags = [&](bf16x8 (&af)[4], bf16x8 (&wf)[2], bool all) {
        if (all) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(af[0]), "+v"(af[1]), "+v"(af[2]), "+v"(af[3]), "+v"(wf[0]), "+v"(wf[1]));
        else asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(af[0]), "+v"(af[1]), "+v"(af[2]), "+v"(af[3]), "+v"(wf[0]), "+v"(wf[1]));
    };
    floatx16 acc[4][2];
    auto mma = [&](const bf16x8 (&af)[4], const bf16x8 (&wf)[2]) {
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) {
                // EPI_VT wants C transposed: with the operands in natural order a lane owns one column of C and four consecutive rows
                if (KIND == EPI_VT) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[i][j], 0, 0, 0);
            }
    };

    // the eight MFMAs of a step with the four direct loads of one half-tile between them, one after every second MFMA: a burst of
    // loads right after the barrier would hold up the MFMAs behind it while the loads queue
    auto mma_dma = [&](const bf16x8 (&af)[4], const bf16x8 (&wf)[2], bool doit, const char *base, int mx, uint32_t pitch, bf16x8 *dst) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
#pragma unroll
            for (int j = 0; j < 2; j++) {
                if (KIND == EPI_VT) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[i][j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (doit) load_piece(base, mx, pitch, dst, i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // ---- FP8 main loop pieces.  One register set: operand i of A (rows i*32..) and j of W are 32 bytes per lane, the chunks
    // 2u and 2u+1 of k-step u (two per k-tile).  The MFMAs of a step run W-block-major, (0,0) (1,0) (2,0) (3,0) (0,1) .. (3,1);
    // as soon as the last MFMA that uses an operand has been issued its registers take the next step's data, so the twelve
    // reads of a step are spread under the step before it: W0 after (3,0), A_i after (i,1), W1 after (3,1). ----
    intx8 A8[4], W8[2];
#define LD8(dst, base, u, OFF)                                                                                     \
    do {                                                                                                           \
        intx4 lo_, hi_;                                                                                            \
        asm volatile("ds_read_b128 %0, %1 offset:" #OFF : "=v"(lo_) : "v"((base) ^ (uint32_t)((u) << 6)));          \
        asm volatile("ds_read_b128 %0, %1 offset:" #OFF : "=v"(hi_) : "v"((base) ^ (uint32_t)(((u) << 6) | 32))); \
        dst = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);                                           \
    } while (0)
#define WAIT8(N, a, w) asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(a), "+v"(w))
#define MMA8(i, j) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(W8[j], A8[i], acc[i][j], 0, 0, 0, 0, 0, 0)
    auto load_step8 = [&](int slot_a, int slot_w, int u) {  // all twelve reads of a step, in the order the waits of a step assume
        const uint32_t pa = a_lane + (uint32_t)slot_a * 32768u, pw = w_lane + (uint32_t)slot_w * 32768u;
        LD8(W8[0], pw, u, 0);
        LD8(A8[0], pa, u, 0);
        LD8(A8[1], pa, u, 4096);
        LD8(A8[2], pa, u, 8192);
        LD8(A8[3], pa, u, 12288);
        LD8(W8[1], pw, u, 4096);
    };

    // ---- prologue: A(0) W(0) A(1) W(1) (and A(2) for the FP8 loop) into slots 0..4 (at least three k-tiles, so all belong to the first tile) ----
    issue_a(0, 0);
    issue_w(0, 1);
    issue_a(1, 2);
    issue_w(1, 3);
    if (F8) {
        issue_a(2, 4);
        asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    } else {  // (the bf16 loop requests A(2) under its first MFMAs)
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    bf16x8 fa0[4], fw0[2], fa1[4], fw1[2];
    int sa = 0;  // slot of A(g); W(g) sits in the next slot
    if (F8) load_step8(0, 1, 0);
    else read_frags(fa0, fw0, 0, 1, 0);

#define SB __builtin_amdgcn_sched_barrier(0)
    for (;;) {  // tiles of this workgroup
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;
        float rinv[4] = {1.0f, 1.0f, 1.0f, 1.0f};
        floatx4 bias4 = {0.0f, 0.0f, 0.0f, 0.0f};  // EPI_F32: bias of this lane's four columns in the epilogue's read-back layout
        if (KIND != EPI_VT && (F8 || epi.row_inv)) {
            const float *rs = F8 ? epi.a_scale : epi.row_inv;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int64_t row = m0 + wm * 128 + i * 32 + frow;
                rinv[i] = rs[row < M ? row : M - 1] * (F8 ? epi.w_scale : 1.0f);
            }
        }
        if (F8) {
            for (int kt = 0; kt < KT; kt++) {
                const int sw = sa + 1 >= RING_SLOTS ? sa + 1 - RING_SLOTS : sa + 1;
                const uint32_t pa = a_lane + (uint32_t)sa * 32768u, pw = w_lane + (uint32_t)sw * 32768u;
                // step 0: its reads are in flight in the order W0 A0 A1 A2 A3 W1 (two each)
                SB; WAIT8(8, A8[0], W8[0]); MMA8(0, 0); SB;
                WAIT8(6, A8[1], W8[0]); MMA8(1, 0); SB;
                WAIT8(4, A8[2], W8[0]); MMA8(2, 0); SB;
                WAIT8(2, A8[3], W8[0]); MMA8(3, 0); SB;
                LD8(W8[0], pw, 1, 0); SB;
                WAIT8(2, A8[0], W8[1]); MMA8(0, 1); SB;
                LD8(A8[0], pa, 1, 0); SB;
                MMA8(1, 1); SB;
                LD8(A8[1], pa, 1, 4096); SB;
                MMA8(2, 1); SB;
                LD8(A8[2], pa, 1, 8192); SB;
                MMA8(3, 1); SB;
                LD8(A8[3], pa, 1, 12288);
                LD8(W8[1], pw, 1, 4096); SB;
                // step 1
                WAIT8(8, A8[0], W8[0]); MMA8(0, 0); SB;
                WAIT8(6, A8[1], W8[0]); MMA8(1, 0); SB;
                WAIT8(4, A8[2], W8[0]); MMA8(2, 0); SB;
                WAIT8(2, A8[3], W8[0]); MMA8(3, 0); SB;
                // every read of A(g), W(g) has been issued; once they have returned and this wave's share of A(g+1), W(g+1) has
                // landed, the barrier releases the two slots (only A(g+2) may stay in flight)
                WAIT8(0, A8[0], W8[1]);
                if (kt + 2 < KT || has_next) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                const int sa1 = sa + 2 >= RING_SLOTS ? sa + 2 - RING_SLOTS : sa + 2;
                const int sw1 = sa + 3 >= RING_SLOTS ? sa + 3 - RING_SLOTS : sa + 3;
                const uint32_t pa1 = a_lane + (uint32_t)sa1 * 32768u, pw1 = w_lane + (uint32_t)sw1 * 32768u;
                const bool more = kt + 1 < KT;  // (a next tile's first operands are read after the epilogue: it needs the registers)
                SB; if (more) LD8(W8[0], pw1, 0, 0); SB;
                if (KIND == EPI_F32 && kt + 2 == KT && epi.bias) {  // see the bf16 loop
                    const int c0 = n0 + wn * 64 + (lane % 16) * 4;
                    const float *src = epi.bias + (c0 + 3 < N ? c0 : 0);
                    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(bias4) : "v"(src) : "memory");
                }
                // the two slots just released take W(g+2) and A(g+3), two loads after each MFMA (not in one burst, which would hold
                // up the MFMAs queued behind it)
                const int gw = kt + 2, ga = kt + 3;
                const char *srcw = gw < KT ? baseW + gw * 128 : baseWn + (gw - KT) * 128;
                const char *srca = ga < KT ? baseA + ga * 128 : baseAn + (ga - KT) * 128;
                const int mxw = gw < KT ? maxw : maxwn, mxa = ga < KT ? maxa : maxan;
                bf16x8 *dstw = smem + sa * SLOT_CHUNKS + wave * 256, *dsta = smem + sw * SLOT_CHUNKS + wave * 256;
                SB; MMA8(0, 1); SB;
                if (more) { LD8(A8[0], pa1, 0, 0); load_piece(srcw, mxw, ldw2, dstw, 0); load_piece(srcw, mxw, ldw2, dstw, 1); } SB;
                MMA8(1, 1); SB;
                if (more) { LD8(A8[1], pa1, 0, 4096); load_piece(srcw, mxw, ldw2, dstw, 2); load_piece(srcw, mxw, ldw2, dstw, 3); } SB;
                MMA8(2, 1); SB;
                if (more) { LD8(A8[2], pa1, 0, 8192); load_piece(srca, mxa, lda2, dsta, 0); load_piece(srca, mxa, lda2, dsta, 1); } SB;
                MMA8(3, 1); SB;
                if (more) { LD8(A8[3], pa1, 0, 12288); LD8(W8[1], pw1, 0, 4096); load_piece(srca, mxa, lda2, dsta, 2); load_piece(srca, mxa, lda2, dsta, 3); } SB;
                if (more) sa = sa1;
            }
        } else
        for (int kt = 0; kt < KT; kt++) {
            const int sw = sa + 1 >= RING_SLOTS ? sa + 1 - RING_SLOTS : sa + 1;
            SB; read_frags(fa1, fw1, sa, sw, 1); wait_frags(fa0, fw0, false); SB;
            {   // A(g+2) into the slot W(g-1) left at the previous barrier
                const int gk = kt + 2;
                const bool cur = gk < KT;
                mma_dma(fa0, fw0, true, cur ? baseA + gk * 128 : baseAn + (gk - KT) * 128, cur ? maxa : maxan, lda2,
                        smem + (sa == 0 ? RING_SLOTS - 1 : sa - 1) * SLOT_CHUNKS + wave * 256);
            }
            SB;
            read_frags(fa0, fw0, sa, sw, 2); wait_frags(fa1, fw1, false); SB;
            mma(fa1, fw1); SB;
            read_frags(fa1, fw1, sa, sw, 3); wait_frags(fa0, fw0, false); SB;
            mma(fa0, fw0); SB;
            // every read of A(g), W(g) has returned; this wave's share of A(g+1), W(g+1) has landed (only A(g+2) may stay in flight)
            wait_frags(fa1, fw1, true);
            if (kt + 2 < KT || has_next) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int sa1 = sa + 2 >= RING_SLOTS ? sa + 2 - RING_SLOTS : sa + 2;
            const int sw1 = sa + 3 >= RING_SLOTS ? sa + 3 - RING_SLOTS : sa + 3;
            SB; if (kt + 1 < KT) read_frags(fa0, fw0, sa1, sw1, 0); SB;  // (a next tile's first fragments are read after the epilogue: it needs the registers)
            if (KIND == EPI_F32 && kt + 2 == KT && epi.bias) {
                // The bias of this lane's four columns (read-back layout of the epilogue) is requested here, just before the
                // tile's last operand loads, by a load the compiler does not track: the wait that ends the last k-tile (all but
                // the four newest loads have landed) covers it.  A tracked load in the epilogue would make the compiler guard
                // the reuse of its registers with a full drain of outstanding loads inside the k-loop.
                const int c0 = n0 + wn * 64 + (lane % 16) * 4;
                const float *src = epi.bias + (c0 + 3 < N ? c0 : 0);
                asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(bias4) : "v"(src) : "memory");
            }
            {   // the slot A(g) left takes W(g+2); after a tile's last k-tile the released slots first stage C
                const int gk = kt + 2;
                const bool cur = gk < KT;
                SB;
                mma_dma(fa1, fw1, kt + 1 < KT, cur ? baseW + gk * 128 : baseWn + (gk - KT) * 128, cur ? maxw : maxwn, ldw2,
                        smem + sa * SLOT_CHUNKS + wave * 256);
                SB;
            }
            if (kt + 1 < KT) sa = sa1;
        }
        // ---- epilogue: slots sa (waves 0..3) and sa+1 (waves 4..7) are free, 8 KB per wave ----
        const int sw = sa + 1 >= RING_SLOTS ? sa + 1 - RING_SLOTS : sa + 1;
        {
            constexpr bool OUT_F32 = KIND >= EPI_F32 && KIND != EPI_VT;
            char *stage = (char *)(smem + (wave < 4 ? sa : sw) * SLOT_CHUNKS) + (wave % 4) * 8192;
            const int64_t wrow0 = m0 + wm * 128;
            const int wcol0 = n0 + wn * 64;
            if (KIND != EPI_VT && (F8 || epi.row_inv)) {
                // folded RMSNorm, reader side: the A operand was gain * x, not yet divided by rms(x); a lane owns row frow of
                // each 32-row block (factors requested at the start of the tile).  FP8 operands: the scales of the row and of W.
#pragma unroll
                for (int i = 0; i < 4; i++)
#pragma unroll
                    for (int j = 0; j < 2; j++)
#pragma unroll
                        for (int v = 0; v < 16; v++) acc[i][j][v] *= rinv[i];
            }
            if (KIND == EPI_VT) {
                // C^T per request: out[(b*N + n) * ldc + s] = C[b*S + s][n] for s < len_b, 0 beyond (values of the context, transposed
                // per head for the attention kernel's second product).  S is a multiple of 64, so the 64 rows of a pass share one request.
                // Two passes of 64 rows: staged as 64 columns x 64 rows (128-byte lines of 8 chunks, chunk c of line r at c ^ (r & 7)).
#pragma unroll
                for (int pass = 0; pass < 2; pass++) {
#pragma unroll
                    for (int ii = 0; ii < 2; ii++)
#pragma unroll
                        for (int j = 0; j < 2; j++) {
                            const int r = j * 32 + frow;
#pragma unroll
                            for (int g = 0; g < 4; g++) {
                                bf16x4 pk;
#pragma unroll
                                for (int e = 0; e < 4; e++) pk[e] = (bf16)acc[pass * 2 + ii][j][4 * g + e];
                                const int c = ii * 4 + g;
                                *(bf16x4 *)(stage + r * 128 + ((c ^ (r & 7)) * 16) + hf * 8) = pk;
                            }
                        }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    const int64_t t0 = wrow0 + pass * 64;  // first of the 64 rows (tokens) of this pass
                    if (t0 < M) {
                        const int64_t b = t0 / epi.vt_S;
                        const int s0 = (int)(t0 - b * epi.vt_S);
                        int len = epi.ctx_len ? epi.ctx_len[b] : epi.vt_S;
                        len = len < 1 ? 1 : (len > epi.vt_S ? epi.vt_S : len);
#pragma unroll 4
                        for (int it = 0; it < 8; it++) {
                            const int r = it * 8 + lane / 8, c = lane % 8;
                            bf16x8 x = *(const bf16x8 *)(stage + r * 128 + ((c ^ (r & 7)) * 16));
                            const int col = wcol0 + r, s = s0 + c * 8;
#pragma unroll
                            for (int e = 0; e < 8; e++) if (s + e >= len) x[e] = (bf16)0.0f;
                            if (col < N) __builtin_nontemporal_store(x, (bf16x8 *)((bf16 *)epi.C + (b * N + col) * epi.ldc + s));
                        }
                    }
                    if (pass == 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                }
            } else if (!OUT_F32) {
                // two passes of 64 rows x 64 columns: 128-byte rows of 8 chunks, chunk c of row r at position c ^ (r & 7)
#pragma unroll
                for (int pass = 0; pass < 2; pass++) {
#pragma unroll
                    for (int ii = 0; ii < 2; ii++) {
                        const int r = ii * 32 + frow;
#pragma unroll
                        for (int j = 0; j < 2; j++)
#pragma unroll
                            for (int g = 0; g < 4; g++) {
                                bf16x4 pk;
#pragma unroll
                                for (int e = 0; e < 4; e++) {
                                    const float x = acc[pass * 2 + ii][j][4 * g + e];
                                    pk[e] = (bf16)(KIND == EPI_SILU ? fast_silu(x) : x);
                                }
                                const int c = j * 4 + g;
                                *(bf16x4 *)(stage + r * 128 + ((c ^ (r & 7)) * 16) + hf * 8) = pk;
                            }
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // wave-private region: no barrier needed
                    if (wrow0 + 128 <= M && wcol0 + 64 <= N) {
                        // the wave's block lies inside C (all but the last row and column of tiles): no bounds tests, one running
                        // address, LDS offsets that are instruction immediates (rows it*8 + lane/8: the swizzle only sees lane/8)
                        const char *rd = stage + (lane / 8) * 128 + (((lane % 8) ^ ((lane / 8) & 7)) * 16);
                        bf16 *wr = (bf16 *)epi.C + (wrow0 + pass * 64 + lane / 8) * epi.ldc + wcol0 + (lane % 8) * 8;
#pragma unroll
                        for (int it = 0; it < 8; it++) {
                            __builtin_nontemporal_store(*(const bf16x8 *)(rd + it * 1024), (bf16x8 *)wr);  // C streams out: not re-read before it leaves the caches
                            wr += 8 * epi.ldc;
                        }
                    } else {
#pragma unroll 4
                        for (int it = 0; it < 8; it++) {
                            const int r = it * 8 + lane / 8, c = lane % 8;
                            const bf16x8 x = *(const bf16x8 *)(stage + r * 128 + ((c ^ (r & 7)) * 16));
                            const int64_t row = wrow0 + pass * 64 + r;
                            const int col = wcol0 + c * 8;
                            if (row < M && col < N) {
                                if (col + 7 < N) __builtin_nontemporal_store(x, (bf16x8 *)((bf16 *)epi.C + row * epi.ldc + col));
                                else for (int e = 0; e < 8 && col + e < N; e++) ((bf16 *)epi.C)[row * epi.ldc + col + e] = x[e];
                            }
                        }
                    }
                    if (pass == 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                }
            } else {
                // four passes of 32 rows x 64 columns: 256-byte rows of 16 chunks, chunk c of row r at position c ^ (r & 15).
                // What a pass adds (residual rows, table rows) is requested before its accumulators are staged, all eight
                // 16-byte pieces at once.  (Requesting them a pass ahead changes nothing: at N = K = 1024 these launches move
                // 12-14 bytes per output element and run at the memory system's mixed read/write rate.)
                constexpr bool HAS_ADD = KIND == EPI_F32_RESID || KIND == EPI_F32_TABLE;  // per-row addends; a bias is one vector per lane
                const int erow = lane / 16, ecol = wcol0 + (lane % 16) * 4;
                // folded RMSNorm, writer side (N % 256 == 0: every column exists)
                const bool emit = HAS_ADD && epi.norm_out != nullptr;
                floatx4 gain4 = {0.0f, 0.0f, 0.0f, 0.0f};
                if (emit) {
                    const bf16x4 g4 = *(const bf16x4 *)((const bf16 *)epi.norm_gain + ecol);
#pragma unroll
                    for (int e = 0; e < 4; e++) gain4[e] = (float)g4[e];
                }
                // the wave's block lies inside C (all but the last row and column of tiles): no bounds tests and running addresses
                const bool interior = wrow0 + 128 <= M && wcol0 + 64 <= N;
#pragma unroll
                for (int pass = 0; pass < 4; pass++) {
                    floatx4 adds[8];
                    if (HAS_ADD && interior) {
                        const int64_t row0 = wrow0 + pass * 32 + erow;
                        if (KIND == EPI_F32_RESID) {
                            const float *rp = epi.resid + row0 * epi.ldr + ecol;
#pragma unroll
                            for (int it = 0; it < 8; it++) adds[it] = *(const floatx4 *)(rp + (int64_t)(it * 4) * epi.ldr);
                        } else {
#pragma unroll
                            for (int it = 0; it < 8; it++)
                                adds[it] = *(const floatx4 *)(epi.table + (epi.tok ? (int64_t)epi.tok[row0 + it * 4] : 0) * N + ecol);
                        }
                    } else if (HAS_ADD) {
#pragma unroll
                        for (int it = 0; it < 8; it++) {
                            const int64_t row = wrow0 + pass * 32 + it * 4 + erow;
                            adds[it] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
                            if (row < M && ecol + 3 < N) {
                                if (KIND == EPI_F32_RESID) adds[it] = *(const floatx4 *)(epi.resid + row * epi.ldr + ecol);
                                if (KIND == EPI_F32_TABLE) adds[it] = *(const floatx4 *)(epi.table + (epi.tok ? (int64_t)epi.tok[row] : 0) * N + ecol);
                            }
                        }
                    }
                    const int r = frow;
#pragma unroll
                    for (int j = 0; j < 2; j++)
#pragma unroll
                        for (int g = 0; g < 4; g++) {
                            floatx4 pk;
#pragma unroll
                            for (int e = 0; e < 4; e++) pk[e] = acc[pass][j][4 * g + e];
                            const int c = j * 8 + g * 2 + hf;
                            *(floatx4 *)(stage + r * 256 + ((c ^ (r & 15)) * 16)) = pk;
                        }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    if (interior) {
                        const int64_t row0 = wrow0 + pass * 32 + erow;
                        char *cp = (char *)epi.C + (row0 * epi.ldc + ecol) * (KIND == EPI_F32 && epi.out_f16 ? 2 : 4);
                        const int64_t cstep = (int64_t)4 * epi.ldc * (KIND == EPI_F32 && epi.out_f16 ? 2 : 4);
                        bf16 *np = emit ? (bf16 *)epi.norm_out + row0 * epi.norm_ld + ecol : nullptr;
                        float *ssp = emit ? epi.norm_ss + row0 * (N / 64) + (wcol0 >> 6) : nullptr;
#pragma unroll
                        for (int it = 0; it < 8; it++) {  // (fully unrolled: the addends must stay in registers)
                            const int rr = it * 4 + erow, c = lane % 16;
                            floatx4 x = *(const floatx4 *)(stage + rr * 256 + ((c ^ (rr & 15)) * 16));
                            if (HAS_ADD) x += adds[it];
                            if (emit) {  // (as below)
                                float sq = x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
                                sq += __shfl_xor(sq, 1, 64);
                                sq += __shfl_xor(sq, 2, 64);
                                sq += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sq), 0x114, 0xf, 0xf, true));
                                sq += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sq), 0x118, 0xf, 0xf, true));
                                if (lane % 16 == 15) ssp[(int64_t)(it * 4) * (N / 64)] = sq;
                            }
                            if (KIND == EPI_F32) x += bias4;
                            if (KIND == EPI_F32 && epi.out_f16) {
                                halfx4 hx;
#pragma unroll
                                for (int e = 0; e < 4; e++) hx[e] = (_Float16)x[e];
                                __builtin_nontemporal_store(hx, (halfx4 *)(cp + it * cstep));
                            } else {
                                __builtin_nontemporal_store(x, (floatx4 *)(cp + it * cstep));
                            }
                            if (emit) {
                                bf16x4 nb;
#pragma unroll
                                for (int e = 0; e < 4; e++) nb[e] = (bf16)(x[e] * gain4[e]);
                                *(bf16x4 *)(np + (int64_t)(it * 4) * epi.norm_ld) = nb;
                            }
                        }
                    } else
#pragma unroll
                    for (int it = 0; it < 8; it++) {  // (fully unrolled: the addends must stay in registers)
                        const int rr = it * 4 + erow, c = lane % 16;
                        floatx4 x = *(const floatx4 *)(stage + rr * 256 + ((c ^ (rr & 15)) * 16));
                        const int64_t row = wrow0 + pass * 32 + rr;
                        const int col = ecol;
                        if (HAS_ADD) x += adds[it];  // (zero where the lane stores nothing or takes the slow path below)
                        if (emit) {  // sum of squares over the row's 64 columns in this wave: the 16 lanes of a DPP row
                            float sq = x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
                            sq += __shfl_xor(sq, 1, 64);
                            sq += __shfl_xor(sq, 2, 64);  // every lane: its quad's sum
                            // row_shr:4 then row_shr:8 (lane i takes lane i-4 / i-8 of its row, 0 if there is none): lane 15 of the
                            // row ends with all four quads
                            sq += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sq), 0x114, 0xf, 0xf, true));
                            sq += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sq), 0x118, 0xf, 0xf, true));
                            if (lane % 16 == 15 && row < M) epi.norm_ss[row * (N / 64) + (wcol0 >> 6)] = sq;
                        }
                        if (row < M && col < N) {
                            if (col + 3 < N) {
                                if (KIND == EPI_F32) x += bias4;
                                if (KIND == EPI_F32 && epi.out_f16) {  // logits for the selection: half precision, 8 bytes per lane, 128 per row
                                    halfx4 hx;
#pragma unroll
                                    for (int e = 0; e < 4; e++) hx[e] = (_Float16)x[e];
                                    __builtin_nontemporal_store(hx, (halfx4 *)((_Float16 *)epi.C + row * epi.ldc + col));
                                } else
                                __builtin_nontemporal_store(x, (floatx4 *)((float *)epi.C + row * epi.ldc + col));
                                if (emit) {
                                    bf16x4 nb;
#pragma unroll
                                    for (int e = 0; e < 4; e++) nb[e] = (bf16)(x[e] * gain4[e]);
                                    *(bf16x4 *)((bf16 *)epi.norm_out + row * epi.norm_ld + col) = nb;
                                }
                            } else {
                                for (int e = 0; e < 4 && col + e < N; e++) {
                                    float y = x[e];
                                    if (KIND == EPI_F32 && epi.bias) y += epi.bias[col + e];
                                    if (KIND == EPI_F32_RESID) y += epi.resid[row * epi.ldr + col + e];
                                    if (KIND == EPI_F32_TABLE) y += epi.table[(epi.tok ? (int64_t)epi.tok[row] : 0) * N + col + e];
                                    if (KIND == EPI_F32 && epi.out_f16) ((_Float16 *)epi.C)[row * epi.ldc + col + e] = (_Float16)y;
                                    else ((float *)epi.C)[row * epi.ldc + col + e] = y;
                                }
                            }
                        }
                    }
                    if (pass < 3) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                }
            }
        }
        if (!has_next) break;
        // ---- the next tile becomes current; the staging slots take its W(1) and A(2) ----
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();  // every wave has read its staged rows back before the slots are overwritten
        asm volatile("" ::: "memory");
        L = Lnext;
        m0 = m0n; n0 = n0n; baseA = baseAn; baseW = baseWn;
        maxa = maxan; maxw = maxwn;
        Lnext = next_live(L + nslots);
        has_next = Lnext < xcd_end;
        if (has_next) {  // (else the "next" sources stay on what is now the current tile)
            tile_coords(Lnext, m0n, n0n);
            tile_sources(m0n, n0n, baseAn, baseWn, maxan, maxwn);
        }
        issue_w(1, sa);
        if (F8) issue_a(2, sw);
        sa = sa + 2 >= RING_SLOTS ? sa + 2 - RING_SLOTS : sa + 2;
        // A(0), W(0) of the new tile landed before its predecessor's last barrier
        if (F8) load_step8(sa, sa + 1 >= RING_SLOTS ? sa + 1 - RING_SLOTS : sa + 1, 0);
        else read_frags(fa0, fw0, sa, sa + 1 >= RING_SLOTS ? sa + 1 - RING_SLOTS : sa + 1, 0);
    }
#undef SB
#undef LD8
#undef WAIT8
#undef MMA8
}

template <int KIND, bool F8 = false>
static int launch_ring_kind(const bf16 *A, int64_t lda, const bf16 *W, int64_t ldw, int64_t M, int N, int K, const GemmEpilogue &epi,
                            hipStream_t st) {
    auto kern = gemm_bf16_ring<KIND, F8>;
    static bool attr_done = false;
    static int n_cu = 0;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, RING_LDS_BYTES) != hipSuccess) return GR4AD_EHIP;
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return GR4AD_EHIP;
        n_cu = prop.multiProcessorCount;
        attr_done = true;
    }
    const int64_t tiles_m = ceil_div64(M, 256);
    const int tiles_n = (N + 255) / 256;
    const int64_t total = tiles_m * tiles_n;
    if (total > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    // one workgroup per compute unit (the ring takes the whole LDS), a multiple of the 8 XCDs
    int64_t grid = n_cu / 8 * 8;
    if (grid < 8) grid = 8;
    if (total < grid) grid = ceil_div64(total, 8) * 8;
    {
        const double operand_bytes = F8 ? ((double)M * K + (double)N * K) : 0.0;  // FP8 operands are half the bytes gemm_bytes counts
        ProfScope ps(F8 ? KC_GEMM_RING_F8 : KC_GEMM_RING, st, 2.0 * (double)M * N * K,
                     gemm_bytes(M, N, K, KIND >= EPI_F32 && KIND != EPI_VT && !epi.out_f16, KIND == EPI_F32_RESID) - operand_bytes);
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), RING_LDS_BYTES, st, A, lda, W, ldw, M, N, K, tiles_m, tiles_n, 4, epi);
    }
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// The persistent kernel stores 16-byte pieces: it needs 16-byte aligned rows of C (and of what the epilogue adds),
// at least three k-tiles, and row pitches whose byte offsets inside a 256-row block fit 32 bits.
static bool ring_ok(int kind, int N, int K, int64_t lda, int64_t ldw, const GemmEpilogue &e) {
    const bool f32 = kind >= EPI_F32;
    if (e.skip_len && e.skip_S < 1) return false;
    if (K < 192 || lda >= (1 << 22) || ldw >= (1 << 22)) return false;
    if (e.out_f16 && kind != EPI_F32) return false;
    if (e.ldc % (f32 ? 4 : 8) || ((uintptr_t)e.C % 16)) return false;
    if (kind == EPI_F32 && e.bias && ((uintptr_t)e.bias % 16)) return false;
    if (kind == EPI_F32_RESID && (e.ldr % 4 || ((uintptr_t)e.resid % 16))) return false;
    if (kind == EPI_F32_TABLE && (N % 4 || ((uintptr_t)e.table % 16))) return false;
    if (e.norm_out) {  // folded RMSNorm, producer side
        if ((kind != EPI_F32_RESID && kind != EPI_F32_TABLE) || N % 256 || !e.norm_gain || !e.norm_ss) return false;
        if (e.norm_ld % 4 || ((uintptr_t)e.norm_out % 8) || ((uintptr_t)e.norm_gain % 8)) return false;
    }
    if (e.row_inv && kind == EPI_VT) return false;  // reader side
    return true;
}

static int launch_ring(const bf16 *A, int64_t lda, const bf16 *W, int64_t ldw, int64_t M, int N, int K, int kind, const GemmEpilogue &epi,
                       hipStream_t st) {
    switch (kind) {
        case EPI_STORE: return launch_ring_kind<EPI_STORE>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_SILU: return launch_ring_kind<EPI_SILU>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_F32: return launch_ring_kind<EPI_F32>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_F32_RESID: return launch_ring_kind<EPI_F32_RESID>(A, lda, W, ldw, M, N, K, epi, st);
        case EPI_VT: return launch_ring_kind<EPI_VT>(A, lda, W, ldw, M, N, K, epi, st);
        default: return launch_ring_kind<EPI_F32_TABLE>(A, lda, W, ldw, M, N, K, epi, st);
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
                            hipStream_t st, int batch = 1, int64_t batch_a = 0, int64_t batch_w = 0, int64_t batch_c = 0) {
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
        if (batch < 1 || batch > 65535) return GR4AD_EUNSUPPORTED;
        ProfScope ps(BM == 256 ? KC_GEMM_256 : KC_GEMM_128, st, 2.0 * (double)M * N * K * batch,
                     batch * gemm_bytes(M, N, K, KIND >= EPI_F32, KIND == EPI_F32_RESID));
        hipLaunchKernelGGL(kern, dim3((unsigned)grid, (unsigned)batch), dim3(NT), smem, st, A, lda, W, ldw, M, N, K, tiles_m, tiles_n, epi, batch_a,
                           batch_w, batch_c);
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

// Batched product on the 128x128 MFMA kernel: for i < batch, C_i[M,N] = A_i[M,K] * W_i[N,K]^T with A_i = A + i*batch_a elements etc.
// bf16 operands; C bf16 or (out_f32) float.  Used by the lazy layers' cross-attention in absorbed form (many small products).
// batch_len (may be NULL), len_bounds: 1 = batch i only needs columns n < batch_len[i] of C_i (the rest may stay unwritten),
// 2 = A_i and W_i are zero from column batch_len[i] (rounded up to 64) on, so the K loop stops there.
int launch_gemm_batched(const void *A, int64_t lda, int64_t batch_a, const void *W, int64_t ldw, int64_t batch_w, void *C, int64_t ldc,
                        int64_t batch_c, int out_f32, int64_t M, int N, int K, int batch, const int32_t *batch_len, int len_bounds,
                        hipStream_t st) {
    if (M <= 0 || N <= 0 || K <= 0 || K % 64 || lda % 8 || ldw % 8 || batch_a % 8 || batch_w % 8 || ((uintptr_t)A % 16) || ((uintptr_t)W % 16))
        return GR4AD_EUNSUPPORTED;
    GemmEpilogue e;
    memset(&e, 0, sizeof(e));
    e.C = C;
    e.ldc = ldc;
    e.out_f32 = out_f32;
    e.batch_len = batch_len;
    e.len_bounds = batch_len ? len_bounds : 0;
    const bf16 *a = (const bf16 *)A, *w = (const bf16 *)W;
    if (M <= 64) {  // few rows per batch: 64-row tiles waste no matrix-core work
        if (out_f32) return launch_mfma_kind<64, 128, 32, 64, EPI_F32>(a, lda, w, ldw, M, N, K, e, st, batch, batch_a, batch_w, batch_c);
        return launch_mfma_kind<64, 128, 32, 64, EPI_STORE>(a, lda, w, ldw, M, N, K, e, st, batch, batch_a, batch_w, batch_c);
    }
    if (out_f32) return launch_mfma_kind<128, 128, 64, 64, EPI_F32>(a, lda, w, ldw, M, N, K, e, st, batch, batch_a, batch_w, batch_c);
    return launch_mfma_kind<128, 128, 64, 64, EPI_STORE>(a, lda, w, ldw, M, N, K, e, st, batch, batch_a, batch_w, batch_c);
}

// Transposed-per-request product for the context values: out[(b*N + n) * ld_out + s] = sum_k A[b*S + s][k] * W[n][k] for
// s < len_b, 0 for len_b <= s < S.  Only the persistent kernel does this; false = shape not covered (caller takes another route).
bool gemm_vt_supported(gr4ad_dtype dtype, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K, int S,
                       const void *out, int64_t ld_out) {
    return dtype == GR4AD_BF16 && K % 64 == 0 && K >= 192 && S % 64 == 0 && M % S == 0 && M >= 256 && N >= 256 && lda % 8 == 0 && ldw % 8 == 0 &&
           lda < (1 << 22) && ldw < (1 << 22) && ((uintptr_t)A % 16) == 0 && ((uintptr_t)W % 16) == 0 && ((uintptr_t)out % 16) == 0 &&
           ld_out % 8 == 0 && ld_out >= S;
}
int launch_gemm_vt(const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K, int S, const int32_t *ctx_len, void *out,
                   int64_t ld_out, hipStream_t st) {
    if (!gemm_vt_supported(GR4AD_BF16, A, lda, W, ldw, M, N, K, S, out, ld_out)) return GR4AD_EUNSUPPORTED;
    GemmEpilogue e;
    memset(&e, 0, sizeof(e));
    e.C = out;
    e.ldc = ld_out;
    e.ctx_len = ctx_len;
    e.vt_S = S;
    e.skip_len = ctx_len;  // key tiles beyond ceil(len / 64) * 64 are never read by the attention kernel
    e.skip_S = S;
    return launch_ring((const bf16 *)A, lda, (const bf16 *)W, ldw, M, N, K, EPI_VT, e, st);
}

// ---------------------------------------------------------------------------
// FP8 products: C = (a_scale[row] * w_scale) * Aq Wq^T with the same epilogues (Aq, Wq: E4M3 bytes; C bf16 or float32)
// ---------------------------------------------------------------------------
static bool ring_f8_ok(int kind, int64_t M, int N, int K, int64_t lda, int64_t ldw, const void *A, const void *W, const GemmEpilogue &e) {
    if (kind < 0 || kind == EPI_VT || e.norm_out || e.row_inv) return false;
    // (there is no mid-size FP8 kernel: a few 256-row tiles on the persistent kernel still beat the plain kernel by far)
    if (M < 64 || N < 256 || K % 128 || K < 384 || lda % 16 || ldw % 16 || ((uintptr_t)A % 16) || ((uintptr_t)W % 16)) return false;
    return ring_ok(kind, N, K, lda, ldw, e);
}

bool gemm_f8_on_persistent_kernel(const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K, const GemmEpilogue &epi) {
    return ring_f8_ok(epilogue_kind(epi), M, N, K, lda, ldw, A, W, epi);
}

int launch_gemm_f8(const void *A, int64_t lda, const float *a_scale, const void *W, int64_t ldw, float w_scale, int64_t M, int N, int K,
                   const GemmEpilogue &epi_in, hipStream_t st) {
    if (M <= 0 || N <= 0 || K <= 0 || !A || !W || !a_scale || !(w_scale > 0.0f)) return GR4AD_EINVAL;
    if (epi_in.norm_out || epi_in.row_inv) return GR4AD_EUNSUPPORTED;
    if (epi_in.out_f16 && !gemm_f8_on_persistent_kernel(A, lda, W, ldw, M, N, K, epi_in)) return GR4AD_EUNSUPPORTED;
    GemmEpilogue epi = epi_in;
    epi.a_scale = a_scale;
    epi.w_scale = w_scale;
    const int kind = epilogue_kind(epi);
    if (gemm_f8_on_persistent_kernel(A, lda, W, ldw, M, N, K, epi)) {
        const bf16 *a = (const bf16 *)A, *w = (const bf16 *)W;  // (the kernel's pointer type; it addresses bytes)
        switch (kind) {
            case EPI_STORE: return launch_ring_kind<EPI_STORE, true>(a, lda, w, ldw, M, N, K, epi, st);
            case EPI_SILU: return launch_ring_kind<EPI_SILU, true>(a, lda, w, ldw, M, N, K, epi, st);
            case EPI_F32: return launch_ring_kind<EPI_F32, true>(a, lda, w, ldw, M, N, K, epi, st);
            case EPI_F32_RESID: return launch_ring_kind<EPI_F32_RESID, true>(a, lda, w, ldw, M, N, K, epi, st);
            default: return launch_ring_kind<EPI_F32_TABLE, true>(a, lda, w, ldw, M, N, K, epi, st);
        }
    }
    dim3 grid((unsigned)ceil_div64(M, 64), (unsigned)((N + 63) / 64));
    if (ceil_div64(M, 64) > 0x7fffffffLL || grid.y > 65535) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_GEMM_SIMPLE, st, 2.0 * (double)M * N * K);
    hipLaunchKernelGGL((gemm_simple<fp8e4m3, bf16>), grid, dim3(256), 0, st, (const fp8e4m3 *)A, lda, (const fp8e4m3 *)W, ldw, M, N, K, epi);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// Kernel choice by shape: bf16 products with 16-byte aligned, K-contiguous operands run on the matrix cores - the persistent
// kernel from 8192 rows and 256 columns on (the 256x256 tile kernel where its epilogue does not cover the layout), 128x128
// tiles below that - everything else on the plain kernel.
static bool mfma_ok(gr4ad_dtype dtype, const void *A, int64_t lda, const void *W, int64_t ldw, int K, int kind) {
    return dtype == GR4AD_BF16 && kind >= 0 && K % 64 == 0 && lda % 8 == 0 && ldw % 8 == 0 && ((uintptr_t)A % 16) == 0 && ((uintptr_t)W % 16) == 0;
}

bool gemm_on_persistent_kernel(gr4ad_dtype dtype, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K,
                               const GemmEpilogue &epi) {
    const int kind = epilogue_kind(epi);
    if (M <= 0 || N <= 0 || K <= 0 || !mfma_ok(dtype, A, lda, W, ldw, K, kind)) return false;
    if (epi.skip_len && M > 0x7fffff00LL) return false;  // (the tile test works on 32-bit row numbers)
    return M >= 8192 && N >= 256 && ring_ok(kind, N, K, lda, ldw, epi);
}

int launch_gemm(gr4ad_dtype dtype, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t M, int N, int K,
                const GemmEpilogue &epi, hipStream_t st) {
    if (M <= 0 || N <= 0 || K <= 0) return GR4AD_EINVAL;
    const int kind = epilogue_kind(epi);
    // only the persistent kernel folds the RMSNorm or writes half-precision logits: never drop such a request silently
    if ((epi.norm_out || epi.row_inv || epi.out_f16) && !gemm_on_persistent_kernel(dtype, A, lda, W, ldw, M, N, K, epi)) return GR4AD_EUNSUPPORTED;
    if (mfma_ok(dtype, A, lda, W, ldw, K, kind)) {
        const bf16 *a = (const bf16 *)A, *w = (const bf16 *)W;
        if (gemm_on_persistent_kernel(dtype, A, lda, W, ldw, M, N, K, epi)) return launch_ring(a, lda, w, ldw, M, N, K, kind, epi, st);
        if (M >= 8192 && N >= 256) return launch_mfma<256, 256, 128, 64>(a, lda, w, ldw, M, N, K, kind, epi, st);
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
