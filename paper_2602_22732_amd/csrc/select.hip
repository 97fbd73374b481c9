// Fused log-softmax + cumulative score + top-k beam selection.
//
// At level t the search keeps the b_t best of the n_t*V_t candidates
// score(i,v) = c_i + log_softmax(z_i)[v] of a request (section 3.2 beam search,
// section 4.2 Dynamic Beam Width).  The selection is two-stage, as TopK Pre-Cut
// (appendix A.2) describes: every beam row first keeps its own min(b_t, V_t)
// best tokens, then the request keeps the b_t best of those.  Both stages are
// exact selections, so the result equals a full sort of all candidates.
// The per-row cut is tightened by a bound per request: the request's first row
// holds its best beam, and that row's own cut already has b_t candidates, so no
// candidate below the worst of them can survive.  The other rows write only what
// reaches that bound (at most their own cut), compacted per request; with beams
// of unequal scores that is a fraction of b_t per row.
//
// Candidates travel between the stages as unique 64-bit keys
//     (order-preserving bits of the fp32 score) << 32 | (0xFFFFFFFF - flat index)
// so "larger key" means "higher score, then lower flat index i*V + v": equal
// scores resolve deterministically and the final order is a plain key sort.
#include <stdlib.h>

#include <algorithm>
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
// The row (V logits) is read once and stays in registers: ITEMS values per thread,
// token v = j*256 + tid.  After the log-sum-exp, the row's min(b_t, V_t) best scores
// are cut out with about two dozen vector operations per logit, so the kernel stays
// bound by the HBM read of the logits:
//   1. a histogram of the scores over ROW_BINS equal-width bins between the row's
//      minimum and maximum (LDS atomics, spread over the bins by the values themselves),
//   2. a scan from the top bin finds the bin T that holds the m-th best score,
//   3. everything above bin T is a candidate; the few scores inside bin T are ranked
//      exactly against each other (64-bit keys, so ties go to the lowest token).
// If bin T is crowded (degenerate rows, e.g. all logits equal) the row falls back to an
// exact radix selection on the score keys that walks two bits at a time and only counts.
#define ROW_BINS 1024
#define ROW_LIST 1024

struct RowShared {
    float f[3][4];
    uint32_t u[2][4][2];
    int wave_tot[4];
    int scan_base, out_gt, out_eq, sel_bin, sel_krem, sel_cnt, list_n;
    int hist[ROW_BINS];
    unsigned long long list[ROW_LIST];
};

__device__ __forceinline__ float block_max_256(float v, RowShared &sh, int slot) {
    v = wave_max(v);
    if (threadIdx.x % 64 == 0) sh.f[slot][threadIdx.x / 64] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh.f[slot][0], sh.f[slot][1]), fmaxf(sh.f[slot][2], sh.f[slot][3]));
}
__device__ __forceinline__ float block_sum_256(float v, RowShared &sh, int slot) {
    v = wave_sum(v);
    if (threadIdx.x % 64 == 0) sh.f[slot][threadIdx.x / 64] = v;
    __syncthreads();
    return (sh.f[slot][0] + sh.f[slot][1]) + (sh.f[slot][2] + sh.f[slot][3]);
}

__device__ __forceinline__ unsigned long long pack_candidate(float score, uint32_t flat) {
    return ((unsigned long long)score_key(score) << 32) | (0xFFFFFFFFu - flat);
}

// Exact fallback: radix selection on the order-preserving keys of the scores held in
// sc[] (padding slots hold -inf and are skipped by the v < V test).
template <int ITEMS>
__device__ __noinline__ void select_row_radix(const float (&sc)[ITEMS], int V, int m, uint32_t flat0, unsigned long long *dst,
                                              RowShared &sh) {
    const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
    uint32_t k_and = 0xFFFFFFFFu, k_or = 0u;
#pragma unroll
    for (int j = 0; j < ITEMS; j++)
        if (j * 256 + tid < V) { const uint32_t k = score_key(sc[j]); k_and &= k; k_or |= k; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        k_and &= __shfl_xor(k_and, o, 64);
        k_or |= __shfl_xor(k_or, o, 64);
    }
    __syncthreads();
    if (lane == 0) { sh.u[0][wv][0] = k_and; sh.u[0][wv][1] = k_or; }
    if (tid == 0) { sh.out_gt = 0; sh.out_eq = 0; }
    __syncthreads();
    k_and = sh.u[0][0][0] & sh.u[0][1][0] & sh.u[0][2][0] & sh.u[0][3][0];
    k_or = sh.u[0][0][1] | sh.u[0][1][1] | sh.u[0][2][1] | sh.u[0][3][1];
    // decided: bits already fixed in `prefix`; a key is still active while (key & decided) == prefix
    const uint32_t diff = k_and ^ k_or;
    uint32_t decided = 0xFFFFFFFFu, prefix = k_and;
    int krem = m, active = V;
    if (diff != 0) {
        const int top = 31 - __clz(diff);
        decided = ~((2u << top) - 1u);  // top == 31 gives 0
        prefix = k_and & decided;
        int slot = 1;
        for (int shb = top & ~1; shb >= 0; shb -= 2) {
            uint32_t c12 = 0, c3 = 0;  // active keys with digit >= 1 (low half), >= 2 (high half), >= 3
#pragma unroll
            for (int j = 0; j < ITEMS; j++) {
                const uint32_t k = score_key(sc[j]);
                const uint32_t d = (k >> shb) & 3u;
                const uint32_t act = (((k ^ prefix) & decided) == 0u && (j * 256 + tid) < V) ? 1u : 0u;
                c12 += (d >= 1u ? act : 0u) + (d >= 2u ? (act << 16) : 0u);
                c3 += d >= 3u ? act : 0u;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                c12 += __shfl_xor(c12, o, 64);
                c3 += __shfl_xor(c3, o, 64);
            }
            if (lane == 0) { sh.u[slot][wv][0] = c12; sh.u[slot][wv][1] = c3; }
            __syncthreads();
            c12 = sh.u[slot][0][0] + sh.u[slot][1][0] + sh.u[slot][2][0] + sh.u[slot][3][0];
            c3 = sh.u[slot][0][1] + sh.u[slot][1][1] + sh.u[slot][2][1] + sh.u[slot][3][1];
            slot ^= 1;  // the next step writes the other slot, so one barrier per step is enough
            const int C1 = (int)(c12 & 0xFFFFu), C2 = (int)(c12 >> 16), C3 = (int)c3;
            uint32_t dsel;
            if (C3 >= krem) { dsel = 3; active = C3; }
            else if (C2 >= krem) { dsel = 2; krem -= C3; active = C2 - C3; }
            else if (C1 >= krem) { dsel = 1; krem -= C2; active = C1 - C2; }
            else { dsel = 0; krem -= C1; active = active - C1; }
            prefix |= dsel << shb;
            decided |= 3u << shb;
            if (active == krem) break;  // every key still active is taken
        }
    }
    // (key & decided) > prefix: above the threshold; == prefix: `active` keys tie at it, krem of them are taken
    const int n_gt = m - krem;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    if (active == krem) {
#pragma unroll
        for (int j = 0; j < ITEMS; j++) {
            const int v = j * 256 + tid;
            const uint32_t kk = score_key(sc[j]) & decided;
            const bool gt = v < V && kk > prefix, eq = v < V && kk == prefix;
            const unsigned long long mg = __ballot(gt), me = __ballot(eq);
            int bg = 0, be = 0;
            if (lane == 0) {
                if (mg) bg = atomicAdd(&sh.out_gt, __popcll(mg));
                if (me) be = atomicAdd(&sh.out_eq, __popcll(me));
            }
            bg = __shfl(bg, 0, 64);
            be = __shfl(be, 0, 64);
            if (gt) dst[bg + __popcll(mg & lt_mask)] = pack_candidate(sc[j], flat0 + (uint32_t)v);
            if (eq) dst[n_gt + be + __popcll(me & lt_mask)] = pack_candidate(sc[j], flat0 + (uint32_t)v);
        }
    } else {
        // more keys tie at the threshold than are needed: take the lowest tokens, in token order
        int base = 0;
#pragma unroll
        for (int j = 0; j < ITEMS; j++) {
            const int v = j * 256 + tid;
            const uint32_t kk = score_key(sc[j]) & decided;
            const bool gt = v < V && kk > prefix;
            const int flag = (v < V && kk == prefix) ? 1 : 0;
            const int incl = block_scan_256(flag, sh.wave_tot);
            if (gt) dst[atomicAdd(&sh.out_gt, 1)] = pack_candidate(sc[j], flat0 + (uint32_t)v);
            const int rank = base + incl - flag;
            if (flag && rank < krem) dst[n_gt + rank] = pack_candidate(sc[j], flat0 + (uint32_t)v);
            if (tid == 255) sh.scan_base = base + incl;
            __syncthreads();
            base = sh.scan_base;
            __syncthreads();
        }
    }
}

template <int ITEMS>
__global__ __launch_bounds__(256) void select_rows(const float *__restrict__ logits, const float *__restrict__ cum, int n, int V, int m,
                                                   unsigned long long *__restrict__ cand) {
    __shared__ RowShared sh;
    extern __shared__ unsigned long long out_stage[];  // m candidates, gathered here and written out in one coalesced sweep
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    const float *z = logits + row * (int64_t)V;
    const float c = cum ? cum[row] : 0.0f;
    for (int i = tid; i < ROW_BINS; i += 256) sh.hist[i] = 0;
    if (tid == 0) { sh.out_gt = 0; sh.list_n = 0; }

    float x[ITEMS];
    float mx = -INFINITY, mn = INFINITY;
#pragma unroll
    for (int j = 0; j < ITEMS; j++) {
        const int v = j * 256 + tid;
        x[j] = v < V ? z[v] : -INFINITY;
        mx = fmaxf(mx, x[j]);
        if (v < V) mn = fminf(mn, x[j]);
    }
    mx = block_max_256(mx, sh, 0);
    mn = -block_max_256(-mn, sh, 1);
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < ITEMS; j++) sum += __expf(x[j] - mx);  // exp(-inf) = 0 for the padding
    const float lse = mx + __logf(block_sum_256(sum, sh, 2));
#pragma unroll
    for (int j = 0; j < ITEMS; j++) x[j] = c + (x[j] - lse);  // scores from here on (padding stays -inf)

    unsigned long long *dst = cand + row * (int64_t)m;
    const uint32_t flat0 = (uint32_t)((row % n) * (int64_t)V);
    if (m >= V) {  // nothing to cut: every token is a candidate
#pragma unroll
        for (int j = 0; j < ITEMS; j++) {
            const int v = j * 256 + tid;
            if (v < V) dst[v] = pack_candidate(x[j], flat0 + (uint32_t)v);
        }
        return;
    }
    // 1. histogram over equal-width bins of [lo, hi]; the bin index is monotone in the score
    const float lo = c + (mn - lse), hi = c + (mx - lse);
    const float inv_w = (hi > lo) ? (float)ROW_BINS / (hi - lo) : 0.0f;
    int bin[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; j++) {
        int bi = (int)((x[j] - lo) * inv_w);
        bi = bi < 0 ? 0 : (bi > ROW_BINS - 1 ? ROW_BINS - 1 : bi);
        bin[j] = bi;
        if (j * 256 + tid < V) atomicAdd(&sh.hist[bi], 1);
    }
    __syncthreads();
    // 2. thread t owns bins 1023-4t .. 1020-4t; inclusive scan from the top bin down
    {
        const int b0 = ROW_BINS - 1 - 4 * tid;
        const int h0 = sh.hist[b0], h1 = sh.hist[b0 - 1], h2 = sh.hist[b0 - 2], h3 = sh.hist[b0 - 3];
        const int incl = block_scan_256(h0 + h1 + h2 + h3, sh.wave_tot);
        int above = incl - (h0 + h1 + h2 + h3);  // scores in bins above this thread's four
        if (above < m && incl >= m) {
            int bsel = b0, cnt = h0;
            if (above + h0 < m) { above += h0; bsel = b0 - 1; cnt = h1;
                if (above + h1 < m) { above += h1; bsel = b0 - 2; cnt = h2;
                    if (above + h2 < m) { above += h2; bsel = b0 - 3; cnt = h3; } } }
            sh.sel_bin = bsel;
            sh.sel_krem = m - above;
            sh.sel_cnt = cnt;
        }
    }
    __syncthreads();
    const int T = sh.sel_bin, krem = sh.sel_krem, cntT = sh.sel_cnt;
    if (cntT > ROW_LIST) {  // crowded threshold bin: exact radix selection over the whole row
        float sc[ITEMS];  // a copy, so that only this branch keeps the scores in addressable memory
#pragma unroll
        for (int j = 0; j < ITEMS; j++) sc[j] = x[j];
        select_row_radix<ITEMS>(sc, V, m, flat0, dst, sh);
        return;
    }
    // 3. bins above T are candidates; bin T goes to the list for exact ranking.  One scan of the
    //    per-thread counts (low half: above T, high half: inside T) gives every thread its slots.
    const int n_gt = m - krem;
    int mine = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; j++) {
        const bool ok = j * 256 + tid < V;
        mine += (ok && bin[j] > T ? 1 : 0) + (ok && bin[j] == T ? (1 << 16) : 0);
    }
    const int incl = block_scan_256(mine, sh.wave_tot);
    int pos_gt = (incl - mine) & 0xFFFF, pos_eq = (incl - mine) >> 16;
#pragma unroll
    for (int j = 0; j < ITEMS; j++) {
        const int v = j * 256 + tid;
        if (v < V && bin[j] > T) out_stage[pos_gt++] = pack_candidate(x[j], flat0 + (uint32_t)v);
        if (v < V && bin[j] == T) sh.list[pos_eq++] = pack_candidate(x[j], flat0 + (uint32_t)v);
    }
    __syncthreads();
    // rank every listed candidate among the cntT listed ones; the krem best go out
    for (int i = tid; i < cntT; i += 256) {
        const unsigned long long mine = sh.list[i];
        int rank = 0;
        for (int q = 0; q < cntT; q++) rank += sh.list[q] > mine ? 1 : 0;
        if (rank < krem) out_stage[n_gt + rank] = mine;
    }
    __syncthreads();
    for (int i = tid; i < m; i += 256) dst[i] = out_stage[i];
}

// ---------------------------------------------------------------------------
// stage A, wavefront form: one wavefront per beam row (V <= 8192)
// ---------------------------------------------------------------------------
// Same cut as select_rows, but a row never leaves one wavefront: no workgroup barrier anywhere, the V logits sit in VEC*4
// registers per lane, read as 16-byte pieces of E = 4 float32 or E = 8 half-precision values (lane l, piece g holds tokens
// (g*64 + l)*E .. +E-1; V % E == 0), every reduction is a wave reduction, and the histogram, the threshold-bin list and the
// staged output live in a private LDS region per wavefront.  The kernel is bound by vector instructions per logit, so the
// common case is kept to a maximum, one exp2 and one comparison per logit: with a request-level bound in force the row is
// swept in the logit domain against a threshold a hair below the exact one, and only the few logits that pass it are turned
// into scores and tested exactly.  Rows that need their own cut (more than m candidates at the bound, or no bound) turn all
// logits into scores, histogram them and rank the threshold bin exactly; score bits are staged raw and turned into sortable
// keys only for the survivors on the way out.
#define WROW_BINS 1024
#define WROW_LIST 512  // threshold-bin candidates ranked exactly; the list reuses the histogram's 4 KB

__device__ __forceinline__ unsigned long long staged_to_key(unsigned long long st) {
    return ((unsigned long long)score_key(__uint_as_float((uint32_t)(st >> 32))) << 32) | (st & 0xFFFFFFFFull);
}

// token held in register i of a lane: piece i / E of the lane, element i % E of the piece
template <int E> __device__ __forceinline__ int wave_tok(int i, int lane) { return ((i / E) * 64 + lane) * E + (i % E); }

// exact fallback on the registers of one wavefront: radix selection on the score keys, two bits per step
template <int VEC, int E>
__device__ __noinline__ void select_row_radix_wave(const float (&sc)[VEC * 4], int V, int m, uint32_t flat0, unsigned long long *stage) {
    const int lane = threadIdx.x % 64;
    uint32_t k_and = 0xFFFFFFFFu, k_or = 0u;
#pragma unroll
    for (int i = 0; i < VEC * 4; i++)
        if (wave_tok<E>(i, lane) < V) { const uint32_t k = score_key(sc[i]); k_and &= k; k_or |= k; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { k_and &= __shfl_xor(k_and, o, 64); k_or |= __shfl_xor(k_or, o, 64); }
    const uint32_t diff = k_and ^ k_or;
    uint32_t decided = 0xFFFFFFFFu, prefix = k_and;
    int krem = m, active = V;
    if (diff != 0) {
        const int top = 31 - __clz(diff);
        decided = ~((2u << top) - 1u);  // top == 31 gives 0
        prefix = k_and & decided;
        for (int shb = top & ~1; shb >= 0; shb -= 2) {
            uint32_t c12 = 0, c3 = 0;  // active keys with digit >= 1 (low half), >= 2 (high half), >= 3
#pragma unroll
            for (int i = 0; i < VEC * 4; i++) {
                const uint32_t k = score_key(sc[i]);
                const uint32_t d = (k >> shb) & 3u;
                const uint32_t act = (((k ^ prefix) & decided) == 0u && wave_tok<E>(i, lane) < V) ? 1u : 0u;
                c12 += (d >= 1u ? act : 0u) + (d >= 2u ? (act << 16) : 0u);
                c3 += d >= 3u ? act : 0u;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) { c12 += __shfl_xor(c12, o, 64); c3 += __shfl_xor(c3, o, 64); }
            const int C1 = (int)(c12 & 0xFFFFu), C2 = (int)(c12 >> 16), C3 = (int)c3;
            uint32_t dsel;
            if (C3 >= krem) { dsel = 3; active = C3; }
            else if (C2 >= krem) { dsel = 2; krem -= C3; active = C2 - C3; }
            else if (C1 >= krem) { dsel = 1; krem -= C2; active = C1 - C2; }
            else { dsel = 0; krem -= C1; active = active - C1; }
            prefix |= dsel << shb;
            decided |= 3u << shb;
            if (active == krem) break;  // every key still active is taken
        }
    }
    // (key & decided) > prefix: above the threshold; == prefix: `active` keys tie there and the krem lowest tokens are taken.
    // Tokens ascend with (piece, lane, element), so a tie's rank is the count of ties in earlier pieces, in lower lanes of
    // this piece, and in lower elements.
    const int n_gt = m - krem;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    int base_gt = 0, base_eq = 0;
#pragma unroll
    for (int g = 0; g < VEC * 4 / E; g++) {
        int my_eq = 0;
        bool gt[E], eq[E];
#pragma unroll
        for (int e = 0; e < E; e++) {
            const bool ok = (g * 64 + lane) * E < V;
            const uint32_t kk = score_key(sc[g * E + e]) & decided;
            gt[e] = ok && kk > prefix;
            eq[e] = ok && kk == prefix;
            my_eq += eq[e] ? 1 : 0;
        }
        int incl = my_eq;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(incl, o, 64); if (lane >= o) incl += t; }
        int rank = base_eq + incl - my_eq;
        base_eq += __shfl(incl, 63, 64);
#pragma unroll
        for (int e = 0; e < E; e++) {
            const unsigned long long mg = __ballot(gt[e]);
            const uint32_t flat = flat0 + (uint32_t)((g * 64 + lane) * E + e);
            const unsigned long long st = ((unsigned long long)__float_as_uint(sc[g * E + e] + 0.0f) << 32) | (0xFFFFFFFFu - flat);
            if (gt[e]) stage[base_gt + __popcll(mg & lt_mask)] = st;
            base_gt += __popcll(mg);
            if (eq[e]) { if (rank < krem) stage[n_gt + rank] = st; rank++; }
        }
    }
}

template <typename LT> struct LogitPiece;  // one 16-byte piece of a row of logits as floats
template <> struct LogitPiece<float> {
    static constexpr int E = 4;
    static __device__ __forceinline__ void unpack(const uint4 &r, float *o) {
        o[0] = __uint_as_float(r.x); o[1] = __uint_as_float(r.y); o[2] = __uint_as_float(r.z); o[3] = __uint_as_float(r.w);
    }
};
template <> struct LogitPiece<_Float16> {
    static constexpr int E = 8;
    static __device__ __forceinline__ void unpack(const uint4 &r, float *o) {
        const halfx8 v = __builtin_bit_cast(halfx8, r);
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = (float)v[e];
    }
};

// The row's own top-m cut.  x[i]: the logit of token wave_tok<E>(i, lane), padding -inf; mx, lse: the row's maximum and
// log-sum-exp; the m best (score, token) pairs go to dst.
template <int VEC, bool FULL, int E>
__device__ __forceinline__ void select_row_own_cut(float (&x)[VEC * 4], float c, float mx, float lse, unsigned long long *__restrict__ dst,
                                                   uint32_t flat0, uint32_t nflat, int V, int m, unsigned long long *list, int lane) {
    constexpr int NX = VEC * 4;
    int *hist = (int *)list;
    unsigned long long *stage = list + 512;
    // scores from here on (padding stays -inf)
    float mn = INFINITY;
#pragma unroll
    for (int i = 0; i < NX; i++) {
        x[i] = c + (x[i] - lse);
        mn = fminf(mn, (FULL || wave_tok<E>(i, lane) < V) ? x[i] : INFINITY);
    }
    if (m >= V) {  // nothing to cut: every token is a candidate
#pragma unroll
        for (int i = 0; i < NX; i++) {
            const int v = wave_tok<E>(i, lane);
            if (FULL || v < V) dst[v] = pack_candidate(x[i], flat0 + (uint32_t)v);
        }
        return;
    }
    // 1. histogram of the scores over equal-width bins of [lo, hi]; the bin index is monotone in the score
    const float lo = -wave_max(-mn), hi = c + (mx - lse);
    const float inv_w = (hi > lo) ? ((float)WROW_BINS - 0.01f) / (hi - lo) : 0.0f;
    const float k0 = -lo * inv_w;
#pragma unroll
    for (int i = 0; i < 4; i++) ((int4 *)hist)[i * 64 + lane] = make_int4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < NX; i++) {
        const uint32_t bi = min((uint32_t)__builtin_fmaf(x[i], inv_w, k0), (uint32_t)(WROW_BINS - 1));  // negative and NaN convert to 0
        if (FULL || wave_tok<E>(i, lane) < V) atomicAdd(&hist[bi], 1);
    }
    // 2. lane l owns bins 1023-16l .. 1008-16l; inclusive scan from the top bin down finds the bin T of the m-th best score
    int h[16];
    {
        const int4 *hp = (const int4 *)(hist + WROW_BINS - 16 - 16 * lane);
#pragma unroll
        for (int i = 0; i < 4; i++) { const int4 t = hp[i]; h[4 * i] = t.x; h[4 * i + 1] = t.y; h[4 * i + 2] = t.z; h[4 * i + 3] = t.w; }
    }
    int mine = 0;
#pragma unroll
    for (int i = 0; i < 16; i++) mine += h[i];
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(incl, o, 64); if (lane >= o) incl += t; }
    int above = incl - mine, selT = 0, selK = 0, selC = 0;
    const bool owner = above < m && incl >= m;
    if (owner) {
#pragma unroll
        for (int i = 15; i >= 0; i--) {  // h[15] is this lane's top bin
            if (selC == 0 && above + h[i] >= m) { selT = WROW_BINS - 16 - 16 * lane + i; selK = m - above; selC = h[i]; }
            if (selC == 0) above += h[i];
        }
    }
    const int src_lane = __ffsll((long long)__ballot(owner)) - 1;
    const int T = __shfl(selT, src_lane, 64), krem = __shfl(selK, src_lane, 64), cntT = __shfl(selC, src_lane, 64);
    if (cntT > WROW_LIST) {  // crowded threshold bin (e.g. all logits equal): exact radix selection
        float sc[NX];  // a copy, so that only this branch keeps the scores in addressable memory
#pragma unroll
        for (int i = 0; i < NX; i++) sc[i] = x[i];
        select_row_radix_wave<VEC, E>(sc, V, m, flat0, stage);
    } else {
        // 3. bins above T go straight to the staged output, bin T to the list (over the dead histogram) for exact ranking
        const int n_gt = m - krem;
        int base_gt = 0, base_eq = 0;
        // The bins are recomputed, not kept: opaque copies of the two constants stop the compiler from holding
        // all NX bin indices of the histogram pass in registers until here.
        float inv_w2 = inv_w, k02 = k0;
        asm volatile("" : "+v"(inv_w2), "+v"(k02));
#pragma unroll
        for (int i = 0; i < NX; i++) {
            const int bi = (int)min((uint32_t)__builtin_fmaf(x[i], inv_w2, k02), (uint32_t)(WROW_BINS - 1));
            const bool ok = FULL || wave_tok<E>(i, lane) < V;
            const bool gt = ok && bi > T, eq = ok && bi == T;
            const unsigned long long mg = __ballot(gt), me = __ballot(eq);
            const unsigned long long st = ((unsigned long long)__float_as_uint(x[i] + 0.0f) << 32) | (nflat - (uint32_t)((i / E) * 64 * E + (i % E)));
            if (gt) stage[base_gt + __builtin_amdgcn_mbcnt_hi((uint32_t)(mg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mg, 0))] = st;
            base_gt += __popcll(mg);
            if (me != 0) {
                if (eq) list[base_eq + __builtin_amdgcn_mbcnt_hi((uint32_t)(me >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)me, 0))] = st;
                base_eq += __popcll(me);
            }
        }
        // rank every listed candidate among the cntT listed ones; the krem best go out
        for (int i = lane; i < cntT; i += 64) {
            const unsigned long long st = list[i], key = staged_to_key(st);
            int rank = 0;
            for (int q = 0; q < cntT; q++) rank += staged_to_key(list[q]) > key ? 1 : 0;
            if (rank < krem) stage[n_gt + rank] = st;
        }
    }
    for (int i = lane; i < m; i += 64) dst[i] = staged_to_key(stage[i]);
}

// One row of logits, already in registers (x[i]: token wave_tok<E>(i, lane); padding -inf), through the cut.  Returns when the
// row's candidates are written.
template <int VEC, bool FULL, int E>
__device__ __forceinline__ void select_one_row_wave(float (&x)[VEC * 4], int64_t vrow, int64_t row, const float *__restrict__ cum, int n, int V,
                                                    int m, unsigned long long *__restrict__ cand, const unsigned long long *__restrict__ bound,
                                                    int *__restrict__ req_count, unsigned long long *list, int lane, int64_t dst_at) {
    constexpr int NX = VEC * 4;
    unsigned long long *stage = list + 512;
    const float c = cum ? cum[row] : 0.0f;
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NX; i++) mx = fmaxf(mx, x[i]);
    mx = wave_max_dpp(mx);
    const float mxl = mx * 1.4426950408889634f;
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < NX; i++) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], 1.4426950408889634f, -mxl));  // padding gives 0
    const float lse = mx + __logf(wave_sum_dpp(sum));

    unsigned long long *dst = cand + (dst_at >= 0 ? dst_at : vrow * (int64_t)m);  // dst_at: where a listed row reserved its m slots
    const uint32_t flat0 = (uint32_t)((row % n) * (int64_t)V);
    // low word of a staged candidate: 0xFFFFFFFF - (flat0 + token)
    const uint32_t nflat = 0xFFFFFFFFu - flat0 - (uint32_t)lane * (uint32_t)E;
    if (bound) {
        // Request-level bound: the request's first row alone has m candidates at or above `bound`, so nothing below it can
        // survive the request's selection.  Rows that have at most m candidates there write exactly those - usually far
        // fewer than m - and skip the histogram; the others fall through to the row's own top-m cut.
        const int64_t req = row / n;
        const float sstar = key_score((uint32_t)(bound[req] >> 32));
        // score(x) = c + (x - lse) >= sstar is tested exactly, but only on the logits that pass a threshold in the logit domain
        // placed a few roundings below the exact one (every candidate at or above the bound passes it)
        const float t0 = (sstar - c) + lse;
        const float thr = t0 - 1e-6f * (fabsf(sstar) + fabsf(c) + fabsf(lse) + fabsf(t0));
        int cnt = 0;
        constexpr int CH = 16;  // logits per test: one wave-uniform branch per CH elements, taken for the few chunks that hold a candidate
#pragma unroll
        for (int i0 = 0; i0 < NX; i0 += CH) {
            unsigned long long any = 0;
#pragma unroll
            for (int u = 0; u < CH; u++) any |= __ballot(x[i0 + u] >= thr);  // padding is -inf
            if (any != 0) {
#pragma unroll
                for (int u = 0; u < CH; u++) {
                    const int i = i0 + u;
                    const float sc = c + (x[i] - lse);
                    const bool hit = sc >= sstar;
                    const unsigned long long mk = __ballot(hit);
                    const unsigned long long st = ((unsigned long long)__float_as_uint(sc + 0.0f) << 32) | (nflat - (uint32_t)((i / E) * 64 * E + (i % E)));
                    const int at = cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(mk >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mk, 0));
                    if (hit && at < m) stage[at] = st;
                    cnt += __popcll(mk);
                }
            }
        }
        const int take = cnt <= m ? cnt : m;
        int base = 0;
        if (lane == 0) base = atomicAdd(&req_count[req], take);
        base = __shfl(base, 0, 64);
        dst = cand + req * ((int64_t)n * m) + base;
        if (cnt <= m) {
            for (int i = lane; i < cnt; i += 64) dst[i] = staged_to_key(stage[i]);
            return;
        }
    }
    select_row_own_cut<VEC, FULL, E>(x, c, mx, lse, dst, flat0, nflat, V, m, list, lane);
}

// FULL: V == VEC*256, every register holds a token (the validity tests fold away).
// row_step: the launch visits rows 0, row_step, 2 row_step, ... of the logits (row_step = n: the first beam of every request).
// bound / req_count (both or neither): per request, a key no survivor can lie below; the launch then writes only
// the candidates that reach it (at most the row's m best), compacted per request behind a running count.
// todo / todo_count (both or neither; then without bound): the launch visits only the listed rows {row, slot}; each gets its
// own cut, written at slot `slot` of its request's segment.  Wavefronts walk their rows with the launch's stride.
template <int VEC, bool FULL, typename LT>
__global__ __launch_bounds__(256, 3) void select_rows_wave(const LT *__restrict__ logits, const float *__restrict__ cum, int64_t rows, int n, int V,
                                                          int m, unsigned long long *__restrict__ cand, int64_t row_step,
                                                          const unsigned long long *__restrict__ bound, int *__restrict__ req_count,
                                                          const int2 *__restrict__ todo, const int *__restrict__ todo_count) {
    constexpr int E = LogitPiece<LT>::E, NX = VEC * 4, G = NX / E;
    extern __shared__ unsigned long long wave_lds[];  // per wavefront: 512 slots of histogram / list, then m slots of staged output
    const int lane = threadIdx.x % 64, wv = threadIdx.x / 64;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t count = todo ? (int64_t)*todo_count : rows;
    unsigned long long *list = wave_lds + (size_t)wv * ((512 + m + 1) & ~1);  // even number of 8-byte slots: 16-byte accesses stay aligned
    // whole wavefronts leave the loop; nothing below synchronises across wavefronts
    for (int64_t at = (int64_t)blockIdx.x * 4 + wv; at < count; at += nwaves) {
        int64_t vrow = at, dst_at = -1;
        if (todo) {
            const int2 t = todo[at];
            vrow = t.x;
            dst_at = (vrow / n) * ((int64_t)n * m) + t.y;
        }
        const uint4 *z = (const uint4 *)(logits + vrow * row_step * (int64_t)V);
        float x[NX];
#pragma unroll
        for (int g = 0; g < G; g++) {
            if (FULL || (g * 64 + lane) * E < V) {
                LogitPiece<LT>::unpack(z[g * 64 + lane], &x[g * E]);
            } else {
#pragma unroll
                for (int e = 0; e < E; e++) x[g * E + e] = -INFINITY;
            }
        }
        select_one_row_wave<VEC, FULL, E>(x, vrow, vrow * row_step, cum, n, V, m, cand, bound, req_count, list, lane, dst_at);
    }
}

// The bounded pass over half-precision logits.  A row stays packed (raw[g]: tokens (g*64 + lane)*8 .. +7; pieces past V
// hold -inf): maximum, log-sum-exp and the sweep for candidates at or above the request's bound read the halves in
// place, and each wavefront asks for its next row before it works on the current one, so the memory latency hides behind the
// arithmetic.  A row with more than m candidates at the bound reserves m slots and is put on the list for
// select_rows_wave, which gives it its own cut; this kernel carries none of that code or its registers.
template <int VEC, bool FULL>
__global__ __launch_bounds__(256, VEC >= 32 ? 2 : (VEC >= 16 ? 3 : 4)) void select_rows_sweep_f16(
    const _Float16 *__restrict__ logits, const float *__restrict__ cum, int64_t rows, int n, int V, int m, unsigned long long *__restrict__ cand,
    const unsigned long long *__restrict__ bound, int *__restrict__ req_count, int2 *__restrict__ todo, int *__restrict__ todo_count) {
    constexpr int NX = VEC * 4, E = 8, G = NX / E;
    extern __shared__ unsigned long long wave_lds[];  // per wavefront: m slots of staged output
    // The row index is made a scalar of the wavefront (rows < 2^31, checked by the host): its cumulative score and bound then
    // come through scalar loads, which do not queue behind the vector loads of the next row.
    const int lane = threadIdx.x % 64, wv = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const uint32_t nwaves = gridDim.x * 4u;
    uint32_t row = blockIdx.x * 4u + (uint32_t)wv;
    if (row >= (uint64_t)rows) return;  // whole wavefronts leave; nothing below synchronises across wavefronts
    unsigned long long *stage = wave_lds + (size_t)wv * m;
    auto request_row = [&](uint32_t r, uint4 (&raw)[G]) {
        const uint4 *z = (const uint4 *)(logits + (int64_t)r * V);
#pragma unroll
        for (int g = 0; g < G; g++) {
            if (FULL || (g * 64 + lane) * E < V) raw[g] = z[g * 64 + lane];
            else raw[g] = make_uint4(0xFC00FC00u, 0xFC00FC00u, 0xFC00FC00u, 0xFC00FC00u);  // halves of -inf
        }
    };
    // per row: request, beam, cumulative score and the bound's score, fetched one row ahead like the logits
    auto row_scalars = [&](uint32_t r, uint32_t &req, uint32_t &beam, float &c, float &sstar) {
        req = r / (uint32_t)n;
        beam = r % (uint32_t)n;
        c = cum ? cum[r] : 0.0f;
        sstar = key_score((uint32_t)(bound[req] >> 32));
    };
    auto pk_max = [](halfx2 a, halfx2 b) {  // (the plain instruction: the generic maximum first quiets both operands)
        halfx2 r;
        asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
        return r;
    };
    uint4 raw[G];
    request_row(row, raw);
    uint32_t req, beam;
    float c, sstar;
    row_scalars(row, req, beam, c, sstar);
    for (;;) {
        const uint64_t next = (uint64_t)row + nwaves;
        const bool more = next < (uint64_t)rows;
        const uint32_t ahead = more ? (uint32_t)next : row;
        uint4 nxt[G];
        // (unconditional - the last row is asked for twice: a branch here would make the compiler wait for these loads at the
        // first use of the current row, as if they had been skipped)
        request_row(ahead, nxt);
        uint32_t req_n, beam_n;
        float c_n, sstar_n;
        row_scalars(ahead, req_n, beam_n, c_n, sstar_n);
        __builtin_amdgcn_sched_barrier(0);  // the loads go out here, not where the instruction scheduler finds the registers cheapest

        halfx2 pmax[G];  // per piece: the maximum of its even and of its odd tokens
#pragma unroll
        for (int g = 0; g < G; g++) {
            const halfx8 v = __builtin_bit_cast(halfx8, raw[g]);
            const halfx2 p0 = {v[0], v[1]}, p1 = {v[2], v[3]}, p2 = {v[4], v[5]}, p3 = {v[6], v[7]};
            pmax[g] = pk_max(pk_max(p0, p1), pk_max(p2, p3));
        }
        halfx2 rm = pmax[0];
#pragma unroll
        for (int g = 1; g < G; g++) rm = pk_max(rm, pmax[g]);
        const float lane_mx = fmaxf((float)rm[0], (float)rm[1]);
        const float mx = wave_max_dpp(lane_mx);
        const float mxl = mx * 1.4426950408889634f;
        float sum = 0.0f;
#pragma unroll
        for (int g = 0; g < G; g++) {
            const halfx8 v = __builtin_bit_cast(halfx8, raw[g]);
#pragma unroll
            for (int e = 0; e < E; e++) sum += __builtin_amdgcn_exp2f(__builtin_fmaf((float)v[e], 1.4426950408889634f, -mxl));  // padding gives 0
        }
        const float lse = mx + __logf(wave_sum_dpp(sum));
        // (opaque to the compiler: otherwise it keeps the NX widened logits of the sum above in registers for the sweep below)
#pragma unroll
        for (int g = 0; g < G; g++) asm volatile("" : "+v"(raw[g].x), "+v"(raw[g].y), "+v"(raw[g].z), "+v"(raw[g].w));

        // score(x) = c + (x - lse) >= sstar is tested exactly, but only inside the pieces whose maximum passes a threshold in the
        // logit domain placed a few roundings below the exact one (every candidate at or above the bound passes it); most
        // rows of a request's weaker beams have no such piece at all
        uint32_t nflat = 0xFFFFFFFFu - beam * (uint32_t)V - (uint32_t)lane * (uint32_t)E;
        asm volatile("" : "+v"(nflat));  // (opaque: keeps the compiler from carrying NX row-independent parts of the token words across rows)
        const float t0 = (sstar - c) + lse;
        const float thr = t0 - 1e-6f * (fabsf(sstar) + fabsf(c) + fabsf(lse) + fabsf(t0));
        int cnt = 0;
        if (__ballot(lane_mx >= thr) != 0) {
#pragma unroll
            for (int g = 0; g < G; g++) {
                const unsigned long long any = __ballot(fmaxf((float)pmax[g][0], (float)pmax[g][1]) >= thr);
                if (any != 0) {
                    const halfx8 v = __builtin_bit_cast(halfx8, raw[g]);
#pragma unroll
                    for (int e = 0; e < E; e++) {
                        const float sc = c + ((float)v[e] - lse);
                        const bool hit = sc >= sstar;
                        const unsigned long long mk = __ballot(hit);
                        const unsigned long long st = ((unsigned long long)__float_as_uint(sc + 0.0f) << 32) | (nflat - (uint32_t)(g * 64 * E + e));
                        const int at = cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(mk >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mk, 0));
                        if (hit && at < m) stage[at] = st;
                        cnt += __popcll(mk);
                    }
                }
            }
        }
        if (cnt > 0) {  // (wavefront-uniform)
            const int take = cnt <= m ? cnt : m;
            int base = 0;
            if (lane == 0) {
                base = atomicAdd(&req_count[req], take);
                if (cnt > m) todo[atomicAdd(todo_count, 1)] = make_int2((int)row, base);  // its m slots are filled by the listed pass
            }
            base = __shfl(base, 0, 64);
            if (cnt <= m) {
                unsigned long long *dst = cand + (int64_t)req * ((int64_t)n * m) + base;
                for (int i = lane; i < cnt; i += 64) dst[i] = staged_to_key(stage[i]);
            }
        }
        if (!more) break;
#pragma unroll
        for (int g = 0; g < G; g++) raw[g] = nxt[g];
        row = (uint32_t)next;
        req = req_n; beam = beam_n; c = c_n; sstar = sstar_n;
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

// every key of a request's candidate list, 16 bytes per lane and four loads in flight (the list is streamed several times)
template <typename F>
__device__ __forceinline__ void for_each_key(const unsigned long long *__restrict__ src, int64_t ncand, F f) {
    const int tid = threadIdx.x;
    if ((((uintptr_t)src) & 15) == 0) {
        const ulonglong2 *src2 = (const ulonglong2 *)src;
        const int64_t pairs = ncand / 2;
        int64_t i = tid;
        for (; i + 3 * SELB_THREADS < pairs; i += 4 * SELB_THREADS) {
            const ulonglong2 a = src2[i], b = src2[i + SELB_THREADS], c = src2[i + 2 * SELB_THREADS], d = src2[i + 3 * SELB_THREADS];
            f(a.x); f(a.y); f(b.x); f(b.y); f(c.x); f(c.y); f(d.x); f(d.y);
        }
        for (; i < pairs; i += SELB_THREADS) { const ulonglong2 a = src2[i]; f(a.x); f(a.y); }
        if ((ncand & 1) && tid == 0) f(src[ncand - 1]);
    } else {
        for (int64_t i = tid; i < ncand; i += SELB_THREADS) f(src[i]);
    }
}

// Usual path of stage B: two sweeps over the candidates.  A sample of one key per thread gives the span of the score bits;
// the first sweep counts the keys in 2048 equal bins of that span (keys outside it fall into the end bins; the bin index is
// monotone in the key, and the counts spread over the bins, unlike the leading radix digit, which most keys of a request
// share), the second collects every key from the threshold bin up into LDS, where a sort finishes the job.  Returns false,
// having selected nothing, when more than SELB_SORT_MAX keys lie from the threshold bin up (the exact radix selection then runs).
__device__ __forceinline__ bool select_request_binned(const unsigned long long *__restrict__ src, int64_t ncand, int k,
                                                      unsigned long long *skeys, int *hist, int *wave_tot, int *sel_digit, int *sel_krem,
                                                      int *sel_cnt, int *out_cnt) {
    const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
    const uint32_t smp = (uint32_t)(src[(int64_t)tid * ncand / SELB_THREADS] >> 32);
    uint32_t smax = smp, smin = smp;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { smax = max(smax, (uint32_t)__shfl_xor((int)smax, o, 64)); smin = min(smin, (uint32_t)__shfl_xor((int)smin, o, 64)); }
    if (lane == 0) { wave_tot[wv] = (int)smax; hist[wv] = (int)smin; }
    __syncthreads();
    for (int q = 0; q < SELB_THREADS / 64; q++) { smax = max(smax, (uint32_t)wave_tot[q]); smin = min(smin, (uint32_t)hist[q]); }
    __syncthreads();
    int nsh = 0;
    while (((smax - smin) >> nsh) >= 2040u) nsh++;
    const long long base = (long long)smin;
    auto digit = [&](unsigned long long key) {
        const long long d = ((((long long)(key >> 32)) - base) >> nsh) + 4;  // floor, also below the sampled minimum
        return (int)(d < 0 ? 0 : (d > 2047 ? 2047 : d));
    };
    for (int i = tid; i < 2048; i += SELB_THREADS) hist[i] = 0;
    if (tid == 0) *out_cnt = 0;
    __syncthreads();
    for_each_key(src, ncand, [&](unsigned long long key) { atomicAdd(&hist[digit(key)], 1); });
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
    if (excl < k && incl >= k) {
        if (excl + hi >= k) { *sel_digit = 2047 - 2 * tid; *sel_krem = k - excl; *sel_cnt = hi; }
        else { *sel_digit = 2046 - 2 * tid; *sel_krem = k - excl - hi; *sel_cnt = lo; }
    }
    __syncthreads();
    const int T = *sel_digit, total_ge = (k - *sel_krem) + *sel_cnt;
    __syncthreads();
    if (total_ge > SELB_SORT_MAX) return false;  // uniform: every thread read the same shared values
    int np = 1;
    while (np < total_ge) np <<= 1;
    for (int i = tid; i < np; i += SELB_THREADS) skeys[i] = 0ull;
    __syncthreads();
    for_each_key(src, ncand, [&](unsigned long long key) {
        if (digit(key) >= T) skeys[atomicAdd(out_cnt, 1)] = key;  // exactly total_ge keys qualify
    });
    __syncthreads();
    bitonic_sort_desc(skeys, np);
    return true;
}

__global__ __launch_bounds__(SELB_THREADS) void select_request(const unsigned long long *__restrict__ cand, int64_t req_stride,
                                                               const int *__restrict__ req_count, int V, int k,
                                                               int32_t *__restrict__ parent, int32_t *__restrict__ tok,
                                                               float *__restrict__ score, const int32_t *__restrict__ sid_old,
                                                               int32_t *__restrict__ sid_new, const int32_t *__restrict__ anc_old,
                                                               int32_t *__restrict__ anc_new, int n, int T, int level) {
    __shared__ unsigned long long skeys[SELB_SORT_MAX];
    __shared__ int hist[2048];
    __shared__ int wave_tot[16];
    __shared__ int sel_digit, sel_krem, sel_cnt, out_cnt;
    const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
    const int64_t b = blockIdx.x;
    const unsigned long long *src = cand + b * req_stride;  // the request's candidates: the first req_count[b] keys of its segment
    const int64_t ncand = req_count[b];
    int kp = 1;
    while (kp < k) kp <<= 1;

    if (ncand <= SELB_SORT_MAX) {
        int np = 1;
        while (np < ncand) np <<= 1;
        for (int i = tid; i < np; i += SELB_THREADS) skeys[i] = i < ncand ? src[i] : 0ull;
        __syncthreads();
        bitonic_sort_desc(skeys, np);
    } else if (select_request_binned(src, ncand, k, skeys, hist, wave_tot, &sel_digit, &sel_krem, &sel_cnt, &out_cnt)) {
        // done: skeys holds the k best in order
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
            for_each_key(src, ncand, [&](unsigned long long key) {
                if (pass == 0 || (key >> shift) == prefix) atomicAdd(&hist[(int)((key >> nshift) & ((1u << w) - 1))], 1);
            });
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
        for_each_key(src, ncand, [&](unsigned long long key) {
            if ((key >> shift) >= prefix) {
                int p = atomicAdd(&out_cnt, 1);
                if (p < kp) skeys[p] = key;
            }
        });
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
        if (anc_new) {  // row (over the whole batch) of the survivor's ancestor at every level so far: the reorder is this index table
            for (int t = 0; t < level; t++) anc_new[(b * k + j) * T + t] = anc_old[(b * n + par) * T + t];
            anc_new[(b * k + j) * T + level] = (int32_t)(b * n + par);
        }
    }
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// what the row kernels of one selection share
struct RowsLaunch {
    hipStream_t st;
    const void *logits;
    int logits_f16;
    const float *cum;
    int n, V, m;
    unsigned long long *cand;
    const unsigned long long *bound;
    int *req_count;
    int2 *todo;
    int *todo_count;
};
static int compute_units() {
    static int n_cu = 0;
    if (!n_cu) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        n_cu = prop.multiProcessorCount;
    }
    return n_cu;
}
// mode 0: every row (stride row_step) its own cut or, with a bound, the bounded cut; mode 1: the listed rows' own cuts
template <int VEC, bool FULL, typename LT>
static int launch_rows_wave_kind(const RowsLaunch &a, int64_t rows, int64_t row_step, int mode) {
    auto kern = select_rows_wave<VEC, FULL, LT>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * (512 + GR4AD_MAX_BEAM + 2) * 8) != hipSuccess) return GR4AD_EHIP;
        attr_done = true;
    }
    const size_t lds = 4 * (size_t)((512 + a.m + 1) & ~1) * sizeof(unsigned long long);  // <= 4 * (4 KB + 32 KB)
    int64_t grid = ceil_div64(rows, 4);  // one wavefront per row, four rows per workgroup
    if (mode == 1) {  // the list is short as a rule: a few workgroups per compute unit walk it
        const int n_cu = compute_units();
        if (!n_cu) return GR4AD_EHIP;
        if (grid > (int64_t)n_cu * 4) grid = (int64_t)n_cu * 4;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, a.st, (const LT *)a.logits, a.cum, rows, a.n, a.V, a.m, a.cand, row_step,
                       mode == 1 ? nullptr : a.bound, mode == 1 ? nullptr : a.req_count, mode == 1 ? (const int2 *)a.todo : nullptr,
                       mode == 1 ? (const int *)a.todo_count : nullptr);
    return GR4AD_OK;
}
// mode 2: the bounded pass over packed half-precision logits, which lists the rows that need their own cut
template <int VEC, bool FULL>
static int launch_rows_sweep_kind(const RowsLaunch &a, int64_t rows) {
    auto kern = select_rows_sweep_f16<VEC, FULL>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * GR4AD_MAX_BEAM * 8) != hipSuccess) return GR4AD_EHIP;
        attr_done = true;
    }
    const int n_cu = compute_units();
    if (!n_cu) return GR4AD_EHIP;
    // wavefronts walk the rows with the launch's stride
    const size_t lds = 4 * (size_t)a.m * sizeof(unsigned long long);
    // About 8 rows per wavefront: measured at a million rows of 8192 logits, 3.6 ms against 4.3 ms with 128 rows per wavefront
    // (as many workgroups as fit the chip at once) and 3.8 ms with one row per wavefront (no next-row prefetch at all).
    int64_t grid = ceil_div64(rows, 32);
    if (grid < (int64_t)n_cu * 16) grid = std::min<int64_t>(ceil_div64(rows, 4), (int64_t)n_cu * 16);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, a.st, (const _Float16 *)a.logits, a.cum, rows,
                       a.n, a.V, a.m, a.cand, a.bound, a.req_count, a.todo, a.todo_count);
    return GR4AD_OK;
}
template <int VEC>
static int launch_rows_vec(const RowsLaunch &a, int64_t rows, int64_t row_step, int mode) {
    const bool full = a.V == VEC * 256;
    if (mode == 2) return full ? launch_rows_sweep_kind<VEC, true>(a, rows) : launch_rows_sweep_kind<VEC, false>(a, rows);
    if (a.logits_f16)
        return full ? launch_rows_wave_kind<VEC, true, _Float16>(a, rows, row_step, mode) : launch_rows_wave_kind<VEC, false, _Float16>(a, rows, row_step, mode);
    return full ? launch_rows_wave_kind<VEC, true, float>(a, rows, row_step, mode) : launch_rows_wave_kind<VEC, false, float>(a, rows, row_step, mode);
}
static int launch_rows(const RowsLaunch &a, int64_t rows, int64_t row_step, int mode) {
    if (a.V <= 1024) return launch_rows_vec<4>(a, rows, row_step, mode);
    if (a.V <= 2048) return launch_rows_vec<8>(a, rows, row_step, mode);
    if (a.V <= 4096) return launch_rows_vec<16>(a, rows, row_step, mode);
    return launch_rows_vec<32>(a, rows, row_step, mode);
}

// Half-precision logits are taken by the wavefront kernel only: 16-byte pieces of 8 values.
bool select_takes_f16(int V) { return V >= 8 && V <= 8192 && V % 8 == 0; }

// bound[b] = smallest of the m keys the first row of request b kept (wavefront per request); count[b] = 0; list count = 0
__global__ __launch_bounds__(256) void request_bound_kernel(const unsigned long long *__restrict__ cand0, int m, int B,
                                                            unsigned long long *__restrict__ bound, int *__restrict__ req_count,
                                                            int *__restrict__ todo_count) {
    const int lane = threadIdx.x % 64;
    const int b = blockIdx.x * 4 + threadIdx.x / 64;
    if (blockIdx.x == 0 && threadIdx.x == 0) *todo_count = 0;  // the list of rows that need their own cut starts empty
    if (b >= B) return;
    unsigned long long mn = ~0ull;
    for (int i = lane; i < m; i += 64) { const unsigned long long k = cand0[(int64_t)b * m + i]; mn = k < mn ? k : mn; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { const unsigned long long t = __shfl_xor(mn, o, 64); mn = t < mn ? t : mn; }
    if (lane == 0) { bound[b] = mn; req_count[b] = 0; }
}
__global__ __launch_bounds__(256) void fill_count_kernel(int *__restrict__ req_count, int B, int v) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b < B) req_count[b] = v;
}

// workspace: candidates [B][n*m] keys, then the first rows' cuts [B][m], the request bounds [B], the request counts [B], the
// count of listed rows (one int in 256 bytes) and the list {row, slot} [B*n]
static inline size_t sel_ws_cand(int B, int n, int m) { return align256((size_t)B * n * m * sizeof(unsigned long long)); }
static inline size_t sel_ws_cand0(int B, int m) { return align256((size_t)B * m * sizeof(unsigned long long)); }
size_t select_workspace_bytes(int B, int n, int V, int k) {
    int m = k < V ? k : V;
    return sel_ws_cand(B, n, m) + sel_ws_cand0(B, m) + align256((size_t)B * sizeof(unsigned long long)) + align256((size_t)B * sizeof(int)) + 256 +
           align256((size_t)B * n * sizeof(int2));
}

int launch_select(const void *logits_any, int logits_f16, const float *cum, int B, int n, int V, int k, void *ws, size_t ws_bytes, int32_t *parent,
                  int32_t *tok, float *score, const int32_t *sid_old, int32_t *sid_new, const int32_t *anc_old, int32_t *anc_new, int T, int level,
                  hipStream_t st) {
    if (B <= 0 || n <= 0 || V <= 0 || k <= 0 || (int64_t)k > (int64_t)n * V) return GR4AD_EINVAL;
    if (logits_f16 && (!select_takes_f16(V) || ((uintptr_t)logits_any % 16))) return GR4AD_EUNSUPPORTED;
    const float *logits = (const float *)logits_any;  // (float32 unless logits_f16: only the wavefront kernel then reads them)
    if (k > GR4AD_MAX_BEAM || V > GR4AD_MAX_CODEBOOK || (int64_t)n * V >= 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    if (ws_bytes < select_workspace_bytes(B, n, V, k) || ((uintptr_t)ws % 8)) return GR4AD_EWORKSPACE;
    const int m = k < V ? k : V;
    const int64_t rows = (int64_t)B * n;
    if (rows > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    unsigned long long *cand = (unsigned long long *)ws;
    unsigned long long *cand0 = (unsigned long long *)((char *)ws + sel_ws_cand(B, n, m));
    unsigned long long *bound = (unsigned long long *)((char *)cand0 + sel_ws_cand0(B, m));
    int *req_count = (int *)((char *)bound + align256((size_t)B * sizeof(unsigned long long)));
    int *todo_count = (int *)((char *)req_count + align256((size_t)B * sizeof(int)));
    int2 *todo = (int2 *)((char *)todo_count + 256);
    const bool wave_path = V <= 8192 && V % 4 == 0 && ((uintptr_t)logits % 16) == 0;
    // Request-level bound (several rows per request, cut smaller than the row): the first row of a request holds its best
    // beam; the m-th best candidate of that row is a score no survivor of the request can lie below.
    const bool bounded = wave_path && n > 1 && k <= V;
    {
        // algorithmic bytes: every logit once; the candidates written depend on the data (between k per request and m per row):
        // the lower bound is counted when the request-level bound is in use
        ProfScope ps(KC_SELECT_ROWS, st, 0.0, (double)rows * V * (logits_f16 ? 2 : 4) + (bounded ? (double)B * k : (double)rows * m) * 8);
        if (wave_path) {
            const RowsLaunch a = {st, logits_any, logits_f16, cum, n, V, m, nullptr, bound, req_count, todo, todo_count};
            RowsLaunch first = a, all = a;
            first.cand = cand0;
            first.bound = nullptr;
            first.req_count = nullptr;
            all.cand = cand;
            int s;
            if (bounded) {
                if ((s = launch_rows(first, B, n, 0))) return s;  // the first row of every request, cut on its own
                GR4AD_LAUNCH_CHECK();
                hipLaunchKernelGGL(request_bound_kernel, dim3((unsigned)((B + 3) / 4)), dim3(256), 0, st, cand0, m, B, bound, req_count, todo_count);
                GR4AD_LAUNCH_CHECK();
                if (logits_f16) {
                    if ((s = launch_rows(all, rows, 1, 2))) return s;
                    GR4AD_LAUNCH_CHECK();
                    if ((s = launch_rows(all, rows, 1, 1))) return s;
                } else {
                    if ((s = launch_rows(all, rows, 1, 0))) return s;
                }
            } else {
                all.bound = nullptr;
                all.req_count = nullptr;
                if ((s = launch_rows(all, rows, 1, 0))) return s;
            }
        } else {
            const size_t stage_bytes = (size_t)m * sizeof(unsigned long long);  // <= 32 KB (GR4AD_MAX_BEAM)
            if (V <= 1024)
                hipLaunchKernelGGL(select_rows<4>, dim3((unsigned)rows), dim3(256), stage_bytes, st, logits, cum, n, V, m, cand);
            else if (V <= 4096)
                hipLaunchKernelGGL(select_rows<16>, dim3((unsigned)rows), dim3(256), stage_bytes, st, logits, cum, n, V, m, cand);
            else if (V <= 8192)
                hipLaunchKernelGGL(select_rows<32>, dim3((unsigned)rows), dim3(256), stage_bytes, st, logits, cum, n, V, m, cand);
            else
                hipLaunchKernelGGL(select_rows<64>, dim3((unsigned)rows), dim3(256), stage_bytes, st, logits, cum, n, V, m, cand);
        }
        GR4AD_LAUNCH_CHECK();
        if (!bounded) {  // every row wrote its m: the request's candidates are the n*m keys of its rows
            hipLaunchKernelGGL(fill_count_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, st, req_count, B, n * m);
            GR4AD_LAUNCH_CHECK();
        }
    }
    ProfScope ps(KC_SELECT_REQUEST, st, 0.0, (bounded ? (double)B * k : (double)rows * m) * 8 + (double)B * k * 12);  // (same convention)
    hipLaunchKernelGGL(select_request, dim3((unsigned)B), dim3(SELB_THREADS), 0, st, (const unsigned long long *)ws, (int64_t)n * m, req_count, V, k,
                       parent, tok, score, sid_old, sid_new, anc_old, anc_new, n, T, level);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// The same selection for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc): the candidate lists, first-row cuts, request bounds and counts live in a fixed device
// array of this library instead of a caller workspace.  Host code never uses the array's name as an address: the device
// address is looked up once per device and kept.  Every call on a GPU shares that GPU's array (overlapping calls race);
// nothing in it has to start at zero - the counts are written by a kernel of every call before they are read.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[GR4AD_SELECT_STATIC_BYTES];

namespace {
const int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device (NULL: not looked up yet)
}  // namespace

extern "C" int gr4ad_op_select_static(const float *logits, const float *cum, int32_t B, int32_t n, int32_t V, int32_t k, int32_t *parent,
                                      int32_t *tok, float *score, void *hip_stream) {
    if (!logits || !parent || !tok || !score) return gr4ad_set_thread_error(GR4AD_EINVAL, "gr4ad_op_select_static: a required pointer is NULL");
    if (B < 1 || n < 1 || V < 1 || k < 1 || (int64_t)k > (int64_t)n * V)
        return gr4ad_set_thread_error(GR4AD_EINVAL, "gr4ad_op_select_static: need B, n, V >= 1 and 1 <= k <= n*V");
    if (k > GR4AD_MAX_BEAM || V > GR4AD_MAX_CODEBOOK)
        return gr4ad_set_thread_error(GR4AD_EUNSUPPORTED, "gr4ad_op_select_static: k > %d or V > %d", GR4AD_MAX_BEAM, GR4AD_MAX_CODEBOOK);
    const int m = k < V ? k : V;
    // (computed in 64 bits before select_workspace_bytes multiplies the sizes)
    if ((double)B * n * m * 8.0 > (double)GR4AD_SELECT_STATIC_BYTES || select_workspace_bytes(B, n, V, k) > (size_t)GR4AD_SELECT_STATIC_BYTES)
        return gr4ad_set_thread_error(GR4AD_EWORKSPACE, "gr4ad_op_select_static: B=%d n=%d V=%d k=%d needs more than the %u bytes of static scratch", B, n,
                                      V, k, (unsigned)GR4AD_SELECT_STATIC_BYTES);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return gr4ad_set_thread_error(GR4AD_EHIP, "gr4ad_op_select_static: hipGetDevice failed");
    if (dev < 0 || dev >= kMaxDevices) return gr4ad_set_thread_error(GR4AD_EUNSUPPORTED, "gr4ad_op_select_static: device index %d", dev);
    if (!g_scratch_ptr[dev]) {  // once per device, with that device current: each GPU holds its own copy of the array
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return gr4ad_set_thread_error(GR4AD_EHIP, "gr4ad_op_select_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    const int s = launch_select(logits, 0, cum, B, n, V, k, g_scratch_ptr[dev], (size_t)GR4AD_SELECT_STATIC_BYTES, parent, tok, score, nullptr, nullptr,
                                nullptr, nullptr, 0, 0, (hipStream_t)hip_stream);
    return s == GR4AD_OK ? s : gr4ad_set_thread_error(s, "gr4ad_op_select_static: selection failed: %s", gr4ad_strerror(s));
}
