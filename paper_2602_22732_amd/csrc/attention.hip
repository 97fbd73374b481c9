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
//  * context_attn_flash_bf16  the lazy layers' cross-attention in absorbed form
//                           (keys = values = the raw context rows, one query of
//                           width d per (position, head)): one pass over the
//                           context, MFMA, online softmax.
//  * self_attn_step<T>      autoregressive self-attention of the new position over
//                           the beam path's earlier positions (at most T keys), read
//                           in place from the buffers their levels wrote, through
//                           the beams' ancestor table (no reorder copy).
//  * trunk_self_attn<T>     causal self-attention over the T trunk positions.
#include <stdlib.h>

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

// ---------------------------------------------------------------------------
// beam-shared flash cross-attention on the matrix cores (bf16)
// ---------------------------------------------------------------------------
// Values transposed per (request, head): vt[b][h][c][s] = V[b][s][h*dh+c] for s < len_b, 0 beyond
// (s runs to Spad = S rounded up to 64), so a tile of V^T is row-major like a tile of K.
__global__ __launch_bounds__(256) void v_transpose_kernel(const bf16 *__restrict__ kv, const int32_t *__restrict__ ctx_len,
                                                          bf16 *__restrict__ vt, int S, int Spad, int d, int src_pitch, int src_col0) {
    __shared__ bf16 tile[64][66];
    const int b = blockIdx.z, c0 = blockIdx.y * 64, s0 = blockIdx.x * 64;
    int len = ctx_len ? ctx_len[b] : S;
    len = len < 1 ? 1 : (len > S ? S : len);
    const int tid = threadIdx.x;
    for (int i = tid; i < 64 * 8; i += 256) {  // 64 rows (s) x 8 chunks of 8 columns
        const int r = i / 8, ch = i % 8, s = s0 + r;
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (s < len) raw = *(const uint4 *)(kv + ((int64_t)b * S + s) * src_pitch + src_col0 + c0 + ch * 8);
        const bf16 *e = (const bf16 *)&raw;
#pragma unroll
        for (int k = 0; k < 8; k++) tile[r][ch * 8 + k] = e[k];
    }
    __syncthreads();
    for (int i = tid; i < 64 * 8; i += 256) {  // 64 rows (c) x 8 chunks of 8 positions
        const int r = i / 8, ch = i % 8;
        uint4 raw;
        bf16 *e = (bf16 *)&raw;
#pragma unroll
        for (int k = 0; k < 8; k++) e[k] = tile[ch * 8 + k][r];
        *(uint4 *)(vt + ((int64_t)b * d + c0 + r) * Spad + s0 + ch * 8) = raw;
    }
}

// One workgroup: NW wavefronts x QT tiles of 32 beams of one (request, head).  The context streams through LDS
// in macro-tiles of SUBS x 64 keys (K [64 x DH] and V^T [DH x 64] per 64 keys), two macro-tiles double-buffered,
// filled by direct global->LDS loads (no staging registers) one whole macro-tile ahead; every beam of the block
// reuses them.  The workgroup meets at a barrier once per macro-tile only: in between, the two wavefronts that
// share a SIMD drift apart, so one's softmax (vector instructions, the larger part) overlaps the other's MFMAs.
// Both products are computed transposed,
//   S^T = K Q^T  (keys x beams)   and   O^T = V^T P^T  (head dims x beams),
// so that each lane owns one beam: its running max / sum are lane-local, P^T leaves the
// accumulators of the first product already in the operand layout of the second, and the
// only cross-lane step is one exchange between the two half-waves.  Key rows enter the
// first product with index bits 2 and 3 swapped, which makes the 8 keys a lane holds for
// one MFMA k-step consecutive (one 16-byte chunk of a V^T row).
template <int DH, int QT, int NW, int SUBS>
__global__ __launch_bounds__(NW * 64, (QT == 1 && SUBS == 1) ? 16 / NW : 1) void cross_attn_flash_bf16(const bf16 *__restrict__ q, int64_t ldq, const bf16 *__restrict__ kv,
                                                                 const bf16 *__restrict__ vt, const int32_t *__restrict__ ctx_len,
                                                                 bf16 *__restrict__ out, int64_t ldo, int n, int S, int Spad, int d,
                                                                 int H, float scale_log2e, int beam_blocks, int64_t total_blocks) {
    constexpr int KCH = DH / 8;                   // 16-byte chunks per K row
    constexpr int K_CHUNKS = 64 * KCH, V_CHUNKS = DH * 8;
    constexpr int STAGE = K_CHUNKS + V_CHUNKS;    // one 64-key tile
    constexpr int MACRO = SUBS * STAGE;
    constexpr int KSTEPS = DH / 16, MT = DH / 32;
    extern __shared__ bf16x8 smem[];              // 2 * MACRO chunks
    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    // Workgroup ids are dealt to the 8 XCDs in turn, each with an L2 of its own.  The beam blocks of one (request, head) read the
    // same keys and values, so they get consecutive slots of ONE XCD: XCD x owns the contiguous range [x*per, (x+1)*per) of the
    // logical blocks (beam block fastest, then head, then request) and its blocks of one (request, head) start together.
    const int64_t per_xcd = (total_blocks + 7) / 8;
    const int64_t logical = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (logical >= total_blocks) return;
    const int beam_block = (int)(logical % beam_blocks);
    const int h = (int)((logical / beam_blocks) % H);
    const int b = (int)(logical / ((int64_t)beam_blocks * H));
    const int frow = lane % 32, hf = lane / 32;
    int len = ctx_len ? ctx_len[b] : S;
    len = len < 1 ? 1 : (len > S ? S : len);
    const int ntiles = (len + 63) / 64;
    const int nmacro = (ntiles + SUBS - 1) / SUBS;
    const int q0 = (beam_block * NW + wave) * (QT * 32);

    // query fragments stay in registers for the whole kernel
    bf16x8 qf[QT][KSTEPS];
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        int row = q0 + qt * 32 + frow;
        if (row > n - 1) row = n - 1;  // rows past the end are computed and dropped
        const bf16 *qr = q + ((int64_t)b * n + row) * ldq + h * DH;
#pragma unroll
        for (int s = 0; s < KSTEPS; s++) qf[qt][s] = *(const bf16x8 *)(qr + 16 * s + 8 * hf);
    }

    // loads of one macro-tile: per 64-key tile, K_CHUNKS/64 wave loads of K rows and V_CHUNKS/64 of V^T rows, dealt round-robin
    // to the wavefronts.  A wave load fills 64 consecutive 16-byte slots; slot p of row r holds chunk p ^ swizzle(r), applied on
    // the global side.  Keys past the context end re-read its last row (masked later); V^T is zero beyond the length.
    // The macro-tiles are requested in ascending order, so each of a wavefront's NL loads keeps a running per-lane source
    // address that advances by a fixed step per macro-tile; only a tile that reaches past row S-1 of the keys (the last one,
    // when S is not a multiple of 64) computes clamped addresses.
    const bf16 *kbase = kv + (int64_t)b * S * 2 * d + h * DH;
    const bf16 *vbase = vt + ((int64_t)b * d + h * DH) * Spad;
    constexpr int KI = K_CHUNKS / 64, VI = V_CHUNKS / 64, PER_TILE = KI + VI, NL = (SUBS * PER_TILE + NW - 1) / NW;
    const bf16 *lsrc[NL];
#pragma unroll
    for (int i = 0; i < NL; i++) {
        const int idx = i * NW + wave;  // wave-uniform
        const int sub = idx / PER_TILE, w = idx % PER_TILE;
        if (w < KI) {
            const int id = w * 64 + lane, r = id / KCH, pslot = id % KCH;
            const int c = pslot ^ ((KCH == 8 ? (r >> 1) : (r >> 2)) & (KCH - 1));
            lsrc[i] = kbase + (int64_t)(sub * 64 + r) * 2 * d + c * 8;
        } else {
            const int id = (w - KI) * 64 + lane, r = id / 8, pslot = id % 8;
            const int c = pslot ^ ((r >> 1) & 7);
            lsrc[i] = vbase + (int64_t)r * Spad + sub * 64 + c * 8;
        }
    }
    const int64_t kstep = (int64_t)SUBS * 64 * 2 * d, vstep = SUBS * 64;  // elements per macro-tile
    auto issue_macro = [&](int macro, int buf) {  // macro = 0, 1, 2, ... in this order
#pragma unroll
        for (int i = 0; i < NL; i++) {
            const int idx = i * NW + wave;
            const int sub = idx / PER_TILE, w = idx % PER_TILE;
            const int tile = macro * SUBS + sub;
            const bf16 *src = lsrc[i];
            lsrc[i] += w < KI ? kstep : vstep;
            if (idx < SUBS * PER_TILE && tile < ntiles) {
                bf16x8 *dst = smem + buf * MACRO + sub * STAGE + (w < KI ? w * 64 : K_CHUNKS + (w - KI) * 64);
                if (w < KI && tile * 64 + 63 > S - 1) {
                    const int id = w * 64 + lane, r = id / KCH, pslot = id % KCH;
                    const int c = pslot ^ ((KCH == 8 ? (r >> 1) : (r >> 2)) & (KCH - 1));
                    int key = tile * 64 + r;
                    if (key > S - 1) key = S - 1;
                    src = kbase + (int64_t)key * 2 * d + c * 8;
                }
                __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)src,
                                                 (void __attribute__((address_space(3))) *)dst, 16, 0, 0);
            }
        }
    };

    float m_run[QT], l_run[QT];
    floatx16 o[QT][MT];
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int v = 0; v < 16; v++) o[qt][mt][v] = 0.0f;
    }
    // key row read by this lane in the first product: bits 2 and 3 of the row index swapped
    const int krow = (frow & 0x13) | ((frow & 4) << 1) | ((frow & 8) >> 1);

    issue_macro(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (nmacro > 1) issue_macro(1, 1);
    for (int tile = 0; tile < ntiles; tile++) {
        const int macro = tile / SUBS, sub_tile = tile % SUBS;
        if (sub_tile == 0 && macro > 0) {
            // the previous macro-tile is read out and this wave's share of the current one has landed: meet, then refill the free buffer
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (macro + 1 < nmacro) issue_macro(macro + 1, (macro + 1) & 1);
        }
        const bf16x8 *sk = smem + (macro & 1) * MACRO + sub_tile * STAGE, *sv = sk + K_CHUNKS;
        // first product: the two 32-key halves are independent accumulation chains, issued in turn; the key fragments of
        // k-step st+1 are read while step st multiplies
        floatx16 s[QT][2];
#pragma unroll
        for (int sub = 0; sub < 2; sub++)
#pragma unroll
            for (int qt = 0; qt < QT; qt++)
#pragma unroll
                for (int v = 0; v < 16; v++) s[qt][sub][v] = 0.0f;
        auto key_frag = [&](int sub, int st) {
            const int r = sub * 32 + krow;
            return sk[r * KCH + ((2 * st + hf) ^ ((KCH == 8 ? (r >> 1) : (r >> 2)) & (KCH - 1)))];
        };
        bf16x8 kf[2][2];
        kf[0][0] = key_frag(0, 0);
        kf[0][1] = key_frag(1, 0);
#pragma unroll
        for (int st = 0; st < KSTEPS; st++) {
            if (st + 1 < KSTEPS) {
                kf[(st + 1) & 1][0] = key_frag(0, st + 1);
                kf[(st + 1) & 1][1] = key_frag(1, st + 1);
            }
#pragma unroll
            for (int sub = 0; sub < 2; sub++)
#pragma unroll
                for (int qt = 0; qt < QT; qt++)
                    s[qt][sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st & 1][sub], qf[qt][st], s[qt][sub], 0, 0, 0);
        }
        // this lane holds, for beam frow of each tile qt, keys tile*64 + 32*sub + 16*(v/8) + 8*hf + v%8.
        // The softmax is the instruction-bound part of the kernel (about three vector instructions per MFMA flop-cycle),
        // so it is kept lean: scores stay raw and the scale enters through one fused multiply-add per element; only a
        // partial last tile is masked; and the running maximum is refreshed lazily -- as long as no score exceeds the
        // maximum in use by more than 2^8 the old one stays, p <= 256 is harmless in fp32 sums and bf16 operands, and
        // the rescaling of O (one multiply per score element) is skipped.
        const int key0 = tile * 64 + 8 * hf;
        const bool partial = tile * 64 + 64 > len;
        bf16x8 pf[QT][4];
#pragma unroll
        for (int qt = 0; qt < QT; qt++) {
            if (partial) {
#pragma unroll
                for (int sub = 0; sub < 2; sub++)
#pragma unroll
                    for (int v = 0; v < 16; v++)
                        if (key0 + 32 * sub + 16 * (v / 8) + (v % 8) >= len) s[qt][sub][v] = -INFINITY;
            }
            float mx = -INFINITY;
#pragma unroll
            for (int sub = 0; sub < 2; sub++)
#pragma unroll
                for (int v = 0; v < 16; v++) mx = fmaxf(mx, s[qt][sub][v]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2e;  // finite: every tile holds at least one valid key
            if (__builtin_amdgcn_ballot_w64(mx > m_run[qt] + 8.0f) != 0) {  // some beam of the wave outgrew its maximum
                const float mnew = mx > m_run[qt] + 8.0f ? mx : m_run[qt];
                const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - mnew);  // m_run = -inf on the first tile gives 0
                m_run[qt] = mnew;
                l_run[qt] *= alpha;
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
#pragma unroll
                    for (int v = 0; v < 16; v++) o[qt][mt][v] *= alpha;
            }
            const float neg_m = -m_run[qt];
            float lsum = 0.0f;
#pragma unroll
            for (int sub = 0; sub < 2; sub++)
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qt][sub][v], scale_log2e, neg_m));
                    lsum += pv;
                    pf[qt][2 * sub + v / 8][v % 8] = (bf16)pv;  // k-step 2*sub + v/8 of the second product
                }
            l_run[qt] += lsum;  // per half-wave partial sum, joined at the end
        }
        // second product; V^T fragments are shared by the QT beam tiles
#pragma unroll
        for (int ks = 0; ks < 4; ks++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const int r = mt * 32 + frow;
                const bf16x8 vf = sv[r * 8 + ((2 * ks + hf) ^ ((r >> 1) & 7))];
#pragma unroll
                for (int qt = 0; qt < QT; qt++) o[qt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qt][ks], o[qt][mt], 0, 0, 0);
            }
    }
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        const float l = l_run[qt] + __shfl_xor(l_run[qt], 32, 64);
        const float inv = 1.0f / l;
        const int row = q0 + qt * 32 + frow;
        if (row < n) {
            bf16 *orow = out + ((int64_t)b * n + row) * ldo + h * DH;
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    bf16x4 pk;
#pragma unroll
                    for (int j = 0; j < 4; j++) pk[j] = (bf16)(o[qt][mt][4 * g + j] * inv);
                    *(bf16x4 *)(orow + mt * 32 + 8 * g + 4 * hf) = pk;
                }
        }
    }
}

size_t cross_attention_workspace_bytes(gr4ad_dtype dtype, int B, int S, int d, int H) {
    const int dh = d / H;
    if (dtype != GR4AD_BF16 || (dh != 32 && dh != 64) || d % 64) return 0;
    const int64_t Spad = (S + 63) / 64 * 64;
    return (size_t)B * d * Spad * sizeof(bf16);
}

int launch_cross_attention_prepare(gr4ad_dtype dtype, const void *kv, const int32_t *ctx_len, void *vt, int B, int S, int d, int H,
                                   hipStream_t st) {
    if (cross_attention_workspace_bytes(dtype, B, S, d, H) == 0) return GR4AD_OK;  // plain kernel reads kv directly
    if (!vt || ((uintptr_t)vt % 16) || ((uintptr_t)kv % 16)) return GR4AD_EWORKSPACE;
    const int Spad = (S + 63) / 64 * 64;
    if (B > 65535 || d / 64 > 65535) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_V_TRANSPOSE, st, 0.0, 2.0 * B * (double)S * d * sizeof(bf16));
    hipLaunchKernelGGL(v_transpose_kernel, dim3(Spad / 64, d / 64, B), dim3(256), 0, st, (const bf16 *)kv, ctx_len, (bf16 *)vt, S, Spad, d, 2 * d,
                       d);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// xt[b][c][s] = x[b][s][c] for s < len_b, zero beyond (s up to the padded length): the operand layout of the
// P*X product of the lazy layers' cross-attention in absorbed form.  x: [B, S, d] bf16, d % 64 == 0.
int launch_context_transpose(const void *x, const int32_t *ctx_len, void *xt, int B, int S, int d, hipStream_t st) {
    const int Spad = (S + 63) / 64 * 64;
    if (B < 1 || S < 1 || d < 64 || d % 64 || B > 65535 || d / 64 > 65535) return GR4AD_EUNSUPPORTED;
    if (!x || !xt || ((uintptr_t)x % 16) || ((uintptr_t)xt % 16)) return GR4AD_EINVAL;
    ProfScope ps(KC_V_TRANSPOSE, st, 0.0, 2.0 * B * (double)S * d * sizeof(bf16));
    hipLaunchKernelGGL(v_transpose_kernel, dim3(Spad / 64, d / 64, B), dim3(256), 0, st, (const bf16 *)x, ctx_len, (bf16 *)xt, S, Spad, d, d, 0);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// Row softmax over the valid keys of a request: one wavefront per row of raw scores sc [rows, ld] (float32);
// row r belongs to request r / rows_per_req.  p[r, s] = softmax_s(scale * sc[r, s]) over s < len, exactly zero
// for len <= s < ld (the product with the values then runs over whole tiles without a mask).
__global__ __launch_bounds__(256) void masked_softmax_rows(const float *__restrict__ sc, bf16 *__restrict__ p, const int32_t *__restrict__ ctx_len,
                                                           int64_t rows, int rows_per_req, int S, int ld, float scale_log2e) {
    const int lane = threadIdx.x % 64;
    const int64_t r = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
    if (r >= rows) return;
    int len = ctx_len ? ctx_len[r / rows_per_req] : S;
    len = len < 1 ? 1 : (len > S ? S : len);
    const float *row = sc + r * ld;
    bf16 *out = p + r * ld;
    const int full = len & ~3;  // whole float4 groups below len
    float mx = -INFINITY;
    for (int s = lane * 4; s < full; s += 256) {
        const float4 v = *(const float4 *)(row + s);
        mx = fmaxf(fmaxf(mx, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
    }
    for (int s = full + lane; s < len; s += 64) mx = fmaxf(mx, row[s]);
    mx = wave_max(mx) * scale_log2e;  // scale > 0: the max commutes with it
    float sum = 0.f;
    for (int s = lane * 4; s < full; s += 256) {
        const float4 v = *(const float4 *)(row + s);
        sum += exp2f(fmaf(v.x, scale_log2e, -mx)) + exp2f(fmaf(v.y, scale_log2e, -mx)) + exp2f(fmaf(v.z, scale_log2e, -mx)) +
               exp2f(fmaf(v.w, scale_log2e, -mx));
    }
    for (int s = full + lane; s < len; s += 64) sum += exp2f(fmaf(row[s], scale_log2e, -mx));
    const float inv = 1.f / wave_sum(sum);
    for (int s = lane * 4; s < ld; s += 256) {  // ld % 4 == 0
        float e[4] = {0.f, 0.f, 0.f, 0.f};
        if (s + 3 < len) {
            const float4 v = *(const float4 *)(row + s);
            e[0] = v.x; e[1] = v.y; e[2] = v.z; e[3] = v.w;
#pragma unroll
            for (int k = 0; k < 4; k++) e[k] = exp2f(fmaf(e[k], scale_log2e, -mx)) * inv;
        } else {
#pragma unroll
            for (int k = 0; k < 4; k++)
                if (s + k < len) e[k] = exp2f(fmaf(row[s + k], scale_log2e, -mx)) * inv;
        }
        bf16x4 o;
#pragma unroll
        for (int k = 0; k < 4; k++) o[k] = (bf16)e[k];
        *(bf16x4 *)(out + s) = o;
    }
}

int launch_masked_softmax(const float *sc, void *p, const int32_t *ctx_len, int64_t rows, int rows_per_req, int S, int ld, float scale,
                          hipStream_t st) {
    if (rows < 1 || rows_per_req < 1 || S < 1 || ld < S || ld % 4 || !sc || !p || ((uintptr_t)sc % 16) || ((uintptr_t)p % 8)) return GR4AD_EINVAL;
    const int64_t grid = ceil_div64(rows, 4);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_SOFTMAX, st, 0.0, (double)rows * S * (sizeof(float) + sizeof(bf16)));
    hipLaunchKernelGGL(masked_softmax_rows, dim3((unsigned)grid), dim3(256), 0, st, sc, (bf16 *)p, ctx_len, rows, rows_per_req, S, ld,
                       scale * 1.4426950408889634f);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// Lazy layers, cross-attention in absorbed form, one pass over the context.  In that form (eq. trunk with
// q_h . (W_k,h x_s) = (W_k,h^T q_h) . x_s and sum_s p_s W_v,h x_s = W_v,h sum_s p_s x_s) every (position, head) of a
// request is a query q' of width D over keys AND values that are the raw context rows:
//     z[b, i, :] = sum_{s < len_b} softmax_s(scale * q'[b, i, :] . x[b, s, :]) x[b, s, :],      i < RQ = positions * heads.
// One workgroup of 8 wavefronts owns a request and streams its rows once, in double-buffered tiles of 32 rows filled
// by direct global->LDS loads (16-byte piece c of tile row r at position c ^ swz(r), applied on the global side).
// Per tile:
//   1. scores^T [32 rows x 32*QT queries]: the contraction over D is split over the 8/QT wavefronts that share a query
//      tile, each with its slice of q' in registers; all but the first leave their partial sums in LDS;
//   2. the first wavefront of each query tile adds the partials in a fixed order and does the online softmax with
//      lane-local running maximum and sum (a lane owns one query), as the beam-shared kernel above does: raw scores,
//      a maximum that is refreshed only when outgrown by 2^8, unrounded terms in the sum, bf16 terms in the product;
//      it leaves P [queries x 32] and the rescale factor of each query in LDS;
//   3. z^T += x^T P^T: every wavefront owns D/8 columns of z for all queries.  The operand x^T (8 rows of one column
//      per lane) comes from the row-major tile through the transposing LDS read (ds_read_b64_tr_b16: of 16 lanes that
//      pass the addresses of a 4 x 16 block of 16-bit words, four words a lane, lane i receives column i).
// Rows past the length re-read the last valid row (finite) and enter with p = 0.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int ctx_swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }  // 16 rows -> 16 values; 4 rows -> 4 groups of 64 bytes

template <int D, int QT>
__global__ __launch_bounds__(512) void context_attn_flash_bf16(const bf16 *__restrict__ qp, const bf16 *__restrict__ x,
                                                               const int32_t *__restrict__ ctx_len, bf16 *__restrict__ z, int RQ, int rq_stride,
                                                               int S, float scale_log2e) {
    constexpr int ROWB = D * 2, CH = D / 8, TILE = 32 * ROWB;  // bytes per row, 16-byte pieces per row, bytes per tile
    constexpr int KSPLIT = 8 / QT, KSL = D / KSPLIT, KSTEPS = KSL / 16;
    constexpr int CW = D / 8, MT = CW / 32;  // columns of z per wavefront
    constexpr int NL = D / 128;              // wave loads per wavefront and tile (32 * CH / 64 dealt to 8 wavefronts)
    constexpr int NPART = QT * (KSPLIT - 1);
    constexpr int PART = 2 * TILE, PBUF = PART + NPART * 4096, ABUF = PBUF + QT * 2048;
    extern __shared__ __attribute__((aligned(16))) char ctx_lds[];  // 2 tiles | partial scores | P | per-query factor
    const int lane = threadIdx.x % 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int b = blockIdx.x;
    const int r32 = lane % 32, g = lane / 32;
    int len = ctx_len ? ctx_len[b] : S;
    len = len < 1 ? 1 : (len > S ? S : len);
    const int ntiles = (len + 31) / 32;
    const bf16 *xb = x + (int64_t)b * S * D;

    // (Everything a lane derives from its id for addressing is recomputed per tile from a value the compiler cannot see through:
    // hoisted out of the tile loop these addresses cost some 50 registers on top of the 192 that hold q' and z, and the spills
    // that follow are scratch loads whose waits drain the tile loads in flight.)
    auto issue_tile = [&](int tile, int buf) {
        unsigned lv = lane;
        asm volatile("" : "+v"(lv));
#pragma unroll
        for (int i = 0; i < NL; i++) {
            const int idx = i * 8 + wave;  // wave-uniform: 64 consecutive 16-byte slots of the tile
            const unsigned id = idx * 64 + lv;
            const int r = id / CH, pos = id % CH;
            int row = tile * 32 + r;
            if (row > len - 1) row = len - 1;
            const bf16 *src = xb + (int64_t)row * D + (pos ^ ctx_swz(r)) * 8;
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)src,
                                             (void __attribute__((address_space(3))) *)(ctx_lds + buf * TILE + idx * 1024), 16, 0, 0);
        }
    };

    // first product: wavefront = (query tile qh, slice kq of the contraction)
    const int kq = wave % KSPLIT, qh = wave / KSPLIT;
    bf16x8 qf[KSTEPS];
    {
        int qrow = qh * 32 + r32;
        if (qrow > RQ - 1) qrow = RQ - 1;  // queries past the end are computed and dropped
        const bf16 *qr = qp + ((int64_t)b * rq_stride + qrow) * D + kq * KSL + 8 * g;
#pragma unroll
        for (int st = 0; st < KSTEPS; st++) qf[st] = *(const bf16x8 *)(qr + 16 * st);
    }
    float m_run = -INFINITY, l_run = 0.0f;

    // second product: wavefront = columns [wave*CW, wave*CW + CW) of z
    floatx16 o[QT][MT];
#pragma unroll
    for (int qt = 0; qt < QT; qt++)
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int v = 0; v < 16; v++) o[qt][mt][v] = 0.0f;
    issue_tile(0, 0);
    issue_tile(1, 1);  // (unconditional, so that the wait for q' is a count the compiler knows: past the length it re-reads the last row)
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NL) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    for (int tile = 0; tile < ntiles; tile++) {
        char *xt = ctx_lds + (tile & 1) * TILE;
        const uint32_t xt0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)ctx_lds + (tile & 1) * TILE;
        unsigned lv = lane;
        asm volatile("" : "+v"(lv));
        const int r32 = lv % 32, g = lv / 32;
        const int xrow_off = r32 * ROWB, xswz = ctx_swz(r32);
        char *part_w = ctx_lds + PART + (qh * (KSPLIT - 1) + (kq > 0 ? kq - 1 : 0)) * 4096 + r32 * 128;  // this wavefront's partial tile (kq > 0)
        const int prow = qh * 32 + r32;                                                                 // P row of this lane's query
        char *p_w = ctx_lds + PBUF + prow * 64 + g * 8;
        // ---- 1. partial scores^T of this wavefront's slice ----
        floatx16 sacc;
#pragma unroll
        for (int v = 0; v < 16; v++) sacc[v] = 0.0f;
#pragma unroll
        for (int st = 0; st < KSTEPS; st++) {
            const bf16x8 xf = *(const bf16x8 *)(xt + xrow_off + (((kq * (KSL / 8) + 2 * st + g) ^ xswz) * 16));
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, qf[st], sacc, 0, 0, 0);
        }
        // this lane: query r32 of the tile, rows 8i + 4g + e at sacc[4i + e]
        if (kq > 0) {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                floatx4 pk;
#pragma unroll
                for (int e = 0; e < 4; e++) pk[e] = sacc[4 * i + e];
                *(floatx4 *)(part_w + (((2 * i + g) ^ (r32 & 7)) * 16)) = pk;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // ---- 2. online softmax (first wavefront of each query tile) ----
        if (kq == 0) {
#pragma unroll
            for (int k = 0; k < KSPLIT - 1; k++)
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const floatx4 pk = *(const floatx4 *)(part_w + k * 4096 + (((2 * i + g) ^ (r32 & 7)) * 16));
#pragma unroll
                    for (int e = 0; e < 4; e++) sacc[4 * i + e] += pk[e];
                }
            if (tile * 32 + 32 > len) {
#pragma unroll
                for (int v = 0; v < 16; v++)
                    if (tile * 32 + 8 * (v / 4) + 4 * g + (v % 4) >= len) sacc[v] = -INFINITY;
            }
            float mx = -INFINITY;
#pragma unroll
            for (int v = 0; v < 16; v++) mx = fmaxf(mx, sacc[v]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2e;  // finite: every tile holds at least one valid row
            float alpha = 1.0f;
            if (mx > m_run + 8.0f) {
                alpha = __builtin_amdgcn_exp2f(m_run - mx);  // m_run = -inf on the first tile gives 0
                m_run = mx;
                l_run *= alpha;
            }
            const float neg_m = -m_run;
            float lsum = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                bf16x4 pk;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[4 * i + e], scale_log2e, neg_m));
                    lsum += pv;
                    pk[e] = (bf16)pv;
                }
                *(bf16x4 *)(p_w + ((i ^ ((prow >> 2) & 3)) * 16)) = pk;  // rows 8i + 4g .. + 3: half g of 16-byte piece i
            }
            l_run += lsum;  // per half-wave partial sum, joined at the end
            if (g == 0) *(float *)(ctx_lds + ABUF + prow * 4) = alpha;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // ---- 3. z^T += x^T P^T ----
        // the 8-byte piece this lane passes to the transposing read h (rows 8g + 4h + i16/4 of a 16-row k-step), before the column tile
        const int i16 = lv % 16, b1 = (lv / 16) & 1;
        int tr_off[2], tr_swz[2];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int sr = 8 * g + 4 * h + i16 / 4;
            tr_off[h] = sr * ROWB + (i16 & 1) * 8;
            tr_swz[h] = ctx_swz(sr);  // (rows 16 apart share the value)
        }
        const int tr_piece = wave * (CW / 8) + 2 * b1 + (i16 % 4) / 2;
#pragma unroll
        for (int qt = 0; qt < QT; qt++) {
            const float a = *(const float *)(ctx_lds + ABUF + (qt * 32 + r32) * 4);
            if (__builtin_amdgcn_ballot_w64(a != 1.0f) != 0) {
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
#pragma unroll
                    for (int v = 0; v < 16; v++) o[qt][mt][v] *= a;
            }
        }
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            bf16x8 pf[QT];
#pragma unroll
            for (int qt = 0; qt < QT; qt++) {
                const int q = qt * 32 + r32;
                pf[qt] = *(const bf16x8 *)(ctx_lds + PBUF + q * 64 + (((2 * ks + g) ^ ((q >> 2) & 3)) * 16));
            }
            // (The transposing reads are inline assembly: issued through the builtin, each would be preceded by a wait for every
            // tile load in flight.  The wait below carries them as operands so that the MFMAs stay behind it.)
            intx2 t[MT][2];
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    const uint32_t addr = xt0 + ks * 16 * ROWB + tr_off[h] + (((tr_piece + mt * 4) ^ tr_swz[h]) * 16);
                    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(t[mt][h]) : "v"(addr));
                }
            if (MT == 4)
                asm volatile("s_waitcnt lgkmcnt(0)"
                             : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[1][0]), "+v"(t[1][1]), "+v"(t[MT - 2][0]), "+v"(t[MT - 2][1]), "+v"(t[MT - 1][0]),
                               "+v"(t[MT - 1][1]));
            else
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[1][0]), "+v"(t[1][1]));
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const intx4 both = __builtin_shufflevector(t[mt][0], t[mt][1], 0, 1, 2, 3);
                const bf16x8 xf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
                for (int qt = 0; qt < QT; qt++) o[qt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, pf[qt], o[qt][mt], 0, 0, 0);
            }
        }
        // ---- the tile is consumed: refill its buffer two tiles ahead, then wait for the next one ----
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (tile + 2 < ntiles) issue_tile(tile + 2, tile & 1);
        if (tile + 1 < ntiles) {
            if (tile + 2 < ntiles) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NL) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // (a one-tile request never waited for its second buffer: no load may outlive the workgroup's LDS)
    // 1 / sum of every query through LDS (the last barrier of the loop is behind every read of the factors)
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);  // (all lanes: the exchange needs both half-waves)
    if (kq == 0 && g == 0) *(float *)(ctx_lds + ABUF + (qh * 32 + r32) * 4) = 1.0f / l_tot;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        const int q = qt * 32 + r32;
        const float inv = *(const float *)(ctx_lds + ABUF + q * 4);
        if (q < RQ) {
            bf16 *zr = z + ((int64_t)b * rq_stride + q) * D + wave * CW + 4 * g;
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    bf16x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; e++) pk[e] = (bf16)(o[qt][mt][4 * i + e] * inv);
                    *(bf16x4 *)(zr + mt * 32 + 8 * i) = pk;
                }
        }
    }
}

// (more than 64 queries per request run as two launches, each reading the context: beyond 128 the stored-score form moves fewer bytes)
bool context_attention_covers(gr4ad_dtype dtype, int RQ, int d) { return dtype == GR4AD_BF16 && (d == 512 || d == 1024) && RQ >= 1 && RQ <= 128; }

template <int D, int QT>
static int launch_context_flash(const bf16 *qp, const bf16 *x, const int32_t *ctx_len, bf16 *z, int B, int RQ, int rq_stride, int S, float scale,
                                hipStream_t st) {  // RQ <= 32 * QT queries per request, rows rq_stride apart from one request to the next
    auto kern = context_attn_flash_bf16<D, QT>;
    constexpr int LDS_BYTES = 2 * 32 * D * 2 + QT * (8 / QT - 1) * 4096 + QT * 2048 + QT * 128;
    static_assert(LDS_BYTES <= 160 * 1024, "the workgroup's LDS");
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess) return GR4AD_EHIP;
        attr_done = true;
    }
    // flops on the padded length S, both products; bytes: the context once, queries and sums once
    ProfScope ps(KC_CONTEXT_ATTN, st, 4.0 * B * (double)RQ * S * D, (2.0 * B * (double)RQ * D + B * (double)S * D) * sizeof(bf16));
    hipLaunchKernelGGL(kern, dim3((unsigned)B), dim3(512), LDS_BYTES, st, qp, x, ctx_len, z, RQ, rq_stride, S, scale * 1.4426950408889634f);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// z [B, RQ, d] = attention of the queries qp [B, RQ, d] over the context rows x [B, S, d] as keys and values (above).
int launch_context_attention(gr4ad_dtype dtype, const void *qp, const void *x, const int32_t *ctx_len, void *z, int B, int RQ, int S, int d,
                             float scale, hipStream_t st) {
    if (!context_attention_covers(dtype, RQ, d) || B < 1 || S < 1) return GR4AD_EUNSUPPORTED;
    if (!qp || !x || !z || ((uintptr_t)qp % 16) || ((uintptr_t)x % 16) || ((uintptr_t)z % 8)) return GR4AD_EINVAL;
    const bf16 *xx = (const bf16 *)x;
    for (int q0 = 0; q0 < RQ; q0 += 64) {  // 64 queries of every request per launch
        const bf16 *q = (const bf16 *)qp + (int64_t)q0 * d;
        bf16 *zz = (bf16 *)z + (int64_t)q0 * d;
        const int nq = RQ - q0 < 64 ? RQ - q0 : 64;
        int s;
        if (d == 1024) s = nq > 32 ? launch_context_flash<1024, 2>(q, xx, ctx_len, zz, B, nq, RQ, S, scale, st)
                                   : launch_context_flash<1024, 1>(q, xx, ctx_len, zz, B, nq, RQ, S, scale, st);
        else s = nq > 32 ? launch_context_flash<512, 2>(q, xx, ctx_len, zz, B, nq, RQ, S, scale, st)
                         : launch_context_flash<512, 1>(q, xx, ctx_len, zz, B, nq, RQ, S, scale, st);
        if (s) return s;
    }
    return GR4AD_OK;
}

template <int DH, int QT, int NW, int SUBS>
static int launch_flash(const bf16 *q, int64_t ldq, const bf16 *kv, const bf16 *vt, const int32_t *ctx_len, bf16 *out, int64_t ldo, int B,
                        int n, int S, int d, int H, hipStream_t st) {
    auto kern = cross_attn_flash_bf16<DH, QT, NW, SUBS>;
    constexpr int LDS_BYTES = 2 * SUBS * (64 * (DH / 8) + DH * 8) * 16;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess) return GR4AD_EHIP;
        attr_done = true;
    }
    const int per_block = NW * QT * 32;
    const int beam_blocks = (n + per_block - 1) / per_block;
    const int64_t total_blocks = (int64_t)beam_blocks * H * B;
    const int64_t grid = (total_blocks + 7) / 8 * 8;
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)DH);
    // flops on the padded length S; bytes: queries and outputs once, keys and values once per request (beam-shared)
    ProfScope ps(KC_XATTN_FLASH, st, 4.0 * B * (double)n * S * d, (2.0 * B * n * d + 2.0 * B * (double)S * d) * sizeof(bf16));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NW * 64), LDS_BYTES, st, q, ldq, kv, vt, ctx_len, out, ldo, n, S, (S + 63) / 64 * 64, d, H, scale_log2e,
                       beam_blocks, total_blocks);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

int launch_cross_attention(gr4ad_dtype dtype, const void *q, int64_t ldq, const void *kv, const void *vt, const int32_t *ctx_len, void *out,
                           int64_t ldo, int B, int n, int S, int d, int H, hipStream_t st) {
    if (B <= 0 || n <= 0 || S <= 0 || d <= 0 || H <= 0 || d % H) return GR4AD_EINVAL;
    const int dh = d / H;
    if (dh > 128) return GR4AD_EUNSUPPORTED;
    if (vt && cross_attention_workspace_bytes(dtype, B, S, d, H) && ldq % 8 == 0 && ldo % 4 == 0 && ((uintptr_t)q % 16) == 0 &&
        ((uintptr_t)out % 8) == 0) {
        const bf16 *qq = (const bf16 *)q, *kk = (const bf16 *)kv, *vv = (const bf16 *)vt;
        bf16 *oo = (bf16 *)out;
        if (dh == 64) {
            // Measured at 256, 512 and 1024 beams per request: 32 beams per wavefront with single 64-key tiles, four wavefronts
            // per SIMD, beat two-tile staging (-25 %) and 64 beams per wavefront (-10 %), which both halve the wavefronts per
            // SIMD: the kernel waits on LDS, barrier and dependent-MFMA latencies, and occupancy is what hides them.  Blocks
            // of 8 wavefronts (256 beams) share each staged tile among twice as many beams and are 3-7 % faster than blocks
            // of 4; they are used where they waste no more beam slots.
            if (n <= 128) return launch_flash<64, 1, 4, 2>(qq, ldq, kk, vv, ctx_len, oo, ldo, B, n, S, d, H, st);
            if ((n + 255) / 256 * 256 == (n + 127) / 128 * 128) return launch_flash<64, 1, 8, 1>(qq, ldq, kk, vv, ctx_len, oo, ldo, B, n, S, d, H, st);
            return launch_flash<64, 1, 4, 1>(qq, ldq, kk, vv, ctx_len, oo, ldo, B, n, S, d, H, st);
        } else {
            if (n <= 128) return launch_flash<32, 1, 4, 2>(qq, ldq, kk, vv, ctx_len, oo, ldo, B, n, S, d, H, st);
            if (n <= 256) return launch_flash<32, 2, 4, 2>(qq, ldq, kk, vv, ctx_len, oo, ldo, B, n, S, d, H, st);
            return launch_flash<32, 2, 8, 4>(qq, ldq, kk, vv, ctx_len, oo, ldo, B, n, S, d, H, st);
        }
    }
    const int64_t rows = (int64_t)B * n;
    const int64_t grid = ceil_div64(rows * H, 4);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    ProfScope ps(KC_XATTN_SIMPLE, st, 4.0 * B * (double)n * S * d, (2.0 * B * n * d + 2.0 * B * (double)S * d) * (dtype == GR4AD_BF16 ? 2 : 4));
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(cross_attn_simple<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)q, ldq, (const bf16 *)kv, ctx_len, (bf16 *)out, ldo, rows, n, S, d, H);
    else
        hipLaunchKernelGGL(cross_attn_simple<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)q, ldq, (const float *)kv, ctx_len, (float *)out, ldo, rows, n, S, d, H);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}

// ---------------------------------------------------------------------------
// self-attention of the new position over the beam path's earlier positions
// ---------------------------------------------------------------------------
// qkv [rows,3d] of the new position; position p < pos of row r is row anc[r*T + p]
// of the [*,3d] buffer level p wrote (keys at column d, values at 2d); the
// query attends to 0..pos.  Beams that share an ancestor read the same row.
// One thread owns 8 consecutive channels of one row (16-byte accesses in bf16); the
// dh/8 threads of a head are neighbouring lanes and join their partial dot products
// with xor-shuffles, so every access of a wavefront is one contiguous stretch.
template <typename T> struct Chunk8;
template <> struct Chunk8<bf16> {
    static __device__ __forceinline__ void load(const bf16 *p, float *o) {
        const bf16x8 v = *(const bf16x8 *)p;
#pragma unroll
        for (int i = 0; i < 8; i++) o[i] = (float)v[i];
    }
    static __device__ __forceinline__ void store(bf16 *p, const float *o) {
        bf16x8 v;
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] = (bf16)o[i];
        *(bf16x8 *)p = v;
    }
};
template <> struct Chunk8<float> {
    static __device__ __forceinline__ void load(const float *p, float *o) {
        const floatx4 a = *(const floatx4 *)p, b = *(const floatx4 *)(p + 4);
#pragma unroll
        for (int i = 0; i < 4; i++) { o[i] = a[i]; o[4 + i] = b[i]; }
    }
    static __device__ __forceinline__ void store(float *p, const float *o) {
        floatx4 a, b;
#pragma unroll
        for (int i = 0; i < 4; i++) { a[i] = o[i]; b[i] = o[4 + i]; }
        *(floatx4 *)p = a;
        *(floatx4 *)(p + 4) = b;
    }
};

template <typename T>
__global__ __launch_bounds__(256) void self_attn_step(const T *__restrict__ qkv, LevelBuffers prev, const int32_t *__restrict__ anc,
                                                      T *__restrict__ out, int64_t rows, int pos, int Tlev, int d, int H) {
    const int cpr = d / 8;        // chunks per row
    const int lph = (d / H) / 8;  // lanes per head: 2, 4, 8 or 16
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = gid < rows * cpr;
    const int64_t row = live ? gid / cpr : rows - 1;  // idle lanes shadow the last row and store nothing
    const int ch = live ? (int)(gid % cpr) : 0;
    const float scale = 1.0f / sqrtf((float)(d / H));
    const T *qr = qkv + row * 3 * d + ch * 8;
    float qv[8], kn[8], vn[8];
    Chunk8<T>::load(qr, qv);
    Chunk8<T>::load(qr + d, kn);
    Chunk8<T>::load(qr + 2 * d, vn);
    const T *kvp[GR4AD_MAX_LEVELS];  // k of position p (v follows d elements later)
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++)
        if (p < pos) kvp[p] = (const T *)prev.p[p] + (int64_t)anc[row * Tlev + p] * 3 * d + d + ch * 8;
    float s[GR4AD_MAX_LEVELS];
    float mx = -INFINITY;
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++) {
        if (p <= pos) {
            float kk[8];
            if (p == pos) {
#pragma unroll
                for (int i = 0; i < 8; i++) kk[i] = kn[i];
            } else {
                Chunk8<T>::load(kvp[p], kk);
            }
            float part = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; i++) part = fmaf(qv[i], kk[i], part);
            for (int o = 1; o < lph; o <<= 1) part += __shfl_xor(part, o, 64);
            s[p] = part * scale;
            mx = fmaxf(mx, s[p]);
        }
    }
    float den = 0.0f;
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++)
        if (p <= pos) { s[p] = __expf(s[p] - mx); den += s[p]; }
    const float inv = 1.0f / den;
    float o8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int p = 0; p < GR4AD_MAX_LEVELS; p++) {
        if (p <= pos) {
            float vv[8];
            if (p == pos) {
#pragma unroll
                for (int i = 0; i < 8; i++) vv[i] = vn[i];
            } else {
                Chunk8<T>::load(kvp[p] + d, vv);
            }
            const float w = s[p] * inv;
#pragma unroll
            for (int i = 0; i < 8; i++) o8[i] = fmaf(w, vv[i], o8[i]);
        }
    }
    if (live) Chunk8<T>::store(out + row * d + ch * 8, o8);
}

int launch_self_attention_step(gr4ad_dtype dtype, const void *qkv, const LevelBuffers &prev, const int32_t *anc, void *out, int64_t rows,
                               int pos, int T, int d, int H, hipStream_t st) {
    // T is the row stride of anc: positions 0..pos-1 are read from it, so pos == T (a step after the last level) is allowed
    if (rows <= 0 || pos < 0 || pos > T || pos >= GR4AD_MAX_LEVELS || T > GR4AD_MAX_LEVELS || d % H) return GR4AD_EINVAL;
    if (pos > 0 && !anc) return GR4AD_EINVAL;
    for (int p = 0; p < pos; p++)
        if (!prev.p[p] || ((uintptr_t)prev.p[p] % 32) || prev.rows[p] < 1) return GR4AD_EINVAL;
    const int dh = d / H;
    if (dh != 16 && dh != 32 && dh != 64 && dh != 128) return GR4AD_EUNSUPPORTED;
    if (((uintptr_t)qkv % 32) || ((uintptr_t)out % 32)) return GR4AD_EUNSUPPORTED;
    const int64_t grid = ceil_div64(rows * (d / 8), 256);
    if (grid > 0x7fffffffLL) return GR4AD_EUNSUPPORTED;
    // reads q,k,v of the new position and the pos earlier (k,v) pairs of the beam's path, writes the output
    // (beams that share an ancestor share its row: an earlier level contributes at most its own size)
    double units = 4.0 * rows;
    for (int p = 0; p < pos; p++) units += 2.0 * (double)(prev.rows[p] > 0 && prev.rows[p] < rows ? prev.rows[p] : rows);
    ProfScope ps(KC_SELF_STEP, st, 4.0 * rows * (double)(pos + 1) * d, units * d * (dtype == GR4AD_BF16 ? 2 : 4));
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(self_attn_step<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)qkv, prev, anc, (bf16 *)out, rows, pos, T, d, H);
    else
        hipLaunchKernelGGL(self_attn_step<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)qkv, prev, anc, (float *)out, rows, pos, T, d, H);
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
    ProfScope ps(KC_TRUNK_SELF, st, 0.0, (double)rows * d * 4 * (dtype == GR4AD_BF16 ? 2 : 4));
    if (dtype == GR4AD_BF16)
        hipLaunchKernelGGL(trunk_self_attn<bf16>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16 *)qkv, (bf16 *)out, rows, T, d, H);
    else
        hipLaunchKernelGGL(trunk_self_attn<float>, dim3((unsigned)grid), dim3(256), 0, st, (const float *)qkv, (float *)out, rows, T, d, H);
    GR4AD_LAUNCH_CHECK();
    return GR4AD_OK;
}
