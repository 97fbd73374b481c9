/* Sanitizer driver of the CPU oracle (test infrastructure): the oracle's source is compiled into this translation unit
 * with -fsanitize=address,undefined and every entry point runs on a small seeded model - the definition, the cached search,
 * the pre-cut search, FP8 mode, the vanilla decoder, ragged context lengths, a rejected beam schedule, the primitives.
 * The three searches must return the same beams.  Exit status 0 = clean and consistent. */
#include "../../oracle/gr4ad_oracle.c"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static float rnd(void) { /* uniform in [-1, 1) */
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(rng_state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *vec(size_t n, float scale) {
    float *p = (float *)malloc(sizeof(float) * n);
    for (size_t i = 0; i < n; i++) p[i] = rnd() * scale;
    return p;
}

static int run(int fp8, int vanilla, int K) {
    enum { d = 16, H = 2, F = 24, L = 3, T = 3, S = 7, B = 3 };
    const int32_t V[T] = {5, 7, 6}, beam[T] = {3, 6, 4}, lens[B] = {7, 1, 4};
    orc_desc ds = {d, H, F, L, K, T, V, 1e-6f, fp8, vanilla};
    orc_layer_w layers[L];
    float *owned[L][13];
    for (int l = 0; l < L; l++) {
        const size_t sz[13] = {d, d * d, d * d, d * d, d * d, d, d * d, d * d, d * d, d * d, d, F * d, d * F};
        for (int i = 0; i < 13; i++) owned[l][i] = vec(sz[i], sz[i] == d ? 1.0f : 0.4f);
        orc_layer_w w = {owned[l][0], owned[l][1], owned[l][2], owned[l][3], owned[l][4], owned[l][5], owned[l][6],
                         owned[l][7], owned[l][8], owned[l][9], owned[l][10], owned[l][11], owned[l][12]};
        layers[l] = w;
    }
    float *pos = vec(T * d, 1), *bos = vec(d, 1), *wg = vec(d * d, 0.4f), *wf = vec(2 * d * d, 0.4f), *ln = vec(d, 1);
    const float *emb[T - 1], *cls[T], *bias[T];
    float *eo[T], *co[T], *bo = vec(V[1], 1);
    for (int t = 0; t < T; t++) { co[t] = vec((size_t)V[t] * d, 0.5f); cls[t] = co[t]; bias[t] = t == 1 ? bo : NULL; }
    for (int t = 0; t + 1 < T; t++) { eo[t] = vec((size_t)V[t] * d, 1); emb[t] = eo[t]; }
    orc_weights w = {pos, bos, emb, vanilla ? NULL : wg, vanilla ? NULL : wf, layers, ln, cls, bias};
    orc_model *m = orc_model_create(&ds, &w);
    if (!m) return 10;
    float *X = vec((size_t)B * S * d, 1);
    const int bT = beam[T - 1], tot = 3 + 6 + 4;
    int32_t sid[3][B * 4 * T], tp[B * 13], tt[B * 13];
    double lp[3][B * 4], ts[B * 13];
    for (int mode = 0; mode < 3; mode++)
        if (orc_decode_batch(m, X, lens, B, S, beam, sid[mode], lp[mode], tp, tt, ts, mode)) return 11;
    for (int mode = 1; mode < 3; mode++) {
        if (memcmp(sid[0], sid[mode], sizeof(int32_t) * B * bT * T)) return 12;
        for (int i = 0; i < B * bT; i++) if (fabs(lp[0][i] - lp[mode][i]) > 1e-9) return 13;
    }
    (void)tot;
    const int32_t bad[T] = {6, 1, 1};
    if (orc_decode_batch(m, X, NULL, B, S, bad, sid[0], lp[0], NULL, NULL, NULL, 0) == 0) return 14;
    orc_req *rq = orc_req_create(m, X, 5);
    double cum[2], dist[2 * 6], last[7];
    const int32_t pre[4] = {1, 2, 4, 0};
    orc_prefix_dists(m, rq, 3, 2, pre, cum, dist);
    if (vanilla) orc_vanilla_ar_seq(m, rq, 2, pre, last); else orc_plain_ar_seq(m, rq, 2, pre, last);
    double s = 0;
    for (int v = 0; v < 6; v++) s += exp(dist[v]);
    if (fabs(s - 1) > 1e-9) return 15;
    orc_req_free(rq);
    orc_model_free(m);
    for (int l = 0; l < L; l++) for (int i = 0; i < 13; i++) free(owned[l][i]);
    free(pos); free(bos); free(wg); free(wf); free(ln); free(bo); free(X);
    for (int t = 0; t < T; t++) free(co[t]);
    for (int t = 0; t + 1 < T; t++) free(eo[t]);
    return 0;
}

int main(void) {
    int rc;
    if ((rc = run(0, 0, 1))) return rc;
    if ((rc = run(0, 0, 0))) return rc + 20;
    if ((rc = run(1, 0, 2))) return rc + 40;
    if ((rc = run(0, 1, 0))) return rc + 60;
    if ((rc = run(1, 1, 0))) return rc + 80;
    /* primitives on their own */
    double z[5] = {0.5, -1, 2, 2, -3}, y[5], sc[6] = {0.1, 0.7, 0.7, -2, 0.3, 0.7}, ks[3];
    int64_t flat[3];
    orc_prim_log_softmax(y, z, 5);
    orc_prim_topk(sc, 2, 3, 3, flat, ks, 1);
    if (flat[0] != 1 || flat[1] != 2 || flat[2] != 5) return 100;
    orc_prim_e4m3(y, z, 5);
    orc_prim_quant_rows(y, z, 1, 5);
    printf("oracle sanitizer driver: ok\n");
    return 0;
}
