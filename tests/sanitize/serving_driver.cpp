// Sanitizer driver of the host-side serving policies (csrc/serving.cpp, compiled into this program with
// -fsanitize=address,undefined): the result cache under four capacity / time-to-live regimes with payload checks, batch
// lookups with repeated keys, and the beam controller through bursts, idle stretches and bad arguments.
// Exit status 0 = clean and consistent.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../../include/gr4ad.h"
#include "../../include/gr4ad_serving.h"

static int cache_rounds() {
    std::mt19937_64 rng(1);
    for (int round = 0; round < 4; round++) {
        const int64_t cap = round == 0 ? 3 : round == 1 ? 50 : round == 2 ? 1000 : 7;
        gr4ad_cache *c;
        if (gr4ad_cache_create(cap, round == 3 ? 0.5 : 5.0, 3, 4, &c)) return 1;
        double t = 0;
        for (int i = 0; i < 60000; i++) {
            t += 0.001 * (double)(rng() % 10);
            const uint64_t key = rng() % (uint64_t)(cap * 3 + 5);
            int32_t sid[12], n;
            float lp[4];
            const int r = gr4ad_cache_lookup(c, key, t, sid, lp, &n);
            if (r < 0) return 2;
            if (r == 1) {
                for (int j = 0; j < n * 3; j++)
                    if (sid[j] != (int32_t)(key * 31 + (uint64_t)j)) return 3;
            } else {
                n = 1 + (int32_t)(rng() % 4);
                for (int j = 0; j < n * 3; j++) sid[j] = (int32_t)(key * 31 + (uint64_t)j);
                for (int j = 0; j < n; j++) lp[j] = -(float)j;
                if (gr4ad_cache_insert(c, key, t, sid, lp, n)) return 4;
            }
            if (i % 1000 == 0) {
                uint64_t keys[9];
                for (auto &k : keys) k = rng() % 6;
                uint8_t hit[9];
                int32_t miss[9], nm;
                if (gr4ad_cache_lookup_batch(c, keys, 9, t, hit, miss, &nm) || nm < 0 || nm > 9) return 5;
            }
        }
        int64_t lk, h, e, ev, ex;
        gr4ad_cache_stats(c, &lk, &h, &e, &ev, &ex);
        if (e > cap || h > lk) return 6;
        gr4ad_cache_free(c);
    }
    gr4ad_cache *c = nullptr;
    if (gr4ad_cache_create(0, 1.0, 3, 4, &c) != GR4AD_EINVAL) return 7;
    gr4ad_cache_free(nullptr);
    return 0;
}

static int tabs_rounds() {
    const int32_t base[3] = {128, 256, 512}, mx[3] = {4096, 4096, 4096}, V[3] = {4096, 4096, 4096};
    gr4ad_tabs_config cfg = {3, base, mx, V, 1000.0, 1.0, 1.6, 0.1, 2.0};
    gr4ad_tabs *ctl;
    if (gr4ad_tabs_create(&cfg, &ctl)) return 1;
    std::mt19937_64 rng(7);
    double t = 0;
    for (int i = 0; i < 20000; i++) {
        t += 0.0005 * (double)(1 + rng() % 20);
        const int burst = (i / 2000) % 2 ? 1 + (int)(rng() % 40) : (int)(rng() % 3);
        if (gr4ad_tabs_observe(ctl, t, burst)) return 2;
        if (i % 7 == 0) {
            int32_t beam[3];
            double scale;
            if (gr4ad_tabs_schedule(ctl, t, 0.25 + 0.75 * (double)(rng() % 100) / 99.0, beam, &scale)) return 3;
            if (scale < 1.0 - 1e-12 || scale > 1.6 + 1e-12 || beam[0] < 128 || beam[2] > 4096) return 4;
        }
    }
    if (gr4ad_tabs_observe(ctl, t - 1.0, 1) != GR4AD_EINVAL) return 5;
    if (gr4ad_tabs_qps(ctl) < 0) return 6;
    gr4ad_tabs_free(ctl);
    gr4ad_tabs_free(nullptr);
    cfg.qps_peak = 0;
    if (gr4ad_tabs_create(&cfg, &ctl) != GR4AD_EINVAL) return 7;
    return 0;
}

int main() {
    int rc;
    if ((rc = cache_rounds())) return rc;
    if ((rc = tabs_rounds())) return 20 + rc;
    printf("serving sanitizer driver: ok\n");
    return 0;
}
