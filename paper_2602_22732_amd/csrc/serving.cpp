// Host-side serving policies around the decoder (section 4.2 of the paper, Efficiency Optimization): the Traffic-Aware
// Adaptive Beam Search controller (section 4.2.1) and the Reco Result Cache (section 4.2.2).  Plain host C++, no GPU calls.
#include <math.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "../../include/gr4ad.h"
#include "../../include/gr4ad_serving.h"

// ---------------------------------------------------------------------------
// TABS: B_t = B_base * f(Q_t, C_avail)
// ---------------------------------------------------------------------------
struct gr4ad_tabs {
    int T;
    int32_t base[GR4AD_MAX_LEVELS], max_beam[GR4AD_MAX_LEVELS], V[GR4AD_MAX_LEVELS];
    double qps_peak, smin, smax, step, tau;
    // traffic estimate: Q before the last interval, that interval's length and arrivals (reports that share a time stamp
    // are merged into it), arrivals stamped with the very first time
    bool started;
    double t, q, q_before, dt_last;
    double n_last, first;
    // scale in use = smin + k * step; time of the last raise
    int64_t k;
    bool raised;
    double t_up;
    std::mutex mu;
};

static int tabs_observe_locked(gr4ad_tabs *c, double t, double n) {
    if (!c->started) {
        c->started = true;
        c->t = t;
        c->first = n;
        return GR4AD_OK;
    }
    if (t < c->t) return GR4AD_EINVAL;
    const double dt = t - c->t;
    if (dt == 0) {
        if (c->dt_last == 0) {
            c->first += n;
            return GR4AD_OK;
        }
        c->n_last += n;
    } else {
        c->q_before = c->q;
        c->dt_last = dt;
        c->n_last = n + c->first;
        c->first = 0;
        c->t = t;
    }
    const double decay = exp(-c->dt_last / c->tau);
    c->q = c->q_before * decay + (c->n_last / c->dt_last) * (1.0 - decay);
    return GR4AD_OK;
}

extern "C" {

int gr4ad_tabs_create(const gr4ad_tabs_config *cfg, gr4ad_tabs **out) {
    if (!cfg || !out || !cfg->beam_base || !cfg->max_beam || !cfg->codebook) return GR4AD_EINVAL;
    if (cfg->n_levels < 1 || cfg->n_levels > GR4AD_MAX_LEVELS) return GR4AD_EINVAL;
    if (!(cfg->qps_peak > 0) || !(cfg->scale_min > 0) || !(cfg->scale_max >= cfg->scale_min) || !(cfg->step > 0) || !(cfg->tau_s > 0))
        return GR4AD_EINVAL;
    for (int t = 0; t < cfg->n_levels; t++)
        if (cfg->beam_base[t] < 1 || cfg->max_beam[t] < 1 || cfg->codebook[t] < 1) return GR4AD_EINVAL;
    gr4ad_tabs *c = new (std::nothrow) gr4ad_tabs();
    if (!c) return GR4AD_ENOMEM;
    c->T = cfg->n_levels;
    for (int t = 0; t < c->T; t++) { c->base[t] = cfg->beam_base[t]; c->max_beam[t] = cfg->max_beam[t]; c->V[t] = cfg->codebook[t]; }
    c->qps_peak = cfg->qps_peak; c->smin = cfg->scale_min; c->smax = cfg->scale_max; c->step = cfg->step; c->tau = cfg->tau_s;
    c->started = false; c->t = 0; c->q = 0; c->q_before = 0; c->dt_last = 0; c->n_last = 0; c->first = 0;
    c->k = 0; c->raised = false; c->t_up = 0;
    *out = c;
    return GR4AD_OK;
}

void gr4ad_tabs_free(gr4ad_tabs *c) { delete c; }

int gr4ad_tabs_observe(gr4ad_tabs *c, double t_s, int32_t n_requests) {
    if (!c || n_requests < 0 || !(t_s == t_s)) return GR4AD_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    return tabs_observe_locked(c, t_s, (double)n_requests);
}

double gr4ad_tabs_qps(const gr4ad_tabs *c) {
    if (!c) return -1.0;
    std::lock_guard<std::mutex> g(const_cast<gr4ad_tabs *>(c)->mu);
    return c->q;
}

int gr4ad_tabs_schedule(gr4ad_tabs *c, double t_s, double c_avail, int32_t *out_beam, double *out_scale) {
    if (!c || !out_beam || !(c_avail > 0) || c_avail > 1.0 || !(t_s == t_s)) return GR4AD_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    int s = tabs_observe_locked(c, t_s, 0.0);
    if (s) return s;
    // decode cost is linear in the scale: the largest scale the available compute sustains at the current traffic
    double target = c->q <= 0 ? c->smax : c_avail * c->qps_peak / c->q;
    if (target > c->smax) target = c->smax;
    if (target < c->smin) target = c->smin;
    const int64_t kq = (int64_t)floor((target - c->smin) / c->step + 1e-9);
    if (kq < c->k) {
        c->k = kq;  // less slack: at once
    } else if (kq > c->k && (!c->raised || t_s - c->t_up >= c->tau)) {
        c->k += 1;  // more slack: one step, at most once per time constant
        c->raised = true;
        c->t_up = t_s;
    }
    const double scale = c->smin + (double)c->k * c->step;
    int64_t prev = 1;
    for (int t = 0; t < c->T; t++) {
        int64_t w = (int64_t)floor((double)c->base[t] * scale + 0.5);
        if (w < 1) w = 1;
        if (w > c->max_beam[t]) w = c->max_beam[t];
        if (w > prev * c->V[t]) w = prev * c->V[t];
        out_beam[t] = (int32_t)w;
        prev = w;
    }
    if (out_scale) *out_scale = scale;
    return GR4AD_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------
// Result cache: open-addressing table of slots, slots chained oldest -> newest
// ---------------------------------------------------------------------------
// The time to live is the same for every entry, so insertion order is expiry order: one list serves both the
// capacity eviction (oldest first) and the order in which entries expire.  Payloads live in two flat arrays indexed by
// slot.  Deletion uses backward-shift, so lookups never meet tombstones.
struct gr4ad_cache {
    int64_t capacity, nslots, mask;  // nslots: power of two >= 2 * capacity
    double ttl;
    int T, max_items;
    struct Slot { uint64_t key; double t; int32_t n; int64_t older, newer; bool used; };
    std::vector<Slot> slots;
    std::vector<int32_t> sid;   // [nslots][max_items * T]
    std::vector<float> lp;      // [nslots][max_items]
    int64_t oldest, newest, entries;
    int64_t lookups, hits, evictions, expired;
    std::mutex mu;
};

namespace {

inline uint64_t mix(uint64_t x) {  // splitmix64 finaliser
    x += 0x9e3779b97f4a7c15ull;
    x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
    x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
    return x ^ (x >> 31);
}

int64_t find_slot(const gr4ad_cache *c, uint64_t key) {
    int64_t i = (int64_t)(mix(key) & (uint64_t)c->mask);
    while (c->slots[i].used) {
        if (c->slots[i].key == key) return i;
        i = (i + 1) & c->mask;
    }
    return -1;
}

void unlink(gr4ad_cache *c, int64_t i) {
    gr4ad_cache::Slot &s = c->slots[i];
    if (s.older >= 0) c->slots[s.older].newer = s.newer; else c->oldest = s.newer;
    if (s.newer >= 0) c->slots[s.newer].older = s.older; else c->newest = s.older;
}

void relink(gr4ad_cache *c, int64_t from, int64_t to) {  // the entry moved from slot `from` to slot `to`
    gr4ad_cache::Slot &s = c->slots[to];
    if (s.older >= 0) c->slots[s.older].newer = to; else c->oldest = to;
    if (s.newer >= 0) c->slots[s.newer].older = to; else c->newest = to;
    (void)from;
}

void erase_slot(gr4ad_cache *c, int64_t i) {
    unlink(c, i);
    c->slots[i].used = false;
    c->entries--;
    // backward shift: pull later members of the probe run into the hole
    int64_t hole = i, j = (i + 1) & c->mask;
    while (c->slots[j].used) {
        const int64_t home = (int64_t)(mix(c->slots[j].key) & (uint64_t)c->mask);
        const bool movable = ((j - home) & c->mask) >= ((j - hole) & c->mask);
        if (movable) {
            c->slots[hole] = c->slots[j];
            const size_t ps = (size_t)c->max_items * c->T, pl = (size_t)c->max_items;
            memcpy(&c->sid[(size_t)hole * ps], &c->sid[(size_t)j * ps], (size_t)c->slots[j].n * c->T * sizeof(int32_t));
            memcpy(&c->lp[(size_t)hole * pl], &c->lp[(size_t)j * pl], (size_t)c->slots[j].n * sizeof(float));
            c->slots[j].used = false;
            relink(c, j, hole);
            hole = j;
        }
        j = (j + 1) & c->mask;
    }
}

// 1 hit, 0 miss; counts the lookup
int lookup_locked(gr4ad_cache *c, uint64_t key, double now, int32_t *out_sid, float *out_lp, int32_t *out_n) {
    c->lookups++;
    const int64_t i = find_slot(c, key);
    if (i < 0) return 0;
    if (now - c->slots[i].t > c->ttl) {
        erase_slot(c, i);
        c->expired++;
        return 0;
    }
    c->hits++;
    const int32_t n = c->slots[i].n;
    if (out_sid) memcpy(out_sid, &c->sid[(size_t)i * c->max_items * c->T], (size_t)n * c->T * sizeof(int32_t));
    if (out_lp) memcpy(out_lp, &c->lp[(size_t)i * c->max_items], (size_t)n * sizeof(float));
    if (out_n) *out_n = n;
    return 1;
}

}  // namespace

extern "C" {

int gr4ad_cache_create(int64_t capacity, double ttl_s, int32_t n_levels, int32_t max_items, gr4ad_cache **out) {
    if (!out || capacity < 1 || capacity > ((int64_t)1 << 40) || !(ttl_s >= 0) || n_levels < 1 || n_levels > GR4AD_MAX_LEVELS || max_items < 1)
        return GR4AD_EINVAL;
    gr4ad_cache *c = new (std::nothrow) gr4ad_cache();
    if (!c) return GR4AD_ENOMEM;
    c->capacity = capacity; c->ttl = ttl_s; c->T = n_levels; c->max_items = max_items;
    int64_t n = 8;
    while (n < 2 * capacity) n <<= 1;
    c->nslots = n; c->mask = n - 1;
    try {
        gr4ad_cache::Slot empty;
        memset(&empty, 0, sizeof(empty));
        empty.older = empty.newer = -1;
        c->slots.assign((size_t)n, empty);
        c->sid.assign((size_t)n * max_items * n_levels, 0);
        c->lp.assign((size_t)n * max_items, 0.0f);
    } catch (const std::bad_alloc &) {
        delete c;
        return GR4AD_ENOMEM;
    }
    c->oldest = c->newest = -1; c->entries = 0;
    c->lookups = c->hits = c->evictions = c->expired = 0;
    *out = c;
    return GR4AD_OK;
}

void gr4ad_cache_free(gr4ad_cache *c) { delete c; }

int gr4ad_cache_insert(gr4ad_cache *c, uint64_t key, double now_s, const int32_t *sid, const float *logprob, int32_t n) {
    if (!c || !sid || !logprob || n < 1 || n > c->max_items || !(now_s == now_s)) return GR4AD_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    int64_t i = find_slot(c, key);
    if (i >= 0) {
        erase_slot(c, i);  // replaced: the new result becomes the newest entry
    } else if (c->entries >= c->capacity) {
        erase_slot(c, c->oldest);
        c->evictions++;
    }
    i = (int64_t)(mix(key) & (uint64_t)c->mask);
    while (c->slots[i].used) i = (i + 1) & c->mask;
    gr4ad_cache::Slot &s = c->slots[i];
    s.key = key; s.t = now_s; s.n = n; s.used = true;
    s.older = c->newest; s.newer = -1;
    if (c->newest >= 0) c->slots[c->newest].newer = i; else c->oldest = i;
    c->newest = i;
    c->entries++;
    memcpy(&c->sid[(size_t)i * c->max_items * c->T], sid, (size_t)n * c->T * sizeof(int32_t));
    memcpy(&c->lp[(size_t)i * c->max_items], logprob, (size_t)n * sizeof(float));
    return GR4AD_OK;
}

int gr4ad_cache_lookup(gr4ad_cache *c, uint64_t key, double now_s, int32_t *out_sid, float *out_logprob, int32_t *out_n) {
    if (!c || !(now_s == now_s)) return GR4AD_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    return lookup_locked(c, key, now_s, out_sid, out_logprob, out_n);
}

int gr4ad_cache_lookup_batch(gr4ad_cache *c, const uint64_t *keys, int32_t B, double now_s, uint8_t *hit, int32_t *miss_index, int32_t *n_miss) {
    if (!c || !keys || !hit || !miss_index || !n_miss || B < 1 || !(now_s == now_s)) return GR4AD_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    // users of this batch whose request is already on the list to decode: a small open-addressing set of indices into keys
    int64_t cap = 16;
    while (cap < 2 * (int64_t)B) cap <<= 1;
    std::vector<int32_t> pending;
    try {
        pending.assign((size_t)cap, -1);
    } catch (const std::bad_alloc &) {
        return GR4AD_ENOMEM;
    }
    int32_t m = 0;
    for (int32_t i = 0; i < B; i++) {
        bool dup = false;  // an earlier request of this batch is being decoded for the same user
        int64_t h = (int64_t)(mix(keys[i]) & (uint64_t)(cap - 1));
        while (pending[h] >= 0 && !dup) {
            dup = keys[pending[h]] == keys[i];
            if (!dup) h = (h + 1) & (cap - 1);
        }
        if (dup) {
            c->lookups++;
            c->hits++;
            hit[i] = 1;
        } else if (lookup_locked(c, keys[i], now_s, nullptr, nullptr, nullptr)) {
            hit[i] = 1;
        } else {
            hit[i] = 0;
            miss_index[m++] = i;
            pending[h] = i;  // h is the empty slot the probe ended on
        }
    }
    *n_miss = m;
    return GR4AD_OK;
}

int gr4ad_cache_stats(const gr4ad_cache *c, int64_t *lookups, int64_t *hits, int64_t *entries, int64_t *evictions, int64_t *expired) {
    if (!c) return GR4AD_EINVAL;
    std::lock_guard<std::mutex> g(const_cast<gr4ad_cache *>(c)->mu);
    if (lookups) *lookups = c->lookups;
    if (hits) *hits = c->hits;
    if (entries) *entries = c->entries;
    if (evictions) *evictions = c->evictions;
    if (expired) *expired = c->expired;
    return GR4AD_OK;
}

}  // extern "C"
