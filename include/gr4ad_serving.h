/*
 * gr4ad_serving.h -- host-side serving policies around gr4ad_decode_batch (C ABI, host memory only, no GPU calls).
 *
 * Two pieces of the paper's deployment (section 4.2, Efficiency Optimization):
 *   - Traffic-Aware Adaptive Beam Search (section 4.2.1): the beam schedule of a call is the base schedule times a
 *     scale B_t = B_base * f(Q_t, C_avail) that grows when traffic is below what the deployment sustains and never
 *     drops below the base schedule at peak (with the defaults of the paper: unchanged at peak, +60 % off-peak).
 *   - Reco Result Cache (section 4.2.2): results of a user's request are reused for that user's later requests inside a
 *     short time window (one minute in the paper), which serves those requests without a decode.
 *
 * The paper leaves f undefined.  The reading taken here: decode cost grows linearly with the beam scale (measured),
 * so the largest scale the available compute sustains at the current traffic is C_avail * qps_peak / Q_t; f is that
 * value clamped to [scale_min, scale_max], rounded down to a multiple of `step` above scale_min, lowered at once and
 * raised by at most one step per time constant.
 *
 * All functions return GR4AD_OK (0) or a negative gr4ad_status unless stated.  Objects are internally locked: calls on
 * one object from several threads are serialised.  Times are seconds on any monotone clock of the caller's choosing.
 */
#ifndef GR4AD_SERVING_H
#define GR4AD_SERVING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- Traffic-Aware Adaptive Beam Search controller (section 4.2.1) -------------------------------------------------- */
typedef struct gr4ad_tabs gr4ad_tabs;

typedef struct {
    int32_t n_levels;          /* T, 1..8 */
    const int32_t *beam_base;  /* host [T]: B_base, the schedule at scale 1 */
    const int32_t *max_beam;   /* host [T]: the decoder's max_beam (upper clamp of every width) */
    const int32_t *codebook;   /* host [T]: V_t (a width never exceeds the previous width times V_t) */
    double qps_peak;           /* requests/s the deployment sustains at scale 1 with all of its compute, > 0 */
    double scale_min;          /* clamp of f from below, > 0 (1.0: never below the base schedule) */
    double scale_max;          /* clamp of f from above, >= scale_min (1.6: the paper's +60 % off-peak) */
    double step;               /* scales are scale_min + k * step, step > 0 */
    double tau_s;              /* time constant of the traffic estimate and shortest time between two raises, > 0 */
} gr4ad_tabs_config;

/* Copies the configuration.  EINVAL on a bad field.  The controller starts at scale_min with Q_t = 0. */
int gr4ad_tabs_create(const gr4ad_tabs_config *cfg, gr4ad_tabs **out);
void gr4ad_tabs_free(gr4ad_tabs *ctl); /* NULL is a no-op */

/* n_requests arrived at time t_s (t_s must not run backwards: EINVAL).  Updates the traffic estimate
 *   Q <- Q * exp(-dt/tau) + (n/dt) * (1 - exp(-dt/tau)),  dt = t_s - time of the previous update
 * Reports that share a time stamp belong to the same interval: the last update is redone with their sum.  Arrivals
 * stamped with the controller's very first time are counted in the first interval. */
int gr4ad_tabs_observe(gr4ad_tabs *ctl, double t_s, int32_t n_requests);

/* Q_t as of the last update; negative on a NULL controller. */
double gr4ad_tabs_qps(const gr4ad_tabs *ctl);

/* The schedule to decode with at time t_s when a fraction c_avail in (0, 1] of the deployment's compute is available:
 * updates the estimate as observe(t_s, 0) would, moves the scale by the rule in the header comment, and writes
 *   out_beam[t] = min(max_beam[t], out_beam[t-1] * V_t, max(1, floor(beam_base[t] * scale + 0.5)))      host [T]
 * and the scale in use to *out_scale (may be NULL). */
int gr4ad_tabs_schedule(gr4ad_tabs *ctl, double t_s, double c_avail, int32_t *out_beam, double *out_scale);

/* ---- Reco Result Cache (section 4.2.2) ------------------------------------------------------------------------------ */
typedef struct gr4ad_cache gr4ad_cache;

/* capacity: most entries held at once (an insert into a full cache evicts the oldest entry); ttl_s: an entry answers
 * lookups up to and including ttl_s seconds after it was inserted; an entry holds up to max_items SIDs of n_levels
 * codes each with their log-probabilities.  EINVAL on non-positive sizes, ENOMEM if the table cannot be allocated. */
int gr4ad_cache_create(int64_t capacity, double ttl_s, int32_t n_levels, int32_t max_items, gr4ad_cache **out);
void gr4ad_cache_free(gr4ad_cache *c); /* NULL is a no-op */

/* Stores (or replaces, making it the newest entry) the result of `key`'s request decoded at now_s:
 * sid host [n, n_levels] int32, logprob host [n] float32, 1 <= n <= max_items. */
int gr4ad_cache_insert(gr4ad_cache *c, uint64_t key, double now_s, const int32_t *sid, const float *logprob, int32_t n);

/* Returns 1 and copies the entry (out_sid host [max_items, n_levels], out_logprob host [max_items], *out_n items;
 * any of the three may be NULL) if `key` has an entry no older than ttl_s; returns 0 otherwise (an entry found
 * expired is dropped); negative on error. */
int gr4ad_cache_lookup(gr4ad_cache *c, uint64_t key, double now_s, int32_t *out_sid, float *out_logprob, int32_t *out_n);

/* A batch of B requests at now_s: hit[i] = 1 if keys[i] is served from the cache (a key that occurs again later in
 * the same batch counts as a hit from its second occurrence on: one decode serves them all), else 0 and i is appended
 * to miss_index; *n_miss = number of requests to decode.  hit, miss_index host [B]. */
int gr4ad_cache_lookup_batch(gr4ad_cache *c, const uint64_t *keys, int32_t B, double now_s, uint8_t *hit, int32_t *miss_index,
                             int32_t *n_miss);

/* counters since creation; any pointer may be NULL */
int gr4ad_cache_stats(const gr4ad_cache *c, int64_t *lookups, int64_t *hits, int64_t *entries, int64_t *evictions, int64_t *expired);

#ifdef __cplusplus
}
#endif
#endif
