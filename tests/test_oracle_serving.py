"""Pins of the serving-policy oracle (section 4.2): closed forms of the traffic estimate and of f, the figures the
paper gives (unchanged at peak, +60 % off-peak, one-minute window), schedule arithmetic, and the cache against a
brute-force scan of the request history."""
import math

import numpy as np

from oracle.serving import CacheOracle, TabsOracle

BASE, MAXB, V = [128, 256, 512], [1024, 1024, 1024], [4096, 4096, 4096]


def test_traffic_estimate_closed_forms():
    o = TabsOracle(BASE, MAXB, V, qps_peak=1000.0, tau_s=10.0)
    # constant rate r from t = 0, whatever the reporting interval: Q(t) = r (1 - exp(-t / tau))
    t, r = 0.0, 640.0
    o.observe(0.0, 0)
    for dt in [0.1, 0.5, 0.02, 3.0, 1.0, 7.5, 0.25] * 6:
        t += dt
        o.observe(t, r * dt)
        assert abs(o.q - r * (1 - math.exp(-t / 10.0))) < 1e-9 * r
    # silence: pure decay
    q0, t0 = o.q, t
    o.observe(t + 25.0, 0)
    assert abs(o.q - q0 * math.exp(-2.5)) < 1e-9 * q0
    # arrivals that share a time stamp are not lost
    a, b = TabsOracle(BASE, MAXB, V, 1000.0), TabsOracle(BASE, MAXB, V, 1000.0)
    a.observe(0.0, 0); a.observe(1.0, 30); a.observe(2.0, 50)
    b.observe(0.0, 0); b.observe(1.0, 10); b.observe(1.0, 20); b.observe(2.0, 50)
    assert abs(a.q - b.q) < 1e-12


def settle(o, rate, c_avail, seconds=400.0, dt=0.5):
    t = o.t or 0.0
    end = t + seconds
    out = None
    while t < end:
        t += dt
        o.observe(t, rate * dt)
        out = o.schedule(t, c_avail)
    return out


def test_peak_keeps_the_base_schedule_and_off_peak_gains_sixty_percent():
    o = TabsOracle(BASE, MAXB, V, qps_peak=1000.0, scale_min=1.0, scale_max=1.6, step=0.1, tau_s=5.0)
    beam, scale = settle(o, 1000.0, 1.0)          # at the sustained peak: unchanged
    assert scale == 1.0 and beam == BASE
    beam, scale = settle(o, 2500.0, 1.0)          # overload never goes below the base schedule
    assert scale == 1.0 and beam == BASE
    beam, scale = settle(o, 300.0, 1.0)           # far off-peak: the paper's +60 %
    assert abs(scale - 1.6) < 1e-9 and beam == [205, 410, 819]
    beam, scale = settle(o, 800.0, 1.0)           # 1000 / 800 = 1.25 -> rounded down to 1.2
    assert abs(scale - 1.2) < 1e-9 and beam == [154, 307, 614]
    beam, scale = settle(o, 800.0, 0.8)           # only 80 % of the compute available: no slack
    assert scale == 1.0
    # steady state: more traffic never widens the beams
    scales = [settle(TabsOracle(BASE, MAXB, V, 1000.0, tau_s=5.0), q, 1.0)[1] for q in range(100, 2000, 100)]
    assert all(x >= y for x, y in zip(scales, scales[1:]))


def test_scale_drops_at_once_and_rises_one_step_per_time_constant():
    o = TabsOracle(BASE, MAXB, V, qps_peak=1000.0, step=0.1, tau_s=10.0)
    o.observe(0.0, 0)
    ups, t = [], 0.0
    while t < 80.0:                                # no traffic: the target is scale_max from the first call
        t += 1.0
        ups.append(o.schedule(t, 1.0)[1])
    changes = [i for i in range(1, len(ups)) if ups[i] != ups[i - 1]]
    assert abs(ups[0] - 1.1) < 1e-9 and abs(ups[-1] - 1.6) < 1e-9
    assert all(b - a == 10 for a, b in zip(changes, changes[1:]))        # one raise every tau seconds
    # a burst: the very next call is back at the base schedule
    o.observe(t + 0.5, 40000)
    assert o.schedule(t + 0.5, 1.0)[1] == 1.0


def test_schedule_clamps():
    o = TabsOracle([600, 900, 40], [1000, 1000, 4096], [64, 2, 4096], qps_peak=10.0, scale_max=2.0, step=0.5, tau_s=1.0)
    o.observe(0.0, 0)
    for t in (1.0, 2.0, 3.0):
        beam, scale = o.schedule(t, 1.0)
    assert scale == 2.0
    # level 1: min(1200, max_beam 1000, 1 * 64) = 64; level 2: min(1800, 1000, 64 * 2) = 128; level 3: 80
    assert beam == [64, 128, 80]
    o2 = TabsOracle([1, 1], [8, 8], [8, 8], qps_peak=10.0, scale_min=0.25, scale_max=1.0, step=0.25, tau_s=1.0)
    o2.observe(0.0, 0)
    assert o2.schedule(0.5, 1.0)[0] == [1, 1]      # floor(0.25 + 0.5) = 0 -> at least 1


def history_scan(history, key, now, ttl):
    """Definition: the user's newest earlier result, if it is young enough."""
    times = [t for k, t in history if k == key]
    return bool(times) and now - max(times) <= ttl


def test_cache_equals_history_scan_when_nothing_is_evicted():
    rng = np.random.default_rng(5)
    c = CacheOracle(capacity=10 ** 6, ttl_s=60.0)
    history, t, hits = [], 0.0, 0
    for _ in range(20000):
        t += rng.exponential(0.05)
        key = int(rng.zipf(1.3)) % 5000
        want = history_scan(history, key, t, 60.0)
        got = c.lookup(key, t) is not None
        assert got == want
        hits += got
        if not got:
            c.insert(key, t, True)
            history.append((key, t))
    assert c.hits == hits and c.lookups == 20000 and 0.05 < hits / 20000 < 0.95


def test_cache_window_boundary_periodic_user_and_eviction_order():
    c = CacheOracle(capacity=3, ttl_s=60.0)
    c.insert(7, 100.0, "a")
    assert c.lookup(7, 160.0) == "a"               # exactly one minute later: still served
    assert c.lookup(7, 160.0 + 1e-6) is None and c.expired == 1 and 7 not in c.entries
    # a user who asks every 20 s with a one-minute window: miss, hit, hit, hit, miss, ...
    c2, pattern = CacheOracle(10, 60.0), []
    for i in range(12):
        got = c2.lookup(1, 20.0 * i) is not None
        pattern.append(int(got))
        if not got:
            c2.insert(1, 20.0 * i, i)
    assert pattern == [0, 1, 1, 1] * 3
    # capacity: the oldest entry goes first; replacing an entry makes it the newest
    c3 = CacheOracle(3, 1e9)
    for k in (1, 2, 3):
        c3.insert(k, float(k), k)
    c3.insert(1, 4.0, "new")                       # refresh 1: order is now 2, 3, 1
    c3.insert(4, 5.0, 4)                           # evicts 2
    assert list(c3.entries) == [3, 1, 4] and c3.evictions == 1 and c3.lookup(1, 6.0) == "new"


def test_batch_lookup_counts_a_repeated_user_once():
    c = CacheOracle(10, 60.0)
    c.insert(5, 0.0, "x")
    hit, miss = c.lookup_batch([9, 5, 9, 8, 9, 5], 1.0)
    assert hit == [0, 1, 1, 0, 1, 1] and miss == [0, 3]
