"""The C library's serving policies (include/gr4ad_serving.h) against the plain-Python oracle on seeded traces, plus
argument validation.  Host code only: no GPU is touched."""
import ctypes as C

import numpy as np
import pytest

from oracle.serving import CacheOracle, TabsOracle
from paper_2602_22732_amd import binding


@pytest.mark.parametrize("seed,kw", [
    (1, dict(qps_peak=1000.0)),
    (2, dict(qps_peak=400.0, scale_min=0.25, scale_max=1.0, step=0.25, tau_s=3.0)),     # a load-adaptive sweep below the base schedule
    (3, dict(qps_peak=2500.0, scale_min=1.0, scale_max=2.0, step=0.05, tau_s=30.0)),
])
def test_tabs_controller_follows_the_oracle_on_a_day_of_traffic(seed, kw):
    rng = np.random.default_rng(seed)
    base, maxb, V = [128, 256, 512], [512, 512, 1024], [4096, 4096, 4096]
    lib_c = binding.TabsController(base, maxb, V, **kw)
    orc = TabsOracle(base, maxb, V, **kw)
    t = 0.0
    for i in range(6000):
        dt = float(rng.choice([0.0, 0.01, 0.05, 0.3, 2.0]))
        t += dt
        # peak / off-peak cycle with bursts
        rate = kw["qps_peak"] * (0.15 + 1.1 * (0.5 + 0.5 * np.sin(t / 40.0)) ** 2) * (3.0 if rng.random() < 0.01 else 1.0)
        n = int(rng.poisson(rate * max(dt, 0.01)))
        lib_c.observe(t, n)
        orc.observe(t, n)
        assert abs(lib_c.qps() - orc.q) <= 1e-9 * max(1.0, orc.q)
        if i % 3 == 0:
            c_avail = float(rng.choice([1.0, 0.9, 0.6]))
            got = lib_c.schedule(t, c_avail)
            want = orc.schedule(t, c_avail)
            assert got[0] == want[0] and abs(got[1] - want[1]) < 1e-12, (i, got, want)
    lib_c.close()


def test_tabs_argument_validation():
    L = binding.lib()
    base, maxb, V = binding._i32arr([4, 4]), binding._i32arr([8, 8]), binding._i32arr([16, 16])
    out = C.c_void_p()

    def make(**over):
        kw = dict(n_levels=2, beam_base=base[1], max_beam=maxb[1], codebook=V[1], qps_peak=10.0, scale_min=1.0, scale_max=1.6, step=0.1, tau_s=1.0)
        kw.update(over)
        return L.gr4ad_tabs_create(C.byref(binding.TabsConfig(**kw)), C.byref(out))

    assert make() == 0
    h = C.c_void_p(out.value)
    for bad in (dict(n_levels=0), dict(n_levels=9), dict(qps_peak=0.0), dict(scale_min=0.0), dict(scale_max=0.5), dict(step=0.0), dict(tau_s=-1.0),
                dict(qps_peak=float("nan"))):
        assert make(**bad) == -1
    assert L.gr4ad_tabs_create(None, C.byref(out)) == -1
    beam = (C.c_int32 * 2)()
    assert L.gr4ad_tabs_observe(h, 5.0, 3) == 0
    assert L.gr4ad_tabs_observe(h, 4.0, 3) == -1          # time runs backwards
    assert L.gr4ad_tabs_observe(h, 6.0, -1) == -1
    assert L.gr4ad_tabs_schedule(h, 6.0, 0.0, beam, None) == -1
    assert L.gr4ad_tabs_schedule(h, 6.0, 1.5, beam, None) == -1
    assert L.gr4ad_tabs_schedule(h, 6.0, 1.0, None, None) == -1
    assert L.gr4ad_tabs_schedule(h, 6.0, 1.0, beam, None) == 0 and list(beam) == [4, 4]
    assert L.gr4ad_tabs_qps(None) < 0 and L.gr4ad_tabs_observe(None, 0.0, 0) == -1
    L.gr4ad_tabs_free(h)
    L.gr4ad_tabs_free(None)


def payload(rng, n, T):
    return rng.integers(0, 4096, (n, T)).astype(np.int32), -np.sort(rng.random(n)).astype(np.float32)


@pytest.mark.parametrize("seed,capacity,ttl,users", [(11, 10 ** 5, 60.0, 3000), (12, 64, 60.0, 500), (13, 5, 1e9, 40), (14, 300, 2.0, 200)])
def test_result_cache_follows_the_oracle_on_a_request_trace(seed, capacity, ttl, users):
    rng = np.random.default_rng(seed)
    T, max_items = 3, 6
    lib_c = binding.ResultCache(capacity, ttl, T, max_items)
    orc = CacheOracle(capacity, ttl)
    t = 0.0
    for i in range(15000):
        t += float(rng.exponential(0.2))
        key = int(rng.zipf(1.2) * 2654435761 % users) if i % 7 else int(rng.integers(0, 2 ** 63))  # a few never-seen users
        want = orc.lookup(key, t)
        got = lib_c.lookup(key, t)
        assert (got is None) == (want is None), i
        if got is not None:
            assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
        else:
            p = payload(rng, int(rng.integers(1, max_items + 1)), T)
            lib_c.insert(key, t, *p)
            orc.insert(key, t, p)
        if i % 500 == 0:
            s = lib_c.stats()
            assert (s["lookups"], s["hits"], s["entries"], s["evictions"], s["expired"]) == (orc.lookups, orc.hits, len(orc.entries), orc.evictions, orc.expired)
    s = lib_c.stats()
    assert s["hits"] == orc.hits and s["evictions"] == orc.evictions and s["expired"] == orc.expired and 0 < s["hits"] < s["lookups"]
    lib_c.close()


def test_result_cache_batches_and_window_boundary():
    rng = np.random.default_rng(3)
    T = 4
    lib_c, orc = binding.ResultCache(100, 60.0, T, 8), CacheOracle(100, 60.0)
    t = 0.0
    for step in range(300):
        t += 1.5
        keys = (rng.zipf(1.4, 32) % 60).astype(np.uint64)
        hit, miss = lib_c.lookup_batch(keys, t)
        want_hit, want_miss = orc.lookup_batch([int(k) for k in keys], t)
        assert hit.tolist() == want_hit and miss.tolist() == want_miss
        for i in miss:                       # the decoded results of the misses go in
            p = payload(rng, 8, T)
            lib_c.insert(int(keys[i]), t, *p)
            orc.insert(int(keys[i]), t, p)
    s = lib_c.stats()
    assert (s["lookups"], s["hits"], s["entries"]) == (orc.lookups, orc.hits, len(orc.entries))
    # one minute, inclusive
    c = binding.ResultCache(4, 60.0, 2, 2)
    c.insert(9, 100.0, [[1, 2]], [-0.5])
    got = c.lookup(9, 160.0)
    assert got is not None and got[0].tolist() == [[1, 2]] and got[1].tolist() == [-0.5]
    assert c.lookup(9, 160.001) is None and c.stats()["expired"] == 1 and c.stats()["entries"] == 0


def test_result_cache_argument_validation():
    L = binding.lib()
    out = C.c_void_p()
    assert L.gr4ad_cache_create(0, 60.0, 3, 4, C.byref(out)) == -1
    assert L.gr4ad_cache_create(10, -1.0, 3, 4, C.byref(out)) == -1
    assert L.gr4ad_cache_create(10, 60.0, 0, 4, C.byref(out)) == -1
    assert L.gr4ad_cache_create(10, 60.0, 3, 0, C.byref(out)) == -1
    assert L.gr4ad_cache_create(10, 60.0, 3, 4, None) == -1
    c = binding.ResultCache(10, 60.0, 3, 4)
    with pytest.raises(binding.Gr4adError):
        c.insert(1, 0.0, np.zeros((5, 3), np.int32), np.zeros(5, np.float32))    # more items than an entry holds
    assert L.gr4ad_cache_lookup(None, 1, 0.0, None, None, None) == -1
    assert L.gr4ad_cache_lookup(c.handle, 1, 0.0, None, None, None) == 0
    assert L.gr4ad_cache_stats(None, None, None, None, None, None) == -1
    L.gr4ad_cache_free(None)
