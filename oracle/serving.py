"""CPU ORACLE of the host-side serving policies (test infrastructure, not the product).

Plain Python, written from the paper's section 4.2 (Efficiency Optimization):

  * TabsOracle  -- Traffic-Aware Adaptive Beam Search (section 4.2.1): B_t = B_base * f(Q_t, C_avail).  The paper leaves f
                   undefined; the reading taken (the same the C library documents): decode cost is linear in the beam
                   scale, so the largest sustainable scale is C_avail * qps_peak / Q_t, clamped to [scale_min, scale_max],
                   rounded down to scale_min + k * step, lowered at once, raised by one step at most once per tau.
                   Q_t is an exponentially weighted arrival rate with time constant tau.
  * CacheOracle -- Reco Result Cache (section 4.2.2): per-user results reused for a bounded interval (TTL), bounded number
                   of entries, oldest entry evicted first.

Only tests may import this module.  It shares no code with the C library.
"""
import math
from collections import OrderedDict


class TabsOracle:
    def __init__(self, beam_base, max_beam, codebook, qps_peak, scale_min=1.0, scale_max=1.6, step=0.1, tau_s=10.0):
        self.base, self.max_beam, self.V = list(beam_base), list(max_beam), list(codebook)
        self.qps_peak, self.smin, self.smax, self.step, self.tau = qps_peak, scale_min, scale_max, step, tau_s
        self.q = 0.0          # Q_t
        self.t = None         # time of the last update
        self.q_before = 0.0   # Q before the last interval, that interval's length and arrivals: reports that share a
        self.dt_last = 0.0    # time stamp belong to the same interval, so the last update is redone with their sum
        self.n_last = 0
        self.first = 0        # arrivals stamped with the very first time (counted in the first interval)
        self.k = 0            # the scale in use is scale_min + k * step
        self.t_up = None      # time of the last raise

    def observe(self, t, n):
        if self.t is None:
            self.t, self.first = t, n
            return
        if t < self.t:
            raise ValueError("time runs backwards")
        dt = t - self.t
        if dt == 0:
            if self.dt_last == 0:          # still at the very first time stamp
                self.first += n
                return
            self.n_last += n
        else:
            self.q_before, self.dt_last, self.n_last = self.q, dt, n + self.first
            self.first = 0
            self.t = t
        # the arrivals of an interval spread evenly over it
        decay = math.exp(-self.dt_last / self.tau)
        self.q = self.q_before * decay + (self.n_last / self.dt_last) * (1.0 - decay)

    def schedule(self, t, c_avail):
        self.observe(t, 0)
        target = self.smax if self.q <= 0 else c_avail * self.qps_peak / self.q
        target = min(self.smax, max(self.smin, target))
        kq = int(math.floor((target - self.smin) / self.step + 1e-9))
        if kq < self.k:
            self.k = kq
        elif kq > self.k and (self.t_up is None or t - self.t_up >= self.tau):
            self.k += 1
            self.t_up = t
        scale = self.smin + self.k * self.step
        beam, prev = [], 1
        for b, mb, v in zip(self.base, self.max_beam, self.V):
            w = max(1, int(math.floor(b * scale + 0.5)))
            w = min(w, mb, prev * v)
            beam.append(w)
            prev = w
        return beam, scale


class CacheOracle:
    def __init__(self, capacity, ttl_s):
        self.capacity, self.ttl = capacity, ttl_s
        self.entries = OrderedDict()   # key -> (time of insertion, payload), oldest first
        self.lookups = self.hits = self.evictions = self.expired = 0

    def insert(self, key, now, payload):
        if key in self.entries:
            del self.entries[key]
        elif len(self.entries) >= self.capacity:
            self.entries.popitem(last=False)
            self.evictions += 1
        self.entries[key] = (now, payload)

    def lookup(self, key, now):
        self.lookups += 1
        e = self.entries.get(key)
        if e is None:
            return None
        if now - e[0] > self.ttl:
            del self.entries[key]
            self.expired += 1
            return None
        self.hits += 1
        return e[1]

    def lookup_batch(self, keys, now):
        hit, miss, seen = [], [], set()
        for i, k in enumerate(keys):
            if k in seen:              # an earlier request of this batch is being decoded for the same user
                self.lookups += 1
                self.hits += 1
                hit.append(1)
                continue
            if self.lookup(k, now) is not None:
                hit.append(1)
            else:
                hit.append(0)
                miss.append(i)
                seen.add(k)
        return hit, miss
