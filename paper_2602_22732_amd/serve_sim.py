"""Serving loop on a synthetic request trace: result cache and traffic-aware beam schedule around gr4ad_decode_batch.

    python -m paper_2602_22732_amd.serve_sim [--config 3] [--ticks 240] [--no-cache] [--no-tabs]

Every policy decision is taken by the C library (include/gr4ad_serving.h) and every decode by gr4ad_decode_batch; this
file only generates the trace, moves results between them and prints one JSON line with what was measured: cache hit
rate, decodes, beam scale in use, GPU time and requests served per second of GPU time.

Trace (seeded, stands in for production traffic): one tick per 0.25 s of trace time; arrivals per tick are Poisson with a
peak / off-peak cycle of 60 s between 0.3 and 1.0 of `--peak-batch`; with probability `--repeat` an arrival is a user drawn
uniformly from the arrivals of the last 45 s, otherwise a new user (section 4.2.2 reports 27.8 % of requests served from a
one-minute cache; the default reproduces about that rate).  A user's context is one of a pool of synthetic contexts of the
configuration's shape.
"""
import argparse
import json
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--ticks", type=int, default=240)
    ap.add_argument("--peak-batch", type=int, default=256, help="mean arrivals per tick at peak (the decoder's max_batch is twice that)")
    ap.add_argument("--repeat", type=float, default=0.28)
    ap.add_argument("--ttl", type=float, default=60.0)
    ap.add_argument("--no-cache", action="store_true")
    ap.add_argument("--no-tabs", action="store_true")
    ap.add_argument("--seed", type=int, default=20260227)
    args = ap.parse_args()

    import torch
    from . import binding, synth

    w = synth.workload(args.config)
    max_batch = 2 * args.peak_batch
    w.B = max_batch
    W = synth.make_weights(w)
    tabs_max = [min(binding_max, int(b * 1.6 + 0.5)) for b, binding_max in zip(w.beam, [4096] * w.T)]
    dec = binding.decoder_for(w, W, max_beam=tabs_max)
    dev = torch.device("cuda:0")
    td = binding.torch_dtype(w.dtype)
    pool_n = 128
    lens_pool = synth.make_lengths(synth.workload(args.config, batch=pool_n))
    pool = torch.empty(pool_n, w.S, w.d, dtype=td, device=dev)
    for r in range(pool_n):
        pool[r] = torch.from_numpy(synth.make_context_request(w, r, int(lens_pool[r]))).to(dev, dtype=td)
    lens_dev = torch.from_numpy(lens_pool).to(dev)
    ws = torch.empty(dec.workspace_bytes(max_batch, w.S, tabs_max), dtype=torch.uint8, device=dev)

    dt_tick = 0.25
    # what one GPU sustains at the base schedule: calibrated on the spot with a full batch
    ctx = pool[torch.arange(max_batch, device=dev) % pool_n].contiguous()
    cl = lens_dev[torch.arange(max_batch, device=dev) % pool_n].contiguous()
    for _ in range(2):
        dec.decode_batch(ctx, cl, w.beam, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        dec.decode_batch(ctx, cl, w.beam, workspace=ws)
    torch.cuda.synchronize()
    qps_base = 3 * max_batch / (time.perf_counter() - t0)
    # the deployment is provisioned for the trace's peak: at peak the GPU is exactly busy at the base schedule
    qps_peak_trace = args.peak_batch / dt_tick
    tabs = binding.TabsController(w.beam, tabs_max, w.V, qps_peak=qps_peak_trace, scale_min=1.0, scale_max=1.6, step=0.1, tau_s=5.0)
    cache = binding.ResultCache(1 << 20, args.ttl, w.T, w.beam[-1] if args.no_tabs else tabs_max[-1])

    rng = np.random.default_rng(args.seed)
    recent = []  # (time, user) of the last 45 s
    next_user = 1
    served = decoded = 0
    gpu_s = host_policy_s = 0.0
    scales = []
    for tick in range(args.ticks):
        t = tick * dt_tick
        load = 0.3 + 0.7 * (0.5 + 0.5 * np.sin(2 * np.pi * t / 60.0))
        n = int(min(max_batch, max(1, rng.poisson(args.peak_batch * load))))
        recent = [(tt, u) for tt, u in recent if t - tt <= 45.0]
        keys = np.empty(n, np.uint64)
        for i in range(n):
            if recent and rng.random() < args.repeat:
                keys[i] = recent[int(rng.integers(len(recent)))][1]
            else:
                keys[i] = next_user
                next_user += 1
        recent.extend((t, int(k)) for k in keys)
        h0 = time.perf_counter()
        tabs.observe(t, n)
        beam, scale = (list(w.beam), 1.0) if args.no_tabs else tabs.schedule(t, 1.0)
        if args.no_cache:
            miss = np.arange(n, dtype=np.int32)
        else:
            _, miss = cache.lookup_batch(keys, t)
        host_policy_s += time.perf_counter() - h0
        scales.append(scale)
        served += n
        if len(miss):
            idx = torch.from_numpy((keys[miss] % pool_n).astype(np.int64)).to(dev)
            ctx = pool[idx].contiguous()
            cl = lens_dev[idx].contiguous()
            torch.cuda.synchronize()
            g0 = time.perf_counter()
            sid, lp = dec.decode_batch(ctx, cl, beam, workspace=ws)
            torch.cuda.synchronize()
            gpu_s += time.perf_counter() - g0
            decoded += len(miss)
            if not args.no_cache:
                sid_h, lp_h = sid.cpu().numpy(), lp.cpu().numpy()
                h0 = time.perf_counter()
                for j, i in enumerate(miss):
                    cache.insert(int(keys[i]), t, sid_h[j], lp_h[j])
                host_policy_s += time.perf_counter() - h0
    stats = cache.stats()
    print(json.dumps({
        "workload": "config %d %s, trace of %d ticks x %.2f s, peak %d arrivals/tick" % (w.cfg_id, w.name, args.ticks, dt_tick, args.peak_batch),
        "cache": not args.no_cache, "tabs": not args.no_tabs, "requests": served, "decoded": decoded,
        "hit_rate": 1.0 - decoded / served, "cache_stats": stats, "mean_beam_scale": float(np.mean(scales)),
        "scale_at_peak": float(np.min(scales)), "scale_off_peak": float(np.max(scales)), "gpu_seconds": gpu_s,
        "requests_per_gpu_second": served / gpu_s, "full_batch_requests_per_s_at_base_schedule": qps_base,
        "host_policy_us_per_request": 1e6 * host_policy_s / served}))


if __name__ == "__main__":
    main()
