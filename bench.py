#!/usr/bin/env python3
"""Benchmark of the LazyAR beam-decode hot path on one MI355X.

A step is one gr4ad_decode_batch call over one batch of synthetic requests that
are already resident in HBM: context K/V projection, lazy pass, and for every
level Fuse, the autoregressive layers, classifier, log-softmax + top-k selection
and beam reorder.  Prints ONE JSON line (requests/s, plus candidates/s,
beam-rows/s, the roofline of the dominant kernel and the CPU oracle timed on
the host cores).

    python bench.py [--config 5] [--scale 1.0] [--steps 5] [--warmup 2] [--no-cpu]

Default: configuration 5 at beam scale 1.0, the largest-batch configuration (2048 requests).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15   # dense bf16 MFMA, FLOP/s
PEAK_FP8_MFMA = 5.0e15    # dense fp8 MFMA, FLOP/s
PEAK_F32_VALU = 157.3e12  # fp32 vector FLOP/s
PEAK_HBM = 8.0e12         # HBM3E, B/s


def algorithmic_flops(w, lens):
    """Algorithmic flops of one batch (1 MAC = 2): what the method must compute."""
    d, F, T, A, K, S = w.d, w.F, w.T, w.A, w.K, w.S
    lens = np.asarray(lens, np.float64)
    R = float(sum(w.rows))
    per_req = {
        "ctx_kv": A * 4.0 * lens.mean() * d * d,
        "lazy": T * K * (12.0 * d * d + 4.0 * d * F + 4.0 * lens.mean() * d),
        "fuse": 0.0 if w.vanilla else R * 2.0 * d * d,
        "ar_gemm": R * A * (12.0 * d * d + 4.0 * d * F),
        "cross_attn": R * A * 4.0 * lens.mean() * d,
        "self_attn": sum(n * A * 4.0 * (t + 1) * d for t, n in enumerate(w.rows)),
        "classifier": sum(n * 2.0 * d * V for n, V in zip(w.rows, w.V)),
    }
    if w.Ve > 0:  # eCPM-token step: one more position of the lazy pass and one more level for the b_T returned beams
        n = float(w.beam[-1])
        per_req["lazy"] *= (T + 1.0) / T
        per_req["fuse"] += 0.0 if w.vanilla else n * 2.0 * d * d
        per_req["ar_gemm"] += n * A * (12.0 * d * d + 4.0 * d * F)
        per_req["cross_attn"] += n * A * 4.0 * lens.mean() * d
        per_req["self_attn"] += n * A * 4.0 * (T + 1) * d
        per_req["classifier"] += n * 2.0 * d * w.Ve
    return {k: v * w.B for k, v in per_req.items()}


def kernel_sources_sha256():
    """Hash of the library's kernel sources (csrc/*, sorted by name): names the code a counter summary was measured on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2602_22732_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def measured_traffic(cfg_id):
    """HBM bytes per decode_batch call and kernel class, measured with rocprofv3 counters (FETCH_SIZE + WRITE_SIZE,
    scaled by a copy kernel of known size), read from the committed summary of that run.  The counters cannot be read
    inside this process, so the summary records the hash of the kernel sources it was measured on; figures of another
    version of the kernels are not reported.  Returns ({kernel: bytes}, note)."""
    import re
    name = "decode_batch_config%d_hbm_traffic.md" % cfg_id
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return {}, "no counter summary profiles/%s" % name
    out, sha = {}, None
    for line in open(path):
        m = re.match(r"^\|\s*(\w+)\s*\|.*\|\s*([0-9.eE+]+)\s*\|\s*$", line)
        if m:
            out[m.group(1)] = float(m.group(2))
        m = re.match(r"^kernel sources sha256:\s*([0-9a-f]{64})", line)
        if m:
            sha = m.group(1)
    if sha != kernel_sources_sha256():
        return {}, "profiles/%s was measured on other kernel sources (sha256 %s): not reported" % (name, sha and sha[:12])
    return out, "rocprofv3 FETCH_SIZE/WRITE_SIZE run of this command, profiles/%s (kernel sources sha256 %s)" % (name, sha[:12])


def cpu_baseline(w, W, lens):
    """Times the CPU oracle as it stands on a bounded sample of the same workload: one request per host thread (the oracle's
    batch driver then runs one request per thread), float32 build (the precision the task states for the oracle; the parity
    tests use the double build of the same source)."""
    import oracle
    from paper_2602_22732_amd import synth
    cores = int(os.environ.get("OMP_NUM_THREADS", 0)) or len(os.sched_getaffinity(0))
    n = min(w.B, max(cores, {1: 4, 2: 64, 3: 16}.get(w.cfg_id, 1)))
    X = synth.make_context(w, lens, requests=range(n))
    o = oracle.Oracle(weights=W, precision="f32", **w.model_kwargs())
    t0 = time.perf_counter()
    o.decode_batch(X, lens[:n], w.beam)
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "requests/s", "cores": cores, "kind": "oracle",
            "sample": "first %d of %d requests of the same workload, one request per thread, oracle decode (float32 build, OpenMP), %.1f s" % (n, w.B, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5 (default: the largest-batch one)")
    ap.add_argument("--scale", type=float, default=1.0, help="beam scale of configuration 5")
    ap.add_argument("--lazy", type=int, default=None, help="number of lazy layers K of the same model (default: the configuration's; 0 = plain autoregressive decoding)")
    ap.add_argument("--vanilla", action="store_true",
                    help="the vanilla autoregressive decoder of section 3.2 on the same weights (input s_{t-1} + p_t, no Fuse, every layer per beam and level)")
    ap.add_argument("--fp8", action="store_true", help="low-precision inference: FP8 (E4M3) operands for the per-beam-row products (default: bf16)")
    ap.add_argument("--value", type=int, default=0, help="append an eCPM-token step with this many value buckets to the model and run it in every call (default: none)")
    ap.add_argument("--beam", type=str, default=None, help="comma-separated beam widths per level instead of the configuration's (Dynamic Beam Width schedules)")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--graph", action="store_true",
                    help="capture the decode call in a HIP graph once and time replays (no per-kernel events: implies --no-profile)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three device-to-device copies of 1 GiB before the warm-up (a kernel of known HBM traffic for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (requests shard data-parallel with no communication; "
              "run one process per GPU to scale out). --gpus %d is not supported." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_22732_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    w = synth.workload(args.config, scale=args.scale, batch=args.batch, lazy=args.lazy, value=args.value, fp8=args.fp8, vanilla=args.vanilla)
    if args.beam:
        beam = [int(b) for b in args.beam.split(",")]
        if len(beam) != w.T or min(beam) < 1:
            print("bench.py: --beam needs %d positive widths" % w.T, file=sys.stderr)
            sys.exit(2)
        w.beam = beam
        w.name += "-beam" + "/".join(map(str, beam))
    W = synth.make_weights(w)
    lens = synth.make_lengths(w)
    dev = torch.device("cuda:0")
    td = binding.torch_dtype(w.dtype)
    ctx = torch.empty(w.B, w.S, w.d, dtype=td, device=dev)
    for r in range(w.B):  # request by request: bounded host memory
        ctx[r] = torch.from_numpy(synth.make_context_request(w, r, int(lens[r]))).to(dev, dtype=td)
    ctx_len = torch.from_numpy(lens).to(dev)
    dec = binding.decoder_for(w, W)
    ws_bytes = dec.workspace_bytes(w.B, w.S, w.beam)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    out_sid = torch.empty(w.B, w.beam[-1], w.T, dtype=torch.int32, device=dev)
    out_lp = torch.empty(w.B, w.beam[-1], dtype=torch.float32, device=dev)
    out_val = torch.empty(w.B, w.beam[-1], w.Ve, dtype=torch.float32, device=dev) if w.Ve > 0 else None

    def step():
        dec.decode_batch(ctx, ctx_len, w.beam, workspace=ws, out_sid=out_sid, out_logprob=out_lp, value=w.Ve > 0, out_value=out_val)

    if args.calibrate_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        c = torch.empty_like(a)
        for _ in range(3):
            c.copy_(a)
        torch.cuda.synchronize()
        del a, c
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        args.no_profile = True
        eager_step = step
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            eager_step()  # (the capture stream's own warm-up)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            eager_step()
        step = graph.replay
        step()
        torch.cuda.synchronize()
    binding.profile_read(reset=True)
    binding.profile_enable(not args.no_profile)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = binding.profile_read(reset=True)
    binding.profile_enable(False)

    ms_per_step = elapsed / args.steps * 1e3
    req_s = w.B * args.steps / elapsed
    flops = algorithmic_flops(w, lens)
    total_flops = sum(flops.values())

    # per-kernel rooflines from the event-timed launches; the dominant kernel (most event time) goes into "roofline"
    traffic, traffic_note = measured_traffic(w.cfg_id) if not (args.lazy is not None or args.fp8 or args.value or args.beam or args.batch or args.vanilla or args.scale != 1.0) \
        else ({}, "counter summaries exist for the default command lines only")
    kernels = {}
    for name, rec in prof.items():
        sec = rec["ms"] * 1e-3
        k = {"ms_per_step": rec["ms"] / args.steps, "launches_per_step": rec["launches"] / args.steps,
             "avg_launch_ms": rec["ms"] / rec["launches"]}
        fl = rec["flops"]
        if name.startswith("cross_attn"):
            fl *= float(np.mean(lens)) / w.S  # the library counts the padded length; the method needs the valid keys only
        if name == "gemm_bf16_ring":
            # likewise the context key/value projections of the A autoregressive layers: counted on B*S rows, needed on the valid ones
            fl -= args.steps * w.A * (w.B * w.S - float(np.sum(lens))) * 2.0 * (2 * w.d) * w.d
        if name == "context_attn_flash_bf16":
            # the lazy layers' one-pass attention: the library counts all S context rows, the kernel reads (and needs) the valid ones
            rec = dict(rec, bytes=rec["bytes"] - rec["launches"] * (w.B * w.S - float(np.sum(lens))) * w.d * 2.0)
            fl = 0.0  # priced against HBM: 4 * RQ flops per context byte pair is far below the machine balance
        if fl > 0 and name.startswith("gemm_fp8"):
            k.update(bound="mfma", achieved=fl / sec / 1e12, peak=PEAK_FP8_MFMA / 1e12, unit="TFLOP/s", frac=fl / sec / PEAK_FP8_MFMA,
                     flops_per_launch=fl / rec["launches"])
        elif fl > 0 and (name.startswith("gemm_bf16") or name.startswith("cross_attn_flash")):
            k.update(bound="mfma", achieved=fl / sec / 1e12, peak=PEAK_BF16_MFMA / 1e12, unit="TFLOP/s", frac=fl / sec / PEAK_BF16_MFMA,
                     flops_per_launch=fl / rec["launches"])
        elif fl > 0 and name.startswith("gemm"):
            k.update(bound="alu", achieved=fl / sec / 1e12, peak=PEAK_F32_VALU / 1e12, unit="TFLOP/s", frac=fl / sec / PEAK_F32_VALU,
                     flops_per_launch=fl / rec["launches"])
        elif rec["bytes"] > 0:
            k.update(bound="hbm", achieved=rec["bytes"] / sec / 1e9, peak=PEAK_HBM / 1e9, unit="GB/s", frac=rec["bytes"] / sec / PEAK_HBM,
                     bytes_per_launch=rec["bytes"] / rec["launches"])
        # the summary holds bytes per decode_batch call; per launch of this class as counted here
        k["traffic"] = traffic[name] / k["launches_per_step"] if name in traffic and k["launches_per_step"] > 0 else None
        kernels[name] = k
    roofline = None
    if prof:
        dom = max(prof, key=lambda n: prof[n]["ms"])
        k = kernels[dom]
        if "bound" in k:
            roofline = {"kernel": dom, "bound": k["bound"], "achieved": k["achieved"], "peak": k["peak"], "unit": k["unit"],
                        "frac": k["frac"], "traffic": k["traffic"], "traffic_source": traffic_note, "avg_launch_ms": k["avg_launch_ms"],
                        "share_of_step": k["ms_per_step"] / ms_per_step}

    out = {
        "metric": "requests_per_s", "value": req_s, "unit": "requests/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8" if w.fp8 else w.dtype, "data": "synthetic",
        "config": {"workload": "config %d %s: B=%d S=%d d=%d L=%d K=%d H=%d F=%d T=%d V=%s beam=%s ctx_len=%s" % (
            w.cfg_id, w.name, w.B, w.S, w.d, w.L, w.K, w.H, w.F, w.T, w.V[0], "/".join(map(str, w.beam)),
            "all %d" % w.S if w.len_min is None else "U[%d,%d]" % (w.len_min, w.S)), "batch": w.B, "beam": list(w.beam), "hip_graph": bool(args.graph)},
        "candidates_per_s": req_s * w.beam[-1], "beam_rows_per_s": req_s * sum(w.rows),
        "algorithmic_tflop_per_step": total_flops / 1e12, "whole_path_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "whole_path_frac_of_bf16_mfma_peak": total_flops / (ms_per_step * 1e-3) / PEAK_BF16_MFMA,
        "workspace_gib": ws_bytes / 2**30,
        "roofline": roofline, "kernels": kernels,
    }
    if not args.no_cpu and w.Ve == 0 and not w.fp8 and not args.graph:  # (the baseline is the oracle as it stands, in its default mode)  # the oracle's batch decode ends at the last SID level
        out["cpu_baseline"] = cpu_baseline(w, W, lens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
