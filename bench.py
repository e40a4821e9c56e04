#!/usr/bin/env python3
"""Benchmark of the DGC hot path on one MI355X.

A step is one pass of the whole path for one worker of an N-worker job on a
paper-shaped gradient set: dgc_compress of the worker's gradient (clipping norm
when the configuration clips, sampled thresholds, streaming update + mask,
emit = extraction + residual + factor masking), then the dense aggregate of N
payloads (the fresh one and N - 1 from other seeded, correlated streams),
merged by element range on chip, workers in order, no float atomics:
dgc_decompress_replace_regions writes it in place of the previous step's
aggregate in one launch (--receive accumulate_clear: the same result from
dgc_decompress_accumulate_regions into a zero buffer followed by
dgc_dense_clear_regions).  Four workers' states
(g, u, v) rotate so that no step finds its operands in the 256 MB last-level
cache.  Inputs are generated on the host once, seeded, and are resident in HBM
before the timed region.

The default workload is the one the headline metric is quoted on: the
ResNet-50-shaped set (25,557,032 fp32 elements in 161 tensors, density 0.1 %,
momentum 0.9, no clipping, N = 16).  --workload lstm | speech time the two
larger sets for the record; --workload speech_warmup times the speech set's
first 20 iterations under the warm-up schedule of densities (25 %, 6.25 %,
1.5625 %, 0.4 %, then 0.1 %), where a step is one iteration at its density.

Prints one JSON line: whole-job throughput in dense gradient elements per
second, the roofline of the dominant kernel (the streaming pass, 20 bytes per
element) from HIP events recorded on the launch stream, and the CPU oracle timed
on a bounded sample of the same workload.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X published peak
BYTES_PER_ELEMENT = 20           # streaming pass: read g, u, v; write u, v (fp32)

WORKLOADS = {
    # name: (set constructor, config, N payloads accumulated, description)
    "resnet50": ("resnet50_set", dict(momentum=0.9, density=0.001, seed=1, num_workers=16), 16,
                 "ResNet-50-shaped gradient set, 161 fp32 tensors, 25,557,032 elements, density 0.001, "
                 "m=0.9, no clipping"),
    "lstm": ("lstm_lm_set", dict(momentum=0.9, density=0.001, seed=1, num_workers=4, clip_threshold=0.25), 4,
             "2-layer LSTM-1500 language-model-shaped set, 11 fp32 tensors, 66,034,000 elements, density 0.001, "
             "m=0.9, clipping 0.25 with N=4"),
    "speech": ("speech_set", dict(momentum=0.9, density=0.001, seed=1, num_workers=8), 8,
               "speech-model-shaped set (7 bidirectional GRU-1200 layers), 62 fp32 tensors, 122,153,069 "
               "elements, density 0.001 (steady state of the warm-up schedule), m=0.9, no clipping"),
    "speech_literal": ("speech_literal_set", dict(momentum=0.9, density=0.001, seed=1, num_workers=8), 8,
                       "speech set read literally from the benchmark's shapes (5 bidirectional GRU-1024 layers), 46 fp32 "
                       "tensors, 90,192,061 elements, density 0.001, m=0.9, no clipping"),
}

# HBM traffic of one streaming-kernel launch on the default workload from rocprofv3 --pmc
# (FETCH_SIZE and WRITE_SIZE runs, each scaled by what the same counter reads for a
# device copy of n floats): 308.3 MB read + 207.9 MB written.  The counters cannot be
# read from inside this process; profiles/stream_kernel_resnet50_hbm_traffic.txt holds
# the run this number comes from.
MEASURED_TRAFFIC_BYTES = {"resnet50": 516176898}


WARMUP_DESCRIPTION = ("speech-model-shaped set, 62 fp32 tensors, 122,153,069 elements, m=0.9, no clipping, N=8, "
                      "iterations 0..19 of the warm-up schedule (densities 0.25, 0.0625, 0.015625, 0.004, then 0.001)")


def run_warmup_schedule(args):
    """The speech set's first 20 iterations: dgc_set_iteration_density, dgc_compress of one
    worker, accumulate of 8 payloads of that density, sparse clear.  --steps counts iterations
    (rounded up to whole passes of 20), --warmup passes nothing but the first pass."""
    import torch
    from paper_1712_01887_amd import binding as B
    from paper_1712_01887_amd import synthetic as S

    dev, N, seed, iters = "cuda", 8, 2025, 20
    gs = S.speech_set()
    n = gs.numel
    scales = S.tensor_scales(gs, seed)
    dgc = B.Dgc(B.make_config(momentum=0.9, density=0.001, seed=1, num_workers=N), gs.offsets, warmup_workspace=True)
    dgc.set_layout(dgc.dgc_recommended_payload_layout(0.25))
    shared = S.gradient(gs, seed, 999, 0, scales)
    g_pool = [torch.from_numpy(S.correlated_gradient(gs, seed, r, 0, shared, scales=scales)).to(dev) for r in range(2)]
    u = torch.zeros(n, device=dev)
    v = torch.zeros(n, device=dev)
    dense = torch.zeros(n, device=dev)
    fresh = [dgc.alloc_payload(dev) for _ in range(2)]
    stage_of = [min(i, 4) for i in range(iters)]
    others = []                                   # per stage: N - 1 payloads of that density
    gw = [torch.from_numpy(S.correlated_gradient(gs, seed, 100 + w, 0, shared, scales=scales)).to(dev)
          for w in range(N - 1)]
    for stage in range(5):
        dgc.dgc_set_iteration_density(stage)
        pls = []
        for w in range(N - 1):
            u.zero_()
            v.zero_()
            pl = dgc.alloc_payload(dev)
            dgc.dgc_compress(gw[w], u, v, pl[0], pl[1], pl[2], pl[3], 0)
            pls.append(pl)
        others.append(pls)
    torch.cuda.synchronize()
    del gw
    u.zero_()
    v.zero_()
    replace = args.receive == "replace"
    plists = {}
    for stage in range(5):
        o = others[stage]
        for q in range(2):
            f = fresh[q]
            plists[(stage, q)] = B.PayloadList([f[0]] + [x[0] for x in o], [f[1]] + [x[1] for x in o],
                                               [f[2]] + [x[2] for x in o])
    prepared = []                                  # iteration i: gradient and payload buffer i & 1
    for i in range(iters):
        before = (i - 1) % iters
        prepared.append(B.PreparedStep(dgc, g_pool[i & 1], u, v, fresh[i & 1], plists[(stage_of[i], i & 1)], dense,
                                       previous=plists[(stage_of[before], before & 1)]))
    for p in prepared:
        p.receive = p.replace if replace else p.accumulate_and_clear

    def one_pass(events=None):
        for i in range(iters):
            dgc.dgc_set_iteration_density(i)
            p = prepared[i]
            if events is not None:
                events[i][0].record()
            p.compress(i)
            if events is not None:
                events[i][1].record()
            p.receive()
            if events is not None:
                events[i][2].record()

    passes = max(1, (args.steps + iters - 1) // iters)
    one_pass()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(passes):
        one_pass()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / (passes * iters) * 1e3
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(iters)]
    one_pass(ev)
    torch.cuda.synchronize()
    per_iteration = [{"iteration": i, "density": [0.25, 0.0625, 0.015625, 0.004, 0.001][stage_of[i]],
                      "compress_us": round(ev[i][0].elapsed_time(ev[i][1]) * 1e3, 1),
                      "replace_us" if replace else "accumulate_and_clear_us":
                          round(ev[i][1].elapsed_time(ev[i][2]) * 1e3, 1)}
                     for i in range(6)]
    out = {
        "metric": "dense gradient elements/s for compress+decompress",
        "value": n / (ms_per_step * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": passes * iters,
        "warmup": iters,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": WARMUP_DESCRIPTION + "; step = one iteration: compress one worker + " +
                               ("aggregate of 8 payloads written in place of the previous one" if replace else
                                "accumulate 8 payloads + sparse clear") + "; workspace with staging arrays",
                   "elements": n, "tensors": len(gs.sizes), "workers_accumulated": N},
        "ms_per_20_iterations": round(ms_per_step * iters, 3),
        "first_iterations": per_iteration,
        "roofline": None,
    }
    print(json.dumps(out))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", choices=sorted(WORKLOADS) + ["speech_warmup"], default="resnet50")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sample-block", type=int, default=None, help="override dgc_config.sample_block")
    ap.add_argument("--refine-alpha", type=float, default=None,
                    help="switch the Section 5 re-threshold on (dgc_config.refine_alpha); off by default")
    ap.add_argument("--sorted", action="store_true",
                    help="emit every tensor's pairs in ascending index order (DGC_FLAG_SORTED_OUTPUT)")
    ap.add_argument("--receive", choices=["replace", "accumulate_clear", "sgd_apply"], default="replace",
                    help="receive side of a step: dgc_decompress_accumulate_regions + dgc_dense_clear_regions, or "
                         "dgc_decompress_replace_regions (the aggregate written in place of the previous one), or "
                         "dgc_sparse_sgd_apply_regions (no aggregate: the dense buffer plays the parameters, lr 1e-3)")
    ap.add_argument("--rotate", type=int, default=4,
                    help="independent (g, u, v) sets the steps rotate through; 4 keeps every step's operands out of the "
                         "last-level cache (the default and the headline), 1 shows the cache-resident case")
    ap.add_argument("--profile-only", action="store_true",
                    help="skip the CPU baseline and the event-instrumented pass (for rocprofv3 runs)")
    return ap.parse_args()


def make_gradient(S, name, gs, seed, worker, shared, scales):
    g = S.correlated_gradient(gs, seed, worker, 0, shared, scales=scales)
    if name == "lstm":      # the embedding gradient touches 700 seeded rows only
        S.zero_inactive_embedding_rows(g, seed, worker, 0)
    return g


def cpu_baseline(name, gs, cfg_kw, n_workers, scales, seed):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    from oracle import dgc_oracle as O
    from paper_1712_01887_amd import synthetic as S

    cfg = O.OracleConfig(**{k: v for k, v in cfg_kw.items() if k != "flags"})   # its payload is always ascending
    u = np.zeros(gs.numel, np.float32)
    v = np.zeros(gs.numel, np.float32)
    grads = [S.gradient(gs, seed, 0, it, scales) for it in range(4)]
    O.compress(grads[0], u, v, gs.offsets, cfg, 0)                     # untimed: first touch of the buffers
    t_comp = 0.0
    iters = 0
    res = None
    while iters < 3 or (t_comp < 10.0 and iters < 400):       # about ten seconds of CPU work
        t0 = time.perf_counter()
        res = O.compress(grads[(iters + 1) % 4], u, v, gs.offsets, cfg, iters + 1)
        t_comp += time.perf_counter() - t0
        iters += 1
    payload = O.flatten_payload(res)
    dense = np.zeros(gs.numel, np.float32)
    reps = 5
    t0 = time.perf_counter()
    for _ in range(reps):
        O.decompress_accumulate(dense, [payload] * n_workers)
        dense[payload[0]] = 0.0                                        # sparse clear, as the GPU step does
    t_acc = (time.perf_counter() - t0) / reps
    per_step = t_comp / iters + t_acc
    return {
        "value": gs.numel / per_step,
        "unit": "elements/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"{iters} compress iterations of the full {name} set "
                  f"({t_comp / iters * 1e3:.0f} ms each) + accumulate/clear of {n_workers} payloads "
                  f"({t_acc * 1e3:.1f} ms), numpy, single thread",
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no collective and this build runs on a "
              "single MI355X; use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1712_01887_amd import binding as B
    from paper_1712_01887_amd import synthetic as S

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    if args.workload == "speech_warmup":
        run_warmup_schedule(args)
        return
    dev = "cuda"
    ROTATE = max(1, args.rotate)
    set_name, cfg_kw, n_workers, description = WORKLOADS[args.workload]
    cfg_kw = dict(cfg_kw)
    gs = getattr(S, set_name)()
    n = gs.numel
    seed = 2025
    scales = S.tensor_scales(gs, seed)
    if args.sample_block:
        cfg_kw["sample_block"] = args.sample_block
    if args.refine_alpha:
        cfg_kw["refine_alpha"] = args.refine_alpha
        description += f", re-threshold when more than {args.refine_alpha:g} k pass"
    if args.sorted:
        cfg_kw["flags"] = cfg_kw.get("flags", 0) | B.DGC_FLAG_SORTED_OUTPUT
        description += ", sorted payload"
    clip = cfg_kw.get("clip_threshold", 0.0) > 0.0

    dgc = B.Dgc(B.make_config(**cfg_kw), gs.offsets)
    layout = dgc.dgc_recommended_payload_layout(cfg_kw["density"])
    dgc.set_layout(layout)

    # ---- inputs, resident in HBM ----------------------------------------------
    shared = S.gradient(gs, seed, 999, 0, scales)
    g_pool = [torch.from_numpy(make_gradient(S, args.workload, gs, seed, r, shared, scales)).to(dev)
              for r in range(ROTATE)]
    u = [torch.zeros(n, device=dev) for _ in range(ROTATE)]
    v = [torch.zeros(n, device=dev) for _ in range(ROTATE)]
    fresh = [dgc.alloc_payload(dev) for _ in range(ROTATE)]
    # N - 1 payloads of other workers: one compress each of a correlated stream
    others = []
    tu = torch.zeros(n, device=dev)
    tv = torch.zeros(n, device=dev)
    for w in range(n_workers - 1):
        gw = torch.from_numpy(make_gradient(S, args.workload, gs, seed, 100 + w, shared, scales)).to(dev)
        tu.zero_()
        tv.zero_()
        pl = dgc.alloc_payload(dev)
        dgc.dgc_compress(gw, tu, tv, pl[0], pl[1], pl[2], pl[3], 0)
        others.append(pl)
    torch.cuda.synchronize()
    del tu, tv, gw
    dense = torch.zeros(n, device=dev)

    # every argument marshalled once: worker r with gradient slot q
    replace = args.receive == "replace"
    if replace and ROTATE < 2:
        print("--receive replace needs --rotate >= 2: the previous step's payload must stay intact", file=sys.stderr)
        sys.exit(2)
    prepared = {}
    plists = [B.PayloadList([f[0]] + [o[0] for o in others], [f[1]] + [o[1] for o in others],
                            [f[2]] + [o[2] for o in others]) for f in fresh]
    for r in range(ROTATE):
        for q in range(ROTATE):
            prepared[(r, q)] = B.PreparedStep(dgc, g_pool[q], u[r], v[r], fresh[r], plists[r], dense,
                                              previous=plists[(r - 1) % ROTATE])
    for p in prepared.values():
        p.receive = {"replace": p.replace, "accumulate_clear": p.accumulate_and_clear,
                     "sgd_apply": p.sgd_apply}[args.receive]

    def step(i):
        r = i % ROTATE
        it = i // ROTATE
        p = prepared[(r, (r + it) % ROTATE)]
        p.compress(it)
        p.receive()

    # ---- warm-up, then the timed region -------------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    if args.profile_only:
        # a plain device copy of known size (n floats in, n floats out) for scaling the
        # FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc runs
        for _ in range(3):
            dense.copy_(g_pool[0])
        dense.zero_()
        for k in range(args.steps):               # the bare streaming kernel, for its duration in the same trace
            r = k % ROTATE
            B.dgc_profile_stream_ceiling(g_pool[(r + k // ROTATE) % ROTATE], u[r], v[r])
        torch.cuda.synchronize()

    # ---- the same steps again with HIP events on the launch stream ----------------------
    roofline = None
    breakdown = {}
    if not args.profile_only:
        dgc.dgc_profile_enable(args.steps)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        base = args.warmup + args.steps
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for k in range(args.steps):
            i = base + k
            r = i % ROTATE
            it = i // ROTATE
            p = prepared[(r, (r + it) % ROTATE)]
            ev[k][0].record()
            p.compress(it)
            ev[k][1].record()
            p.receive()
            ev[k][2].record()
        torch.cuda.synchronize()
        profiled_ms = (time.perf_counter() - t1) / args.steps * 1e3
        calls, norm_ms, select_ms, stream_ms, emit_ms = dgc.dgc_profile_collect()
        dgc.dgc_profile_disable()
        stream_avg_ms = stream_ms / calls
        achieved = BYTES_PER_ELEMENT * n / (stream_avg_ms * 1e-3) / 1e9
        roofline = {
            "bound": "hbm",
            "kernel": "stream_kernel",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
            "algorithmic_bytes": BYTES_PER_ELEMENT * n,
            "avg_kernel_us": round(stream_avg_ms * 1e3, 2),
        }
        # the box's own ceiling for this traffic: the bare three-read / two-write kernel on the same
        # rotating buffers, timed the same way (u and v are not needed any more)
        cev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        for k in range(args.warmup + args.steps):
            r = k % ROTATE
            if k >= args.warmup:
                cev[k - args.warmup][0].record()
            B.dgc_profile_stream_ceiling(g_pool[(r + k // ROTATE) % ROTATE], u[r], v[r])
            if k >= args.warmup:
                cev[k - args.warmup][1].record()
        torch.cuda.synchronize()
        ceil_ms = sum(e[0].elapsed_time(e[1]) for e in cev) / args.steps
        ceiling = BYTES_PER_ELEMENT * (n // 1024 * 1024) / (ceil_ms * 1e-3) / 1e9
        roofline["practical_ceiling"] = {
            "kernel": "ceiling_kernel (3 arrays read, 2 written, non-temporal, same tiling, no table, no mask)",
            "achieved": round(ceiling, 1), "unit": "GB/s", "avg_kernel_us": round(ceil_ms * 1e3, 2),
            "stream_kernel_frac_of_it": round(achieved / ceiling, 4)}
        comp = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
        acc = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
        per_step = sorted(e[0].elapsed_time(e[2]) for e in ev)
        breakdown = {
            "step_us_median_by_events": round(per_step[len(per_step) // 2] * 1e3, 2),
            "step_us_best_by_events": round(per_step[0] * 1e3, 2),
            "compress_us": round(comp * 1e3, 2),
            "norm_kernel_us": round(norm_ms / calls * 1e3, 2) if clip else None,
            "select_kernel_us": round(select_ms / calls * 1e3, 2),
            "stream_kernel_us": round(stream_avg_ms * 1e3, 2),
            "emit_kernel_us": round(emit_ms / calls * 1e3, 2),
            {"replace": "replace_us", "accumulate_clear": "accumulate_and_clear_us",
             "sgd_apply": "sgd_apply_us"}[args.receive]: round(acc * 1e3, 2),
            "ms_per_step_with_events": round(profiled_ms, 5),
        }
        if clip:
            nb = 4 * n / (norm_ms / calls * 1e-3) / 1e9
            breakdown["norm_kernel_GBps"] = round(nb, 1)

    counts = max(1, int(fresh[0][2].sum().item()))   # (payload counters: untouched by the ceiling probe)
    step_bytes = (BYTES_PER_ELEMENT + (4 if clip else 0)) * n
    out = {
        "metric": "dense gradient elements/s for compress+decompress",
        "value": n / (ms_per_step * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": description + (f"; step = compress one worker + aggregate of {n_workers} payloads written in "
                                       "place of the previous one" if replace else
                                       f"; step = compress one worker + sparse SGD apply of {n_workers} payloads"
                                       if args.receive == "sgd_apply" else
                                       f"; step = compress one worker + accumulate {n_workers} payloads + sparse clear"),
            "elements": n,
            "tensors": len(gs.sizes),
            "workers_accumulated": n_workers,
            "rotating_states": ROTATE,
            "pairs_per_payload": counts,
        },
        "algorithmic_GBps_whole_step": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "compression_ratio": {"ours_8B_pairs": round(4.0 * n / (8 * counts), 1),
                              "ours_6B_entries": round(4.0 * n / (6 * counts), 1),
                              "paper_resnet50": 277, "paper_range": "270-600"},
        "breakdown": breakdown,
        "roofline": roofline,
    }
    if not (args.no_cpu_baseline or args.profile_only):
        out["cpu_baseline"] = cpu_baseline(args.workload, gs, cfg_kw, n_workers, scales, seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
