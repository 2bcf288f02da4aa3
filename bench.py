#!/usr/bin/env python3
"""Benchmark of the DiLoCo outer-synchronisation path on one MI355X.

One "step" is one pass of the whole hot path over the full 10B-shaped parameter set
(42 layers, hidden 4096, FFN 14336, GQA 32/8, vocabulary 128256: 10,211,381,248 fp32 elements in
381 tensors) with W = 4 coded peer contributions:
    diloco_pseudograd_quantize (fp32 theta_local)     17 B / element
    int8_reduce_chunk          (W = 4, recomputing)    9 B / element
    outer_nesterov_step        (coded delta)          17 B / element
All inputs are synthetic, seeded, and already resident in HBM when timing starts.  `value` is the
algorithmic bytes of the K timed steps divided by their wall time.  The roofline object reports
the kernel that takes the most time, timed with HIP events recorded by the library around it.
The CPU oracle is timed on a bounded sample (one decoder layer's tensors) as a baseline only.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "pseudo-grad quantise+int8 reduce+outer step: GB/s & % HBM peak, 10B"
HBM_PEAK_GBS = 8000.0
LR, BETA = 0.7, 0.9

# algorithmic bytes per element of each streaming kernel
KERNEL_BYTES = {
    "stage1_stats(pseudograd fp32)": 8,     # reads theta_outer, theta_local
    "stage1_quant(pseudograd fp32)": 9,     # reads both again, writes 1 code
    "stage2_stats(reduce W=4)": 4,          # reads 4 code streams
    "stage2_quant(reduce W=4)": 5,          # reads 4 code streams, writes 1 code
    "stage3_outer(coded)": 17,              # reads code, theta, momentum; writes theta, momentum
}
STAGE_BYTES = {"stage1": 17, "stage2": 9, "stage3": 17}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration (0, 1 or 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise copy of 2^28 fp32 (1 GiB read, 1 GiB written) so that "
                         "profiler byte counters can be scaled against a kernel of known traffic")
    ap.add_argument("--cpu-layers", type=int, default=4,
                    help="decoder layers in the CPU-oracle sample (218,112,000 elements each)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (peers are int8 buffers in local HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2412_01152_amd import binding as B
    from paper_2412_01152_amd import synth

    B.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = args.config
    sizes = synth.config_segment_sizes(cfg)
    off = synth.offsets_from_sizes(sizes)
    N, T = off[-1], len(sizes)
    W = 4 if cfg == 2 else synth.config_peers(cfg)
    kind = synth.config_delta_kind(cfg)
    log(f"[bench] config {cfg}: N={N} T={T} W={W}; allocating")

    t0 = time.time()
    theta = torch.empty(N, dtype=torch.float32, device=dev)
    local = torch.empty(N, dtype=torch.float32, device=dev)
    mom = torch.zeros(N, dtype=torch.float32, device=dev)
    peer_codes = [torch.empty(N, dtype=torch.uint8, device=dev) for _ in range(W)]
    peer_luts = [torch.empty((T, 256), dtype=torch.float32, device=dev) for _ in range(W)]
    codes1 = torch.empty(N, dtype=torch.uint8, device=dev)
    lut1 = torch.empty((T, 256), dtype=torch.float32, device=dev)
    codes2 = torch.empty(N, dtype=torch.uint8, device=dev)
    lut2 = torch.empty((T, 256), dtype=torch.float32, device=dev)
    qp = B.new_qparams(T, dev)
    ws = B.new_workspace(T, dev)
    synth.fill_theta_outer(theta)
    # peers 1..W-1 first (their theta_local passes through the one scratch buffer), peer 0 last so
    # that `local` ends up holding this worker's weights
    for p in list(range(1, W)) + [0]:
        synth.fill_theta_local(local, theta, p, kind)
        B.pseudograd_quantize(theta, local, off, codes_out=peer_codes[p], lut_out=peer_luts[p],
                              qparams_out=qp, workspace=ws)
        torch.cuda.synchronize()
        log(f"[bench] peer {p} ready ({time.time() - t0:.1f}s)")

    # ---- CPU oracle on a bounded sample, before theta is modified (baseline only) -------------
    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = cpu_oracle_baseline(np, torch, synth, theta, local, off, sizes, cfg, W, args.cpu_layers)

    def step(events=None):
        if events is not None:
            B.profile_passes(events[0])
        B.pseudograd_quantize(theta, local, off, codes_out=codes1, lut_out=lut1, qparams_out=qp, workspace=ws)
        if events is not None:
            B.profile_passes(events[1])
        B.reduce_chunk(peer_codes, peer_luts, off, W, codes_out=codes2, lut_out=lut2, qparams_out=qp,
                       workspace=ws)
        if events is not None:
            B.profile_passes(events[2])
        B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=off, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        n_cal = 1 << 28                      # 1 GiB read + 1 GiB written, one launch
        src = local[:n_cal]
        dst = torch.empty(n_cal, dtype=torch.float32, device=dev)
        for _ in range(3):
            torch.neg(src, out=dst)          # the only negation kernel in the run: easy to find
        torch.cuda.synchronize()
        del dst

    # HIP events: created by torch (one dummy record makes the handle exist), recorded by the library
    def make_events():
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for e in evs:
            e.record()
        return evs

    all_events = [[make_events() for _ in range(3)] for _ in range(args.steps)]
    handles = [[[e.cuda_event for e in stage] for stage in st] for st in all_events]
    torch.cuda.synchronize()

    t_start = time.perf_counter()
    for k in range(args.steps):
        step(handles[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    B.profile_passes(None)

    ms_per_step = elapsed * 1e3 / args.steps
    step_bytes = sum(STAGE_BYTES.values()) * N
    value = step_bytes / (elapsed / args.steps) / 1e9

    KERNEL_BYTES.pop("stage2_stats(reduce W=4)")
    KERNEL_BYTES.pop("stage2_quant(reduce W=4)")
    kb = dict(list(KERNEL_BYTES.items())[:2])
    kb[f"stage2_stats(reduce W={W})"] = W
    kb[f"stage2_quant(reduce W={W})"] = W + 1
    kb["stage3_outer(coded)"] = 17
    KERNEL_BYTES.clear()
    KERNEL_BYTES.update(kb)
    STAGE_BYTES["stage2"] = 2 * W + 1
    step_bytes = sum(STAGE_BYTES.values()) * N
    value = step_bytes / (elapsed / args.steps) / 1e9
    names = list(KERNEL_BYTES)
    dur = {n: [] for n in names}
    stage_ms = {"stage1": [], "stage2": [], "stage3": []}
    for st in all_events:
        s1, s2, s3 = st
        dur[names[0]].append(s1[0].elapsed_time(s1[1]))
        dur[names[1]].append(s1[2].elapsed_time(s1[3]))
        dur[names[2]].append(s2[0].elapsed_time(s2[1]))
        dur[names[3]].append(s2[2].elapsed_time(s2[3]))
        dur[names[4]].append(s3[0].elapsed_time(s3[1]))
        stage_ms["stage1"].append(s1[0].elapsed_time(s1[3]))
        stage_ms["stage2"].append(s2[0].elapsed_time(s2[3]))
        stage_ms["stage3"].append(s3[0].elapsed_time(s3[1]))
    for k in range(args.steps):
        log("[bench] step %2d: " % k + "  ".join(f"{dur[n][k]:7.3f}" for n in names) + "  ms")
    kernels = {}
    for n in names:
        avg = float(np.mean(dur[n]))
        kernels[n] = {"avg_ms": round(avg, 4), "GB/s": round(KERNEL_BYTES[n] * N / (avg * 1e-3) / 1e9, 1),
                      "frac_of_peak": round(KERNEL_BYTES[n] * N / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        log(f"[bench] {n:34s} avg {avg:8.3f} ms  {kernels[n]['GB/s']:8.1f} GB/s  "
            f"{100 * kernels[n]['frac_of_peak']:.1f}% of peak")
    stages = {}
    for s, v in stage_ms.items():
        avg = float(np.mean(v))
        stages[s] = {"avg_ms": round(avg, 4), "GB/s": round(STAGE_BYTES[s] * N / (avg * 1e-3) / 1e9, 1)}
        log(f"[bench] {s}: {avg:.3f} ms  {stages[s]['GB/s']:.1f} GB/s ({100 * stages[s]['GB/s'] / HBM_PEAK_GBS:.1f}%)")
    dominant = max(names, key=lambda n: kernels[n]["avg_ms"])
    achieved = kernels[dominant]["GB/s"]
    traffic = measured_traffic_bytes(dominant) if cfg == 2 else None
    result = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config{cfg}: 10B-shaped parameter set, {N} fp32 elements in {T} tensors, "
                               f"W={W} coded peers, delta={kind}, lr={LR}, momentum={BETA}"
                   if cfg == 2 else f"config{cfg}: N={N} T={T} W={W} delta={kind}",
                   "elements": N, "segments": T, "peers": W, "bytes_per_element_per_step": sum(STAGE_BYTES.values())},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "algorithmic_bytes_per_launch": KERNEL_BYTES[dominant] * N},
        "kernels": kernels, "stages": stages,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(result), flush=True)


def measured_traffic_bytes(kernel_name):
    """HBM bytes per launch of `kernel_name` from the committed rocprofv3 counter summary
    (profiles/hbm_traffic_config2.txt: FETCH_SIZE and WRITE_SIZE in KiB per dispatch and the factors
    that a plain copy of known size gave for the same counters).  None if the file or the row is
    missing: the figure is measured offline, never estimated here."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_config2.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("#") or "|" not in line:
            continue
        cols = [c.strip() for c in line.split("|")]
        if cols[0] == kernel_name and len(cols) >= 5:
            fetch_kib, write_kib, fetch_factor, write_factor = (float(c) for c in cols[1:5])
            return round((fetch_kib / fetch_factor + write_kib / write_factor) * 1024.0)
    return None


def cpu_oracle_baseline(np, torch, synth, theta, local, off, sizes, cfg, W, layers):
    """Times the oracle's three stages on the first decoder layers of the same workload
    (9 tensors, 218,112,000 elements per layer), copied down from the device."""
    import oracle
    from oracle import build as obuild
    obuild.build(force=False)
    if cfg == 2:
        first, last = 1, 1 + 9 * max(1, layers)      # tensor 0 is the embedding
    else:
        first, last = 0, min(len(sizes), 9)
    a, b = off[first], off[last]
    sample_off = [o - a for o in off[first:last + 1]]
    n = b - a
    th = theta[a:b].cpu().numpy()
    lo = local[a:b].cpu().numpy()
    # contributions of the other peers: the oracle makes its own codes from freshly generated
    # theta_local slices (setup, untimed); nothing the GPU library produced is used
    pcs, pls = [], []
    scratch = torch.empty(n, dtype=torch.float32, device=theta.device)
    threads = oracle.num_threads()
    t_setup = time.perf_counter()
    for p in range(1, W):
        synth.fill_theta_local(scratch, theta[a:b], p, synth.config_delta_kind(cfg), seed=synth.BASE_SEED + 1)
        c, l, _, _ = oracle.pseudograd_quantize(th, scratch.cpu().numpy(), sample_off)
        pcs.append(c)
        pls.append(l)
    del scratch
    log(f"[bench] cpu baseline: sample of {n} elements, {threads} threads, setup {time.perf_counter() - t_setup:.1f}s")
    t1 = time.perf_counter()
    c0, l0, _, _ = oracle.pseudograd_quantize(th, lo, sample_off)
    t2 = time.perf_counter()
    acc, c2, l2, _ = oracle.reduce([c0] + pcs, [l0] + pls, sample_off, W)
    t3 = time.perf_counter()
    m = np.zeros(n, dtype=np.float32)
    th2 = th.copy()
    t4 = time.perf_counter()
    oracle.outer_step(th2, m, LR, BETA, delta_codes=c2, delta_luts=l2, seg_offsets=sample_off)
    t5 = time.perf_counter()
    secs = (t2 - t1) + (t3 - t2) + (t5 - t4)
    bpe = 17 + 2 * W + 1 + 17
    gbs = bpe * n / secs / 1e9
    log(f"[bench] cpu baseline: stage1 {t2 - t1:.2f}s stage2 {t3 - t2:.2f}s stage3 {t5 - t4:.2f}s -> {gbs:.2f} GB/s")
    return {"value": round(gbs, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"first {max(1, layers) if cfg == 2 else 1} decoder layer(s) of the same workload "
                      f"({n} elements in {len(sample_off) - 1} tensors, W={W}), same {bpe} B/element "
                      f"accounting; wall seconds per stage: {t2 - t1:.2f}/{t3 - t2:.2f}/{t5 - t4:.2f} "
                      f"(about {secs * threads:.0f} core-seconds)",
            "seconds": round(secs, 3)}


if __name__ == "__main__":
    main()
