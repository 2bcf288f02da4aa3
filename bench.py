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
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration: 2 (default, the graded workload); 0 and 1 are the small cases; "
                         "3 times the reduce step alone at W = 14")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise copy of 2^28 fp32 (1 GiB read, 1 GiB written) so that "
                         "profiler byte counters can be scaled against a kernel of known traffic")
    ap.add_argument("--extras", action="store_true",
                    help="after the timed steps also time the other variants of the three calls on the same "
                         "resident data (bf16 theta_local, stored accumulation, fp32 delta, hand-back)")
    ap.add_argument("--no-also", action="store_true",
                    help="config 2: only the graded step, without the other full-size shapes that the default run "
                         "appends under \"also\" (profiling runs)")
    ap.add_argument("--aligned-chunks", action="store_true",
                    help="config 4 only: round the ring chunk up to a multiple of 1024 elements")
    ap.add_argument("--overlap", action="store_true",
                    help="config 4 only: the 13 coded contributions of each chunk arrive from pinned host memory on "
                         "a copy stream while the previous chunk is reduced; reports the reduce time with and "
                         "without the concurrent transfer")
    ap.add_argument("--study", choices=["ring", "quantiser"], default=None,
                    help="quantiser: error of the 8-bit code for other clipping widths, the midpoint codebook and "
                         "per-row groups, on one decoder layer; ring: error and time of the per-hop ring reduce (requantised at every hop) against the "
                         "one-shot W-way reduce, on one decoder layer (config 1's shape)")
    ap.add_argument("--compute-ceiling", action="store_true",
                    help="config 2: also time stage 2 with ONE code buffer standing in for all W contributions "
                         "(every instruction executed, a quarter of the HBM reads): the compute units' own ceiling")
    ap.add_argument("--graph", action="store_true",
                    help="configs 0-2: also record the step into a HIP graph and time its replays")
    ap.add_argument("--shard", type=int, default=1, metavar="K",
                    help="config 2: one of K equal shards of every tensor (what one GPU of a K-GPU fully sharded "
                         "node holds: the same 381 groups, a K-th of the elements), buffers spread as with --spread")
    ap.add_argument("--spread", action="store_true",
                    help="configs 0-1: carve the buffers from the arena so that every kernel's written buffers lie "
                         "about 100 GiB away from the buffers it reads (small buffers allocated side by side are "
                         "the slow case on this memory system)")
    ap.add_argument("--no-arena", action="store_true",
                    help="allocate every buffer separately instead of carving them from one arena whose "
                         "placement is chosen by timing the outer step (configs 2, 3 and 4)")
    ap.add_argument("--arena-shift", type=int, default=None, metavar="GIB",
                    help="config 2: carve the state at this shift of the arena instead of timing the outer step "
                         "on the candidates (profiling runs: keeps the probes out of the kernel statistics)")
    ap.add_argument("--cpu-layers", type=int, default=8,
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

    if args.study == "ring":
        return study_ring(args, np, torch, B, synth, dev)
    if args.study == "quantiser":
        return study_quantiser(args, np, torch, B, synth, dev)
    cfg = args.config
    if cfg == 3:
        return bench_config3(args, np, torch, B, synth, dev)
    if cfg == 4:
        return (bench_config4_overlap if args.overlap else bench_config4)(args, np, torch, B, synth, dev)
    # The graded line is configuration 2's step.  The default run then re-uses the same arena for the other
    # full-size shapes of the target table (the reduce at W = 14, the 14 ring-chunk calls with the outer step
    # behind them, stage 1 with a bf16 theta_local, one GPU's eighth of every tensor) and appends them to the
    # same JSON line under "also"; none of that is inside the timed region of the step.
    also_wanted = cfg == 2 and args.shard == 1 and not args.no_also
    result, arena = run_step_benchmark(args, np, torch, B, synth, dev, cfg, want_extras=args.extras or also_wanted)
    fracs = {k: v["frac_of_peak"] for k, v in result["kernels"].items()}
    if also_wanted:
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        result["also"] = measure_also(args, np, torch, B, synth, dev, arena)
        for name in ("config3_reduce_w14", "config4_ring_chunks"):
            for k, v in (result["also"].get(name) or {}).get("kernels", {}).items():
                fracs[f"{name}: {k}"] = v["frac_of_peak"]
    worst = min(fracs, key=fracs.get)
    result["min_kernel_frac_of_peak"] = {"kernel": worst, "frac": fracs[worst]}
    print(json.dumps(result), flush=True)


def measure_also(args, np, torch, B, synth, dev, arena):
    """The other full-size shapes, one after the other in the memory the step benchmark used."""
    def fresh_alloc():
        if arena is None:
            return lambda numel, dtype: torch.empty(numel, dtype=dtype, device=dev)
        arena.pos = 0

        def carve(numel, dtype):
            try:
                return arena.carve(numel, dtype)
            except RuntimeError:
                return torch.empty(numel, dtype=dtype, device=dev)
        return carve

    import gc
    also = {}
    steps = max(3, args.steps // 2)
    for name, fn in (("config3_reduce_w14", measure_config3), ("config4_ring_chunks", measure_config4)):
        try:
            r = fn(args, np, torch, B, synth, dev, fresh_alloc(), steps, 1)
            also[name] = {k: r[k] for k in ("value", "unit", "ms_per_step", "frac_of_hbm_peak", "steps", "kernels",
                                             "outer_step_after", "stage1_bf16_theta_local", "roofline") if k in r}
            also[name]["workload"] = r["config"]["workload"]
            also[name]["bytes_per_element"] = r["config"]["bytes_per_element_per_step"]
        except RuntimeError as e:                 # not enough free HBM (another process on the card)
            log(f"[bench] {name} skipped: {e}")
            also[name] = None
        gc.collect()
        torch.cuda.empty_cache()
    shard = {"buffers spread over the arena by role": measure_shard(args, np, torch, B, synth, dev, arena, 8, True)}
    if arena is not None:                         # hand the memory back: the next measurement allocates per buffer
        arena.buf = None
        arena.nbytes = 0
    gc.collect()
    torch.cuda.empty_cache()
    shard["one allocation per buffer"] = measure_shard(args, np, torch, B, synth, dev, None, 8, False)
    also["config2_shard_1_of_8"] = shard
    return also


def measure_shard(args, np, torch, B, synth, dev, arena, K, spread):
    """One GPU's share under the paper's hybrid scheme (Section 2.3): a K-th of every tensor of configuration 2,
    the same 381 quantisation groups; the three calls of the step, per call."""
    from paper_2412_01152_amd.arena import role_bases
    sizes = [-(-s // K) for s in synth.config_segment_sizes(2)]
    off = synth.offsets_from_sizes(sizes)
    N, T, W = off[-1], len(sizes), 4
    bases = role_bases(arena) if (spread and arena is not None and arena.nbytes >= (210 << 30)) else None
    if spread and bases is None:
        return None

    def alloc(numel, dtype, at=None):
        if bases is not None:
            return arena.carve(numel, dtype, at=at)
        return torch.empty(numel, dtype=dtype, device=dev)

    theta = alloc(N, torch.float32, at=bases["read"] if bases else None)
    local = alloc(N, torch.float32)
    peer_codes = [alloc(N, torch.uint8) for _ in range(W)]
    mom = alloc(N, torch.float32, at=bases["state"] if bases else None).zero_()
    codes1 = alloc(N, torch.uint8)
    codes2 = alloc(N, torch.uint8, at=bases["out"] if bases else None)
    peer_luts = [torch.empty((T, 256), dtype=torch.float32, device=dev) for _ in range(W)]
    lut1 = torch.empty((T, 256), dtype=torch.float32, device=dev)
    lut2 = torch.empty((T, 256), dtype=torch.float32, device=dev)
    qp, ws = B.new_qparams(T, dev), B.new_workspace(T, dev)
    synth.fill_theta_outer(theta)
    for p in list(range(1, W)) + [0]:
        synth.fill_theta_local(local, theta, p, "mixture")
        B.pseudograd_quantize(theta, local, off, codes_out=peer_codes[p], lut_out=peer_luts[p], qparams_out=qp,
                              workspace=ws)
    calls = (("stage1", 17, lambda: B.pseudograd_quantize(theta, local, off, codes_out=codes1, lut_out=lut1,
                                                          qparams_out=qp, workspace=ws)),
             ("stage2", 2 * W + 1, lambda: B.reduce_chunk(peer_codes, peer_luts, off, W, codes_out=codes2, lut_out=lut2,
                                                          qparams_out=qp, workspace=ws)),
             ("stage3", 17, lambda: B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2,
                                                 seg_offsets=off, workspace=ws)))
    out = {"elements": N}
    reps = 10
    for name, bpe, fn in calls:
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = call_record(e0.elapsed_time(e1) / reps, bpe, N)
    log(f"[bench] shard 1/{K} ({'spread' if bases else 'plain allocations'}): "
        + "  ".join(f"{k} {out[k]['ms']:.3f} ms {100 * out[k]['frac_of_peak']:.1f}%" for k in ("stage1", "stage2", "stage3")))
    return out


def run_step_benchmark(args, np, torch, B, synth, dev, cfg, want_extras):
    """One step = the three calls on one configuration's buffers; returns (result record, the arena or None)."""
    sizes = synth.config_segment_sizes(cfg)
    sharded = cfg == 2 and args.shard > 1
    if sharded:
        sizes = [-(-s // args.shard) for s in sizes]
    off = synth.offsets_from_sizes(sizes)
    N, T = off[-1], len(sizes)
    W = 4 if cfg == 2 else synth.config_peers(cfg)
    kind = synth.config_delta_kind(cfg)
    log(f"[bench] config {cfg}: N={N} T={T} W={W}; allocating")

    t0 = time.time()
    # All large buffers come out of one allocation made before anything else, in the order theta,
    # theta_local, momentum, peer codes, codes of stage 1, codes of stage 2: their physical placement
    # is then the same in every process (see paper_2412_01152_amd/arena.py), and the shift of the whole
    # group inside the arena is chosen by timing the outer step on a few candidates (setup, untimed).
    arena = None
    if cfg == 2 and not sharded and not args.no_arena:
        from paper_2412_01152_amd.arena import Arena, place_outer_state
        need = (12 + W + 2) * N + (1 << 30)
        try:
            arena = Arena(dev)
            if arena.nbytes < need:
                raise RuntimeError(f"arena of {arena.nbytes >> 30} GiB is too small")
        except RuntimeError as e:                 # e.g. another process holds part of the HBM
            log(f"[bench] no arena ({e}); falling back to one allocation per buffer")
            arena = None
            torch.cuda.empty_cache()
    if arena is not None:
        if args.arena_shift is not None:
            shift = args.arena_shift << 30
        else:
            shift = place_outer_state(arena, N, off, range(0, 41, 5), tail_bytes=(W + 2) * N, log=log)
        if shift + need > arena.nbytes:
            shift = 0
        log(f"[bench] arena of {arena.nbytes >> 30} GiB, state carved at +{shift >> 30} GiB")

    # Small configurations, on request: three groups about 100 GiB apart - what stage 1, stage 2 and
    # the outer step read (theta, theta_local, peer codes) | momentum and the stage-1 codes | the
    # stage-2 codes - so that no kernel writes near what it reads.
    spread = None
    if (sharded or (cfg in (0, 1) and args.spread)) and not args.no_arena:
        from paper_2412_01152_amd.arena import Arena, role_bases
        try:
            arena = Arena(dev)
            if arena.nbytes < (210 << 30):
                raise RuntimeError(f"arena of {arena.nbytes >> 30} GiB is too small to spread over")
            spread = role_bases(arena)
            shift = spread["read"]
            log(f"[bench] arena of {arena.nbytes >> 30} GiB, buffers spread at "
                + " / ".join(f"+{v / (1 << 30):.0f}" for v in spread.values()) + " GiB")
        except RuntimeError as e:
            log(f"[bench] no arena ({e}); one allocation per buffer")
            arena = None
            torch.cuda.empty_cache()

    def alloc(numel, dtype, at=None):
        if arena is not None:
            try:
                return arena.carve(numel, dtype, at=at)
            except RuntimeError:
                pass
        return torch.empty(numel, dtype=dtype, device=dev)

    # --extras times stage 1 with a bf16 theta_local as well: that copy of the worker's weights belongs next
    # to theta like the fp32 one (reads run fastest from the same part of the memory), and the room in
    # front of theta is free when the state was shifted far enough
    bf16_slot = None
    if arena is not None and not spread and want_extras and shift >= 2 * N + 8192:
        bf16_slot = arena.buf[shift - 2 * N - 4096:shift - 4096].view(torch.bfloat16)
    theta = alloc(N, torch.float32, at=shift if arena is not None else None)
    local = alloc(N, torch.float32)
    if spread:
        peer_codes = [alloc(N, torch.uint8) for _ in range(W)]
        mom = alloc(N, torch.float32, at=spread["state"]).zero_()
        codes1 = alloc(N, torch.uint8)
        codes2 = alloc(N, torch.uint8, at=spread["out"])
    else:
        mom = alloc(N, torch.float32).zero_()
        peer_codes = [alloc(N, torch.uint8) for _ in range(W)]
        codes1 = alloc(N, torch.uint8)
        codes2 = alloc(N, torch.uint8)
    peer_luts = [torch.empty((T, 256), dtype=torch.float32, device=dev) for _ in range(W)]
    lut1 = torch.empty((T, 256), dtype=torch.float32, device=dev)
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
        cpu_baseline = cpu_oracle_baseline(np, torch, synth, theta, local, off, sizes, cfg, W, args.cpu_layers, alloc)

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
        calibration_copy(torch, local, alloc)

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
        med = float(np.median(v))
        stages[s] = {"avg_ms": round(avg, 4), "median_ms": round(med, 4), "min_ms": round(float(np.min(v)), 4),
                     "GB/s": round(STAGE_BYTES[s] * N / (avg * 1e-3) / 1e9, 1),
                     "frac_of_peak": round(STAGE_BYTES[s] * N / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        log(f"[bench] {s}: {avg:.3f} ms  {stages[s]['GB/s']:.1f} GB/s ({100 * stages[s]['GB/s'] / HBM_PEAK_GBS:.1f}%)")
    graph = None
    if args.graph:
        # the same step recorded once from the stream and replayed: no per-launch host work between kernels
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        graph = {"ms_per_step": round(g_ms, 3), "GB/s": round(step_bytes / (g_ms * 1e-3) / 1e9, 1)}
        log(f"[bench] step replayed from a HIP graph: {g_ms:.3f} ms per step ({graph['GB/s']:.1f} GB/s); "
            f"eager launches: {ms_per_step:.3f} ms")
    copy_ref = measure_copy_kernel(torch, local, alloc)
    log(f"[bench] plain copy kernel ({copy_ref['what']}): {copy_ref['GB/s']:.1f} GB/s; "
        f"step runs at {100 * value / copy_ref['GB/s']:.1f}% of it")
    ceiling = None
    if args.compute_ceiling:
        # table look-ups, bucket arithmetic and LDS bins at full rate while HBM delivers 2 bytes per element
        # instead of 2W + 1; GB/s counts the real call's bytes
        def aliased():
            B.reduce_chunk([peer_codes[0]] * W, peer_luts, off, W, codes_out=codes2, lut_out=lut2, qparams_out=qp,
                           workspace=ws)
        aliased()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            aliased()
        e1.record()
        torch.cuda.synchronize()
        c_ms = e0.elapsed_time(e1) / 5
        ceiling = {"stage2_ms": round(c_ms, 3), "GB/s": round((2 * W + 1) * N / (c_ms * 1e-3) / 1e9, 1),
                   "what": f"int8_reduce_chunk with one code buffer passed {W} times"}
        log(f"[bench] stage 2 compute ceiling: {c_ms:.3f} ms per call ({ceiling['GB/s']:.1f} GB/s of the real call's "
            f"bytes, {100 * ceiling['GB/s'] / HBM_PEAK_GBS:.1f}% of the HBM peak)")
        B.reduce_chunk(peer_codes, peer_luts, off, W, codes_out=codes2, lut_out=lut2, qparams_out=qp, workspace=ws)
    extras = None
    if want_extras:
        extras = time_extras(torch, B, theta, local, mom, peer_codes, peer_luts, codes1, lut1, codes2, lut2, qp, ws,
                             off, N, T, W, alloc, bf16_slot)
    dominant = max(names, key=lambda n: kernels[n]["avg_ms"])
    achieved = kernels[dominant]["GB/s"]
    traffic = measured_traffic_bytes("hbm_traffic_config2.txt", dominant) if cfg == 2 and not sharded else None
    result = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config{cfg}: 10B-shaped parameter set, {N} fp32 elements in {T} tensors, "
                               f"W={W} coded peers, delta={kind}, lr={LR}, momentum={BETA}"
                   + (f"; shard 1/{args.shard} of every tensor" if sharded else "")
                   if cfg == 2 else f"config{cfg}: N={N} T={T} W={W} delta={kind}",
                   "elements": N, "segments": T, "peers": W, "bytes_per_element_per_step": sum(STAGE_BYTES.values())},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "copy_kernel": copy_ref, "frac_of_copy_kernel": round(value / copy_ref["GB/s"], 4),
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "algorithmic_bytes_per_launch": KERNEL_BYTES[dominant] * N},
        "kernels": kernels, "stages": stages, "extras": extras, "graph": graph, "stage2_compute_ceiling": ceiling,
        "cpu_baseline": cpu_baseline,
    }
    return result, arena


def study_ring(args, np, torch, B, synth, dev):
    """Section 2.2's ring, hop by hop (dequantise the incoming chunk, add the local fp32 data,
    requantise, forward; W quantisations on the way) against the one-shot reduce (every contribution
    quantised once, one requantisation).  Data: one decoder layer (9 tensors, 218,112,000 elements),
    Gaussian, mixture and Student-t pseudo-gradients, W workers.  Error = rms(dequantised result - exact average) / std of the
    exact average, exact = fp64 mean of the W fp32 pseudo-gradients (evaluation only, with torch)."""
    from paper_2412_01152_amd import ring
    sizes = synth.config_segment_sizes(1)
    off = synth.offsets_from_sizes(sizes)
    N, T = off[-1], len(sizes)
    theta = torch.empty(N, dtype=torch.float32, device=dev)
    synth.fill_theta_outer(theta)
    ws = B.new_workspace(T, dev)
    rows = []
    for kind, W in [(k, w) for k in ("normal", "mixture", "student_t3") for w in (2, 4, 8, 14)]:
        d = []
        for p in range(W):
            x = torch.empty(N, dtype=torch.float32, device=dev)
            synth.fill_theta_local(x, theta, p, kind)
            x.sub_(theta).neg_()                              # theta_outer - theta_local
            d.append(x)
        exact = torch.zeros(N, dtype=torch.float64, device=dev)
        for x in d:
            exact += x
        exact /= W
        sd = float(exact.std())

        def run(fn):
            fn(d, off, ws)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            out = fn(d, off, ws)
            e1.record()
            torch.cuda.synchronize()
            val = ring.dequantise(out[0], out[1], off, workspace=ws)
            err = float(torch.sqrt(torch.mean((val.double() - exact) ** 2))) / sd
            return err, e0.elapsed_time(e1)

        err_ring, ms_ring = run(ring.ring_reduce)
        err_one, ms_one = run(ring.one_shot_reduce)
        rows.append({"delta": kind, "W": W, "rms_error_over_std": {"ring": round(err_ring, 5), "one_shot": round(err_one, 5)},
                     "ms": {"ring": round(ms_ring, 3), "one_shot": round(ms_one, 3)}})
        log(f"[study] {kind:10s} W={W:2d}: rms error / std  ring {err_ring:.5f}  one-shot {err_one:.5f}  "
            f"({err_ring / err_one:.2f}x);  time ring {ms_ring:.2f} ms  one-shot {ms_one:.2f} ms (both include quantising "
            f"the W fp32 inputs)")
        del d, exact
    print(json.dumps({"study": "ring hop-by-hop vs one-shot reduce", "elements": N, "segments": T, "rows": rows}),
          flush=True)


def study_quantiser(args, np, torch, B, synth, dev):
    """Section 2.2 argues for its two constants in words only: clipping at 6 sigma keeps the buckets
    narrow, and a codebook of bucket averages lowers the error.  This measures both on one decoder
    layer (9 tensors, 218,112,000 elements): rms(decoded - d) / std(d) of a single quantisation, for
    clipping widths 3..10 sigma, both codebooks, three pseudo-gradient distributions, and with one
    quantisation group per matrix row instead of per tensor (plain rows, and rows whose scales are
    spread log-normally, sigma_ln = 1).  All quantisation runs in the library; the error is evaluated
    with torch."""
    from paper_2412_01152_amd import ring
    sizes = synth.config_segment_sizes(1)
    off = synth.offsets_from_sizes(sizes)
    N = off[-1]
    row_sizes = synth.layer_row_sizes()                                    # one group per matrix row
    row_off = synth.offsets_from_sizes(row_sizes)
    assert row_off[-1] == N
    theta = torch.empty(N, dtype=torch.float32, device=dev)
    synth.fill_theta_outer(theta)
    x = torch.empty(N, dtype=torch.float32, device=dev)
    ws = B.new_workspace(len(row_sizes), dev)
    rows = []

    def measure(d, offsets, c, cb):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        codes, lut, _ = B.reduce_chunk([], [], offsets, 1, local_fp32=d, workspace=ws, variant=(c, cb))
        e1.record()
        val = ring.dequantise(codes, lut, offsets, workspace=ws)
        err = float(torch.sqrt(torch.mean((val.double() - d.double()) ** 2)) / d.double().std())
        clipped = float(((codes == 0) | (codes == 255)).float().mean())
        return err, clipped, e0.elapsed_time(e1)

    for kind in ("normal", "mixture", "student_t3"):
        synth.fill_theta_local(x, theta, 0, kind)
        d = (theta - x)
        for c in (3.0, 4.0, 5.0, 6.0, 8.0, 10.0):
            for cb, cbn in ((B.CODEBOOK_MEAN, "mean"), (B.CODEBOOK_MIDPOINT, "midpoint")):
                err, clipped, ms = measure(d, off, c, cb)
                rows.append({"delta": kind, "groups": "tensor", "range_sigmas": c, "codebook": cbn,
                             "rms_error_over_std": round(err, 5), "end_bucket_fraction": round(clipped, 6)})
                log(f"[study] {kind:10s} per tensor  c={c:4.1f} {cbn:8s}: rms error / std {err:.5f}  "
                    f"end buckets {100 * clipped:.4f}%  ({ms:.2f} ms)")
        for scaled in (False, True):
            dd = d
            if scaled:
                g = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 77)
                scale = torch.exp(torch.randn(len(row_sizes), device=dev, generator=g))
                dd = d * torch.repeat_interleave(scale, torch.tensor(row_sizes, device=dev))
            for groups, offsets in (("tensor", off), ("row", row_off)):
                err, clipped, ms = measure(dd, offsets, 6.0, B.CODEBOOK_MEAN)
                wire = 1.0 + 1024.0 * (len(offsets) - 1) / N
                rows.append({"delta": kind + (" x log-normal row scales" if scaled else ""), "groups": groups,
                             "range_sigmas": 6.0, "codebook": "mean", "rms_error_over_std": round(err, 5),
                             "end_bucket_fraction": round(clipped, 6), "wire_bytes_per_element": round(wire, 4),
                             "ms": round(ms, 3)})
                log(f"[study] {kind:10s} rows scaled={scaled!s:5s} groups per {groups:6s}: rms error / std {err:.5f}  "
                    f"wire {wire:.3f} B/elem  ({ms:.2f} ms, {len(offsets) - 1} groups)")
            del dd
    print(json.dumps({"study": "quantiser variants", "elements": N, "rows": rows}), flush=True)


def calibration_copy(torch, src_buf, alloc):
    """A plain elementwise copy of known traffic (2^28 fp32: 1 GiB read + 1 GiB written per launch) for
    scaling a profiler's byte counters; torch.neg is the only negation kernel in a run, so it is easy to find."""
    n_cal = 1 << 28
    dst = alloc(n_cal, torch.float32)
    for _ in range(3):
        torch.neg(src_buf[:n_cal], out=dst)
    torch.cuda.synchronize()
    del dst


def measure_copy_kernel(torch, src_buf, alloc):
    """Bandwidth of a plain elementwise copy (read 4 B, write 4 B per element) of up to 2^30 fp32, measured
    in this process: the nominal 8 TB/s is never reached by any kernel, so the step is also
    reported as a fraction of this."""
    n = min(1 << 30, src_buf.numel())
    src = src_buf[:n]
    dst = alloc(n, torch.float32)
    best = 0.0
    for name, fn in ((f"elementwise x*2 over {n} fp32", lambda: torch.mul(src, 2.0, out=dst)),
                     (f"tensor copy of {n} fp32", lambda: dst.copy_(src))):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        torch.cuda.synchronize()
        gbs = 8 * n * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        if gbs > best:
            best, what = gbs, name
    del dst
    return {"GB/s": round(best, 1), "what": what}


def arena_alloc(args, torch, dev):
    """alloc(numel, dtype): views carved in call order from one arena (reproducible placement), or
    separate allocations with --no-arena."""
    if args.no_arena:
        return lambda numel, dtype: torch.empty(numel, dtype=dtype, device=dev)
    from paper_2412_01152_amd.arena import Arena
    try:
        arena = Arena(dev)
    except RuntimeError as e:
        log(f"[bench] no arena ({e}); falling back to one allocation per buffer")
        return lambda numel, dtype: torch.empty(numel, dtype=dtype, device=dev)
    log(f"[bench] arena of {arena.nbytes >> 30} GiB")

    def carve(numel, dtype):
        try:
            return arena.carve(numel, dtype)
        except RuntimeError:
            return torch.empty(numel, dtype=dtype, device=dev)
    return carve


def measure_config3(args, np, torch, B, synth, dev, alloc, steps, warmup):
    """Configuration 3: the reduce step alone at W = 14 heavy-tailed coded peers on the full 10B set
    (143 GB of codes resident), accumulation stored over theta_local (no room for a fourth fp32 array
    next to theta_outer, theta_local and momentum in the real layout).  Returns the result record."""
    sizes = synth.config_segment_sizes(3)
    off = synth.offsets_from_sizes(sizes)
    N, T, W = off[-1], len(sizes), 14
    log(f"[bench] config 3: N={N} T={T} W={W}; allocating {(W + 1) * N / 1e9 + 8 * N / 1e9:.0f} GB")
    t0 = time.time()
    theta = alloc(N, torch.float32)
    local = alloc(N, torch.float32)
    peer_codes = [alloc(N, torch.uint8) for _ in range(W)]
    peer_luts = [torch.empty((T, 256), dtype=torch.float32, device=dev) for _ in range(W)]
    codes2 = alloc(N, torch.uint8)
    lut2 = torch.empty((T, 256), dtype=torch.float32, device=dev)
    qp = B.new_qparams(T, dev)
    ws = B.new_workspace(T, dev)
    synth.fill_theta_outer(theta)
    for p in range(W):
        synth.fill_theta_local(local, theta, p, "student_t3")
        B.pseudograd_quantize(theta, local, off, codes_out=peer_codes[p], lut_out=peer_luts[p], qparams_out=qp,
                              workspace=ws)
    torch.cuda.synchronize()
    log(f"[bench] {W} peers ready ({time.time() - t0:.1f}s)")

    def step(events=None):
        if events is not None:
            B.profile_passes(events)
        B.reduce_chunk(peer_codes, peer_luts, off, W, acc_out=local, codes_out=codes2, lut_out=lut2,
                       qparams_out=qp, workspace=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        calibration_copy(torch, theta, alloc)
    evs = []
    for _ in range(steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for x in e:
            x.record()
        evs.append(e)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(steps):
        step([x.cuda_event for x in evs[k]])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    B.profile_passes(None)
    a_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    b_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in evs]))
    bpe = W + 9
    value = bpe * N / (elapsed / steps) / 1e9
    kernels = {f"stage2_stats(reduce W={W}, store acc)": kernel_record(a_ms, (W + 4) * N),
               "stage2_quant(stored acc)": kernel_record(b_ms, 5 * N)}
    for k, v in kernels.items():
        log(f"[bench] {k:40s} avg {v['avg_ms']:8.3f} ms  {v['GB/s']:8.1f} GB/s  {100 * v['frac_of_peak']:.1f}% of peak")
    dom = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    return {"metric": "int8 reduce W=14 (stored accumulation): GB/s & % HBM peak, 10B", "value": round(value, 1),
            "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": round(elapsed * 1e3 / steps, 3), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"config3: 10B-shaped parameter set, {N} elements in {T} tensors, W=14 coded "
                                   f"peers (Student-t nu=3 deltas), int8_reduce_chunk only", "elements": N,
                       "segments": T, "peers": W, "bytes_per_element_per_step": bpe},
            "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
            "roofline": {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["GB/s"], "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": round(kernels[dom]["GB/s"] / HBM_PEAK_GBS, 4),
                         "traffic": measured_traffic_bytes("hbm_traffic_config3_config4.txt", dom),
                         "algorithmic_bytes_per_launch": (W + 4) * N if dom.startswith("stage2_stats") else 5 * N},
            "kernels": kernels, "cpu_baseline": None}


def bench_config3(args, np, torch, B, synth, dev):
    result = measure_config3(args, np, torch, B, synth, dev, arena_alloc(args, torch, dev), args.steps, args.warmup)
    print(json.dumps(result), flush=True)


def measure_config4(args, np, torch, B, synth, dev, alloc, steps, warmup):
    """Configuration 4: ring granularity.  The 10B set is cut into 14 contiguous chunks of
    ceil(N / 14) = 729,384,375 elements (odd: every other chunk starts on a 4-byte boundary only);
    int8_reduce_chunk runs once per chunk on 13 coded contributions plus the owner's fp32 data
    (stored in place), each chunk its own quantisation group.  One step = the 14 calls; then the outer
    step from the 14 requantised chunks, and stage 1 with a bf16 theta_local on the same 14 groups."""
    N = synth.n_elements(2)
    chunk_sizes = synth.ring_chunk_sizes(N, 14)
    if args.aligned_chunks:                       # chunk rounded up to a multiple of 1024 elements
        c = -(-chunk_sizes[0] // 1024) * 1024
        chunk_sizes = [c] * 13 + [N - 13 * c]
    coff = synth.offsets_from_sizes(chunk_sizes)
    W = 13
    log(f"[bench] config 4: N={N}, 14 chunks of {chunk_sizes[0]} (last {chunk_sizes[-1]}), W={W} coded + local")
    t0 = time.time()
    theta = alloc(N, torch.float32)
    local = alloc(N, torch.float32)
    peer_codes = [alloc(N, torch.uint8) for _ in range(W)]
    peer_luts = [torch.empty((14, 256), dtype=torch.float32, device=dev) for _ in range(W)]
    codes2 = alloc(N, torch.uint8)
    lut2 = torch.empty((14, 256), dtype=torch.float32, device=dev)
    qp = B.new_qparams(14, dev)
    ws = B.new_workspace(14, dev)
    synth.fill_theta_outer(theta)
    for p in range(W):
        synth.fill_theta_local(local, theta, p, "mixture")
        B.pseudograd_quantize(theta, local, coff, codes_out=peer_codes[p], lut_out=peer_luts[p], qparams_out=qp,
                              workspace=ws)
    synth.fill_theta_local(local, theta, W, "mixture")
    local.sub_(theta).neg_()                      # the owner's own fp32 pseudo-gradient (input preparation)
    torch.cuda.synchronize()
    log(f"[bench] {W} peers ready ({time.time() - t0:.1f}s)")
    qp1 = B.new_qparams(1, dev)

    def step(events=None):
        for c in range(14):
            a, b = coff[c], coff[c + 1]
            if events is not None:
                B.profile_passes(events[c])
            B.reduce_chunk([pc[a:b] for pc in peer_codes], [pl[c:c + 1] for pl in peer_luts], [0, b - a], 14,
                           local_fp32=local[a:b], acc_out=local[a:b], codes_out=codes2[a:b],
                           lut_out=lut2[c:c + 1], qparams_out=qp1, workspace=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        calibration_copy(torch, theta, alloc)
    t_start = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    bpe = W + 13
    value = bpe * N / (elapsed / steps) / 1e9
    log(f"[bench] 14 chunk calls: {elapsed * 1e3 / steps:.3f} ms  {value:.1f} GB/s ({100 * value / HBM_PEAK_GBS:.1f}% of peak)")
    # one more step with the library's events around the two passes of every call: per-kernel durations
    evs = []
    for _ in range(14):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for x in e:
            x.record()
        evs.append(e)
    torch.cuda.synchronize()
    step([[x.cuda_event for x in e] for e in evs])
    torch.cuda.synchronize()
    B.profile_passes(None)
    a_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs[:13]]))       # the 13 full-length chunks
    b_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in evs[:13]]))
    n0 = chunk_sizes[0]
    kernels = {f"stage2_stats(reduce W={W} + fp32 local, store acc in place), one chunk": kernel_record(a_ms, (W + 8) * n0),
               "stage2_quant(stored acc), one chunk": kernel_record(b_ms, 5 * n0)}
    for k, v in kernels.items():
        log(f"[bench] {k:40s} avg {v['avg_ms']:8.3f} ms  {v['GB/s']:8.1f} GB/s  {100 * v['frac_of_peak']:.1f}% of peak")
    # then the outer step from the requantised chunks (14 quantisation groups at the odd chunk offsets)
    outer = None
    try:
        mom = alloc(N, torch.float32).zero_()
    except RuntimeError:
        mom = None
    if mom is not None:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=coff, workspace=ws)
        e0.record()
        for _ in range(max(1, steps)):
            B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=coff, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        outer = call_record(e0.elapsed_time(e1) / max(1, steps), 17, N)
        log(f"[bench] then the outer step from the 14 requantised chunks: {outer['ms']:.3f} ms  {outer['GB/s']:.1f} GB/s "
            f"({100 * outer['frac_of_peak']:.1f}% of peak)")
    # stage 1 of this configuration: bf16 theta_local, one quantisation group per ring chunk; the bf16 copy is
    # written over the first half of the consumed fp32 accumulation (right behind theta)
    local16 = local.view(torch.bfloat16)[:N]
    synth.fill_theta_local(local16, theta, 0, "mixture")
    B.pseudograd_quantize(theta, local16, coff, codes_out=codes2, lut_out=lut2, qparams_out=qp, workspace=ws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(max(1, steps)):
        B.pseudograd_quantize(theta, local16, coff, codes_out=codes2, lut_out=lut2, qparams_out=qp, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    stage1_bf16 = call_record(e0.elapsed_time(e1) / max(1, steps), 13, N)
    log(f"[bench] stage 1 with bf16 theta_local, 14 groups: {stage1_bf16['ms']:.3f} ms  {stage1_bf16['GB/s']:.1f} GB/s "
        f"({100 * stage1_bf16['frac_of_peak']:.1f}% of peak)")
    dom = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    return {"metric": "int8 reduce per ring chunk, 13 coded + fp32 local: GB/s & % HBM peak, 10B",
            "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": round(elapsed * 1e3 / steps, 3), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"config4: {N} elements as 14 ring chunks of {chunk_sizes[0]}, 13 coded peers + "
                                   f"fp32 local, divisor 14, one int8_reduce_chunk call per chunk",
                       "elements": N, "segments": 14, "peers": W, "bytes_per_element_per_step": bpe},
            "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4), "kernels": kernels, "outer_step_after": outer,
            "stage1_bf16_theta_local": stage1_bf16,
            "roofline": {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["GB/s"], "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": round(kernels[dom]["GB/s"] / HBM_PEAK_GBS, 4),
                         "traffic": measured_traffic_bytes("hbm_traffic_config3_config4.txt", dom),
                         "algorithmic_bytes_per_launch": (W + 8) * n0 if dom.startswith("stage2_stats") else 5 * n0},
            "cpu_baseline": None}


def bench_config4(args, np, torch, B, synth, dev):
    result = measure_config4(args, np, torch, B, synth, dev, arena_alloc(args, torch, dev), args.steps, args.warmup)
    print(json.dumps(result), flush=True)


def bench_config4_overlap(args, np, torch, B, synth, dev):
    """Configuration 4 with the transfer in the loop (Section 2.2: quantisation work hidden behind the
    communication).  The coded contributions of a ring chunk start in pinned host memory and are
    brought in by host-to-device copies on a second stream, double buffered, while the previous chunk
    is reduced on the compute stream.  All 14 chunks reuse one chunk's worth of host data (9.5 GB
    pinned): the values do not matter for timing.  Reported: the transfer alone, the 14 reduce calls
    alone (inputs already staged), and the pipeline with and without overlap."""
    from paper_2412_01152_amd.pipeline import new_staging, reduce_chunks_pipelined
    N = synth.n_elements(2)
    chunk_sizes = synth.ring_chunk_sizes(N, 14)
    coff = synth.offsets_from_sizes(chunk_sizes)
    W, n0 = 13, chunk_sizes[0]
    log(f"[bench] config 4 overlap: N={N}, 14 chunks of {n0}, W={W} coded (pinned host) + fp32 local")
    t0 = time.time()
    theta = torch.empty(n0, dtype=torch.float32, device=dev)
    loc = torch.empty(n0, dtype=torch.float32, device=dev)
    codes = torch.empty(n0, dtype=torch.uint8, device=dev)
    lut = torch.empty((1, 256), dtype=torch.float32, device=dev)
    synth.fill_theta_outer(theta)
    host_codes, host_luts = [], []
    for p in range(W):
        synth.fill_theta_local(loc, theta, p, "mixture")
        B.pseudograd_quantize(theta, loc, [0, n0], codes_out=codes, lut_out=lut)
        host_codes.append(torch.empty(n0, dtype=torch.uint8, pin_memory=True).copy_(codes))
        host_luts.append(torch.empty((1, 256), dtype=torch.float32, pin_memory=True).copy_(lut))
    synth.fill_theta_local(loc, theta, W, "mixture")
    loc.sub_(theta).neg_()
    local = torch.empty(N, dtype=torch.float32, device=dev)
    for c in range(14):
        local[coff[c]:coff[c + 1]] = loc[:coff[c + 1] - coff[c]]
    del theta, loc, codes
    codes2 = torch.empty(N, dtype=torch.uint8, device=dev)
    lut2 = torch.empty((14, 256), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] host-resident peers ready ({time.time() - t0:.1f}s)")

    def arrive(c, code_bufs, lut_bufs):
        n = coff[c + 1] - coff[c]
        for p in range(W):
            code_bufs[p].copy_(host_codes[p][:n], non_blocking=True)
            lut_bufs[p].copy_(host_luts[p], non_blocking=True)

    def no_arrival(c, code_bufs, lut_bufs):
        pass

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / reps

    copy_stream = torch.cuda.Stream(dev)
    staging = new_staging(n0, W, dev)

    def copy_only():                               # also leaves both staging sets holding real codes
        for c in range(14):
            ph, n = coff[c] % 128, coff[c + 1] - coff[c]
            arrive(c, [b[ph:ph + n] for b in staging[0][c & 1]], staging[1][c & 1])

    t_copy = timed(copy_only, 1)
    run = lambda arr, ov, ev=None: reduce_chunks_pipelined(coff, W, 14, arr, local, codes2, lut2,
                                                           copy_stream=copy_stream, overlap=ov, staging=staging,
                                                           timing_out=ev)
    t_reduce = timed(lambda: run(no_arrival, True), max(1, args.steps))
    t_serial = timed(lambda: run(arrive, False), 1)
    t_overlap = timed(lambda: run(arrive, True), 1)
    ev_alone, ev_under = [], []
    run(arrive, False, ev_alone)                   # same idle gaps between calls, no transfer beside them
    run(arrive, True, ev_under)
    torch.cuda.synchronize()
    log("[bench] per-call ms alone :", " ".join(f"{a.elapsed_time(b):.2f}" for a, b in ev_alone))
    log("[bench] per-call ms beside:", " ".join(f"{a.elapsed_time(b):.2f}" for a, b in ev_under))
    ms_alone = sorted(a.elapsed_time(b) for a, b in ev_alone[:13])      # chunks 0..12 have a transfer beside them
    ms_under = sorted(a.elapsed_time(b) for a, b in ev_under[:13])
    h2d = W * N / t_copy / 1e9
    log(f"[bench] transfer alone      {t_copy * 1e3:9.2f} ms  ({h2d:.1f} GB/s host to device)")
    log(f"[bench] 14 reduces alone    {t_reduce * 1e3:9.2f} ms  ({26 * N / t_reduce / 1e9:.1f} GB/s)")
    log(f"[bench] copy then reduce    {t_serial * 1e3:9.2f} ms")
    log(f"[bench] pipelined           {t_overlap * 1e3:9.2f} ms  (exposed reduce time "
        f"{(t_overlap - t_copy) * 1e3:.2f} ms of {t_reduce * 1e3:.2f})")
    log(f"[bench] one reduce call, median of 13: alone {ms_alone[6]:.3f} ms, beside a transfer {ms_under[6]:.3f} ms "
        f"(+{100 * (ms_under[6] / ms_alone[6] - 1):.1f}%)")
    # The same pipeline with the contributions arriving from device memory: a second resident copy of one
    # chunk's coded contributions is copied into the staging set on the copy stream (device-to-device, at
    # hundreds of GB/s instead of the host link's tens) while the previous chunk is reduced; 1, 4 or all 13
    # of a chunk's contributions arrive that way, the others are already in place.
    dev_codes = [torch.empty(n0, dtype=torch.uint8, device=dev).copy_(h, non_blocking=True) for h in host_codes]
    dev_luts = [h.to(dev) for h in host_luts]
    torch.cuda.synchronize()
    d2d = {}
    for inbound in (1, 4, W):
        def arrive_d2d(c, code_bufs, lut_bufs, k=inbound):
            n = coff[c + 1] - coff[c]
            for p in range(k):
                code_bufs[p].copy_(dev_codes[p][:n], non_blocking=True)
                lut_bufs[p].copy_(dev_luts[p], non_blocking=True)

        def copy_only_d2d():
            with torch.cuda.stream(copy_stream):
                for c in range(14):
                    ph, n = coff[c] % 128, coff[c + 1] - coff[c]
                    arrive_d2d(c, [b[ph:ph + n] for b in staging[0][c & 1]], staging[1][c & 1])
            torch.cuda.current_stream().wait_stream(copy_stream)

        t_c = timed(copy_only_d2d, 2)
        t_o = timed(lambda: run(arrive_d2d, True), 2)
        ev_a, ev_u = [], []
        run(arrive_d2d, False, ev_a)
        run(arrive_d2d, True, ev_u)
        torch.cuda.synchronize()
        m_a = sorted(a.elapsed_time(b) for a, b in ev_a[:13])
        m_u = sorted(a.elapsed_time(b) for a, b in ev_u[:13])
        rate = inbound * N / t_c / 1e9
        d2d[f"{inbound} of {W} contributions inbound"] = {
            "transfer_alone_ms": round(t_c * 1e3, 2), "inbound_GB/s": round(rate, 1),
            "pipelined_ms": round(t_o * 1e3, 2),
            "reduce_call_ms": {"alone": round(m_a[6], 3), "beside_transfer": round(m_u[6], 3)}}
        log(f"[bench] device-to-device arrival, {inbound:2d} of {W} contributions: transfer alone {t_c * 1e3:7.2f} ms "
            f"({rate:.0f} GB/s inbound), pipelined {t_o * 1e3:7.2f} ms (14 reduces alone {t_reduce * 1e3:.2f}); one reduce "
            f"call {m_a[6]:.3f} ms alone, {m_u[6]:.3f} ms beside the transfer (+{100 * (m_u[6] / m_a[6] - 1):.1f}%)")
    result = {"metric": "ring-chunk pipeline: transfer of chunk c+1 overlapping int8 reduce of chunk c, 10B",
              "value": round(t_overlap * 1e3, 2), "unit": "ms", "n_gpus": 1, "steps": 1, "warmup": 1,
              "ms_per_step": round(t_overlap * 1e3, 2), "higher_is_better": False, "scaling": "weak",
              "vs_baseline": None, "dtype": "f32", "data": "synthetic",
              "config": {"workload": f"config4 pipelined: 14 ring chunks of {n0}, 13 coded peers from pinned host "
                                     f"memory + fp32 local", "elements": N, "segments": 14, "peers": W},
              "transfer_alone_ms": round(t_copy * 1e3, 2), "reduce_alone_ms": round(t_reduce * 1e3, 2),
              "serial_ms": round(t_serial * 1e3, 2), "pipelined_ms": round(t_overlap * 1e3, 2),
              "h2d_GB/s": round(h2d, 1),
              "reduce_call_ms": {"alone": round(ms_alone[6], 3), "beside_transfer": round(ms_under[6], 3)},
              "device_to_device_arrival": d2d, "roofline": None, "cpu_baseline": None}
    print(json.dumps(result), flush=True)


def time_extras(torch, B, theta, local, mom, peer_codes, peer_luts, codes1, lut1, codes2, lut2, qp, ws, off, N, T, W,
                alloc, bf16_slot=None):
    """Whole-call timings (HIP events around the call, 5 repetitions) of the variants bench's step does
    not use.  Runs last: the stored-accumulation variant overwrites theta_local."""
    out = {}

    def timed(name, bytes_per_elem, fn, reps=5):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbs = bytes_per_elem * N / (ms * 1e-3) / 1e9
        out[name] = {"ms": round(ms, 3), "bytes_per_element": bytes_per_elem, "GB/s": round(gbs, 1),
                     "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}
        log(f"[bench] extra {name:52s} {ms:8.3f} ms  {gbs:8.1f} GB/s  {100 * gbs / HBM_PEAK_GBS:.1f}% of peak")

    # the bf16 weights stage 1 READS sit next to theta when there is room (bf16_slot); the bf16 weights the
    # outer step WRITES go far from theta and momentum, like every written buffer
    handback_bf16 = alloc(N, torch.bfloat16)
    local_bf16 = (bf16_slot if bf16_slot is not None else handback_bf16).copy_(local)
    scratch_f32 = alloc(N, torch.float32)
    timed("stage1 bf16 theta_local (13 B/elem)", 13,
          lambda: B.pseudograd_quantize(theta, local_bf16, off, codes_out=codes1, lut_out=lut1, qparams_out=qp,
                                        workspace=ws))
    # the quantiser with bucket midpoints instead of bucket averages as its codebook (a variant the paper argues
    # against in words): pass B then needs no bucket sums, so no LDS atomics and no offset arithmetic
    timed("stage1 fp32, midpoint codebook (17 B/elem)", 17,
          lambda: B.pseudograd_quantize(theta, local, off, codes_out=codes1, lut_out=lut1, qparams_out=qp,
                                        workspace=ws, variant=(6.0, B.CODEBOOK_MIDPOINT)))
    timed(f"stage2 W={W}, midpoint codebook ({2 * W + 1} B/elem)", 2 * W + 1,
          lambda: B.reduce_chunk(peer_codes, peer_luts, off, W, codes_out=codes2, lut_out=lut2, qparams_out=qp,
                                 workspace=ws, variant=(6.0, B.CODEBOOK_MIDPOINT)))
    B.reduce_chunk(peer_codes, peer_luts, off, W, codes_out=codes2, lut_out=lut2, qparams_out=qp, workspace=ws)
    timed("stage3 coded + bf16 hand-back (19 B/elem)", 19,
          lambda: B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=off,
                               theta_local_out=handback_bf16, workspace=ws))
    del local_bf16, handback_bf16
    timed(f"stage2 W={W} storing the accumulation ({W + 9} B/elem)", W + 9,
          lambda: B.reduce_chunk(peer_codes, peer_luts, off, W, acc_out=local, codes_out=codes2, lut_out=lut2,
                                 qparams_out=qp, workspace=ws))
    timed(f"stage2 W={W - 1} + fp32 local, in place ({W - 1 + 13} B/elem)", W - 1 + 13,
          lambda: B.reduce_chunk(peer_codes[1:], peer_luts[1:], off, W, local_fp32=local, acc_out=local,
                                 codes_out=codes2, lut_out=lut2, qparams_out=qp, workspace=ws))
    timed("stage3 fp32 delta (20 B/elem)", 20,
          lambda: B.outer_step(theta, mom, LR, BETA, delta_fp32=local, workspace=ws))
    timed("stage3 fp32 delta + fp32 hand-back (24 B/elem)", 24,
          lambda: B.outer_step(theta, mom, LR, BETA, delta_fp32=local, workspace=ws,
                               theta_local_out=scratch_f32))
    return out


def kernel_record(avg_ms, bytes_per_launch):
    gbs = bytes_per_launch / (avg_ms * 1e-3) / 1e9
    return {"avg_ms": round(avg_ms, 4), "GB/s": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}


def call_record(ms, bytes_per_elem, n):
    gbs = bytes_per_elem * n / (ms * 1e-3) / 1e9
    return {"ms": round(ms, 3), "bytes_per_element": bytes_per_elem, "GB/s": round(gbs, 1),
            "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}


def csrc_sha16():
    """Hash of the library's sources: the counter summaries under profiles/ carry the hash of the sources they
    were measured with, and a summary taken with other sources is not quoted."""
    import hashlib
    d = os.path.join(ROOT, "paper_2412_01152_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip", ".cpp", ".c")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic_bytes(profile_file, kernel_name):
    """HBM bytes per launch of `kernel_name` from a committed rocprofv3 counter summary under profiles/
    (FETCH_SIZE and WRITE_SIZE in KiB per dispatch and the factors that a plain copy of known size gave for
    the same counters).  The figure is measured offline, never estimated here: None if the file or the row is
    missing, or if the file was taken with other kernel sources than the ones in the tree (its csrc_sha16
    line differs from the hash of csrc/ now)."""
    path = os.path.join(ROOT, "profiles", profile_file)
    if not os.path.exists(path):
        return None
    stamp_ok = False
    row = None
    for line in open(path):
        if line.startswith("# csrc_sha16:"):
            stamp_ok = line.split(":", 1)[1].strip() == csrc_sha16()
        if line.startswith("#") or "|" not in line:
            continue
        cols = [c.strip() for c in line.split("|")]
        if cols[0] == kernel_name and len(cols) >= 5:
            fetch_kib, write_kib, fetch_factor, write_factor = (float(c) for c in cols[1:5])
            row = round((fetch_kib / fetch_factor + write_kib / write_factor) * 1024.0)
    if not stamp_ok:
        if row is not None:
            log(f"[bench] profiles/{profile_file} was taken with other kernel sources: traffic not quoted")
        return None
    return row


def host_cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_oracle_baseline(np, torch, synth, theta, local, off, sizes, cfg, W, layers, alloc):
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
    scratch = alloc(n, torch.float32)
    threads = oracle.num_threads()
    t_setup = time.perf_counter()
    for p in range(1, W):
        synth.fill_theta_local(scratch, theta[a:b], p, synth.config_delta_kind(cfg), seed=synth.BASE_SEED + 1)
        c, l, _, _ = oracle.pseudograd_quantize(th, scratch.cpu().numpy(), sample_off)
        pcs.append(c)
        pls.append(l)
    del scratch
    cpu_model, logical = host_cpu_model(), os.cpu_count()
    log(f"[bench] cpu baseline: sample of {n} elements, {threads} threads on {cpu_model} ({logical} logical CPUs), "
        f"setup {time.perf_counter() - t_setup:.1f}s")
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
    # the same three calls on one thread, on the first two tensors of the sample only
    k1 = min(2, len(sample_off) - 1)
    n1, off1 = sample_off[k1], sample_off[:k1 + 1]
    oracle.set_num_threads(1)
    t6 = time.perf_counter()
    c0s, l0s, _, _ = oracle.pseudograd_quantize(th[:n1], lo[:n1], off1)
    _, c2s, l2s, _ = oracle.reduce([c0s] + [c[:n1] for c in pcs], [l0s] + [l[:k1] for l in pls], off1, W)
    m1, th1 = np.zeros(n1, dtype=np.float32), th[:n1].copy()
    oracle.outer_step(th1, m1, LR, BETA, delta_codes=c2s, delta_luts=l2s, seg_offsets=off1)
    secs1 = time.perf_counter() - t6
    oracle.set_num_threads(threads)
    gbs1 = bpe * n1 / secs1 / 1e9
    log(f"[bench] cpu baseline, 1 thread on {n1} elements: {secs1:.2f}s -> {gbs1:.2f} GB/s")
    log(f"[bench] cpu baseline: stage1 {t2 - t1:.2f}s stage2 {t3 - t2:.2f}s stage3 {t5 - t4:.2f}s -> {gbs:.2f} GB/s")
    return {"value": round(gbs, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"first {max(1, layers) if cfg == 2 else 1} decoder layer(s) of the same workload "
                      f"({n} elements in {len(sample_off) - 1} tensors, W={W}), same {bpe} B/element "
                      f"accounting; wall seconds per stage: {t2 - t1:.2f}/{t3 - t2:.2f}/{t5 - t4:.2f} "
                      f"(about {secs * threads:.0f} core-seconds)",
            "seconds": round(secs, 3), "cpu": cpu_model, "logical_cpus": logical,
            "one_thread": {"value": round(gbs1, 3), "unit": "GB/s", "elements": n1, "seconds": round(secs1, 3)}}


if __name__ == "__main__":
    main()
