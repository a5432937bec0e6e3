#!/usr/bin/env python3
"""Benchmark of the secret-shared ReLU hot path on one MI355X.

A step is one pass of hb_relu over the headline workload: the 17 ReLU input tensors of ResNet18 on
3x32x32 images at batch 512 (285,212,672 elements, 2^16 fixed point, int64 shares), slice
(k, m) = (12, 20), every tensor with its own seed, issued through hb_relu_batch (one kernel launch for
the 17 tensors).  Inputs and outputs are resident in HBM before the timed region starts.  The GPU's clocks
ramp up over the first tens of milliseconds of load, so a fixed pre-warm of the same workload (about 0.4 s)
runs before the counted warm-up steps.  Prints ONE JSON line:

  value / ms_per_step   the headline run (w = 8)
  roofline              the headline kernel against the HBM peak (32 B per element; the metric's fraction)
  roofline_alu          the same launch against its vector-ALU issue floor at the clock measured in this run
  roofline_w64          hb_relu at (0, 64) on the first tensor: HBM fraction and issue floor
  configs               every named workload: time per call, elements/s, HBM fraction, opened bits per element
  cpu_baseline(_w64)    the CPU oracle on this machine's host cores, bounded samples
  extra                 the other entry points

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-extra]
    python bench.py --microbench      # instruction issue costs, streaming probes, socket power: a text report
"""
import argparse
import glob
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

ROOT_SEED = 0x2309048750000001
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
BYTES_PER_ELEMENT = 32         # two int64 shares read, two written
SIMDS = 256 * 4                # compute units x SIMDs per compute unit


def profile_constants():
    """`@const name = value` lines of the rocprofv3 summaries under profiles/ (counter readings and microbenchmark
    results that the live run cannot measure itself)."""
    out = {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        with open(path) as f:
            for line in f:
                m = re.match(r"^@const\s+(\S+)\s*=\s*([-+0-9.eE]+)\s*(#.*)?$", line.strip())
                if m:
                    out[m.group(1)] = float(m.group(2))
    return out


def kernel_name(w, op="relu", batched=False):
    if w <= 32:
        return "hb::%s<%d, %s>" % ("tile_batch_kernel" if batched else "tile_kernel", w, op)
    return "hb::group_kernel<%d, %s, vec>" % (w, op)


def party_path_bytes(n, k, m):
    """Bytes the party-faithful path must move for one ReLU: what each of its kernels reads and writes once
    (shares, per-group state words, wire words, per-element DReLU shares, results), both parties."""
    w = m - k
    L = min(64 // w, 32)
    R = 0 if w == 1 else (w - 1).bit_length()
    G = (n + L - 1) // L
    b2a = (n + 63) // 64
    words = 2 * n + 2 * G * (2 + 2)                                   # slice: read shares; write S, P, two wire words
    for r in range(R):                                               # round: read state + both wires' previous message;
        words += 2 * G * ((1 + 4 if r == 0 else 2 + 8) + 2 + 4)      #        write G, P and four wire words
    words += 2 * G * (2 + (4 if R else 4) + 1)                       # sign: read S, G, the last G-update opening; write Z
    words += 2 * (G + b2a)                                           # B2A: read Z, write packed bits
    words += 2 * (n + 2 * b2a + n + 2 * n)                           # multiply send: read share, B2A words; write D, 2 wire words
    words += 2 * (4 * n + n)                                         # result: read both wires' multiply words, write result
    return 8 * words


def _time_launches(fn, torch, warm_ms=120.0, meas_ms=150.0, max_reps=4000):
    """Average duration in ms of `fn` (one call) by events on the current stream: the same load runs for
    `warm_ms` beforehand so the clocks have settled, then for about `meas_ms` between the events."""
    fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    e1.record()
    torch.cuda.synchronize()
    one = max(e0.elapsed_time(e1), 0.002)
    for _ in range(min(max_reps, int(warm_ms / one) + 1)):
        fn()
    reps = min(max_reps, int(meas_ms / one) + 1)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _clock_under(load_fn, torch, probes, dev, launch_ms, spins=400000, reps=3):
    """Shader clock (MHz) while `load_fn` launches run back to back.  A one-wavefront probe on a second stream takes
    a wave slot when one frees up and times a fixed dependent chain of about 15 ms (many launches long: the clock
    moves under the power limit, and windows of a millisecond read anything from 1.75 to 2.15 GHz) against the
    100 MHz counter; launches of the load are enqueued before it (60 ms) and after it (40 ms), so it never runs next
    to an idle GPU.  Median of `reps` probes."""
    side = torch.cuda.Stream()
    before = max(4, int(60.0 / launch_ms))
    after = max(4, int(40.0 / launch_ms))
    readings = []
    for _ in range(reps):
        stamps = torch.zeros(2, dtype=torch.int64, device=dev)
        torch.cuda.synchronize()
        for _ in range(before):
            load_fn()
        with torch.cuda.stream(side):
            probes.clock_probe(spins, stamps)
        for _ in range(after):
            load_fn()
        torch.cuda.synchronize()
        ticks = stamps.cpu().tolist()
        readings.append(100.0 * ticks[0] / max(ticks[1], 1))
    return sorted(readings)[len(readings) // 2]


def _issue_floor(consts, prefix, waves, launch_ms, clock_mhz):
    """The launch priced in SIMD issue cycles: vector-ALU instructions per wavefront (counter reading) split
    into classes (compiler listing of the kernel), each class at the cost measured for it ALONE on all
    compute units (a lower bound: mixed streams run slower), against elapsed cycles x 1024 SIMDs at the clock
    measured in this run."""
    need = [prefix + ".valu_insts_per_wave", prefix + ".frac_two_operand", prefix + ".frac_bitop3",
            "issue.cycles_two_operand", "issue.cycles_bitop3", "issue.cycles_full_rate"]
    if clock_mhz is None or any(k not in consts for k in need):
        return None
    per_wave = consts[prefix + ".valu_insts_per_wave"]
    f2, f3 = consts[prefix + ".frac_two_operand"], consts[prefix + ".frac_bitop3"]
    floor_cycles = per_wave * (f2 * consts["issue.cycles_two_operand"] + f3 * consts["issue.cycles_bitop3"] +
                               (1.0 - f2 - f3) * consts["issue.cycles_full_rate"])
    available = launch_ms * 1e-3 * clock_mhz * 1e6 * SIMDS          # SIMD cycles of the launch
    needed = floor_cycles * waves
    return {"bound": "alu", "achieved": needed / (launch_ms * 1e-3) / 1e9, "peak": clock_mhz * 1e6 * SIMDS / 1e9,
            "unit": "G SIMD issue cycles/s", "frac": needed / available,
            "gap_to_issue_floor_pct": 100.0 * (1.0 - needed / available),
            "shader_clock_mhz_in_this_run": clock_mhz,
            "valu_insts_per_wave": per_wave, "wavefronts_per_launch": waves,
            "issue_floor_cycles_per_wave": floor_cycles,
            "measured_cycles_per_instruction": available / (per_wave * waves),
            "class_costs_alone": {"two_operand": consts["issue.cycles_two_operand"],
                                  "bitop3": consts["issue.cycles_bitop3"],
                                  "multiplier_64bit_three_operand": consts["issue.cycles_full_rate"]},
            "class_fractions": {"two_operand": f2, "bitop3": f3, "multiplier_64bit_three_operand": 1.0 - f2 - f3},
            "valu_busy_pct_profiled": consts.get(prefix + ".valu_busy_pct"),
            "peak_derivation": "1024 SIMDs x the shader clock measured while this kernel runs"}


def _socket_power():
    """Socket power in W from amd-smi (None when the tool is missing or prints something else)."""
    try:
        out = subprocess.run(["amd-smi", "metric", "-p"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True,
                             timeout=20).stdout
    except (OSError, subprocess.SubprocessError):
        return None
    m = re.search(r"SOCKET_POWER\s*:\s*([0-9.]+)", out)
    return float(m.group(1)) if m else None


def microbench(torch, hb, probes, workloads, dev):
    """Text report: issue cost of instruction classes and of mixed streams, streaming ceilings, socket power."""
    say = lambda s="": print(s, flush=True)
    say("# microbenchmarks on %s (python bench.py --microbench)" % torch.cuda.get_device_name(0))
    say("# issue cost: all 256 compute units, 64-instruction unrolled streams on eight independent registers,")
    say("# SIMD cycles per wave64 instruction = duration x shader clock (measured inside the launch) / instructions per SIMD")
    names = probes.issue_probe_names()
    alone = probes.issue_class_count()
    say("%-66s %5s %9s %9s %8s" % ("stream", "w/SIMD", "ms", "MHz", "cycles"))
    for i, name in enumerate(names):
        groups16 = name.startswith("16-wave")
        for wps in ((8, 4) if groups16 else ((8, 2, 1) if i < alone else (8,))):
            iters = (256 if groups16 else 2048) if i >= alone else 2048
            r = probes.issue_probe(i, wps, iters)
            say("%-66s %5d %9.3f %9.0f %8.2f" % (name, wps, r["ms"], r["mhz"], r["cycles_per_instruction"]))
    say()
    say("# streaming: out0 = x0 + x1, out1 = x0 ^ x1 over 2^25 int64 elements (32 B per element), 16-byte accesses")
    n = 1 << 25
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    x0 = torch.randint(-2**62, 2**62, (n,), generator=g, device=dev, dtype=torch.int64)
    x1 = torch.randint(-2**62, 2**62, (n,), generator=g, device=dev, dtype=torch.int64)
    o0, o1 = torch.empty_like(x0), torch.empty_like(x1)
    for nt in (True, False):
        for xcd in (False, True):
            ms = _time_launches(lambda: probes.stream_copy(x0, x1, o0, o1, nt, xcd), torch, 200.0, 200.0)
            say("%-22s %-44s %8.4f ms %8.1f GB/s" % ("non-temporal" if nt else "plain loads/stores",
                                                     "each XCD a contiguous eighth" if xcd else "consecutive blocks stream neighbours",
                                                     ms, 32.0 * n / ms / 1e6))
    ms = _time_launches(lambda: hb.hb_open(x0, x1, False, out=o0), torch, 200.0, 200.0)
    say("%-22s %-44s %8.4f ms %8.1f GB/s" % ("hb_open", "24 B per element", ms, 24.0 * n / ms / 1e6))
    say()
    say("# socket power (amd-smi metric -p, SOCKET_POWER), two readings between 1.2 s and 2.5 s into a steady load of about 4 s")
    say("%-44s %8s %8s" % ("load", "W", "W"))
    torch.cuda.synchronize()
    time.sleep(3.0)
    say("%-44s %8s" % ("idle (3 s after the last kernel)", _socket_power()))

    def under(name, enqueue):
        # the launches are enqueued from a second host thread (the launch queue is finite, so enqueueing seconds of
        # work blocks its caller) while this thread reads the power
        import threading
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()

        def feed():
            with torch.cuda.stream(stream):
                enqueue()
        th = threading.Thread(target=feed)
        th.start()
        time.sleep(1.2)
        p1 = _socket_power()
        time.sleep(0.4)
        p2 = _socket_power()
        th.join()
        torch.cuda.synchronize()
        say("%-44s %8s %8s" % (name[:44], p1, p2))
        return p2

    spec = workloads.resnet18_cifar_batch512()[0]
    _, s0, s1 = workloads.materialize_on_device(spec, dev)
    q0, q1 = torch.empty_like(s0), torch.empty_like(s1)
    idle = _socket_power()
    for idx in [names.index(t) for t in ("v_xor_b32", "v_bitop3_b32", "v_mul_lo_u32", "v_mad_u64_u32", "v_lshrrev_b64",
                                         "16-wave groups: xor x128 / mul_lo x128, free-running",
                                         "16-wave groups: xor x128 / mul_lo x128, barrier after each run")]:
        iters = 256 if names[idx].startswith("16-wave") else 2048
        r = probes.issue_probe(idx, 8, iters)
        launches = max(1, int(4000.0 / r["ms"]))
        p = under(names[idx] + " on all compute units", lambda: probes.issue_load(idx, 8, iters, launches))
        if p and idle:
            rate = r["instructions_per_wave"] * 8 * SIMDS / (r["ms"] * 1e-3)       # wavefront-instructions per second
            say("%-44s %8.2f nJ per wavefront-instruction above idle (%.2f cycles each at %.0f MHz)"
                % ("", (p - idle) / rate * 1e9, r["cycles_per_instruction"], r["mhz"]))
    ms = _time_launches(lambda: hb.hb_relu(s0, s1, 12, 20, 7, q0, q1), torch)
    under("hb_relu w = 8, 2^25 elements", lambda: [hb.hb_relu(s0, s1, 12, 20, 7, q0, q1) for _ in range(int(4000.0 / ms))])
    ms = _time_launches(lambda: hb.hb_drelu(s0, s1, 12, 20, 7, q0, q1), torch)
    under("hb_drelu w = 8, 2^25 elements", lambda: [hb.hb_drelu(s0, s1, 12, 20, 7, q0, q1) for _ in range(int(4000.0 / ms))])
    ms = _time_launches(lambda: hb.hb_relu(s0, s1, 0, 64, 7, q0, q1), torch)
    under("hb_relu w = 64, 2^25 elements", lambda: [hb.hb_relu(s0, s1, 0, 64, 7, q0, q1) for _ in range(int(4000.0 / ms))])
    ms = _time_launches(lambda: hb.hb_open(s0, s1, False, out=q0), torch)
    under("hb_open, 2^25 elements", lambda: [hb.hb_open(s0, s1, False, out=q0) for _ in range(int(4000.0 / ms))])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="only the headline run (profiling passes)")
    ap.add_argument("--microbench", action="store_true", help="print the microbenchmark report and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (both parties are simulated on it; there is no "
                 "sharded or multi-rank path) -- run with --gpus 1")

    import torch
    from paper_2309_04875_amd import hb, probes, workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    hb.load()       # fails loudly when the HIP library has not been built
    probes.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.microbench:
        microbench(torch, hb, probes, workloads, dev)
        return
    consts = profile_constants()

    # ---- inputs resident in HBM ------------------------------------------------------------
    specs = workloads.resnet18_cifar_batch512()
    tensors = []
    for spec in specs:
        _, s0, s1 = workloads.materialize_on_device(spec, dev)
        tensors.append((spec, s0, s1, torch.empty_like(s0), torch.empty_like(s1),
                        hb.hb_tensor_seed(ROOT_SEED, spec.tensor_id)))
    n_total = sum(s.n for s in specs)
    k, m = specs[0].k, specs[0].m
    waves_headline = sum((s.n + 511) // 512 for s in specs)       # a wavefront takes 64 groups of 8 elements at w = 8
    torch.cuda.synchronize()

    batch = hb.make_batch([(s0, s1, o0, o1, spec.k, spec.m, seed) for (spec, s0, s1, o0, o1, seed) in tensors])

    def step():
        return hb.hb_relu_batch(batch)

    # fixed pre-warm (not counted): the same workload until the clocks have settled
    t_end = time.perf_counter() + 0.4
    while time.perf_counter() < t_end:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; a HIP event pair on the launch stream brackets each step's launch ----
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for (a, b) in events:
        a.record()
        opened = step()
        b.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = n_total / (ms_per_step * 1e-3)

    launch_ms = [a.elapsed_time(b) for (a, b) in events]      # one launch of hb::tile_batch_kernel<8, relu> per step
    avg_launch_ms = sum(launch_ms) / len(launch_ms)
    bytes_per_launch = BYTES_PER_ELEMENT * n_total
    achieved_gbs = bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9

    traffic = None
    if consts.get("headline.elements") == n_total and "headline.fetch_kib" in consts and "headline.write_kib" in consts:
        traffic = 1024.0 * (consts["headline.fetch_kib"] * consts.get("counter.fetch_scale", 1.0) +
                            consts["headline.write_kib"] * consts.get("counter.write_scale", 1.0))
    roofline = {"bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved_gbs / HBM_PEAK_GBS, "traffic": traffic,
                "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by what the "
                                "counter reads for a streaming kernel of known size; profiles/)",
                "kernel": kernel_name(8, "relu", True), "avg_launch_ms": avg_launch_ms,
                "algorithmic_bytes_per_launch": bytes_per_launch, "algorithmic_bytes_per_element": BYTES_PER_ELEMENT,
                "target_frac": 0.60, "target_met": achieved_gbs / HBM_PEAK_GBS >= 0.60,
                "valu_busy_pct_profiled": consts.get("headline.valu_busy_pct"),
                "mean_occupancy_per_cu_profiled": consts.get("headline.mean_occupancy_per_cu"),
                "vgprs": consts.get("headline.vgprs")}

    clock_mhz = None if args.no_extra else _clock_under(step, torch, probes, dev, avg_launch_ms)
    roofline_alu = _issue_floor(consts, "headline", waves_headline, avg_launch_ms, clock_mhz)
    if roofline_alu is not None:
        roofline_alu["kernel"] = kernel_name(8, "relu", True)

    spec0, s0, s1, o0, o1, seed0 = tensors[0]
    bits_w8 = opened / n_total
    bits_full_ring = hb.hb_opened_bits(True, 0, 64, 1)
    extra = {"shader_clock_mhz_under_headline_kernel": clock_mhz,
             "opened_bits_per_element": bits_w8,
             "opened_bits_ratio_vs_sec_2_3_unpacked_accounting": hb.BASELINE_BITS_PER_ELEMENT / bits_w8,
             "opened_bits_ratio_vs_this_library_at_0_64": bits_full_ring / bits_w8}
    configs = [{"name": "cfg3 resnet18 32x32 batch 512, (12,20) [headline, timed region]", "elements": n_total,
                "widths": [8], "calls": "one hb_relu_batch (1 launch)", "us_per_call": avg_launch_ms * 1e3,
                "elements_per_s": n_total / (avg_launch_ms * 1e-3), "hbm_frac": achieved_gbs / HBM_PEAK_GBS,
                "opened_bits_per_element": bits_w8, "kernel": kernel_name(8, "relu", True)}]
    roofline_w64 = None
    cpu_w64 = None

    if not args.no_extra:
        # ---- w = 64 (the other width the metric names): hb_relu at (0, 64) on the first tensor (2^25 elements) ----
        def relu64():
            hb.hb_relu(s0, s1, 0, 64, seed0, o0, o1)
        ms64 = _time_launches(relu64, torch, 200.0, 300.0)
        gbs64 = BYTES_PER_ELEMENT * spec0.n / (ms64 * 1e-3) / 1e9
        clock64 = _clock_under(relu64, torch, probes, dev, ms64)
        roofline_w64 = {"bound": "hbm", "achieved": gbs64, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": gbs64 / HBM_PEAK_GBS, "kernel": kernel_name(64), "elements": spec0.n,
                        "elements_per_s": spec0.n / (ms64 * 1e-3), "avg_launch_ms": ms64,
                        "opened_bits_per_element": bits_full_ring,
                        "valu_insts_per_element": consts.get("w64.valu_insts_per_wave"),
                        "valu_busy_pct_profiled": consts.get("w64.valu_busy_pct"),
                        "mean_occupancy_per_cu_profiled": consts.get("w64.mean_occupancy_per_cu"),
                        "vgprs": consts.get("w64.vgprs"),
                        "binding": _issue_floor(consts, "w64", (spec0.n + 63) // 64, ms64, clock64)}

        # ---- the other named workloads ---------------------------------------------------------------------
        def add_config(name, n, widths, calls, ms, bits, kern):
            configs.append({"name": name, "elements": n, "widths": widths, "calls": calls, "us_per_call": ms * 1e3,
                            "elements_per_s": n / (ms * 1e-3), "hbm_frac": BYTES_PER_ELEMENT * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "opened_bits_per_element": bits, "kernel": kern})

        # cfg 1 and cfg 2 are launch-bound: the per-call figure is the prepared-set call (hb_plan_run: arguments
        # checked once at hb_plan_create, each call only enqueues); the plain calls, which check every pointer on
        # every call, and a HIP-graph replay are in `extra`
        for (kk, mm) in ((0, 64), (12, 20)):                      # cfg 1: flat 65,536
            sp = workloads.flat_normal(65536, kk, mm)
            _, a, b = workloads.materialize_on_device(sp, dev)
            c, d = torch.empty_like(a), torch.empty_like(b)
            plan = hb.hb_plan_create([(a, b, c, d, kk, mm, ROOT_SEED)], True)
            ms = _time_launches(plan.run, torch, 30.0, 60.0)
            add_config("cfg1 flat 65,536, (%d,%d)" % (kk, mm), sp.n, [mm - kk], "one hb_plan_run (1 launch)", ms,
                       hb.hb_opened_bits(True, kk, mm, 1), kernel_name(mm - kk) if mm - kk > 32 else "hb::small_batch_kernel<%d, relu>" % (mm - kk))
            ms = _time_launches(lambda: hb.hb_relu(a, b, kk, mm, ROOT_SEED, c, d), torch, 30.0, 60.0)
            extra["flat_65536_w%d_us_plain_hb_relu_call" % (mm - kk)] = ms * 1e3
            hb.hb_plan_destroy(plan)
        small = []                                                # cfg 2: one image, 17 tensors, per-tensor (k, m)
        for sp in workloads.resnet18_cifar():
            _, a, b = workloads.materialize_on_device(sp, dev)
            small.append((a, b, torch.empty_like(a), torch.empty_like(b), sp.k, sp.m, hb.hb_tensor_seed(ROOT_SEED, sp.tensor_id)))
        n_small = sum(t[0].numel() for t in small)
        small_batch = hb.make_batch(small)
        bits_small = hb.hb_relu_batch(small_batch) / n_small
        plan = hb.hb_plan_create(small_batch, True)
        ms = _time_launches(plan.run, torch, 30.0, 60.0)
        add_config("cfg2 resnet18 32x32 one image, per-tensor (k,m)", n_small, [8], "one hb_plan_run (1 launch)", ms, bits_small,
                   "hb::small_batch_kernel<8, relu>")
        ms = _time_launches(lambda: hb.hb_relu_batch(small_batch), torch, 30.0, 60.0)
        extra["one_image_set_us_plain_batched_call"] = ms * 1e3
        ms = _time_launches(lambda: [hb.hb_relu(a, b, kk, mm, sd, c, d) for (a, b, c, d, kk, mm, sd) in small], torch, 30.0, 60.0)
        extra["one_image_set_us_per_tensor_calls"] = ms * 1e3
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(20):
                    plan.run()
        torch.cuda.synchronize()
        ms = _time_launches(graph.replay, torch, 30.0, 60.0)
        extra["one_image_set_us_per_call_in_a_graph_of_20"] = ms * 1e3 / 20.0
        hb.hb_plan_destroy(plan)
        del graph, small, small_batch, plan
        sweep = workloads.width_sweep()                           # cfg 4: flat 2^26, six widths, one pair of buffers
        _, a, b = workloads.materialize_on_device(sweep[0], dev)
        c, d = torch.empty_like(a), torch.empty_like(b)
        for sp in sweep:
            ms = _time_launches(lambda: hb.hb_relu(a, b, sp.k, sp.m, ROOT_SEED, c, d), torch, 100.0, 150.0)
            add_config("cfg4 width sweep flat 2^26, (%d,%d)" % (sp.k, sp.m), sp.n, [sp.w], "one hb_relu", ms,
                       hb.hb_opened_bits(True, sp.k, sp.m, 1), kernel_name(sp.w))
        del a, b, c, d
        big = []                                                  # cfg 5: 224x224 at batch 64, per-tensor (k, m)
        for sp in workloads.resnet18_imagenet():
            _, a, b = workloads.materialize_on_device(sp, dev)
            big.append((a, b, torch.empty_like(a), torch.empty_like(b), sp.k, sp.m, hb.hb_tensor_seed(ROOT_SEED, sp.tensor_id)))
        n_big = sum(t[0].numel() for t in big)
        big_batch = hb.make_batch(big)
        bits_big = hb.hb_relu_batch(big_batch) / n_big
        ms = _time_launches(lambda: hb.hb_relu_batch(big_batch), torch, 100.0, 150.0)
        widths5 = sorted({t[5] - t[4] for t in big})
        add_config("cfg5 resnet18 224x224 batch 64, per-tensor (k,m)", n_big, widths5,
                   "one hb_relu_batch (%d launches)" % len(widths5), ms, bits_big,
                   ", ".join(kernel_name(w, "relu", True) for w in widths5))
        del big, big_batch
        torch.cuda.empty_cache()

        # ---- side figures: the other entry points on the first tensor of the headline set -------------------
        def per_tensor_step():
            for (spec, a, b, c, d, seed) in tensors:
                hb.hb_relu(a, b, spec.k, spec.m, seed, c, d)
        ms = _time_launches(per_tensor_step, torch)
        extra["relu_w8_elems_per_s_one_launch_per_tensor"] = n_total / (ms * 1e-3)
        # the same set on the shared-mask dealer layout (3w opened bits per prefix round, 4 dealer words fewer per group)
        ms = _time_launches(lambda: hb.hb_relu_batch_ex(batch, hb.HB_DEALER_SHARED_MASK), torch)
        extra["relu_w8_shared_mask_elems_per_s"] = n_total / (ms * 1e-3)
        extra["relu_w8_shared_mask_hbm_frac"] = BYTES_PER_ELEMENT * n_total / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        extra["relu_w8_shared_mask_opened_bits_per_element"] = hb.hb_opened_bits_ex(True, k, m, 1, hb.HB_DEALER_SHARED_MASK)
        # three and four parties on the first tensor: 16 p bytes per element, (p - 1) adders
        for parties in (3, 4):
            more = [torch.randint(-(1 << 62), 1 << 62, (spec0.n,), dtype=torch.int64, device=dev)
                    for _ in range(parties - 2)]
            sh = [s0, s1] + more
            outs = [o0, o1] + [torch.empty_like(t) for t in more]
            ms = _time_launches(lambda: hb.hb_relu_mp(sh, k, m, seed0, outs), torch)
            extra["relu_mp%d_w8_elems_per_s" % parties] = spec0.n / (ms * 1e-3)
            extra["relu_mp%d_w8_hbm_frac" % parties] = 16 * parties * spec0.n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
            extra["relu_mp%d_w8_opened_bits_per_element_per_link" % parties] = hb.hb_opened_bits_mp(True, parties, k, m, 1)
            del more, sh, outs
        def drelu8():
            hb.hb_drelu(s0, s1, k, m, seed0, o0, o1)
        ms = _time_launches(drelu8, torch)
        extra["drelu_w8_shader_clock_mhz"] = _clock_under(drelu8, torch, probes, dev, ms)
        extra["drelu_w8_elems_per_s"] = spec0.n / (ms * 1e-3)
        extra["drelu_w8_hbm_frac"] = BYTES_PER_ELEMENT * spec0.n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        ms = _time_launches(lambda: hb.hb_open(s0, s1, False, out=o0), torch)
        extra["open_copy_ceiling_gbs"] = 24 * spec0.n / (ms * 1e-3) / 1e9
        ms = _time_launches(lambda: probes.stream_copy(s0, s1, o0, o1, True, False), torch)
        extra["stream_2in_2out_ceiling_gbs"] = 32 * spec0.n / (ms * 1e-3) / 1e9
        roofline["frac_of_2in_2out_copy_ceiling"] = achieved_gbs / extra["stream_2in_2out_ceiling_gbs"]
        roofline_w64["frac_of_2in_2out_copy_ceiling"] = gbs64 / extra["stream_2in_2out_ceiling_gbs"]
        ws = torch.empty(hb.hb_party_workspace_bytes(spec0.n, k, m), dtype=torch.uint8, device=dev)
        ms = _time_launches(lambda: hb.hb_relu_party(s0, s1, k, m, seed0, o0, o1, ws), torch)
        extra["relu_party_w8_elems_per_s"] = spec0.n / (ms * 1e-3)
        extra["relu_party_w8_bytes_per_element"] = party_path_bytes(spec0.n, k, m) / spec0.n
        extra["relu_party_w8_hbm_frac"] = party_path_bytes(spec0.n, k, m) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        extra["relu_party_w8_wire_bytes_per_element_per_party"] = 8 * hb.hb_party_wire_words(spec0.n, k, m) / spec0.n
        del ws
        xf = torch.randn(spec0.n, device=dev, dtype=torch.float32)
        yf = torch.empty_like(xf)
        ms = _time_launches(lambda: hb.hb_sim_relu_f32(xf, k, m, seed0, 1, yf), torch)
        extra["sim_relu_f32_w8_elems_per_s"] = spec0.n / (ms * 1e-3)       # 8 B per element; bound by VALU like hb_relu
        del xf, yf
        counts = torch.empty(64, dtype=torch.int64, device=dev)
        ms = _time_launches(lambda: hb.hb_eco_scan(s0, s1, counts), torch)
        extra["eco_scan_elems_per_s"] = spec0.n / (ms * 1e-3)
        extra["eco_scan_hbm_frac"] = 16 * spec0.n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS      # 16 B read per element
        extra["eco_scan_zero_error_m"] = hb.hb_eco_choose(counts)

    # ---- CPU baseline: the oracle as it stands on this machine's host cores, bounded samples ------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        cores = min(len(os.sched_getaffinity(0)), 16)
        sample = tensors[:2]                     # tensors 0 and 1 of the workload: 2 x 2^25 elements
        host = [(sp, a.cpu().numpy(), b.cpu().numpy(), sd) for (sp, a, b, _, _, sd) in sample]
        c0 = time.perf_counter()
        for (sp, a, b, sd) in host:
            oracle.evaluate(a, b, sp.k, sp.m, sd, oracle.WHAT_RELU, threads=cores)
        c1 = time.perf_counter()
        n_cpu = sum(sp.n for (sp, _, _, _) in host)
        sp, a, b, sd = host[0]
        n_one = 1 << 23                          # one thread on the first 2^23 elements of tensor 0
        d0 = time.perf_counter()
        oracle.evaluate(a[:n_one], b[:n_one], sp.k, sp.m, sd, oracle.WHAT_RELU, threads=1)
        d1 = time.perf_counter()
        cpu = {"value": n_cpu / (c1 - c0), "unit": "elements/s", "cores": cores, "kind": "oracle",
               "sample": "tensors 0-1 of the workload in full (%d elements), hb_relu at (12,20), "
                         "element range split over %d threads" % (n_cpu, cores),
               "one_core_value": n_one / (d1 - d0)}
        if not args.no_extra:
            n64 = 1 << 25                        # the whole first tensor at (0, 64)
            c0 = time.perf_counter()
            oracle.evaluate(a[:n64], b[:n64], 0, 64, sd, oracle.WHAT_RELU, threads=cores)
            c1 = time.perf_counter()
            n_one = 1 << 21
            d0 = time.perf_counter()
            oracle.evaluate(a[:n_one], b[:n_one], 0, 64, sd, oracle.WHAT_RELU, threads=1)
            d1 = time.perf_counter()
            cpu_w64 = {"value": n64 / (c1 - c0), "unit": "elements/s", "cores": cores, "kind": "oracle",
                       "sample": "tensor 0 of the workload in full (%d elements), hb_relu at (0,64), element range "
                                 "split over %d threads" % (n64, cores),
                       "one_core_value": n_one / (d1 - d0)}

    out = {
        "metric": "secret-shared ReLU elems/s at w=8 and w=64; % of HBM roofline",
        "value": value,
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {"workload": "resnet18_cifar32_relu_set_batch512_k12_m20 (17 tensors, 285,212,672 elements, w=8)",
                   "elements": n_total, "k": k, "m": m, "launches_per_step": 1, "tensors_per_step": len(tensors),
                   "root_seed": ROOT_SEED, "prewarm_s": 0.4},
        "roofline": roofline,
        "roofline_alu": roofline_alu,
        "roofline_w64": roofline_w64,
        "cpu_baseline": cpu,
        "cpu_baseline_w64": cpu_w64,
        "configs": configs,
        "extra": extra,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
