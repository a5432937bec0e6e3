#!/usr/bin/env python3
"""Benchmark of the secret-shared ReLU hot path on one MI355X.

A step is one pass of hb_relu over the headline workload: the 17 ReLU input tensors of ResNet18 on
3x32x32 images at batch 512 (285,212,672 elements, 2^16 fixed point, int64 shares), slice
(k, m) = (12, 20), every tensor with its own seed, issued through hb_relu_batch (one kernel launch for
the 17 tensors).  Inputs and outputs are resident in HBM before the timed region starts.  The GPU's clocks
ramp up over the first tens of milliseconds of load, so the default warm-up is 50 steps.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

ROOT_SEED = 0x2309048750000001
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
BYTES_PER_ELEMENT = 32         # two int64 shares read, two written

# HBM traffic of one launch of hb::tile_batch_kernel<8, relu> on this workload, from the rocprofv3 --pmc runs
# summarised in profiles/tile_batch_kernel_w8_relu_resnet18_b512.txt: FETCH_SIZE 2228395.7 KiB scaled by 2.0
# (what the counter under-reads for a plain streaming kernel of known size), WRITE_SIZE 4456448.1 KiB scaled by 1.0.
PROFILED_TRAFFIC_BYTES = (2228395.7 * 2.0 + 4456448.1 * 1.0) * 1024.0
PROFILED_ELEMENTS = 285212672
# Vector-ALU instructions per wavefront of the same kernel (SQ_INSTS_VALU / SQ_WAVES, profiles/
# tile_kernel_w8_w64_valu_counters.txt); a wavefront covers 512 elements.
VALU_INSTS_PER_WAVE = 2069.6
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9      # CUs x SIMDs x lanes per clock x 2.4 GHz = 39.3e12 32-bit lane-ops/s


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


def _time_launches(fn, reps, torch):
    """Average duration in ms of `fn` (one launch) over `reps` launches, by events on the current stream."""
    for _ in range(max(1, reps // 2)):      # same load beforehand, so the clocks have settled
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the side measurements (profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (both parties are simulated on it; there is no "
                 "sharded or multi-rank path) -- run with --gpus 1")

    import torch
    from paper_2309_04875_amd import hb, workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    hb.load()   # fails loudly when the HIP library has not been built
    dev = "cuda:0"
    torch.cuda.set_device(0)

    # ---- inputs resident in HBM ------------------------------------------------------------
    specs = workloads.resnet18_cifar_batch512()
    tensors = []
    for spec in specs:
        _, s0, s1 = workloads.materialize_on_device(spec, dev)
        tensors.append((spec, s0, s1, torch.empty_like(s0), torch.empty_like(s1),
                        hb.hb_tensor_seed(ROOT_SEED, spec.tensor_id)))
    n_total = sum(s.n for s in specs)
    k, m = specs[0].k, specs[0].m
    torch.cuda.synchronize()

    batch = hb.make_batch([(s0, s1, o0, o1, spec.k, spec.m, seed) for (spec, s0, s1, o0, o1, seed) in tensors])

    def step():
        return hb.hb_relu_batch(batch)

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
    kernel_ms_per_step = avg_launch_ms
    bytes_per_launch = BYTES_PER_ELEMENT * n_total
    achieved_gbs = bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
    valu_lane_ops = VALU_INSTS_PER_WAVE * 64.0 * (n_total / 512.0)     # instructions x lanes x wavefronts

    # ---- the shader clock the GPU sustains under this kernel: a one-wavefront probe on a second stream while
    # steps of the workload run (the board is power-limited under this load; nominal clock 2.4 GHz) -----------
    def clock_under(load_fn, launches):
        side = torch.cuda.Stream()
        stamps = torch.zeros(2, dtype=torch.int64, device=dev)
        torch.cuda.synchronize()
        for _ in range(launches):
            load_fn()
        with torch.cuda.stream(side):
            hb.hb_clock_probe(3000, stamps)
        for _ in range(launches):
            load_fn()
        torch.cuda.synchronize()
        ticks = stamps.cpu().tolist()
        return 100.0 * ticks[0] / max(ticks[1], 1)

    core_clock_mhz = clock_under(step, 3) if not args.no_extra else None

    # ---- side figures, outside the timed region ---------------------------------------------
    spec0, s0, s1, o0, o1, seed0 = tensors[0]
    extra = {"opened_bits_per_element": opened / n_total,
             "opened_bits_vs_64bit_baseline": hb.BASELINE_BITS_PER_ELEMENT / (opened / n_total)}
    if not args.no_extra:
        def per_tensor_step():
            for (spec, a, b, c, d, seed) in tensors:
                hb.hb_relu(a, b, spec.k, spec.m, seed, c, d)
        ms = _time_launches(per_tensor_step, 40, torch)
        extra["relu_w8_elems_per_s_one_launch_per_tensor"] = n_total / (ms * 1e-3)
        # the same set on the shared-mask dealer layout (3w opened bits per prefix round, 4 dealer words fewer per group)
        ms = _time_launches(lambda: hb.hb_relu_batch_ex(batch, hb.HB_DEALER_SHARED_MASK), 60, torch)
        extra["relu_w8_shared_mask_elems_per_s"] = n_total / (ms * 1e-3)
        extra["relu_w8_shared_mask_hbm_frac"] = BYTES_PER_ELEMENT * n_total / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        extra["relu_w8_shared_mask_opened_bits_per_element"] = hb.hb_opened_bits_ex(True, k, m, 1, hb.HB_DEALER_SHARED_MASK)
        # three and four parties on the first tensor: 16 p bytes per element, (p - 1) adders
        for parties in (3, 4):
            more = [torch.randint(-(1 << 62), 1 << 62, (spec0.n,), dtype=torch.int64, device=dev)
                    for _ in range(parties - 2)]
            sh = [s0, s1] + more
            outs = [o0, o1] + [torch.empty_like(t) for t in more]
            ms = _time_launches(lambda: hb.hb_relu_mp(sh, k, m, seed0, outs), 40, torch)
            extra["relu_mp%d_w8_elems_per_s" % parties] = spec0.n / (ms * 1e-3)
            extra["relu_mp%d_w8_hbm_frac" % parties] = 16 * parties * spec0.n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
            extra["relu_mp%d_w8_opened_bits_per_element_per_link" % parties] = hb.hb_opened_bits_mp(True, parties, k, m, 1)
            del more, sh, outs
        ms = _time_launches(lambda: hb.hb_relu(s0, s1, 0, 64, seed0, o0, o1), 60, torch)
        extra["relu_w64_elems_per_s"] = spec0.n / (ms * 1e-3)
        extra["relu_w64_hbm_frac"] = BYTES_PER_ELEMENT * spec0.n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        ms = _time_launches(lambda: hb.hb_drelu(s0, s1, k, m, seed0, o0, o1), 300, torch)
        extra["drelu_w8_shader_clock_mhz"] = clock_under(lambda: hb.hb_drelu(s0, s1, k, m, seed0, o0, o1), 40)
        extra["drelu_w8_elems_per_s"] = spec0.n / (ms * 1e-3)
        extra["drelu_w8_hbm_frac"] = BYTES_PER_ELEMENT * spec0.n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        ms = _time_launches(lambda: hb.hb_open(s0, s1, False, out=o0), 300, torch)
        extra["open_copy_ceiling_gbs"] = 24 * spec0.n / (ms * 1e-3) / 1e9
        ws = torch.empty(hb.hb_party_workspace_bytes(spec0.n, k, m), dtype=torch.uint8, device=dev)
        ms = _time_launches(lambda: hb.hb_relu_party(s0, s1, k, m, seed0, o0, o1, ws), 40, torch)
        extra["relu_party_w8_elems_per_s"] = spec0.n / (ms * 1e-3)
        extra["relu_party_w8_bytes_per_element"] = party_path_bytes(spec0.n, k, m) / spec0.n
        extra["relu_party_w8_hbm_frac"] = party_path_bytes(spec0.n, k, m) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        extra["relu_party_w8_wire_bytes_per_element_per_party"] = 8 * hb.hb_party_wire_words(spec0.n, k, m) / spec0.n
        del ws
        xf = torch.randn(spec0.n, device=dev, dtype=torch.float32)
        yf = torch.empty_like(xf)
        ms = _time_launches(lambda: hb.hb_sim_relu_f32(xf, k, m, seed0, 1, yf), 100, torch)
        extra["sim_relu_f32_w8_elems_per_s"] = spec0.n / (ms * 1e-3)       # 8 B per element; bound by VALU like hb_relu
        del xf, yf
        # the one-image set (17 tensors, 557,056 elements, per-tensor (k, m)) is launch-bound: per-tensor calls, the
        # batched call (one launch per distinct width) and the batched call replayed from a HIP graph
        small = []
        for spec in workloads.resnet18_cifar():
            _, a, b = workloads.materialize_on_device(spec, dev)
            small.append((a, b, torch.empty_like(a), torch.empty_like(b), spec.k, spec.m,
                          hb.hb_tensor_seed(ROOT_SEED, spec.tensor_id)))
        n_small = sum(t[0].numel() for t in small)
        small_batch = hb.make_batch(small)
        ms = _time_launches(lambda: [hb.hb_relu(a, b, kk, mm, sd, c, d) for (a, b, c, d, kk, mm, sd) in small], 200, torch)
        extra["one_image_set_us_per_tensor_calls"] = ms * 1e3
        ms = _time_launches(lambda: hb.hb_relu_batch(small_batch), 200, torch)
        extra["one_image_set_us_batched_call"] = ms * 1e3
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                hb.hb_relu_batch(small_batch)
        torch.cuda.synchronize()
        ms = _time_launches(graph.replay, 200, torch)
        extra["one_image_set_us_graph_replay"] = ms * 1e3
        extra["one_image_set_elements"] = n_small
        del graph, small, small_batch
        counts = torch.empty(64, dtype=torch.int64, device=dev)
        ms = _time_launches(lambda: hb.hb_eco_scan(s0, s1, counts), 300, torch)
        extra["eco_scan_elems_per_s"] = spec0.n / (ms * 1e-3)
        extra["eco_scan_hbm_frac"] = 16 * spec0.n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS      # 16 B read per element
        extra["eco_scan_zero_error_m"] = hb.hb_eco_choose(counts)

    # ---- CPU baseline: the oracle as it stands on this machine's host cores, bounded sample ------
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
                   "root_seed": ROOT_SEED},
        # The kernel is bound by vector-ALU instruction issue (VALUBusy 99 %), not by HBM: `roofline` prices the launch
        # against the chip's 32-bit integer lane-op rate (instructions per wavefront from SQ_INSTS_VALU / SQ_WAVES);
        # `roofline_hbm` is the same launch against the HBM peak, the fraction the metric names.
        "roofline": {"bound": "alu", "achieved": valu_lane_ops / (avg_launch_ms * 1e-3) / 1e12,
                     "peak": VALU_PEAK_LANE_OPS / 1e12, "unit": "T lane-ops/s",
                     "frac": valu_lane_ops / (avg_launch_ms * 1e-3) / VALU_PEAK_LANE_OPS,
                     "traffic": PROFILED_TRAFFIC_BYTES if n_total == PROFILED_ELEMENTS else None,
                     "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)",
                     "kernel": "hb::tile_batch_kernel<8, relu>",
                     "avg_launch_ms": avg_launch_ms, "kernel_ms_per_step": kernel_ms_per_step,
                     "valu_lane_ops_per_element": VALU_INSTS_PER_WAVE / 8.0,
                     "valu_lane_ops_per_launch": valu_lane_ops,
                     "peak_derivation": "256 CUs x 4 SIMDs x 16 lanes per clock x 2.4 GHz",
                     "shader_clock_mhz_under_this_kernel": core_clock_mhz},
        "roofline_hbm": {"bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": achieved_gbs / HBM_PEAK_GBS,
                         "traffic": PROFILED_TRAFFIC_BYTES if n_total == PROFILED_ELEMENTS else None,
                         "algorithmic_bytes_per_launch": bytes_per_launch,
                         "algorithmic_bytes_per_element": BYTES_PER_ELEMENT},
        "cpu_baseline": cpu,
        "extra": extra,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
