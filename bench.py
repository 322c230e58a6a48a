#!/usr/bin/env python3
"""One-GPU benchmark of the SpC layer hot path (pack+sort -> feature-row permutation ->
kernel-map build -> weight re-layout -> feature computation) on synthetic clouds.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--dataflow os|ws]

A "step" is one pass of the whole path over one cloud, inputs already resident in HBM.
Prints ONE JSON line (see the keys below); `value` is whole-path throughput in
Mvoxel-offsets/s = |V_q| * K^3 / step time.  Per-phase numbers, the roofline of the
dominant kernel and the CPU oracle timed on the host cores ride along.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0   # MI355X dense fp16/bf16 MFMA
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E
PEAK_FP32_TFLOPS = 157.3


def _recorded_traffic(cfg: int, kernel: str):
    """HBM bytes per launch of the dominant kernel, as measured by the rocprofv3 --pmc runs whose
    summary is kept under profiles/ (a line 'traffic_bytes_per_launch <kernel> <bytes>')."""
    path = os.path.join(ROOT, "profiles", "cfg%d_pmc_traffic.txt" % cfg)
    try:
        with open(path) as f:
            for line in f:
                t = line.split()
                if len(t) == 3 and t[0] == "traffic_bytes_per_launch" and t[1] == kernel:
                    return float(t[2])
    except OSError:
        pass
    return None


def measured_peaks(torch, B) -> dict:
    """The machine's own denominators, next to the data-sheet ones: a plain copy kernel over 1 GiB (read + write
    bytes per second) and a register-resident fp16 MFMA loop on every wave of the chip."""
    dev = torch.device("cuda:0")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    best_copy, best_mfma = 0.0, 0.0
    for rep in range(4):
        a, b = ev(), ev()
        a.record()
        nbytes = B.spc_probe_copy(src, dst)
        b.record()
        torch.cuda.synchronize()
        if rep:
            best_copy = max(best_copy, 2.0 * nbytes / (a.elapsed_time(b) * 1e-3) / 1e9)
        a, b = ev(), ev()
        a.record()
        flops = B.spc_probe_mfma(20000, sink)
        b.record()
        torch.cuda.synchronize()
        if rep:
            best_mfma = max(best_mfma, flops / (a.elapsed_time(b) * 1e-3) / 1e12)
    return {"copy_kernel_GBps": best_copy, "mfma_f16_loop_TFLOPs": best_mfma,
            "datasheet": {"hbm_GBps": PEAK_HBM_GBS, "mfma_f16_TFLOPs": PEAK_MFMA_F16_TFLOPS}}


def bench_network(args, torch, B, synth) -> int:
    """Configuration 4: the 25-layer UNet-style stack.  A step = pack+sort, feature-row permutation,
    network-wide kernel-map build on HIP streams, and the 25 feature computations."""
    from paper_2511_20834_amd.network import SpcNetwork
    dev = torch.device("cuda:0")
    coords_np = synth.cloud("lidar")
    n = coords_np.shape[0]
    layers = synth.unet_layers()
    W_np = synth.unet_weights(layers)
    F_np = synth.features(n, 4, np.float16, seed=synth.SEED_BASE + 300)
    desc = B.spc_pack_desc_fit(coords_np[:, 1:].min(0), coords_np[:, 1:].max(0), 1, 16, 16)
    coords = torch.from_numpy(coords_np).to(dev)
    F_raw = torch.from_numpy(F_np).to(dev)
    net = SpcNetwork(layers, [torch.from_numpy(w).to(dev) for w in W_np], dataflow=B.DATAFLOW_OS)
    ws = torch.empty(B.spc_pack_workspace_bytes(n, desc), dtype=torch.uint8, device=dev)
    keys = torch.empty(n, dtype=torch.int32, device=dev)
    perm = torch.empty(n, dtype=torch.int32, device=dev)
    F = torch.empty_like(F_raw)
    # the timed graph uses the pipelined builder (levels on one stream, searches on another, layers wait for their
    # own map: 0.485 ms per step); the join-all builder took 0.544 ms on two streams, 0.566 on four, 0.60 on one
    streams = [torch.cuda.current_stream(), torch.cuda.Stream(), torch.cuda.Stream()]
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(flags=0, marks=None, forward=True, keep=False):
        if marks:
            marks[0].record()
        B.spc_pack_coords(coords, desc, True, 0, None, ws, keys, perm)
        B.spc_permute_rows(F_raw, perm, F)
        if marks:
            marks[1].record()
        net.build_maps(keys, desc, streams, flags)
        if marks:
            marks[2].record()
        y = net.forward(F) if forward else None
        if marks:
            marks[3].record()
        y = y.clone() if keep else None
        net.destroy_maps()
        return y

    # sizes (fetched once; they do not change between steps)
    B.spc_pack_coords(coords, desc, True, 0, None, ws, keys, perm)
    maps = net.build_maps(keys, desc, streams)
    vo = sum(m.n_out * m.kvol for m in maps)
    flops = sum(2.0 * float(m.nnz().sum()) * l["cin"] * l["cout"] for m, l in zip(maps, layers))
    level_sizes = sorted({(l["in_stride"], m.n_in if not l["transposed"] else m.n_out) for m, l in zip(maps, layers)})
    net.destroy_maps()
    tuned = None
    if args.tune:
        # one-time tuning of the per-layer dataflow threshold on this cloud (not part of a step)
        B.spc_permute_rows(F_raw, perm, F)
        t0 = time.perf_counter()
        rows = net.tune(keys, desc, F)
        tuned = {"seconds": time.perf_counter() - t0,
                 "layers": {name: {"best_t": best, "us": {str(t): round(v, 1) for t, v in times.items()}} for name, best, times in rows}}
    def timed(fn, reps):
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    # ---- eager launches: the host enqueues ~150 kernels and as many event operations per step
    for _ in range(args.warmup):
        step()
    part = {"eager_ms_per_step": timed(step, args.steps)}
    for name, flags in (("streams", 0), ("sequential", B.NET_SEQUENTIAL)):
        marks = [[ev() for _ in range(4)] for _ in range(min(args.steps, 30))]
        for m in marks:
            step(flags, m)
        torch.cuda.synchronize()
        part["eager_build_ms_" + name] = float(np.mean([m[1].elapsed_time(m[2]) for m in marks]))
        part["eager_forward_ms"] = float(np.mean([m[2].elapsed_time(m[3]) for m in marks]))
        part["pack_sort_permute_ms"] = float(np.mean([m[0].elapsed_time(m[1]) for m in marks]))

    # ---- the same step recorded once into a HIP graph and replayed (the timed configuration)
    caps = {}
    for name, flags in (("streams", B.NET_PIPELINED), ("sequential", B.NET_SEQUENTIAL)):
        caps[name] = net.capture_step(coords, F_raw, desc, streams[1:], flags)
        for _ in range(args.warmup):
            caps[name].replay()
        part["graph_ms_per_step_" + name] = timed(caps[name].replay, args.steps)
    ms_per_step = part["graph_ms_per_step_streams"]
    part["graph_speedup_streams_over_sequential"] = part["graph_ms_per_step_sequential"] / ms_per_step
    # the replayed step must reproduce the eager step bit for bit
    y_eager = step(keep=True)
    torch.cuda.synchronize()
    caps["streams"].replay()
    torch.cuda.synchronize()
    part["graph_equals_eager"] = bool(torch.equal(caps["streams"].output[:caps["streams"].n_out()], y_eager))
    part["forward_useful_TFLOPs"] = flops / (part["eager_forward_ms"] * 1e-3) / 1e12
    # ---- serving view: independent scenes in flight, one captured single-stream step per scene, replayed
    # round-robin on the scenes' own streams (most layers of the stack are too small to fill the chip alone)
    if args.scene_streams > 1:
        scenes = []
        try:  # an extra view: a failure here must not cost the headline line
            scenes = [net.capture_step(coords, F_raw, desc, None, B.NET_SEQUENTIAL) for _ in range(args.scene_streams)]
            ok = True
            for rep in range(2):
                for sc in scenes:
                    sc.output.zero_()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for i in range(args.steps):
                    sc = scenes[i % len(scenes)]
                    with torch.cuda.stream(sc.stream):
                        sc.replay()
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                ok = ok and all(bool(torch.equal(sc.output[:sc.n_out()], y_eager)) for sc in scenes[:min(len(scenes), args.steps)])
            part["scenes_in_flight"] = {"streams": len(scenes), "ms_per_step": dt * 1e3 / args.steps,
                                        "value": vo * args.steps / dt / 1e6, "equals_one_at_a_time": ok}
        except Exception as e:  # noqa: BLE001
            part["scenes_in_flight"] = {"error": "%s: %s" % (type(e).__name__, e)}
        torch.cuda.synchronize()
        for sc in scenes:
            sc.destroy()
    result = {
        "metric": "SpC UNet-style stack (pack+sort, network-wide kmap build, 25 feature layers) Mvoxel-offsets/s",
        "value": vo / (ms_per_step * 1e-3) / 1e6, "unit": "Mvoxel-offsets/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "cfg4: lidar cloud, %d voxels, 25-layer UNet-style stack, 13 kernel maps built pipelined on 2 streams, OS dataflow, "
                               "step replayed from a HIP graph" % n,
                   "n_voxels": n, "levels": level_sizes, "voxel_offsets": vo, "useful_flops": flops},
        "parts": part, "tuning": tuned,
        "roofline": {"kernel": "conv_os_splitk_kernel + conv_os_phase_kernel (all 25 layers)", "bound": "mfma",
                     "achieved": part["forward_useful_TFLOPs"],
                     "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s", "frac": part["forward_useful_TFLOPs"] / PEAK_MFMA_F16_TFLOPS,
                     "traffic": None},
    }
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, choices=[0, 1, 2, 3, 4])
    ap.add_argument("--dataflow", default="auto", choices=["auto", "os", "ws"])
    ap.add_argument("--hybrid-t", type=int, default=None,
                    help="single-layer configurations: threshold of the hybrid dual dataflow (offsets with L1 norm < t run "
                         "output-stationary, the others weight-stationary); --config 4: ignored")
    ap.add_argument("--sym", action="store_true",
                    help="single-layer configurations with --dataflow ws: build the symmetric half-map (submanifold layers)")
    ap.add_argument("--voxels", type=int, default=0,
                    help="single-layer configurations: replace the configuration's cloud by a uniformly random scene of this many "
                         "voxels in a [n, n, 200] volume at 1.25 %% density (the random-scene size sweep)")
    ap.add_argument("--tune", action="store_true", help="--config 4: tune the per-layer threshold on the cloud first and report it")
    ap.add_argument("--key-bits", type=int, default=0, choices=[0, 64],
                    help="configs 0-3: 64 forces 64-bit packed keys (default: 32 bits when the scene fits)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--scene-streams", type=int, default=3,
                    help="configs 0-3: also time independent scenes in flight on this many streams (0 or 1: skip)")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the copy-kernel and MFMA-loop measurements of the machine's own peaks")
    ap.add_argument("--copy-probe-mb", type=int, default=0,
                    help="run one plain device copy of this many MiB before the warm-up (calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2511_20834_amd import binding as B
    from paper_2511_20834_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    if args.config == 4:
        return bench_network(args, torch, B, synth)
    cfg = synth.CONFIGS[args.config]
    K, s_l, cin, cout = cfg["K"], cfg["layer_stride"], cfg["cin"], cfg["cout"]
    K3 = K ** 3
    tdt = {"f32": torch.float32, "f16": torch.float16}[cfg["dtype"]]
    coords_np = synth.scaled_random_cloud(args.voxels) if args.voxels > 0 else synth.cloud(cfg["cloud"])
    n = coords_np.shape[0]
    F_np, W_np = synth.layer_tensors(args.config, n)
    dataflow = {"os": B.DATAFLOW_OS, "ws": B.DATAFLOW_WS}.get(args.dataflow)
    if dataflow is None:
        dataflow = B.DATAFLOW_OS  # with per-block offset skipping OS wins on all four single-layer configurations
    layout = B.LAYOUT_OS if dataflow == B.DATAFLOW_OS else B.LAYOUT_WS
    if args.hybrid_t is not None:
        layout = B.LAYOUT_BOTH
    if args.sym:
        layout |= B.LAYOUT_WS_SYM

    lo, hi = coords_np[:, 1:].min(0), coords_np[:, 1:].max(0)
    reach = ((K - 1) // 2) if K % 2 else (K - 1)
    desc = B.spc_pack_desc_fit(lo, hi, int(coords_np[:, 0].max()) + 1, s_l, reach, args.key_bits)

    dev = torch.device("cuda:0")
    coords = torch.from_numpy(coords_np).to(dev)
    F_raw = torch.from_numpy(F_np).to(dev)
    W = torch.from_numpy(W_np).to(dev)
    ws = torch.empty(B.spc_pack_workspace_bytes(n, desc), dtype=torch.uint8, device=dev)
    keys = torch.empty(n, dtype=torch.int32 if desc.key_bits == 32 else torch.int64, device=dev)
    perm = torch.empty(n, dtype=torch.int32, device=dev)
    use_packed = tdt != torch.float32 and cin % 16 == 0 and cout in (32, 64, 128, 256)
    Wp = torch.empty_like(W)

    # sizes that only exist after a first build (strided layers produce |V_q| on the device)
    B.spc_pack_coords(coords, desc, True, 0, None, ws, keys, perm)
    km0 = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout)
    n_out = km0.n_out
    nnz = int(km0.nnz().sum())
    km0.destroy()
    out = torch.empty((n_out, cout), dtype=tdt, device=dev)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    phases = ("pack_sort", "kmap_build", "conv")
    # Weights are constant during inference: their re-layout into MFMA operand order is done once,
    # like loading the model, and is not part of a step.
    if use_packed:
        B.spc_conv_prepare_weights(W, Wp)
    conv_flags = B.CONV_PACKED_WEIGHTS if use_packed else 0
    F_sorted = torch.empty_like(F_raw) if args.sym else None

    def step(marks=None):
        """One layer on one cloud: pack + sort the coordinates, build the kernel map (with the sort
        permutation folded in, so the feature rows are gathered from the caller's order), features."""
        if marks is not None:
            marks[0].record()
        B.spc_pack_coords(coords, desc, True, 0, None, ws, keys, perm)
        if marks is not None:
            marks[1].record()
        if args.sym:  # a symmetric half-map numbers inputs and outputs alike: the feature rows are moved instead
            B.spc_permute_rows(F_raw, perm, F_sorted)
            km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout)
        else:
            km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout, in_perm=perm)
        if marks is not None:
            marks[2].record()
        B.spc_conv_forward(km, F_sorted if args.sym else F_raw, Wp if use_packed else W, dataflow, conv_flags, out=out,
                           hybrid_t=args.hybrid_t)
        if marks is not None:
            marks[3].record()
        km.destroy()

    if args.copy_probe_mb > 0:
        # plain copy kernel (probe_copy_kernel): reads and writes a known byte count
        src = torch.ones(args.copy_probe_mb * 1024 * 1024 // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        B.spc_probe_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps, no per-phase events inside
    t0 = time.perf_counter()
    e_start, e_end = ev(), ev()
    e_start.record()
    for _ in range(args.steps):
        step()
    e_end.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = max(e_start.elapsed_time(e_end), 0.0) / args.steps
    ms_per_step_wall = wall * 1e3 / args.steps

    # ---- per-phase durations (separate pass: events between the calls, same stream)
    n_prof = min(args.steps, 50)
    marks = [[ev() for _ in range(4)] for _ in range(n_prof)]
    for i in range(n_prof):
        step(marks[i])
    torch.cuda.synchronize()
    phase_ms = {p: float(np.mean([marks[i][j].elapsed_time(marks[i][j + 1]) for i in range(n_prof)]))
                for j, p in enumerate(phases)}

    # ---- each phase alone, 20 invocations back to back between two events (the launch of one hides under the
    # kernels of the one before): the rate the phase sustains, beside the duration it has inside a step
    def back_to_back(fn, reps=20, rounds=3):
        best = float("inf")
        for _ in range(rounds):
            a, b = ev(), ev()
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b) / reps)
        return best

    def build_once():
        if args.sym:
            B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout).destroy()
        else:
            B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout, in_perm=perm).destroy()

    B.spc_pack_coords(coords, desc, True, 0, None, ws, keys, perm)
    km_b = (B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout) if args.sym
            else B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout, in_perm=perm))
    loop_ms = {
        "pack_sort": back_to_back(lambda: B.spc_pack_coords(coords, desc, True, 0, None, ws, keys, perm)),
        "kmap_build": back_to_back(build_once),
        "conv": back_to_back(lambda: B.spc_conv_forward(km_b, F_sorted if args.sym else F_raw, Wp if use_packed else W, dataflow,
                                                        conv_flags, out=out, hybrid_t=args.hybrid_t)),
    }
    km_b.destroy()

    voxel_offsets = n_out * K3
    flops = 2.0 * nnz * cin * cout
    value = voxel_offsets / (ms_per_step * 1e-3) / 1e6
    conv_tflops = flops / (phase_ms["conv"] * 1e-3) / 1e12
    key_b = desc.key_bits // 8
    if layout == B.LAYOUT_OS:
        map_bytes = n * key_b + n_out * key_b + n_out * K3 * 4
    else:
        map_bytes = n * key_b + n_out * key_b + nnz * 8 + K3 * 4
    kmap_gbs = map_bytes / (phase_ms["kmap_build"] * 1e-3) / 1e9
    # compulsory bytes of the feature kernel: every input and output row once, the weights once, the map once
    elt = 4 if tdt == torch.float32 else 2
    conv_bytes = (n * cin + n_out * cout + K3 * cin * cout) * elt + (n_out * K3 * 4 if layout == B.LAYOUT_OS else nnz * 8)
    conv_gbs = conv_bytes / (phase_ms["conv"] * 1e-3) / 1e9
    if tdt == torch.float32:
        roof = {"kernel": "conv_%s_simple_kernel" % ("os" if dataflow == B.DATAFLOW_OS else "ws"), "bound": "alu",
                "achieved": conv_tflops, "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s",
                "frac": conv_tflops / PEAK_FP32_TFLOPS, "traffic": None}
    else:
        # the library's choice between its two OS kernels (prefer_splitk in csrc/conv.hip): the split-k kernel for
        # kernels larger than 4x4x4, for layers whose tiles fill fewer than 64 phase workgroups (16 row blocks
        # each, per slab of 64 or 32 output channels), and for layers with little work behind every tile
        n_slabs = cout // 64 if cout % 64 == 0 else cout // 32
        phase_wgs = ((n_out + 31) // 32 + 15) // 16 * n_slabs
        splitk = K3 > 64 or phase_wgs < 64 or cout % 64 != 0 or phase_wgs * cin < 7000
        os_kernel = "conv_os_splitk_kernel" if splitk else "conv_os_phase_kernel"
        kname = os_kernel if dataflow == B.DATAFLOW_OS else "conv_ws_mfma_kernel"
        # Which roof binds: the layer's arithmetic intensity (useful flops per compulsory byte) against the machine
        # balance (2.5 PFLOP/s / 8 TB/s = 312 flop/B).  Below it the HBM roof is the nearer one and is the one
        # reported; the other roof's fraction rides along in "parts".  Both use the duration of the feature phase
        # measured with HIP events on the launch stream (the kernel plus its launch; the kernel's own duration from
        # rocprofv3 is in profiles/).
        intensity = flops / conv_bytes
        if intensity < PEAK_MFMA_F16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            roof = {"kernel": kname, "bound": "hbm", "achieved": conv_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": conv_gbs / PEAK_HBM_GBS, "traffic": None}
        else:
            roof = {"kernel": kname, "bound": "mfma", "achieved": conv_tflops, "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
                    "frac": conv_tflops / PEAK_MFMA_F16_TFLOPS, "traffic": None}
        roof["flop_per_byte"] = intensity
        roof["timed"] = "feature phase, HIP events on the launch stream, mean of %d steps" % n_prof

    # the counters were taken on the configuration's own cloud, dataflow and key width
    own_workload = args.voxels <= 0 and dataflow == B.DATAFLOW_OS and args.hybrid_t is None and desc.key_bits == 32
    roof["traffic"] = _recorded_traffic(args.config, roof["kernel"]) if own_workload else None

    result = {
        "metric": "SpC layer hot path (pack+sort, kmap build, feature computation) Mvoxel-offsets/s",
        "value": value, "unit": "Mvoxel-offsets/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_wall": ms_per_step_wall, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": "cfg%d: %s cloud, %d voxels -> %d outputs, K=%d, layer stride %d, C %d->%d, %s, dataflow %s"
                   % (args.config, "uniform random" if args.voxels > 0 else cfg["cloud"], n, n_out, K, s_l, cin, cout, cfg["dtype"],
                      ("hybrid t=%d" % args.hybrid_t) if args.hybrid_t is not None else
                      ("OS" if dataflow == B.DATAFLOW_OS else "WS")),
                   "n_voxels": n, "n_out": n_out, "K": K, "cin": cin, "cout": cout, "nnz": nnz,
                   "key_bits": desc.key_bits},
        "parts": {"phase_ms": phase_ms, "phase_back_to_back_ms": loop_ms,
                  "kmap_build_back_to_back_frac_of_hbm_peak": map_bytes / (loop_ms["kmap_build"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                  "kmap_build_Mvoxel_offsets_per_s": voxel_offsets / (phase_ms["kmap_build"] * 1e-3) / 1e6,
                  "kmap_build_algorithmic_GBps": kmap_gbs, "kmap_build_frac_of_hbm_peak": kmap_gbs / PEAK_HBM_GBS,
                  "conv_useful_TFLOPs": conv_tflops, "conv_frac_of_mfma_peak": conv_tflops / PEAK_MFMA_F16_TFLOPS,
                  "conv_compulsory_GBps": conv_gbs, "conv_frac_of_hbm_peak": conv_gbs / PEAK_HBM_GBS},
        "roofline": roof,
    }

    # ---- serving view: independent scenes in flight.  Each stream owns a copy of the inputs, its buffers and a
    # captured graph of the same step; replays go round-robin over the streams, so the latency-bound sort and
    # search kernels of one scene run next to the feature kernel of another.  Reported beside the headline, which
    # stays the one-scene-at-a-time number.
    # (the step can be captured when the library's own sort runs: up to 8 Mi voxels, see include/spc.h)
    capturable = n <= 8192 * 1024
    if args.scene_streams > 1 and capturable and dataflow == B.DATAFLOW_OS and not args.sym and args.hybrid_t is None:
        class Scene:
            def __init__(self):
                self.coords, self.F = coords.clone(), F_raw.clone()
                self.ws, self.keys, self.perm, self.out = (torch.empty_like(ws), torch.empty_like(keys),
                                                           torch.empty_like(perm), torch.empty_like(out))
                self.stream, self.maps, self.graph = torch.cuda.Stream(), [], None

            def step(self, keep):
                B.spc_pack_coords(self.coords, desc, True, 0, None, self.ws, self.keys, self.perm)
                km = B.spc_build_kmap(self.keys, desc, K, 1, s_l, 0, layout, in_perm=self.perm)
                B.spc_conv_forward(km, self.F, Wp if use_packed else W, dataflow, conv_flags, out=self.out)
                if keep:
                    self.maps.append(km)  # the graph's kernels use the map's buffers
                else:
                    km.destroy()

            def capture(self):
                with torch.cuda.stream(self.stream):
                    self.step(False)
                torch.cuda.synchronize()
                self.graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(self.graph, stream=self.stream, capture_error_mode="relaxed"):
                    self.step(True)
                torch.cuda.synchronize()

        scenes = []
        try:  # an extra view: a failure here must not cost the headline line
            scenes = [Scene() for _ in range(args.scene_streams)]
            for sc in scenes:
                sc.capture()
            expect = out.clone()
            ok = True
            for rep in range(2):  # replays are checked against the eager result, twice, with cleared outputs
                for sc in scenes:
                    sc.out.zero_()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for i in range(args.steps):
                    sc = scenes[i % len(scenes)]
                    with torch.cuda.stream(sc.stream):
                        sc.graph.replay()
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                ok = ok and all(bool(torch.equal(sc.out, expect)) for sc in scenes[:min(len(scenes), args.steps)])
            result["parts"]["scenes_in_flight"] = {"streams": len(scenes), "ms_per_step": dt * 1e3 / args.steps,
                                                   "value": voxel_offsets * args.steps / dt / 1e6,
                                                   "equals_one_at_a_time": ok}
        except Exception as e:  # noqa: BLE001
            result["parts"]["scenes_in_flight"] = {"error": "%s: %s" % (type(e).__name__, e)}
        torch.cuda.synchronize()
        for sc in scenes:
            sc.graph = None
            for km in sc.maps:
                km.destroy()

    if not args.no_check:
        import oracle
        cs, operm = oracle.sort_coords(coords_np)
        oc, M = oracle.layer(cs, K, 1, s_l)
        rows = np.random.default_rng(0).choice(n_out, size=min(n_out, 512), replace=False)
        ref = oracle.conv(M[rows], F_np[operm].astype(np.float64), W_np.astype(np.float64))
        got = out[torch.from_numpy(rows).to(dev)].cpu().double().numpy()
        err = float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))
        result["check"] = {"rows": int(len(rows)), "max_rel_err": err, "ok": bool(err <= (1e-5 if tdt == torch.float32 else 1e-2))}

    if not args.no_peaks:
        result["parts"]["peaks_measured"] = measured_peaks(torch, B)

    if not args.no_cpu_baseline:
        import oracle
        F64, W64 = F_np.astype(np.float64), W_np.astype(np.float64)
        best = None
        t_all = time.perf_counter()
        reps = 0
        while reps < 3 or (time.perf_counter() - t_all < 10.0 and reps < 20):
            t = time.perf_counter()
            cs, operm = oracle.sort_coords(coords_np)
            oc, M = oracle.layer(cs, K, 1, s_l)
            oracle.conv(M, F64[operm], W64)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
            reps += 1
        result["cpu_baseline"] = {"value": len(oc) * K3 / best / 1e6, "unit": "Mvoxel-offsets/s",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": "whole workload (sort + hash-map kernel map + fp64 features), best of %d runs" % reps,
                                  "seconds": best}
        # the same on one thread (one run; the sort is single-threaded either way)
        threads = oracle.num_threads()
        oracle.set_threads(1)
        t = time.perf_counter()
        cs, operm = oracle.sort_coords(coords_np)
        oc, M = oracle.layer(cs, K, 1, s_l)
        oracle.conv(M, F64[operm], W64)
        one = time.perf_counter() - t
        oracle.set_threads(threads)
        result["cpu_baseline"]["single_thread"] = {"value": len(oc) * K3 / one / 1e6, "seconds": one}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
