#!/usr/bin/env python3
"""Benchmark of the mixed-precision GEMV / small-batch GEMM hot path on one MI355X.

Default workload (configs[1] of the benchmark spec): the four batch-1 matrix-vector products of one
Llama2-7B decoder layer (fused QKV 12288x4096, O 4096x4096, gate+up 22016x4096, down 4096x11008)
against 2/4/16-bit weights: g1 = 64, g2 = 16, 10 % 4-bit groups, 0.5 % fp16 outliers in 2-bit groups.
One step = those four launches on one layer copy.  Byte-identical copies of the packed layer live at
different addresses in HBM (32 copies, 2.2 GB) and the steps rotate over them, so every launch
streams its weights from HBM and not from the 256 MB last-level cache.

Other workloads (same protocol): --config 3 (Llama3-8B shapes, g1 = 128), --config 4 (Llama2-70B
slices, 80 layer copies = 22.5 GB resident, one step = a full 320-launch decode sweep), --batch M
(small-batch product), --sweep (configs[2]: batch x 4-bit fraction x outlier fraction on the
Llama2-7B layer; the table goes to stderr and into the JSON line's config.sweep).

Prints ONE JSON line on stdout; everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "effective weight GB/s and % HBM roofline, mixed-prec GEMV batch 1 (Llama2-7B)"
MODEL = {1: "Llama2-7B", 2: "Llama2-7B", 3: "Llama3-8B", 4: "Llama2-70B"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(spec, n4, nnz, M=1):
    """Bytes one product must move: codes, (s_int, z1), (s2, z2), CSR words and row pointers, X and Y."""
    import mpq_synth as synth
    by = synth.stored_bytes(spec, n4, nnz)
    return by["total"] + M * (2 * spec.K + 2 * spec.N)


class Layer:
    """One layer's matrices packed once and replicated `copies` times in device memory."""

    def __init__(self, torch, mpq, synth, specs, copies, M, dev):
        self.mats = []
        self.copies = copies
        self.multi = False   # True: the layer's products go out as one multi-problem launch
        t0 = time.time()
        for spec in specs:
            lg = synth.make_matrix(spec)
            pk = mpq.pack_logical(lg)
            first = torch.from_numpy(pk.blob).to(dev)
            m = dict(spec=spec, lg=lg, pk=pk, blobs=[first] + [first.clone() for _ in range(copies - 1)],
                     hdr=np.ascontiguousarray(pk.header))
            self.mats.append(m)
            log(f"[setup] {spec.name}: {spec.N}x{spec.K} g1={spec.g1} n4={pk.n4} nnz={pk.nnz} "
                f"packed={pk.blob.size / 1e6:.3f} MB ({time.time() - t0:.1f}s)")
        self.packed_bytes = sum(m["pk"].blob.size for m in self.mats)
        self.set_batch(torch, synth, M, dev)

    def set_batch(self, torch, synth, M, dev):
        """Activations and outputs for batch M (the weights stay as they are)."""
        self.M = M
        for m in self.mats:
            spec, pk = m["spec"], m["pk"]
            m["X"] = synth.make_x(spec.seed, M, spec.K)
            m["bytes"] = algorithmic_bytes(spec, pk.n4, pk.nnz, M)
            m["x"] = torch.from_numpy(m["X"].view(np.int16).copy()).to(dev)
            m["y"] = [torch.zeros(M * spec.N, dtype=torch.int16, device=dev) for _ in range(min(self.copies, 4))]
        self.step_bytes = sum(m["bytes"] for m in self.mats)
        # one workspace for all products of the stream (they run one after the other), as large as
        # the most demanding matrix asks for
        import paper_2311_16442_amd as mpq
        need = max(mpq.gemm_workspace_size(m["hdr"], M) for m in self.mats) if M > 1 else 0
        self.workspace = torch.empty(need, dtype=torch.uint8, device=dev) if need else None
        self.workspace_bytes = need
        torch.cuda.synchronize()

    def launch_layer(self, mpq, layer, stream):
        if self.multi:
            k = layer % len(self.mats[0]["y"])
            mpq.gemv_multi([m["hdr"] for m in self.mats], [m["blobs"][layer] for m in self.mats],
                           [m["x"] for m in self.mats], [m["y"][k] for m in self.mats], stream=stream)
            return
        for m in self.mats:
            y = m["y"][layer % len(m["y"])]
            if self.M == 1:
                mpq.gemv(m["hdr"], m["blobs"][layer], m["x"], y, stream=stream)
            else:
                mpq.gemm(m["hdr"], m["blobs"][layer], m["x"], y, self.M, stream=stream, workspace=self.workspace)


def time_rotations(torch, mpq, layer, stream, rotations, warm_rotations, use_graph):
    """Seconds (wall) and milliseconds (HIP events on the launch stream) for `rotations` passes over all copies."""
    graph = None
    with torch.cuda.stream(stream):
        layer.launch_layer(mpq, 0, stream)
        stream.synchronize()
        if use_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for c in range(layer.copies):
                    layer.launch_layer(mpq, c, stream)

        def rotation():
            if graph is not None:
                graph.replay()
            else:
                for c in range(layer.copies):
                    layer.launch_layer(mpq, c, stream)

        for _ in range(warm_rotations):
            rotation()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        ev0.record(stream)
        for _ in range(rotations):
            rotation()
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_start
        return wall, ev0.elapsed_time(ev1), graph is not None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=1024)
    ap.add_argument("--config", type=int, default=1, choices=[1, 3, 4],
                    help="1 = Llama2-7B layer (headline), 3 = Llama3-8B shapes, 4 = Llama2-70B 80-layer sweep")
    ap.add_argument("--batch", type=int, default=1, help="batch rows M (1 = GEMV)")
    ap.add_argument("--sweep", action="store_true",
                    help="configs[2]: M x 4-bit fraction x outlier fraction on the Llama2-7B layer")
    ap.add_argument("--g1", type=int, default=None, help="first-order group size instead of the configuration's (16, 32, 64, 128)")
    ap.add_argument("--g2", type=int, default=None, help="second-order group size instead of the configuration's")
    ap.add_argument("--g2-axis", type=int, default=None, choices=[0, 1],
                    help="0 = second-order pairs along K (the configurations), 1 = shared by g2 rows (the paper's axis)")
    ap.add_argument("--f4", type=float, default=None, help="fraction of 4-bit groups instead of the configuration's")
    ap.add_argument("--p-o", type=float, default=None, help="outlier probability instead of the configuration's")
    ap.add_argument("--multi", action="store_true",
                    help="one multi-problem launch per step (mpq_gemv_multi) instead of one launch per matrix; M = 1 only")
    ap.add_argument("--no-graph", action="store_true", help="launch from Python instead of replaying a HIP graph")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="do one 1 GiB device-to-device copy first (reference for FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on exactly one GPU (no collectives); use --gpus 1")
        sys.exit(2)

    import torch

    import mpq_synth as synth
    import paper_2311_16442_amd as mpq

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.Stream()
    M = args.batch

    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        log(f"[calibration] device copy of {src.numel() * 4} bytes done")
        del src, dst

    sweep = None
    if args.sweep:
        sweep = []
        for f4 in (0.0, 0.10, 0.25):
            for p_o in (0.0, 0.005, 0.015):
                lay = Layer(torch, mpq, synth, synth.config_specs(2, f4=f4, p_o=p_o), 16, 1, dev)
                for Ms in (1, 4, 16, 32):
                    lay.set_batch(torch, synth, Ms, dev)
                    wall, ev_ms, _ = time_rotations(torch, mpq, lay, stream, 8, 4, not args.no_graph)
                    us = wall * 1e6 / (8 * lay.copies)
                    row = {"M": Ms, "f4": f4, "p_o": p_o, "us_per_layer": round(us, 2),
                           "GB/s": round(lay.step_bytes / us / 1e3, 1), "MB": round(lay.step_bytes / 1e6, 2)}
                    sweep.append(row)
                    log("[sweep]", json.dumps(row))
                del lay
                torch.cuda.empty_cache()

    copies = 80 if args.config == 4 else 32
    import dataclasses
    specs = synth.config_specs(args.config, f4=args.f4, p_o=args.p_o)
    over = {k: v for k, v in (("g1", args.g1), ("g2", args.g2), ("g2_axis", args.g2_axis)) if v is not None}
    specs = [dataclasses.replace(sp, **over) for sp in specs]
    layer = Layer(torch, mpq, synth, specs, copies, M, dev)
    layer.multi = bool(args.multi)
    assert not (args.multi and M != 1), "--multi is the matrix-vector product only"
    log(f"[setup] {copies} layer copies resident: {copies * layer.packed_bytes / 1e9:.2f} GB; "
        f"algorithmic bytes per layer {layer.step_bytes / 1e6:.3f} MB")
    # a step: one layer (configs 1, 3) or one decode sweep over all 80 resident layers (config 4)
    layers_per_step = copies if args.config == 4 else 1
    if args.config == 4:
        rotations = max(1, min(args.steps, 64))
        warm_rot = max(1, min(args.warmup, 8))
    else:
        rotations = max(1, args.steps // copies)
        warm_rot = max(1, (args.warmup + copies - 1) // copies)
    wall, ev_ms, graphed = time_rotations(torch, mpq, layer, stream, rotations, warm_rot, not args.no_graph)
    steps = rotations * copies // layers_per_step
    warm = warm_rot * copies // layers_per_step
    step_bytes = layer.step_bytes * layers_per_step
    per_layer = 1 if args.multi else len(layer.mats)
    launches = rotations * copies * per_layer
    ms_per_step = wall * 1e3 / steps
    value = step_bytes / (wall / steps) / 1e9
    # dominant kernel = the product kernel (the only kernel in the timed region); its average launch
    # duration from HIP events on the launch stream over the timed region
    avg_launch_us = ev_ms * 1e3 / launches
    bytes_per_launch = layer.step_bytes / per_layer
    achieved = bytes_per_launch / (avg_launch_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "kernel": ("mpq_gemv_multi_kernel" if args.multi else "mpq_gemv_kernel" if M == 1 else "mpq_mm_kernel or mpq_mms_kernel + mpq_mms_finish_kernel") + " (every product of the step)", "avg_launch_us": round(avg_launch_us, 3),
                "bytes_per_launch": round(bytes_per_launch)}
    traffic_file = os.path.join(ROOT, "profiles", "gemv_llama2_7b_traffic.json")
    if args.config == 1 and M == 1 and not over and not args.multi and args.f4 is None and args.p_o is None and os.path.exists(traffic_file):
        try:
            roofline["traffic"] = json.load(open(traffic_file)).get("hbm_bytes_per_launch")
        except Exception:  # noqa: BLE001 - a malformed note must not break the benchmark line
            pass

    cpu = None
    if not args.no_cpu:
        import oracle
        sample = min(layer.mats, key=lambda m: m["spec"].N * m["spec"].K)   # smallest matrix of the layer
        om = oracle.Matrix.from_logical(sample["lg"])
        cores = oracle.max_threads()
        tc = time.perf_counter()
        reps = 0
        while time.perf_counter() - tc < 10.0 or reps < 2:
            ref = om.gemm(sample["X"], threads=cores)
            reps += 1
        cpu_s = (time.perf_counter() - tc) / reps
        # correctness of what was timed: the last launch wrote y[(copies - 1) % len(y)]
        got = sample["y"][(copies - 1) % len(sample["y"])].cpu().numpy().view(np.float16).astype(np.float64)
        got = got.reshape(M, sample["spec"].N)
        rms = float(np.sqrt(np.mean(ref ** 2)))
        err = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 0.05 * rms)))
        log(f"[check] {sample['spec'].name} output of the timed run vs oracle: max rel err {err:.2e}")
        assert err <= 2e-3, err
        cpu = {"value": round(sample["bytes"] / cpu_s / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
               "sample": f"oracle product (fp64 accumulation, OpenMP over rows) of the {sample['spec'].N}x{sample['spec'].K} "
                         f"{sample['spec'].name} matrix of the same layer at M={M}, {reps} repetitions, {cpu_s * 1e3:.1f} ms each"}

    spec0 = layer.mats[0]["spec"]
    workload = ("configs[%d]: %s %s, %d launches per step (%s), batch M=%d, g1=%d g2=%d%s f4=%.0f%% p_o=%.1f%%, "
                "%d layer copies %s" % (
                    args.config, MODEL[args.config],
                    "decode sweep over 80 resident layers" if args.config == 4 else "decoder layer",
                    per_layer * layers_per_step,
                    ", ".join(f"{m['spec'].N}x{m['spec'].K}" for m in layer.mats), M, spec0.g1, spec0.g2,
                    " (pairs shared by g2 rows)" if spec0.g2_axis == 1 else "", 100 * spec0.f4, 100 * spec0.p_o, copies,
                    "resident (22.5 GB), each read once per step" if args.config == 4 else "rotated (cold last-level cache)"))
    config = {"workload": workload, "bytes_per_step": step_bytes,
              "launch": "hipGraph replay" if graphed else "python", "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2)}
    if sweep is not None:
        config["sweep"] = sweep
    out = {"metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warm,
           "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f16", "data": "synthetic", "config": config, "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
