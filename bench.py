#!/usr/bin/env python3
"""Benchmark of the mixed-precision GEMV / small-batch GEMM hot path on one MI355X.

Default workload (configs[1] of the benchmark spec): the four batch-1 matrix-vector products of one
Llama2-7B decoder layer (fused QKV 12288x4096, O 4096x4096, gate+up 22016x4096, down 4096x11008)
against 2/4/16-bit weights: g1 = 64, g2 = 16, 10 % 4-bit groups, 0.5 % fp16 outliers in 2-bit groups.
One step = those four launches on one layer copy.  Byte-identical copies of the packed layer live at
different addresses in HBM (32 copies, 2.2 GB) and the steps rotate over them, so every launch
streams its weights from HBM and not from the 256 MB last-level cache.

Timing protocol.  The rotation over the copies is captured in a HIP graph and replayed.  Whatever
--warmup says, at least 1024 steps run untimed first (the shader clock needs about that long to
settle); then EXACTLY --steps steps are timed (whole rotations plus one shorter graph for the rest).

Next to the product, the same run measures what the memory system delivers (roofline.ceiling): one
read-only pass over 4 GiB, and a read-only pass over the SAME packed bytes in the SAME launch pattern
(one launch per matrix, same rotation, same graph protocol).

Other workloads (same protocol): --config 3 (Llama3-8B shapes, g1 = 128), --config 4 (Llama2-70B
slices, 80 layers = 22.5 GB resident, one step = a full 320-launch decode sweep; layer l is layer 0 with
its 16-row blocks rotated by l), --token (configs 1 and 3: a whole decode step over 32 layers drawn
with their own seeds, plus lm_head for config 3, as ONE graph: ms per token), --batch M (small-batch
product), --sweep (configs[2]: batch x 4-bit fraction x outlier fraction on the Llama2-7B layer; the
table goes to stderr and into the JSON line's config.sweep).

Prints ONE JSON line on stdout; everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MIN_WARM_STEPS = 1024
METRIC = "effective weight GB/s and % HBM roofline, mixed-prec GEMV batch 1 (Llama2-7B)"
MODEL = {1: "Llama2-7B", 2: "Llama2-7B", 3: "Llama3-8B", 4: "Llama2-70B"}
KERNEL_NAMES = {1: "mpq_gemvp_kernel", 2: "mpq_gemv_kernel", 3: "mpq_mm_kernel", 4: "mpq_mms_kernel + mpq_mms_finish_kernel"}
TRAFFIC_FILE = os.path.join("profiles", "gemv_llama2_7b_traffic.json")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(spec, n4, nnz, M=1):
    """Bytes one product must move: codes, (s_int, z1), (s2, z2), CSR words and row pointers, X and Y."""
    import mpq_synth as synth
    by = synth.stored_bytes(spec, n4, nnz)
    return by["total"] + M * (2 * spec.K + 2 * spec.N)


class Layer:
    """The matrices of a layer, packed, with `copies` device blobs each.

    distinct = "copies":  byte-identical copies at different addresses (cold last-level cache);
    distinct = "seeds":   every copy is a layer of its own, drawn from the recipe with its layer index;
    distinct = "rotated": copy l is copy 0 with its 16-row records rotated by l (a different matrix with the
                          same header) - for the 80-layer sweep, where drawing 80 x 855 M weights on the
                          host would take minutes."""

    def __init__(self, torch, mpq, synth, specs, copies, M, dev, distinct="copies", config=1):
        self.mats = []
        self.copies = copies
        self.multi = False   # True: the layer's products go out as one multi-problem launch
        self.dequant = None  # 0 / 1: the steps dequantize (without / with outliers) instead of multiplying
        t0 = time.time()
        for mi, spec in enumerate(specs):
            lg = synth.make_matrix(spec)
            pk = mpq.pack_logical(lg)
            first = torch.from_numpy(pk.blob).to(dev)
            blobs, hdrs = [first], [np.ascontiguousarray(pk.header)]
            nbytes = [algorithmic_bytes(spec, pk.n4, pk.nnz, M)]
            for c in range(1, copies):
                if distinct == "seeds":
                    spec_c = dataclasses.replace(spec, seed=synth.matrix_seed(config, mi, c))
                    lg_c = synth.make_matrix(spec_c)
                    pk_c = mpq.pack_logical(lg_c)
                    blobs.append(torch.from_numpy(pk_c.blob).to(dev))
                    hdrs.append(np.ascontiguousarray(pk_c.header))
                    nbytes.append(algorithmic_bytes(spec_c, pk_c.n4, pk_c.nnz, M))
                elif distinct == "rotated":
                    assert spec.N % 16 == 0
                    off, rec, cnt = mpq.blob_tiles(pk.header)
                    b = first.clone()
                    tiles = first[off: off + rec * cnt].view(cnt, rec)
                    b[off: off + rec * cnt].view(cnt, rec).copy_(torch.roll(tiles, shifts=c % cnt, dims=0))
                    blobs.append(b)
                    hdrs.append(hdrs[0])
                    nbytes.append(nbytes[0])
                else:
                    blobs.append(first.clone())
                    hdrs.append(hdrs[0])
                    nbytes.append(nbytes[0])
            self.mats.append(dict(spec=spec, lg=lg, pk=pk, blobs=blobs, hdrs=hdrs, hdr=hdrs[0], nbytes=nbytes))
            log(f"[setup] {spec.name}: {spec.N}x{spec.K} g1={spec.g1} n4={pk.n4} nnz={pk.nnz} "
                f"packed={pk.blob.size / 1e6:.3f} MB x {copies} ({distinct}) ({time.time() - t0:.1f}s)")
        self.packed_bytes = sum(m["pk"].blob.size for m in self.mats)
        self.set_batch(torch, synth, M, dev)

    def set_batch(self, torch, synth, M, dev):
        """Activations and outputs for batch M (the weights stay as they are)."""
        import paper_2311_16442_amd as mpq
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
        need = max(mpq.gemm_workspace_size(m["hdr"], M) for m in self.mats) if M > 1 else 0
        self.workspace = torch.empty(need, dtype=torch.uint8, device=dev) if need else None
        torch.cuda.synchronize()

    def kernels(self, torch, mpq):
        """Which kernel every matrix of the layer runs (one call each through the reporting entry point)."""
        names = []
        for m in self.mats:
            rep = mpq.gemm_planned(m["hdr"], m["blobs"][0], m["x"], m["y"][0], self.M, workspace=self.workspace)
            names.append(KERNEL_NAMES.get(rep.kernel, str(rep.kernel)))
        torch.cuda.synchronize()
        return names

    def launch_layer(self, mpq, layer, stream, stream_only=False):
        if self.dequant is not None and not stream_only:
            for m in self.mats:
                mpq.dequant(m["hdrs"][layer], m["blobs"][layer], self.wout, add_outliers=bool(self.dequant), stream=stream)
            return
        if stream_only:   # the same bytes in the same launch pattern, read and nothing else
            for m in self.mats:
                mpq.stream_probe(m["blobs"][layer], stream=stream)
            return
        if self.multi:
            k = layer % len(self.mats[0]["y"])
            mpq.gemv_multi([m["hdrs"][layer] for m in self.mats], [m["blobs"][layer] for m in self.mats],
                           [m["x"] for m in self.mats], [m["y"][k] for m in self.mats], stream=stream)
            return
        for m in self.mats:
            y = m["y"][layer % len(m["y"])]
            if self.M == 1:
                mpq.gemv(m["hdrs"][layer], m["blobs"][layer], m["x"], y, stream=stream)
            else:
                mpq.gemm(m["hdrs"][layer], m["blobs"][layer], m["x"], y, self.M, stream=stream, workspace=self.workspace)


def time_steps(torch, mpq, layer, stream, layer_steps, warm_layer_steps, use_graph, stream_only=False):
    """Runs >= warm_layer_steps untimed, then exactly layer_steps timed passes over one layer copy each
    (copies in rotation).  Returns (wall seconds, event milliseconds on the launch stream, warm steps run, graphed)."""
    copies = layer.copies
    full, rest = divmod(layer_steps, copies)
    warm_rot = (warm_layer_steps + copies - 1) // copies
    g_full = g_rest = None
    with torch.cuda.stream(stream):
        layer.launch_layer(mpq, 0, stream, stream_only)
        stream.synchronize()
        if use_graph:
            g_full = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_full, stream=stream):
                for c in range(copies):
                    layer.launch_layer(mpq, c, stream, stream_only)
            if rest:
                g_rest = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g_rest, stream=stream):
                    for c in range(rest):
                        layer.launch_layer(mpq, c, stream, stream_only)

        def run(count, graph):
            if graph is not None:
                graph.replay()
            else:
                for c in range(count):
                    layer.launch_layer(mpq, c, stream, stream_only)

        for _ in range(warm_rot):
            run(copies, g_full)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        ev0.record(stream)
        for _ in range(full):
            run(copies, g_full)
        if rest:
            run(rest, g_rest)
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_start
    return wall, ev0.elapsed_time(ev1), warm_rot * copies, use_graph


def measure_ceiling(torch, mpq, layer, stream, dev, layer_steps, use_graph):
    """What the memory system delivers: a 4 GiB read-only pass, and the packed bytes of the workload read
    (and nothing else) in the workload's own launch pattern."""
    big = torch.empty(4 << 30, dtype=torch.uint8, device=dev)
    big.fill_(1)
    with torch.cuda.stream(stream):
        mpq.stream_probe(big, stream=stream)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        stream.synchronize()
        ev0.record(stream)
        for _ in range(4):
            mpq.stream_probe(big, stream=stream)
        ev1.record(stream)
        stream.synchronize()
    big_gbs = 4 * big.numel() / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del big
    torch.cuda.empty_cache()
    steps = min(layer_steps, 2048)
    wall, ev_ms, _, _ = time_steps(torch, mpq, layer, stream, steps, 256, use_graph, stream_only=True)
    us = ev_ms * 1e3 / steps
    return {"read_4GiB_GBs": round(big_gbs, 1),
            "same_launches_read_only_us_per_layer": round(us, 3),
            "same_launches_read_only_GBs": round(layer.step_bytes / us / 1e3, 1),
            "note": "one read-only launch per matrix over its packed blob, same rotation and graph protocol; "
                    "GB/s counts the same algorithmic bytes as `value`"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=1024)
    ap.add_argument("--config", type=int, default=1, choices=[1, 3, 4],
                    help="1 = Llama2-7B layer (headline), 3 = Llama3-8B shapes, 4 = Llama2-70B 80-layer sweep")
    ap.add_argument("--batch", type=int, default=1, help="batch rows M (1 = GEMV)")
    ap.add_argument("--token", action="store_true",
                    help="configs 1 and 3: one step = a decode step over 32 layers drawn with their own seeds "
                         "(+ lm_head for config 3) as one graph; reports ms per token")
    ap.add_argument("--dequant", type=int, default=None, choices=[0, 1],
                    help="time mpq_dequant (0 = dense part, 1 = with the outliers added) on the layer's matrices instead of "
                         "the product; bytes = packed bytes read + 2 bytes per weight written")
    ap.add_argument("--sweep", action="store_true",
                    help="configs[2]: M x 4-bit fraction x outlier fraction on the Llama2-7B layer")
    ap.add_argument("--g1", type=int, default=None, help="first-order group size instead of the configuration's (16, 32, 64, 128)")
    ap.add_argument("--g2", type=int, default=None, help="second-order group size instead of the configuration's")
    ap.add_argument("--g2-axis", type=int, default=None, choices=[0, 1],
                    help="0 = second-order pairs along K (the configurations), 1 = shared by g2 rows (the paper's axis)")
    ap.add_argument("--meta", type=int, default=None, choices=[0, 1],
                    help="1 = the paper's aligned metadata (16-bit word per three 2-bit groups, byte-padded second-order "
                         "zero; needs --g1 16), 0 = byte-wide scales and zero points (the configurations)")
    ap.add_argument("--f4", type=float, default=None, help="fraction of 4-bit groups instead of the configuration's")
    ap.add_argument("--p-o", type=float, default=None, help="outlier probability instead of the configuration's")
    ap.add_argument("--multi", action="store_true",
                    help="one multi-problem launch per step (mpq_gemv_multi) instead of one launch per matrix; M = 1 only. "
                         "An upper bound for products that do not depend on each other, never the headline")
    ap.add_argument("--no-graph", action="store_true", help="launch from Python instead of replaying a HIP graph")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the read-only bandwidth legs")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="do one 1 GiB device-to-device copy first (reference for FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on exactly one GPU (no collectives); use --gpus 1")
        sys.exit(2)
    if args.steps < 1:
        log("bench.py: --steps must be at least 1")
        sys.exit(2)

    import torch

    import mpq_synth as synth
    import paper_2311_16442_amd as mpq

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.Stream()
    M = args.batch
    use_graph = not args.no_graph

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
                    wall, ev_ms, _, _ = time_steps(torch, mpq, lay, stream, 8 * lay.copies, 4 * lay.copies, use_graph)
                    us = ev_ms * 1e3 / (8 * lay.copies)
                    row = {"M": Ms, "f4": f4, "p_o": p_o, "us_per_layer": round(us, 2),
                           "GB/s": round(lay.step_bytes / us / 1e3, 1), "MB": round(lay.step_bytes / 1e6, 2)}
                    sweep.append(row)
                    log("[sweep]", json.dumps(row))
                del lay
                torch.cuda.empty_cache()

    assert not (args.token and args.config == 4), "--token is for configs 1 and 3 (config 4 is a whole sweep already)"
    assert not (args.multi and M != 1), "--multi is the matrix-vector product only"
    copies = 80 if args.config == 4 else 32
    distinct = "rotated" if args.config == 4 else "seeds" if args.token else "copies"
    specs = synth.config_specs(args.config, f4=args.f4, p_o=args.p_o)
    over = {k: v for k, v in (("g1", args.g1), ("g2", args.g2), ("g2_axis", args.g2_axis), ("meta", args.meta)) if v is not None}
    specs = [dataclasses.replace(sp, **over) for sp in specs]
    head = None
    if args.token and args.config == 3:      # the head is used once per token, not once per layer
        head = Layer(torch, mpq, synth, [sp for sp in specs if sp.name == "lm_head"], 2, M, dev)
    if args.token:
        specs = [sp for sp in specs if sp.name != "lm_head"]
    layer = Layer(torch, mpq, synth, specs, copies, M, dev, distinct=distinct, config=args.config)
    layer.multi = bool(args.multi)
    kernel_names = ["mpq_gemv_multi_kernel"] if args.multi else layer.kernels(torch, mpq)
    if args.dequant is not None:
        layer.dequant = args.dequant
        layer.wout = torch.zeros(max(m["spec"].N * m["spec"].K for m in layer.mats), dtype=torch.int16, device=dev)
        # groups of 16 or 32 columns go through the kernel that writes whole output lines (unit tables of up to 14 KiB)
        def dequant_kernel(m):
            h = np.asarray(m["hdrs"][0]).view(np.int32)
            table = 32 * (64 // m["spec"].g1) * int(h[13] + h[14]) if m["spec"].g1 < 64 else 0   # 32 bytes per piece and block
            return "mpq_dequant_lines_kernel" if 0 < table <= 14336 else "mpq_dequant_kernel"
        kernel_names = [dequant_kernel(m) for m in layer.mats]
        for m in layer.mats:      # what a dequantization moves: the packed bytes in, two bytes per weight out
            m["bytes"] = m["bytes"] - M * (2 * m["spec"].K + 2 * m["spec"].N) + 2 * m["spec"].N * m["spec"].K
        layer.step_bytes = sum(m["bytes"] for m in layer.mats)
    log(f"[setup] {copies} layers resident: {copies * layer.packed_bytes / 1e9:.2f} GB; "
        f"algorithmic bytes per layer {layer.step_bytes / 1e6:.3f} MB; kernels {kernel_names}")

    # a step: one layer (configs 1, 3), or one pass over all resident layers (config 4 and --token)
    whole_stack = args.config == 4 or args.token
    layers_per_step = copies if whole_stack else 1
    layer_steps = args.steps * layers_per_step
    warm_layer_steps = max(args.warmup * layers_per_step, MIN_WARM_STEPS)
    if head is not None:
        # the head rides along as one more launch per step: time it on its own protocol and add it
        wall_h, ev_h, _, _ = time_steps(torch, mpq, head, stream, max(2 * (args.steps // 2), 2), 16, use_graph)
        head_us = ev_h * 1e3 / max(2 * (args.steps // 2), 2)
    wall, ev_ms, warm_run, graphed = time_steps(torch, mpq, layer, stream, layer_steps, warm_layer_steps, use_graph)
    steps = args.steps
    warm = warm_run // layers_per_step
    step_bytes = layer.step_bytes * layers_per_step
    if distinct == "seeds":
        step_bytes = sum(sum(m["nbytes"]) for m in layer.mats)
    step_s = wall / steps
    if head is not None:
        step_bytes += head.step_bytes
        step_s += head_us * 1e-6
        ev_ms += head_us * 1e-3 * steps
    per_layer = 1 if args.multi else len(layer.mats)
    launches = steps * (layers_per_step * per_layer + (1 if head is not None else 0))
    ms_per_step = step_s * 1e3
    value = step_bytes / step_s / 1e9
    # dominant kernel = the product kernel (the only kernel in the timed region); its average launch
    # duration from HIP events on the launch stream over the timed region
    avg_launch_us = ev_ms * 1e3 / launches
    bytes_per_launch = step_bytes * steps / launches
    achieved = bytes_per_launch / (avg_launch_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "kernel": " / ".join(sorted(set(kernel_names))) + " (every product of the step: " + ", ".join(
                    f"{m['spec'].name} {k}" for m, k in zip(layer.mats, kernel_names)) + ")" if not args.multi else kernel_names[0],
                "avg_launch_us": round(avg_launch_us, 3), "bytes_per_launch": round(bytes_per_launch)}
    default_workload = (args.config == 1 and M == 1 and not over and not args.multi and not args.token
                        and args.f4 is None and args.p_o is None and args.dequant is None)
    if default_workload and os.path.exists(os.path.join(ROOT, TRAFFIC_FILE)):
        try:
            roofline["traffic"] = json.load(open(os.path.join(ROOT, TRAFFIC_FILE))).get("hbm_bytes_per_launch")
            roofline["traffic_source"] = (TRAFFIC_FILE + ": rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                                          "read from the file, not measured in this run")
        except Exception:  # noqa: BLE001 - a malformed note must not break the benchmark line
            pass
    if not args.no_ceiling and not args.multi and args.dequant is None:
        roofline["ceiling"] = measure_ceiling(torch, mpq, layer, stream, dev, layer_steps, use_graph)
        roofline["ceiling"]["frac_of_same_launches_read_only"] = round(value / roofline["ceiling"]["same_launches_read_only_GBs"], 4)

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
        # correctness of what is timed: one more product on copy 0 (the copy the oracle holds)
        layer.dequant = None
        y0 = torch.zeros(M * sample["spec"].N, dtype=torch.int16, device=dev)
        mpq.gemm(sample["hdr"], sample["blobs"][0], sample["x"], y0, M, workspace=layer.workspace)
        torch.cuda.synchronize()
        got = y0.cpu().numpy().view(np.float16).astype(np.float64).reshape(M, sample["spec"].N)
        rms = float(np.sqrt(np.mean(ref ** 2)))
        err = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 0.05 * rms)))
        log(f"[check] {sample['spec'].name} product vs oracle: max rel err {err:.2e}")
        assert err <= 2e-3, err
        cpu = {"value": round(sample["bytes"] / cpu_s / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
               "sample": f"oracle product (fp64 accumulation, OpenMP over rows) of the {sample['spec'].N}x{sample['spec'].K} "
                         f"{sample['spec'].name} matrix of the same layer at M={M}, {reps} repetitions, {cpu_s * 1e3:.1f} ms each"}

    spec0 = layer.mats[0]["spec"]
    shapes = ", ".join(f"{m['spec'].N}x{m['spec'].K}" for m in layer.mats)
    if args.token:
        what = f"decode step over {copies} layers drawn with their own seeds" + (" plus lm_head 128256x4096" if head is not None else "")
        residency = "every layer read once per step"
    elif args.config == 4:
        what = "decode sweep over 80 resident layers (layer l = layer 0 with its 16-row blocks rotated by l)"
        residency = "resident (22.5 GB), each read once per step"
    else:
        what = "decoder layer"
        residency = "byte-identical layer copies rotated (cold last-level cache)"
    workload = ("configs[%d]: %s %s, %d launches per step (%s), batch M=%d, g1=%d g2=%d%s f4=%.0f%% p_o=%.1f%%, %d %s" % (
        args.config, MODEL[args.config], what, launches // steps, shapes, M, spec0.g1, spec0.g2,
        (" (pairs shared by g2 rows)" if spec0.g2_axis == 1 else "") + (" aligned metadata (Sec. 3.3)" if spec0.meta == 1 else ""), 100 * spec0.f4, 100 * spec0.p_o, copies, residency))
    config = {"workload": workload, "bytes_per_step": step_bytes,
              "launch": "hipGraph replay" if graphed else "python", "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
              "requested": {"steps": args.steps, "warmup": args.warmup},
              "warmup_rule": f"at least {MIN_WARM_STEPS} layer passes run untimed whatever --warmup says"}
    if args.token:
        config["ms_per_token"] = round(ms_per_step, 5)
    if args.multi:
        config["note"] = "one launch for the four products: only legitimate for products that do not depend on each other"
    if args.dequant is not None:
        config["note"] = ("mpq_dequant %s outliers instead of the product: bytes = packed bytes read + 2 bytes per weight written"
                          % ("with" if args.dequant else "without"))
    if sweep is not None:
        config["sweep"] = sweep
    out = {"metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warm,
           "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f16", "data": "synthetic", "config": config, "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
