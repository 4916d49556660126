#!/usr/bin/env python3
"""Phase timeline of the batch-1 kernels on one MI355X, from the timeline build of the library.

The timeline build (paper_2311_16442_amd/libmpq_timeline.so: the product sources compiled with
-DMPQ_TIMELINE) reads the 100 MHz wall clock at the phase boundaries of the two matrix-vector kernels;
the first and the last wave of every workgroup write their stamps to a buffer.  This program runs the
products of a decoder layer as bench.py does (copies of every matrix rotated so that the last-level
cache holds other data, the other products of the layer launched in between), collects the stamps of
one launch per repetition and prints, per shape and phase, the median and the 5 % .. 95 % range over
workgroups and repetitions, in microseconds after the first wave of the launch started.

  python timeline.py [--config 1|3|4] [--path 0|1|2] [--waves W] [--tiles n] [--reps 40]
  python timeline.py --dequant 0|1 [--config 1|3|4]
  python timeline.py --batch M [--config 1|3|4]

--path: 0 = the library's choice per shape, 1 = plane-sum kernel, 2 = per-weight kernel.
--batch: the two kernels of the K-range batch path (shapes that the library routes there at that M): when the
unit table, the gathered activations and the first block are there, when the blocks are done, when the partial sums
are written; and the phases of the second kernel (outlier product, sum over the ranges).
--dequant: the dequantization kernel instead (0 = dense part, 1 = with the outliers): per wave, the time it
spends issuing its batches' requests, waiting for a block's words, and decoding, turning and storing; when
the waves end, by how many workgroups shared their compute unit.
"""
import argparse
import ctypes as C
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PHASES = {
    2: ["start", "requests issued", "staged operands landed", "barrier 1", "outliers done", "block 1 fetched", "block 2 fetched",
        "block 3 fetched", "blocks done", "barrier 2", "end"],
    1: ["start", "requests issued", "staged operands landed", "barrier 1", "activations split", "outliers done", "barrier 2",
        "block 1 done", "blocks done", "barrier 3", "end"],
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1, choices=[1, 3, 4])
    ap.add_argument("--path", type=int, default=0, choices=[0, 1, 2])
    ap.add_argument("--reps", type=int, default=40)
    ap.add_argument("--waves", type=int, default=0, help="waves per workgroup (0 = the library's choice)")
    ap.add_argument("--tiles", type=int, default=0, help="tiles per workgroup (0 = the library's choice)")
    ap.add_argument("--dequant", type=int, default=None, choices=[0, 1])
    ap.add_argument("--batch", type=int, default=None)
    args = ap.parse_args()
    import torch
    import mpq_synth as synth
    import paper_2311_16442_amd as mpq
    lib_path = os.path.join(os.path.dirname(mpq.LIB_PATH), "libmpq_timeline.so")
    if not os.path.exists(lib_path):
        raise SystemExit(f"{lib_path} is missing: python paper_2311_16442_amd/build.py --timeline")
    L = C.CDLL(lib_path)
    L.mpq_gemm_planned.restype = C.c_int
    L.mpq_gemm_planned.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p,
                                   C.POINTER(mpq.Plan), C.POINTER(mpq.Report)]
    L.mpq_timeline_buffer.restype = C.c_int
    L.mpq_timeline_buffer.argtypes = [C.c_void_p]
    if args.dequant is not None:
        return dequant_timeline(args, torch, synth, mpq, L)
    if args.batch is not None:
        return batch_timeline(args, torch, synth, mpq, L)
    shapes = []
    for spec in synth.config_specs(args.config):
        if spec.name == "lm_head":
            continue
        pk = mpq.pack_logical(synth.make_matrix(spec))
        copies = max(3, min(12, int(1.5e9 // pk.blob.size)))
        blobs = [torch.from_numpy(pk.blob).cuda() for _ in range(copies)]
        X = torch.from_numpy(synth.make_x(1, 1, spec.K).view(np.int16).copy()).cuda()
        Y = torch.zeros(spec.N, dtype=torch.int16, device="cuda")
        shapes.append((spec, np.ascontiguousarray(pk.header), blobs, X, Y))
    buf = torch.zeros(8192 * 32, dtype=torch.int64, device="cuda")
    plan = mpq.Plan(gemv_path=args.path, gemv_waves=args.waves, gemv_tiles=args.tiles)
    rep = mpq.Report()

    def launch(sh, i):
        spec, hdr, blobs, X, Y = sh
        st = L.mpq_gemm_planned(hdr.ctypes.data, blobs[i % len(blobs)].data_ptr(), X.data_ptr(), Y.data_ptr(), 1, None, 0, None,
                                C.byref(plan), C.byref(rep))
        assert st == 0, st

    print(f"# config {args.config}, gemv_path {args.path}, {args.reps} repetitions (the first 10 left out); microseconds after the first wave of the launch started")
    print("# median [5 % .. 95 %] over workgroups and repetitions; first wave / last wave of a workgroup")
    for sh in shapes:
        spec = sh[0]
        acc = []
        for i in range(args.reps):
            assert L.mpq_timeline_buffer(None) == 0
            for other in shapes:
                launch(other, i + 1)
            torch.cuda.synchronize()
            buf.zero_()
            torch.cuda.synchronize()
            assert L.mpq_timeline_buffer(buf.data_ptr()) == 0
            launch(sh, i)
            torch.cuda.synchronize()
            if 2 * rep.workgroups * 16 > buf.numel():
                raise SystemExit("stamp buffer too small")
            if i >= 10:
                acc.append(buf.cpu().numpy().reshape(-1, 16)[: 2 * rep.workgroups].astype(np.float64))
        names = PHASES[rep.kernel]
        kernel = {1: "plane-sum kernel", 2: "per-weight kernel"}[rep.kernel]
        spans = np.array([(d[:, 10].max() - d[:, 0].min()) / 100.0 for d in acc])
        early = np.median([np.sum((d[0::2, 0] - d[:, 0].min()) / 100.0 < 3.0) for d in acc])  # a second generation starts later
        print(f"\n{spec.name} {spec.N}x{spec.K}: {kernel}, {rep.waves} waves x {rep.workgroups} workgroups, {rep.tiles_per_workgroup} tile(s) each; "
              f"first start to last end {np.median(spans):.2f} us [{spans.min():.2f} .. {spans.max():.2f}]; "
              f"{early:.0f} workgroups started within 3 us of the first")
        for wsel, label in ((0, "first wave"), (1, "last wave")):
            rows = []
            for d in acc:
                dd = (d[wsel::2, :11] - d[:, 0].min()) / 100.0
                dd[d[wsel::2, :11] == 0] = np.nan
                rows.append(dd)
            dd = np.concatenate(rows, axis=0)
            nb = np.concatenate([d[wsel::2, 11] for d in acc])
            print(f"  {label} ({np.median(nb):.0f} blocks, at most {nb.max():.0f}):")
            for k, nm in enumerate(names):
                col = dd[:, k]
                if np.all(np.isnan(col)):
                    continue
                print(f"    {nm:24s} {np.nanmedian(col):6.2f}  [{np.nanpercentile(col, 5):5.2f} .. {np.nanpercentile(col, 95):5.2f}]")


def batch_timeline(args, torch, synth, mpq, L):
    M = args.batch
    L.mpq_gemm_workspace_size.restype = C.c_int
    L.mpq_gemm_workspace_size.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]
    us = lambda ticks: ticks / 100.0
    first = ["start", "unit table there", "requests issued", "own gather landed", "barrier: activations there",
             "transposed activations written", "blocks done (last group)", "partial sums written", "all waves' blocks done (last group)", "gather requests issued"]
    print(f"# config {args.config}, batch {M}: K-range kernel (first and last wave of every workgroup) and its second kernel;")
    print("# microseconds after the first wave of the first kernel started; median [5 % .. 95 %]")
    for spec in synth.config_specs(args.config):
        if spec.name == "lm_head":
            continue
        pk = mpq.pack_logical(synth.make_matrix(spec))
        hdr = np.ascontiguousarray(pk.header)
        blobs = [torch.from_numpy(pk.blob).cuda() for _ in range(4)]
        X = torch.from_numpy(synth.make_x(1, M, spec.K).view(np.int16).copy()).cuda()
        Y = torch.zeros(M * spec.N, dtype=torch.int16, device="cuda")
        need = C.c_size_t(0)
        assert L.mpq_gemm_workspace_size(hdr.ctypes.data, M, C.byref(need)) == 0
        ws = torch.empty(max(256, need.value), dtype=torch.uint8, device="cuda")
        rep = mpq.Report()
        buf = torch.zeros(8192 * 2 * 16, dtype=torch.int64, device="cuda")
        for rnd in range(2):
            for i in range(4):
                if rnd == 1 and i == 3:
                    torch.cuda.synchronize()
                    assert L.mpq_timeline_buffer(buf.data_ptr()) == 0
                st = L.mpq_gemm_planned(hdr.ctypes.data, blobs[i].data_ptr(), X.data_ptr(), Y.data_ptr(), M, ws.data_ptr(), ws.numel(),
                                        None, None, C.byref(rep))
                assert st == 0, st
        torch.cuda.synchronize()
        assert L.mpq_timeline_buffer(None) == 0
        if rep.kernel != 4:
            print(f"\n{spec.name} {spec.N}x{spec.K}: not routed to the K-range kernel at this batch size")
            continue
        a = buf.cpu().numpy().reshape(-1, 16).astype(np.float64)
        k1, k2 = a[: 2 * 4096], a[2 * 4096:]
        n1 = int(rep.workgroups)
        k1, k2 = k1[: 2 * n1], k2[k2[:, 8] > 0]
        t0 = k1[:, 0].min()
        print(f"\n{spec.name} {spec.N}x{spec.K}: {rep.workgroups} workgroups of {rep.waves} waves; first kernel ends {us(k1[:, 7].max() - t0):.2f}, "
              f"second kernel starts {us(k2[:, 8].min() - t0):.2f} and ends {us(k2[:, 12].max() - t0):.2f}")
        w_first, w_last = k1[0::2], k1[1::2]   # records alternate: first wave, last wave of a workgroup
        for k, nm in enumerate(first):
            ca, cb = us(w_first[:, k] - t0), us(w_last[:, k] - t0)
            print(f"    {nm:32s} first wave {np.median(ca):6.2f}  [{np.percentile(ca, 5):5.2f} .. {np.percentile(ca, 95):5.2f}]"
                  f"   last wave {np.median(cb):6.2f}  [{np.percentile(cb, 5):5.2f} .. {np.percentile(cb, 95):5.2f}]")
        t2 = k2[:, 8].min()
        for k, nm in ((8, "second kernel: start"), (9, "words, row starts, first sums there"), (10, "outlier product done"), (12, "end")):
            col = us(k2[:, k] - t2)
            print(f"    {nm:32s} {np.median(col):6.2f}  [{np.percentile(col, 5):5.2f} .. {np.percentile(col, 95):5.2f}]   (after the second kernel's first wave)")


def dequant_timeline(args, torch, synth, mpq, L):
    L.mpq_dequant.restype = C.c_int
    L.mpq_dequant.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
    us = lambda ticks: ticks / 100.0
    print(f"# config {args.config}, mpq_dequant with add_outliers = {args.dequant}: stamps of the first and the last wave of every workgroup,")
    print("# one launch after three others on rotating copies of blob and output; microseconds")
    for spec in synth.config_specs(args.config):
        if spec.name == "lm_head":
            continue
        pk = mpq.pack_logical(synth.make_matrix(spec))
        hdr = np.ascontiguousarray(pk.header)
        blobs = [torch.from_numpy(pk.blob).cuda() for _ in range(4)]
        outs = [torch.empty(spec.N * spec.K, dtype=torch.int16, device="cuda") for _ in range(4)]
        buf = torch.zeros(4096 * 2 * 16, dtype=torch.int64, device="cuda")
        for rnd in range(2):
            for i in range(4):
                if rnd == 1 and i == 3:
                    torch.cuda.synchronize()
                    assert L.mpq_timeline_buffer(buf.data_ptr()) == 0
                assert L.mpq_dequant(hdr.ctypes.data, blobs[i].data_ptr(), outs[i].data_ptr(), args.dequant, None) == 0
        torch.cuda.synchronize()
        assert L.mpq_timeline_buffer(None) == 0
        a = buf.cpu().numpy().reshape(-1, 16)
        a = a[a[:, 11] > 0]
        t0 = a[:, 0].min()
        end = us(a[:, 4] - t0)
        print(f"\n{spec.name} {spec.N}x{spec.K}: {len(a)} waves recorded, {a[:, 11].min()} to {a[:, 11].max()} blocks each; "
              f"start median {us(np.median(a[:, 0] - t0)):.2f} max {us((a[:, 0] - t0).max()):.2f}; "
              f"end median {np.median(end):.2f}, 5 % {np.percentile(end, 5):.2f}, 95 % {np.percentile(end, 95):.2f}, max {end.max():.2f}")
        for k, name in ((1, "issuing the batches' requests"), (2, "waiting for blocks' words"), (3, "decode, turn, stores")):
            tot = us(a[:, k])
            print(f"  {name:32s} per wave: median {np.median(tot):6.2f}  [5 % {np.percentile(tot, 5):6.2f} .. 95 % {np.percentile(tot, 95):6.2f}]"
                  f"   per block {np.median(us(a[:, k]) / a[:, 11]):.2f}")
        # where the waves ran (HW_ID: compute unit bits 8-11, shader array bit 12, shader engine bits 13-15; XCC_ID bits 0-3)
        hw, xcc = a[:, 12], a[:, 13] & 0xF
        cu = xcc * 1000 + ((hw >> 13) & 7) * 100 + ((hw >> 12) & 1) * 50 + ((hw >> 8) & 0xF)
        ids, cnt = np.unique(cu, return_counts=True)
        for n in np.unique(cnt):
            sel = np.isin(cu, ids[cnt == n])
            print(f"  {np.sum(cnt == n):3d} compute units with {n // 2} workgroups: their waves end at median {np.median(end[sel]):.2f}, max {end[sel].max():.2f}")


if __name__ == "__main__":
    main()
