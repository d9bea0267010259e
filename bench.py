#!/usr/bin/env python3
"""Benchmark of the whole decode path on one MI355X.

A step is one jpgd_decode_batch call over one synthetic workload: unstuff, synchronisation (intra and
inter), scan, write (with DC), pixels -- inputs already resident in HBM, outputs left in HBM.
Prints ONE JSON line (see README / DESIGN.md, "Measurement").

  python bench.py                       # benchmark configs[1]: one 1920x1088 4:4:4 q90 image
  python bench.py --config 5            # other workloads (1..5), for the notes in the design doc
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

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM bytes per launch (read + written) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for a plain copy of known size; taken from the summaries in profiles/ (same commands).
# Share of the chip's vector issue slots the kernel uses and lanes switched on per vector instruction, from the SQ
# counters in the same summaries (the entropy kernels are bound by dependent instruction issue, not by HBM).
MEASURED_ISSUE = {
    ("hd1088_444_q90", "sync_intra"): {"valu_issue_frac": 0.114, "lanes_per_valu_instr": 41.2},
    ("uhd16k_420_q92_flat_random", "sync_intra"): {"valu_issue_frac": 0.429, "lanes_per_valu_instr": 40.6},
}

MEASURED_TRAFFIC = {
    ("hd1088_444_q90", "sync_intra"): 1.747e6,
    ("hd1088_444_q90", "write"): 14.65e6,
    ("hd1088_444_q90", "pixels"): 18.89e6,
    ("uhd16k_420_q92_flat_random", "sync_intra"): 84.75e6,
    ("uhd16k_420_q92_flat_random", "write"): 1122.0e6,
    ("uhd16k_420_q92_flat_random", "pixels"): 796.3e6,
}


def algorithmic_bytes(kernel: str, Bs: int, B: int, S: int, K: int, out_bytes: int) -> int:
    """Bytes the method itself must move per launch ("Kernels"): Bs stuffed bytes, B unstuffed
    bytes, S subsequences (16-byte records), K data units (128 bytes of int16 each), out_bytes of pixels."""
    return {
        "unstuff_count": Bs,
        "unstuff_scan": 8 * (Bs // 4096 + 1),
        "unstuff_scatter": Bs + B,
        "sync_intra": B + 16 * S,
        "sync_inter": 16 * (S // 256 + 1),
        "scan_totals": 16 * S,
        "scan_prefix": 32 * (S // 256 + 1),
        "write": B + 16 * S + 128 * K,
        "pixels": 128 * K + out_bytes,
    }[kernel]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 of BASELINE.json (default 2 = configs[1])")
    ap.add_argument("--subseq-bits", type=int, default=0)
    ap.add_argument("--overlap", type=int, default=-1)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle timing; 0 skips it")
    ap.add_argument("--limit", type=int, default=0, help="images of the batch config to use (0 = all)")
    ap.add_argument("--restart-interval", type=int, default=0, metavar="MCUS",
                    help="encode the workload with restart markers every MCUS MCUs (-1 = one MCU row); the "
                         "configurations themselves have none")
    ap.add_argument("--quality", type=int, default=0,
                    help="encode the (single-image) workload at this quality instead of the configuration's")
    ap.add_argument("--planar", action="store_true",
                    help="component planes instead of RGB (JPGD_F_PLANAR): the paper's own output format")
    ap.add_argument("--include-h2d", action="store_true",
                    help="also time steps that first copy the compressed bytes from pinned host memory (reported as "
                         "'with_h2d'; never as 'value')")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of decoding, run plain device copies of this many MiB (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (nothing here is distributed)" % args.gpus,
              file=sys.stderr)
        return 2

    import torch
    import paper_2111_09219_amd as J
    from workloads import CONFIGS, config_jpeg
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the decoder has no CPU path", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "copies": 5, "gbs": round(2 * n / 1e9 / dt, 1)}))
        return 0

    c = args.config
    wl = CONFIGS[c]
    ri = args.restart_interval
    if ri < 0:
        mcu_w = 8 if wl["subsampling"] in ("gray", "444") else 16
        ri = (wl["width"] + mcu_w - 1) // mcu_w
    enc = config_jpeg(c, limit=args.limit or None, restart_interval=ri) if c == 4 else config_jpeg(c, restart_interval=ri, quality=args.quality or None)
    files = [e.data for e in enc] if isinstance(enc, list) else [enc.data]
    flags = J.F_PLANAR if args.planar else 0
    cfg = J.Config.make(subseq_bits=args.subseq_bits, overlap=None if args.overlap < 0 else args.overlap, flags=flags)
    batch = J.prepare_batch(files, cfg, device="cuda:0")
    Bs = batch.compressed_bytes
    pixels = batch.pixels_total
    K = int(sum(i.total_units for i in batch.infos))
    if args.planar:   # luma plane plus (ncomp - 1) chroma planes at their own resolution
        out_bytes = int(sum(i.width * i.height + (i.ncomp - 1) * (-(-i.width // i.hsamp[0])) * (-(-i.height // i.vsamp[0]))
                            for i in batch.infos))
    else:
        out_bytes = int(sum(i.width * i.height * i.ncomp for i in batch.infos))

    # warm-up; its last steps time every kernel to find the dominant one
    cfg_all = J.Config.make(subseq_bits=args.subseq_bits, overlap=None if args.overlap < 0 else args.overlap,
                            flags=flags, timing_mask=(1 << len(J.KERNELS)) - 1)
    split = np.zeros(len(J.KERNELS))
    nsplit = max(1, min(5, args.warmup))
    rep = None
    nwarm = max(args.warmup, nsplit + 1)
    for w in range(nwarm):
        if w >= nwarm - nsplit:   # the last warm-up steps: clocks and caches are settled by then
            rep = batch.decode(cfg=cfg_all)
            split += np.array(list(rep.kernel_ms))
        else:
            rep = batch.decode()
    split /= nsplit
    dominant = int(np.argmax(split))
    S = rep.n_subseq
    B = Bs  # unstuffed length is within 0.5 % of the stuffed one; the bound is used for the byte counts

    cfg_dom = J.Config.make(subseq_bits=args.subseq_bits, overlap=None if args.overlap < 0 else args.overlap,
                            flags=flags, timing_mask=1 << dominant)
    dom_ms = 0.0
    dom_launches = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        # the dominant kernel is bracketed with HIP events in every fourth step of the timed region: the two
        # event records cost the stream about ten microseconds, which is several percent of a small decode
        if k % 4 == 0:
            rep = batch.decode(cfg=cfg_dom)
            dom_ms += rep.kernel_ms[dominant]
            dom_launches += rep.launches[dominant]
        else:
            rep = batch.decode(cfg=cfg)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    mbps = Bs / 1e6 / (ms_per_step / 1e3)
    mpix = pixels / 1e6 / (ms_per_step / 1e3)

    with_h2d = None
    if args.include_h2d:
        host = batch.d_scans.cpu().pin_memory()
        for _ in range(5):
            batch.d_scans.copy_(host, non_blocking=True)
            batch.decode()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            batch.d_scans.copy_(host, non_blocking=True)
            batch.decode()
        torch.cuda.synchronize()
        ms_h = (time.perf_counter() - t1) * 1e3 / args.steps
        with_h2d = {"ms_per_step": round(ms_h, 5), "mb_per_s": round(Bs / 1e6 / (ms_h / 1e3), 2),
                    "note": "each step copies the compressed bytes from pinned host memory on the same stream first"}
        # the same with two sets of buffers: while one batch is decoded, the next one's bytes are copied on a
        # second stream (the decode call holds the host until its verdict, so the copy is enqueued before it)
        other = J.prepare_batch(files, cfg, device="cuda:0")
        sets = [batch, other]
        copy_stream = torch.cuda.Stream()
        ready = [torch.cuda.Event(), torch.cuda.Event()]
        done = [torch.cuda.Event(), torch.cuda.Event()]
        main = torch.cuda.current_stream()

        def enqueue_copy(k):
            with torch.cuda.stream(copy_stream):
                copy_stream.wait_event(done[k])          # the set's previous decode has finished reading
                sets[k].d_scans.copy_(host, non_blocking=True)
                ready[k].record(copy_stream)

        def pipelined(steps):
            for k in (0, 1):
                done[k].record(main)
            enqueue_copy(0)
            for i in range(steps):
                k = i & 1
                enqueue_copy(k ^ 1)
                main.wait_event(ready[k])
                sets[k].decode()
                done[k].record(main)
            torch.cuda.synchronize()

        pipelined(6)
        t2 = time.perf_counter()
        pipelined(args.steps)
        ms_o = (time.perf_counter() - t2) * 1e3 / args.steps
        with_h2d["overlapped_ms_per_step"] = round(ms_o, 5)
        with_h2d["overlapped_mb_per_s"] = round(Bs / 1e6 / (ms_o / 1e3), 2)
        # from the files, as the paper times it (Section 5: parsing, allocation and transfer included): header
        # parsing and packing of the entropy-coded segments on the host, tensors from torch's caching allocator
        # (after the first step an allocation is a look-up), copy from pageable memory, decode
        del other, sets
        n_files = max(3, min(args.steps, 30))
        for _ in range(2):
            J.prepare_batch(files, cfg, device="cuda:0").decode()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(n_files):
            J.prepare_batch(files, cfg, device="cuda:0").decode()
        torch.cuda.synchronize()
        ms_f = (time.perf_counter() - t3) * 1e3 / n_files
        with_h2d["from_files_ms_per_step"] = round(ms_f, 5)
        with_h2d["from_files_mb_per_s"] = round(Bs / 1e6 / (ms_f / 1e3), 2)

    dom_name = J.KERNELS[dominant]
    dom_avg_ms = dom_ms / max(1, dom_launches)
    alg = algorithmic_bytes(dom_name, Bs, B, S, K, out_bytes)
    achieved = alg / 1e9 / (dom_avg_ms / 1e3) if dom_avg_ms > 0 else 0.0

    kernels = {}
    for k, name in enumerate(J.KERNELS):
        if rep.launches[k] == 0:
            continue
        ab = algorithmic_bytes(name, Bs, B, S, K, out_bytes)
        kernels[name] = {"ms": round(float(split[k]), 5), "alg_bytes": ab,
                         "hbm_gbs": round(ab / 1e9 / (split[k] / 1e3), 2) if split[k] > 0 else None}

    cpu = None
    if args.cpu_seconds > 0:
        from oracle import OracleImage
        t_start = time.perf_counter()
        done_bytes = 0
        done_pixels = 0
        reps = 0
        imgs = files if len(files) > 1 else files * 1000
        for f in imgs:
            o = OracleImage(f)
            coef = o.coefficients()
            o.pixels(coef)
            done_bytes += int(o.info.scan_len)
            done_pixels += o.width * o.height
            reps += 1
            if time.perf_counter() - t_start > args.cpu_seconds:
                break
        cpu_dt = time.perf_counter() - t_start
        cpu = {"value": round(done_bytes / 1e6 / cpu_dt, 3), "unit": "MB/s", "cores": 1, "kind": "oracle",
               "mpixel_per_s": round(done_pixels / 1e6 / cpu_dt, 3),
               "sample": "%d full decode(s) (entropy decode + double-precision pixels) of the same file(s), %.1f s, "
                         "single thread" % (reps, cpu_dt)}

    line = {
        "metric": "compressed MB/s per image (whole decode path, data resident in HBM)",
        "value": round(mbps, 2),
        "unit": "MB/s",
        "mpixel_per_s": round(mpix, 2),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32 bit-parsing + fp32 IDCT (int16 coefficients, u8 pixels)",
        "data": "synthetic",
        "config": {"workload": "configs[%d] %s: %d image(s) %dx%d %s q%s%s, %d compressed bytes" % (
            c - 1, wl["name"], len(files), wl["width"], wl["height"], wl["subsampling"], wl["quality"],
            (" optimized Huffman" if wl["optimize"] else "") + (" restart interval %d MCUs" % ri if ri else "") + (" re-encoded at q%d" % args.quality if args.quality else ""), Bs),
            "subseq_bits": rep.subseq_bits, "subsequences": S, "sequences": rep.n_sequences,
            "inter_rounds": rep.inter_rounds, "redo": rep.redo, "output": "planes" if args.planar else "rgb"},
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                     "traffic": MEASURED_TRAFFIC.get((wl["name"], dom_name)) if not (args.subseq_bits or ri or args.quality) else None,
                     "issue": MEASURED_ISSUE.get((wl["name"], dom_name)) if not (args.subseq_bits or ri or args.quality) else None,
                     "avg_launch_ms": round(dom_avg_ms, 5), "timed_launches": dom_launches,
                     "alg_bytes_per_launch": alg},
        "cpu_baseline": cpu,
        "kernels": kernels,
        "with_h2d": with_h2d,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
