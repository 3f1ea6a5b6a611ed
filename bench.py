#!/usr/bin/env python3
"""Benchmark of the PCR decode path on one MI355X.

A step is one pass of the whole path (index, marker parse, unstuff, progressive Huffman decode
of scans 1..k, refinement, de-quantise, IDCT, chroma replication, YCbCr->RGB, store) over the
whole workload: 4096 variable-size progressive JPEGs in 4 records of 1024, record bytes already
resident in device memory.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--images N] [--no-cpu-baseline] [--no-baseline-files]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

# The records of a step are decoded on one HIP stream each.  HIP multiplexes its streams over
# GPU_MAX_HW_QUEUES hardware queues (default 4); with four, pairs of the record streams were measured to
# share a queue and run one after the other.  Sixteen queues give the four record streams and the four
# streams of the loader measured further down one each.  Must be set before the HIP runtime starts.
if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 16:
    os.environ["GPU_MAX_HW_QUEUES"] = "16"

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
SCAN_GROUPS = (1, 2, 5, 10)    # the scan groups the paper tabulates (Tables 1 and 2)
HEADLINE_K = 10


def scan_tables(files):
    """Per file: cumulative compressed bytes per scan; per image: geometry for byte accounting."""
    import pcrgen
    return np.array([pcrgen.split_scans(f) for f in files], dtype=np.int64)


def algorithmic_bytes(ends, shapes, k):
    """Bytes the method itself must move for scan group k (per image, summed):
    compressed prefix read once, each coefficient position covered by scans <= k written once and
    read once (2 bytes each), pixels written once.  10-scan 4:2:0 script: DC for all components
    at k=1, luma positions 1..5 at k=2, Cr 1..63 at k=3, Cb 1..63 at k=4, all luma from k=5."""
    comp = ends[:, k - 1].sum()
    out = 0
    touched = 0          # int16 elements
    for (W, H) in shapes:
        mx, my = -(-W // 16), -(-H // 16)
        yb, cb = 4 * mx * my, mx * my
        ycov = (1 if k >= 1 else 0) + (5 if k >= 2 else 0) + (58 if k >= 5 else 0)
        crcov = 1 + (63 if k >= 3 else 0)
        cbcov = 1 + (63 if k >= 4 else 0)
        touched += yb * ycov + cb * (crcov + cbcov)
        out += W * H * 3
    return dict(compressed=int(comp), touched=int(2 * touched), out=int(out),
                path=int(comp + 2 * 2 * touched + out), entropy=int(comp + 2 * touched))


# rocprofv3 counters of the dominant kernel, k_ac_refine, per launch (mean of its two launches per
# record: scans 6, 8, 9, then scan 10) for record 0 of the default workload at scan group 10; summaries
# under profiles/.  FETCH_SIZE reads 0.5 KiB per KiB a plain copy kernel fetches and WRITE_SIZE 1.0, so the
# fetch figure is scaled by 2.  They describe the kernel as it stood when they were taken and are set to
# None whenever k_ac_refine changes, until the counters are read again.
AC_REFINE_PMC = {
    "salu_insts_per_launch": 0.5 * (831.8e6 + 634.4e6),
    "valu_insts_per_launch": 0.5 * (267.3e6 + 207.4e6),
    "fetch_bytes_per_launch": 0.5 * (278348.8 + 240598.3) * 1024 * 2.0,
    "write_bytes_per_launch": 0.5 * (160126.8 + 103962.1) * 1024 * 1.0,
}
SALU_PEAK_GINSTS = 256 * 2.4      # one scalar instruction per cycle per compute unit, 256 CUs, 2.4 GHz
# all kernels of one decode of record 0 at scan group 10 (same counter run): scalar / vector instructions
RECORD0_INSTS = {"scalar": 2881.7e6, "vector": 1708.8e6}

# Algorithmic work of the entropy kernels: Huffman-coded symbols per launch, counted with the CPU build of the
# decoders (tests/host_emul) on record 0 of the default workload, and the scalar operations the serial chain of
# this design needs per symbol at the very least (fetch the packed word of the current bit offset, test it, take
# its length, add it to the position, apply the position update, test for the end of the block and of the
# window).  Everything else a symbol needs is data-parallel work of the lanes.
SYMBOLS_RECORD0 = {"dc_first": [3981894], "ac_first": [62868359], "ac_refine": [53792045, 46598601]}
CHAIN_OPS_PER_SYMBOL = 8


def dominant_kernel_roofline(args, ends0, alone_ms, over_ms, alone, n_img, probe):
    """Roofline object for k_ac_refine, the kernel with the largest share of the step at scan group 10
    (at scan groups without AC refinement scans: k_ac_first, else k_dc_first)."""
    k = args.scan_group
    name = "ac_refine" if alone["ac_refine"][1] else ("ac_first" if alone["ac_first"][1] else "dc_first")
    ms = alone_ms[name]
    # what the method itself makes this kernel move: the entropy-coded bytes of its scans, read once
    # (refinement scans of the 10-scan script: 6, 8, 9, 10; AC first: 2..5; DC first: 1)
    scans = {"ac_refine": [6, 8, 9, 10], "ac_first": [2, 3, 4, 5], "dc_first": [1]}[name]
    sizes = np.diff(np.concatenate([np.zeros((ends0.shape[0], 1), dtype=np.int64), ends0], axis=1), axis=1)
    launches_per_call = max(1, alone[name][1] // 3)
    alg = float(sum(sizes[:, j - 1].sum() for j in scans if j <= k)) / launches_per_call
    default = args.images == 4096 and k == HEADLINE_K and name == "ac_refine"
    pmc = AC_REFINE_PMC if default else None
    sym = (sum(SYMBOLS_RECORD0[name]) / len(SYMBOLS_RECORD0[name])) if (args.images == 4096 and k == HEADLINE_K) else None
    achieved = (CHAIN_OPS_PER_SYMBOL * sym / (ms * 1e-3) / 1e9) if sym else None
    out = {
        "kernel": "k_%s (one record of %d images decoded alone, mean of its %d launches per decode)" % (name, ends0.shape[0], launches_per_call),
        "bound": "alu",
        "achieved": achieved, "peak": SALU_PEAK_GINSTS, "unit": "G scalar operations/s",
        "frac": (achieved / SALU_PEAK_GINSTS) if achieved else None,
        "traffic": (pmc["fetch_bytes_per_launch"] + pmc["write_bytes_per_launch"]) if pmc else None,
        "algorithmic": {"symbols_per_launch": sym, "chain_operations_per_symbol": CHAIN_OPS_PER_SYMBOL,
                        "symbols_per_s": (sym / (ms * 1e-3)) if sym else None},
        "issued": {"scalar_insts_per_launch": pmc["salu_insts_per_launch"] if pmc else None,
                   "vector_insts_per_launch": pmc["valu_insts_per_launch"] if pmc else None,
                   "G_scalar_insts_per_s": (pmc["salu_insts_per_launch"] / (ms * 1e-3) / 1e9) if pmc else None,
                   "frac_of_peak": (pmc["salu_insts_per_launch"] / (ms * 1e-3) / 1e9 / SALU_PEAK_GINSTS) if pmc else None},
        "peak_measured": probe,
        "ms_per_launch": ms, "ms_per_launch_overlapped": over_ms[name],
        "hbm_view": {"algorithmic_bytes_per_launch": alg, "achieved_GBps": alg / (ms * 1e-3) / 1e9,
                     "frac_of_8TBps": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "note": "a serial Huffman decoder is bound by scalar-ALU issue (one wavefront per stream), not by HBM.  achieved = "
                "symbols per launch x the scalar operations the serial chain needs per symbol / the launch duration measured "
                "here with HIP events (record alone); peak = 256 CUs x 1 scalar instruction per cycle x 2.4 GHz; peak_measured "
                "= the library's dependent-scalar-chain probe in this run; issued = what the kernel really executes "
                "(rocprofv3 counters, profiles/)",
    }
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--images", type=int, default=4096, help="images of the workload to use (default: all 4096)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-baseline-files", action="store_true", help="skip the leg that decodes the same images as non-progressive files")
    ap.add_argument("--scan-group", type=int, default=HEADLINE_K)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain elementwise copy of 256 MiB (untimed), the yardstick for rocprofv3's FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the decode path shards by record with no exchange between GPUs, "
              "and this build runs on a single MI355X; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import pcrgen
    import paper_1911_00472_amd as pkg
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    pkg.lib()

    t0 = time.time()
    records, files = pcrgen.make_workload("imagenet_like", limit=args.images)
    Ws, Hs = pcrgen.workload_shapes("imagenet_like", limit=args.images)
    shapes = list(zip((int(w) for w in Ws), (int(h) for h in Hs)))
    ends = scan_tables(files)
    n_img = len(files)
    gen_s = time.time() - t0
    print("[bench] generated %d images (mean %.1f kB) in %d records, %.1f s" % (n_img, ends[:, -1].mean() / 1000, len(records), gen_s),
          file=sys.stderr, flush=True)

    t0 = time.perf_counter()
    handles = [pkg.pcr_open(r, 0) for r in records]
    torch.cuda.synchronize()
    open_ms = (time.perf_counter() - t0) * 1e3 / len(records)
    outs = [torch.empty(int(h.output_layout()[-1]), dtype=torch.uint8, device="cuda") for h in handles]
    # one stream per record: records are independent, so their kernels may overlap (default priority)
    streams = [torch.cuda.Stream() for _ in handles]

    def step(k):
        for h, o, st in zip(handles, outs, streams):
            h.decode_batch(k, out=o, stream=st.cuda_stream)

    if args.calibrate_copy:
        # a kernel that reads 256 MiB and writes 256 MiB, nothing else: what the HBM counters read for it
        # gives the factor by which the same counters of the decode kernels are scaled
        a = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 1, out=b)
        torch.cuda.synchronize()
        print("[bench] calibration copy: elementwise kernel, %d bytes read, %d bytes written" % (a.numel(), b.numel()), file=sys.stderr, flush=True)
        del a, b

    # ---- parity spot check against the oracle before anything is timed ----
    import oracle
    step(HEADLINE_K)
    torch.cuda.synchronize()
    lay = handles[0].output_layout()
    host = outs[0].cpu().numpy()
    for i in (0, 1, min(7, handles[0].n - 1)):
        _, p0, info = oracle.decode_record_image(records[0], i, HEADLINE_K, want_coef=False)
        got = host[int(lay[i]):int(lay[i + 1])].reshape(info.H, info.W, info.nc).astype(int)
        assert np.abs(got - p0).max() <= 1, "parity check failed for image %d" % i

    def timed(k, steps, warmup):
        for _ in range(warmup):
            step(k)
        torch.cuda.synchronize()
        for h in handles:
            h.enable_stage_timing(True)          # starts a new event history on every handle
        t = time.perf_counter()
        for _ in range(steps):
            step(k)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        # HIP events the library recorded on each record's own stream around every kernel of the timed
        # steps.  The records of a step overlap, so an interval here also holds the time a kernel spent
        # sharing the GPU with the other records' kernels.
        over = {n: [0.0, 0] for n in pkg.STAGE_NAMES}
        for h in handles:
            calls, hist = h.stage_ms_history()
            for n, (ms, launches) in hist.items():
                over[n][0] += ms
                over[n][1] += launches
        # the same with record 0 decoded ALONE on its stream: every kernel has the GPU to itself, which is
        # also what rocprofv3 reports (it serialises dispatches)
        handles[0].enable_stage_timing(True)
        for _ in range(3):
            handles[0].decode_batch(k, out=outs[0], stream=streams[0].cuda_stream)
        torch.cuda.synchronize()
        calls, alone = handles[0].stage_ms_history()
        return dt / steps, over, alone, calls

    # ---- fidelity upgrades: from the planes of scan group a to scan group b, decoding only the new scans ----
    def upgrade_step(k):
        for h, o, st in zip(handles, outs, streams):
            h.upgrade_batch(k, out=o, stream=st.cuda_stream)

    chain = [k for k in SCAN_GROUPS]
    reps = max(2, args.steps // 2)
    acc = {(a, b): 0.0 for a, b in zip(chain[:-1], chain[1:])}
    for _ in range(reps + 1):                                   # the first round warms the plans up
        step(chain[0])
        torch.cuda.synchronize()
        for a, b in zip(chain[:-1], chain[1:]):
            t = time.perf_counter()
            upgrade_step(b)
            torch.cuda.synchronize()
            if _ > 0:
                acc[(a, b)] += (time.perf_counter() - t) / reps

    # ---- from pinned host memory: upload of the prefix fidelity k needs + bind + decode, one loader slot per record ----
    # (the record bytes sit in the slots' pinned staging buffers before the clock starts: what a reader
    # with O_DIRECT would have put there; every step uploads them again and re-binds the slots' handles)
    streamed = {}
    cap = max(len(r) for r in records)
    with pkg.Loader(len(records), cap) as ld:
        for k in SCAN_GROUPS:
            need = []
            for j, rec in enumerate(records):
                ok, nb = pkg.prefix_length(rec[:24 + 8 * 64], k)
                assert ok
                need.append(nb)
                ld.staging(j)[:nb] = np.frombuffer(rec, np.uint8)[:nb]
            host_s = [0.0]

            def stream_step():
                for j in range(len(records)):
                    t1 = time.perf_counter()
                    ld.upload(j, need[j])
                    host_s[0] += time.perf_counter() - t1
                    ld.decode(j, k, outs[j])

            stream_step()
            for j in range(len(records)):
                ld.wait(j)
            reps_s = max(5, args.steps)
            host_s[0] = 0.0
            t = time.perf_counter()
            for _ in range(reps_s):
                stream_step()
            for j in range(len(records)):
                ld.wait(j)
            dt = (time.perf_counter() - t) / reps_s
            streamed[str(k)] = {"images_per_s": n_img / dt, "ms_per_step": dt * 1e3, "uploaded_MB_per_step": sum(need) / 1e6,
                                "host_to_device_GBps": sum(need) / dt / 1e9, "ms_per_step_inside_upload_calls": host_s[0] / reps_s * 1e3}
    torch.cuda.synchronize()

    # ---- training tail: decode, then one random box per image resized to 224 x 224, flipped, normalised, fp16 NCHW ----
    rng = np.random.default_rng(1911_00472)
    crop_t, tails = [], []
    box_bytes = 0
    for h in handles:
        bx = np.zeros((h.n, 5), np.int32)
        for i in range(h.n):
            W, H = h.image_info(i)[:2]
            area = rng.uniform(0.08, 1.0) * W * H                 # the usual random-resized-crop recipe
            ratio = np.exp(rng.uniform(np.log(3 / 4), np.log(4 / 3)))
            w = int(min(W, max(1, round(np.sqrt(area * ratio))))); hh = int(min(H, max(1, round(np.sqrt(area / ratio)))))
            bx[i] = (rng.integers(0, W - w + 1), rng.integers(0, H - hh + 1), w, hh, rng.integers(0, 2))
            box_bytes += w * hh * 3
        crop_t.append(torch.from_numpy(bx).cuda())
        tails.append(torch.empty((h.n, 3, 224, 224), dtype=torch.float16, device="cuda"))
    MEAN, ISTD = (0.485, 0.456, 0.406), (1 / 0.229, 1 / 0.224, 1 / 0.225)

    def tail_step(k):                                               # (one call: the pixel kernel skips strips outside the boxes)
        for h, o, st, c, t in zip(handles, outs, streams, crop_t, tails):
            h.decode_crop_batch(k, c, 224, 224, MEAN, ISTD, pixels=o, out=t, stream=st.cuda_stream)

    def tail_step_two_calls(k):
        for h, o, st, c, t in zip(handles, outs, streams, crop_t, tails):
            h.decode_batch(k, out=o, stream=st.cuda_stream)
            h.crop_resize_batch(o, c, 224, 224, MEAN, ISTD, out=t, stream=st.cuda_stream)

    tail_step(args.scan_group)
    torch.cuda.synchronize()
    reps_t = max(3, args.steps)
    t = time.perf_counter()
    for _ in range(reps_t):
        tail_step(args.scan_group)
    torch.cuda.synchronize()
    dt_tail = (time.perf_counter() - t) / reps_t
    tail_step_two_calls(args.scan_group)
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(reps_t):
        tail_step_two_calls(args.scan_group)
    torch.cuda.synchronize()
    dt_tail2 = (time.perf_counter() - t) / reps_t
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(streams[0]):
        e0.record()
        for _ in range(10):
            handles[0].crop_resize_batch(outs[0], crop_t[0], 224, 224, MEAN, ISTD, out=tails[0], stream=streams[0].cuda_stream)
        e1.record()
    torch.cuda.synchronize()
    tail_ms = e0.elapsed_time(e1) / 10
    tail_bytes = box_bytes / len(handles) + handles[0].n * 3 * 224 * 224 * 2
    training_tail = {"out": "float16 [n, 3, 224, 224]", "images_per_s_decode_plus_tail": n_img / dt_tail, "ms_per_step_decode_plus_tail": dt_tail * 1e3,
                     "ms_per_step_decode_then_tail_as_two_calls": dt_tail2 * 1e3,
                     "scan_group": args.scan_group, "tail_kernel_ms_per_record_alone": tail_ms,
                     "tail_kernel_algorithmic_GBps": tail_bytes / (tail_ms * 1e-3) / 1e9,
                     "tail_kernel_frac_of_hbm_peak": tail_bytes / (tail_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "note": "algorithmic bytes of the tail kernel: the pixels of each image's box read once + the half-precision output written once"}

    # ---- the whole input pipeline: pinned host bytes -> upload + bind -> decode -> crop / resize / normalise -> fp16 ----
    with pkg.Loader(len(records), cap) as ld:
        k = args.scan_group
        need = []
        for j, rec in enumerate(records):
            ok, nb = pkg.prefix_length(rec[:24 + 8 * 64], k)
            need.append(nb)
            ld.staging(j)[:nb] = np.frombuffer(rec, np.uint8)[:nb]

        def pipeline_step():
            for j in range(len(records)):
                ld.upload(j, need[j])
                ld.decode_crop(j, k, crop_t[j], 224, 224, MEAN, ISTD, outs[j], tails[j])

        pipeline_step()
        for j in range(len(records)):
            ld.wait(j)
        reps_p = max(5, args.steps)
        t = time.perf_counter()
        for _ in range(reps_p):
            pipeline_step()
        for j in range(len(records)):
            ld.wait(j)
        dt_pipe = (time.perf_counter() - t) / reps_p
    training_tail["images_per_s_from_pinned_host_memory"] = n_img / dt_pipe
    training_tail["ms_per_step_from_pinned_host_memory"] = dt_pipe * 1e3
    torch.cuda.synchronize()

    # ---- fidelity estimate: similarity of each scan group's pictures to the full ones (record 0) ----
    G0 = handles[0].G
    with torch.cuda.stream(streams[0]):
        full0 = handles[0].decode_batch(G0, stream=streams[0].cuda_stream).clone()
        scores0 = torch.empty(handles[0].n, dtype=torch.float32, device="cuda")
        mean_score = {}
        for k in [g for g in SCAN_GROUPS if g < G0]:
            handles[0].decode_batch(k, out=outs[0], stream=streams[0].cuda_stream)
            handles[0].msssim_batch(outs[0], full0, out=scores0, stream=streams[0].cuda_stream)
            mean_score[str(k)] = float(scores0.mean().item())
        e0.record()
        for _ in range(5):
            handles[0].msssim_batch(outs[0], full0, out=scores0, stream=streams[0].cuda_stream)
        e1.record()
    torch.cuda.synchronize()
    sim_ms = e0.elapsed_time(e1) / 5
    fidelity_estimate = {"measure": "multi-scale structural similarity on luma against scan group %d, mean over the record's images" % G0,
                         "mean_score_by_scan_group": mean_score, "ms_per_record": sim_ms,
                         "pixel_GBps": 2 * full0.numel() / (sim_ms * 1e-3) / 1e9,
                         "note": "pixel_GBps counts both batches read once; the kernel reads every scale from the uint8 pixels (about 5 x 1.7 reads with tile halos)"}
    del full0

    per_k = {}
    for k in SCAN_GROUPS:
        if k == args.scan_group:
            continue
        per_k[k] = timed(k, max(2, args.steps // 2), 1)
    per_k[args.scan_group] = timed(args.scan_group, args.steps, args.warmup)

    upgrades = {}
    for (a, b), sec_ab in acc.items():
        upgrades["%d->%d" % (a, b)] = {"ms_per_step": sec_ab * 1e3, "fresh_decode_ms_per_step": per_k[b][0] * 1e3}

    def per_launch(d):
        return {n: (ms / launches if launches else 0.0) for n, (ms, launches) in d.items()}

    report = {}
    for k in sorted(per_k):
        sec, over, alone, calls = per_k[k]
        ab = algorithmic_bytes(ends, shapes, k)
        report[str(k)] = {
            "images_per_s": n_img / sec,
            "ms_per_step": sec * 1e3,
            "output_GBps": ab["out"] / sec / 1e9,
            "algorithmic_GBps": ab["path"] / sec / 1e9,
            "hbm_roofline_frac": ab["path"] / sec / 1e9 / HBM_PEAK_GBS,
            "must_move_floor_GBps": (ab["compressed"] + ab["out"]) / sec / 1e9,
            "stage_ms_one_record_alone": {n: ms / calls for n, (ms, launches) in alone.items()},
            "kernel_ms_per_launch_alone": per_launch(alone),
            "kernel_ms_per_launch_overlapped": per_launch(over),
        }
    sec, over, alone, calls = per_k[args.scan_group]
    ab = algorithmic_bytes(ends, shapes, args.scan_group)
    n0 = handles[0].n
    # what the chip sustains on chains of dependent scalar instructions (the library's own probe kernel), best of
    # 8, 16 and 32 wavefronts per CU: the practical ceiling next to the nominal one
    probe = max(pkg.probe_scalar_issue_rate(w) for w in (8, 16, 32))
    # what a plain device-to-device copy reaches on this machine (the second denominator for the HBM figures)
    ca = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cb = torch.empty_like(ca)
    cb.copy_(ca)
    torch.cuda.synchronize()
    ce0, ce1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ce0.record()
    for _ in range(5):
        cb.copy_(ca)
    ce1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * ca.numel() / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    del ca, cb
    roofline = dominant_kernel_roofline(args, ends[:n0], per_launch(alone), per_launch(over), alone, n_img, probe)

    # (the two legs below come after everything the headline figures are taken from)
    # ---- the same images as baseline (non-progressive) files: what the decode of a progressive file costs over it ----
    baseline = None
    if not args.no_baseline_files:
        seq_records, seq_files = pcrgen.make_workload("imagenet_like", limit=args.images, script="sequential")
        seq_handles = [pkg.pcr_open(r, 0) for r in seq_records]
        torch.cuda.synchronize()

        def seq_step():
            for h, o, st in zip(seq_handles, outs, streams):
                h.decode_batch(1, out=o, stream=st.cuda_stream)

        seq_step()
        torch.cuda.synchronize()
        lay_s = seq_handles[0].output_layout()
        host = outs[0].cpu().numpy()
        for i in (0, min(5, seq_handles[0].n - 1)):
            _, p0, info = oracle.decode_record_image(seq_records[0], i, 1, want_coef=False)
            got = host[int(lay_s[i]):int(lay_s[i + 1])].reshape(info.H, info.W, info.nc).astype(int)
            assert np.abs(got - p0).max() <= 1, "parity check failed for baseline image %d" % i
        reps_b = max(5, args.steps)
        t = time.perf_counter()
        for _ in range(reps_b):
            seq_step()
        torch.cuda.synchronize()
        dt_seq = (time.perf_counter() - t) / reps_b
        seq_handles[0].enable_stage_timing(True)
        for _ in range(3):
            seq_handles[0].decode_batch(1, out=outs[0], stream=streams[0].cuda_stream)
        torch.cuda.synchronize()
        calls_b, alone_b = seq_handles[0].stage_ms_history()
        baseline = {"files": "the same %d images (same quantised coefficients) as sequential Huffman files, mean %.1f kB" % (n_img, np.mean([len(f) for f in seq_files]) / 1e3),
                    "images_per_s": n_img / dt_seq, "ms_per_step": dt_seq * 1e3,
                    "stage_ms_one_record_alone": {n: v[0] / calls_b for n, v in alone_b.items() if v[1]},
                    "note": "one wavefront per image (no restart intervals): a single pass, no refinement scans"}
        for h in seq_handles:
            h.close()
        del seq_handles, seq_records, seq_files

    # ---- the same images with restart intervals in every scan: more independent streams per image ----
    with_restarts = None
    if not args.no_baseline_files:
        RI = 128
        rst_records, rst_files = pcrgen.make_workload("imagenet_like", limit=args.images, restart=RI)
        rst_handles = [pkg.pcr_open(r, 0) for r in rst_records]
        torch.cuda.synchronize()
        rst_rates = {}
        for k in SCAN_GROUPS:
            def rst_step():
                for h, o, st in zip(rst_handles, outs, streams):
                    h.decode_batch(k, out=o, stream=st.cuda_stream)
            rst_step(); rst_step()
            torch.cuda.synchronize()
            if k == HEADLINE_K:
                host = outs[0].cpu().numpy()
                lay_r = rst_handles[0].output_layout()
                _, p0, info = oracle.decode_record_image(rst_records[0], 3, k, want_coef=False)
                got = host[int(lay_r[3]):int(lay_r[4])].reshape(info.H, info.W, info.nc).astype(int)
                assert np.abs(got - p0).max() <= 1, "parity check failed for the image with restart intervals"
            reps_r = max(5, args.steps)
            t = time.perf_counter()
            for _ in range(reps_r):
                rst_step()
            torch.cuda.synchronize()
            dt_r = (time.perf_counter() - t) / reps_r
            rst_handles[0].enable_stage_timing(True)
            for _ in range(3):
                rst_handles[0].decode_batch(k, out=outs[0], stream=streams[0].cuda_stream)
            torch.cuda.synchronize()
            calls_r, alone_r = rst_handles[0].stage_ms_history()
            rst_handles[0].enable_stage_timing(False)
            rst_rates[str(k)] = {"images_per_s": n_img / dt_r, "ms_per_step": dt_r * 1e3,
                                 "ms_one_record_alone": sum(v[0] for v in alone_r.values()) / calls_r}
        with_restarts = {"files": "the same %d images, same scans, a restart marker every %d MCUs of each scan; mean %.1f kB (%.2f %% more bytes)"
                                  % (n_img, RI, np.mean([len(f) for f in rst_files]) / 1e3, 100.0 * (sum(map(len, rst_files)) / float(ends[:, -1].sum()) - 1.0)),
                         "per_scan_group": rst_rates,
                         "note": "what an encoder that knows the decoder can add: each restart interval is a stream of its own, so one image's "
                                 "scan is decoded by several wavefronts; not the headline workload (stock encoders write no restart markers)"}
        for h in rst_handles:
            h.close()
        del rst_handles, rst_records, rst_files

    cpu = None
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        # bounded sample: every record of the workload once, a few seconds of wall time on 16 threads
        t = time.perf_counter()
        sample = 0
        for rec_bytes, h in zip(records, handles):
            oracle.decode_record(rec_bytes, args.scan_group, images=range(h.n), threads=threads, want_coef=False)
            sample += h.n
        dt = time.perf_counter() - t
        cpu = {"value": sample / dt, "unit": "images/s", "cores": threads, "kind": "oracle",
               "sample": "all %d images of the workload once at scan group %d, %d threads, %.1f s wall (%.0f CPU-seconds)"
                         % (sample, args.scan_group, threads, dt, dt * threads)}

    line = {
        "metric": "decoded_images_per_sec_at_scan_group_%d" % args.scan_group,
        "value": n_img / sec, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int16 coefficients, fp32 IDCT/colour, u8 pixels", "data": "synthetic",
        "config": {"workload": "imagenet_like: %d RGB images, width/height uniform in [300,500], 4:2:0, quality 90, "
                               "10-scan progressive, mean %.0f kB, %d records of <=1024" % (n_img, ends[:, -1].mean() / 1000, len(records)),
                   "scan_group": args.scan_group, "images": n_img, "records": len(records)},
        "output_GBps": ab["out"] / sec / 1e9,
        "open_ms_per_record": open_ms,
        "path_roofline": {"bound": "hbm", "achieved": ab["path"] / sec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": ab["path"] / sec / 1e9 / HBM_PEAK_GBS, "device_copy_GBps_measured": copy_gbps,
                          "frac_of_measured_copy": ab["path"] / sec / 1e9 / copy_gbps},
        "path_issue": ({"scalar_insts_per_step": RECORD0_INSTS["scalar"] * len(records), "vector_insts_per_step": RECORD0_INSTS["vector"] * len(records),
                        "G_scalar_insts_per_s": RECORD0_INSTS["scalar"] * len(records) / sec / 1e9,
                        "frac_of_peak": RECORD0_INSTS["scalar"] * len(records) / sec / 1e9 / SALU_PEAK_GINSTS,
                        "frac_of_measured_peak": RECORD0_INSTS["scalar"] * len(records) / sec / 1e9 / probe,
                        "note": "instructions of one record (rocprofv3 counters of record 0) x records, over the timed step: how "
                                "busy the scalar units are when the records overlap"}
                       if (args.images == 4096 and args.scan_group == HEADLINE_K) else None),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "per_scan_group": report,
        "fidelity_upgrade": upgrades,
        "from_pinned_host_memory": streamed,
        "training_tail": training_tail,
        "fidelity_estimate": fidelity_estimate,
        "baseline_sequential_files": baseline,
        "with_restart_intervals": with_restarts,
    }
    for h in handles:
        h.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
