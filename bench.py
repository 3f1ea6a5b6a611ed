#!/usr/bin/env python3
"""Benchmark of the PCR decode path on one MI355X.

A step is one pass of the whole path (index, marker parse, unstuff, progressive Huffman decode of scans 1..k,
refinement, de-quantise, IDCT, chroma replication, YCbCr->RGB, store) over the whole workload, record bytes already
resident in device memory, every record on a HIP stream of its own.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--scan-group k] [--images N]
                    [--extras] [--no-cpu-baseline] [--no-default-queues]

Workloads (synthetic stand-ins for the paper's datasets, Table 1 / Table 3):
    imagenet_like (default, the headline)  4096 RGB images 300..500 px, 4:2:0, 4 records, scan groups 1..10
    rgb256        1024 RGB 256 x 256, 1 record, scan groups 1..10
    gray64        64 gray 64 x 64, 1 record, scan groups 1, 3, 6
    hires1024     1024 RGB 1024 x 1024 with a restart interval per MCU row, 8 records, scan groups 1, 5, 10
    ham_like      2048 RGB 600 x 450, 4:4:4, quality 95, 2 records, scan groups 1..10; also streamed from pinned host
                  memory with the record parsed on the device
"""
import argparse
import json
import os
import subprocess
import sys
import tempfile
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# The records of a step are decoded on one HIP stream each.  HIP multiplexes its streams over GPU_MAX_HW_QUEUES
# hardware queues (default 4); streams that share a queue run one after the other.  Sixteen queues give every record
# stream (and the loader's) one of its own.  Must be set before the HIP runtime starts; `--keep-queues` (used by the
# child process that measures HIP's default) leaves the environment alone.
if "--keep-queues" not in sys.argv and int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 16:
    os.environ["GPU_MAX_HW_QUEUES"] = "16"

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
SALU_PEAK_GINSTS = 256 * 2.4   # one scalar instruction per cycle per compute unit, 256 CUs, 2.4 GHz
WORKLOAD_SCAN_GROUPS = {"imagenet_like": tuple(range(1, 11)), "rgb256": tuple(range(1, 11)), "gray64": (1, 3, 6),
                        "hires1024": (1, 5, 10), "ham_like": tuple(range(1, 11))}
TABLE_SCAN_GROUPS = (1, 2, 5, 10)     # the scan groups the paper tabulates (Tables 1 and 2)

VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12   # vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane operations/s
                                                    # (the chip's 157.3 TFLOP/s of packed fp32 FMA is this figure x 2 x 2)

# rocprofv3 counters of the kernels of ONE decode of record 0 of the default workload at scan group 10, read off the
# summaries under profiles/ (which give the commands).  FETCH_SIZE reads 0.5 KiB per KiB a plain copy kernel fetches
# and WRITE_SIZE 1.0 (profiles/), so fetched bytes are the counter x 2.  They describe the kernels as they stood when
# the counters were taken: an entry is removed (-> null in the output) whenever its kernel changes.
PMC = {
    # mean of the two launches of one decode (profiles/decode_kernels_imagenet_like_k10_counters.md)
    "ac_refine_lanes": {"salu": 36.4e6, "valu": 160.6e6, "fetch_bytes": 499.5e6, "write_bytes": 324.6e6,
                        "source": "profiles/decode_kernels_imagenet_like_k10_counters.md (SQ_INSTS_SALU, SQ_INSTS_VALU, FETCH_SIZE x 2.0, WRITE_SIZE x 1.0)"},
}
# all kernels of that decode, same counter run
RECORD0_INSTS = {"scalar": 228.5e6, "vector": 764.3e6, "source": "profiles/decode_kernels_imagenet_like_k10_counters.md (whole decode)"}

# The work of one Huffman-coded symbol, at the very least.
# One wavefront per unit (pcr_entropy.h): the serial chain -- fetch the packed word of the current bit offset, test it,
# take its length, add it to the position, apply the position update, test for the end of the block and of the window
# (8 scalar operations); everything else a symbol needs is data-parallel work of the lanes.
CHAIN_OPS_PER_SYMBOL = 8
# One lane per unit (pcr_lanes.h), in operations of that lane.  AC first scan: window, table index, look-up, split the
# entry into length / run / size (3), the appended bits (2), their sign extension (3), position, element address (2),
# point transform, store, buffer advance (3), end-of-band test (2): 21.  AC refinement: window, index, look-up, split
# (3), zeros from the position on (2), the n-th of them by halving a 64-bit mask (6 x 3), the new coefficient's bit and
# sign (4), the history positions passed: mask and count (4), their correction bits: extract and merge (5), buffer
# advance (3), position, end-of-block test: 46.
LANE_OPS_PER_SYMBOL = {"ac_first": 21, "ac_refine": 46}


def read_scan_script(jpeg):
    """[(components, Ss, Se, Ah, Al)] of a file's scans and its component sampling factors, from its SOF / SOS headers."""
    p, comps, scans = 2, {}, []
    order = []
    while p + 4 <= len(jpeg):
        assert jpeg[p] == 0xFF
        m = jpeg[p + 1]
        if m == 0xFF:
            p += 1
            continue
        if m == 0xD9:
            break
        L = int.from_bytes(jpeg[p + 2:p + 4], "big")
        s = p + 4
        if m in (0xC0, 0xC1, 0xC2):
            for c in range(jpeg[s + 5]):
                comps[jpeg[s + 6 + 3 * c]] = (jpeg[s + 7 + 3 * c] >> 4, jpeg[s + 7 + 3 * c] & 15)
                order.append(jpeg[s + 6 + 3 * c])
        p += 2 + L
        if m == 0xDA:
            ns = jpeg[s]
            cs = [order.index(jpeg[s + 1 + 2 * j]) for j in range(ns)]
            scans.append((cs, jpeg[s + 1 + 2 * ns], jpeg[s + 2 + 2 * ns], jpeg[s + 3 + 2 * ns] >> 4, jpeg[s + 3 + 2 * ns] & 15))
            while True:                                   # skip the entropy-coded data
                p = jpeg.index(b"\xff", p)
                if jpeg[p + 1] == 0 or 0xD0 <= jpeg[p + 1] <= 0xD7 or jpeg[p + 1] == 0xFF:
                    p += 2 if jpeg[p + 1] != 0xFF else 1
                    continue
                break
    return scans, [comps[c] for c in order]


def algorithmic_bytes(ends, shapes, script, sampling, k):
    """Bytes the method itself must move for scan group k (summed over the images): compressed prefix read once, each
    coefficient position covered by scans <= k written once and read once (2 bytes each), pixels written once."""
    nc = len(sampling)
    hmax, vmax = max(h for h, _ in sampling), max(v for _, v in sampling)
    cov = [set() for _ in range(nc)]
    for cs, Ss, Se, Ah, Al in script[:k]:
        for c in cs:
            cov[c].update(range(Ss, Se + 1))
    comp = int(ends[:, min(k, ends.shape[1]) - 1].sum())
    out = touched = 0
    for (W, H) in shapes:
        mx, my = -(-W // (8 * hmax)), -(-H // (8 * vmax))
        for c in range(nc):
            touched += mx * sampling[c][0] * my * sampling[c][1] * len(cov[c])
        out += W * H * nc
    return dict(compressed=comp, touched=int(2 * touched), out=int(out), path=int(comp + 2 * 2 * touched + out), entropy=int(comp + 2 * touched))


def scan_levels(script):
    """Dependency level (1-based) of every scan: one more than the deepest earlier scan that shares a component and
    overlaps in band -- the launches of the entropy kernels follow these levels."""
    lv = []
    for g, (cs, Ss, Se, Ah, Al) in enumerate(script):
        d = 1
        for q in range(g):
            cq, sq, eq, _, _ = script[q]
            if set(cs) & set(cq) and sq <= Se and Ss <= eq:
                d = max(d, lv[q] + 1)
        lv.append(d)
    return lv


def stage_of(scan):
    cs, Ss, Se, Ah, Al = scan
    if Ss == 0 and Se == 63:
        return "sequential"
    if Ss == 0:
        return "dc_first" if Ah == 0 else None            # DC refinement has no serial decode
    return "ac_first" if Ah == 0 else "ac_refine"


class Job:
    """One workload resident on the device: handles, output buffers, one stream per record."""

    lane_decoders = 0                                       # --lane-decoders: pcr_set_lane_decoders of every handle (0: the library's choice)

    def __init__(self, torch, pkg, records, on_device=False):
        self.torch, self.pkg, self.records = torch, pkg, records
        t0 = time.perf_counter()
        if on_device:                                       # bytes already in device memory: index and markers parsed on the device
            self.dev = [torch.frombuffer(bytearray(r), dtype=torch.uint8).cuda() for r in records]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.handles = [pkg.pcr_open_device(d) for d in self.dev]
        else:
            self.handles = [pkg.pcr_open(r, 0) for r in records]
        torch.cuda.synchronize()
        self.open_ms = (time.perf_counter() - t0) * 1e3 / len(records)
        for h in self.handles:
            h.set_lane_decoders(Job.lane_decoders)
        self.outs = [torch.empty(int(h.output_layout()[-1]), dtype=torch.uint8, device="cuda") for h in self.handles]
        self.streams = [torch.cuda.Stream() for _ in self.handles]          # default priority
        self.n_img = sum(h.n for h in self.handles)

    def step(self, k):
        for h, o, st in zip(self.handles, self.outs, self.streams):
            h.decode_batch(k, out=o, stream=st.cuda_stream)

    def close(self):
        for h in self.handles:
            h.close()

    def timed(self, k, steps, warmup, single_steps=10):
        """(mean s per step over `steps` steps in one bracket, [s of single steps], stage times overlapped, stage times
        of record 0 decoded alone, calls)."""
        torch, pkg = self.torch, self.pkg
        for _ in range(warmup):
            self.step(k)
        torch.cuda.synchronize()
        for h in self.handles:
            h.enable_stage_timing(False)
        t = time.perf_counter()
        for _ in range(steps):
            self.step(k)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t) / steps
        singles = []
        for _ in range(single_steps):
            t = time.perf_counter()
            self.step(k)
            torch.cuda.synchronize()
            singles.append(time.perf_counter() - t)
        # HIP events the library records on each record's own stream around every kernel.  The records of a step
        # overlap, so an interval here also holds the time a kernel spent sharing the GPU with the other records'.
        for h in self.handles:
            h.enable_stage_timing(True)
        for _ in range(3):
            self.step(k)
        torch.cuda.synchronize()
        over = {n: [0.0, 0] for n in pkg.STAGE_NAMES}
        for h in self.handles:
            calls, hist = h.stage_ms_history()
            for n, (ms, launches) in hist.items():
                over[n][0] += ms
                over[n][1] += launches
        # the same with record 0 decoded ALONE: every kernel has the GPU to itself (what rocprofv3 reports as well)
        h0 = self.handles[0]
        h0.enable_stage_timing(True)
        for _ in range(3):
            h0.decode_batch(k, out=self.outs[0], stream=self.streams[0].cuda_stream)
        torch.cuda.synchronize()
        calls, alone = h0.stage_ms_history()
        for h in self.handles:
            h.enable_stage_timing(False)
        return dt, singles, over, alone, calls


def per_launch(d):
    return {n: (ms / launches if launches else 0.0) for n, (ms, launches) in d.items()}


def dominant_kernel_roofline(workload, k, script, symbols0, ends0, alone, calls, over, probe, default_config, lanes):
    """Roofline object for the kernel with the largest share of a record's decode at scan group k.  lanes: the AC scans were
    decoded with one lane per unit (else one wavefront per unit)."""
    stage_ms = {n: ms / calls for n, (ms, launches) in alone.items()}
    name = max(stage_ms, key=lambda n: stage_ms[n])
    launches_per_call = max(1, alone[name][1] // calls)
    ms = alone[name][0] / max(1, alone[name][1])
    over_ms = per_launch(over)[name]
    entropy = name in ("dc_first", "ac_first", "ac_refine", "sequential")
    by_lane = lanes and name in LANE_OPS_PER_SYMBOL
    scans = [g for g, sc in enumerate(script[:k]) if stage_of(sc) == name]
    sizes = np.diff(np.concatenate([np.zeros((ends0.shape[0], 1), dtype=np.int64), ends0], axis=1), axis=1)
    alg_bytes = float(sum(sizes[:, g].sum() for g in scans)) / launches_per_call if entropy else None
    sym = (float(sum(symbols0[:, g].sum() for g in scans)) / launches_per_call) if (entropy and symbols0 is not None) else None
    pmc = PMC.get(name + ("_lanes" if by_lane else "")) if default_config else None
    out = {"kernel": "k_%s%s (record 0 decoded alone, mean of its %d launches per decode)" % (name, "_lanes" if by_lane else "", launches_per_call),
           "share_of_a_lone_record_decode": stage_ms[name] / sum(stage_ms.values()),
           "ms_per_launch": ms, "ms_per_launch_overlapped": over_ms, "peak_measured_G_scalar_insts_per_s": probe}
    hbm_view = ({"algorithmic_bytes_per_launch": alg_bytes, "achieved_GBps": alg_bytes / (ms * 1e-3) / 1e9,
                 "frac_of_8TBps": alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "note": "the entropy-coded bytes of the launch's scans, read once"} if entropy else None)
    if by_lane:
        ops = LANE_OPS_PER_SYMBOL[name]
        achieved = ops * sym / (ms * 1e-3) / 1e12 if sym else None
        out.update({
            "bound": "alu", "achieved": achieved, "peak": VALU_PEAK_TLANEOPS, "unit": "T lane operations/s",
            "frac": achieved / VALU_PEAK_TLANEOPS if achieved else None,
            "frac_is": "algorithmic vector-lane operations (symbols x %d operations of the lane that decodes them) / launch duration / vector "
                       "ALU peak (256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz).  A lane-per-unit launch on its own is bound by the latency of one "
                       "symbol after another in its longest unit, not by issue: what it leaves idle the decodes of the other records use "
                       "(ms_per_launch_overlapped; path_issue gives the whole step); `issued` gives the same launch by executed instructions" % ops,
            "traffic": (pmc["fetch_bytes"] + pmc["write_bytes"]) if pmc else None,
            "algorithmic": {"symbols_per_launch": sym, "lane_operations_per_symbol": ops,
                            "symbols_per_s": sym / (ms * 1e-3) if sym else None,
                            "source": "pcrgen.workload_symbol_counts (the encoder's own count of the Huffman-coded symbols of the scans of this launch)"},
            "issued": ({"vector_insts_per_launch": pmc["valu"], "scalar_insts_per_launch": pmc["salu"],
                        "vector_insts_per_symbol_per_lane": pmc["valu"] * 64 / sym if sym else None,
                        "T_lane_operations_per_s": pmc["valu"] * 64 / (ms * 1e-3) / 1e12,
                        "frac_of_peak": pmc["valu"] * 64 / (ms * 1e-3) / 1e12 / VALU_PEAK_TLANEOPS, "source": pmc["source"]} if pmc else None),
            "hbm_view": hbm_view,
        })
    elif entropy:
        achieved = CHAIN_OPS_PER_SYMBOL * sym / (ms * 1e-3) / 1e9 if sym else None
        out.update({
            "bound": "alu", "achieved": achieved, "peak": SALU_PEAK_GINSTS, "unit": "G scalar operations/s",
            "frac": achieved / SALU_PEAK_GINSTS if achieved else None,
            "frac_is": "algorithmic scalar operations (symbols x %d operations of the serial chain) / launch duration / nominal scalar "
                       "issue peak (256 CUs x 1 per cycle x 2.4 GHz); `issued` and `hbm_view` give the same launch by executed "
                       "instructions and by algorithmic bytes" % CHAIN_OPS_PER_SYMBOL,
            "traffic": (pmc["fetch_bytes"] + pmc["write_bytes"]) if pmc else None,
            "algorithmic": {"symbols_per_launch": sym, "chain_operations_per_symbol": CHAIN_OPS_PER_SYMBOL,
                            "symbols_per_s": sym / (ms * 1e-3) if sym else None,
                            "source": "pcrgen.workload_symbol_counts (the encoder's own count of the Huffman-coded symbols of the scans of this launch)"},
            "issued": ({"scalar_insts_per_launch": pmc["salu"], "vector_insts_per_launch": pmc["valu"],
                        "scalar_insts_per_symbol": pmc["salu"] / sym if sym else None,
                        "G_scalar_insts_per_s": pmc["salu"] / (ms * 1e-3) / 1e9,
                        "frac_of_peak": pmc["salu"] / (ms * 1e-3) / 1e9 / SALU_PEAK_GINSTS, "source": pmc["source"]} if pmc else None),
            "hbm_view": hbm_view,
        })
    else:                                                   # a data-parallel kernel: bytes against HBM (achieved is filled in by the caller)
        out.update({"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                    "frac_is": "algorithmic bytes of the kernel / launch duration / 8 TB/s",
                    "traffic": (pmc["fetch_bytes"] + pmc["write_bytes"]) if pmc else None})
    return out, name


def oracle_rates(oracle, records, k, threads, per_record):
    """Oracle images/s at scan group k on the first `per_record` images of every record."""
    t = time.perf_counter()
    n = 0
    for rec in records:
        cnt = min(per_record, oracle.record_header(rec)["n"])
        oracle.decode_record(rec, k, images=range(cnt), threads=threads, want_coef=False)
        n += cnt
    dt = time.perf_counter() - t
    return n / dt, n, dt


def measure_default_queues(records, k, steps, warmup):
    """The same step in a child process that leaves GPU_MAX_HW_QUEUES at HIP's default (4): what a program measures
    that does not set it.  The records travel through a temporary file."""
    with tempfile.TemporaryDirectory() as tmp:
        path = os.path.join(tmp, "records.bin")
        with open(path, "wb") as f:
            for r in records:
                f.write(len(r).to_bytes(8, "little"))
                f.write(r)
        env = dict(os.environ)
        env.pop("GPU_MAX_HW_QUEUES", None)
        try:
            out = subprocess.run([sys.executable, os.path.abspath(__file__), "--keep-queues", "--child-records", path, "--scan-group", str(k), "--lane-decoders", str(Job.lane_decoders),
                                  "--steps", str(steps), "--warmup", str(warmup)], env=env, capture_output=True, text=True, timeout=300)
            return json.loads(out.stdout.strip().splitlines()[-1])
        except Exception as e:                              # the figure is a side note: never fail the benchmark over it
            return {"error": repr(e)[:200]}


def child_main(args):
    import torch
    import paper_1911_00472_amd as pkg
    records = []
    with open(args.child_records, "rb") as f:
        while True:
            head = f.read(8)
            if len(head) < 8:
                break
            records.append(f.read(int.from_bytes(head, "little")))
    job = Job(torch, pkg, records)
    for _ in range(args.warmup):
        job.step(args.scan_group)
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(args.steps):
        job.step(args.scan_group)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t) / args.steps
    job.close()
    print(json.dumps({"GPU_MAX_HW_QUEUES": os.environ.get("GPU_MAX_HW_QUEUES", "unset (HIP default 4)"), "ms_per_step": dt * 1e3,
                      "images_per_s": job.n_img / dt}))


def streamed_from_pinned(torch, pkg, records, outs, scan_groups, n_img, steps):
    """From pinned host memory: upload of the prefix fidelity k needs + bind (index and markers parsed on the device)
    + decode, one loader slot per record; every step uploads the bytes again and re-binds the slots' handles."""
    streamed = {}
    cap = max(len(r) for r in records)
    with pkg.Loader(len(records), cap) as ld:
        for k in scan_groups:
            need = []
            for j, rec in enumerate(records):
                ok, nb = pkg.prefix_length(rec[:24 + 8 * 64], k)
                assert ok
                need.append(nb)
                ld.staging(j)[:nb] = np.frombuffer(rec, np.uint8)[:nb]

            def stream_step():
                for j in range(len(records)):
                    ld.upload(j, need[j])
                    ld.decode(j, k, outs[j])

            stream_step()
            for j in range(len(records)):
                ld.wait(j)
            reps = max(5, steps)
            t = time.perf_counter()
            for _ in range(reps):
                stream_step()
            for j in range(len(records)):
                ld.wait(j)
            dt = (time.perf_counter() - t) / reps
            streamed[str(k)] = {"images_per_s": n_img / dt, "ms_per_step": dt * 1e3, "uploaded_MB_per_step": sum(need) / 1e6,
                                "host_to_device_GBps": sum(need) / dt / 1e9}
    torch.cuda.synchronize()
    return streamed


def extras(torch, pkg, pcrgen, oracle, job, args, ends, per_k_ms, k):
    """Measurements beyond the decode path proper (fidelity upgrade, training tail, similarity scores, the same images
    as baseline files and with restart intervals); imagenet_like only, with --extras."""
    handles, outs, streams, records, n_img = job.handles, job.outs, job.streams, job.records, job.n_img
    res = {}
    chain = list(TABLE_SCAN_GROUPS)
    reps = max(2, args.steps // 2)
    acc = {(a, b): 0.0 for a, b in zip(chain[:-1], chain[1:])}
    for it in range(reps + 1):                                   # the first pass warms the plans up
        job.step(chain[0])
        torch.cuda.synchronize()
        for a, b in zip(chain[:-1], chain[1:]):
            t = time.perf_counter()
            for h, o, st in zip(handles, outs, streams):
                h.upgrade_batch(b, out=o, stream=st.cuda_stream)
            torch.cuda.synchronize()
            if it > 0:
                acc[(a, b)] += (time.perf_counter() - t) / reps
    res["fidelity_upgrade"] = {"%d->%d" % ab: {"ms_per_step": s * 1e3, "fresh_decode_ms_per_step": per_k_ms.get(ab[1])} for ab, s in acc.items()}

    # the same step with every record's decode call captured into a HIP graph (one replay per record instead of 6 - 14
    # kernel launches): what the launch overhead is worth at each scan group
    graphed = {}
    for kk in TABLE_SCAN_GROUPS:
        job.step(kk)
        torch.cuda.synchronize()
        graphs = []
        for h, o, st in zip(handles, outs, streams):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                h.decode_batch(kk, out=o, stream=st.cuda_stream)
            graphs.append(g)
        torch.cuda.synchronize()

        def replay_all():                                           # (a replay runs on the current stream: each record on its own)
            for g, st in zip(graphs, streams):
                with torch.cuda.stream(st):
                    g.replay()
        replay_all()
        torch.cuda.synchronize()
        reps_g = max(5, args.steps)
        t = time.perf_counter()
        for _ in range(reps_g):
            replay_all()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t) / reps_g
        graphed[str(kk)] = {"ms_per_step": dt * 1e3, "images_per_s": n_img / dt, "eager_ms_per_step": per_k_ms.get(kk)}
        del graphs
    res["decode_calls_replayed_from_graphs"] = graphed

    # training tail: one random box per image resized to 224 x 224, flipped, normalised, fp16 NCHW
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
    def tail_step():                                               # one kernel: the full-resolution pixels never reach memory
        for h, st, c, t in zip(handles, streams, crop_t, tails):
            h.decode_crop_batch(k, c, 224, 224, MEAN, ISTD, pixels=None, out=t, stream=st.cuda_stream)

    def tail_step_working_buffer():
        for h, o, st, c, t in zip(handles, outs, streams, crop_t, tails):
            h.decode_crop_batch(k, c, 224, 224, MEAN, ISTD, pixels=o, out=t, stream=st.cuda_stream)

    def tail_step_two_calls():
        for h, o, st, c, t in zip(handles, outs, streams, crop_t, tails):
            h.decode_batch(k, out=o, stream=st.cuda_stream)
            h.crop_resize_batch(o, c, 224, 224, MEAN, ISTD, out=t, stream=st.cuda_stream)

    times = []
    for fn in (tail_step, tail_step_working_buffer, tail_step_two_calls):
        fn()
        torch.cuda.synchronize()
        reps_t = max(3, args.steps)
        t = time.perf_counter()
        for _ in range(reps_t):
            fn()
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t) / reps_t)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(streams[0]):
        e0.record()
        for _ in range(10):
            handles[0].crop_resize_batch(outs[0], crop_t[0], 224, 224, MEAN, ISTD, out=tails[0], stream=streams[0].cuda_stream)
        e1.record()
    torch.cuda.synchronize()
    tail_ms = e0.elapsed_time(e1) / 10
    tail_bytes = box_bytes / len(handles) + handles[0].n * 3 * 224 * 224 * 2
    res["training_tail"] = {"out": "float16 [n, 3, 224, 224]", "scan_group": k, "images_per_s_decode_plus_tail": n_img / times[0],
                            "ms_per_step_decode_plus_tail": times[0] * 1e3, "ms_per_step_through_a_working_buffer": times[1] * 1e3,
                            "ms_per_step_decode_then_tail_as_two_calls": times[2] * 1e3,
                            "tail_kernel_ms_per_record_alone": tail_ms, "tail_kernel_algorithmic_GBps": tail_bytes / (tail_ms * 1e-3) / 1e9,
                            "tail_kernel_frac_of_hbm_peak": tail_bytes / (tail_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    cap = max(len(r) for r in records)
    with pkg.Loader(len(records), cap) as ld:
        need = []
        for j, rec in enumerate(records):
            ok, nb = pkg.prefix_length(rec[:24 + 8 * 64], k)
            need.append(nb)
            ld.staging(j)[:nb] = np.frombuffer(rec, np.uint8)[:nb]

        def pipeline_step():
            for j in range(len(records)):
                ld.upload(j, need[j])
                ld.decode_crop(j, k, crop_t[j], 224, 224, MEAN, ISTD, None, tails[j])

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
    res["training_tail"]["images_per_s_from_pinned_host_memory"] = n_img / dt_pipe
    torch.cuda.synchronize()

    # fidelity estimate: similarity of each scan group's pictures to the full ones (record 0)
    G0 = handles[0].G
    with torch.cuda.stream(streams[0]):
        full0 = handles[0].decode_batch(G0, stream=streams[0].cuda_stream).clone()
        scores0 = torch.empty(handles[0].n, dtype=torch.float32, device="cuda")
        mean_score = {}
        for kk in [g for g in TABLE_SCAN_GROUPS if g < G0]:
            handles[0].decode_batch(kk, out=outs[0], stream=streams[0].cuda_stream)
            handles[0].msssim_batch(outs[0], full0, out=scores0, stream=streams[0].cuda_stream)
            mean_score[str(kk)] = float(scores0.mean().item())
        e0.record()
        for _ in range(5):
            handles[0].msssim_batch(outs[0], full0, out=scores0, stream=streams[0].cuda_stream)
        e1.record()
    torch.cuda.synchronize()
    res["fidelity_estimate"] = {"measure": "multi-scale structural similarity on luma against scan group %d, mean over record 0" % G0,
                                "mean_score_by_scan_group": mean_score, "ms_per_record": e0.elapsed_time(e1) / 5}
    # ... and with the smoothing of DC-only components, which matters at the first scan group (luma is DC-only there)
    with torch.cuda.stream(streams[0]):
        handles[0].decode_batch_smooth(1, out=outs[0], stream=streams[0].cuda_stream)
        handles[0].msssim_batch(outs[0], full0, out=scores0, stream=streams[0].cuda_stream)
        smooth_score = float(scores0.mean().item())
    torch.cuda.synchronize()
    t = time.perf_counter()
    reps_s = max(5, args.steps)
    for _ in range(reps_s):
        for h, o, st in zip(handles, outs, streams):
            h.decode_batch_smooth(1, out=o, stream=st.cuda_stream)
    torch.cuda.synchronize()
    res["fidelity_estimate"]["scan_group_1_smoothed"] = {"mean_score": smooth_score, "ms_per_step": (time.perf_counter() - t) / reps_s * 1e3,
                                                         "plain_ms_per_step": per_k_ms.get(1)}
    del full0

    # the same images as baseline (non-progressive) files, and with restart intervals in every scan
    for label, kw, ks in (("baseline_sequential_files", dict(script="sequential"), (1,)), ("with_restart_intervals", dict(restart=128), TABLE_SCAN_GROUPS)):
        recs, files = pcrgen.make_workload("imagenet_like", limit=args.images, **kw)
        hs = [pkg.pcr_open(r, 0) for r in recs]
        torch.cuda.synchronize()
        rates = {}
        for kk in ks:
            def other_step():
                for h, o, st in zip(hs, outs, streams):
                    h.decode_batch(kk, out=o, stream=st.cuda_stream)
            other_step(); other_step()
            torch.cuda.synchronize()
            lay = hs[0].output_layout()
            host = outs[0].cpu().numpy()
            _, p0, info = oracle.decode_record_image(recs[0], 3, kk, want_coef=False)
            got = host[int(lay[3]):int(lay[4])].reshape(info.H, info.W, info.nc).astype(int)
            assert np.abs(got - p0).max() <= 1, "parity check failed (%s)" % label
            reps_b = max(5, args.steps)
            t = time.perf_counter()
            for _ in range(reps_b):
                other_step()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t) / reps_b
            rates[str(kk)] = {"images_per_s": n_img / dt, "ms_per_step": dt * 1e3}
        res[label] = {"mean_file_kB": float(np.mean([len(f) for f in files]) / 1e3), "per_scan_group": rates}
        for h in hs:
            h.close()
        del hs, recs, files
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="imagenet_like", choices=sorted(WORKLOAD_SCAN_GROUPS))
    ap.add_argument("--images", type=int, default=None, help="use only the first N images of the workload")
    ap.add_argument("--scan-group", type=int, default=None, help="the scan group `value` is quoted at (default: the highest)")
    ap.add_argument("--entry-interval", type=int, default=64, help="MCUs between the entry points the record writer stores (record version 2)")
    ap.add_argument("--only", action="store_true", help="time only the scan group of --scan-group (for profiler runs)")
    ap.add_argument("--extras", action="store_true", help="also: fidelity upgrades, training tail, similarity scores, baseline files, restart intervals")
    ap.add_argument("--lane-decoders", type=int, default=0, choices=(-1, 0, 1),
                    help="shape of the AC entropy decoders: 0 the library's choice (by units per launch and records open), 1 one lane per unit "
                         "wherever possible, -1 one wavefront per unit")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-default-queues", action="store_true", help="skip the child process that measures the step with HIP's default number of hardware queues")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain elementwise copy of 256 MiB (untimed), the yardstick for rocprofv3's FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--keep-queues", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--child-records", default=None, help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the decode path shards by record with no exchange between GPUs, "
              "and this build runs on a single MI355X; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    Job.lane_decoders = args.lane_decoders
    if args.child_records:
        return child_main(args)

    import torch
    import pcrgen
    import paper_1911_00472_amd as pkg
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    pkg.lib()
    name = args.workload
    scan_groups = WORKLOAD_SCAN_GROUPS[name]
    headline_k = args.scan_group or scan_groups[-1]
    if headline_k not in scan_groups:
        scan_groups = tuple(sorted(set(scan_groups) | {headline_k}))
    if args.only:
        scan_groups = (headline_k,)

    t0 = time.time()
    records, files = pcrgen.make_workload(name, limit=args.images)
    Ws, Hs = pcrgen.workload_shapes(name, limit=args.images)
    shapes = list(zip((int(w) for w in Ws), (int(h) for h in Hs)))
    ends = np.array([pcrgen.split_scans(f) for f in files], dtype=np.int64)
    script, sampling = read_scan_script(files[0])
    n0 = len(files) if len(records) == 1 else pcrgen.WORKLOADS[name]["per_record"]
    symbols0 = pcrgen.workload_symbol_counts(name, limit=min(n0, len(files)))          # record 0's images
    print("[bench] %s: %d images (mean %.1f kB) in %d records, generated in %.1f s" % (name, len(files), ends[:, -1].mean() / 1000, len(records), time.time() - t0),
          file=sys.stderr, flush=True)

    # The records the library's own writer makes of these files: the same image bytes, plus entry points about every
    # 128 MCUs of every scan (record version 2), which the decoder uses as it uses restart intervals.  `value` is
    # measured on them; the plain records (no entry points: one serial stream per scan) are timed further down.
    plain_records = records
    per_record = pcrgen.WORKLOADS[name]["per_record"]
    labels = (np.arange(len(files)) * 7919) % 1000
    t0 = time.time()
    records = [pkg.record_write_indexed(files[a:a + per_record], labels[a:a + per_record], args.entry_interval) for a in range(0, len(files), per_record)]
    index_s = time.time() - t0
    entry_bytes = sum(len(r) for r in records) - sum(len(r) for r in plain_records)

    job = Job(torch, pkg, records, on_device=(name == "ham_like"))
    n_img = job.n_img

    if args.calibrate_copy:
        a = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 1, out=b)
        torch.cuda.synchronize()
        print("[bench] calibration copy: elementwise kernel, %d bytes read, %d bytes written" % (a.numel(), b.numel()), file=sys.stderr, flush=True)
        del a, b

    # ---- parity spot check against the oracle before anything is timed ----
    import oracle
    job.step(headline_k)
    torch.cuda.synchronize()
    lay = job.handles[0].output_layout()
    host = job.outs[0].cpu().numpy()
    for i in (0, 1, min(7, job.handles[0].n - 1)):
        _, p0, info = oracle.decode_record_image(records[0], i, headline_k, want_coef=False)
        got = host[int(lay[i]):int(lay[i + 1])].reshape(info.H, info.W, info.nc).astype(int)
        assert np.abs(got - p0).max() <= 1, "parity check failed for image %d" % i

    per_k = {}
    for k in scan_groups:
        if k != headline_k:
            per_k[k] = job.timed(k, max(3, args.steps // 2), 2)
    per_k[headline_k] = job.timed(headline_k, args.steps, args.warmup)      # EXACTLY --steps steps after --warmup warm-up steps

    threads = min(16, os.cpu_count() or 1)
    report = {}
    for k in sorted(per_k):
        sec, singles, over, alone, calls = per_k[k]
        ab = algorithmic_bytes(ends, shapes, script, sampling, k)
        report[str(k)] = {
            "images_per_s": n_img / sec, "ms_per_step": sec * 1e3,
            "ms_per_step_median_of_single_steps": float(np.median(singles)) * 1e3, "ms_per_step_min_of_single_steps": float(np.min(singles)) * 1e3,
            "output_GBps": ab["out"] / sec / 1e9, "algorithmic_GBps": ab["path"] / sec / 1e9,
            "hbm_roofline_frac": ab["path"] / sec / 1e9 / HBM_PEAK_GBS,
            "must_move_floor_GBps": (ab["compressed"] + ab["out"]) / sec / 1e9,
            "compressed_MB": ab["compressed"] / 1e6,
            "stage_ms_one_record_alone": {n: ms / calls for n, (ms, launches) in alone.items() if launches},
            "kernel_ms_per_launch_overlapped": {n: v for n, v in per_launch(over).items() if v},
        }
        if not args.no_cpu_baseline:
            rate, cnt, dt = oracle_rates(oracle, records, k, threads, max(16, 256 // len(records)))
            report[str(k)]["oracle_images_per_s"] = rate
            report[str(k)]["gpu_over_oracle"] = n_img / sec / rate
    sec, singles, over, alone, calls = per_k[headline_k]
    ab = algorithmic_bytes(ends, shapes, script, sampling, headline_k)

    probe = max(pkg.probe_scalar_issue_rate(w) for w in (8, 16, 32))
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

    default_config = name == "imagenet_like" and args.images is None and headline_k == 10 and args.entry_interval == ap.get_default("entry_interval")
    nrec0 = job.handles[0].n
    job.handles[0].decode_batch(headline_k, out=job.outs[0], stream=job.streams[0].cuda_stream)
    torch.cuda.synchronize()
    lane_launches, wave_launches = job.handles[0].last_decoder_shapes()
    roofline, dom = dominant_kernel_roofline(name, headline_k, script, symbols0, ends[:nrec0], alone, calls, over, probe, default_config,
                                             lane_launches > 0 and wave_launches == 0)
    if roofline["bound"] == "hbm":                            # data-parallel kernel: its algorithmic bytes for record 0
        ab0 = algorithmic_bytes(ends[:nrec0], shapes[:nrec0], script, sampling, headline_k)
        kb = {"pixel": ab0["touched"] + ab0["out"], "unstuff": 2 * ab0["compressed"]}.get(dom)
        if kb:
            roofline["achieved"] = kb / (roofline["ms_per_launch"] * 1e-3) / 1e9
            roofline["frac"] = roofline["achieved"] / HBM_PEAK_GBS
    # the pixel kernel on its own against HBM (the one stage the byte model calls bandwidth-bound)
    ab0 = algorithmic_bytes(ends[:nrec0], shapes[:nrec0], script, sampling, headline_k)
    pix_ms = alone["pixel"][0] / max(1, alone["pixel"][1])
    pixel_kernel = {"ms_per_launch_alone": pix_ms, "algorithmic_bytes": ab0["touched"] + ab0["out"],
                    "achieved_GBps": (ab0["touched"] + ab0["out"]) / (pix_ms * 1e-3) / 1e9,
                    "frac_of_8TBps": (ab0["touched"] + ab0["out"]) / (pix_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "note": "coefficients covered by scans <= k read once (2 bytes each) + pixels written once, record 0 alone"}

    cpu = None
    if not args.no_cpu_baseline:
        rate16, cnt16, dt16 = oracle_rates(oracle, records, headline_k, threads, 1 << 30 if name == "imagenet_like" else max(64, 1024 // len(records)))
        rate1, cnt1, dt1 = oracle_rates(oracle, records, headline_k, 1, max(4, 96 // len(records)))
        cpu = {"value": rate16, "unit": "images/s", "cores": threads, "kind": "oracle",
               "sample": "%d images of the workload (the first of every record) once at scan group %d, %d threads, %.1f s wall" % (cnt16, headline_k, threads, dt16),
               "one_thread": {"value": rate1, "unit": "images/s", "cores": 1,
                              "sample": "%d images at scan group %d, %.1f s" % (cnt1, headline_k, dt1)}}

    line = {
        "metric": "decoded_images_per_sec_at_scan_group_%d" % headline_k,
        "value": n_img / sec, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int16 coefficients, fp32 IDCT/colour, u8 pixels", "data": "synthetic",
        "config": {"workload": "%s: %d images, mean %.0f kB, %d records, sampling %s, %d scans" % (name, n_img, ends[:, -1].mean() / 1000, len(records),
                                                                                                  "x".join("%d%d" % s for s in sampling), len(script)),
                   "scan_group": headline_k, "images": n_img, "records": len(records),
                   "records_opened": "from device memory (index and markers parsed on the device)" if name == "ham_like" else "from host bytes",
                   "record_version": 2, "entry_interval_mcus": args.entry_interval, "entry_point_bytes_share": entry_bytes / float(sum(len(r) for r in records)),
                   "record_writer_s": index_s},
        "ms_per_step_median_of_single_steps": float(np.median(singles)) * 1e3, "ms_per_step_min_of_single_steps": float(np.min(singles)) * 1e3,
        "output_GBps": ab["out"] / sec / 1e9,
        "open_ms_per_record": job.open_ms,
        "path_roofline": {"bound": "hbm", "achieved": ab["path"] / sec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": ab["path"] / sec / 1e9 / HBM_PEAK_GBS, "device_copy_GBps_measured": copy_gbps,
                          "frac_of_measured_copy": ab["path"] / sec / 1e9 / copy_gbps,
                          "by_scan_group": {k: v["hbm_roofline_frac"] for k, v in report.items()}},
        "path_issue": ({"scalar_insts_per_step": RECORD0_INSTS["scalar"] * len(records), "vector_insts_per_step": RECORD0_INSTS["vector"] * len(records),
                        "G_scalar_insts_per_s": RECORD0_INSTS["scalar"] * len(records) / sec / 1e9,
                        "G_vector_insts_per_s": RECORD0_INSTS["vector"] * len(records) / sec / 1e9,
                        "scalar_frac_of_peak": RECORD0_INSTS["scalar"] * len(records) / sec / 1e9 / SALU_PEAK_GINSTS,
                        "vector_frac_of_peak": RECORD0_INSTS["vector"] * len(records) * 64 / sec / 1e12 / VALU_PEAK_TLANEOPS,
                        "note": "instructions executed per step (rocprofv3, record 0 x records) over the step time; each unit issues "
                                "614 G wavefront instructions/s at most", "source": RECORD0_INSTS["source"]}
                       if (default_config and RECORD0_INSTS and lane_launches > 0 and wave_launches == 0) else None),
        "ac_decoder_shape": {"lane_per_unit_launches": lane_launches, "wavefront_per_unit_launches": wave_launches},
        "roofline": roofline,
        "pixel_kernel": pixel_kernel,
        "cpu_baseline": cpu,
        "per_scan_group": report,
    }
    if name == "ham_like" or args.extras:
        line["from_pinned_host_memory"] = streamed_from_pinned(torch, pkg, records, job.outs, scan_groups if name == "ham_like" else TABLE_SCAN_GROUPS,
                                                               n_img, args.steps)
    if args.extras and name == "imagenet_like":
        line.update(extras(torch, pkg, pcrgen, oracle, job, args, ends, {kk: v[0] * 1e3 for kk, v in per_k.items()}, headline_k))
    job.close()
    del job
    torch.cuda.synchronize()
    # the same files in plain records (version 1, what the input generator writes: no entry points)
    pjob = Job(torch, pkg, plain_records)
    plain = {}
    for k in ([] if args.only else sorted(set(TABLE_SCAN_GROUPS) & set(scan_groups))):
        psec, psingles, _, palone, pcalls = pjob.timed(k, max(3, args.steps // 2), 2, single_steps=5)
        plain[str(k)] = {"images_per_s": n_img / psec, "ms_per_step": psec * 1e3,
                         "ms_one_record_alone": sum(ms for ms, _ in palone.values()) / pcalls}
    pjob.close()
    del pjob
    line["plain_records_without_entry_points"] = plain
    if not args.no_default_queues and len(records) > 1:
        line["with_default_hardware_queues"] = measure_default_queues(records, headline_k, args.steps, args.warmup)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
