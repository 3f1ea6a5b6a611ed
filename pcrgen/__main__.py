"""`python -m pcrgen symbols <workload> [--images N] [--record-size R]`: Huffman-coded symbols per scan of a workload's
files, as the encoder counts them while writing (the work figure a decoder's throughput is quoted against)."""
import argparse

import numpy as np

import pcrgen


def main():
    ap = argparse.ArgumentParser(prog="python -m pcrgen")
    ap.add_argument("what", choices=["symbols"])
    ap.add_argument("workload", choices=sorted(pcrgen.WORKLOADS))
    ap.add_argument("--images", type=int, default=None, help="only the first N images")
    ap.add_argument("--record-size", type=int, default=1024, help="images per record, for the per-record sums")
    a = ap.parse_args()
    cnt = pcrgen.workload_symbol_counts(a.workload, limit=a.images)
    n, g = cnt.shape
    print("%s: %d images, %d scans; Huffman-coded symbols per scan" % (a.workload, n, g))
    print("record | images | " + " | ".join("scan %d" % (s + 1) for s in range(g)) + " | all scans")
    for r0 in range(0, n, a.record_size):
        part = cnt[r0:r0 + a.record_size]
        print("%6d | %6d | " % (r0 // a.record_size, part.shape[0]) + " | ".join("%d" % int(v) for v in part.sum(axis=0)) + " | %d" % int(part.sum()))
    print("   all | %6d | " % n + " | ".join("%d" % int(v) for v in cnt.sum(axis=0)) + " | %d" % int(cnt.sum()))
    print("mean per image: " + ", ".join("%.0f" % v for v in cnt.mean(axis=0)))


if __name__ == "__main__":
    main()
