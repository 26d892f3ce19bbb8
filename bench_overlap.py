#!/usr/bin/env python3
"""Do the matrix cores, the vector units and the HBM stream overlap on this machine?

    python3 bench_overlap.py

Runs the library's measurement aids (owq_probe_mfma, owq_probe_alu, owq_probe_read: registers-only matrix
instructions, registers-only fp32 arithmetic, a read-only 128-bit stream over 12 rotating buffers of 127 MB, the
size of one 3-bit 9216 x 36864 layer) alone and in pairs on two streams of the default priority, and prints the
microseconds per round.  A pair that overlaps takes about as long as its longer member, one that does not takes
the sum.  Context for the batched path's figures: a kernel that issues a call's matrix instructions and streams
its codes is bounded by what this prints for that pair."""
from __future__ import annotations

import time

import torch

from paper_2306_02272_amd import binding as B

LAYER_BYTES = 127_401_984


def main() -> int:
    if not torch.cuda.is_available():
        raise SystemExit("bench_overlap.py needs a GPU")
    dev = torch.device("cuda:0")
    word = torch.zeros(4, dtype=torch.float32, device=dev)
    bufs = [torch.zeros(LAYER_BYTES, dtype=torch.uint8, device=dev) for _ in range(12)]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()          # default priority

    def mfma(stream, wgs, trips):
        return lambda: B.owq_probe_mfma(word.data_ptr(), wgs, trips, stream.cuda_stream)

    def alu(stream, wgs, trips):
        return lambda: B.owq_probe_alu(word.data_ptr(), wgs, trips, stream.cuda_stream)

    def read(stream, launches):
        def go():
            for i in range(launches):
                B.owq_probe_read(bufs[i % len(bufs)].data_ptr(), LAYER_BYTES, 512, stream.cuda_stream)
        return go

    def per_round(fns, rounds=40):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.1:                   # untimed: clocks, code upload
            for f in fns:
                f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(rounds):                                 # enqueued in turn, so both queues fill together
            for f in fns:
                f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / rounds * 1e6

    cases = [
        ("matrix probe, 128 workgroups x 640 trips (half the chip)", [mfma(s1, 128, 640)]),
        ("the same on two streams", [mfma(s1, 128, 640), mfma(s2, 128, 640)]),
        ("matrix probe, 256 workgroups x 320 trips", [mfma(s1, 256, 320)]),
        ("read stream, 8 launches x 127 MB", [read(s2, 8)]),
        ("matrix probe + read stream", [mfma(s1, 256, 320), read(s2, 8)]),
        ("vector probe, 256 workgroups x 2000 trips", [alu(s1, 256, 2000)]),
        ("vector probe + read stream", [alu(s1, 256, 2000), read(s2, 8)]),
        ("vector probe + matrix probe", [alu(s1, 256, 2000), mfma(s2, 256, 320)]),
    ]
    for name, fns in cases:
        print(f"{name:60s} {per_round(fns):9.2f} us per round", flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
