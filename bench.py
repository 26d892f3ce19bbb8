#!/usr/bin/env python3
"""Throughput of the OWQ mixed-precision linear layer on one MI355X.

A step is one pass of the hot path over one token: every layer of the workload
is called once through the C ABI (owq_linear), batch 1, on synthetic layers and
activations that are already resident in HBM.  Successive steps use different
packed copies of the layers (distinct addresses, more than the 256 MB of
last-level cache in total), as successive decoder blocks of a model would, so
that the weights really come from HBM.

The workloads named search-* time the other entry point, owq_search_config (the configuration
search that produces a layer's step sizes, zero points and codes from fp16 weights): a step is one
call over the whole matrix, the bound is the vector units (fp32 operations against the published
fp32 vector peak).

Prints ONE JSON line.  value = algorithmic bytes of a step / time of a step (GB/s);
roofline.achieved = algorithmic bytes (or, on the tile layout, floating-point operations) per
call / mean duration of a call from HIP events on the launch stream; roofline.traffic = HBM
bytes per call from rocprofv3's FETCH_SIZE and WRITE_SIZE (profiles/traffic.json, written by
bench_traffic.py); cpu_baseline = the CPU oracle timed on a bounded sample of the same step.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
CALIB_BYTES = 256 << 20

WORKLOADS = {
    # name: (index in the list of benchmark configurations, layer indices, description, packed layout, default batch)
    "opt6.7b-ffn": (2, [0, 1], "configs[2]: OPT-6.7B-like FFN pair, fc1 4096->16384 (k=32) + fc2 16384->4096 (k=128), 3-bit, group 128", 0, 1),
    "opt6.7b-attn": (1, [0], "configs[1]: OPT-6.7B-like attention projection 4096->4096, 3-bit per-channel, k=32", 0, 1),
    "target": (5, [0], "bandwidth-target layer 16384->4096, 3-bit per-channel, k=128", 0, 1),
    "llama13b": (3, [0, 1, 2], "configs[3]: LLaMA-13B-like q/k/v/o, gate/up, down, 4-bit group 128, k=1%", 0, 1),
    "tiny": (0, [0], "configs[0]: 1024->1024, 4-bit per-channel, k=8", 0, 1),
    "unseen-7168": (6, [0], "a shape no launch model was fitted on: 7168->7168 (hidden size not a power of two), 3-bit group 128, k=72", 0, 1),
    "unseen-wide-ffn": (6, [1, 2], "a shape no launch model was fitted on: very wide FFN pair 8192->28672 (4-bit group 128, k=82) + 28672->8192 (4-bit per-channel, k=287)", 0, 1),
    "opt66b-ffn": (4, [0, 1], "configs[4]: OPT-66B-like FFN pair, fc1 9216->36864 (k=64) + fc2 36864->9216 (k=256), 3-bit per-channel, tile layout (matrix cores)", 1, 64),
}


def algorithmic_bytes(spec, batch: int, layout: int = 0) -> int:
    """Bytes one call has to move: codes + (scale, zero) + weak columns + indices + x + y.
    Storage-favoured layout (2): codes of the columns that are not weak only, and a dword of
    weak-column bookkeeping per 8 input columns instead of the indices."""
    groups = 1 if spec.group_size == 0 else -(-spec.d_in // spec.group_size)
    cols = spec.d_in - spec.k if layout == 2 else spec.d_in
    index_bytes = 4 * (-(-spec.d_in // 8)) if layout == 2 else 4 * spec.k
    return (spec.d_out * cols * spec.bits // 8 + 4 * spec.d_out * groups + 2 * spec.d_out * spec.k
            + index_bytes + 2 * batch * (spec.d_in + spec.d_out))


def pmc_calibration(torch, stream):
    """A plain copy of known size (reads CALIB_BYTES, writes CALIB_BYTES per launch) for bench_traffic.py."""
    src = torch.arange(CALIB_BYTES // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 1, out=dst)            # an elementwise kernel of torch's own: copy with +1
    stream.synchronize()


def blas_threads():
    """Threads the oracle's numpy matrix products use."""
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return os.cpu_count() or 1


def stored_traffic(workload):
    """HBM bytes per call that bench_traffic.py measured for this workload, or None."""
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        return json.load(open(tpath)).get(workload)
    except Exception:
        return None


FP32_VECTOR_PEAK_TFLOPS = 157.3
SEARCH_WORKLOADS = {
    # name: (d_out, d_in, k, bits, group size, grid n_lo x n_hi, shrink, description)
    "search-opt6.7b-fc1": (16384, 4096, 32, 3, 128, 16, 16, 0.4,
                           "configuration search for an OPT-6.7B-like fc1 (16384 x 4096 fp16 weights, k=32 weak "
                           "columns left out), 3-bit, group 128, 16 x 16 grid of narrowed ranges"),
    "search-opt6.7b-fc1-row": (16384, 4096, 32, 3, 0, 16, 16, 0.4,
                               "configuration search for an OPT-6.7B-like fc1 (16384 x 4096 fp16 weights, k=32 weak "
                               "columns left out), 3-bit, one scale per row, 16 x 16 grid of narrowed ranges"),
}
SEARCH_FLOP = 7          # per weight and grid point: multiply, round, clamp, two fused multiply-adds


def bench_search(args) -> int:
    """A step = one owq_search_config call over the whole weight matrix, resident in HBM."""
    import numpy as np
    import torch

    from paper_2306_02272_amd import binding as B
    from synth import make_weights

    B.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    d_out, d_in, k, bits, gs, n_lo, n_hi, shrink, desc = SEARCH_WORKLOADS[args.workload]
    w_host, idx_host = make_weights(d_out, d_in, k, seed=2000)
    w = torch.from_numpy(w_host).cuda()
    idx = torch.from_numpy(idx_host).cuda()
    n_g = 1 if gs == 0 else -(-d_in // gs)
    scale = torch.empty((d_out, n_g), dtype=torch.float16, device="cuda")
    zero = torch.empty_like(scale)
    codes = torch.empty((d_out, d_in), dtype=torch.uint8, device="cuda")
    err = torch.empty((d_out, n_g), dtype=torch.float32, device="cuda")
    sd = B.SearchDesc(d_out, d_in, bits, gs, k, n_lo, n_hi, shrink)
    stream = torch.cuda.Stream()
    raw = stream.cuda_stream
    steps, warmup = min(args.steps, 200), min(args.warmup, 20)

    def run(n):
        for _ in range(n):
            B.owq_search_config(sd, w.data_ptr(), idx.data_ptr(), scale.data_ptr(), zero.data_ptr(), codes.data_ptr(),
                                err.data_ptr(), 0, raw)

    with torch.cuda.stream(stream):
        if args.pmc_calib:
            pmc_calibration(torch, stream)
        run(warmup)
        stream.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(stream)
        run(steps)
        ev1.record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # what the vector units issue of the search's own five instructions on registers only, same run
        word = torch.zeros(1, dtype=torch.float32, device="cuda")
        alu_wgs, alu_trips = 256 * 8, 4096
        B.owq_probe_alu(word.data_ptr(), alu_wgs, alu_trips, raw)
        stream.synchronize()
        ea0, ea1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ea0.record(stream)
        for _ in range(5):
            B.owq_probe_alu(word.data_ptr(), alu_wgs, alu_trips, raw)
        ea1.record(stream)
        stream.synchronize()
        bare_tips = alu_wgs * 256 * alu_trips * 160 * 5 / (ea0.elapsed_time(ea1) * 1e-3) / 1e12
    wall_s, event_s = t1 - t0, ev0.elapsed_time(ev1) * 1e-3
    assert torch.isfinite(err).all() and int(codes.max()) <= (1 << bits) - 1
    weights = d_out * (d_in - k)
    flops = SEARCH_FLOP * weights * n_lo * n_hi
    avg_launch_s = event_s / steps
    tflops = flops / avg_launch_s / 1e12
    result = {
        "metric": f"configuration search, G weights/s ({n_lo} x {n_hi} grid points each), {bits}-bit",
        "value": round(weights * steps / wall_s / 1e9, 3), "unit": "Gweights/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(wall_s / steps * 1e3, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": desc, "d_out": d_out, "d_in": d_in, "k": k, "group_size": gs, "grid": [n_lo, n_hi],
                   "shrink": shrink, "launch_mode": "eager"},
        "roofline": {"bound": "alu", "achieved": round(tflops, 1), "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / FP32_VECTOR_PEAK_TFLOPS, 4), "traffic": stored_traffic(args.workload),
                     "kernel": f"owq_search_kernel<{-(-n_lo * n_hi // 64)}, {0 if gs == 0 or gs > 1024 else -(-gs // 64)}>",
                     "avg_launch_us": round(avg_launch_s * 1e6, 1), "flops_per_launch": flops,
                     "instructions_per_s": round(5 * weights * n_lo * n_hi / avg_launch_s / 1e12, 2),
                     "achievable": {"kind": "register-only loop of the same five fp32 instructions (T lane-instructions/s), same run",
                                    "instructions_per_s": round(bare_tips, 2),
                                    "frac_of_it": round(5 * weights * n_lo * n_hi / avg_launch_s / 1e12 / bare_tips, 4)}},
    }
    if not args.no_cpu_baseline:
        from oracle import search
        rows, c0 = 0, time.perf_counter()
        while time.perf_counter() - c0 < 10.0:        # whole rows until about ten seconds have gone by
            search.search_config(w_host[rows:rows + 1], idx_host, bits, gs, n_lo, n_hi, shrink)
            rows += 1
        c1 = time.perf_counter()
        result["cpu_baseline"] = {"value": round(rows * (d_in - k) / (c1 - c0) / 1e9, 9), "unit": "Gweights/s",
                                  "cores": 1, "kind": "oracle",
                                  "sample": f"the first {rows} of {d_out} rows, in {c1 - c0:.2f} s"}
    print(json.dumps(result), flush=True)
    return 0


BACKWARD_WORKLOADS = {
    # name: (index in the list of benchmark configurations, layer indices, tokens, description)
    "backward-opt6.7b-ffn": (2, [0, 1], 512, "backward (dX and dWw, weak-column tuning) of configs[2]'s OPT-6.7B-like FFN "
                                             "pair, 3-bit, group 128, 512 tokens, tile layout"),
    "backward-llama13b": (3, [0, 1, 2], 512, "backward (dX and dWw, weak-column tuning) of configs[3]'s LLaMA-13B-like q/k/v/o, "
                                             "gate/up and down projections, 4-bit, group 128, 512 tokens, tile layout"),
}


def bench_backward(args) -> int:
    """A step = owq_linear_backward (dX and dWw) of every layer of the workload for one batch of tokens."""
    import numpy as np
    import torch

    from paper_2306_02272_amd import binding as B
    from synth import CONFIGS, make_layer, make_x

    B.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg, layer_ids, batch, desc = BACKWARD_WORKLOADS[args.workload]
    if args.batch:
        batch = args.batch
    specs = [CONFIGS[cfg][i] for i in layer_ids]
    layers = [make_layer(s) for s in specs]
    lins = [B.OwqLinear(L, layout=1) for L in layers]
    rng = np.random.default_rng(5)
    xs_host = [make_x(L, batch) for L in layers]
    dys_host = [rng.normal(0, 0.05, size=(batch, L.d_out)).astype(np.float16) for L in layers]
    xs = [torch.from_numpy(x).cuda() for x in xs_host]
    dys = [torch.from_numpy(d).cuda() for d in dys_host]
    dxs = [torch.empty((batch, L.d_in), dtype=torch.float16, device="cuda") for L in layers]
    dwws = [torch.empty((L.d_out, L.k), dtype=torch.float32, device="cuda") for L in layers]
    wss = [torch.empty(B.owq_backward_workspace_bytes(lin.handle, batch), dtype=torch.uint8, device="cuda") for lin in lins]
    stream = torch.cuda.Stream()
    raw = stream.cuda_stream
    steps, warmup = min(args.steps, 200), min(args.warmup, 20)

    def run(n):
        for _ in range(n):
            for lin, x, dy, dx, dww, ws in zip(lins, xs, dys, dxs, dwws, wss):
                B.owq_linear_backward(lin.handle, dy.data_ptr(), x.data_ptr(), dx.data_ptr(), dww.data_ptr(), batch,
                                      ws.data_ptr(), int(ws.numel()), raw)

    with torch.cuda.stream(stream):
        if args.pmc_calib:
            pmc_calibration(torch, stream)
        run(warmup)
        stream.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(stream)
        run(steps)
        ev1.record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    wall_s, event_s = t1 - t0, ev0.elapsed_time(ev1) * 1e-3
    for dx in dxs:
        assert torch.isfinite(dx).all()
    # dense product + the two weak-column products
    flops_step = sum(2 * batch * sp.d_out * sp.d_in + 4 * batch * sp.d_out * sp.k for sp in specs)
    calls = steps * len(specs)
    avg_call_s = event_s / calls
    tflops = flops_step / len(specs) / avg_call_s / 1e12
    result = {
        "metric": f"backward of the {specs[0].bits}-bit OWQ linear (dX, dWw), tokens/s, {batch} tokens",
        "value": round(batch * steps / wall_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(wall_s / steps * 1e3, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 operands (dy x step size rounded to f16), f32 accumulate", "data": "synthetic",
        "config": {"workload": desc, "batch": batch, "layers": [s.name for s in specs], "launch_mode": "eager"},
        "us_per_call": round(wall_s / calls * 1e6, 3),
        "roofline": {"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / MFMA_F16_PEAK_TFLOPS, 4), "traffic": stored_traffic(args.workload),
                     "kernel": f"owq_bwd_product<{specs[0].bits}> (+ stage, sum, weak, dww)",
                     "avg_launch_us": round(avg_call_s * 1e6, 3), "flops_per_launch": flops_step // len(specs)},
    }
    if not args.no_cpu_baseline:
        from oracle import backward
        # a bounded sample: the first tokens of the batch and the first rows of every layer
        nt, c0, reps = min(batch, 8), time.perf_counter(), 0
        while True:
            for L, x, dy in zip(layers, xs_host, dys_host):
                rows = max(1, L.d_out // 8)
                backward.owq_backward_ref(L.codes[:rows], L.scale[:rows], L.zero[:rows], L.group_size, L.weak_idx,
                                          L.weak_w[:rows], x[:nt], dy[:nt, :rows])
            reps += 1
            if time.perf_counter() - c0 >= 10.0:
                break
        c1 = time.perf_counter()
        result["cpu_baseline"] = {"value": round(reps * nt / 8 / (c1 - c0), 3), "unit": "tokens/s", "cores": blas_threads(),
                                  "kind": "oracle",
                                  "sample": f"{reps} x ({nt} tokens, the first eighth of the output rows of each layer) "
                                            f"in {c1 - c0:.2f} s"}
    print(json.dumps(result), flush=True)
    for lin in lins:
        lin.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="opt6.7b-ffn", choices=sorted(WORKLOADS) + sorted(SEARCH_WORKLOADS) + sorted(BACKWARD_WORKLOADS))
    ap.add_argument("--batch", type=int, default=0, help="tokens per call (default: the workload's own)")
    ap.add_argument("--layout", type=int, default=-1, help="0 = single-token layout, 1 = tile layout, 2 = storage-favoured single-token layout (default: the workload's own)")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"],
                    help="graph: the K timed steps are one HIP graph launch; eager: K*layers launches from Python")
    ap.add_argument("--footprint-gb", type=float, default=1.5, help="total bytes of packed copies to rotate over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tasks", type=int, default=0,
                    help="N > 0: owq_linear_multi with N sets of weak columns and random task ids per token")
    ap.add_argument("--pmc-calib", action="store_true",
                    help="also run a few plain device copies of 256 MiB, for scaling rocprofv3's byte counters")
    ap.add_argument("--replays", type=int, default=7, help="timed replays of the K steps; the median one is reported")
    ap.add_argument("--ramp-ms", type=float, default=100.0,
                    help="untimed replays of the same steps before the timed ones, until the GPU has been busy this long")
    ap.add_argument("--lead-in", type=int, default=1, choices=(0, 1),
                    help="1: every timed replay is enqueued straight behind an untimed one (GPU never idle at its start) and the "
                         "line's value is the HIP-event time of its K steps; 0: every replay starts on an idle GPU and the value "
                         "is the host clock around synchronize -> K steps -> synchronize")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the context figures (one packed copy, single launch, read-only stream, empty launch)")
    ap.add_argument("--launch", default="", help="rtw,rsplit,waves,depth override for every layer (tuning)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    if args.workload in SEARCH_WORKLOADS:
        return bench_search(args)
    if args.workload in BACKWARD_WORKLOADS:
        return bench_backward(args)

    import numpy as np
    import torch

    from paper_2306_02272_amd import binding as B
    from synth import CONFIGS, make_layer, make_x

    B.lib()                                       # no library, no benchmark
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg, layer_ids, desc, layout, batch = WORKLOADS[args.workload]
    specs = [CONFIGS[cfg][i] for i in layer_ids]
    if args.batch:
        batch = args.batch
    if args.layout >= 0:
        layout = args.layout

    layers = [make_layer(s) for s in specs]
    xs_host = [make_x(L, batch) for L in layers]
    bytes_per_layer = [algorithmic_bytes(s, batch, layout) for s in specs]
    step_bytes = sum(bytes_per_layer)

    # packed copies to rotate over
    first = [B.OwqLinear(L, layout=layout) for L in layers]
    packed_total = sum(int(f.buf.numel()) for f in first)
    copies = max(1, int(-(-args.footprint_gb * 1e9 // packed_total)))
    sets = [first] + [[B.OwqLinear(L, packed=f.buf, layout=layout) for L, f in zip(layers, first)]
                      for _ in range(copies - 1)]
    if args.launch:
        rtw, rsplit, waves, depth = (int(v) for v in (args.launch.split(",") + ["0", "0", "0"])[:4])
        for st in sets:
            for lin in st:
                B.owq_set_launch(lin.handle, rtw, rsplit, waves, depth)
    tables = None
    if args.tasks > 0:
        rng = np.random.default_rng(1)
        tables = [[lin.add_weak_sets([rng.normal(0, 0.02, size=(L.d_out, L.k)).astype(np.float16)
                                      for _ in range(args.tasks)]) for lin, L in zip(st, layers)] for st in sets]
        task_ids = torch.from_numpy(rng.integers(0, args.tasks, size=batch).astype(np.int32)).cuda()
    xs = [torch.from_numpy(x).cuda() for x in xs_host]
    ys = [torch.empty((batch, s.d_out), dtype=torch.float16, device="cuda") for s in specs]

    probe_out = [torch.empty_like(y) for y in ys]
    stream = torch.cuda.Stream()                  # default priority
    raw = stream.cuda_stream
    # what a call reads of a packed layer: all of it but the tile layout's scratch area
    read_bytes = [int(f.info().off_scratch or f.buf.numel()) & ~15 for f in first]

    def run_steps(first_step: int, n: int, ncopies: int = copies):
        for t in range(first_step, first_step + n):
            st = sets[t % ncopies]
            for i, (lin, x, y) in enumerate(zip(st, xs, ys)):
                if tables is None:
                    B.owq_linear(lin.handle, x.data_ptr(), y.data_ptr(), batch, raw)
                else:
                    tab = tables[t % ncopies][i][0]
                    B.owq_linear_multi(lin.handle, tab.data_ptr(), args.tasks, task_ids.data_ptr(), x.data_ptr(),
                                       y.data_ptr(), batch, raw)

    def read_steps(first_step: int, n: int, workgroups: int):
        """The same bytes, read only: one 128-bit read launch per layer call."""
        for t in range(first_step, first_step + n):
            for lin, nbytes in zip(sets[t % copies], read_bytes):
                B.owq_probe_read(lin.buf.data_ptr(), nbytes, workgroups, raw)

    def read_write_steps(first_step: int, n: int, workgroups: int):
        """The same reads, and each launch ends on a store of the size of the layer's output."""
        for t in range(first_step, first_step + n):
            for lin, nbytes, y in zip(sets[t % copies], read_bytes, probe_out):
                B.owq_probe_read_write(lin.buf.data_ptr(), nbytes, workgroups, y.data_ptr(), int(y.numel()) * 2 & ~15, raw)

    # the matrix instructions of one call's dense product, on registers only: 512 workgroups of four waves,
    # 16 instructions of 32768 flops per trip (padding the batch to the 32 or 64 tokens the kernel multiplies)
    probe_word = torch.zeros(4, dtype=torch.float32, device="cuda")
    mfma_tokens = 32 if batch <= 32 else 64 * -(-batch // 64)
    mfma_trips = [max(1, round(2 * mfma_tokens * sp.d_out * sp.d_in / (512 * 4 * 16 * 32768))) for sp in specs]

    def mfma_steps(first_step: int, n: int):
        for _ in range(n):
            for trips in mfma_trips:
                B.owq_probe_mfma(probe_word.data_ptr(), 512, trips, raw)

    def empty_steps(first_step: int, n: int):
        for _ in range(n * len(specs)):
            B.owq_probe_empty(raw)

    def timed(body, replays, lead_in=None):
        """body(first_step, n) enqueues n steps.  Graph mode: the n steps are one graph, replayed `replays` times,
        every replay bracketed by synchronisation; eager mode: enqueued from Python every time.  Before the timed
        replays the same steps run untimed until the GPU has been busy for --ramp-ms milliseconds (at least once:
        that also uploads the graph): a run of a few steps is over before the chip has reached its clocks, and would
        read up to 10 % slower than the same steps in a long run.  With a lead-in (--lead-in, the default) every timed
        replay is enqueued straight behind an untimed replay of the same steps, with no synchronisation between the
        two: the events then time exactly the K steps as they run in a job that keeps the GPU fed, without the
        microseconds a first launch on an idle GPU takes to start (6 us of a 280 us region at 20 steps); the host
        clock then brackets both replays.  Returns the (wall seconds, event seconds) pairs."""
        lead_in = args.lead_in if lead_in is None else lead_in
        graph = None
        if args.mode == "graph":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                body(args.warmup, args.steps)
        def once():
            if graph is not None:
                graph.replay()
            else:
                body(args.warmup, args.steps)
        r0 = time.perf_counter()
        untimed = 0
        while untimed == 0 or (time.perf_counter() - r0) * 1e3 < args.ramp_ms:
            once()
            stream.synchronize()
            untimed += 1
        ramp.setdefault("untimed_replays", untimed)      # of the layer's own steps: the first call of this function
        # events made (and recorded once) ahead of the timed region: creating one costs microseconds of idle GPU
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(replays)]
        for e0, e1 in events:
            e0.record(stream)
            e1.record(stream)
        out = []
        for ev0, ev1 in events:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if lead_in:
                once()
            ev0.record(stream)
            once()
            ev1.record(stream)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            out.append((t1 - t0, ev0.elapsed_time(ev1) * 1e-3))
        return out

    def median_of(pairs, key=0):
        order = sorted(range(len(pairs)), key=lambda i: pairs[i][key])
        return pairs[order[len(order) // 2]]

    context = {}
    ramp = {}
    with torch.cuda.stream(stream):
        if args.pmc_calib:
            pmc_calibration(torch, stream)
        run_steps(0, args.warmup)
        stream.synchronize()
        runs = timed(run_steps, args.replays)
        idle = timed(run_steps, 3, lead_in=0) if args.lead_in else None
        if not args.no_context and tables is None:
            # (1) the same steps on ONE packed copy: the weights then come from the last-level cache
            one = median_of(timed(lambda f, n: run_steps(f, n, 1), 3))
            context["one_copy_cache_resident"] = {"us_per_call": round(one[1] / (args.steps * len(specs)) * 1e6, 3),
                                                  "gbs": round(step_bytes * args.steps / one[1] / 1e9, 1)}
            # (2) one call at a time: events around a single eager launch, rotating copies
            lat = []
            for t in range(24):
                lin, x, y = sets[t % copies][t % len(specs)], xs[t % len(specs)], ys[t % len(specs)]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                stream.synchronize()
                e0.record(stream)
                B.owq_linear(lin.handle, x.data_ptr(), y.data_ptr(), batch, raw)
                e1.record(stream)
                stream.synchronize()
                lat.append(e0.elapsed_time(e1) * 1e3)
            context["single_launch_us"] = round(sorted(lat)[len(lat) // 2], 3)
            # (3) what the machine does on the same bytes without any arithmetic, and on nothing at all
            best = None
            for wgs in (256, 512, 1024):
                r = median_of(timed(lambda f, n: read_steps(f, n, wgs), 3))
                if best is None or r[1] < best[1]:
                    best = (wgs, r[1])
            rw = median_of(timed(lambda f, n: read_write_steps(f, n, best[0]), 3))
            context["read_write_stream_us"] = round(rw[1] / (args.steps * len(specs)) * 1e6, 3)
            empty = median_of(timed(empty_steps, 3))
            context["read_only_stream"] = {"workgroups": best[0],
                                           "us_per_call": round(best[1] / (args.steps * len(specs)) * 1e6, 3),
                                           "gbs": round(sum(read_bytes) * args.steps / best[1] / 1e9, 1)}
            context["empty_launch_us"] = round(empty[1] / (args.steps * len(specs)) * 1e6, 3)
            if layout == 1 and batch > 16:
                mf = median_of(timed(mfma_steps, 3))
                mf_flops = sum(512 * 4 * 16 * 32768 * t for t in mfma_trips) * args.steps
                context["mfma_only"] = {"us_per_call": round(mf[1] / (args.steps * len(specs)) * 1e6, 3),
                                        "tflops": round(mf_flops / mf[1] / 1e12, 1)}
    # with a lead-in the K steps are timed by the events (the host clock brackets two replays); without, by the host clock
    key = 1 if args.lead_in else 0
    wall_s, event_s = median_of(runs, key)
    step_s = (event_s if args.lead_in else wall_s) / args.steps
    ms_per_step = step_s * 1e3
    value = step_bytes / step_s / 1e9
    walls = sorted(r[key] for r in runs)

    # parity of the last step against the oracle is checked in tests; here only a finite-ness guard
    for y in ys:
        assert torch.isfinite(y).all()

    launches = args.steps * len(specs)
    avg_launch_s = event_s / launches
    achieved = (step_bytes / len(specs)) / avg_launch_s / 1e9
    traffic = stored_traffic(args.workload)
    info = first[0].info()
    flops_per_step = sum(2 * batch * sp.d_out * (sp.d_in + sp.k) for sp in specs)
    small = layout == 1 and batch <= 16 and not args.launch     # the one-launch kernel of the tile layout: bound by the weight stream
    if layout == 1 and not small:
        # three kernels per call; the matrix kernel dominates.  The figure charges the whole call to it.
        tflops = flops_per_step / len(specs) / avg_launch_s / 1e12
        roofline = {"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tflops / MFMA_F16_PEAK_TFLOPS, 4), "traffic": traffic,
                    "kernel": f"owq_tile_mma<{specs[0].bits},{2 if batch > 32 else 1}> (+ stage, finish)",
                    "avg_launch_us": round(avg_launch_s * 1e6, 3),
                    "flops_per_launch": flops_per_step // len(specs),
                    "hbm_gbs": round(achieved, 1), "hbm_frac": round(achieved / HBM_PEAK_GBS, 4),
                    "workgroups": info.workgroups}
        if "mfma_only" in context:
            # the matrix instructions of the same calls issued from registers, nothing read or written: what the
            # matrix cores deliver at the clock the chip holds under them; and the call's bytes at the read-only
            # stream's rate
            mo, ro = context["mfma_only"], context["read_only_stream"]
            roofline["achievable"] = {"kind": "the same 32x32x16 fp16 matrix instructions on registers only, same stream and launch mode",
                                      "tflops": mo["tflops"], "us_per_call": mo["us_per_call"],
                                      "frac_of_it": round(tflops / mo["tflops"], 4),
                                      "read_only_stream_us_per_call": ro["us_per_call"], "read_only_stream_gbs": ro["gbs"],
                                      "empty_launch_us": context["empty_launch_us"]}
    else:
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                    "kernel": (f"owq_tile_small<{specs[0].bits}> (+ owq_tile_small_sum)" if small
                               else f"owq_gemv_kernel<{specs[0].bits},{info.prefetch_depth}>"),
                    "avg_launch_us": round(avg_launch_s * 1e6, 3),
                    "bytes_per_launch": step_bytes // len(specs)}
        if "read_only_stream" in context:
            # the same bytes read by a kernel that computes nothing, same stream, same launch mode, same run
            ro = context["read_only_stream"]
            roofline["achievable"] = {"kind": "read-only 128-bit stream over the same packed copies", "gbs": ro["gbs"],
                                      "us_per_call": ro["us_per_call"], "workgroups": ro["workgroups"],
                                      "frac_of_it": round(achieved / ro["gbs"], 4),
                                      "empty_launch_us": context["empty_launch_us"],
                                      "with_output_store_us_per_call": context["read_write_stream_us"]}
    result = {
        # the headline metric; other workloads say their own code width and batch
        "metric": f"effective HBM GB/s (% of peak) + us/call, {specs[0].bits}-bit OWQ linear, batch {batch}",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 activations x 3/4-bit codes, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": desc, "batch": batch, "layers": [s.name for s in specs],
                   "packed_copies": copies, "launch_mode": args.mode, "tasks": args.tasks,
                   "bytes_per_step": step_bytes},
        "pct_of_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "us_per_call": round(step_s * args.steps / launches * 1e6, 3),
        # every replay is the same K steps; the line reports the median one (ms_per_step x steps = its wall time)
        "replays": {"n": len(walls), "ms_per_step_min": round(walls[0] / args.steps * 1e3, 6),
                    "ms_per_step_median": round(ms_per_step, 6), "ms_per_step_max": round(walls[-1] / args.steps * 1e3, 6),
                    # untimed replays of the same K steps in front of the timed ones (graph upload, clocks)
                    "untimed_before": ramp.get("untimed_replays", 0), "ramp_ms": args.ramp_ms,
                    "timed_by": ("HIP events around the K steps, enqueued straight behind an untimed replay of the same steps"
                                 if args.lead_in else "host clock around synchronize, K steps, synchronize")},
        "roofline": roofline,
    }
    if idle is not None:
        # the same K steps started on an idle GPU, every replay between two synchronisations: host clock and events
        iw, ie = median_of(idle)
        result["replays"]["idle_start"] = {"n": len(idle), "ms_per_step_host_clock": round(iw / args.steps * 1e3, 6),
                                           "ms_per_step_events": round(ie / args.steps * 1e3, 6)}
    for key in ("one_copy_cache_resident", "single_launch_us"):
        if key in context:
            result[key] = context[key]

    if not args.no_cpu_baseline:
        from oracle import owq_ref
        threads = blas_threads()
        # a bounded sample of the same step: the first `rows` output rows of every layer (all of
        # them when the step is small), repeated until about ten seconds have gone by
        work = sum(sp.d_out * sp.d_in * batch for sp in specs)
        frac = min(1.0, 2.0e9 / work)
        reps, c0 = 0, time.perf_counter()
        while True:
            for L, x in zip(layers, xs_host):
                rows = max(1, int(L.d_out * frac))
                owq_ref.owq_linear_ref(L.codes[:rows], L.scale[:rows], L.zero[:rows], L.group_size,
                                       L.weak_idx, L.weak_w[:rows], x)
            reps += 1
            if time.perf_counter() - c0 >= 10.0:
                break
        c1 = time.perf_counter()
        cpu_steps = reps * frac
        result["cpu_baseline"] = {"value": round(step_bytes * cpu_steps / (c1 - c0) / 1e9, 4), "unit": "GB/s",
                                  "cores": int(threads), "kind": "oracle",
                                  "sample": f"{reps} x the first {100 * frac:.1f} % of the output rows of each of the "
                                            f"{len(specs)} layers, batch {batch}, in {c1 - c0:.2f} s"}
    print(json.dumps(result), flush=True)
    for st in sets:
        for lin in st:
            lin.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
