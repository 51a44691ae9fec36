#!/usr/bin/env python3
"""Benchmark of the any-precision GEMV hot path on one MI355X.

Workload (the configuration the headline metric is quoted on): the three linear-layer shapes of
Llama-2-7B (4096x4096, 11008x4096, 4096x11008), 8-bit parent, batch 1, every bit-width b = 3..8.
One step = one ap_gemv per (shape, b): 18 calls.  Inputs are seeded and synthetic (uniform 8-bit
indices, sorted N(0, 0.02) binary16 tables, N(0, 1) binary16 activations) and resident in HBM
before the timed region.  Every call of a step reads a different device copy of its matrix, and a
copy is reused only after several hundred MB of other traffic, so the numbers are HBM-cold
(neither the 256 MB last-level cache nor the L2 holds the data).

Prints ONE JSON line: effective GB/s over the timed steps (algorithmic bytes / elapsed), with the
roofline of the dominant kernel and the CPU oracle timed beside it.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
# HBM bytes per launch of gemv_kernel<b,1>, averaged over the three shapes of the headline workload:
# FETCH_SIZE and WRITE_SIZE from two `rocprofv3 --pmc` runs of this script, each scaled by what the
# counter reads for a plain transfer of known size (ap_probe_read for reads: factor 1.9993;
# the runtime's buffer copy for writes: factor 0.4965).  Source: profiles/gemv_config2_hbm_traffic.txt
MEASURED_TRAFFIC_BYTES = {3: 13773926, 4: 18266645, 5: 22924189, 6: 27796687, 7: 33070470, 8: 39167242}
COPIES = 7      # device copies of every packed matrix (rotation period)


def large_batch(args, np, torch, B, inputs, dev):
    """Dequantise kernel (HBM-bound: reads b/8 bytes, writes 2 bytes per weight) and the
    dequantise + rocBLAS FP16 GEMM path, on the Llama-2-7B shapes."""
    sp = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rows = []
    for (M, K) in inputs.CONFIGS[2]["shapes"]:
        idx, luts, _ = inputs.make_case(2, M, K)
        pm = B.ap_pack(idx, luts, device=dev)
        copies = [pm] + [pm.clone() for _ in range(COPIES - 1)]
        works = [torch.empty(M * K * 2, dtype=torch.uint8, device=dev) for _ in range(4)]
        for b in range(3, 9):
            def issue(n):
                for r in range(n):
                    st = B.lib.ap_dequantize(copies[r % COPIES].handle, b, works[r % 4].data_ptr(), sp)
                    if st != 0:
                        raise RuntimeError("ap_dequantize failed")
            issue(8)
            torch.cuda.synchronize()
            samples = []
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                issue(28)
                e1.record()
                torch.cuda.synchronize()
                samples.append(e0.elapsed_time(e1) * 1e3 / 28)
            us = sorted(samples)[1]
            nbytes = M * K * b // 8 + M * (2 << b) + M * K * 2
            row = dict(M=M, K=K, b=b, dequant_us=round(us, 2), dequant_bytes=nbytes,
                       dequant_GBps=round(nbytes / us / 1e3, 1), frac_of_peak=round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4))
            if b in (4, 8):
                for batch in (16, 64, 256, 512):
                    x = torch.randn((batch, K), dtype=torch.float16, device=dev)
                    y = torch.empty((batch, M), dtype=torch.float16, device=dev)
                    for r in range(3):
                        B.lib.ap_gemm(pm.handle, b, x.data_ptr(), y.data_ptr(), batch, works[0].data_ptr(),
                                      works[0].numel(), sp)
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for r in range(10):
                        B.lib.ap_gemm(copies[r % COPIES].handle, b, x.data_ptr(), y.data_ptr(), batch,
                                      works[r % 4].data_ptr(), works[0].numel(), sp)
                    e1.record()
                    torch.cuda.synchronize()
                    row["gemm_us_batch%d" % batch] = round(e0.elapsed_time(e1) * 1e3 / 10, 2)
            rows.append(row)
            print("  %5dx%-5d b=%d dequantise %7.2f us  %7.1f GB/s (%4.1f%% of 8 TB/s)  %s" %
                  (M, K, b, us, row["dequant_GBps"], 100 * row["frac_of_peak"],
                   " ".join("batch%s=%.1fus" % (k[13:], v) for k, v in row.items() if k.startswith("gemm_us"))),
                  file=sys.stderr)
        for c in copies:
            c.close()
    print(json.dumps(dict(metric="dequantise kernel GB/s (b/8 bytes read + 2 bytes written per weight) and "
                                 "dequantise + dense FP16 GEMM latency", unit="GB/s", n_gpus=1, data="synthetic",
                          rows=rows)))


def decode_step(args, np, torch, B, inputs, dev):
    """Config 4: all 224 matrices of a 7B-shaped model resident, one bit-width per decode step.

    Layer 0's seven matrices are drawn and packed; the other 31 layers are device copies of them
    (distinct addresses are what the memory system sees; 6.5 GB of slices + 1.4 GB of tables).
    Each step issues the 224 batch-1 GEMVs of one token at that step's bit-width, replayed from one
    HIP graph per bit-width; no repacking between steps.
    """
    layer = []
    for k, (M, K) in enumerate(inputs.DECODE_LAYER_SHAPES):
        idx, luts, x = inputs.make_case(4, M, K, salt=k)
        pm = B.ap_pack(idx, luts, device=dev)
        xd = torch.from_numpy(x).to(dev)
        yd = torch.empty((1, M), dtype=torch.float16, device=dev)
        layer.append((M, K, pm, xd, yd))
    model = [[(M, K, pm if l == 0 else pm.clone(), xd, yd) for (M, K, pm, xd, yd) in layer]
             for l in range(inputs.DECODE_LAYERS)]
    cap = torch.cuda.Stream()
    sp = ctypes.c_void_p(cap.cuda_stream)

    def issue(b):
        for lay in model:
            for (M, K, pm, xd, yd) in lay:
                if B.lib.ap_gemv(pm.handle, b, xd.data_ptr(), yd.data_ptr(), 1, sp) != 0:
                    raise RuntimeError("ap_gemv failed")

    # fused: matrices that share their input go out in one launch (q,k,v | o | gate,up | down):
    # 4 launches per layer instead of 7.  Each matrix keeps its own output buffer.
    youts = [[torch.empty((1, M), dtype=torch.float16, device=dev) for (M, K, pm, xd, yd) in lay] for lay in model]
    fused_items = []
    for lay, ys in zip(model, youts):
        for grp in ([0, 1, 2], [3], [4, 5], [6]):
            fused_items.append(B.make_items([(lay[i][2], lay[i][3], ys[i]) for i in grp]))

    def issue_fused(b):
        for arr in fused_items:
            if B.lib.ap_gemv_multi(arr, len(arr), b, 1, sp) != 0:
                raise RuntimeError("ap_gemv_multi failed")

    # work lists (ap_gemv_list): a whole layer per launch (7 items), and 32 items per launch (the 224
    # matrices of config 4 are independent of each other: 7 launches per step)
    layer_lists, wide_lists = {}, {}
    for b in range(3, 9):
        quads = [(lay[i][2], b, lay[i][3], ys[i]) for lay, ys in zip(model, youts) for i in range(len(lay))]
        layer_lists[b] = [B.make_list(quads[k:k + 7]) for k in range(0, len(quads), 7)]
        wide_lists[b] = [B.make_list(quads[k:k + 32]) for k in range(0, len(quads), 32)]

    def issue_lists(lists):
        def fn(b):
            for arr in lists[b]:
                if B.lib.ap_gemv_list(arr, len(arr), sp) != 0:
                    raise RuntimeError("ap_gemv_list failed")
        return fn

    seq = inputs.decode_bit_sequence(64)
    results = {}
    for name, fn in (("separate", issue), ("fused", issue_fused), ("layer_list", issue_lists(layer_lists)),
                     ("list32", issue_lists(wide_lists))):
        graphs = {}
        with torch.cuda.stream(cap):
            for b in range(3, 9):
                fn(b)
                cap.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=cap):
                    fn(b)
                graphs[b] = g
        torch.cuda.synchronize()
        per_b = {b: [] for b in range(3, 9)}
        for b in seq[:6]:
            graphs[b].replay()
        torch.cuda.synchronize()
        for b in seq:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            graphs[b].replay()
            e1.record()
            torch.cuda.synchronize()
            per_b[b].append(e0.elapsed_time(e1) * 1e3)
        rows = []
        for b in range(3, 9):
            nbytes = inputs.DECODE_LAYERS * sum(inputs.algorithmic_bytes(M, K, b) for (M, K) in inputs.DECODE_LAYER_SHAPES)
            if per_b[b]:
                us = float(np.median(per_b[b]))
                rows.append(dict(b=b, steps=len(per_b[b]), us_per_step=round(us, 1), bytes=nbytes,
                                 GBps=round(nbytes / us / 1e3, 1), frac_of_peak=round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)))
                print("  decode step (%s) b=%d: %8.1f us (median of %d)  %7.1f GB/s  %5.1f%% of 8 TB/s" %
                      (name, b, us, len(per_b[b]), nbytes / us / 1e3, 100 * nbytes / us / 1e3 / HBM_PEAK_GBPS),
                      file=sys.stderr)
        results[name] = rows
    print(json.dumps(dict(metric="7B-shaped decode step latency by bit-width (224 batch-1 GEMVs per step; "
                                 "'fused' = 128 launches: q,k,v | o | gate,up | down per layer; 'layer_list' = 32 "
                                 "launches of one layer's 7 matrices; 'list32' = 7 launches of 32 matrices)",
                          unit="us/step", n_gpus=1, data="synthetic", sequence=seq, per_bit_width=results)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=210)
    ap.add_argument("--warmup", type=int, default=105)
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of replaying HIP graphs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--detail", action="store_true", help="also print a per-(shape, b) table to stderr")
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 5],
                    help="benchmark configuration to run (default 2 = the headline workload)")
    ap.add_argument("--batch", type=int, default=1, help="batch size (exploration only; headline is 1)")
    ap.add_argument("--streams", type=int, default=1,
                    help="capture the independent calls of a step round robin on this many streams (parallel graph branches)")
    ap.add_argument("--variant", type=int, default=0,
                    help="kernel-selection override for A/B runs (ap_set_option AP_OPT_VARIANT; 0 = the dispatcher's choice)")
    ap.add_argument("--weights", choices=["uniform", "quantised"], default="uniform",
                    help="uniform: uniform random indices and random tables (headline recipe); quantised: "
                         "indices and tables from the incremental-upscaling quantiser on heavy-tailed weights "
                         "(exploration: same bytes, non-uniform index statistics)")
    ap.add_argument("--large-batch", action="store_true",
                    help="instead of the headline line: the dequantise kernel and the dequantise + dense GEMM "
                         "path (batch 16..512) on the headline shapes; prints one JSON line")
    ap.add_argument("--decode-step", action="store_true",
                    help="instead of the headline line: the 7B-shaped decode step (32 layers x 7 matrices packed "
                         "once, a seeded sequence of per-step bit-widths); prints one JSON line with per-b latency")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2402_10517_amd import binding as B
    from paper_2402_10517_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.decode_step:
        decode_step(args, np, torch, B, inputs, dev)
        return
    if args.large_batch:
        large_batch(args, np, torch, B, inputs, dev)
        return
    cfg = inputs.CONFIGS[args.config]
    shapes = cfg["shapes"]
    batch = args.batch
    bits = list(range(3, 9))

    # ---- inputs resident in HBM -------------------------------------------------------------
    cases = []
    for (M, K) in shapes:
        idx, luts, x = inputs.make_case(args.config, M, K, batch=batch, sigma=cfg["sigma"])
        if args.weights == "quantised":
            W, S = inputs.make_dense_weights(args.config, M, K, sigma=cfg["sigma"])
            idx, luts = B.ap_quantize(W, S, 3, 8, 10)
            del W, S
        pm = B.ap_pack(idx, luts, device=dev)
        ncopies = max(2, min(COPIES, int(2.5e9 // pm.buf.numel())))
        copies = [pm] + [pm.clone() for _ in range(ncopies - 1)]
        if args.variant:
            for c in copies:
                c.set_options(variant=args.variant)
        xd = torch.from_numpy(x).to(dev)
        yd = torch.empty((batch, M), dtype=torch.float16, device=dev)
        cases.append(dict(M=M, K=K, idx=idx, luts=luts, x=x, copies=copies, xd=xd, yd=yd))
    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)

    side = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else []
    # one output buffer per call of a step: the calls are independent (no two write the same memory)
    youts = {(b, i): torch.empty((batch, cs["M"]), dtype=torch.float16, device=dev) for b in bits for i, cs in enumerate(cases)}

    def issue_step(phase, main=None):
        """The 18 calls of one step; `phase` selects which device copies they read.  With side streams
        the calls go round robin over them, forked from and joined to `main`."""
        c = phase * len(bits)
        k = 0
        for s_ in side:
            s_.wait_stream(main)
        for b in bits:
            for i, cs in enumerate(cases):
                pm = cs["copies"][c % len(cs["copies"])]
                spk = ctypes.c_void_p(side[k % len(side)].cuda_stream) if side else sp
                k += 1
                st = B.lib.ap_gemv(pm.handle, b, cs["xd"].data_ptr(), youts[(b, i)].data_ptr(), batch, spk)
                if st != 0:
                    raise RuntimeError("ap_gemv failed: %s" % B.strerror(st))
            c += 1
        for s_ in side:
            main.wait_stream(s_)

    step_bytes = sum(inputs.algorithmic_bytes(cs["M"], cs["K"], b, batch) for cs in cases for b in bits)

    graphs = None
    cycle_graph = None
    if not args.no_graph:
        # one captured graph per rotation phase, plus one graph holding a whole rotation cycle
        # (COPIES consecutive steps) so that long runs pay the replay cost once per cycle;
        # captured on a side stream as torch requires
        graphs = []
        cap = torch.cuda.Stream()
        sp_save = sp
        with torch.cuda.stream(cap):
            sp = ctypes.c_void_p(cap.cuda_stream)
            for phase in range(COPIES):
                issue_step(phase, cap)     # eager warm-up on the capture stream
            cap.synchronize()
            for phase in range(COPIES):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=cap):
                    issue_step(phase, cap)
                graphs.append(g)
            cycle_graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(cycle_graph, stream=cap):
                for phase in range(COPIES):
                    issue_step(phase, cap)
        sp = sp_save
        torch.cuda.synchronize()

    def run_steps(first, count):
        """Steps first .. first+count-1 in order; whole rotation cycles are replayed as one graph."""
        i = first
        while i < first + count:
            if graphs is None:
                issue_step(i % COPIES, stream)
                i += 1
            elif i % COPIES == 0 and i + COPIES <= first + count:
                cycle_graph.replay()
                i += COPIES
            else:
                graphs[i % COPIES].replay()
                i += 1

    run_steps(0, args.warmup)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    run_steps(args.warmup, args.steps)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms = e0.elapsed_time(e1)
    ms_per_step = ms / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel durations, live, with events on the launch stream ---------------------------
    # N back-to-back launches of one (shape, b) over rotating copies between two events (median of 3
    # such runs); the average includes the dispatch gap between dependent launches, so it bounds the
    # kernel time from above.
    per_call = []
    reps = 5 * COPIES
    for b in bits:
        for cs in cases:
            nc = len(cs["copies"])
            for r in range(nc):
                B.lib.ap_gemv(cs["copies"][r].handle, b, cs["xd"].data_ptr(), cs["yd"].data_ptr(), batch, sp)
            torch.cuda.synchronize()
            samples = []
            for _ in range(3):
                a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a0.record()
                for r in range(reps):
                    B.lib.ap_gemv(cs["copies"][r % nc].handle, b, cs["xd"].data_ptr(), cs["yd"].data_ptr(), batch, sp)
                a1.record()
                torch.cuda.synchronize()
                samples.append(a0.elapsed_time(a1) * 1e3 / reps)
            us = sorted(samples)[1]
            nbytes = inputs.algorithmic_bytes(cs["M"], cs["K"], b, batch)
            per_call.append(dict(M=cs["M"], K=cs["K"], b=b, us=round(us, 3), bytes=nbytes,
                                 GBps=round(nbytes / us / 1e3, 1),
                                 frac_of_peak=round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)))
    # counter calibration launches (outside every timed region): a plain read of known size with the
    # slice loads' access shape, so that a rocprofv3 --pmc run of this script holds its own reference
    probe = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    for _ in range(4):
        if B.lib.ap_probe_read(probe.data_ptr(), probe.numel(), sp) != 0:
            raise RuntimeError("ap_probe_read failed")
    torch.cuda.synchronize()

    # dominant kernel = the bit-width whose launches take the most time in a step
    by_b = {}
    for pc in per_call:
        d = by_b.setdefault(pc["b"], dict(us=0.0, bytes=0, n=0))
        d["us"] += pc["us"]
        d["bytes"] += pc["bytes"]
        d["n"] += 1
    dom_b = max(by_b, key=lambda k: by_b[k]["us"])
    dom = by_b[dom_b]
    achieved = dom["bytes"] / dom["us"] / 1e3
    roofline = dict(bound="hbm", kernel="gemv_kernel<%d,%d>" % (dom_b, batch), achieved=round(achieved, 1),
                    peak=HBM_PEAK_GBPS, unit="GB/s", frac=round(achieved / HBM_PEAK_GBPS, 4),
                    bytes_per_launch=dom["bytes"] // dom["n"],
                    avg_launch_us=round(dom["us"] / dom["n"], 3),
                    traffic=MEASURED_TRAFFIC_BYTES.get(dom_b)
                    if args.config == 2 and batch == 1 and args.weights == "uniform" else None)

    # ---- the oracle on the host cores, on a bounded sample of the same workload ----------------
    cpu = None
    if not args.no_cpu:
        import oracle
        cs = cases[0]
        t_cpu, n_bytes, n_calls = 0.0, 0, 0
        while t_cpu < 10.0 and n_calls < 3000:
            for b in bits:
                t1 = time.perf_counter()
                oracle.gemv(cs["idx"], cs["luts"][b], b, cs["x"])
                t_cpu += time.perf_counter() - t1
                n_bytes += inputs.algorithmic_bytes(cs["M"], cs["K"], b)
                n_calls += 1
        cpu = dict(value=round(n_bytes / t_cpu / 1e9, 4), unit="GB/s", cores=oracle.num_threads(),
                   kind="oracle",
                   sample="%d oracle calls on the 4096x4096 matrix, b=3..8 round robin, batch 1 (%.1f s)"
                          % (n_calls, t_cpu),
                   us_per_call=round(t_cpu / n_calls * 1e6, 1))

    out = dict(metric="any-precision GEMV effective GB/s, b=3..8, batch 1 (HBM-cold)", value=round(value, 1),
               unit="GB/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(ms_per_step, 5), higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f16 tables and activations, f32 accumulate", data="synthetic",
               config=dict(workload=("configs[1]: Llama-2-7B linears 4096x4096, 11008x4096, 4096x11008; "
                                     "8-bit parent, b=3..8, batch 1; one step = 18 ap_gemv calls")
                           if args.config == 2 and batch == 1 and args.weights == "uniform" else
                           "exploration: config %d (%s) shapes %s, batch %d, %s weights"
                           % (args.config, cfg["name"], shapes, batch, args.weights),
                           calls_per_step=len(bits) * len(cases), bytes_per_step=step_bytes,
                           device_copies=COPIES, launch="hip-graph" if graphs is not None else "python-loop"),
               frac_of_hbm_peak=round(value / HBM_PEAK_GBPS, 4), us_per_call=round(ms_per_step * 1e3 / (len(bits) * len(cases)), 3),
               wall_ms=round(wall_ms, 2), roofline=roofline, cpu_baseline=cpu, per_call=per_call)
    if args.detail:
        for pc in per_call:
            print("  %5dx%-5d b=%d  %8.2f us  %7.1f GB/s  %5.1f%% of 8 TB/s" %
                  (pc["M"], pc["K"], pc["b"], pc["us"], pc["GBps"], 100 * pc["frac_of_peak"]), file=sys.stderr)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
