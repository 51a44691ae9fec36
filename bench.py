#!/usr/bin/env python3
"""Benchmark of the any-precision GEMV hot path on one MI355X.

Workload of the headline (the configuration the metric is quoted on): the three linear-layer shapes of
Llama-2-7B (4096x4096, 11008x4096, 4096x11008), 8-bit parent, batch 1, every bit-width b = 3..8: 18
matrix-vector products per step.  They are independent of each other, so a step issues them the way the
library offers for independent products: one ap_gemv_list call for all 18 (a list of mixed bit-widths,
as a server decoding several queries at different precisions would issue), replayed from a HIP graph.  The same step as 18 separate ap_gemv calls on one stream is timed beside it
(`serial`), and every (shape, b) of the 7B, 13B and 70B shapes is timed as single calls (`per_call`).
Inputs are seeded and synthetic (uniform 8-bit indices, sorted N(0, sigma) binary16 tables, N(0, 1)
binary16 activations) and resident in HBM before any timed region.  Every call reads a different device
copy of its matrix, and a copy is reused only after several hundred MB of other traffic, so all numbers
are HBM-cold (neither the 256 MB last-level cache nor the L2 holds the data).

Prints ONE JSON line: effective GB/s over the timed steps (algorithmic bytes / elapsed), the roofline of
the dominant kernel, the CPU oracle timed beside it, and the per-call, small-batch and decode-step rows.
"""
import argparse
import ctypes
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
COPIES = 7      # device copies of every packed matrix of the headline (rotation period)
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gemv_config2_hbm_traffic.txt")


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel`, from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE, each scaled by what the counter reads for a plain transfer of known size); None if the
    summary holds no line for it.  Returns (bytes, commit the profile was taken at)."""
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None, None
    m = re.search(r"^traffic_bytes_per_launch\s+%s\s*=\s*(\d+)" % re.escape(kernel), text, re.M)
    c = re.search(r"^taken_at_commit\s*=\s*(\w+)", text, re.M)
    return (int(m.group(1)) if m else None), (c.group(1) if c else None)


def timed_launches(torch, fn, reps, samples=3):
    """Median over `samples` of the average duration (us) of `reps` back-to-back launches between two
    events on the current stream (the launch stream)."""
    out = []
    for _ in range(samples):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for r in range(reps):
            fn(r)
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) * 1e3 / reps)
    return sorted(out)[len(out) // 2]


def probe_issue(torch, B, sp):
    """Issue rates of the instruction kinds the dequantising kernels consist of (ap_probe_issue): 2048 workgroups
    of 256 threads = 32 waves per CU, 8 per SIMD; every wave runs `passes` passes of one group of instructions."""
    kinds = [(0, "8 ds_read_b32, own bank per lane", 8, 0), (1, "8 ds_read_b32, 2-way bank conflict", 8, 0),
             (2, "8 ds_bpermute_b32", 8, 0), (3, "4 ds_read_b128", 4, 0), (4, "32 v_perm_b32", 0, 32),
             (5, "8 ds_read_b32 + 32 v_perm_b32", 8, 32), (6, "8 ds_bpermute_b32 + 32 v_perm_b32", 8, 32)]
    passes, waves_per_cu, waves_per_simd = 2000, 2048 * 4 / 256, 2048 * 4 / 1024
    rows = []
    for kind, what, n_lds, n_valu in kinds:
        def launch(_r, kind=kind):
            if B.lib.ap_probe_issue(kind, passes, sp) != 0:
                raise RuntimeError("ap_probe_issue failed")
        if B.lib.ap_probe_issue(kind, 10, sp) != 0:
            raise RuntimeError("ap_probe_issue failed")
        torch.cuda.synchronize()
        us = timed_launches(torch, launch, 3)
        row = dict(kind=kind, group=what, us=round(us, 1))
        if n_lds:
            row["ns_per_lds_instruction_per_cu"] = round(us * 1e3 / (waves_per_cu * passes * n_lds), 3)
        if n_valu:
            row["ns_per_valu_instruction_per_simd"] = round(us * 1e3 / (waves_per_simd * passes * n_valu), 3)
        rows.append(row)
        print("  kind %d  %-36s %8.1f us%s%s" % (
            kind, what, us,
            "  %6.2f ns per LDS instruction and CU" % row["ns_per_lds_instruction_per_cu"] if n_lds else "",
            "  %6.2f ns per VALU instruction and SIMD" % row["ns_per_valu_instruction_per_simd"] if n_valu else ""),
            file=sys.stderr)
    print(json.dumps(dict(metric="issue rates of LDS and VALU instruction groups (2048 workgroups x 256 threads, %d passes)"
                          % passes, unit="us", n_gpus=1, rows=rows)))


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
            def issue(r):
                if B.lib.ap_dequantize(copies[r % COPIES].handle, b, works[r % 4].data_ptr(), sp) != 0:
                    raise RuntimeError("ap_dequantize failed")
            for r in range(8):
                issue(r)
            torch.cuda.synchronize()
            us = timed_launches(torch, issue, 28)
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
                    row["gemm_us_batch%d" % batch] = round(timed_launches(
                        torch, lambda r: B.lib.ap_gemm(copies[r % COPIES].handle, b, x.data_ptr(), y.data_ptr(), batch,
                                                       works[r % 4].data_ptr(), works[0].numel(), sp), 10, samples=1), 2)
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


def decode_step_rows(np, torch, B, inputs, dev, modes, replays, batch=1):
    """Config 4: all 224 matrices of a 7B-shaped model resident, one bit-width per decode step.

    Layer 0's seven matrices are drawn and packed; the other 31 layers are device copies of them
    (distinct addresses are what the memory system sees; 6.5 GB of slices + 1.4 GB of tables).  Each
    step issues the 224 batch-1 products of one token at that step's bit-width, replayed from one HIP
    graph per bit-width and issue mode; no repacking between steps.  Issue modes:
      separate    224 ap_gemv calls
      fused       ap_gemv_multi for the matrices of a layer that share their input: q,k,v | o | gate,up |
                  down (4 calls per layer; respects the data dependencies inside a real decoder layer)
      layer_list  one ap_gemv_list call per layer (7 matrices; config 4 treats the products as independent)
      list32      ap_gemv_list calls of 32 matrices (7 calls per step)
    `batch` > 1: the same step for `batch` tokens at once (the list modes then call ap_gemv_list_batch).
    Returns {mode: [row per bit-width]}.
    """
    layer = []
    for k, (M, K) in enumerate(inputs.DECODE_LAYER_SHAPES):
        idx, luts, x = inputs.make_case(4, M, K, salt=k, batch=batch)
        pm = B.ap_pack(idx, luts, device=dev)
        layer.append((M, K, pm, torch.from_numpy(x).to(dev)))
    model = [[(M, K, pm if l == 0 else pm.clone(), xd) for (M, K, pm, xd) in layer]
             for l in range(inputs.DECODE_LAYERS)]
    youts = [[torch.empty((batch, M), dtype=torch.float16, device=dev) for (M, K, pm, xd) in lay] for lay in model]
    cap = torch.cuda.Stream()
    sp = ctypes.c_void_p(cap.cuda_stream)
    fused_items = [B.make_items([(lay[i][2], lay[i][3], ys[i]) for i in grp])
                   for lay, ys in zip(model, youts) for grp in ([0, 1, 2], [3], [4, 5], [6])]
    lists = {}
    for b in range(3, 9):
        quads = [(lay[i][2], b, lay[i][3], ys[i]) for lay, ys in zip(model, youts) for i in range(len(lay))]
        lists[("layer_list", b)] = [B.make_list(quads[k:k + 7]) for k in range(0, len(quads), 7)]
        lists[("list32", b)] = [B.make_list(quads[k:k + 32]) for k in range(0, len(quads), 32)]

    def issue(mode, b):
        if mode == "separate":
            for lay, ys in zip(model, youts):
                for (M, K, pm, xd), y in zip(lay, ys):
                    if B.lib.ap_gemv(pm.handle, b, xd.data_ptr(), y.data_ptr(), batch, sp) != 0:
                        raise RuntimeError("ap_gemv failed")
        elif mode == "fused":
            for arr in fused_items:
                if B.lib.ap_gemv_multi(arr, len(arr), b, batch, sp) != 0:
                    raise RuntimeError("ap_gemv_multi failed")
        else:
            for arr in lists[(mode, b)]:
                if B.lib.ap_gemv_list_batch(arr, len(arr), batch, sp) != 0:
                    raise RuntimeError("ap_gemv_list_batch failed")

    seq = inputs.decode_bit_sequence(replays)
    results = {}
    for mode in modes:
        graphs = {}
        with torch.cuda.stream(cap):
            for b in range(3, 9):
                issue(mode, b)
                cap.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=cap):
                    issue(mode, b)
                graphs[b] = g
        torch.cuda.synchronize()
        per_b = {b: [] for b in range(3, 9)}
        for b in range(3, 9):
            graphs[b].replay()
        torch.cuda.synchronize()
        for b in list(seq) + list(range(3, 9)):   # the seeded sequence, then every bit-width once more
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            graphs[b].replay()
            e1.record()
            torch.cuda.synchronize()
            per_b[b].append(e0.elapsed_time(e1) * 1e3)
        rows = []
        for b in range(3, 9):
            nbytes = inputs.DECODE_LAYERS * sum(inputs.algorithmic_bytes(M, K, b, batch) for (M, K) in inputs.DECODE_LAYER_SHAPES)
            us = float(np.median(per_b[b]))
            rows.append(dict(b=b, steps=len(per_b[b]), us_per_step=round(us, 1), bytes=nbytes,
                             GBps=round(nbytes / us / 1e3, 1), frac_of_peak=round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)))
            print("  decode step (%s) b=%d: %8.1f us (median of %d)  %7.1f GB/s  %5.1f%% of 8 TB/s" %
                  (mode, b, us, len(per_b[b]), nbytes / us / 1e3, 100 * nbytes / us / 1e3 / HBM_PEAK_GBPS),
                  file=sys.stderr)
        results[mode] = rows
        del graphs
    for lay in model:
        for (M, K, pm, xd) in lay:
            pm.close()
    return results, seq


def per_call_rows(torch, B, inputs, dev, config, batches, bits, sp, variant=0, detail=False, waves=0, mfma_min_batch=0,
                  warm=False):
    """Single ap_gemv calls of every shape of `config`: back-to-back launches over rotating device
    copies between two events (median of 3 runs); the average includes the dispatch gap between
    dependent launches, so it is at least the kernel's own duration."""
    cfg = inputs.CONFIGS[config]
    rows = []
    for (M, K) in cfg["shapes"]:
        idx, luts, x = inputs.make_case(config, M, K, batch=max(batches), sigma=cfg["sigma"])
        pm = B.ap_pack(idx, luts, device=dev)
        del idx, luts
        ncopies = max(3, min(COPIES, int(0.9e9 // pm.buf.numel()) + 1))
        copies = [pm] + [pm.clone() for _ in range(ncopies - 1)]
        if variant:
            for c in copies:
                c.set_options(variant=variant)
        if waves:
            for c in copies:
                c.set_options(waves=waves)
        if mfma_min_batch:
            for c in copies:
                c.set_options(mfma_min_batch=mfma_min_batch)
        for batch in batches:
            xd = torch.from_numpy(x[:batch].copy()).to(dev)
            yd = torch.empty((batch, M), dtype=torch.float16, device=dev)
            for b in bits:
                def call(r):
                    if B.lib.ap_gemv(copies[r % ncopies].handle, b, xd.data_ptr(), yd.data_ptr(), batch, sp) != 0:
                        raise RuntimeError("ap_gemv failed")
                for r in range(ncopies):
                    call(r)
                torch.cuda.synchronize()
                reps = max(10, min(5 * COPIES, int(2e9 // inputs.algorithmic_bytes(M, K, b, batch))))
                us = timed_launches(torch, call, reps)
                nbytes = inputs.algorithmic_bytes(M, K, b, batch)
                rows.append(dict(config=config, M=M, K=K, b=b, batch=batch, us=round(us, 3), bytes=nbytes,
                                 GBps=round(nbytes / us / 1e3, 1), frac_of_peak=round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)))
                if warm:   # the same device copy every call: the matrix stays in the 256 MB last-level cache
                    rows[-1]["us_cache_warm"] = round(timed_launches(torch, lambda r: call(0), reps), 3)
                if detail:
                    print("  %5dx%-5d b=%d batch %d  %8.2f us  %7.1f GB/s  %5.1f%% of 8 TB/s" %
                          (M, K, b, batch, us, nbytes / us / 1e3, 100 * nbytes / us / 1e3 / HBM_PEAK_GBPS), file=sys.stderr)
        for c in copies:
            c.close()
        del copies, pm
        torch.cuda.empty_cache()
    return rows


ORACLE_ONE_THREAD = r"""
import json, sys, time
sys.path.insert(0, %r)
import oracle
from paper_2402_10517_amd import inputs
idx, luts, x = inputs.make_case(2, 4096, 4096)
t, n, nbytes = 0.0, 0, 0
while t < %f:
    for b in range(3, 9):
        t1 = time.perf_counter()
        oracle.gemv(idx, luts[b], b, x)
        t += time.perf_counter() - t1
        n += 1
        nbytes += inputs.algorithmic_bytes(4096, 4096, b)
print(json.dumps(dict(t=t, n=n, nbytes=nbytes, threads=oracle.num_threads())))
"""


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=210)
    ap.add_argument("--warmup", type=int, default=105)
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of replaying HIP graphs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-extra", action="store_true",
                    help="headline only: skip the 13B / 70B per-call rows, the small-batch rows and the decode step")
    ap.add_argument("--detail", action="store_true", help="also print the per-call tables to stderr")
    ap.add_argument("--issue", choices=["list", "serial", "list3"], default="list",
                    help="how the timed step issues its 18 products: one ap_gemv_list call (default), 18 ap_gemv "
                         "calls on one stream, or (exploration) one ap_gemv_list call per bit-width")
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 5],
                    help="exploration: per-call timing of this configuration only (2 = the full default run)")
    ap.add_argument("--batch", type=int, default=1, help="exploration: batch size of --config 3|5 runs")
    ap.add_argument("--waves", type=int, default=0, help="exploration: waves per row group (ap_set_option AP_OPT_WAVES_PER_GROUP)")
    ap.add_argument("--mfma-min-batch", type=int, default=0,
                    help="exploration: smallest batch for the one-row-per-lane matrix-core kernel (AP_OPT_MFMA_MIN_BATCH; 9 = never)")
    ap.add_argument("--per-call-only", action="store_true",
                    help="exploration: only the single-call timing of --config (2 included) at --batch")
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
                    help="instead of the headline line: the 7B-shaped decode step in every issue mode; one JSON line")
    ap.add_argument("--probe-issue", action="store_true",
                    help="instead of the headline line: issue rates of the LDS and VALU instructions the kernels "
                         "are made of (ap_probe_issue); one JSON line")
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
    bits = list(range(3, 9))
    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)
    if args.probe_issue:
        probe_issue(torch, B, sp)
        return
    if args.decode_step:
        res, seq = decode_step_rows(np, torch, B, inputs, dev, ["separate", "fused", "layer_list", "list32"],
                                    64 if args.batch == 1 else 18, batch=args.batch)
        print(json.dumps(dict(metric="7B-shaped decode step latency by bit-width (224 GEMVs of batch %d per step) per issue mode"
                              % args.batch, unit="us/step", n_gpus=1, data="synthetic", sequence=seq, per_bit_width=res)))
        return
    if args.large_batch:
        large_batch(args, np, torch, B, inputs, dev)
        return
    if args.config != 2 or args.per_call_only:
        rows = per_call_rows(torch, B, inputs, dev, args.config, [args.batch], bits, sp, args.variant, detail=True,
                             waves=args.waves, mfma_min_batch=args.mfma_min_batch)
        print(json.dumps(dict(metric="exploration: single ap_gemv calls", config=args.config, batch=args.batch,
                              variant=args.variant, per_call=rows)))
        return

    # ---- headline inputs resident in HBM ------------------------------------------------------
    cfg = inputs.CONFIGS[2]
    cases = []
    for (M, K) in cfg["shapes"]:
        idx, luts, x = inputs.make_case(2, M, K, sigma=cfg["sigma"])
        if args.weights == "quantised":
            W, S = inputs.make_dense_weights(2, M, K, sigma=cfg["sigma"])
            idx, luts = B.ap_quantize(W, S, 3, 8, 10)
            del W, S
        pm = B.ap_pack(idx, luts, device=dev)
        copies = [pm] + [pm.clone() for _ in range(COPIES - 1)]
        if args.variant:
            for c in copies:
                c.set_options(variant=args.variant)
        cases.append(dict(M=M, K=K, idx=idx, luts=luts, x=x, copies=copies, xd=torch.from_numpy(x).to(dev)))
    # one output buffer per product of a step (no two write the same memory)
    youts = {(b, i): torch.empty((1, cs["M"]), dtype=torch.float16, device=dev) for b in bits for i, cs in enumerate(cases)}
    # the list of bit-width b in rotation phase p reads copy (p * 6 + b - 3) % COPIES of every matrix
    lists = {(p, b): B.make_list([(cs["copies"][(p * len(bits) + b - 3) % COPIES], b, cs["xd"], youts[(b, i)])
                                  for i, cs in enumerate(cases)])
             for p in range(COPIES) for b in bits}

    lists18 = {p: B.make_list([(cs["copies"][(p * len(bits) + b - 3) % COPIES], b, cs["xd"], youts[(b, i)])
                               for b in bits for i, cs in enumerate(cases)]) for p in range(COPIES)}

    def issue_step(phase, sp_, mode):
        """The 18 products of one step; `phase` selects which device copies they read."""
        if mode == "list":   # one call for all 18 products (a list of mixed bit-widths)
            arr = lists18[phase]
            st = B.lib.ap_gemv_list(arr, len(arr), sp_)
            if st != 0:
                raise RuntimeError("ap_gemv_list failed: %s" % B.strerror(st))
            return
        for b in bits:
            if mode == "list3":
                arr = lists[(phase, b)]
                st = B.lib.ap_gemv_list(arr, len(arr), sp_)
                if st != 0:
                    raise RuntimeError("ap_gemv_list failed: %s" % B.strerror(st))
            else:
                for i, cs in enumerate(cases):
                    pm = cs["copies"][(phase * len(bits) + b - 3) % COPIES]
                    st = B.lib.ap_gemv(pm.handle, b, cs["xd"].data_ptr(), youts[(b, i)].data_ptr(), 1, sp_)
                    if st != 0:
                        raise RuntimeError("ap_gemv failed: %s" % B.strerror(st))

    step_bytes = sum(inputs.algorithmic_bytes(cs["M"], cs["K"], b) for cs in cases for b in bits)

    def time_steps(mode, steps, warmup):
        """`steps` timed steps after `warmup` untimed ones; one captured graph per rotation phase plus one
        graph holding a whole rotation cycle (COPIES consecutive steps), captured on a side stream."""
        graphs, cycle = None, None
        if not args.no_graph:
            graphs = []
            cap = torch.cuda.Stream()
            spc = ctypes.c_void_p(cap.cuda_stream)
            with torch.cuda.stream(cap):
                for phase in range(COPIES):
                    issue_step(phase, spc, mode)      # eager warm-up on the capture stream
                cap.synchronize()
                for phase in range(COPIES):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=cap):
                        issue_step(phase, spc, mode)
                    graphs.append(g)
                cycle = torch.cuda.CUDAGraph()
                with torch.cuda.graph(cycle, stream=cap):
                    for phase in range(COPIES):
                        issue_step(phase, spc, mode)
            torch.cuda.synchronize()

        def run(first, count):
            i = first
            while i < first + count:
                if graphs is None:
                    issue_step(i % COPIES, sp, mode)
                    i += 1
                elif i % COPIES == 0 and i + COPIES <= first + count:
                    cycle.replay()
                    i += COPIES
                else:
                    graphs[i % COPIES].replay()
                    i += 1

        run(0, warmup)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        run(warmup, steps)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        ms = e0.elapsed_time(e1) / steps
        return ms, wall_ms

    ms_per_step, wall_ms = time_steps(args.issue, args.steps, args.warmup)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    other = "serial" if args.issue != "serial" else "list"
    o_ms, _ = time_steps(other, max(7, args.steps // 3), max(7, args.warmup // 3))
    other_row = dict(issue=other, value=round(step_bytes / (o_ms * 1e-3) / 1e9, 1), unit="GB/s", ms_per_step=round(o_ms, 5),
                     frac_of_hbm_peak=round(step_bytes / (o_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4))

    # ---- the dominant kernel of the timed step, live, with events on the launch stream -----------
    # A list call launches its kernel once per class of row length (rows that need the same number of
    # waves): here two launches per call, the 4096-column matrices and the 11008-column ones.  N
    # back-to-back calls over rotating copies between two events; per launch = per call / launches.
    def call18(r):
        arr = lists18[r % COPIES]
        if B.lib.ap_gemv_list(arr, len(arr), sp) != 0:
            raise RuntimeError("ap_gemv_list failed")
    for r in range(COPIES):
        call18(r)
    torch.cuda.synchronize()
    list_us = timed_launches(torch, call18, 5 * COPIES)
    # one launch per class of waves per row group (one wave per span of 2048 columns up to 4 spans, half as many
    # for 5 to 8 spans, 8 beyond)
    def list_waves(K):
        n = (K + 2047) // 2048
        return (n + 1) // 2 if 5 <= n <= 8 else min(8, n)
    list_launches = len({list_waves(cs["K"]) for cs in cases})
    list_call = dict(products=len(bits) * len(cases), launches=list_launches, us=round(list_us, 3), bytes=step_bytes,
                     GBps=round(step_bytes / list_us / 1e3, 1), frac_of_peak=round(step_bytes / list_us / 1e3 / HBM_PEAK_GBPS, 4))
    per_call = per_call_rows(torch, B, inputs, dev, 2, [1], bits, sp, args.variant, args.detail, warm=True)
    # counter calibration launches (outside every timed region): a plain read of known size with the slice
    # loads' access shape, so that a rocprofv3 --pmc run of this script holds its own reference (for
    # writes: the device-to-device copies of the packed matrices made above)
    probe = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    for _ in range(4):
        if B.lib.ap_probe_read(probe.data_ptr(), probe.numel(), sp) != 0:
            raise RuntimeError("ap_probe_read failed")
    torch.cuda.synchronize()
    del probe
    # streaming-read ceiling: the same plain read kernel over 240 MB pieces of a 960 MB buffer in rotation
    # (HBM-cold like the products), back-to-back launches between two events
    big = torch.empty(960 << 20, dtype=torch.uint8, device=dev)
    piece = 240 << 20

    def read_piece(r):
        if B.lib.ap_probe_read(big.data_ptr() + (r % 4) * piece, piece, sp) != 0:
            raise RuntimeError("ap_probe_read failed")
    for r in range(4):
        read_piece(r)
    torch.cuda.synchronize()
    read_us = timed_launches(torch, read_piece, 20)
    read_ceiling = dict(bytes=piece, us=round(read_us, 2), GBps=round(piece / read_us / 1e3, 1),
                        frac_of_peak=round(piece / read_us / 1e3 / HBM_PEAK_GBPS, 4))
    del big
    torch.cuda.empty_cache()
    if args.issue == "list":
        kernel = "gemv_list_kernel<0,1,512>"   # template arguments: 0 = list of mixed bit-widths, 1 = batch 1
        dom_bytes, dom_us = step_bytes // list_launches, list_us / list_launches
    else:
        by_b = {}
        for pc in per_call:
            d = by_b.setdefault(pc["b"], dict(us=0.0, bytes=0, n=0))
            d["us"] += pc["us"]
            d["bytes"] += pc["bytes"]
            d["n"] += 1
        dom_b = max(by_b, key=lambda k: by_b[k]["us"])
        kernel = "gemv_kernel<%d,1>" % dom_b
        dom_bytes, dom_us = by_b[dom_b]["bytes"] // by_b[dom_b]["n"], by_b[dom_b]["us"] / by_b[dom_b]["n"]
    traffic, traffic_commit = measured_traffic(kernel) if args.weights == "uniform" and not args.variant else (None, None)
    achieved = dom_bytes / dom_us / 1e3
    roofline = dict(bound="hbm", kernel=kernel, achieved=round(achieved, 1), peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBPS, 4), frac_of_read_ceiling=round(achieved / read_ceiling["GBps"], 4),
                    bytes_per_launch=dom_bytes,
                    avg_launch_us=round(dom_us, 3), traffic=traffic, traffic_from="profiles/gemv_config2_hbm_traffic.txt"
                    + (" @ " + traffic_commit if traffic_commit else ""))

    # ---- the other configurations: single calls on the 13B and 70B shapes, small batches, decode step
    extra = {}
    if not args.no_extra:
        per_call += per_call_rows(torch, B, inputs, dev, 3, [1], bits, sp, args.variant, args.detail)
        per_call += per_call_rows(torch, B, inputs, dev, 5, [1], bits, sp, args.variant, args.detail)
        idx, luts, x = inputs.make_case(5, 28672, 8192, batch=8, sigma=0.01)
        pm = B.ap_pack(idx, luts, device=dev)
        del idx, luts
        copies = [pm, pm.clone(), pm.clone()]
        small = []
        for batch in (2, 4, 8, 16):   # 16 = two passes of 8 rows
            xd = torch.from_numpy(np.concatenate([x, x])[:batch].copy()).to(dev)
            yd = torch.empty((batch, 28672), dtype=torch.float16, device=dev)
            for b in bits:
                def call(r):
                    if B.lib.ap_gemv(copies[r % 3].handle, b, xd.data_ptr(), yd.data_ptr(), batch, sp) != 0:
                        raise RuntimeError("ap_gemv failed")
                for r in range(3):
                    call(r)
                torch.cuda.synchronize()
                us = timed_launches(torch, call, 12)
                nbytes = inputs.algorithmic_bytes(28672, 8192, b, batch)
                b1 = [pc["us"] for pc in per_call if (pc["M"], pc["K"], pc["b"]) == (28672, 8192, b)][0]
                small.append(dict(M=28672, K=8192, b=b, batch=batch, us=round(us, 2), x_batch1=round(us / b1, 3),
                                  GBps=round(nbytes / us / 1e3, 1), frac_of_peak=round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)))
        for c in copies:
            c.close()
        del copies, pm
        torch.cuda.empty_cache()
        extra["small_batch"] = small
        dec, seq = decode_step_rows(np, torch, B, inputs, dev, ["fused", "layer_list", "list32"], 18)
        extra["decode_step"] = dict(workload="configs[3]: 32 layers x 7 matrices packed once, one bit-width per step, "
                                             "batch 1; us per step by issue mode (fused = q,k,v | o | gate,up | down per "
                                             "layer; layer_list = one ap_gemv_list per layer; list32 = 32 matrices per call)",
                                    sequence=seq, per_bit_width=dec)
        dec8, _ = decode_step_rows(np, torch, B, inputs, dev, ["separate", "fused", "list32"], 6, batch=8)
        extra["decode_step_batch8"] = dict(workload="the same model and step for 8 tokens at once (batch 8): 224 ap_gemv calls, "
                                                    "ap_gemv_multi per group of equal row length (4 calls per layer), or "
                                                    "ap_gemv_list_batch with 32 matrices per call",
                                           per_bit_width=dec8)

    # ---- the oracle on the host cores, on a bounded sample of the same workload ------------------
    cpu = None
    if not args.no_cpu:
        import oracle
        cs = cases[0]
        t_cpu, n_bytes, n_calls = 0.0, 0, 0
        while t_cpu < 8.0 and n_calls < 3000:
            for b in bits:
                t1 = time.perf_counter()
                oracle.gemv(cs["idx"], cs["luts"][b], b, cs["x"])
                t_cpu += time.perf_counter() - t1
                n_bytes += inputs.algorithmic_bytes(cs["M"], cs["K"], b)
                n_calls += 1
        cpu = dict(value=round(n_bytes / t_cpu / 1e9, 4), unit="GB/s", cores=oracle.num_threads(), kind="oracle",
                   sample="%d oracle calls on the 4096x4096 matrix, b=3..8 round robin, batch 1 (%.1f s)" % (n_calls, t_cpu),
                   us_per_call=round(t_cpu / n_calls * 1e6, 1))
        # the same sample on one thread (a child process: the thread count of the OpenMP runtime is fixed at start-up)
        try:
            env = dict(os.environ, OMP_NUM_THREADS="1")
            out = subprocess.run([sys.executable, "-c", ORACLE_ONE_THREAD % (ROOT, 6.0)], env=env, capture_output=True,
                                 text=True, timeout=120, check=True).stdout
            r1 = json.loads(out.strip().splitlines()[-1])
            cpu["one_thread"] = dict(value=round(r1["nbytes"] / r1["t"] / 1e9, 4), unit="GB/s", cores=r1["threads"],
                                     us_per_call=round(r1["t"] / r1["n"] * 1e6, 1),
                                     sample="%d calls, same matrix (%.1f s)" % (r1["n"], r1["t"]))
        except Exception as e:   # the baseline is a report, not a gate
            cpu["one_thread"] = dict(error=str(e)[:200])

    issue_text = {"list": "one ap_gemv_list call (a list of mixed bit-widths)", "serial": "18 ap_gemv calls on one stream",
                  "list3": "one ap_gemv_list call per bit-width (3 matrices each)"}[args.issue]
    out = dict(metric="any-precision GEMV effective GB/s, b=3..8, batch 1 (HBM-cold)", value=round(value, 1),
               unit="GB/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(ms_per_step, 5), higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f16 tables and activations, f32 accumulate", data="synthetic",
               config=dict(workload=("configs[1]: Llama-2-7B linears 4096x4096, 11008x4096, 4096x11008; 8-bit parent, "
                                     "b=3..8, batch 1; one step = 18 independent products, issued as " + issue_text)
                           if args.weights == "uniform" and not args.variant else
                           "exploration: config 2 shapes, batch 1, %s weights, variant %d" % (args.weights, args.variant),
                           products_per_step=len(bits) * len(cases), bytes_per_step=step_bytes, issue=args.issue,
                           device_copies=COPIES, launch="hip-graph" if not args.no_graph else "python-loop"),
               frac_of_hbm_peak=round(value / HBM_PEAK_GBPS, 4), us_per_product=round(ms_per_step * 1e3 / (len(bits) * len(cases)), 3),
               wall_ms=round(wall_ms, 2), roofline=roofline, cpu_baseline=cpu, other_issue=other_row,
               list_call=list_call, read_ceiling=read_ceiling, per_call=per_call, **extra)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
