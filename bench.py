#!/usr/bin/env python3
"""Benchmark of the simulated low-bit-width-accumulator GEMM on one MI355X.

A "step" is one pass of the hot path over the default workload: every convolution (as an im2col
GEMM) and the FC layer of a ResNet-50 forward pass at batch 64, 224x224 (54 GEMMs,
2.617e11 LBA-MACs), with FP8 E4M3 operands, Q_prod = M7E5 (b=15) and the 12-bit accumulator
Q_acc = M7E4 (b=7), biases folded by the per-tensor power-of-two scales, sequential order,
floor rounding (the paper's LBA rounding, Sec. 3).  Inputs are synthetic and resident in HBM
before the timed region.  Prints ONE JSON line.

Other workloads (for profiling, not the headline): --workload conv (ResNet-18 3x3 conv 64->64 at
batch 32), bert (BERT-base linears at 4096 tokens), gemm4096 (4096^3; --acc E,M sweeps the accumulator
format), config1 (one 64x64x256 GEMM: launch latency), layer:MxNxK (one GEMM of that shape with the ResNet-50
data recipe: per-shape profiles).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# 256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz = 78.6e12 full-rate VALU lane-ops per second: the
# rate behind the published 157.3 TFLOP/s FP32 vector peak (an FMA counts two flops).
PEAK_LANE_OPS = 256 * 4 * 32 * 2.4e9
# Counter-derived figures (HBM bytes per launch from calibrated FETCH_SIZE / WRITE_SIZE runs, VALU instructions
# issued per MAC from SQ_INSTS_VALU, the rate the issue-rate probe sustains with a kernel's own instruction mix)
# are not measured by this script: they come from profiles/roofline_counters.json, written by
# paper_2401_14110_amd/rocprof_record.py from rocprofv3 runs of this script, and are reported only when the
# record's workload and kernel name are the ones that ran here; otherwise the fields are null.
COUNTER_RECORDS = os.path.join(ROOT, "profiles", "roofline_counters.json")
PROD_FMT = (5, 7, 15)
ACC_FMT = (4, 7, 7)


def counter_record(workload_key, kernel_name):
    """The record of rocprof_record.py for this workload and kernel, or None."""
    try:
        with open(COUNTER_RECORDS) as f:
            data = json.load(f)
    except (OSError, ValueError):
        return None
    for rec in data.get("records", []):
        if rec.get("workload_key") == workload_key and kernel_name in rec.get("kernels", {}):
            return dict(rec["kernels"][kernel_name], commit=rec.get("commit"), probe=data.get("valu_probe", {}))
    return None


def cpu_baseline(layer, qp, qa, C_gpu, order=0, threads=None, budget_macs=2.0e9):
    """The oracle, as it stands, on a bounded slab of one layer; also a parity check of the slab."""
    import numpy as np
    from oracle import lba_ref
    if not threads:
        threads = min(16, os.cpu_count() or 1)
    budget_macs = budget_macs * min(1.0, threads / 8.0)           # keeps the leg near 10-30 s
    rows = int(min(layer["M"], max(1, budget_macs // (layer["N"] * layer["K"]))))
    A = layer["A"][:rows].cpu().numpy()
    B = layer["B"].cpu().numpy()
    t0 = time.perf_counter()
    if "fa" in layer:
        want = lba_ref.gemm_in(A, B, lba_ref.InFmt(*layer["fa"]), lba_ref.InFmt(*layer["fb"]), lba_ref.QFmt(*qp),
                               lba_ref.QFmt(*qa), order=order, nthreads=threads)
    else:
        want = lba_ref.gemm(A, B, lba_ref.QFmt(*qp), lba_ref.QFmt(*qa), order=order, nthreads=threads)
    dt = time.perf_counter() - t0
    got = C_gpu[:rows].cpu().numpy()
    parity = bool(np.array_equal(got.view(np.uint32), want.view(np.uint32)))
    macs = rows * layer["N"] * layer["K"]
    # the same oracle on one thread, on a sixteenth of the slab
    rows1 = max(1, rows // 16)
    t0 = time.perf_counter()
    if "fa" in layer:
        lba_ref.gemm_in(A[:rows1], B, lba_ref.InFmt(*layer["fa"]), lba_ref.InFmt(*layer["fb"]), lba_ref.QFmt(*qp),
                        lba_ref.QFmt(*qa), order=order, nthreads=1)
    else:
        lba_ref.gemm(A[:rows1], B, lba_ref.QFmt(*qp), lba_ref.QFmt(*qa), order=order, nthreads=1)
    dt1 = time.perf_counter() - t0
    return {"value": macs / dt, "unit": "LBA-MAC/s", "cores": threads, "kind": "oracle",
            "sample": "first %d rows of %s (M=%d,N=%d,K=%d), %.3g MACs, %.1f s" %
                      (rows, layer["name"], layer["M"], layer["N"], layer["K"], macs, dt),
            "value_1_thread": rows1 * layer["N"] * layer["K"] / dt1,
            "sample_1_thread": "first %d rows, %.1f s" % (rows1, dt1),
            "bit_exact_vs_gpu": parity}


def make_parser():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--round", default="floor", choices=["floor", "rne"])
    ap.add_argument("--order", default="seq", choices=["seq", "chunk16"],
                    help="accumulation order: one sequential chain (default) or the paper's chunks of 16")
    ap.add_argument("--acc", default=None, metavar="E,M",
                    help="accumulator format with b = 2^(E-1)-1 instead of the 12-bit M7E4 (format sweeps)")
    ap.add_argument("--in-fmt", default=None, metavar="E,M",
                    help="operands in that 8-bit format with per-tensor flex bias (3,4 = the paper's M4E3) through lba_gemm_in")
    ap.add_argument("--implicit", action="store_true",
                    help="resnet50 / conv workloads: convolutions straight from NHWC activation tensors (lba_conv2d)")
    ap.add_argument("--bwd", action="store_true",
                    help="time lba_gemm_bwd (forward chain + both event planes) instead of lba_gemm")
    ap.add_argument("--of-only", action="store_true", help="with --bwd: ask for the overflow plane only")
    ap.add_argument("--diff", type=float, default=None, metavar="EPS2",
                    help="with --bwd: time lba_gemm_bwd_diff (C + the DIFF plane for that threshold) instead")
    ap.add_argument("--grad", default=None, choices=["identity", "immediate", "recursive", "premapped"],
                    help="time lba_grad (dX and dW with that estimator's coefficients; the OF planes / last-overflow "
                         "indices are computed before the timed region) instead of lba_gemm; 2 MACs per forward MAC; "
                         "premapped: the immediate estimator through lba_grad_premapped, with the brick maps left by "
                         "lba_gemm_bwd_ws before the timed region")
    ap.add_argument("--ws", action="store_true",
                    help="with --grad identity / recursive: time lba_grad_ws with a workspace of lba_grad_workspace_bytes_fast bytes (split sums combined there)")
    ap.add_argument("--maps", action="store_true", help="with --bwd: time lba_gemm_bwd_ws (also leaves the brick maps) instead")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-threads", type=int, default=0, help="threads of the oracle leg (default: min(16, cores))")
    ap.add_argument("--per-layer", action="store_true", help="also print a per-layer table to stderr")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the steps, run a 1 GiB fill and a 1 GiB add (references for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--results", default=None, metavar="FILE",
                    help="append one JSON line per GEMM of the workload (shape, formats, rounding, order, kernel, time, MAC/s, "
                         "checksum of the complete output and its verdict against the offline oracle checksum of "
                         "tests/golden/full_digests.txt); forward call on E4M3 operands only")
    ap.add_argument("--dump-kernels", default=None, metavar="FILE",
                    help="write the kernels of one step (name, launches, MACs, algorithmic bytes, issue slots per MAC) as "
                         "JSON: the input rocprof_record.py pairs with the profiler's per-kernel counters")
    ap.add_argument("--paper-biases", action="store_true",
                    help="Q_prod = M7E4 b=12, Q_acc = M7E4 b=10: the paper's own bias pair (Sec. 3.1) instead of M7E5 b=15 / M7E4 b=7")
    ap.add_argument("--suite", default=None, metavar="OUT.md",
                    help="run every configuration of the summary table (SUITE below) one after the other and write the table "
                         "to OUT.md and the JSON lines to OUT.jsonl")
    return ap


def run(args):
    """One benchmark configuration; returns the dictionary of the JSON line."""
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU (every output chain is independent; "
                         "rows of A and of C would shard across GPUs with B replicated and nothing exchanged). Use --gpus 1.")
    import torch
    from paper_2401_14110_amd import binding as lb
    from paper_2401_14110_amd import inputs
    lb.lib()
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    rnd = 0 if args.round == "floor" else 1
    order = 0 if args.order == "seq" else 1

    acc_fmt = ACC_FMT
    prod_fmt = PROD_FMT
    if args.paper_biases:
        prod_fmt, acc_fmt = (4, 7, 12), (4, 7, 10)
    if args.acc:
        e, m = (int(v) for v in args.acc.split(","))
        acc_fmt = (e, m, 2 ** (e - 1) - 1)
    in_fmt = tuple(int(v) for v in args.in_fmt.split(",")) if args.in_fmt else None
    if args.diff is not None and (not args.bwd or args.of_only or args.in_fmt or args.grad):
        raise SystemExit("bench.py: --diff goes with --bwd alone (E4M3 operands)")
    with_masks = 2 if args.diff is not None else ((3 if (args.of_only and order == 0) else 1) if args.bwd else 0)
    if in_fmt and (args.grad or (args.bwd and order == 1)):
        raise SystemExit("bench.py: --in-fmt times lba_gemm_in or lba_gemm_bwd_in (sequential order)")
    if args.implicit and (in_fmt or args.grad or args.diff is not None or args.maps or (args.bwd and (order == 1 or rnd != 0))):
        raise SystemExit("bench.py: --implicit times lba_conv2d, or with --bwd lba_conv2d_bwd under floor rounding and the sequential order")
    layers = inputs.make_conv_workload(args.workload, dev) if args.implicit else inputs.make_workload(args.workload, dev, in_fmt=in_fmt)
    cmax = max(l["M"] * l["N"] for l in layers)
    Cbuf = torch.empty(cmax, dtype=torch.float32, device=dev)
    for l in layers:
        if in_fmt:                                          # biases stay in real units: the library folds the flex biases
            l["qp"], l["qa"] = prod_fmt + (rnd,), acc_fmt + (rnd,)
            l["fa"], l["fb"] = in_fmt + (l["ta"],), in_fmt + (l["tb"],)
            l["plan"] = lb.lba_plan_query_in(l["M"], l["N"], l["K"], l["fa"], l["fb"], l["qp"], l["qa"], order, with_masks)
            l["kname"] = lb.lba_plan_kernel_name_in(l["M"], l["N"], l["K"], l["fa"], l["fb"], l["qp"], l["qa"], order, with_masks)
            if args.bwd and args.of_only:
                fwd = lb.lba_plan_query_in(l["M"], l["N"], l["K"], l["fa"], l["fb"], l["qp"], l["qa"], order, 0)
                l["plan"] = dict(l["plan"], valu_per_mac_x100=fwd["valu_per_mac_x100"])
        else:
            l["qp"], l["qa"], _ = inputs.folded_formats(l["ta"], l["tb"], prod_fmt, acc_fmt, rnd)
            l["plan"] = lb.lba_plan_query(l["M"], l["N"], l["K"], l["qp"], l["qa"], order, with_masks)
            l["kname"] = lb.lba_plan_kernel_name(l["M"], l["N"], l["K"], l["qp"], l["qa"], order, with_masks)
            if args.bwd and args.of_only and order == 0:
                # priced like the forward call: k-tiles that cannot overflow run the forward tile (3 slots per MAC);
                # tiles that can add a clamp, a compare and a carry-in add per MAC, which this count leaves out
                fwd = lb.lba_plan_query(l["M"], l["N"], l["K"], l["qp"], l["qa"], order, 0)
                l["plan"] = dict(l["plan"], valu_per_mac_x100=fwd["valu_per_mac_x100"])
            if args.implicit:
                l["kname"] = conv_kernel_name(l["kname"])
        l["C"] = Cbuf[: l["M"] * l["N"]].view(l["M"], l["N"])
        l["macs"] = l["M"] * l["N"] * l["K"]
    if args.grad:
        ste = {"identity": 0, "immediate": 1, "recursive": 2, "premapped": 1}[args.grad]
        premapped = args.grad == "premapped"
        stream = torch.cuda.current_stream().cuda_stream
        Gbuf = torch.randn(cmax, dtype=torch.float32, device=dev)
        dXbuf = torch.empty(max(l["M"] * l["K"] for l in layers), dtype=torch.float32, device=dev)
        dWbuf = torch.empty(max(l["N"] * l["K"] for l in layers), dtype=torch.float32, device=dev)
        for l in layers:
            l["macs"] *= 2                                     # dX and dW
            # VALU issue slots per masked MAC (one wave instruction = 64 MACs; half-rate forms count 2).  Vector
            # kernel, identity / recursive: v_fmac with a scalar operand 2 (+ one v_cmp, recursive).  Immediate: priced
            # at its floor, one full-rate v_fmac per 64 terms (a block without a blocked coefficient); blocks with
            # blocked coefficients add two v_readlane per instruction, which this count leaves out
            l["plan"] = dict(l["plan"], kernel=2, prod_mode=ste, valu_per_mac_x100=(200, 100, 400)[ste])
            # identity and (sequential) recursive coefficients are constant inside a k tile: lba_grad runs them as a
            # dense product on the matrix cores when rows of G are aligned
            # ... and so are the bricks of the immediate estimator that hold no overflow (lba_grad_ws; on this workload,
            # whose formats fit the data, that is every brick; the pass over the plane that finds them is inside the
            # timed call)
            if l["N"] % 4 == 0 and (ste == 0 or ste == 1 or l["K"] <= 12288):
                l["plan"] = dict(l["plan"], kernel=3, valu_per_mac_x100=0)
            l["of"] = l["last"] = None
            if premapped:
                _, l["of"], _, l["ws"] = lb.gemm_bwd_ws(l["A"], l["B"], l["qp"], l["qa"], want_c=False, want_uf=False)
            elif ste:
                _, l["of"], _ = lb.gemm_bwd(l["A"], l["B"], l["qp"], l["qa"], want_c=False)
            if ste == 2:
                l["last"] = lb.last_overflow(l["of"], l["K"])
                l["of"] = None
        wsbuf = torch.empty(max(256, max(lb.lba_grad_workspace_bytes_fast(l["M"], l["N"], l["K"]) for l in layers)), dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()

        def launch(l):
            if premapped:
                rc = lb.lba_grad_premapped(Gbuf.data_ptr(), l["A"].data_ptr(), l["B"].data_ptr(), l["of"].data_ptr(),
                                           dXbuf.data_ptr(), dWbuf.data_ptr(), l["M"], l["N"], l["K"], l["ws"].data_ptr(), l["ws"].numel(), stream)
            elif ste == 1 or args.ws:
                rc = lb.lba_grad_ws(Gbuf.data_ptr(), l["A"].data_ptr(), l["B"].data_ptr(),
                                    l["of"].data_ptr() if l["of"] is not None else None,
                                    l["last"].data_ptr() if l["last"] is not None else None,
                                    dXbuf.data_ptr(), dWbuf.data_ptr(), l["M"], l["N"], l["K"], ste, wsbuf.data_ptr(), wsbuf.numel(), stream)
            else:
                rc = lb.lba_grad(Gbuf.data_ptr(), l["A"].data_ptr(), l["B"].data_ptr(),
                                 l["of"].data_ptr() if l["of"] is not None else None,
                                 l["last"].data_ptr() if l["last"] is not None else None,
                                 dXbuf.data_ptr(), dWbuf.data_ptr(), l["M"], l["N"], l["K"], ste, stream)
            if rc != 0:
                raise RuntimeError(lb.lba_strerror(rc))
    total_macs = sum(l["macs"] for l in layers)
    if args.grad:
        pass
    elif args.bwd:
        wmax = max(lb.lba_mask_words(l["M"], l["N"], l["K"]) for l in layers)
        of_buf = torch.empty(wmax, dtype=torch.int32, device=dev)
        uf_buf = torch.empty(wmax, dtype=torch.int32, device=dev)
        stream = torch.cuda.current_stream().cuda_stream
        if args.maps:
            ws_buf = torch.empty(max(256, max(lb.lba_grad_workspace_bytes(l["M"], l["N"], l["K"]) for l in layers)), dtype=torch.uint8, device=dev)

        if order == 1:
            w2max = max(lb.lba_mask_words_level2(l["M"], l["N"], l["K"]) for l in layers)
            of2_buf = torch.empty(w2max, dtype=torch.int32, device=dev)
            uf2_buf = torch.empty(w2max, dtype=torch.int32, device=dev)

        def launch(l):
            if args.diff is not None:
                rc = lb.lba_gemm_bwd_diff(l["A"].data_ptr(), l["B"].data_ptr(), l["C"].data_ptr(), of_buf.data_ptr(),
                                          l["M"], l["N"], l["K"], l["qp"], l["qa"], order, args.diff, stream)
            elif args.implicit:
                rc = lb.lba_conv2d_bwd(l["X"].data_ptr(), l["B"].data_ptr(), l["C"].data_ptr(), of_buf.data_ptr(),
                                       None if args.of_only else uf_buf.data_ptr(), l["desc"], l["cout"], l["qp"], l["qa"], order, stream)
            elif in_fmt:
                rc = lb.lba_gemm_bwd_in(l["A"].data_ptr(), l["B"].data_ptr(), l["C"].data_ptr(), of_buf.data_ptr(),
                                        None if args.of_only else uf_buf.data_ptr(), l["M"], l["N"], l["K"],
                                        l["fa"], l["fb"], l["qp"], l["qa"], order, stream)
            elif order == 1:
                rc = lb.lba_gemm_bwd_chunked(l["A"].data_ptr(), l["B"].data_ptr(), l["C"].data_ptr(), of_buf.data_ptr(),
                                             uf_buf.data_ptr(), of2_buf.data_ptr(), uf2_buf.data_ptr(),
                                             l["M"], l["N"], l["K"], l["qp"], l["qa"], stream)
            elif args.maps:
                rc = lb.lba_gemm_bwd_ws(l["A"].data_ptr(), l["B"].data_ptr(), l["C"].data_ptr(), of_buf.data_ptr(),
                                        None if args.of_only else uf_buf.data_ptr(), l["M"], l["N"], l["K"], l["qp"], l["qa"],
                                        ws_buf.data_ptr(), ws_buf.numel(), stream)
            else:
                rc = lb.lba_gemm_bwd(l["A"].data_ptr(), l["B"].data_ptr(), l["C"].data_ptr(), of_buf.data_ptr(),
                                     None if args.of_only else uf_buf.data_ptr(), l["M"], l["N"], l["K"], l["qp"], l["qa"], order, stream)
            if rc != 0:
                raise RuntimeError(lb.lba_strerror(rc))
    else:
        stream0 = torch.cuda.current_stream().cuda_stream

        def launch(l):
            if args.implicit:
                rc = lb.lba_conv2d(l["X"].data_ptr(), l["B"].data_ptr(), l["C"].data_ptr(), l["desc"], l["cout"],
                                   l["qp"], l["qa"], order, stream0)
                if rc != 0:
                    raise RuntimeError(lb.lba_strerror(rc))
            elif in_fmt:
                rc = lb.lba_gemm_in(l["A"].data_ptr(), l["B"].data_ptr(), l["C"].data_ptr(), l["M"], l["N"], l["K"],
                                    l["fa"], l["fb"], l["qp"], l["qa"], order, stream0)
                if rc != 0:
                    raise RuntimeError(lb.lba_strerror(rc))
            else:
                lb.gemm(l["A"], l["B"], l["qp"], l["qa"], order=order, out=l["C"])

    def one_step(events=None):
        for i, l in enumerate(layers):
            if events is not None:
                events[i][0].record()
            launch(l)
            if events is not None:
                events[i][1].record()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(ev[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    if args.copy_calibration:
        # two kernels of known traffic: a fill (writes 1 GiB) and an add (reads 1 GiB, writes 1 GiB)
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()

    ms_per_step = wall * 1e3 / args.steps
    value = total_macs * args.steps / wall

    # per-launch durations (HIP events on the launch stream: torch's current stream is the one every call is given),
    # grouped by the kernel that ran
    def synthetic_name(p):
        fam = ("fast_diff" if args.diff is not None else "fast_bwd" if args.bwd else "fast") if p["kernel"] == 0 else "gen"
        return "lba_%s%s_kernel<%dx%d,bk%d,prod_mode=%d,%s>" % (fam, "_mixed" if p.get("tail_blocks", 0) > 0 else "", p["thread_m"],
                                                                 p["thread_n"], p["tile_k"], p["prod_mode"], "rne" if p["round"] else "floor")

    groups = {}
    per_layer_ms = [0.0] * len(layers)
    step_ms = [0.0] * args.steps
    for s in range(args.steps):
        for i, l in enumerate(layers):
            ms = ev[s][i][0].elapsed_time(ev[s][i][1])
            per_layer_ms[i] += ms / args.steps
            step_ms[s] += ms
            p = l["plan"]
            key = ("lba_grad_kernel<%s>" % args.grad) if args.grad else l.get("kname") or synthetic_name(p)
            if args.grad:
                key = (key, p["kernel"])
            g = groups.setdefault(key, dict(ms=0.0, macs=0, launches=0, bytes=0, ops=p["valu_per_mac_x100"] / 100.0, plan_kernel=p["kernel"]))
            g["ms"] += ms
            g["macs"] += l["macs"]
            if args.grad:     # g (and the plane or the last-overflow indices) once per product, codes once, outputs once
                per_prod = 4 * l["M"] * l["N"] + {"identity": 0, "immediate": l["M"] * l["N"] * ((l["K"] + 31) // 32) * 4,
                                                  "premapped": 0,     # the plane is read only inside marked bricks
                                                  "recursive": 4 * l["M"] * l["N"]}[args.grad]
                g["bytes"] += 2 * per_prod + 5 * (l["M"] * l["K"] + l["N"] * l["K"])
            else:
                g["bytes"] += l["M"] * l["K"] + l["N"] * l["K"] + 4 * l["M"] * l["N"]   # A, B once, C once
                if args.bwd:                                                         # + one bit per MAC and plane
                    planes = 1 if (args.diff is not None or args.of_only) else 2
                    g["bytes"] += 4 * planes * lb.lba_mask_words(l["M"], l["N"], l["K"])
                    if order == 1:
                        g["bytes"] += 4 * 2 * lb.lba_mask_words_level2(l["M"], l["N"], l["K"])
            g["launches"] += 1
    step_ms.sort()
    median_ms = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    dom_key = max(groups, key=lambda k: groups[k]["ms"])
    dom = groups[dom_key]
    dom_name = dom_key[0] if isinstance(dom_key, tuple) else dom_key
    achieved = dom["macs"] * dom["ops"] / (dom["ms"] * 1e-3)
    workload_key = "%s:%s:%s:%s:acc=%d,%d" % (
        args.workload, ("grad-" + args.grad) if args.grad else ("diff" if args.diff is not None else ("bwd-of" if args.of_only else "bwd")) if args.bwd else "fwd",
        args.round, args.order, acc_fmt[0], acc_fmt[1]) + (":in=%d,%d" % in_fmt if in_fmt else "") + (":implicit" if args.implicit else "") + (
        ":paper-biases" if args.paper_biases else "") + (":maps" if args.maps else "") + (":ws" if args.ws else "")
    rec = counter_record(workload_key, dom_name)
    probe_rate = None
    if rec and rec.get("probe_mix"):
        probe_rate = rec["probe"].get(rec["probe_mix"], {}).get("lane_ops_per_s")
    roofline = {
        "bound": "alu", "achieved": achieved / 1e12, "peak": PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
        "frac": achieved / PEAK_LANE_OPS,
        "peak_measured": probe_rate / 1e12 if probe_rate else None,
        "frac_of_measured": achieved / probe_rate if probe_rate else None,
        "traffic": rec.get("traffic_bytes_per_launch") if rec else None,
        "kernel": dom_name,
        "algorithmic_bytes": dom["bytes"] / dom["launches"],
        "valu_slots_per_mac": dom["ops"],
        "issued_valu_per_mac": rec.get("issued_valu_per_mac") if rec else None,
        "counters_from": ("profiles/roofline_counters.json @ %s" % rec.get("commit")) if rec else None,
        "avg_launch_ms": dom["ms"] / dom["launches"],
        "launches": dom["launches"], "mac_per_s": dom["macs"] / (dom["ms"] * 1e-3),
        "time_share": dom["ms"] / sum(g["ms"] for g in groups.values()),
    }
    if args.dump_kernels:
        with open(args.dump_kernels, "w") as f:
            json.dump({"workload_key": workload_key, "steps": args.steps, "warmup": args.warmup,
                       "kernels": {(k[0] if isinstance(k, tuple) else k): dict(
                           launches_per_step=g["launches"] // args.steps, macs_per_step=g["macs"] // args.steps,
                           algorithmic_bytes_per_step=g["bytes"] // args.steps, slots_per_mac=g["ops"],
                           avg_launch_ms_events=g["ms"] / g["launches"]) for k, g in groups.items()}}, f, indent=1)

    if args.grad and dom["plan_kernel"] == 3:
        # three bfloat16 MFMA passes per FP32 x FP8 product (g is split exactly into three bfloat16 pieces):
        # issued flops = 3 x 2 per masked MAC, against the dense bfloat16 peak of the matrix cores
        issued = dom["macs"] * 6 / (dom["ms"] * 1e-3)
        roofline.update({"bound": "mfma", "achieved": issued / 1e12, "peak": 2500.0, "unit": "TFLOP/s", "frac": issued / 2.5e15,
                         "kernel": "lba_grad_dense_kernel<%s> (v_mfma_f32_32x32x16_bf16, 3 passes%s)" % (
                             args.grad, "; lba_grad_ws: the whole call, with the pass over the plane and the vector kernel's bricks" if args.grad == "immediate" else
                             "; lba_grad_premapped: the whole call, with the vector kernel's bricks" if args.grad == "premapped" else ""),
                         "algorithmic_tflops": dom["macs"] * 2 / (dom["ms"] * 1e-3) / 1e12, "valu_slots_per_mac": None,
                         "peak_measured": None, "frac_of_measured": None})

    if args.results and not (args.bwd or args.grad or in_fmt or args.implicit):
        from paper_2401_14110_amd.digest import digest
        gold = {}
        for line in open(os.path.join(ROOT, "tests", "golden", "full_digests.txt")):
            f = line.split()
            if f and not line.startswith("#"):
                gold[(f[0], int(f[1]), f[5], f[6], int(f[7]))] = (int(f[8], 16), int(f[9], 16), int(f[10], 16))
        with open(args.results, "a") as out_f:
            for i, l in enumerate(layers):
                launch(l)
                torch.cuda.synchronize()
                d = digest(l["C"])
                want = gold.get((args.workload, i, ",".join(map(str, l["qp"])), ",".join(map(str, l["qa"])), order))
                if want is None:
                    verdict = "no offline oracle checksum for this case"
                elif (digest(l["A"]), digest(l["B"])) != want[:2]:
                    verdict = "inputs differ from the ones the oracle checksum was made from"
                else:
                    verdict = "bit-exact (complete output)" if d == want[2] else "MISMATCH"
                out_f.write(json.dumps({"workload": args.workload, "layer": i, "name": l["name"], "M": l["M"], "N": l["N"], "K": l["K"],
                                        "qprod": l["qp"], "qacc": l["qa"], "round": args.round, "order": args.order,
                                        "kernel": l.get("kname"), "slots_per_mac": l["plan"]["valu_per_mac_x100"] / 100.0,
                                        "ms": per_layer_ms[i], "mac_per_s": l["macs"] / (per_layer_ms[i] * 1e-3),
                                        "digest_C": "%016x" % d, "parity": verdict}) + "\n")

    if args.per_layer:
        for i, l in enumerate(layers):
            p = l["plan"]
            sys.stderr.write("%-24s M=%-7d N=%-5d K=%-5d %8.3f ms %7.3f TMAC/s  tile %dx%dx%d pm=%d grid=%dx%d\n" % (
                l["name"], l["M"], l["N"], l["K"], per_layer_ms[i], l["macs"] / per_layer_ms[i] / 1e9,
                p["tile_m"], p["tile_n"], p["tile_k"], p["prod_mode"], p["grid_x"], p["grid_y"]))

    out = {
        "metric": "simulated LBA-MACs/sec on one MI355X", "value": value, "unit": "LBA-MAC/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median_events": median_ms, "value_median_events": total_macs / (median_ms * 1e-3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32-carrier/fp8-in",
        "data": "synthetic",
        "config": {"workload": {"resnet50": "ResNet-50 forward, batch 64, 224x224: 53 convs (im2col) + FC as 54 LBA GEMMs",
                                "conv": "ResNet-18 3x3 conv 64->64, batch 32, 56x56 (M=100352,N=64,K=576)",
                                "bert": "BERT-base linears, 4096 tokens", "gemm4096": "4096^3 GEMM",
                                "config1": "single GEMM M=N=64, K=256, operands scaled to max|x|=448"}.get(
                                    args.workload, "single GEMM %s, ReLU activations, He weights" % args.workload),
                   "macs_per_step": total_macs, "qprod": "M%dE%d b=%d" % (prod_fmt[1], prod_fmt[0], prod_fmt[2]), "qacc": "M%dE%d b=%d" % (acc_fmt[1], acc_fmt[0], acc_fmt[2]) + (" (12-bit)" if acc_fmt == ACC_FMT else ""),
                   "call": ("%s, %s estimator: dX and dW (2 masked MACs per forward MAC)" % ({"immediate": "lba_grad_ws", "premapped": "lba_grad_premapped"}.get(args.grad, "lba_grad_ws" if args.ws else "lba_grad"), "immediate" if args.grad == "premapped" else args.grad)) if args.grad else ("lba_gemm_bwd_diff (C + DIFF plane, eps2 = %g)" % args.diff) if args.diff is not None else ("lba_gemm_bwd_chunked (C + four planes)" if order == 1 else (("lba_gemm_bwd_ws" if args.maps else ("lba_conv2d_bwd" if args.implicit else "lba_gemm_bwd")) + (" (C + OF plane)" if args.of_only else " (C + OF and UF planes)"))) if args.bwd else ("lba_conv2d" if args.implicit else "lba_gemm"), "round": args.round, "order": "sequential" if order == 0 else "chunks of 16", "scale": "per-tensor power of two, folded into b",
                   "conv": "implicit im2col from NHWC activations (lba_conv2d)" if args.implicit else "operand A is the written-out im2col matrix",
                   "operands": ("E%dM%d codes with per-tensor flex bias (lba_gemm_in)" % in_fmt) if in_fmt else "E4M3"},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline and not args.grad and not args.implicit:
        # a mid-sized layer whose output is still in the shared buffer: recompute it last
        pick = max(range(len(layers)), key=lambda i: (layers[i]["K"] == 576, layers[i]["M"]))
        l = layers[pick]
        launch(l)
        torch.cuda.synchronize()
        out["cpu_baseline"] = cpu_baseline(l, l["qp"], l["qa"], l["C"], order, args.cpu_threads)
    return out


# The configurations of profiles/all_configs_summary.md: (section, label, flags).
SUITE = [
    ("main", "1: 64x64x256, nearest-even (launch latency)", "--workload config1 --round rne --steps 200 --warmup 20"),
    ("main", "1: same, chunks of 16 (K-parallel kernel)", "--workload config1 --round rne --order chunk16 --steps 200 --warmup 20"),
    ("main", "2: ResNet-18 conv 100352x64x576, floor", "--workload conv --steps 20"),
    ("main", "2: same, nearest-even", "--workload conv --round rne --steps 20"),
    ("main", "3: ResNet-50 sweep, 54 GEMMs, floor (headline)", ""),
    ("main", "3: same, nearest-even", "--round rne"),
    ("main", "3: same, chunks of 16", "--order chunk16"),
    ("main", "3: same, chunks of 16, the paper's biases (10, 12)", "--order chunk16 --paper-biases"),
    ("main", "4: BERT-base linears, floor", "--workload bert --steps 10"),
    ("main", "4: same, nearest-even", "--workload bert --round rne --steps 10"),
    ("main", "2: lba_gemm_bwd (C + 2 planes)", "--workload conv --bwd --steps 3 --warmup 1"),
    ("main", "3: lba_gemm_bwd (C + 2 planes), ResNet-50 sweep", "--bwd --steps 3 --warmup 1"),
    ("main", "3: same, nearest-even", "--bwd --round rne --steps 3 --warmup 1"),
    ("main", "4: lba_gemm_bwd (C + 2 planes)", "--workload bert --bwd --steps 3 --warmup 1"),
    ("main", "5: 4096^3 lba_gemm_bwd, Q_acc M3E4", "--workload gemm4096 --acc 4,3 --bwd --steps 3 --warmup 1"),
    ("main", "5: 4096^3 lba_gemm_bwd, Q_acc M7E4", "--workload gemm4096 --acc 4,7 --bwd --steps 3 --warmup 1"),
    ("main", "5: same, nearest-even", "--workload gemm4096 --acc 4,7 --round rne --bwd --steps 3 --warmup 1"),
    ("main", "5: 4096^3 lba_gemm_bwd, Q_acc M10E6", "--workload gemm4096 --acc 6,10 --bwd --steps 3 --warmup 1"),
    ("wide", "lba_gemm_bwd, OF plane only, ResNet-50 sweep", "--bwd --of-only --steps 5"),
    ("wide", "same, BERT-base linears", "--workload bert --bwd --of-only --steps 5"),
    ("wide", "same, ResNet-18 conv", "--workload conv --bwd --of-only --steps 10"),
    ("wide", "same, 4096^3, Q_acc M7E4", "--workload gemm4096 --acc 4,7 --bwd --of-only --steps 3 --warmup 1"),
    ("wide", "same, 4096^3, Q_acc M7E5", "--workload gemm4096 --acc 5,7 --bwd --of-only --steps 3 --warmup 1"),
    ("wide", "lba_gemm_bwd_diff (C + DIFF plane, eps2 = 0.25), 4096^3, Q_acc M7E4", "--workload gemm4096 --acc 4,7 --bwd --diff 0.25 --steps 3 --warmup 1"),
    ("wide", "same, nearest-even", "--workload gemm4096 --acc 4,7 --round rne --bwd --diff 0.25 --steps 3 --warmup 1"),
    ("wide", "same, chunks of 16", "--workload gemm4096 --acc 4,7 --bwd --diff 0.25 --order chunk16 --steps 3 --warmup 1"),
    ("wide", "same, Q_acc M7E5, nearest-even", "--workload gemm4096 --acc 5,7 --round rne --bwd --diff 0.25 --steps 3 --warmup 1"),
    ("wide", "same, BERT-base linears, M7E4", "--workload bert --bwd --diff 0.25 --steps 3 --warmup 1"),
    ("wide", "same, ResNet-50 sweep, M7E4", "--bwd --diff 0.25 --steps 3 --warmup 1"),
    ("wide", "lba_gemm_bwd_chunked (C + 4 planes), 4096^3", "--workload gemm4096 --acc 4,7 --bwd --order chunk16 --steps 3 --warmup 1"),
    ("wide", "same, BERT-base linears", "--workload bert --bwd --order chunk16 --steps 3 --warmup 1"),
    ("wide", "lba_gemm_in, M4E3 flex-bias operands, ResNet-50 sweep, floor", "--in-fmt 3,4"),
    ("wide", "same, chunks of 16", "--in-fmt 3,4 --order chunk16"),
    ("wide", "same, BERT-base linears", "--in-fmt 3,4 --workload bert --steps 10"),
    ("wide", "same, ResNet-50 sweep, nearest-even (Q_prod rounds the 10-bit products to nearest)", "--in-fmt 3,4 --round rne --steps 5 --warmup 1"),
    ("wide", "lba_gemm_bwd_in, M4E3 operands, OF plane only, ResNet-50 sweep", "--in-fmt 3,4 --bwd --of-only --steps 5"),
    ("wide", "same, both planes, BERT-base linears", "--in-fmt 3,4 --workload bert --bwd --steps 3 --warmup 1"),
    ("wide", "lba_conv2d from NHWC activations, ResNet-50 sweep", "--implicit"),
    ("wide", "same, ResNet-18 conv", "--implicit --workload conv --steps 20"),
    ("wide", "lba_conv2d_bwd (Y + 2 planes) from NHWC activations, ResNet-50 sweep", "--implicit --bwd --steps 3 --warmup 1"),
    ("grad", "lba_grad, identity estimator, ResNet-50 sweep (dX and dW)", "--grad identity --steps 3 --warmup 1"),
    ("grad", "lba_grad, recursive estimator", "--grad recursive --steps 3 --warmup 1"),
    ("grad", "lba_grad_ws, identity estimator (split sums combined in the workspace)", "--grad identity --ws --steps 3 --warmup 1"),
    ("grad", "lba_grad_ws, recursive estimator", "--grad recursive --ws --steps 3 --warmup 1"),
    ("grad", "lba_grad_ws, immediate estimator (pass over the plane + matrix cores + vector kernel)", "--grad immediate --steps 3 --warmup 1"),
    ("grad", "lba_grad, identity estimator, 4096^3", "--workload gemm4096 --grad identity --steps 3 --warmup 1"),
    ("grad", "lba_grad, recursive estimator, 4096^3", "--workload gemm4096 --grad recursive --steps 3 --warmup 1"),
    ("grad", "lba_grad_ws, immediate estimator, 4096^3", "--workload gemm4096 --grad immediate --steps 3 --warmup 1"),
    ("grad", "lba_grad_premapped (maps left by lba_gemm_bwd_ws), immediate estimator, ResNet-50 sweep", "--grad premapped --steps 3 --warmup 1"),
    ("grad", "same, 4096^3", "--workload gemm4096 --grad premapped --steps 3 --warmup 1"),
    ("grad", "same, BERT-base linears", "--workload bert --grad premapped --steps 5 --warmup 2"),
    ("main", "3: lba_gemm_bwd_ws (C + 2 planes + brick maps), ResNet-50 sweep", "--bwd --maps --steps 3 --warmup 1"),
    ("main", "5: same, 4096^3, Q_acc M7E4", "--workload gemm4096 --acc 4,7 --bwd --maps --steps 3 --warmup 1"),
] + [("grad", "%s, %s estimator, %s" % ("lba_grad_ws" if e == "immediate" else "lba_grad", e, n), "--workload %s --grad %s --steps 5 --warmup 2" % (w, e))
     for w, n in (("bert", "BERT-base linears"), ("conv", "ResNet-18 conv")) for e in ("identity", "recursive", "immediate")
] + [("sweep", "%s E%d M%d" % (r, e, m), "--workload gemm4096 --acc %d,%d --round %s --steps 5 --warmup 1" % (e, m, r))
     for r in ("floor", "rne") for e in (4, 5, 6) for m in range(3, 11)]


def run_suite(path):
    """Every configuration of SUITE in this process; writes the summary table and the JSON lines."""
    import gc
    import torch
    ap = make_parser()
    rows = []
    with open(os.path.splitext(path)[0] + ".jsonl", "w") as jl:
        for section, label, flags in SUITE:
            a = ap.parse_args(flags.split() + ["--no-cpu-baseline"])
            out = run(a)
            out["suite"] = {"section": section, "label": label, "flags": flags}
            jl.write(json.dumps(out) + "\n")
            jl.flush()
            rows.append((section, label, flags, out))
            sys.stderr.write("%-80s %8.3f TMAC/s\n" % (label[:80], out["value"] / 1e12))
            gc.collect()
            torch.cuda.empty_cache()

    def line(label, flags, d):
        r = d["roofline"]
        return "| %s | `%s` | %.3f | %.4f | %s | %s | %.3f |" % (
            label, flags or "(none)", d["value"] / 1e12, d["ms_per_step"], r["kernel"].split(" (")[0],
            ("%.1f" % r["valu_slots_per_mac"]) if r.get("valu_slots_per_mac") else "mfma", r["frac"])

    w = []
    w.append("# All five configurations on one MI355X: throughput of the library calls\n")
    w.append("Written by `python bench.py --suite profiles/all_configs_summary.md` (one process, one box; every row is one")
    w.append("configuration of `bench.py` with the flags shown, inputs resident in HBM, HIP events per launch, wall time over the")
    w.append("steps for the rate; the JSON lines are written beside it as `.jsonl`).  `frac` is the dominant kernel's VALU issue")
    w.append("slots per second over the 78.64e12 peak, with the slot count per MAC the planner states for the loop without the")
    w.append("accumulator clamp and without the overflow test (k-tiles in which a sum can reach R_OF add 2 slots per MAC, or 6")
    w.append("with event planes, which the count leaves out: their `frac` under-reports); `mfma`: issued bfloat16 flops over the")
    w.append("2.5e15 peak of the matrix cores.  Parity of all of these configurations is what the GPU tests check.\n")
    for section, title in (("main", "The five configurations"), ("wide", "Widened rows"), ("grad", "Gradient products (2 masked MACs per forward MAC)")):
        w.append("## %s\n" % title)
        w.append("| configuration | bench.py flags | 1e12 MAC/s | ms/step | dominant kernel | slots/MAC | frac |")
        w.append("|---|---|---|---|---|---|---|")
        for sec, label, flags, d in rows:
            if sec == section:
                w.append(line(label, flags, d))
        w.append("")
    w.append("## Configuration 5: accumulator-width sweep on 4096^3 (68.7e9 MACs per call)\n")
    w.append("`python bench.py --workload gemm4096 --acc E,M [--round rne] --steps 5 --warmup 1`, b = 2^(E-1)-1, Q_prod = M7E5 b=15,")
    w.append("biases folded by the operand scales.  Entries: 1e12 LBA-MAC/s (ms per call); `o`: the round-to-odd variant of the")
    w.append("scaled kernel, `g`: the general kernel.\n")
    cells = {l: d for sec, l, f, d in rows if sec == "sweep"}
    for r, title in (("floor", "Floor (the paper's LBA rounding)"), ("rne", "Nearest-even")):
        w.append("%s:\n" % title)
        w.append("| E \\ M | 3 | 4 | 5 | 6 | 7 | 8 | 9 | 10 |")
        w.append("|---|---|---|---|---|---|---|---|---|")
        for e in (4, 5, 6):
            cs = []
            for m in range(3, 11):
                d = cells["%s E%d M%d" % (r, e, m)]
                k = d["roofline"]["kernel"]
                tag = "g" if "gen_kernel" in k else ("o" if k.startswith("lba_fast_kernel") and k.rstrip(">").split(", ")[4] == "3" else "")
                cs.append("%.2f%s (%.2f)" % (d["value"] / 1e12, tag, d["ms_per_step"]))
            w.append("| %d | %s |" % (e, " | ".join(cs)))
        w.append("")
    with open(path, "w") as f:
        f.write("\n".join(w))


def conv_kernel_name(name):
    """The kernel lba_conv2d / lba_conv2d_bwd launch where the row-major call of the same shape and formats launches
    `name`: E4M3 tensors run the same tiles and grids through the instantiations that gather im2col rows."""
    for plain, conv in (("lba_fast_mixed_kernel<", "lba_fast_conv_mixed_kernel<"), ("lba_fast_bwd_mixed_kernel<", "lba_fast_bwd_conv_mixed_kernel<")):
        if name.startswith(plain):
            return conv + name[len(plain):]
    if (name.startswith("lba_fast_kernel<") or name.startswith("lba_fast_bwd_kernel<")) and name.endswith(", 0>"):
        return name[:-4] + ", 2>"
    return name


def main():
    args = make_parser().parse_args()
    if args.suite:
        run_suite(args.suite)
        return
    print(json.dumps(run(args)))


if __name__ == "__main__":
    main()
