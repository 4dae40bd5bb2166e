#!/usr/bin/env python3
"""Benchmark of the quantized-operator hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c2|c3] [--tag int8|fp16]

One "step" is one pass of the whole hot path over one batch of the workload: for every
linear operator of the workload, forward (absmax + quantize of X and W, GEMM with fused
dequantize + bias) and backward (absmax + stochastic-rounding quantize of dY, dX GEMM, dW
GEMM, bias gradient).  Inputs are seeded synthetic tensors already resident in HBM.
Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"int8": 5000.0, "fp16": 2500.0}          # dense MFMA peak of MI355X, TOP/s and TFLOP/s
HBM_PEAK_GBS = 8000.0
# HBM-side bytes per forward-GEMM launch come from the committed rocprofv3 --pmc summaries (FETCH_SIZE and
# WRITE_SIZE, scaled by a plain 512 MiB copy): a line "forward_gemm_traffic_bytes_per_launch: N" in each file.
TRAFFIC_PROFILE = {("c5", "int8", "f16"): "config5_int8_hbm_traffic.md", ("c5", "fp16", "f16"): "config5_fp16_hbm_traffic.md"}


def measured_traffic(workload: str, tag: str, ydtype: str):
    name = TRAFFIC_PROFILE.get((workload, tag, ydtype))
    if name is None:
        return None
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("forward_gemm_traffic_bytes_per_launch:"):
                return int(line.split(":")[1].strip())
    except OSError:
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_workload(name: str):
    from paper_2407_02327_amd import workloads as wl
    if name == "c5":
        c = wl.config5()
        return "config5: BERT-large-scale linears 16384x1024->4096 and 16384x4096->1024", [c["up"], c["down"]]
    if name == "c2":
        return "config2: BERT-base FFN linear 4096x768->3072", [wl.config2()]
    if name == "c3":
        return "config3: ResNet-50 3x3 conv as im2col GEMM M=200704 K=576 N=64", [wl.config3()]
    raise SystemExit(f"unknown workload {name}")


class EventLog:
    """Pairs of events around named launches, recorded on the stream the launch goes to (ms after sync)."""

    def __init__(self):
        import torch
        self.torch = torch
        self.pairs = []

    def run(self, name, fn, stream):
        a = self.torch.cuda.Event(enable_timing=True)
        b = self.torch.cuda.Event(enable_timing=True)
        a.record(stream)
        fn()
        b.record(stream)
        self.pairs.append((name, a, b))

    def totals(self):
        out = {}
        for name, a, b in self.pairs:
            t, n = out.get(name, (0.0, 0))
            out[name] = (t + a.elapsed_time(b), n + 1)
        return out


def cpu_baseline(cases, tag, tokens: int):
    """The oracle, as it stands, on a row-subset of the same workload (the first `tokens` rows of every operator)."""
    import numpy as np
    from oracle import qsync_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    ops = 0
    t0 = time.perf_counter()
    for c in cases:
        m = min(tokens, c.x.shape[0])
        orc.operator_fwd_bwd(tag, c.x[:m], c.w, c.bias, c.dy[:m], c.w_gran, c.dy_round, seed=c.philox_seed,
                             y_dtype=np.float16, dx_dtype=np.float16, dw_dtype=np.float32)
        ops += 6 * m * c.w.shape[0] * c.w.shape[1]
    dt = time.perf_counter() - t0
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": int(cores), "kind": "oracle",
            "sample": f"first {tokens} rows of each operator (of {cases[0].x.shape[0]}), whole operator fwd+bwd "
                      f"incl. absmax/quantize, {dt:.1f} s"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a step takes under a millisecond and the shader clock needs tens of milliseconds to leave its idle state:
    # the defaults keep the timed region at about 0.15 s behind 40 ms of warm-up
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c5", choices=["c5", "c2", "c3"])
    ap.add_argument("--conv-input", default="nhwc", choices=["nhwc", "patches", "implicit"],
                    help="workload c3 with tag int8: start each step from the NHWC activation (quantize it once, "
                         "expand int8 codes into the patch matrix), from the fp16 patch matrix, or run the convolution "
                         "itself (implicit: forward and data gradient gather patches inside the GEMM, dX is the NHWC "
                         "gradient [M,C] instead of the patch gradient [M,9C])")
    ap.add_argument("--tag", default="int8", choices=["int8", "fp16"])
    ap.add_argument("--bwd-tag", default=None, choices=[None, "fp16"],
                    help="fp16 with --tag int8: the paper's pairing, FP16 backward on the dequantized saved codes")
    ap.add_argument("--ydtype", default="f16", choices=["f16", "f32"], help="forward output type")
    ap.add_argument("--cpu-tokens", type=int, default=16384, help="rows per operator given to the CPU oracle")
    ap.add_argument("--streams", type=int, default=1,
                    help="streams over which the workload's independent operators are spread in the timed region "
                         "(1 = one after the other, as a dependent training step would run them)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-extra-passes", action="store_true",
                    help="skip the passes that follow the timed region (per-phase breakdown, operators on separate "
                         "streams): keeps a profile of the run limited to the timed, serial region")
    ap.add_argument("--w-side-stream", type=int, default=0,
                    help="1: an operator's weight conversion runs on a side stream beside its activation conversion "
                         "(measured: the cross-stream join costs about what the overlap saves)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 512 MiB device copy (known traffic) so that rocprofv3 --pmc FETCH_SIZE / "
                         "WRITE_SIZE readings can be scaled")
    ap.add_argument("--gemm-persistent", default="auto", choices=["auto", "0", "1"],
                    help="tuning: 1 launches the persistent 256x256 GEMM kernel whenever a GEMM is eligible (default: never)")
    ap.add_argument("--transposed-copies", default="auto", choices=["auto", "0", "1"],
                    help="tag int8: 1 makes the quantizer also write the transposed activation / gradient codes and the "
                         "weight-gradient GEMM read those; 0 / auto: one row-major copy, transposed on the way into the "
                         "matrix-instruction fragments")
    ap.add_argument("--no-fp16-pass", action="store_true",
                    help="default run (config 5, tag int8): skip the second timed pass with tag fp16")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); run with --gpus 1", file=sys.stderr)
        raise SystemExit(2)
    return args


def run(args):
    """One timed pass (warm-up, K steps) of the workload under args.tag plus, unless args.no_extra_passes, the
    untimed extra passes; returns the dictionary of the JSON line."""
    import torch
    from paper_2407_02327_amd.build import ensure_built
    ensure_built(rebuild_if_stale=True)              # a library older than its sources is rebuilt (or the run fails)
    from paper_2407_02327_amd import qsync as Q
    if args.gemm_persistent != "auto":
        Q.qsync_debug_set_gemm_persistent(int(args.gemm_persistent))
    from paper_2407_02327_amd.operator import QLinear

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    tag = Q.INT8 if args.tag == "int8" else Q.FP16
    desc, cases = build_workload(args.workload)
    log(f"workload: {desc}; tag {args.tag}")
    ydt = torch.float16 if args.ydtype == "f16" else torch.float32
    tdt = {"float16": torch.float16, "float32": torch.float32}
    ops_objs, dev_in = [], []
    for c in cases:
        M, N, K = c.mnk
        op = QLinear(tag, M, N, K, x_dtype=tdt[str(c.x.dtype)], dy_dtype=tdt[str(c.dy.dtype)], y_dtype=ydt,
                     dx_dtype=torch.float16, dw_dtype=torch.float32,
                     w_gran=Q.PER_ROW if c.w_gran == "row" else Q.PER_TENSOR,
                     dy_round=Q.ROUND_STOCHASTIC if c.dy_round == "stochastic" else Q.ROUND_NEAREST,
                     philox_seed=c.philox_seed, bwd_tag=(Q.FP16 if args.bwd_tag == "fp16" and tag == Q.INT8 else None),
                     transposed_copies=(True if args.transposed_copies == "1" else None))
        if c.nhwc is not None and args.conv_input == "implicit":
            from paper_2407_02327_amd.operator import QConv3x3
            b_, h_, w_, c_ = c.nhwc.shape
            op = QConv3x3(tag, b_, h_, w_, c_, N, x_dtype=tdt[str(c.nhwc.dtype)], y_dtype=ydt, dx_dtype=torch.float16,
                          dw_dtype=torch.float32, w_gran=Q.PER_ROW if c.w_gran == "row" else Q.PER_TENSOR,
                          dy_round=Q.ROUND_STOCHASTIC if c.dy_round == "stochastic" else Q.ROUND_NEAREST,
                          philox_seed=c.philox_seed)
            op.convert_x_nhwc, op.gemm_fwd = op.convert_x, op.conv_fwd
            op.gemm_bwd = (lambda o: lambda dy, st=None: (o.conv_dgrad(st), o.conv_wgrad(st)))(op)
        ops_objs.append(op)
        nhwc = c.nhwc is not None and ((tag == Q.INT8 and args.conv_input == "nhwc") or args.conv_input == "implicit")
        x_in = torch.from_numpy(c.nhwc if nhwc else c.x).cuda()
        op.convert_act = op.convert_x_nhwc if nhwc else op.convert_x
        dev_in.append((x_in, torch.from_numpy(c.w).cuda(), torch.from_numpy(c.dy).cuda()))
    torch.cuda.synchronize()

    ev = EventLog()
    main = torch.cuda.current_stream()
    # The operators of a workload are independent of each other, so each gets its own stream
    # (default priority): the HBM-bound conversion kernels of one overlap the MFMA-bound GEMMs
    # of the other.  The small weight-conversion kernels of an operator run on a side stream
    # beside its activation conversion.
    nstreams = max(1, min(args.streams, len(ops_objs)))
    op_streams = [main] + [torch.cuda.Stream() for _ in range(len(ops_objs) - 1)]
    side_streams = [torch.cuda.Stream() for _ in ops_objs]

    def step(record: str, nstreams=nstreams, base=None):
        """record: "none", "gemm_fwd" (events around the forward GEMM only: the timed region) or "all".
        base: the stream of the first operator (default: the current stream at start-up)."""
        def run(name, fn, st):
            if record == "all" or record == name:
                ev.run(name, fn, st)
            else:
                fn()
        first = main if base is None else base
        streams = [first] + op_streams[1:]
        for st in streams[1:nstreams]:
            st.wait_stream(first)
        for i, (op, (x, w, dy)) in enumerate(zip(ops_objs, dev_in)):
            st, side = streams[i % nstreams], side_streams[i]
            if args.w_side_stream:
                side.wait_stream(st)
                op.convert_w(w, side)
                run("convert_x", lambda: op.convert_act(x, st), st)
                st.wait_stream(side)
            else:
                run("convert_x", lambda: (op.convert_w(w, st), op.convert_act(x, st)), st)
            run("gemm_fwd", lambda: op.gemm_fwd(st), st)
            run("convert_dy", lambda: op.convert_dy(dy, st), st)
            run("gemm_bwd", lambda: op.gemm_bwd(dy, st), st)
        for st in streams[1:nstreams]:
            first.wait_stream(st)

    def step_model_order():
        """The operators as consecutive layers of one model: all forwards, then the backwards in reverse order;
        a layer's weight-gradient GEMM runs on a side stream (default priority) beside the next layer's gradient
        conversion and data-gradient GEMM on the main stream."""
        side = side_streams[0]
        for op, (x, w, dy) in zip(ops_objs, dev_in):
            op.convert_w(w, main)
            op.convert_act(x, main)
            op.gemm_fwd(main)
        for op, (x, w, dy) in reversed(list(zip(ops_objs, dev_in))):
            op.convert_dy(dy, main)
            side.wait_stream(main)
            op.gemm_bwd_part("dw", dy, side)
            op.gemm_bwd_part("dx", dy, main)
        main.wait_stream(side)

    def step_dw_beside_next():
        """The serial step, except that every weight-gradient GEMM (nothing downstream needs it before the
        optimizer) runs on a side stream (default priority) beside whatever the main stream does next: the data
        gradient, then the next operator's conversions."""
        side = side_streams[0]
        for op, (x, w, dy) in zip(ops_objs, dev_in):
            op.convert_w(w, main)
            op.convert_act(x, main)
            op.gemm_fwd(main)
            op.convert_dy(dy, main)
            side.wait_stream(main)
            op.gemm_bwd_part("dw", dy, side)
            op.gemm_bwd_part("dx", dy, main)
        main.wait_stream(side)

    def step_weights_ahead():
        """The serial step, except that the weight conversions of the second and later operators (they depend on
        the weights only, which a training step knows from its start) run on a side stream (default priority)
        while the first operator's forward GEMM runs on the main stream."""
        side = side_streams[0]
        pairs = list(zip(ops_objs, dev_in))
        for i, (op, (x, w, dy)) in enumerate(pairs):
            if i == 0:
                op.convert_w(w, main)
                op.convert_act(x, main)
                side.wait_stream(main)
                for op2, (_, w2, _) in pairs[1:]:
                    op2.convert_w(w2, side)
            else:
                op.convert_act(x, main)
                main.wait_stream(side)
            op.gemm_fwd(main)
            op.convert_dy(dy, main)
            op.gemm_bwd(dy, main)

    if args.pmc_calibration:
        src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Timed region: K whole steps; HIP events bracket only the forward GEMM launches (the dominant
    # kernel of the roofline figure), because every event pair costs the stream a few microseconds.
    for _ in range(args.warmup):
        step("none")
    torch.cuda.synchronize()
    # (An event pair costs the stream about 3 us; with events around both forward GEMMs of every step that was
    # 3 % of the step, so every fourth step carries them.)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step("gemm_fwd" if i % 4 == 0 else "none")
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    fwd_ms = ev.totals()["gemm_fwd"][0] / len(range(0, args.steps, 4))

    gemm_ops = sum(6 * c.mnk[0] * c.mnk[1] * c.mnk[2] for c in cases)          # three GEMMs, 2MNK each
    value = gemm_ops / (ms_per_step * 1e-3) / 1e12

    # Extra (outside the timed region above): the same K steps with every operator on its own stream,
    # so that one operator's HBM-bound conversion kernels overlap the other's MFMA-bound GEMMs.
    overlapped = None
    if len(ops_objs) > 1 and nstreams == 1 and not args.no_extra_passes:
        for _ in range(max(2, args.warmup)):
            step("none", len(ops_objs))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step("none", len(ops_objs))
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t1) * 1e3 / args.steps
        overlapped = {"operator_streams": len(ops_objs), "ms_per_step": round(ms2, 4),
                      "value": round(gemm_ops / (ms2 * 1e-3) / 1e12, 3), "unit": "TOPS"}
    # Extra (outside the timed region): the same serial step captured once in a HIP graph and replayed
    # (the library only enqueues kernels: no allocation, no memset, no host copy inside a step).
    graph_replay = None
    if not args.no_extra_passes and not args.w_side_stream:
        saved_offsets = [getattr(o, "offset", 0) for o in ops_objs]
        cap = torch.cuda.Stream()
        cap.wait_stream(main)
        with torch.cuda.stream(cap):
            step("none", 1, base=cap)
        main.wait_stream(cap)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=cap):
            step("none", 1, base=torch.cuda.current_stream())
        for _ in range(max(2, args.warmup)):
            g.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        ms4 = (time.perf_counter() - t1) * 1e3 / args.steps
        graph_replay = {"ms_per_step": round(ms4, 4), "value": round(gemm_ops / (ms4 * 1e-3) / 1e12, 3), "unit": "TOPS",
                        "note": "one serial step captured in a HIP graph, replayed (every replay reuses the captured Philox offsets)"}
        for o, off in zip(ops_objs, saved_offsets):
            if hasattr(o, "offset"):
                o.offset = off
    model_order = None
    if len(ops_objs) > 1 and not args.no_extra_passes and all(hasattr(o, "gemm_bwd_part") for o in ops_objs):
        for _ in range(max(2, args.warmup)):
            step_model_order()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step_model_order()
        torch.cuda.synchronize()
        ms3 = (time.perf_counter() - t1) * 1e3 / args.steps
        model_order = {"schedule": "forward of every operator, then backward in reverse order; each weight-gradient GEMM on "
                                   "a side stream beside the next operator's gradient conversion", "ms_per_step": round(ms3, 4),
                       "value": round(gemm_ops / (ms3 * 1e-3) / 1e12, 3), "unit": "TOPS"}
    dw_beside = None
    if len(ops_objs) > 1 and not args.no_extra_passes and all(hasattr(o, "gemm_bwd_part") for o in ops_objs):
        for _ in range(max(2, args.warmup)):
            step_dw_beside_next()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step_dw_beside_next()
        torch.cuda.synchronize()
        ms6 = (time.perf_counter() - t1) * 1e3 / args.steps
        dw_beside = {"schedule": "serial step; each weight-gradient GEMM on a side stream beside the data gradient and the "
                                 "next operator's conversions", "ms_per_step": round(ms6, 4),
                     "value": round(gemm_ops / (ms6 * 1e-3) / 1e12, 3), "unit": "TOPS"}
    weights_ahead = None
    if len(ops_objs) > 1 and not args.no_extra_passes and not args.w_side_stream:
        for _ in range(max(2, args.warmup)):
            step_weights_ahead()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step_weights_ahead()
        torch.cuda.synchronize()
        ms5 = (time.perf_counter() - t1) * 1e3 / args.steps
        weights_ahead = {"schedule": "serial step; the later operators' weight conversions on a side stream beside the "
                                     "first operator's forward GEMM", "ms_per_step": round(ms5, 4),
                         "value": round(gemm_ops / (ms5 * 1e-3) / 1e12, 3), "unit": "TOPS"}
    # Extra (outside the timed region): the matrix-instruction rate the GPU sustains with no memory traffic
    # (register operands), with constant and with pseudo-random operand values: context for roofline.frac.
    mfma_probe = None
    if not args.no_extra_passes:
        scratch = torch.empty(512 * 256, dtype=torch.int32, device="cuda")
        mfma_probe = {"unit": "TOPS" if tag == Q.INT8 else "TFLOP/s", "kernel": "qsync_probe_mfma (512 x 4 wavefronts, "
                      "back-to-back 32x32 matrix instructions on register operands)"}
        modes = [("constant_operands", 0), ("random_operands", 1)]
        if tag == Q.FP16:
            modes.append(("random_operands_second_subnormal", 2))
        for key, rnd_ops in modes:
            Q.qsync_probe_mfma(tag, rnd_ops, 2000, scratch, main)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
            ops = Q.qsync_probe_mfma(tag, rnd_ops, 50000, scratch, main)
            e1.record(main)
            torch.cuda.synchronize()
            mfma_probe[key] = round(ops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
        del scratch
        # the workload's forward GEMMs alone, back to back, on the codes of the last step and on constant
        # operands (every code / half = 1): the same instruction stream at the same addresses, only the
        # operand values differ
        lin_ops = [o for o in ops_objs if hasattr(o, "gemm_bwd_part")]
        if lin_ops:
            def gemm_rate():
                for o in lin_ops:
                    o.gemm_fwd(main)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(main)
                for _ in range(10):
                    for o in lin_ops:
                        o.gemm_fwd(main)
                e1.record(main)
                torch.cuda.synchronize()
                return sum(2 * o.M * o.N * o.K for o in lin_ops) * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e12
            mfma_probe["forward_gemms_back_to_back"] = round(gemm_rate(), 1)
            saved = [(o.xq, o.wq) for o in lin_ops]
            for o in lin_ops:        # xq may alias the caller's input (binary16 tag): swap in fresh buffers
                o.xq, o.wq = torch.ones_like(o.xq), torch.ones_like(o.wq)
            mfma_probe["forward_gemms_back_to_back_constant_operands"] = round(gemm_rate(), 1)
            for o, (xq_, wq_) in zip(lin_ops, saved):
                o.xq, o.wq = xq_, wq_
    # Extra (outside the timed region): the quantize kernel alone on the largest gradient tensor of the
    # workload, 20 back-to-back launches each; "cold" rotates through enough input/output sets to exceed
    # 512 MB (nothing is left in the memory-side cache), "warm" reuses one set.
    quant_iso = None
    dequant_iso = None
    if tag == Q.INT8 and args.bwd_tag is None and not args.no_extra_passes:
        big = max(range(len(cases)), key=lambda i: cases[i].dy.size)
        op, dy = ops_objs[big], dev_in[big][2]
        Mq, Nq = op.M, op.N
        one_copy = bool(getattr(op, "rowmajor_bwd", False))          # the form this run's step uses
        bytes_one, bytes_two = dy.numel() * (dy.element_size() + 1), dy.numel() * (dy.element_size() + 2)
        bytes_per = bytes_one if one_copy else bytes_two
        nset = max(2, int(math.ceil((512 << 20) / bytes_one)) + 1)
        sets = [(dy.clone(), torch.empty(Mq, Nq, dtype=torch.int8, device="cuda"), torch.empty(Nq, Mq, dtype=torch.int8, device="cuda"))
                for _ in range(nset)]
        quant_iso = {"tensor": f"dY [{Mq},{Nq}] {str(dy.dtype).replace('torch.', '')}",
                     "bytes": "read + codes" if one_copy else "read + codes + transposed codes",
                     "bytes_per_launch": int(bytes_per), "sets_rotated_cold": nset}
        other = {"bytes": "read + codes + transposed codes" if one_copy else "read + codes",
                 "bytes_per_launch": int(bytes_two if one_copy else bytes_one)}
        quant_iso["other_form"] = other
        for dest, single, nbytes in ((quant_iso, one_copy, bytes_per), (other, not one_copy, other["bytes_per_launch"])):
            for rname, rnd in (("rtn", Q.ROUND_NEAREST), ("sr", Q.ROUND_STOCHASTIC)):
                for mode in ("cold", "warm"):
                    def one(i):
                        x_, q_, qt_ = sets[i % nset] if mode == "cold" else sets[0]
                        Q.qsync_quantize(x_, Mq, Nq, Nq, Q.INT8, 8, Q.PER_TENSOR, rnd, 1, 0, op.idy, q_, None if single else qt_, main)
                    for i in range(5):
                        one(i)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(main)
                    for i in range(20):
                        one(i)
                    e1.record(main)
                    torch.cuda.synchronize()
                    us = e0.elapsed_time(e1) / 20 * 1e3
                    gbs = nbytes / (us * 1e-6) / 1e9
                    dest[f"{rname}_{mode}"] = {"us": round(us, 1), "GBps": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}
        # reference on the same machine: a plain device copy moving the same bytes (read 2 B, write 2 B per element)
        csets = [(s_[0], torch.empty_like(s_[0])) for s_ in sets]
        for mode in ("cold", "warm"):
            def onec(i):
                a_, b_ = csets[i % nset] if mode == "cold" else csets[0]
                b_.copy_(a_)
            for i in range(5):
                onec(i)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
            for i in range(20):
                onec(i)
            e1.record(main)
            torch.cuda.synchronize()
            gbs = dy.numel() * 2 * dy.element_size() / (e0.elapsed_time(e1) / 20 * 1e-3) / 1e9
            quant_iso[f"plain_copy_{mode}"] = {"GBps": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}
        del sets, csets
        # the standalone dequantizer on raw accumulators of the same shape: int32 -> fp16 with the per-column
        # scale and bias of a per-output-channel operator (read 4 B, write 2 B per element)
        dq_bytes = Mq * Nq * 6
        nset = max(2, int(math.ceil((512 << 20) / dq_bytes)) + 1)
        dsets = [(torch.randint(-2**20, 2**20, (Mq, Nq), dtype=torch.int32, device="cuda"),
                  torch.empty(Mq, Nq, dtype=torch.float16, device="cuda")) for _ in range(nset)]
        csv_, cbv_ = torch.rand(Nq, device="cuda"), torch.rand(Nq, device="cuda")
        dequant_iso = {"tensor": f"int32 accumulators [{Mq},{Nq}] -> float16, per-column scale + bias",
                       "bytes_per_launch": int(dq_bytes), "sets_rotated_cold": nset}
        for mode in ("cold", "warm"):
            def oned(i):
                a_, y_ = dsets[i % nset] if mode == "cold" else dsets[0]
                Q.qsync_dequantize(a_, Mq, Nq, Nq, None, csv_, 1e-6, cbv_, y_, main)
            for i in range(5):
                oned(i)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
            for i in range(20):
                oned(i)
            e1.record(main)
            torch.cuda.synchronize()
            gbs = dq_bytes / (e0.elapsed_time(e1) / 20 * 1e-3) / 1e9
            dequant_iso[mode] = {"GBps": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}
        del dsets

    # Extra: the forward GEMM collecting max |Y| in its epilogue, against the pass over Y that a directly chained
    # consumer would otherwise need (forward GEMM + absmax of Y  vs  forward GEMM with the maximum + two divisions).
    epilogue_max = None
    epilogue_codes = None
    if not args.no_extra_passes and tag == Q.INT8:
        lin_ops = [o for o in ops_objs if hasattr(o, "gemm_bwd_part")]
        if lin_ops:
            o = lin_ops[0]
            am = torch.zeros(1, dtype=torch.float32, device="cuda")
            s_, i_, a_ = (torch.empty(1, dtype=torch.float32, device="cuda") for _ in range(3))
            wsa = torch.zeros(max(256, Q.qsync_absmax_workspace_bytes(o.M, o.N, Q.PER_TENSOR)), dtype=torch.uint8, device="cuda")

            def separate():
                Q.qsync_qlinear_fwd(o.tag, o.M, o.N, o.K, o.xq, o.sx, o.wq, o.sw, o.w_gran, o.bias, o.y, None, o.ws_fwd, main)
                Q.qsync_absmax_scale(o.y, o.M, o.N, o.N, Q.PER_TENSOR, 8, s_, i_, a_, None, wsa, main)

            def fused():
                Q.qsync_qlinear_fwd_amax(o.tag, o.M, o.N, o.K, o.xq, o.sx, o.wq, o.sw, o.w_gran, o.bias, o.y, None, am,
                                         o.ws_fwd, main)
                Q.qsync_scale_from_amax(am, 8, s_, i_, True, main)

            res = {}
            for name, fn in (("gemm_then_absmax_us", separate), ("gemm_with_maximum_then_scale_us", fused)):
                for _ in range(3):
                    fn()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(main)
                for _ in range(20):
                    fn()
                e1.record(main)
                torch.cuda.synchronize()
                res[name] = round(e0.elapsed_time(e1) / 20 * 1e3, 1)
            epilogue_max = {"operator": "%dx%d->%d, Y %s" % (o.M, o.K, o.N, str(o.y.dtype).replace("torch.", "")), **res}
            # the consumer's codes from the producer's epilogue against the consumer's own quantize pass over Y
            # (row-major codes in both cases; scale given)
            yq = torch.empty(o.M, o.N, dtype=torch.int8, device="cuda")
            inv_ = torch.full((1,), 20.0, dtype=torch.float32, device="cuda")

            def separate_q():
                Q.qsync_qlinear_fwd(o.tag, o.M, o.N, o.K, o.xq, o.sx, o.wq, o.sw, o.w_gran, o.bias, o.y, None, o.ws_fwd, main)
                Q.qsync_quantize(o.y, o.M, o.N, o.N, Q.INT8, 8, Q.PER_TENSOR, Q.ROUND_NEAREST, 0, 0, inv_, yq, None, main)

            def fused_q():
                Q.qsync_qlinear_fwd_codes(o.tag, o.M, o.N, o.K, o.xq, o.sx, o.wq, o.sw, o.w_gran, o.bias, o.y, 8, inv_, yq, None,
                                          o.ws_fwd, main)

            res = {}
            for name, fn in (("gemm_then_quantize_us", separate_q), ("gemm_with_codes_us", fused_q)):
                for _ in range(3):
                    fn()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(main)
                for _ in range(20):
                    fn()
                e1.record(main)
                torch.cuda.synchronize()
                res[name] = round(e0.elapsed_time(e1) / 20 * 1e3, 1)
            epilogue_codes = {"operator": epilogue_max["operator"], **res}

    # Extra (outside the timed region): a fully instrumented pass for the per-phase breakdown.
    per_step = {"gemm_fwd": fwd_ms}
    if not args.no_extra_passes:
        ev2 = EventLog()
        ev, ev_timed = ev2, ev
        nb = min(args.steps, 20)          # (thousands of live events slow the recording itself down)
        for _ in range(nb):
            step("all")
        torch.cuda.synchronize()
        per_step = {k: v[0] / nb for k, v in ev2.totals().items()}        # ms per step per class
        ev = ev_timed
    # dominant kernel: the MFMA GEMM.  gemm_bwd also holds the bias-gradient column sum, so the
    # roofline figure uses the forward GEMM launches alone (one launch per operator per step).
    fwd_ops = sum(2 * c.mnk[0] * c.mnk[1] * c.mnk[2] for c in cases)
    achieved = fwd_ops / (fwd_ms * 1e-3) / 1e12
    peak = PEAK[args.tag]
    if mfma_probe is not None:
        mfma_probe["forward_gemm_frac_of_random_operand_rate"] = round(achieved / mfma_probe["random_operands"], 4)
    # HBM-bound side: absmax + quantize of dY (read twice, write the codes, and their transpose when that is kept)
    esz = cases[0].dy.dtype.itemsize
    # (the convolution operator keeps its codes in NHWC only; its weight gradient gathers them)
    ncopies = [1 if (getattr(o, "rowmajor_bwd", False) or not hasattr(o, "rowmajor_bwd")) else 2 for o in ops_objs]
    dy_bytes = sum(c.dy.size * (2 * esz + n) for c, n in zip(cases, ncopies))
    quant_gbs = dy_bytes / (per_step["convert_dy"] * 1e-3) / 1e9 if "convert_dy" in per_step else None

    out = {
        "metric": "qlinear fwd+bwd TOPS (whole step incl. absmax/quantize/dequantize)",
        "value": round(value, 3), "unit": "TOPS" if args.tag == "int8" else "TFLOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.tag if args.tag == "int8" else "f16", "data": "synthetic",
        "config": {"workload": desc, "tag": args.tag, "y_dtype": args.ydtype, "dx_dtype": "f16", "dw_dtype": "f32",
                   "w_scale": "per-output-channel",
                   "dy_rounding": "stochastic (Philox4x32-10)" if args.bwd_tag is None else "none (FP16 backward)",
                   "bwd_tag": args.bwd_tag or args.tag,
                   "operator_streams": nstreams,
                   "activation_and_gradient_codes": "row-major only" if min(ncopies) == 1 else "row-major + transposed copy",
                   **({"conv_input": args.conv_input if (tag == Q.INT8 or args.conv_input == "implicit") else "patches"}
                      if any(c.nhwc is not None for c in cases) else {})},
        "roofline": {"bound": "mfma", "kernel": "gemm_nt_kernel (forward GEMM launches; HIP events on every 4th timed step)",
                     "achieved": round(achieved, 2), "peak": peak, "unit": "TOP/s" if args.tag == "int8" else "TFLOP/s",
                     "frac": round(achieved / peak, 4),
                     "traffic": measured_traffic(args.workload, args.tag, args.ydtype),
                     "algorithmic_bytes": int(sum((c.mnk[0] + c.mnk[1]) * c.mnk[2] * (1 if args.tag == "int8" else 2)
                                                  + c.mnk[0] * c.mnk[1] * (2 if args.ydtype == "f16" else 4)
                                                  for c in cases) / len(cases))},
        "breakdown_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "breakdown_note": "separate pass after the timed region with events around every phase (the events "
                          "themselves lengthen that pass); convert_x includes the weight conversion",
        "quantize_dy": None if quant_gbs is None else
                       {"GBps": round(quant_gbs, 1), "frac_hbm": round(quant_gbs / HBM_PEAK_GBS, 4),
                        "bytes": "absmax read + quantize read + codes" + ("" if min(ncopies) == 1 else " + transposed codes")},
        "quantize_alone": quant_iso,
        "dequantize_alone": dequant_iso,
        "mfma_probe": mfma_probe,
        "operators_on_separate_streams": overlapped,
        "hip_graph_replay": graph_replay,
        "model_order_dw_on_side_stream": model_order,
        "weights_converted_ahead_on_side_stream": weights_ahead,
        "dw_on_side_stream_beside_next_operator": dw_beside,
        "epilogue_maximum": epilogue_max,
        "epilogue_codes": epilogue_codes,
    }
    if quant_iso is not None:
        # the HBM-bound kernels against the published 8 TB/s, cold (inputs and outputs rotated through > 512 MB)
        out["roofline_quantize"] = {"bound": "hbm", "kernel": "quantize kernel, stochastic rounding, " + quant_iso["tensor"]
                                    + ", " + quant_iso["bytes"] + ", cold",
                                    "achieved": quant_iso["sr_cold"]["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": quant_iso["sr_cold"]["frac_hbm"], "algorithmic_bytes": quant_iso["bytes_per_launch"]}
        out["roofline_quantize_nearest"] = {"bound": "hbm", "kernel": "quantize kernel, round to nearest, " + quant_iso["tensor"]
                                            + ", " + quant_iso["bytes"] + ", cold",
                                            "achieved": quant_iso["rtn_cold"]["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                            "frac": quant_iso["rtn_cold"]["frac_hbm"],
                                            "algorithmic_bytes": quant_iso["bytes_per_launch"]}
    if dequant_iso is not None:
        out["roofline_dequantize"] = {"bound": "hbm", "kernel": "dequantize_cols_kernel, " + dequant_iso["tensor"] + ", cold",
                                      "achieved": dequant_iso["cold"]["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": dequant_iso["cold"]["frac_hbm"], "algorithmic_bytes": dequant_iso["bytes_per_launch"]}
    if "gemm_bwd" in per_step:
        out["gemm_only_TOPS"] = round(gemm_ops / ((per_step["gemm_fwd"] + per_step["gemm_bwd"]) * 1e-3) / 1e12, 2)
    if not args.no_cpu:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(cases, tag, args.cpu_tokens)
    return out


def main():
    args = parse_args()
    out = run(args)
    # The metric names INT8 and FP16: the default run times the same workload a second time under the FP16 tag
    # (its own warm-up and K steps, its own HIP events around the forward GEMMs) and reports it beside the INT8 line.
    if args.tag == "int8" and args.workload == "c5" and args.bwd_tag is None and not args.no_fp16_pass:
        import copy
        a16 = copy.copy(args)
        a16.tag, a16.no_cpu, a16.no_extra_passes = "fp16", True, True
        o16 = run(a16)
        out["fp16_tag"] = {k: o16[k] for k in ("metric", "value", "unit", "ms_per_step", "steps", "warmup", "dtype",
                                               "config", "roofline")}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
