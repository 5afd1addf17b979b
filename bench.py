#!/usr/bin/env python3
"""Benchmark of the MBConv training step (forward + backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--policy recompute|store]
                    [--mode train|eval]

A step is one forward plus one backward through the C ABI on seeded synthetic inputs that are
already resident in HBM.  The default workload is benchmark config 4, the largest one: the 16
MBConv blocks of EfficientNet-B0 chained at batch 64 (block i's output is block i+1's input,
backward in reverse order, one scratch workspace shared by all blocks); its first block is the
layer the paper measured.  Prints ONE JSON line:
  value         images/s over the whole job
  roofline      the slowest kernel of the step, timed live with HIP events recorded on the launch
                stream inside the timed region (less the measured gap of an empty event pair),
                against the HBM roofline (algorithmic bytes); `traffic` is the HBM byte count
                rocprofv3 measured for that launch, read from profiles/hbm_traffic_per_step.md
  roofline_next the next slowest steps, from the untimed survey
  step_roofline algorithmic bytes of the whole step / ms_per_step against the HBM peak
  gemm          the 1x1 convolutions of the blocks whose GEMMs lie above the fp32 ridge
                (chain blocks 7-16): flops and time, and per matrix-core instruction family
                (fp32 MFMA; bf16 MFMA on three-plane splits of the fp32 operands, six issued
                flops per flop of the contraction) the issued rate against that family's peak
  other_configs the single-block configs 1-3 (images/s, slowest kernel, roofline fraction)
  cpu_baseline  the fp64 CPU oracle timed on this host (a reported baseline, not a target)
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_F32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix rate, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix rate, published
F32_RIDGE = MFMA_F32_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)  # flop per byte

# HBM bytes per launch as rocprofv3 --pmc measured them (FETCH_SIZE, WRITE_SIZE, scaled by the
# same counters' reading on a plain copy of known size): one Markdown table row per
# (workload, step), written from the profiler's output; bench.py only reads it.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_step.md")

NO_EXPAND_STEPS = ("expand_conv", "bn1_finalize", "bn1_bwd_finalize", "expand_dgrad", "expand_wgrad")
GEMM_STEPS = ("expand_conv", "proj_conv", "proj_dgrad", "proj_wgrad", "expand_dgrad", "expand_wgrad")


def measured_traffic(workload: str, step: str):
    """Bytes (fetch + write) the profiler counted for one launch of `step`, or None."""
    try:
        with open(TRAFFIC_TABLE) as fh:
            for line in fh:
                cells = [c.strip() for c in line.split("|")]
                if len(cells) >= 8 and cells[1] == workload and cells[2] == step:
                    return int(round((float(cells[5]) + float(cells[6])) * 2 ** 20))
    except (OSError, ValueError):
        pass
    return None


def _fused(s):
    """Shapes for which one kernel computes both gradients of a 1x1 conv (narrow side <= 32
    channels, wide side <= 256, plane a multiple of four): the step named *_dgrad is that kernel."""
    fused_proj = s.Cout <= 32 and s.Cout < s.Cexp <= 256 and (s.Ho * s.Wo) % 4 == 0
    fused_exp = s.has_expand and s.Cin <= 32 and s.Cin < s.Cexp <= 256 and (s.H * s.W) % 4 == 0
    return fused_proj, fused_exp


def step_bytes(s) -> dict:
    """Bytes each step must move by the fusion plan (each tensor it consumes or produces
    crosses HBM once), for the steps with an activation-sized operand."""
    b = 2 if s.dtype == "bf16" else 4
    X = s.N * s.Cin * s.H * s.W
    E = s.N * s.Cexp * s.H * s.W
    D = s.N * s.Cexp * s.Ho * s.Wo
    P = s.N * s.Cout * s.Ho * s.Wo
    res = P if s.residual else 0
    fused_proj, fused_exp = _fused(s)
    table = {
        "expand_conv": X + E, "dw_fwd": E + D, "se_pool": D, "proj_conv": D + P,
        "bn3_apply": 2 * P + res, "bn3_bwd_reduce": 2 * P,
        "proj_dgrad": 2 * P + 2 * D if fused_proj else 2 * P + D,
        "proj_wgrad": 2 * P + D, "gate_sums": 2 * D,
        "dw_bwd": (2 * D + 2 * E) if s.has_expand else (2 * D + 2 * X + res),
        "expand_dgrad": 2 * E + 2 * X + res if fused_exp else 2 * E + X + res,
        "expand_wgrad": 2 * E + X,
    }
    if fused_proj:
        del table["proj_wgrad"]  # what is left of the step is the sum over the splits
    if fused_exp:
        del table["expand_wgrad"]
    if not s.has_expand:
        for n in ("expand_conv", "expand_dgrad", "expand_wgrad"):
            table.pop(n, None)
    if not getattr(s, "has_se", True):
        table.pop("se_pool", None)
    return {n: v * b for n, v in table.items()}


def algorithmic_bytes(s, step: str):
    return step_bytes(s).get(step)


def step_flops(s) -> dict:
    """Multiply-add flops of the 1x1-convolution steps (2 per multiply-add)."""
    fe = 2 * s.N * s.H * s.W * s.Cin * s.Cexp
    fp = 2 * s.N * s.Ho * s.Wo * s.Cexp * s.Cout
    fused_proj, fused_exp = _fused(s)
    t = {"proj_conv": fp, "proj_dgrad": 2 * fp if fused_proj else fp}
    if not fused_proj:
        t["proj_wgrad"] = fp
    if s.has_expand:
        t.update({"expand_conv": fe, "expand_dgrad": 2 * fe if fused_exp else fe})
        if not fused_exp:
            t["expand_wgrad"] = fe
    return t


def gemm_is_mfma_bound(s) -> bool:
    """True when the block's 1x1 convolutions lie above the fp32 ridge (flops per byte of a
    1x1 conv: 2*Ci*Co per pixel over (Ci+Co)*4 bytes)."""
    if s.dtype != "f32" or not s.has_expand:
        return False
    return 2.0 * s.Cin * s.Cexp / ((s.Cin + s.Cexp) * 4.0) > F32_RIDGE


class HipEvents:
    """HIP events through the runtime's C API (torch.cuda.Event only sees torch's stream)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]

    def create(self) -> C.c_void_p:
        ev = C.c_void_p()
        rc = self.hip.hipEventCreate(C.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed ({rc})")
        return ev

    def elapsed_ms(self, a, b) -> float:
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)

    def record(self, ev, stream):
        rc = self.hip.hipEventRecord(ev, C.c_void_p(stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed ({rc})")

    def pair_overhead_ms(self, stream, work, reps=20) -> float:
        """Time between two events recorded back to back behind queued work: the part of an
        event-bracketed kernel time that is not the kernel (median of `reps`)."""
        import torch
        a, b = self.create(), self.create()
        vals = []
        for _ in range(reps):
            work()
            self.record(a, stream)
            self.record(b, stream)
            torch.cuda.synchronize()
            vals.append(self.elapsed_ms(a, b))
        self.destroy(a)
        self.destroy(b)
        return sorted(vals)[len(vals) // 2]


def cpu_baseline(shape, tensors, eval_mode=False):
    """The oracle, as it stands, on this host: passes over the same workload, at least one and
    then as many as fit into about ten seconds (five at most); the median pass is reported."""
    from oracle import oracle as orc
    times, begin = [], time.perf_counter()
    while len(times) < 5 and (not times or time.perf_counter() - begin + times[-1] < 10.0):
        t0 = time.perf_counter()
        if eval_mode:
            orc.mbconv_forward_eval(shape, tensors)
        else:
            orc.mbconv_step(shape, tensors)
        times.append(time.perf_counter() - t0)
    dt = sorted(times)[len(times) // 2]
    what = "evaluation-mode forward" if eval_mode else "forward+backward"
    return {"value": shape.N / dt, "unit": "images/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"fp64 {what} of the full workload batch ({shape.N} images), median of "
                      f"{len(times)} passes, {dt:.2f} s wall each"}


def cpu_baseline_chain(batch: int):
    """One fp64 oracle pass (forward through the 16 blocks, then backward) over the chain at
    `batch` images, same seeds as the GPU run; every tape is freed as soon as its block's
    backward has run."""
    import numpy as np
    from mbconv_inputs import b0_chain, make_block_inputs
    from oracle import oracle as orc
    shapes = b0_chain(N=batch)
    t0 = time.perf_counter()
    recs, x = [], None
    for i, s in enumerate(shapes):
        t = make_block_inputs(s, seed=i, with_x=(i == 0), with_dout=(i == len(shapes) - 1))
        if i > 0:
            t["x"] = x
        f = orc.mbconv_forward(s, t)
        x = f.out
        recs.append((s, t, f.tape))
    dout = np.asarray(recs[-1][1]["dout"], dtype=np.float64)
    while recs:
        s, t, tape = recs.pop()
        dout = orc.mbconv_backward(s, t, tape, dout).dx
        del tape, t
    dt = time.perf_counter() - t0
    return {"value": batch / dt, "unit": "images/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"one fp64 forward+backward pass over the 16-block chain at batch {batch} "
                      f"(seeded input generation included), {dt:.1f} s wall"}


def cpu_baseline_one_thread(shape, eval_mode=False):
    """The oracle on ONE thread, in a child process (OMP_NUM_THREADS=1), on a quarter of the batch."""
    import subprocess
    n = max(shape.N // 4, 1)
    code = (
        "import sys, time; sys.path.insert(0, %r)\n"
        "from dataclasses import replace\n"
        "from mbconv_inputs import CONFIGS, make_block_inputs\n"
        "from oracle import oracle as orc\n"
        "s = replace(CONFIGS[%d], N=%d); t = make_block_inputs(s, 0)\n"
        "t0 = time.perf_counter()\n"
        "%s\n"
        "print(time.perf_counter() - t0, orc.num_threads())\n"
    ) % (ROOT, next(k for k, v in __import__("mbconv_inputs").CONFIGS.items() if v == shape), n,
         "orc.mbconv_forward_eval(s, t)" if eval_mode else "orc.mbconv_step(s, t)")
    env = dict(os.environ, OMP_NUM_THREADS="1")
    out = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, check=True)
    dt, threads = out.stdout.split()
    return {"value": n / float(dt), "unit": "images/s", "cores": int(threads),
            "sample": f"{n} images, {float(dt):.1f} s wall"}


def _roofline_entry(kernel, nbytes, ms):
    ach = nbytes / (ms * 1e-3) / 1e9
    return {"kernel": kernel, "kernel_ms": round(ms, 5), "achieved": round(ach, 1),
            "frac": round(ach / HBM_PEAK_GBS, 4), "algorithmic_bytes": nbytes}


def run_chain(args) -> dict:
    """Benchmark config 4: the 16 MBConv blocks of EfficientNet-B0 chained (block i's output is
    block i+1's input; backward in reverse order), one scratch workspace shared by all blocks."""
    import torch
    from mbconv_inputs import b0_chain, make_block_inputs
    from paper_2110_10802_amd import binding as B
    from paper_2110_10802_amd.harness import DeviceBlock

    B.load()
    shapes = b0_chain()
    policy = B.MBCONV_STORE if args.policy == "store" else B.MBCONV_RECOMPUTE
    scratch_bytes = max(B.mbconv_workspace_size(B.make_desc(s, policy))[1] for s in shapes)
    scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device="cuda")
    blocks, ctx = [], []
    for i, s in enumerate(shapes):
        t = make_block_inputs(s, seed=i, with_x=(i == 0), with_dout=(i == len(shapes) - 1))
        blk = DeviceBlock(s, t, policy=policy, scratch=scratch)
        if i == 0:
            x0 = blk.to_device(t["x"])
        if i == len(shapes) - 1:
            dlast = blk.to_device(t["dout"])
        blocks.append(blk)
    stream = torch.cuda.current_stream().cuda_stream
    for i, blk in enumerate(blocks):
        ctx.append({
            "blk": blk, "desc": blk.desc, "params": B._fill(B.Params(), blk.params),
            "running": B._fill(B.BNState(), blk.running) if blk.running else None,
            "grads": B._fill(B.Grads(), blk.grads),
            "x": x0 if i == 0 else blocks[i - 1].out,
            "dout": dlast if i == len(blocks) - 1 else blocks[i + 1].dx,
        })
    only = args.only_block - 1 if args.only_block else None

    def step(probe=None, probe_block=-1):
        for i, c in enumerate(ctx):
            if only is not None and i != only:
                continue
            pr = probe if (i == probe_block and probe.step <= 9) else None
            B.mbconv_forward_probed(c["desc"], c["params"], c["running"], c["x"], c["blk"].out,
                                    c["blk"].saved, scratch, stream, pr)
        for i in range(len(ctx) - 1, -1, -1):
            if only is not None and i != only:
                continue
            c = ctx[i]
            pr = probe if (i == probe_block and probe.step > 9) else None
            B.mbconv_backward_probed(c["desc"], c["params"], c["x"], c["dout"], c["blk"].saved,
                                     scratch, c["blk"].dx, c["grads"], stream, pr)

    if only is not None:
        # one block of the chain alone, at its real shape and on its real input (for profiling):
        # the blocks before it run once to produce that input, the block after it is given a
        # random upstream gradient
        for i, c in enumerate(ctx[:only]):
            B.mbconv_forward_probed(c["desc"], c["params"], c["running"], c["x"], c["blk"].out,
                                    c["blk"].saved, scratch, stream, None)
        if only < len(ctx) - 1:
            ctx[only]["dout"].normal_()
    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    ev = HipEvents()
    overhead_ms = ev.pair_overhead_ms(stream, step, reps=5)
    e0, e1 = ev.create(), ev.create()
    survey = []
    for i, c in enumerate(ctx):
        if args.no_survey:
            break
        row = {}
        if only is not None and i != only:
            survey.append(row)
            continue
        prev_reps = None
        for name, sid in B.STEPS.items():
            if not shapes[i].has_expand and name in NO_EXPAND_STEPS:
                continue
            reps = []
            for _ in range(3):
                step(B.Probe(sid, e0, e1), i)
                torch.cuda.synchronize()
                reps.append(ev.elapsed_ms(e0, e1))
            if prev_reps is not None and all(r == prev_reps[-1] for r in reps):
                continue  # the step did not occur (its events still hold the previous step's last times)
            prev_reps = reps
            row[name] = sorted(reps)[1]
        survey.append(row)
        s = shapes[i]
        print(f"block {i + 1:2d} {s.Cin}->{s.Cexp}->{s.Cout} {s.H}x{s.W} k{s.k}s{s.stride}: "
              f"{sum(row.values()) * 1e3:7.1f}us  " +
              " ".join(f"{n}={v * 1e3:.0f}" for n, v in row.items()), file=sys.stderr)
    ev.destroy(e0)
    ev.destroy(e1)
    def chain_bytes(i, n):
        # (where a block's two weight gradients share one launch, the survey has no proj_wgrad
        # step and the expand_wgrad step moves the bytes of both)
        b = algorithmic_bytes(shapes[i], n)
        if b is not None and n == "expand_wgrad" and survey and survey[i] and "proj_wgrad" not in survey[i]:
            b += step_bytes(shapes[i]).get("proj_wgrad", 0)
        return b

    cand = [(i, n) for i, row in enumerate(survey) for n in row if chain_bytes(i, n) is not None]
    if args.probe_step or args.no_survey:
        default_probe = f"{only + 1}:dw_bwd" if only is not None else "2:dw_bwd"
        bi, dominant = (args.probe_step or default_probe).split(":")
        bi = int(bi) - 1
    else:
        bi, dominant = max(cand, key=lambda c: survey[c[0]][c[1]])
    # the dominant kernel is timed inside the timed region on every fourth step (an event pair
    # stretches its step by the gap between two event records)
    pairs = [(ev.create(), ev.create()) for _ in range((args.steps + 3) // 4)]
    probes = [B.Probe(B.STEPS[dominant], a, b) for a, b in pairs]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % 4 == 0:
            step(probes[i // 4], bi)
        else:
            step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kern_ms_raw = sum(ev.elapsed_ms(a, b) for a, b in pairs) / len(pairs)
    for a, b in pairs:
        ev.destroy(a)
        ev.destroy(b)
    kern_ms = max(kern_ms_raw - overhead_ms, 1e-6)
    nbytes = chain_bytes(bi, dominant)
    achieved = nbytes / (kern_ms * 1e-3) / 1e9
    N = shapes[0].N
    active = [s for i, s in enumerate(shapes) if only is None or i == only]
    total_bytes = sum(sum(step_bytes(s).values()) for s in active)
    workload = "config4" if only is None else f"config4-block{only + 1}"
    result = {
        "metric": "mbconv_fwd_bwd_images_per_sec", "value": N / (ms_per_step * 1e-3),
        "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload, "block": f"N{N} EfficientNet-B0 chain of 16 MBConv blocks, "
                   "32ch 112x112 in" + ("" if only is None else f"; block {only + 1} alone"),
                   "policy": args.policy},
        "roofline": {"bound": "hbm", "kernel": f"block{bi + 1}:{dominant}", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic("config4", f"block{bi + 1}:{dominant}"),
                     "kernel_ms": kern_ms, "kernel_ms_with_event_gap": kern_ms_raw,
                     "event_gap_ms": overhead_ms, "algorithmic_bytes": nbytes},
        # bytes of every step of every block by the fusion plan over the measured step time: how
        # far the whole step is from streaming its tensors once at the HBM peak
        "step_roofline": {"bound": "hbm", "algorithmic_bytes": total_bytes,
                          "achieved": round(total_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                          "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": round(total_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
    }
    if survey:
        net = lambda i, n: max(survey[i][n] - overhead_ms, 1e-6)
        nxt = sorted((c for c in cand if c != (bi, dominant)), key=lambda c: -survey[c[0]][c[1]])[:3]
        result["roofline_next"] = [_roofline_entry(f"block{i + 1}:{n}", chain_bytes(i, n),
                                                   net(i, n)) for i, n in nxt]
        # 1x1 convolutions above the fp32 ridge: the matrix-core roofline applies to these.  The
        # library says which instruction family serves each launch: the fp32 MFMA, or the bf16
        # MFMA on three-plane splits of the fp32 operands, which issues six times the flops of
        # the contraction on the bf16 matrix cores; each family is priced against its own peak.
        rows = []
        for i, s in enumerate(shapes):
            if not gemm_is_mfma_bound(s) or not survey[i]:
                continue
            fl = step_flops(s)
            for n in GEMM_STEPS:
                if n in fl and n in survey[i]:
                    eng = B.ENGINES[B.mbconv_step_engine(ctx[i]["desc"], B.STEPS[n])]
                    f = fl[n]
                    if n == "expand_wgrad" and "proj_wgrad" in fl and "proj_wgrad" not in survey[i]:
                        f += fl["proj_wgrad"]  # the two weight gradients share this launch
                    rows.append((i, n, f, net(i, n), eng))
        if rows:
            issue = {"mfma_f32": (1, MFMA_F32_PEAK_TFLOPS), "mfma_bf16x3": (6, MFMA_BF16_PEAK_TFLOPS),
                     "mfma_bf16": (1, MFMA_BF16_PEAK_TFLOPS)}
            tot_f, tot_ms = sum(r[2] for r in rows), sum(r[3] for r in rows)
            tf = lambda f, ms: f / (ms * 1e-3) / 1e12
            slow = max(rows, key=lambda r: r[3])
            worst = min(rows, key=lambda r: r[2] / r[3])
            best = max(rows, key=lambda r: r[2] / r[3])
            ent = lambda r: {"kernel": f"block{r[0] + 1}:{r[1]}", "engine": r[4], "flops": r[2],
                             "kernel_ms": round(r[3], 5), "achieved": round(tf(r[2], r[3]), 1),
                             "frac": round(tf(r[2], r[3]) * issue[r[4]][0] / issue[r[4]][1], 4)}
            engines = {}
            for e in sorted({r[4] for r in rows}):
                sel = [r for r in rows if r[4] == e]
                f, ms = sum(r[2] for r in sel), sum(r[3] for r in sel)
                engines[e] = {"launches": len(sel), "flops": f, "issued_flops": f * issue[e][0],
                              "ms": round(ms, 5), "achieved": round(tf(f, ms), 1),
                              "issued": round(tf(f, ms) * issue[e][0], 1), "peak": issue[e][1],
                              "frac": round(tf(f, ms) * issue[e][0] / issue[e][1], 4)}
            result["gemm"] = {"bound": "mfma", "unit": "TFLOP/s",
                              "blocks": sorted({r[0] + 1 for r in rows}), "launches": len(rows),
                              "flops": tot_f, "ms": round(tot_ms, 5),
                              "achieved": round(tf(tot_f, tot_ms), 1),
                              # context: the contraction's own flops against the fp32 MFMA peak,
                              # the ceiling of a kernel that multiplies in fp32
                              "vs_f32_mfma_peak": round(tf(tot_f, tot_ms) / MFMA_F32_PEAK_TFLOPS, 4),
                              "engines": engines,
                              "slowest": ent(slow), "lowest_frac": ent(worst), "highest_frac": ent(best)}
        result["block_ms_survey"] = [round(sum(max(v - overhead_ms, 0.0) for v in r.values()), 5)
                                     for r in survey]
        result["launch_steps"] = sum(len(r) for r in survey)
    del blocks, ctx, scratch
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline and only is None:
        result["cpu_baseline"] = cpu_baseline_chain(N)
    return result


# Workloads of the operator benchmarks (--op).  The paper gives no tensor sizes for these in its
# text; the shapes are those of the networks it takes them from: a YOLOv4 backbone activation
# for Mish, BERT-large's hidden states for layer normalisation, its attention scores for softmax.
OP_WORKLOADS = {
    "mish": {"n": 8 * 64 * 304 * 304, "what": "8x64x304x304 activation"},
    "layernorm": {"rows": 8 * 512, "cols": 1024, "what": "4096 rows x 1024 (batch 8, sequence 512, hidden 1024)"},
    "softmax": {"rows": 8 * 16 * 512, "cols": 512, "what": "65536 rows x 512 (batch 8, 16 heads, 512x512 scores)"},
}


def run_op(args) -> dict:
    """One step = forward + backward of the operator on resident fp32 tensors."""
    import numpy as np
    import torch
    from paper_2110_10802_amd import dnnops as D

    D.load()
    w = OP_WORKLOADS[args.op]
    rng = np.random.default_rng(0)
    stream = torch.cuda.current_stream().cuda_stream
    dev = "cuda:0"
    if args.op == "mish":
        n = w["n"]
        x = torch.from_numpy((rng.standard_normal(n) * 2).astype(np.float32)).to(dev)
        dy = torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(dev)
        y, dx = torch.empty_like(x), torch.empty_like(x)
        fwd = lambda: D.mish_forward(x, y, n, stream)
        bwd = lambda: D.mish_backward(x, dy, dx, n, stream)
        elems, fbytes, bbytes = n, 8 * n, 12 * n
    else:
        rows, cols = w["rows"], w["cols"]
        x = torch.from_numpy((rng.standard_normal((rows, cols)) * 2).astype(np.float32)).to(dev)
        dy = torch.from_numpy(rng.standard_normal((rows, cols)).astype(np.float32)).to(dev)
        y, dx = torch.empty_like(x), torch.empty_like(x)
        elems = rows * cols
        if args.op == "layernorm":
            g = torch.from_numpy((1 + 0.1 * rng.standard_normal(cols)).astype(np.float32)).to(dev)
            b = torch.from_numpy((0.1 * rng.standard_normal(cols)).astype(np.float32)).to(dev)
            mean, rstd = torch.empty(rows, device=dev), torch.empty(rows, device=dev)
            dg, db = torch.empty_like(g), torch.empty_like(g)
            scratch = torch.empty(D.layernorm_backward_scratch_bytes(rows, cols), dtype=torch.uint8,
                                  device=dev)
            fwd = lambda: D.layernorm_forward(x, g, b, 1e-5, rows, cols, y, mean, rstd, stream)
            bwd = lambda: D.layernorm_backward(x, dy, g, mean, rstd, rows, cols, dx, dg, db, scratch,
                                               stream)
        else:
            fwd = lambda: D.softmax_forward(x, y, rows, cols, stream)
            bwd = lambda: D.softmax_backward(y, dy, dx, rows, cols, stream)
        fbytes, bbytes = 8 * elems, 12 * elems
    for _ in range(max(args.warmup, 1)):
        fwd()
        bwd()
    torch.cuda.synchronize()
    ev = HipEvents()
    pairs = [(ev.create(), ev.create(), ev.create()) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, m, b_ in pairs:
        ev.record(a, stream)
        fwd()
        ev.record(m, stream)
        bwd()
        ev.record(b_, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    f_ms = sorted(ev.elapsed_ms(a, m) for a, m, _ in pairs)[len(pairs) // 2]
    b_ms = sorted(ev.elapsed_ms(m, b_) for _, m, b_ in pairs)[len(pairs) // 2]
    # the slower direction is the roofline kernel (one launch per direction; the layer-norm
    # backward adds two small second-stage launches, counted in its time)
    kname, kms, kbytes = ("backward", b_ms, bbytes) if b_ms >= f_ms else ("forward", f_ms, fbytes)
    achieved = kbytes / (kms * 1e-3) / 1e9
    result = {
        "metric": f"{args.op}_fwd_bwd_gelements_per_sec", "value": elems / (ms_per_step * 1e-3) / 1e9,
        "unit": "Gelements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.op}: {w['what']}"},
        "roofline": {"bound": "hbm", "kernel": f"{args.op}_{kname}", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "kernel_ms": kms, "algorithmic_bytes": kbytes,
                     "forward_ms": f_ms, "backward_ms": b_ms,
                     "forward_gbs": fbytes / (f_ms * 1e-3) / 1e9,
                     "backward_gbs": bbytes / (b_ms * 1e-3) / 1e9},
    }
    if not args.no_cpu_baseline:
        from oracle import dnnops as orc
        xs = x.detach().cpu().numpy().astype(np.float64)
        dys = dy.detach().cpu().numpy().astype(np.float64)
        if args.op == "mish":
            xs, dys = xs[:1 << 24], dys[:1 << 24]  # a bounded sample: 16 Mi elements
        c0 = time.perf_counter()
        if args.op == "mish":
            orc.mish_fwd(xs)
            orc.mish_bwd(xs, dys)
        elif args.op == "layernorm":
            gam = g.cpu().numpy().astype(np.float64)
            _, mo, ro = orc.layernorm_fwd(xs, gam, b.cpu().numpy().astype(np.float64), 1e-5)
            orc.layernorm_bwd(xs, dys, gam, mo, ro)
        else:
            orc.softmax_bwd(orc.softmax_fwd(xs), dys)
        dt = time.perf_counter() - c0
        result["cpu_baseline"] = {"value": xs.size / dt / 1e9, "unit": "Gelements/s",
                                  "cores": os.cpu_count(), "kind": "oracle",
                                  "sample": f"one fp64 forward+backward over {xs.size} elements, {dt:.1f} s wall"}
    return result


def run_block(args, config: int, steps: int, warmup: int, with_cpu: bool, distribution: bool = True) -> dict:
    """One of the single-block workloads (configs 0-3 and the MobileNet-V2 block)."""
    import torch
    from mbconv_inputs import CONFIGS, make_block_inputs
    from paper_2110_10802_amd import binding as B
    from paper_2110_10802_amd.harness import DeviceBlock

    B.load()  # fails loudly if the HIP library has not been built
    shape = CONFIGS[config]
    tensors = make_block_inputs(shape, seed=0)
    policy = B.MBCONV_STORE if args.policy == "store" else B.MBCONV_RECOMPUTE
    blk = DeviceBlock(shape, tensors, policy=policy)
    x = blk.to_device(tensors["x"])
    dout = blk.to_device(tensors["dout"])
    stream = torch.cuda.current_stream().cuda_stream
    params = B._fill(B.Params(), blk.params)
    running = B._fill(B.BNState(), blk.running)
    grads = B._fill(B.Grads(), blk.grads)
    desc = blk.desc

    evalm = args.mode == "eval"
    if evalm:
        eval_ws = torch.empty(B.mbconv_eval_workspace_size(desc), dtype=torch.uint8, device="cuda")

    def step(probe=None):
        if evalm:
            B.mbconv_forward_eval_probed(desc, params, running, x, blk.out, eval_ws, stream, probe)
            return
        fprobe = probe if probe is not None and probe.step <= 9 else None
        bprobe = probe if probe is not None and probe.step > 9 else None
        B.mbconv_forward_probed(desc, params, running, x, blk.out, blk.saved, blk.scratch, stream,
                                fprobe)
        B.mbconv_backward_probed(desc, params, x, dout, blk.saved, blk.scratch, blk.dx, grads,
                                 stream, bprobe)

    for _ in range(max(warmup, 1)):
        step()
    torch.cuda.synchronize()

    ev = HipEvents()
    # untimed survey: duration of every step, to find the slowest kernel
    survey = {}
    e0, e1 = ev.create(), ev.create()
    prev_reps = None
    for name, sid in B.STEPS.items():
        if not shape.has_expand and name in NO_EXPAND_STEPS:
            continue
        if not getattr(shape, "has_se", True) and name == "se_pool":
            continue
        if evalm and (sid > 9 or name in ("bn2_finalize", "bn3_finalize")
                      or (name == "bn1_finalize" and not shape.has_expand)):
            continue  # backward steps, and finalise steps that do not occur in evaluation mode
        reps = []
        for _ in range(3):
            step(B.Probe(sid, e0, e1))
            torch.cuda.synchronize()
            reps.append(ev.elapsed_ms(e0, e1))
        if prev_reps is not None and all(r == prev_reps[-1] for r in reps):
            continue  # the step did not occur (its events still hold the previous step's last times)
        prev_reps = reps
        survey[name] = sorted(reps)[1]
    ev.destroy(e0)
    ev.destroy(e1)
    dominant = args.probe_step or max(
        (n for n in survey if algorithmic_bytes(shape, n) is not None), key=lambda n: survey[n])
    print(f"config {config} per-step ms (untimed survey): " +
          ", ".join(f"{n}={v * 1e3:.1f}us" for n, v in survey.items()), file=sys.stderr)

    # the dominant kernel is timed inside the timed region on every fourth step (an event pair
    # stretches the step by the gap between two event records, about 2 % of this one)
    pairs = [(ev.create(), ev.create()) for _ in range((steps + 3) // 4)]
    sid = B.STEPS[dominant]
    probes = [B.Probe(sid, a, b) for a, b in pairs]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(probes[i // 4] if i % 4 == 0 else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    kern_ms_raw = sum(ev.elapsed_ms(a, b) for a, b in pairs) / len(pairs)
    for a, b in pairs:
        ev.destroy(a)
        ev.destroy(b)
    step_stats = None
    if distribution:
        # distribution of the step time: a second, separate pass with one event between
        # consecutive steps (kept out of the timed loop, whose wall clock it would stretch); median
        # and a 95 % non-parametric confidence interval of the median from the order statistics
        marks = [ev.create() for _ in range(steps + 1)]
        ev.record(marks[0], stream)
        for i in range(steps):
            step()
            ev.record(marks[i + 1], stream)
        torch.cuda.synchronize()
        per_step = sorted(ev.elapsed_ms(marks[i], marks[i + 1]) for i in range(steps))
        for m in marks:
            ev.destroy(m)
        k = len(per_step)
        half = 0.98 * (k ** 0.5)  # 1.96 * sqrt(k) / 2
        lo_i, hi_i = max(int(k / 2 - half), 0), min(int(k / 2 + half) + 1, k - 1)
        step_stats = {"median": per_step[k // 2], "ci95": [per_step[lo_i], per_step[hi_i]],
                      "min": per_step[0], "max": per_step[-1]}
    # an event pair around a kernel also spans the gap between two event records; that gap is
    # measured with an empty pair behind the same queued work and taken off
    overhead_ms = ev.pair_overhead_ms(stream, step)
    kern_ms = max(kern_ms_raw - overhead_ms, 1e-6)

    if args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    nbytes = algorithmic_bytes(shape, dominant)
    achieved = nbytes / (kern_ms * 1e-3) / 1e9
    workload = f"config{config}"
    total_bytes = sum(v for n, v in step_bytes(shape).items() if not evalm or B.STEPS[n] <= 9)
    net = lambda n: max(survey[n] - overhead_ms, 1e-6)
    result = {
        "metric": "mbconv_eval_fwd_images_per_sec" if evalm else "mbconv_fwd_bwd_images_per_sec",
        "value": shape.N / (ms_per_step * 1e-3),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": workload, "block": f"N{shape.N} {shape.Cin}->{shape.Cexp}->{shape.Cout} "
                   f"{shape.H}x{shape.W} k{shape.k}s{shape.stride} se{shape.Cse} "
                   f"res{int(shape.residual)}" + ("" if getattr(shape, "has_se", True) else " no-se") +
                   (" relu6" if getattr(shape, "activation", "swish") == "relu6" else ""),
                   "policy": args.policy, "mode": args.mode},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(workload if args.policy == "recompute" and not evalm
                                                 else f"{workload}-{args.policy}-{args.mode}", dominant),
                     "kernel_ms": kern_ms, "kernel_ms_with_event_gap": kern_ms_raw,
                     "event_gap_ms": overhead_ms, "algorithmic_bytes": nbytes},
        # the next slowest steps, from the untimed survey (event gap taken off): on config 1 three
        # kernels lie within 2 us of each other and the survey's order among them varies from run
        # to run, so the line shows all of them whichever one `roofline` names
        "roofline_next": [
            _roofline_entry(n, algorithmic_bytes(shape, n), net(n))
            for n in sorted((m for m in survey if m != dominant and algorithmic_bytes(shape, m) is not None),
                            key=lambda m: -survey[m])[:3]],
        "step_roofline": {"bound": "hbm", "algorithmic_bytes": total_bytes,
                          "achieved": round(total_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                          "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": round(total_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "step_ms_survey": {n: round(v, 5) for n, v in survey.items()},
        "launch_steps": len(survey),
    }
    if step_stats is not None:
        result["step_ms_distribution"] = {
            k_: ([round(v_, 5) for v_ in v] if isinstance(v, list) else round(v, 5))
            for k_, v in step_stats.items()}
    if with_cpu:
        result["cpu_baseline"] = cpu_baseline(shape, tensors, evalm)
        if args.cpu_1thread:
            result["cpu_baseline"]["one_thread"] = cpu_baseline_one_thread(shape, evalm)
    del blk
    torch.cuda.empty_cache()
    return result


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, choices=[0, 1, 2, 3, 4, 5],
                    help="4 (default): the EfficientNet-B0 chain of 16 MBConv blocks, the largest "
                         "workload; 0-3: single MBConv blocks; 5: a MobileNet-V2 inverted-residual "
                         "block (ReLU6, no SE) with config 1's tensor shapes")
    ap.add_argument("--policy", default="recompute", choices=["recompute", "store"])
    ap.add_argument("--mode", default="train", choices=["train", "eval"],
                    help="train: forward+backward (the headline metric); eval: the evaluation-mode "
                         "forward alone (BN with running statistics), configs 0-3")
    ap.add_argument("--op", default=None, choices=["mish", "layernorm", "softmax"],
                    help="benchmark one of the paper's other memory-bound operators (forward + "
                         "backward) instead of the MBConv step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="config 4 only: do not also run the single-block configs 1-3")
    ap.add_argument("--cpu-1thread", action="store_true",
                    help="also time the oracle on one thread (on a quarter of the batch; slow)")
    ap.add_argument("--probe-step", default=None,
                    help="time this step for the roofline instead of the slowest one "
                         "(config 4: BLOCK:STEP)")
    ap.add_argument("--no-survey", action="store_true",
                    help="config 4 only: skip the per-block survey (the roofline kernel is then "
                         "--probe-step BLOCK:STEP, default 2:dw_bwd)")
    ap.add_argument("--only-block", type=int, default=0,
                    help="config 4 only: time block B (1-16) of the chain alone, at its real shape "
                         "and on its real input (for profiling one block)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (for scaling rocprofv3 "
                         "FETCH_SIZE/WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    if args.op:
        print(json.dumps(run_op(args)))
        return 0
    if args.config != 4:
        print(json.dumps(run_block(args, args.config, args.steps, args.warmup,
                                   not args.no_cpu_baseline)))
        return 0
    if args.mode != "train":
        print("bench.py: --mode eval covers the single-block configs 0-3", file=sys.stderr)
        return 2
    result = run_chain(args)
    if args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_others and not args.only_block:
        # the single-block configs in the same run, so that one line shows every workload
        others = {}
        saved_probe, args.probe_step = args.probe_step, None
        for cfg in (1, 2, 3):
            r = run_block(args, cfg, max(args.steps, 50), max(args.warmup, 5),
                          not args.no_cpu_baseline, distribution=False)
            keep = {k: r[k] for k in ("value", "unit", "ms_per_step", "dtype", "steps", "roofline_next",
                                      "step_roofline", "launch_steps") if k in r}
            keep["block"] = r["config"]["block"]
            keep["roofline"] = {k: r["roofline"][k] for k in ("kernel", "achieved", "frac", "traffic",
                                                              "kernel_ms", "algorithmic_bytes")}
            if "cpu_baseline" in r:
                keep["cpu_baseline"] = r["cpu_baseline"]
            others[f"config{cfg}"] = keep
        args.probe_step = saved_probe
        result["other_configs"] = others
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
