"""Writes profiles/hbm_traffic_per_step.md, the table bench.py reads `roofline.traffic` from.

    python -m paper_2110_10802_amd.hbm_traffic_table <dir>

<dir> holds the output of eight rocprofv3 counter passes (the commands are repeated in the table's
header): <dir>/c<config>_<COUNTER>/t_counter_collection.csv for config 4, 1, 2, 3 and COUNTER in
FETCH_SIZE, WRITE_SIZE, each run with bench.py's --pmc-calibration option (a 256 MiB device copy
whose counter readings give the scale of the counter).  Every launch of the library is attributed
to its (block, step) by launch order: a step of the library launches a fixed sequence of kernels.
Run from the repository root (it imports bench.py for the algorithmic byte counts)."""
import csv, os, re, sys, statistics
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from mbconv_inputs import b0_chain, CONFIGS
if len(sys.argv) != 2:
    sys.exit(__doc__)
base = sys.argv[1]

FWD = [("expand_conv", r"x3_prep|conv_x3|conv_xw|conv_pe|conv_pr|conv_big|conv_bf|conv1x1_kernel|splitk_finish"),
       ("bn1_finalize", r"bn_finalize"),
       ("dw_fwd", r"dw4_fwd|dwr_fwd|dw2_fwd|dw_fwd_k"),
       ("bn2_finalize", r"bn_finalize"),
       ("se_pool", r"OpPool"),
       ("se_fc", r"se_fwd|fill_kernel"),
       ("proj_conv", r"x3_prep|conv_x3|conv_pe|conv_pr|conv_big|conv_bf|conv1x1_kernel|splitk_finish"),
       ("bn3_finalize", r"bn_finalize"),
       ("bn3_apply", r"bn_apply")]
BWD = [("bn3_bwd_reduce", r"OpDot"),
       ("bn3_bwd_finalize", r"bn_bwd_finalize"),
       ("proj_dgrad", r"wgrad_lt_kernel<.*true>|projbwd_wave|conv_x3|conv_xw|conv_pe|conv_pr|conv_big|conv_bf|conv1x1_kernel|splitk_finish"),
       ("proj_wgrad", r"wgrad_lt_kernel<.*false>|wgrad_x3|wgrad_big|wgrad_bf|wgrad1x1|wgrad_cl|reduce_splits"),
       ("gate_sums", r"OpGate"),
       ("se_bwd", r"se_bwd|bn2_bwd_nose"),
       ("dw_bwd", r"dw4_bwd|dwr_bwd|dw2_bwd|dw_bwd_kernel"),
       ("dw_wgrad_reduce", r"dw_bwd_finalize|reduce_planes"),
       ("expand_dgrad", r"bwd1x1_lt|bwd1x1_x3|conv_x3|conv_pe|conv_pr|conv_big|conv_bf|conv1x1_kernel|splitk_finish"),
       ("expand_wgrad", r"wgrad_lt|wgrad_x3|wgrad_big|wgrad_bf|wgrad1x1|wgrad_cl|reduce_splits")]
NOEXP = {"expand_conv", "bn1_finalize", "expand_dgrad", "expand_wgrad"}

def read(cfg, ctr):
    rows = list(csv.DictReader(open(f"{base}/c{cfg}_{ctr}/t_counter_collection.csv")))
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    cal = max((float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"]), default=0.0)
    lib = [(r["Kernel_Name"], float(r["Counter_Value"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
           for r in rows if "mbk" in r["Kernel_Name"]]
    return lib, cal

def attribute(seq, shapes):
    """seq: kernel names of one step in launch order -> list of (block index, step, [dispatch indices])"""
    out, i = [], 0
    def run(bi, steps, s):
        nonlocal i
        for name, pat in steps:
            if not s.has_expand and name in NOEXP:
                continue
            idx, mains = [], 0
            while i < len(seq) and re.search(pat, seq[i]):
                # a step never swallows the kernel that starts the next step of the same family:
                # stop at one main kernel (+ the weight-image launch ahead of it and its
                # second-stage helpers)
                helper = re.search(r"x3_prep|splitk_finish|reduce_splits|se_bwd_batch", seq[i]) or \
                    (name == "se_bwd" and "se_bwd" in seq[i])
                if not helper:
                    if mains:
                        break
                    mains += 1
                idx.append(i)
                i += 1
            if idx:
                out.append((bi, name, idx))
    for bi, s in enumerate(shapes):
        run(bi, FWD, s)
    for bi in range(len(shapes) - 1, -1, -1):
        run(bi, BWD, shapes[bi])
    assert i == len(seq), f"unattributed dispatch {i} of {len(seq)}: {seq[i][:80]}"
    return out

lines = ["# HBM traffic per launch, by step: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE", "",
         "Commands (from the repo root on the MI355X box, after cd /tmp && export TMPDIR=/tmp && cd <repo>), one pass per counter:", "",
         "  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o t -- python3 bench.py --config 4 --steps 1 --warmup 1 --no-survey --no-others --no-cpu-baseline --pmc-calibration",
         "  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out> -o t -- python3 bench.py --config 4 --steps 1 --warmup 1 --no-survey --no-others --no-cpu-baseline --pmc-calibration",
         "  (and the same two passes with --config 1|2|3 --steps 4 --warmup 1 --no-cpu-baseline --pmc-calibration)", "",
         "Both counters read KiB per dispatch.  They are scaled by what the same counter reads for the plain 256 MiB device",
         "copy the calibration option appends to the run (262144 KiB each way): the factor is given per workload below.",
         "A launch is attributed to its (block, step) by launch order: every step of the library launches a fixed sequence",
         "of kernels.  Median over the steps of the run; a step with two launches (a convolution and the sum over its split",
         "partial tiles, the two SE backward kernels, the weight-image launch ahead of a block's first convolution) is their",
         "sum.  us = kernel time inside the counter run (serialised by the",
         "profiler).  bench.py reads `traffic` for its roofline kernel from this table, which",
         "`python -m paper_2110_10802_amd.hbm_traffic_table <out>` writes from the eight passes' csv files.", "",
         "| workload | step | kernel | us | fetch MiB | write MiB | algorithmic MiB |",
         "|---|---|---|---|---|---|---|"]
import importlib
bench = importlib.import_module("bench")
notes = []
for cfg in (4, 1, 2, 3):
    f, fcal = read(cfg, "FETCH_SIZE")
    w, wcal = read(cfg, "WRITE_SIZE")
    assert [x[0] for x in f] == [x[0] for x in w], "launch sequences of the two passes differ"
    sf, sw = 262144.0 / fcal, 262144.0 / wcal
    shapes = b0_chain() if cfg == 4 else [CONFIGS[cfg]]
    # length of one step: the sequence repeats
    names = [x[0] for x in f]
    L = next(l for l in range(10, len(names) + 1) if len(names) % l == 0 and names[:l] * (len(names) // l) == names)
    reps = len(names) // L
    att = attribute(names[:L], shapes)
    notes.append(f"config {cfg}: {L} launches per step, {reps} steps in the run; copy calibration FETCH_SIZE={fcal:.0f} WRITE_SIZE={wcal:.0f} -> fetch x{sf:.3f}, write x{sw:.3f}")
    for bi, step, idx in att:
        fm = statistics.median(sum(f[r * L + i][1] for i in idx) for r in range(reps)) * sf / 1024
        wm = statistics.median(sum(w[r * L + i][1] for i in idx) for r in range(reps)) * sw / 1024
        us = statistics.median(sum(f[r * L + i][2] for i in idx) for r in range(reps))
        alg = bench.algorithmic_bytes(shapes[bi], step)
        main = next((i for i in idx if "x3_prep" not in names[i]), idx[0])
        kern = re.sub(r"^void |mbk::|mbk_r6::", "", names[main]).split("(")[0][:60]
        key = f"block{bi + 1}:{step}" if cfg == 4 else step
        lines.append(f"| config{cfg} | {key} | `{kern}` | {us:.1f} | {fm:.1f} | {wm:.1f} | {alg / 2**20:.1f} |" if alg else
                     f"| config{cfg} | {key} | `{kern}` | {us:.1f} | {fm:.1f} | {wm:.1f} | - |")
hdr = lines.index("| workload | step | kernel | us | fetch MiB | write MiB | algorithmic MiB |")
lines[hdr:hdr] = notes + [""]
open(os.path.join(ROOT, "profiles", "hbm_traffic_per_step.md"), "w").write("\n".join(lines) + "\n")
print("\n".join(notes))
