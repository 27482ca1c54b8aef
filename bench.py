"""Benchmark of the convolution hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--dtype f32|bf16]
                    [--workload resnet50|inception_v3] [--layers all|4,8,13,18]
                    [--table] [--table-dir DIR] [--no-cpu] [--no-ceilings] [--no-detail]

A "step" is one pass of the whole hot path over one minibatch: forward,
backward-by-data and weight update (partial + reduce) of every layer in the
workload, on tensors already resident in HBM in the blocked layout.  The default
workload is the full layer set the headline metric is quoted on: all 20
ResNet-50 layers of Table I at N = 256 (the four 3x3 layers, the fifteen 1x1
layers and the 7x7 first layer), seeded synthetic inputs.  With no --dtype the
run times that workload twice: in fp32 (the headline: value, ms_per_step,
roofline, cpu_baseline) and in bf16 (the "bf16" object of the same line); both
carry per-class (3x3 / 1x1 / conv1) rates per pass (timed in a separate pass after
the clock has stopped: events around all 60 calls of a step cost 0.45 ms of stream
time, so the timed steps bracket the forward launches only).  "measured_ceilings" holds
what this device sustains on an MFMA issue loop, a 1 GiB copy and an L2 -> LDS
streaming loop.  Prints ONE JSON line.

--table additionally times every requested layer/pass on its own (in the cycling
loop and repeated back to back) and writes a per-layer table (TFLOP/s, % of MFMA
peak, % of the layer's roofline ceiling at the published and at the measured
ceilings) as JSON into --table-dir and as text to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

# (kernel arguments in device memory: see paper_1808_05567_amd/__init__.py; set before the HIP
# runtime initialises, unless the environment says otherwise)
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK = {"f32": 157.3, "bf16": 2500.0}   # TFLOP/s, dense, published MI355X figures
HBM_PEAK = 8.0                                # TB/s
N_BATCH = 256


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--dtype", default=None, choices=["f32", "bf16"],
                    help="one type only (default: fp32 as the headline plus a bf16 block)")
    ap.add_argument("--workload", default="resnet50", choices=["resnet50", "inception_v3"],
                    help="layer table: ResNet-50 (Table I of the paper) or the distinct "
                         "Inception-v3 shapes (second workload; --layers all)")
    ap.add_argument("--layers", default=None,
                    help="comma-separated layer ids of the workload, or 'all' (the default)")
    ap.add_argument("--batch", type=int, default=N_BATCH)
    ap.add_argument("--table", action="store_true")
    ap.add_argument("--table-dir", default=os.path.join(ROOT, "gpurun_out"),
                    help="where --table writes layers_<workload>_<dtype>.json")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-detail", action="store_true",
                    help="timed steps only: no separate per-pass pass, no shader-clock sampling "
                         "(profiler runs, where every launch is counted)")
    ap.add_argument("--no-ceilings", action="store_true")
    ap.add_argument("--cpu-batch", type=int, default=0,
                    help="minibatch of the oracle's timed sample (default: sized to the workload)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch a plain 1 GiB device copy (reference for HBM counters)")
    ap.add_argument("--summarize-pmc", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: turn two rocprofv3 --pmc counter_collection CSVs "
                         "(FETCH_SIZE, WRITE_SIZE) of a --calib-copy run into a traffic summary")
    ap.add_argument("--summarize-counters", metavar="COUNTER_CSV",
                    help="no GPU work: turn a rocprofv3 --pmc counter_collection CSV (GRBM_GUI_ACTIVE, "
                         "SQ_VALU_MFMA_BUSY_CYCLES, SQ_LDS_BANK_CONFLICT, SQ_LDS_IDX_ACTIVE, SQ_INSTS_LDS, "
                         "SQ_WAIT_INST_LDS, SQ_WAVE_CYCLES, SQ_BUSY_CYCLES) into a per-kernel table")
    ap.add_argument("--lib-gemm", action="store_true",
                    help="context only, no conv work: time the vendor library's plain GEMM "
                         "(torch.matmul) at the GEMM shapes the layers' forward passes would have "
                         "after an im2col expansion that is NOT timed")
    ap.add_argument("--out", default=None)
    return ap.parse_args()


CALIB_BYTES = 1 << 30
# committed counter summaries (HBM bytes per dispatch) by workload: (layers, dtype) -> file
L1X1 = "2,3,5,6,7,9,10,11,12,14,15,16,17,19,20"
TRAFFIC_FILE = {(ly, dt): "igemm_upd_%s_resnet50_%s_n256_hbm_traffic.json" % (dt, wl)
                for wl, ly in (("all", "all"), ("3x3", "4,8,13,18"), ("1x1", L1X1))
                for dt in ("f32", "bf16")}


def summarize_pmc(fetch_csv, write_csv, out):
    """Average HBM bytes per dispatch of every kernel, from FETCH_SIZE / WRITE_SIZE
    (KiB per dispatch), each scaled by what the same counter reads for the 1 GiB copy."""
    import collections
    import csv

    def load(path, counter):
        acc = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] == counter:
                acc[r["Kernel_Name"]].append(float(r["Counter_Value"]))
        return ({k: sum(v) / len(v) for k, v in acc.items()}, {k: len(v) for k, v in acc.items()},
                {k: max(v) for k, v in acc.items()})

    fetch, calls, fetch_max = load(fetch_csv, "FETCH_SIZE")
    write, _, write_max = load(write_csv, "WRITE_SIZE")
    # the calibration copy: the largest dispatch of torch's copy kernel (the same kernel also
    # serves a few tiny copies, so its largest reading is taken, not its mean)
    copy = [k for k in fetch if "copy" in k.lower() or "elementwise" in k.lower()]
    copy = max(copy, key=lambda k: fetch_max[k]) if copy else None
    f_scale = (CALIB_BYTES / 1024.0) / fetch_max[copy] if copy else 1.0
    w_scale = (CALIB_BYTES / 1024.0) / write_max[copy] if copy and write_max.get(copy) else 1.0
    rows = {}
    for k in fetch:
        rows[k] = {"calls": calls[k], "fetch_bytes": fetch[k] * 1024 * f_scale,
                   "write_bytes": write.get(k, 0.0) * 1024 * w_scale}
    summary = {"copy_kernel": copy, "copy_bytes_each_way": CALIB_BYTES,
               "fetch_scale": f_scale, "write_scale": w_scale, "kernels": rows}
    if out:
        with open(out, "w") as f:
            json.dump(summary, f, indent=1)
    for k, r in sorted(rows.items(), key=lambda kv: -kv[1]["fetch_bytes"]):
        print("%-90s calls %4d  fetch %9.1f MB  write %9.1f MB" % (
            k[:90], r["calls"], r["fetch_bytes"] / 1e6, r["write_bytes"] / 1e6))
    print("scales: fetch %.4f write %.4f (copy kernel: %s)" % (f_scale, w_scale, copy))


def summarize_counters(path, out):
    """Per kernel (averages over its dispatches): matrix-core utilisation = MFMA busy cycles
    of all SIMDs / (1024 SIMDs x the kernel's duration in clocks; GRBM_GUI_ACTIVE sums the 8
    XCDs), LDS bank-conflict cycles as a share of the LDS-active cycles, the share of wave
    time spent waiting for LDS instructions, LDS instructions per dispatch."""
    import collections
    import csv
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        acc[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    lines = ["%-88s %6s %9s %8s %10s %9s %11s" % ("kernel", "calls", "clocks", "MFMA %", "LDS confl %",
                                                 "LDS wait %", "LDS insts")]
    rows = []
    for k, v in acc.items():
        if "convmi" not in k:
            continue
        m = {c: sum(x) / len(x) for c, x in v.items()}
        clocks = m.get("GRBM_GUI_ACTIVE", 0.0) / 8.0
        if clocks <= 0:
            continue
        mfma = 100.0 * m.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / (1024.0 * clocks)
        idx = m.get("SQ_LDS_IDX_ACTIVE", 0.0)
        confl = 100.0 * m.get("SQ_LDS_BANK_CONFLICT", 0.0) / idx if idx else 0.0
        wc = m.get("SQ_WAVE_CYCLES", 0.0)
        wait = 100.0 * m.get("SQ_WAIT_INST_LDS", 0.0) / wc if wc else 0.0
        rows.append((clocks * len(v["GRBM_GUI_ACTIVE"]), "%-88s %6d %9.0f %8.1f %10.1f %9.2f %11.0f" % (
            k[:88], len(v["GRBM_GUI_ACTIVE"]), clocks, mfma, confl, wait, m.get("SQ_INSTS_LDS", 0.0))))
    lines += [t for _, t in sorted(rows, reverse=True)]
    text = "\n".join(lines) + "\n"
    if out:
        with open(out, "a") as f:
            f.write(text)
    print(text, end="")


def algorithmic_bytes(l, N, es, which):
    """Each operand once: I + W + O (dW fp32 for the update pass).  An unpadded 1x1 filter
    with a stride reads (forward, update) only the N*C*P*Q input pixels it samples; its
    backward pass still writes all of dI (the zeros included)."""
    sampled = l.R == 1 and l.S == 1 and l.stride > 1 and l.pads == (0, 0) and which != "bwd"
    i = N * l.C * (l.P * l.Q if sampled else l.H * l.W) * es
    o = N * l.K * l.P * l.Q * es
    w = l.K * l.C * l.R * l.S
    return i + o + w * (4 if which == "upd" else es)


def written_bytes(l, N, es, which):
    """The part of algorithmic_bytes that is the pass's result."""
    if which == "fwd":
        return N * l.K * l.P * l.Q * es
    if which == "bwd":
        return N * l.C * l.H * l.W * es
    return l.K * l.C * l.R * l.S * 4


def layer_class(l):
    """The three families of Table I the target names separately."""
    if l.R == 1 and l.S == 1:
        return "1x1"
    return "conv1" if l.C <= 4 else "%dx%d" % (l.R, l.S)


def make_layers(ids, N, dtype_names, workload="resnet50"):
    """One resident layer set per requested type, all fed from the same generated host
    arrays (bf16: rounded once, to nearest even, by the upload's type conversion)."""
    import torch
    from paper_1808_05567_amd import conv, inputs
    out = {d: [] for d in dtype_names}
    for lid in ids:
        l = inputs.layer(lid, workload)
        I = inputs.gen_input(N, l.C, l.H, l.W, lid)
        Wt = inputs.gen_weights(l.K, l.C, l.R, l.S, lid)
        dO = inputs.gen_outgrad(N, l.K, l.P, l.Q, lid)
        for d in dtype_names:
            dt = conv.CONV_BF16 if d == "bf16" else conv.CONV_F32
            L = conv.ConvLayer(N, l.C, l.K, l.H, l.W, l.R, l.S, l.stride, l.pad, dtype=dt)
            # separate resident buffers per pass so that no pass overwrites another's input
            L.set_input(I)
            L.set_weights(Wt)
            L.x_blk = L.in_blk
            L.dy_blk = torch.empty_like(L.out_blk)
            L.out_blk, keep = L.dy_blk, L.out_blk
            L.set_outgrad(dO)
            L.out_blk = keep
            L.dx_blk = torch.empty_like(L.in_blk)
            out[d].append((l, L))
        del I, Wt, dO
    torch.cuda.synchronize()
    return out


def launch(L, which):
    from paper_1808_05567_amd import conv
    if which == "fwd":
        conv.conv_fwd(L.h, L.x_blk, L.wt_blk, L.out_blk, L.ws)
    elif which == "bwd":
        conv.conv_bwd_data(L.h, L.dy_blk, L.wt_blk, L.dx_blk, L.ws)
    else:
        conv.conv_upd(L.h, L.x_blk, L.dy_blk, L.dwt_blk, L.ws)


PASSES = ("fwd", "bwd", "upd")


def bound_calls(layers):
    """The same three C-ABI calls per layer with their arguments marshalled once: a bf16 step
    is about 5 ms of GPU work in some 120 kernel launches, so per-call Python work in the timed
    loop (pointer look-ups, stream queries) must stay well below that."""
    import ctypes
    import torch
    from paper_1808_05567_amd import conv
    lib = conv.load()
    vp = ctypes.c_void_p
    st = vp(torch.cuda.current_stream().cuda_stream)
    calls = []
    for l, L in layers:
        p = {k: vp(getattr(L, k).data_ptr()) for k in ("x_blk", "wt_blk", "out_blk", "dy_blk", "dx_blk",
                                                       "dwt_blk", "ws")}
        calls.append((l.id, "fwd", lib.conv_fwd, (L.h, p["x_blk"], p["wt_blk"], p["out_blk"], p["ws"], st)))
        calls.append((l.id, "bwd", lib.conv_bwd_data, (L.h, p["dy_blk"], p["wt_blk"], p["dx_blk"], p["ws"], st)))
        calls.append((l.id, "upd", lib.conv_upd, (L.h, p["x_blk"], p["dy_blk"], p["dwt_blk"], p["ws"], st)))
    return calls


DETAIL_STEPS = 10


def time_workload(layers, N, steps, warmup, detail=True):
    """W untimed steps, then exactly K timed steps between two synchronisations.  In the timed
    steps only the launches of the dominant kernel (the forward launches) sit between two events
    on the stream the kernels run on (torch's current stream is the one handed to the library):
    an event record costs about 4 us of stream time, and a pair around each of the 60 calls of
    a step is 0.45 ms, a tenth of a bf16 step.  The durations of the other passes come from a
    separate pass of DETAIL_STEPS steps after the clock has stopped, with a pair around every
    launch.  Returns wall seconds, the mean forward durations (ms) of the timed steps per layer
    id, the mean durations per (layer id, pass) of the detail pass, and the shader clock the
    compute units ran at during a step (sampled afterwards, next to three more steps)."""
    import torch

    calls = bound_calls(layers)

    def new_events(n_steps, which):
        evs = [{i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                for i, c in enumerate(calls) if c[1] in which} for _ in range(n_steps)]
        # (recorded once, which is what allocates them, before any clock starts)
        for row in evs:
            for a, b in row.values():
                a.record()
                b.record()
        return evs

    def run(evs):
        for row in evs:
            for i, (_, _, fn, args) in enumerate(calls):
                pair = row.get(i)
                if pair:
                    pair[0].record()
                rc = fn(*args)
                if pair:
                    pair[1].record()
                if rc != 0:
                    raise RuntimeError("conv call failed with status %d" % rc)

    def means(evs):
        return {(calls[i][0], calls[i][1]): sum(row[i][0].elapsed_time(row[i][1]) for row in evs) / len(evs)
                for i in evs[0]}

    evs = new_events(steps, ("fwd",))
    for _ in range(warmup):
        for _, _, fn, args in calls:
            assert fn(*args) == 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(evs)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    fwd = means(evs)
    if not detail:
        return wall, fwd, None, None
    evs = new_events(DETAIL_STEPS, PASSES)
    torch.cuda.synchronize()
    run(evs)
    torch.cuda.synchronize()

    def one_step():
        for _, _, fn, args in calls:
            fn(*args)
    clock = shader_clock_under(one_step, wall * 1e3 / steps)
    return wall, fwd, means(evs), clock


_SIDE_STREAM = None


def shader_clock_under(work, work_ms):
    """Shader clock (MHz; median, lowest and highest of the 8 XCDs) while `work` keeps the
    device busy: one sleeping wave per XCD on a second stream counts shader cycles against the
    constant 100 MHz clock (conv_ceiling_shader_clock).  `work` (work_ms of device time) is
    queued n times back to back, n - 2 of them at least a millisecond; the window is 0.8 of
    those n - 2, begins while the first is under way and ends before the last does (short
    kernels: the gaps between launches are inside the window, a few per cent of it).  Not part
    of any timed region: the eight waves take a register-file share on eight CUs.  None if no
    second stream could be made to run next to the work."""
    import math
    import torch
    from paper_1808_05567_amd import conv
    global _SIDE_STREAM
    ticks = torch.zeros(16, dtype=torch.int64, device="cuda")
    n = max(1, int(math.ceil(1.0 / max(work_ms, 1e-3))))
    # The runtime maps streams onto a few hardware queues; a second stream that shares the main
    # stream's queue runs behind the work instead of next to it.  Keep the first stream whose
    # sampler demonstrably ended before the work did.
    for attempt in range(8):
        side = _SIDE_STREAM or torch.cuda.Stream()
        e_side, e_main = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        work()
        conv.conv_ceiling_shader_clock(8, min(1000000, max(50, int(n * work_ms * 800))), ticks, stream=side)
        e_side.record(side)
        for _ in range(n + 1):
            work()
        e_main.record()
        torch.cuda.synchronize()
        if e_side.elapsed_time(e_main) > 0:
            _SIDE_STREAM = side
            break
        _SIDE_STREAM = None
    else:
        return None
    t = ticks.cpu().view(8, 2).double()
    mhz = sorted((t[:, 0] / (t[:, 1] / 100.0)).tolist())
    return {"median": round(0.5 * (mhz[3] + mhz[4])), "min": round(mhz[0]), "max": round(mhz[-1])}


def summarize(layers, N, dtype_name, wall, fwd, per, steps, traffic_file):
    """Whole-workload rate, per-class rates and the roofline block of the dominant kernel."""
    peak = MFMA_PEAK[dtype_name]
    flops_step = sum(3 * l.flops(N) for l, _ in layers)
    ms_per_step = wall * 1e3 / steps
    value = flops_step / (wall / steps) / 1e12

    def rate(ls, which, src=None):
        fl = sum(l.flops(N) for l in ls)
        ms = sum((src or per)[(l.id, which)] for l in ls)
        return fl / (ms * 1e-3) / 1e12

    per_class = {}
    for cls in sorted({layer_class(l) for l, _ in layers} if per else ()):
        ls = [l for l, _ in layers if layer_class(l) == cls]
        tf = {w: rate(ls, w) for w in PASSES}
        allp = sum(3 * l.flops(N) for l in ls) / (sum(per[(l.id, w)] for l in ls for w in PASSES) * 1e-3) / 1e12
        per_class[cls] = {"layers": [l.id for l in ls],
                          "per_pass_tflops": {w: round(tf[w], 2) for w in PASSES},
                          "per_pass_pct_of_mfma_peak": {w: round(100 * tf[w] / peak, 1) for w in PASSES},
                          "tflops": round(allp, 2), "pct_of_mfma_peak": round(100 * allp / peak, 1)}
    # Dominant kernel: the implicit-GEMM kernel (for a first layer its resident-filter form:
    # the same tiles and MFMA layout).  A forward launch is exactly one launch of it,
    # so the forward events of the timed steps are its launch durations: achieved =
    # algorithmic flops of the forward launches / their summed duration.
    all_l = [l for l, _ in layers]
    achieved = rate(all_l, "fwd", fwd)
    # HBM bytes per implicit-GEMM launch (forward and backward launches together: the counter
    # run cannot tell them apart), from the committed rocprofv3 counter summary of this same
    # workload; null when there is none.
    traffic = None
    if traffic_file and os.path.exists(traffic_file):
        try:
            ks = json.load(open(traffic_file))["kernels"]
            ig = [(v["calls"], v["fetch_bytes"] + v["write_bytes"]) for k, v in ks.items()
                  if "igemm_kernel" in k or "igemm_stem_kernel" in k]
            traffic = round(sum(c * b for c, b in ig) / sum(c for c, _ in ig))
        except Exception:
            traffic = None
    roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), "traffic": traffic,
                "kernel": "igemm_kernel (the forward launches of the workload's layers)",
                "per_pass_tflops": {w: round(rate(all_l, w), 2) for w in PASSES} if per else None}
    es = 2 if dtype_name == "bf16" else 4
    alg = {w: sum(algorithmic_bytes(l, N, es, w) for l in all_l) for w in PASSES}
    roofline["algorithmic_bytes_per_step"] = alg
    return {"value": round(value, 3), "ms_per_step": round(ms_per_step, 4),
            "pct_of_mfma_peak": round(100 * value / peak, 2), "per_class": per_class,
            "roofline": roofline}


def measure_ceilings():
    """What this device sustains on loops that do nothing else (kernels of the library's own
    ceilings.hip, timed here with events): MFMA issue per type, a 1 GiB copy, L2 -> LDS
    streaming in the forward kernel's staging pattern."""
    import torch
    from paper_1808_05567_amd import conv

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b)
            best = ms if best is None else min(best, ms)
        return best * 1e-3

    out = {}
    blocks, iters = 256 * 2, 20000      # two waves per SIMD on every CU
    sink = torch.empty(256 * 32 * 256, dtype=torch.float32, device="cuda")
    for name, dt, k in (("mfma_f32_tflops", conv.CONV_F32, 2), ("mfma_bf16_tflops", conv.CONV_BF16, 16)):
        it = iters if dt == conv.CONV_BF16 else iters // 2
        s = timed(lambda: conv.conv_ceiling_mfma(dt, blocks, it, sink))
        out[name] = round(blocks * 4 * it * 8 * 2 * 32 * 32 * k / s / 1e12, 1)
        # the same loop kept up for a tenth of a second (the short run above ends before power
        # management has settled), and the shader clock meanwhile
        reps = max(1, int(0.03 / s))

        def burst():
            for _ in range(reps):
                conv.conv_ceiling_mfma(dt, blocks, it, sink)
        s = timed(burst, reps=3) / reps
        out[name.replace("_tflops", "_sustained_tflops")] = round(
            blocks * 4 * it * 8 * 2 * 32 * 32 * k / s / 1e12, 1)
        out[name.replace("_tflops", "_sustained_shader_clock_mhz")] = shader_clock_under(burst, s * reps * 1e3)
    src = torch.empty(CALIB_BYTES, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    s = timed(lambda: conv.conv_ceiling_copy(dst, src, CALIB_BYTES))
    out["hbm_copy_tbps"] = round(2 * CALIB_BYTES / s / 1e12, 2)
    s = timed(lambda: conv.conv_ceiling_read(src, CALIB_BYTES, sink))
    out["hbm_read_tbps"] = round(CALIB_BYTES / s / 1e12, 2)
    s = timed(lambda: conv.conv_ceiling_write(dst, CALIB_BYTES))
    out["hbm_write_tbps"] = round(CALIB_BYTES / s / 1e12, 2)
    del dst
    win = 96 * 1024
    for wgs in (1, 2):
        for regs in (False, True):
            it, nb = 4000, 256 * wgs
            s = timed(lambda: conv.conv_ceiling_l2_to_lds(src, 256 * win, nb, it, sink, regs))
            out["l2_to_lds_tbps_%dwg_per_cu_%s" % (wgs, "via_registers" if regs else "lds_direct")] = round(
                nb * it * 16384 / s / 1e12, 2)
    # 1024 workgroups on 2048 windows: the 256 windows an XCD's workgroups touch (24 MiB) do not
    # fit its 4 MiB L2, all of them (192 MiB) fit the 256 MiB last-level cache -- the rate at
    # which tiles come in from beyond the L2
    for regs in (False, True):
        it, nb = 2000, 1024
        s = timed(lambda: conv.conv_ceiling_l2_to_lds(src, 2048 * win, nb, it, sink, regs))
        out["beyond_l2_to_lds_tbps_4wg_per_cu_%s" % ("via_registers" if regs else "lds_direct")] = round(
            nb * it * 16384 / s / 1e12, 2)
    # LDS operand reads (bytes per clock and CU at the 2.4 GHz the peaks are quoted at): lanes on
    # consecutive chunks, and over a staged tile of 14-pixel rows 16 chunks apart (the 14x14
    # 3x3 layers), where lanes of one 16-lane pass share banks
    for key, row_len, pitch in (("lds_read_bytes_per_clk_cu_contiguous", 0, 0),
                                ("lds_read_bytes_per_clk_cu_rows_of_14_pitch_16", 14, 16)):
        it, nb = 20000, 256
        s = timed(lambda: conv.conv_ceiling_lds_read(nb, it, sink, row_len, pitch))
        out[key] = round(nb * 512 * it * 8 * 16 / s / 256 / 2.4e9, 1)
    del src, sink
    out["note"] = ("MFMA: 512 workgroups x 4 waves (two waves per SIMD), eight independent 32x32 "
                   "accumulator tiles per wave; copy: 1 GiB, read + write bytes counted; L2->LDS: "
                   "workgroups of 4 waves streaming 96 KiB windows that hit the L2 but not the "
                   "32 KiB L1, with loads that write into LDS or through registers; beyond L2: "
                   "the same with more windows per XCD than its L2 holds; LDS reads: one workgroup "
                   "of 8 waves per CU, eight 16-byte reads per lane in flight; shader clock: one "
                   "sleeping wave per XCD on a second stream counting shader cycles against the "
                   "100 MHz clock while the loop runs (the published peaks assume 2400 MHz)")
    return out


def cpu_baseline(ids, n_cpu, workload="resnet50"):
    """The fp64 oracle, as it stands, on a bounded sample: the same layers and
    passes at a reduced minibatch (per-image cost does not depend on N)."""
    import numpy as np
    import oracle
    from paper_1808_05567_amd import inputs
    flops = 0.0
    secs = 0.0
    for lid in ids:
        l = inputs.layer(lid, workload)
        I = inputs.gen_input(n_cpu, l.C, l.H, l.W, lid).astype(np.float64)
        Wt = inputs.gen_weights(l.K, l.C, l.R, l.S, lid).astype(np.float64)
        dO = inputs.gen_outgrad(n_cpu, l.K, l.P, l.Q, lid).astype(np.float64)
        t0 = time.perf_counter()
        oracle.fwd(I, Wt, l.stride, l.pad)
        oracle.bwd_data(dO, Wt, l.H, l.W, l.stride, l.pad)
        oracle.upd(I, dO, l.R, l.S, l.stride, l.pad)
        secs += time.perf_counter() - t0
        flops += 3 * l.flops(n_cpu)
    return {"value": round(flops / secs / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "layers %s, fwd+bwd_data+upd, fp64 naive loops, minibatch %d instead of %d "
                      "(%.1f s of CPU time)" % (",".join(map(str, ids)), n_cpu, N_BATCH, secs)}


def lib_gemm_context(args):
    """The vendor BLAS on [K x C*R*S] . [C*R*S x N*P*Q] for each layer: what a GEMM library
    reaches on this machine at the same sizes with the expanded matrix already in memory.  Context
    for the MFMA fractions of the conv kernels; nothing here is part of the product path."""
    import torch
    from paper_1808_05567_amd import inputs
    tdt = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    torch.backends.cuda.matmul.allow_tf32 = False
    peak = MFMA_PEAK[args.dtype]
    shapes = [("L%d" % i, inputs.layer(i)) for i in (int(x) for x in args.layers.split(","))]
    rows = [(nm, l.K, args.batch * l.P * l.Q, l.C * l.R * l.S) for nm, l in shapes]
    rows.append(("8192^3", 8192, 8192, 8192))
    for nm, M, N, K in rows:
        a = torch.randn(M, K, device="cuda", dtype=tdt)
        b = torch.randn(K, N, device="cuda", dtype=tdt)
        for _ in range(5):
            a @ b
        torch.cuda.synchronize()
        evs = []
        for _ in range(20):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            a @ b
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ms = sorted(x.elapsed_time(y) for x, y in evs)[10]
        tf = 2.0 * M * N * K / ms / 1e9
        print("# lib gemm %-7s %s M=%d N=%d K=%d: %.3f ms %8.1f TF/s %5.1f%% of MFMA peak" % (
            nm, args.dtype, M, N, K, ms, tf, 100 * tf / peak), file=sys.stderr)
        del a, b


def main():
    args = parse()
    if args.lib_gemm:
        args.dtype = args.dtype or "f32"
        args.layers = args.layers or "4,8,13,18"
        lib_gemm_context(args)
        return
    if args.summarize_pmc:
        summarize_pmc(args.summarize_pmc[0], args.summarize_pmc[1], args.out)
        return
    if args.summarize_counters:
        summarize_counters(args.summarize_counters, args.out)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1808_05567_amd import inputs
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.layers is None:
        args.layers = "all"
    if args.layers == "all":
        ids = [l.id for l in inputs.WORKLOADS[args.workload]]
    else:
        ids = [int(x) for x in args.layers.split(",")]
    N = args.batch
    dtypes = [args.dtype] if args.dtype else ["f32", "bf16"]
    head = dtypes[0]
    sets = make_layers(ids, N, dtypes, args.workload)

    ceilings = None
    if not args.no_ceilings:
        ceilings = measure_ceilings()
    if args.calib_copy:
        src = torch.empty(CALIB_BYTES, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    wname = "ResNet-50 Table I" if args.workload == "resnet50" else "Inception-v3 (distinct shapes)"
    summ, pers = {}, {}
    for d in dtypes:
        wall, fwd, per, clock = time_workload(sets[d], N, args.steps, args.warmup, detail=not args.no_detail)
        tf = None
        if args.workload == "resnet50" and N == N_BATCH and (args.layers, d) in TRAFFIC_FILE:
            tf = os.path.join(ROOT, "profiles", TRAFFIC_FILE[(args.layers, d)])
        summ[d] = summarize(sets[d], N, d, wall, fwd, per, args.steps, tf)
        summ[d]["shader_clock_mhz_during_step"] = clock
        pers[d] = per

    h = summ[head]
    result = {
        "metric": "conv TFLOPS per pass (fwd/bwd/upd) on %s layers; %% of MFMA peak" % (
            "ResNet-50" if args.workload == "resnet50" else "Inception-v3"),
        "value": h["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": h["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": head, "data": "synthetic",
        "config": {"workload": "%s, layers %s (%d layers), N=%d, %s, fwd+bwd_data+upd per layer, "
                               "blocked tensors resident in HBM" % (wname, args.layers, len(ids), N, head),
                   "pct_of_mfma_peak": h["pct_of_mfma_peak"], "per_class": h["per_class"],
                   "shader_clock_mhz_during_step": h["shader_clock_mhz_during_step"],
                   "timing": "value and ms_per_step: the K timed steps, with an event pair around the "
                             "forward launches only (roofline.achieved); per_class and per_pass figures: a "
                             "separate pass of %d steps with an event pair around every launch (an event "
                             "record costs about 4 us of stream time)" % DETAIL_STEPS,
                   "runtime_env": {"HIP_FORCE_DEV_KERNARG": os.environ.get("HIP_FORCE_DEV_KERNARG")}},
        "roofline": h["roofline"],
    }
    for d in dtypes[1:]:
        result[d] = {"workload": "the same layers and passes, N=%d, %s tensors, fp32 accumulation, "
                                 "fp32 weight gradients" % (N, d),
                     "value": summ[d]["value"], "unit": "TFLOP/s", "ms_per_step": summ[d]["ms_per_step"],
                     "steps": args.steps, "warmup": args.warmup,
                     "pct_of_mfma_peak": summ[d]["pct_of_mfma_peak"], "per_class": summ[d]["per_class"],
                     "shader_clock_mhz_during_step": summ[d]["shader_clock_mhz_during_step"],
                     "roofline": summ[d]["roofline"]}
    if ceilings:
        result["measured_ceilings"] = ceilings

    if args.table and not args.no_detail:
        for d in dtypes:
            layer_table(args, sets[d], N, d, pers[d], ceilings)

    for d in dtypes:
        for _, L in sets[d]:
            L.close()
    if not args.no_cpu:
        n_cpu = args.cpu_batch or (32 if len(ids) > 8 else 128)
        result["cpu_baseline"] = cpu_baseline(ids, n_cpu, args.workload)
    print(json.dumps(result), flush=True)


def layer_table(args, layers, N, dtype_name, per, ceilings):
    """Per layer and pass: the cycling loop's duration (operands evicted from the 256 MB
    last-level cache between launches: cold), the same launch repeated back to back (warm),
    % of the published MFMA peak, % of the layer's own ceiling min(MFMA peak, AI x HBM rate)
    at the published figures and at the measured ones, and the shader clock the compute units
    ran at while the launch was repeated (the peaks assume 2400 MHz)."""
    import torch
    from paper_1808_05567_amd import conv as _conv
    es = 2 if dtype_name == "bf16" else 4
    peak = MFMA_PEAK[dtype_name]
    m_peak = (ceilings or {}).get("mfma_%s_tflops" % dtype_name)
    m_rd = (ceilings or {}).get("hbm_read_tbps")
    m_wr = (ceilings or {}).get("hbm_write_tbps")
    warm, clk = {}, {}
    for l, L in layers:
        for which in PASSES:
            launch(L, which)
            evs = []
            for _ in range(max(3, args.steps)):
                a0 = torch.cuda.Event(enable_timing=True)
                a1 = torch.cuda.Event(enable_timing=True)
                a0.record()
                launch(L, which)
                a1.record()
                evs.append((a0, a1))
            torch.cuda.synchronize()
            warm[(l.id, which)] = sum(x.elapsed_time(y) for x, y in evs) / len(evs)
            # the shader clock while this kernel runs (back to back, a window inside the middle launch)
            c = shader_clock_under(lambda: launch(L, which), warm[(l.id, which)])
            clk[(l.id, which)] = c["median"] if c else 0

    def row(l, which, ms, by, extra=None, wr=None):
        tf = l.flops(N) / (ms * 1e-3) / 1e12
        ceil = min(peak, l.flops(N) / by * HBM_PEAK)
        r = {"layer": l.id, "pass": which, "ms": round(ms, 4), "tflops": round(tf, 2),
             "pct_mfma_peak": round(100 * tf / peak, 1),
             "ceiling_tflops": round(ceil, 1), "pct_ceiling": round(100 * tf / ceil, 1),
             "alg_GBps": round(by / (ms * 1e-3) / 1e9, 1)}
        if m_peak and m_rd and m_wr:
            # (the measured ceiling: what is read at the measured read rate, what is written at
            # the measured write rate, one after the other)
            wr = written_bytes(l, N, es, which) if wr is None else wr
            secs = (by - wr) / (m_rd * 1e12) + wr / (m_wr * 1e12)
            mc = min(m_peak, l.flops(N) / secs / 1e12)
            r["measured_ceiling_tflops"] = round(mc, 1)
            r["pct_measured_ceiling"] = round(100 * tf / mc, 1)
        if extra:
            r.update(extra)
        return r

    rows = []
    for l, L in layers:
        for which in PASSES:
            rows.append(row(l, which, per[(l.id, which)], algorithmic_bytes(l, N, es, which),
                            {"ms_warm": round(warm[(l.id, which)], 4), "shader_clock_mhz": clk[(l.id, which)]}))
    # forward pass with bias + residual + ReLU fused into its store, timed on its own
    # (dy_blk, a tensor of the output's shape, stands in for the residual)
    for l, L in layers:
        bias = torch.zeros(L.info.Kp, dtype=torch.float32, device="cuda")
        kw = dict(bias=bias, residual=L.dy_blk, relu=True, ws=L.ws)
        _conv.conv_fwd_fused(L.h, L.x_blk, L.wt_blk, L.out_blk, **kw)
        evs = []
        for _ in range(args.steps):
            a0 = torch.cuda.Event(enable_timing=True)
            a1 = torch.cuda.Event(enable_timing=True)
            a0.record()
            _conv.conv_fwd_fused(L.h, L.x_blk, L.wt_blk, L.out_blk, **kw)
            a1.record()
            evs.append((a0, a1))
        torch.cuda.synchronize()
        ms = sum(x.elapsed_time(y) for x, y in evs) / len(evs)
        rows.append(row(l, "fwd_fused", ms,
                        algorithmic_bytes(l, N, es, "fwd") + N * l.K * l.P * l.Q * es,
                        wr=written_bytes(l, N, es, "fwd")))
    # layout conversion, timed on its own (the passes work on resident blocked tensors)
    for l, L in layers:
        nchw = torch.empty((N, l.C, l.H, l.W), dtype=L.tdtype, device="cuda")
        nkpq = torch.empty((N, l.K, l.P, l.Q), dtype=L.tdtype, device="cuda")
        for name, fn, src, dst, by in (
                ("pack_in", _conv.conv_pack_in, nchw, L.x_blk, 2 * nchw.numel() * es),
                ("unpack_out", _conv.conv_unpack_out, L.out_blk, nkpq, 2 * nkpq.numel() * es)):
            fn(L.h, src, dst)
            a0 = torch.cuda.Event(enable_timing=True)
            a1 = torch.cuda.Event(enable_timing=True)
            a0.record()
            for _ in range(5):
                fn(L.h, src, dst)
            a1.record()
            torch.cuda.synchronize()
            ms = a0.elapsed_time(a1) / 5
            rows.append({"layer": l.id, "pass": name, "ms": round(ms, 4), "tflops": 0.0,
                         "pct_mfma_peak": 0.0, "ceiling_tflops": 0.0, "pct_ceiling": 0.0,
                         "alg_GBps": round(by / (ms * 1e-3) / 1e9, 1)})
        del nchw, nkpq
    os.makedirs(args.table_dir, exist_ok=True)
    path = os.path.join(args.table_dir, "layers_%s%s.json" % (
        "" if args.workload == "resnet50" else args.workload + "_", dtype_name))
    with open(path, "w") as f:
        json.dump(rows, f, indent=1)
    for r in rows:
        print("# %-4s L%-2d %-10s %8.3f ms %8.2f TF/s %5.1f%% peak %5.1f%% of ceiling%s %7.1f GB/s%s" % (
            dtype_name, r["layer"], r["pass"], r["ms"], r["tflops"], r["pct_mfma_peak"], r["pct_ceiling"],
            " (%5.1f%% of measured)" % r["pct_measured_ceiling"] if "pct_measured_ceiling" in r else "",
            r["alg_GBps"], "  warm %8.3f ms  %4d MHz" % (r["ms_warm"], r["shader_clock_mhz"]) if "ms_warm" in r else ""),
            file=sys.stderr)


if __name__ == "__main__":
    main()
