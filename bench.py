#!/usr/bin/env python3
"""Benchmark of libunit on one MI355X.

Default workload (the one the headline metric is quoted on): the 53 conv layers of a
ResNet-50-shaped network at batch 1, int8 x int8 -> int32, each layer run through the whole
hot path (pack_act NCHW -> blocked NHWC, tile selection, implicit-GEMM MFMA kernel, split
reduce where selected, NCHW int32 epilogue).  One "step" is one pass over all 53 layers;
`value` is 2*MACs / time in TOPS and `ms_per_step` is the ResNet-50-shape batch-1 time.

The same JSON line carries `roofline` (HIP events around the timed steps themselves: the
kernels the step launches, nothing else), `per_layer` (each unique shape's call timed alone,
with its own roofline time and fraction), `cold_ms_per_step` (the same step rotating over more
than 512 MB of layer buffers), `cpu_baseline` (the CPU oracle on a bounded sample) and `others`
(the compute-bound configurations: GEMM 4096^3 and the large conv, int8 and fp16, each with its
own MFMA roofline fraction).  `--step-only` runs just the timed steps (for profiling: every
kernel the profiler then sees belongs to a step).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"i8": 5000.0, "u8i8": 5000.0, "f16": 2500.0, "bf16": 2500.0, "fp8": 5000.0}        # dense MFMA TOPS / TFLOPS (published MI355X)
HBM_GBS = 8000.0
# HBM-side bytes per launch (per step for the layer set) of the main kernel, from the committed
# rocprofv3 counter runs (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, factors from a 256 MiB copy in the
# same run); files profiles/igemm_*.md.  Not measurable live, so carried as constants.
TRAFFIC = {"resnet50_i8_b1": 139.9e6, "gemm_i8_4096": 167.9e6, "gemm_f16_4096": 268.6e6, "large_conv_i8": 138.7e6}
COLD_BYTES = 512 << 20     # the cold step rotates over layer-buffer sets totalling more than this


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet50_i8_b1",
                    choices=["resnet50_i8_b1", "gemm_i8_4096", "large_conv_i8", "gemm_f16_4096",
                             "large_conv_f16", "resnet50_f16_b16", "table1_ablation", "conv3d_resnet18",
                             "gemm_i8_8192", "gemm_f16_8192"])
    ap.add_argument("--no-others", action="store_true", help="skip the secondary configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--step-only", action="store_true",
                    help="layer-set workloads: run only the warm-up and the timed steps (no per-layer timing loops, no "
                         "cold rotation, no other configurations, no CPU baseline), so that a profile of the run holds "
                         "the step's kernels only")
    ap.add_argument("--phase-probe", action="store_true",
                    help="ResNet-50 batch-1 set on the instrumented library (make -C paper_2101_08458_amd/csrc probe): per-layer "
                         "time stamps of the main kernel's phases inside the replayed 53-layer graph; with a gemm_* workload, "
                         "the phases of that GEMM's rounds of workgroups; prints its own JSON line")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (counter calibration for profiles)")
    return ap.parse_args()


class ConvCase:
    """Device-resident buffers and launch closures for one conv layer."""

    def __init__(self, torch, unit, wl, sh, n, dtype, config_id, layer_id):
        self.sh, self.n, self.dtype = sh, n, dtype
        self.unit = unit
        dev = "cuda:0"
        i8 = dtype == "i8"
        self.ut = unit.UNIT_I8 if i8 else unit.UNIT_F16
        x, w = (wl.conv_inputs_i8 if i8 else wl.conv_inputs_f16)(sh, n, config_id, layer_id)
        tdt = torch.int8 if i8 else torch.int16
        self.x = torch.from_numpy(x.view(np.int8 if i8 else np.int16)).to(dev)
        wd = torch.from_numpy(w.view(np.int8 if i8 else np.int16)).to(dev)
        self.d = unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
        p, q = unit.unit_conv2d_out_dims(self.d)
        self.p, self.q = p, q
        self.xp = torch.empty(unit.unit_packed_act_bytes(n, sh.c, sh.h, sh.w, self.ut), dtype=torch.uint8, device=dev)
        self.wp = torch.empty(unit.unit_packed_weights_bytes(self.d, self.ut), dtype=torch.uint8, device=dev)
        (unit.unit_pack_weights_i8 if i8 else unit.unit_pack_weights_f16)(self.d, wd, self.wp)
        self.y = torch.empty((n, sh.k, p, q), dtype=torch.int32 if i8 else torch.float32, device=dev)
        self.ws = torch.empty(max(unit.unit_conv2d_wpacked_workspace(self.d, self.ut), 256), dtype=torch.uint8, device=dev)
        es = 1 if i8 else 2
        self.macs = wl.macs(sh, n)
        self.bytes = (x.size + w.size) * es + self.y.numel() * 4      # each operand once, output once
        self.info = unit.unit_select_conv2d(self.d, self.ut)
        self.pack()
        torch.cuda.synchronize()

    def clone(self, torch):
        """Same layer on fresh device buffers (same values): for rotating over more memory than the caches hold."""
        import copy
        c = copy.copy(self)
        c.x, c.wp = self.x.clone(), self.wp.clone()
        c.xp, c.y, c.ws = torch.empty_like(self.xp), torch.empty_like(self.y), torch.empty_like(self.ws)
        return c

    def pack(self):
        u, sh = self.unit, self.sh
        (u.unit_pack_act_i8 if self.dtype == "i8" else u.unit_pack_act_f16)(self.n, sh.c, sh.h, sh.w, self.x, self.xp)

    def conv(self):
        u = self.unit
        if self.dtype == "i8":
            u.unit_conv2d_packed_i8(self.d, self.xp, self.wp, self.y, None, None, None, self.ws)
        else:
            u.unit_conv2d_packed_f16(self.d, self.xp, self.wp, self.y, self.ws)

    def api(self):
        """NCHW activations in, NCHW accumulators out, weights pre-packed: one library call
        (pack_act + conv, or the fused NCHW-direct kernel where the shape allows it)."""
        u = self.unit
        if self.dtype == "i8":
            u.unit_conv2d_wpacked_i8(self.d, self.x, self.wp, self.y, None, None, self.ws)
        else:
            u.unit_conv2d_wpacked_f16(self.d, self.x, self.wp, self.y, self.ws)


class GemmCase:
    _KINDS = {   # dtype -> (inputs, numpy view, element bytes, unit_dtype name, entry point)
        "i8": ("gemm_inputs_i8", np.int8, 1, "UNIT_I8", "unit_matmul_i8"),
        "f16": ("gemm_inputs_f16", np.int16, 2, "UNIT_F16", "unit_matmul_f16"),
        "bf16": ("gemm_inputs_bf16", np.int16, 2, "UNIT_BF16", "unit_matmul_bf16"),
        "u8i8": ("gemm_inputs_u8i8", None, 1, "UNIT_U8I8", "unit_matmul_u8i8"),
        "fp8": ("gemm_inputs_fp8", None, 1, "UNIT_FP8", "unit_matmul_fp8"),
    }

    def __init__(self, torch, unit, wl, m, n, k, dtype):
        dev = "cuda:0"
        gen, view, es, ut, fn = self._KINDS[dtype]
        integer = dtype in ("i8", "u8i8")
        self.unit, self.dtype, self.m, self.n, self.k = unit, dtype, m, n, k
        A, B = getattr(wl, gen)(m, n, k)
        self.A = torch.from_numpy(A.view(view) if view else A).to(dev)
        self.B = torch.from_numpy(B.view(view) if view else B).to(dev)
        self.C = torch.empty((m, n), dtype=torch.int32 if integer else torch.float32, device=dev)
        ut = getattr(unit, ut)
        self.fn = getattr(unit, fn)
        self.ws = torch.empty(max(unit.unit_matmul_workspace(m, n, k, k, k, ut), 256), dtype=torch.uint8, device=dev)
        self.macs = m * n * k
        self.bytes = (m * k + n * k) * es + m * n * 4
        self.info = unit.unit_select_matmul(m, n, k, ut)
        torch.cuda.synchronize()

    def run(self):
        self.fn(self.m, self.n, self.k, self.A, self.k, self.B, self.k, self.C, self.n, self.ws)


RAMP_MS = 30.0   # the GPU needs ~10 ms of work after an idle spell before its clocks are back up


def ramp_up(torch, replay, min_ms=RAMP_MS):
    """Untimed replays until `min_ms` of wall time have passed: after idling (input generation on the
    host) the first ~10 ms of kernels run 10-17 % slow, which is a property of the idle clocks, not of
    the kernels."""
    t0 = time.perf_counter()
    if (t0 - _last_busy[0]) * 1e3 < 5.0:          # the GPU was busy a moment ago: still at speed
        return
    while (time.perf_counter() - t0) * 1e3 < min_ms:
        replay()
        torch.cuda.synchronize()


_last_busy = [0.0]


def mark_busy():
    _last_busy[0] = time.perf_counter()


def event_ms(torch, fn, reps, warm=2):
    """Average device time of one fn() from a HIP event pair around a graph of `reps`
    back-to-back calls on torch's current stream (the stream the library launches on)."""
    g = capture(torch, fn, reps)
    ramp_up(torch, g.replay)
    for _ in range(warm):
        g.replay()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    g.replay()
    b.record()
    torch.cuda.synchronize()
    mark_busy()
    return a.elapsed_time(b) / reps


def capture(torch, fn, reps=1):
    """Record `reps` calls of fn() into a HIP graph (the library launches on torch's current
    stream, which is the capturing stream inside the context).  Replaying it runs exactly the
    same kernels without the per-launch host cost of the Python binding."""
    fn()                                   # first call outside capture: one-time function attributes
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(reps):
            fn()
    return g


def wall_ms(torch, fn, steps, warmup, use_graph=True):
    """Wall-clock time per call: `warmup` untimed calls, then exactly `steps` timed ones between
    two device synchronisations."""
    run = capture(torch, fn).replay if use_graph else fn
    ramp_up(torch, run)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    mark_busy()
    return (time.perf_counter() - t0) * 1e3 / steps


def timed_steps(torch, replay, steps, warmup):
    """`warmup` untimed steps, then exactly `steps` timed ones between two device synchronisations.
    Returns (wall ms per step, HIP-event ms per step); the events are recorded on torch's current
    stream, which is the stream the library launches on and the graph replays on."""
    ramp_up(torch, replay)
    for _ in range(warmup):
        replay()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    a.record()
    for _ in range(steps):
        replay()
    b.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    mark_busy()
    return wall, a.elapsed_time(b) / steps


def roof_us(macs, byts, dtype):
    """Roofline time of one layer: the larger of its MFMA time and its HBM time at the published peaks."""
    return max(2.0 * macs / (PEAK[dtype] * 1e12), byts / (HBM_GBS * 1e9)) * 1e6


def mfma_ceiling(torch, unit):
    """What the matrix units sustain with nothing else running (unit_measure_mfma: the large tile's MFMA
    sequence on register-resident operands), on constant and on uniformly random operands, for a launch
    with as many MFMAs as the 4096^3 matmul and for a long one.  The clock is what the waves measured
    in-kernel (core cycles per 100 MHz real-time tick)."""
    res = []
    counters = torch.zeros(unit.UNIT_MEASURE_COUNTERS_BYTES // 8, dtype=torch.int64, device="cuda:0")
    for dtype, ut, kb in (("i8", unit.UNIT_I8, 32), ("f16", unit.UNIT_F16, 16)):
        for rnd in (0, 1):
            for steps in (4096 * (1 if dtype == "i8" else 2) // 128, 2048):
                fn = lambda: unit.unit_measure_mfma(ut, steps, rnd, counters)
                reps = 20 if steps < 1000 else 3
                ms = event_ms(torch, fn, reps)
                c = counters.cpu().numpy().reshape(-1, 4)
                ops = 256 * 8 * steps * 32 * 2.0 * 32 * 32 * kb
                res.append({"dtype": dtype, "operands": "random" if rnd else "constant", "steps": steps,
                            "us": round(ms * 1e3, 1), "value": round(ops / (ms * 1e-3) / 1e12, 1),
                            "unit": "TOPS" if dtype == "i8" else "TFLOPS",
                            "frac_of_nominal_peak": round(ops / (ms * 1e-3) / 1e12 / PEAK[dtype], 4),
                            "shader_clock_MHz": round(float(c[:, 0].sum()) / max(float(c[:, 1].sum()), 1.0) * 100.0)})
    return res


def phase_probe(torch, unit, wl, dtype="i8", n=1, config_id=3):
    """Where the 53-layer step's time goes, from inside the kernels: the instrumented library stamps the cycle and the
    100 MHz real-time counters at the main kernel's phase boundaries in every wave (UNIT_STAMP in csrc/igemm.hpp); the
    step is captured as usual, every layer writing to a probe region of its own, and replayed."""
    import ctypes
    lib = unit.load()
    layers = wl.resnet50_convs()
    seq = [ConvCase(torch, unit, wl, sh, n, dtype, config_id, idx) for idx, sh in enumerate(layers)]
    slot = 1 << 18                                       # uint64 per layer: up to 16384 waves x 16 stamps
    probe = torch.zeros(len(seq) * slot, dtype=torch.int64, device="cuda:0")
    lib.unit_probe_set.restype, lib.unit_probe_set.argtypes = None, [ctypes.c_void_p]

    def step():
        for i, c in enumerate(seq):
            lib.unit_probe_set(probe.data_ptr() + i * slot * 8)
            c.api()
        lib.unit_probe_set(None)
    g = capture(torch, step)
    for _ in range(20):
        g.replay()
    torch.cuda.synchronize()
    probe.zero_()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    g.replay()
    b.record()
    torch.cuda.synchronize()
    P = probe.cpu().numpy().reshape(len(seq), slot)
    rows, prev_end = [], None
    keys = ("gap_us", "skew_us", "prologue_math_us", "prologue_issue_us", "prologue_wait_us", "loop_us", "drain_us",
            "epilogue_issue_us", "stores_ack_us", "span_us")
    tot = dict.fromkeys(keys, 0.0)
    for i, c in enumerate(seq):
        mode = unit.unit_conv2d_input_mode(c.d, c.ut, c.x)
        info = unit.unit_select_conv2d_input(c.d, c.ut, mode)
        nw = (info.workgroups // info.split_k) * info.waves_m * info.waves_n * info.waves_k
        p = P[i, :nw * 16].reshape(nw, 16)
        rt = p[:, 8:16].astype(np.float64) / 100.0        # microseconds (100 MHz counter)
        rt = rt[rt[:, 0] > 0]
        # stamp order in time: 0 entry, 6 arithmetic done, 7 tiles requested, 1 loop start, 2 loop end, 3 drained,
        # 4 stores issued, 5 stores acknowledged (with a reduction split the slices share the region: last writer wins)
        t = rt[:, [0, 6, 7, 1, 2, 3, 4, 5]]
        start, end = t[:, 0].min(), t[:, 7].max()
        d = np.diff(t, axis=1).mean(axis=0)
        r = {"layer": i, "shape": list(layers[i]), "input": ("packed", "direct", "direct-shifted")[mode],
             "workgroups": info.workgroups, "split": info.split_k,
             "gap_us": round(start - prev_end, 2) if prev_end is not None else 0.0,
             "skew_us": round(t[:, 0].mean() - start, 2)}
        for k, v in zip(keys[2:9], d):
            r[k] = round(float(v), 2)
        r["span_us"] = round(end - start, 2)
        # shader clock over the loop: core cycles per real-time tick
        cyc = p[:, :8].astype(np.float64)[p[:, 8] > 0]
        # (only without a reduction split: its slices share a probe region, and the cycle counters of different XCDs differ)
        r["loop_clock_MHz"] = (round(float((cyc[:, 2] - cyc[:, 1]).mean() / max((rt[:, 2] - rt[:, 1]).mean(), 1e-9)))
                               if info.split_k == 1 else None)
        # small-tile step loop: mean cycles per step a wave waits for its own loads, at the barrier, and for its
        # fragment reads (sums kept by the instrumented kernel in cycle slots 3-6)
        steps_run = cyc[:, 6]
        if steps_run.min() > 0:
            r["steps"] = int(steps_run.max())
            loop_cyc = (cyc[:, 2] - cyc[:, 1]) / steps_run
            r["cycles_per_step"] = {"total": round(float(loop_cyc.mean())) if info.split_k == 1 else None,
                                    "wait_loads": round(float((cyc[:, 3] / steps_run).mean())),
                                    "barrier": round(float((cyc[:, 4] / steps_run).mean())),
                                    "wait_fragments": round(float((cyc[:, 5] / steps_run).mean()))}
        prev_end = end
        rows.append(r)
        for k in keys:
            tot[k] += r[k]
    return {"metric": f"phase time stamps inside the replayed 53-layer step ({dtype}, batch {n})", "unit": "us",
            "probed_step_us": round(a.elapsed_time(b) * 1e3, 1),
            "note": "gap = last wave of the previous main kernel to first wave of this one (contains any pack_act / "
                    "splitk_reduce launched in between); the instrumented kernels are a few percent slower than the product's",
            "sums_us": {k: round(v, 1) for k, v in tot.items()}, "layers": rows}


def phase_probe_gemm(torch, unit, wl, dtype, size):
    """Phase stamps of the large-tile kernel on one size^3 GEMM (instrumented library): per round of 256 workgroups,
    when its waves pass each phase boundary, and the median length of each phase of a wave."""
    import ctypes
    lib = unit.load()
    lib.unit_probe_set.restype, lib.unit_probe_set.argtypes = None, [ctypes.c_void_p]
    c = GemmCase(torch, unit, wl, size, size, size, dtype)
    info = c.info
    nwpg = info.waves_m * info.waves_n * info.waves_k
    nw = info.workgroups * nwpg
    probe = torch.zeros(nw * 16, dtype=torch.int64, device="cuda:0")
    ramp_up(torch, c.run)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        c.run()
    b.record()
    torch.cuda.synchronize()
    plain_us = a.elapsed_time(b) * 100.0
    lib.unit_probe_set(probe.data_ptr())
    for _ in range(3):
        c.run()
    torch.cuda.synchronize()
    a.record()
    c.run()
    b.record()
    torch.cuda.synchronize()
    lib.unit_probe_set(None)
    P = probe.cpu().numpy().reshape(info.workgroups, nwpg, 16)
    rt = P[:, :, 8:16].astype(np.float64)[:, :, [0, 6, 7, 1, 2, 3, 4, 5]] / 100.0     # microseconds, in time order
    cyc = P[:, :, :8].astype(np.float64)
    t0 = rt[:, :, 0].min()
    order = np.argsort(rt[:, :, 0].min(axis=1))
    names = ("entry", "arithmetic_done", "tiles_requested", "loop_start", "loop_end", "drained", "stores_issued", "stores_acked")
    phases = ("prologue_math_us", "prologue_issue_us", "prologue_wait_us", "loop_us", "drain_us", "epilogue_issue_us", "stores_ack_us")
    es = 1 if dtype == "i8" else 2
    steps = (size * es + info.block_k_bytes - 1) // info.block_k_bytes
    mfma_k = 32 if dtype == "i8" else 16
    mfma_cycles = info.block_m * info.block_n * (info.block_k_bytes // es) // (32 * 32 * mfma_k) * 32 // 4
    rounds = []
    for r in range(0, info.workgroups, 256):
        sel = order[r:r + 256]
        d = rt[sel]
        row = {"workgroups": len(sel)}
        for i, nm in enumerate(names):
            row[nm] = [round(float(d[:, :, i].min() - t0), 2), round(float(np.median(d[:, :, i]) - t0), 2),
                       round(float(d[:, :, i].max() - t0), 2)]
        for i, nm in enumerate(phases):
            row[nm] = round(float(np.median(d[:, :, i + 1] - d[:, :, i])), 2)
        lc = cyc[sel][:, :, 2] - cyc[sel][:, :, 1]              # core cycles of the loop, per wave
        lt = d[:, :, 4] - d[:, :, 3]
        row["loop_clock_MHz"] = round(float(lc.mean() / max(lt.mean(), 1e-9)))
        row["loop_cycles_per_step"] = round(float(lc.mean()) / steps)
        # every XCD runs at a clock of its own under the power limit (workgroup id % 8 = XCD)
        row["per_xcd"] = [{"xcd": x, "loop_us": round(float(np.median(lt[sel % 8 == x])), 1),
                           "clock_MHz": round(float((lc[sel % 8 == x] / lt[sel % 8 == x]).mean()))} for x in range(8)]
        rounds.append(row)
    return {"metric": f"phase time stamps of one {dtype} GEMM {size}^3", "unit": "us", "tile": tile_str(info),
            "steps_per_tile": steps,
            # MFMA issue cycles one SIMD needs for a step of the tile (32 cycles per 32x32 MFMA, four SIMDs per workgroup):
            # loop_cycles_per_step below is to be read against this
            "mfma_cycles_per_step": mfma_cycles,
            "unprobed_us": round(plain_us, 1), "probed_us": round(a.elapsed_time(b) * 1e3, 1),
            "kernel_span_us": round(float(rt[:, :, 7].max() - t0), 2),
            "note": "per boundary [min, median, max] over the waves of the round, from the first wave's entry; workgroups "
                    "sorted by entry time, 256 to a round",
            "rounds": rounds}


def tile_str(info):
    tail = f" + tail 256x{info.tail_block_n} wg{info.tail_workgroups}" if info.tail_block_n else ""
    return (f"{info.block_m}x{info.block_n}x{info.block_k_bytes}B waves {info.waves_m}x{info.waves_n}x{info.waves_k} "
            f"mfma{info.mfma} split{info.split_k} wg{info.workgroups}{tail}")


def mfma_roofline(dtype, macs, ms, traffic=None):
    tops = 2.0 * macs / (ms * 1e-3) / 1e12
    return {"bound": "mfma", "achieved": round(tops, 2), "peak": PEAK[dtype],
            "unit": "TOP/s" if dtype == "i8" else "TFLOP/s", "frac": round(tops / PEAK[dtype], 4), "traffic": traffic}


def cpu_baseline(wl, budget_s=12.0):
    """The CPU oracle, as it stands, on whole passes over the same ResNet-50-shaped layer set
    (batch 1) until about `budget_s` seconds of host time are used; at least one full pass."""
    import oracle
    oracle.build()
    layers = wl.resnet50_convs()
    inputs = [wl.conv_inputs_i8(sh, 1, 3, idx) for idx, sh in enumerate(layers)]
    macs, secs, passes = 0, 0.0, 0
    while secs < budget_s:
        for sh, (x, w) in zip(layers, inputs):
            t0 = time.perf_counter()
            oracle.conv2d_i8(x, w, (sh.stride,) * 2, (sh.pad,) * 2)
            secs += time.perf_counter() - t0
            macs += wl.macs(sh)
        passes += 1
    res = {"value": round(2.0 * macs / secs / 1e12, 5), "unit": "TOPS", "cores": oracle.num_threads(),
           "kind": "oracle", "sample": f"{passes} full passes over the 53 ResNet-50-shaped int8 conv layers at "
                                       f"batch 1, {macs / 1e9:.2f} GMAC in {secs:.2f} s, OpenMP direct loops"}
    # the single conv of config 1 (1x64x56x56 * 64x64x3x3) on all cores and on one thread
    x, w = wl.conv_inputs_i8(wl.CONFIG1, 1, 1, 0)
    full = oracle.num_threads()

    def best_of(reps):
        best = 1e30
        for _ in range(reps):
            t0 = time.perf_counter()
            oracle.conv2d_i8(x, w, (1, 1), (1, 1))
            best = min(best, time.perf_counter() - t0)
        return best
    res["config1_ms_all_cores"] = round(best_of(5) * 1e3, 3)
    oracle.set_num_threads(1)
    try:
        res["config1_ms_single_thread"] = round(best_of(3) * 1e3, 3)
    finally:
        oracle.set_num_threads(full)
    return res


def conv3d_resnet18(torch, unit, wl, out):
    """The paper's conv3d experiment (Section VI-C): every 2-D convolution of a ResNet-18-shaped
    network lifted to 3-D.  The paper does not give the depth; here every layer gets an input depth
    of 8 and a cubic kernel (kernel depth = R, depth stride = stride, depth pad = pad).  Batch 1,
    int8 -> int32 and fp16 -> fp32, NCDHW in -> NKOPQ out through unit_conv3d_* (packs both
    operands inside the call)."""
    from paper_2101_08458_amd.resnet18_int8 import layer_list
    shapes = []
    for _, sh in layer_list():
        if sh not in shapes:
            shapes.append(sh)
    rows = []
    for dtype in ("i8", "f16"):
        i8 = dtype == "i8"
        ut = unit.UNIT_I8 if i8 else unit.UNIT_F16
        for idx, sh in enumerate(shapes):
            depth = 8
            g = wl.rng(7, idx)
            shape_x, shape_w = (1, sh.c, depth, sh.h, sh.w), (sh.k, sh.c, sh.r, sh.r, sh.s)
            if i8:
                x, w = wl.int8_activations(g, shape_x), wl.int8_weights(g, shape_w)
            else:
                x = wl.f16_activations(g, shape_x).view(np.int16)
                w = wl.f16_weights(g, shape_w, sh.c * sh.r ** 3).view(np.int16)
            d = unit.conv3d_desc(1, sh.c, depth, sh.h, sh.w, sh.k, sh.r, sh.r, sh.s,
                                 (sh.stride,) * 3, (sh.pad,) * 3)
            o, p, q = unit.unit_conv3d_out_dims(d)
            xd, wd = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(w).to("cuda:0")
            y = torch.empty((1, sh.k, o, p, q), dtype=torch.int32 if i8 else torch.float32, device="cuda:0")
            ws = torch.empty(max(unit.unit_conv3d_workspace(d, ut), 256), dtype=torch.uint8, device="cuda:0")
            f = (lambda: unit.unit_conv3d_i8(d, xd, wd, y, ws)) if i8 else (lambda: unit.unit_conv3d_f16(d, xd, wd, y, ws))
            us = event_ms(torch, f, 10) * 1e3
            macs = sh.k * o * p * q * sh.c * sh.r ** 2 * sh.s
            rows.append({"dtype": dtype, "shape": [sh.c, depth, sh.h, sh.w, sh.k, sh.r, sh.stride, sh.pad],
                         "out": [o, p, q], "us": round(us, 2), "gmac": round(macs / 1e9, 3),
                         "value": round(2.0 * macs / us / 1e6, 2)})
            del xd, wd, y, ws
    tot = {dt: sum(r["us"] for r in rows if r["dtype"] == dt) for dt in ("i8", "f16")}
    mac = {dt: sum(r["gmac"] for r in rows if r["dtype"] == dt) for dt in ("i8", "f16")}
    out.update({"metric": "int8 conv3d TOPS", "unit": "TOPS", "dtype": "i8",
                "value": round(2.0 * mac["i8"] * 1e9 / (tot["i8"] * 1e-6) / 1e12, 2),
                "ms_per_step": round(tot["i8"] / 1e3, 4),
                "fp16_tflops": round(2.0 * mac["f16"] * 1e9 / (tot["f16"] * 1e-6) / 1e12, 2),
                "fp16_ms": round(tot["f16"] / 1e3, 4),
                "config": {"workload": "unique conv layers of a ResNet-18-shaped network lifted to 3-D "
                                       "(input depth 8, cubic kernels), batch 1, unit_conv3d_* calls"},
                "layers": rows})


def table1_ablation(torch, unit, wl, out):
    """The paper's per-kernel experiment (Table I layers; its GPU ablation Generic -> +SplitK
    -> +Tune, Section VI-B) on this hardware: batch 1, kernel only (packed operands).
    Generic = one fixed tile (64x64, 2x2 waves) without a reduction split; +SplitK = the same
    tile with the best grid split; +Tune = best tile and split of the sweep; selector = what
    the library's rule picks.  Fused H*W (the paper's FuseDim) is inherent in the implicit
    GEMM and cannot be switched off."""
    unit.unit_debug_force_tile(-1, -1)
    splits = [1, 2, 3, 4, 6, 8, 12]
    rows = []
    for dtype in ("f16", "i8"):
        for idx, sh in enumerate(wl.TABLE1):
            c = ConvCase(torch, unit, wl, sh, 1, dtype, 6, idx)

            def timed(tile, split):
                unit.unit_debug_force_tile(tile, split)
                try:
                    if unit.unit_select_conv2d(c.d, c.ut).split_k != split:
                        return None
                    need = unit.unit_conv2d_packed_workspace(c.d, c.ut)
                    if need > c.ws.numel():
                        c.ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
                    return event_ms(torch, c.conv, 20) * 1e3
                finally:
                    unit.unit_debug_force_tile(-1, -1)

            generic = timed(3, 1)
            splitk = min(t for t in (timed(3, s) for s in splits) if t is not None)
            tuned = min(t for t in (timed(tl, s) for tl in (1, 2, 3, 4, 9, 12) for s in splits) if t is not None)
            need = unit.unit_conv2d_packed_workspace(c.d, c.ut)
            if need > c.ws.numel():
                c.ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
            auto = event_ms(torch, c.conv, 20) * 1e3
            rows.append({"dtype": dtype, "layer": idx + 1, "shape": list(sh), "generic_us": round(generic, 2),
                         "splitk_us": round(splitk, 2), "tuned_us": round(tuned, 2), "selector_us": round(auto, 2),
                         "selector_tile": tile_str(unit.unit_select_conv2d(c.d, c.ut))})
            del c
    out.update({"metric": "Table I conv layers, batch 1, kernel-only us per layer", "unit": "us", "dtype": "f16+i8",
                "config": {"workload": "16 conv layers of the paper's Table I, batch 1, packed operands"},
                "value": round(sum(r["selector_us"] for r in rows if r["dtype"] == "f16"), 2),
                "higher_is_better": False, "layers": rows})
    for dt in ("f16", "i8"):
        sel = [r for r in rows if r["dtype"] == dt]
        gm = lambda key: float(np.exp(np.mean([np.log(r["generic_us"] / r[key]) for r in sel])))
        out[f"geomean_speedup_over_generic_{dt}"] = {"splitk": round(gm("splitk_us"), 3), "tuned": round(gm("tuned_us"), 3),
                                                      "selector": round(gm("selector_us"), 3)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2101_08458_amd import unit, workloads as wl
    if args.phase_probe:
        unit.LIB_PATH = os.path.join(os.path.dirname(unit.LIB_PATH), "libunit_probe.so")
        if not os.path.exists(unit.LIB_PATH):
            print("bench.py --phase-probe needs the instrumented library: make -C paper_2101_08458_amd/csrc probe", file=sys.stderr)
            sys.exit(2)
    unit.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.phase_probe:
        if args.workload.startswith("gemm_"):
            _, dt, size = args.workload.split("_")
            print(json.dumps(phase_probe_gemm(torch, unit, wl, dt, int(size))))
        elif args.workload == "resnet50_f16_b16":
            print(json.dumps(phase_probe(torch, unit, wl, "f16", 16, 4)))
        else:
            print(json.dumps(phase_probe(torch, unit, wl)))
        return

    if args.copy_calibration_mib:
        src = torch.ones(args.copy_calibration_mib << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "data": "synthetic"}
    others = []

    def conv_set(dtype, n, config_id):
        """The 53 layers, each with buffers and values of its own (as in a network: no two layers share weights
        or activations, so a repeated shape gains nothing from the caches), plus the first case of every unique
        shape for the per-layer table."""
        layers = wl.resnet50_convs()
        seq = [ConvCase(torch, unit, wl, sh, n, dtype, config_id, idx) for idx, sh in enumerate(layers)]
        uniq = {}
        for sh, c in zip(layers, seq):
            uniq.setdefault(sh, c)
        return layers, seq, uniq

    def run_conv_set(dtype, n, config_id, steps, warmup, step_only=False, cold=True):
        layers, seq, uniq = conv_set(dtype, n, config_id)

        def step():
            for c in seq:
                c.api()
        g = capture(torch, step)
        ms, ev_ms = timed_steps(torch, g.replay, steps, warmup)
        macs = sum(c.macs for c in seq)
        byts = sum(c.bytes for c in seq)
        res = {"ms": ms, "event_ms": ev_ms, "macs": macs, "bytes": byts}
        if step_only:
            return res
        res["eager_ms"] = wall_ms(torch, step, max(steps // 10, 3), 2, use_graph=False)
        # per unique shape, each call alone (a graph of 50 back-to-back calls of the same layer: warm caches):
        # api = the call the step makes; conv / pack = the packed-path kernels of the same layer, for comparison
        t_conv = t_pack = t_api = 0.0
        per_layer = []
        for sh, c in uniq.items():
            mult = sum(1 for s in layers if s == sh)
            tc = event_ms(torch, c.conv, 50)
            tp = event_ms(torch, c.pack, 50)
            ta = event_ms(torch, c.api, 50)
            t_conv += mult * tc
            t_pack += mult * tp
            t_api += mult * ta
            mode = unit.unit_conv2d_input_mode(c.d, c.ut, c.x)
            ru = roof_us(c.macs, c.bytes, dtype)
            per_layer.append({"shape": list(sh), "x": mult, "api_us": round(ta * 1e3, 2),
                              "roof_us": round(ru, 3), "frac": round(ru / (ta * 1e3), 4),
                              "bytes": c.bytes, "GBps": round(c.bytes / (ta * 1e-3) / 1e9, 1),
                              "packed_conv_us": round(tc * 1e3, 2), "pack_us": round(tp * 1e3, 2),
                              "tile": tile_str(unit.unit_select_conv2d_input(c.d, c.ut, mode)),
                              "input": ("packed", "direct", "direct-shifted")[mode]})
        res.update({"t_conv": t_conv, "t_pack": t_pack, "t_api": t_api, "per_layer": per_layer})
        if cold:
            # the same step on rotating buffer sets totalling more than COLD_BYTES, so that no layer finds its
            # operands in L2 or the Infinity Cache from an earlier step
            sets = [seq]
            while len(sets) * byts <= COLD_BYTES:
                sets.append([c.clone(torch) for c in seq])

            def rotation():
                for cases in sets:
                    for c in cases:
                        c.api()
            gc = capture(torch, rotation)
            _, cold_ev = timed_steps(torch, gc.replay, max(steps // len(sets), 5), 2)
            res["cold_ms"] = cold_ev / len(sets)
            res["cold_sets"] = len(sets)
            del gc, sets
            torch.cuda.empty_cache()
        return res

    wlname = args.workload
    if wlname == "conv3d_resnet18":
        conv3d_resnet18(torch, unit, wl, out)
        print(json.dumps(out))
        return
    if wlname == "table1_ablation":
        table1_ablation(torch, unit, wl, out)
        print(json.dumps(out))
        return
    if wlname in ("resnet50_i8_b1", "resnet50_f16_b16"):
        dtype, n, cid = ("i8", 1, 3) if wlname == "resnet50_i8_b1" else ("f16", 16, 4)
        r = run_conv_set(dtype, n, cid, args.steps, args.warmup, step_only=args.step_only)
        ms, macs, byts = r["ms"], r["macs"], r["bytes"]
        tops = 2.0 * macs / (ms * 1e-3) / 1e12
        out.update({
            "metric": "int8 conv2d TOPS" if dtype == "i8" else "fp16 conv2d TFLOPS",
            "value": round(tops, 3), "unit": "TOPS" if dtype == "i8" else "TFLOPS",
            "ms_per_step": round(ms, 4), "dtype": dtype,
            "pct_of_mfma_peak": round(100.0 * tops / PEAK[dtype], 3),
            "config": {"workload": f"53 conv layers of a ResNet-50-shaped network, batch {n}, "
                                   f"{'int8->int32' if dtype == 'i8' else 'fp16->fp32'}, NCHW in -> NCHW out per layer "
                                   "(one unit_conv2d_wpacked call: pack_act + implicit-GEMM conv [+ split reduce], or the "
                                   "kernel reading NCHW directly where the shape allows it: see per_layer.input), "
                                   "weights pre-packed, every layer on buffers of its own",
                       "layers": 53, "batch": n, "gmacs_per_step": round(macs / 1e9, 3)},
            "launch": "one HIP graph per step (all kernels of the 53 layers), replayed",
            "event_ms_per_step": round(r["event_ms"], 4),
        })
        # The roofline figure is taken over the timed steps themselves: algorithmic bytes of the 53 layers (each
        # operand once, each output once) / HIP-event time of a step, i.e. all 53 main-kernel launches plus the
        # pack_act and split-reduce launches the step needs and the gaps between launches.
        gbs = byts / (r["event_ms"] * 1e-3) / 1e9
        out["roofline"] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_GBS, "unit": "GB/s",
                           "frac": round(gbs / HBM_GBS, 4), "traffic": TRAFFIC.get(wlname),
                           "algorithmic_bytes": byts,
                           "kernel": "igemm_kernel: the 53 launches of one step, with the step's pack_act and "
                                     "splitk_reduce launches and the inter-launch gaps inside the measured time",
                           "note": "sum of algorithmic bytes (x + w + y once per layer) / HIP-event time of one timed step"}
        if not args.step_only:
            t_roof = sum(l["roof_us"] * l["x"] for l in r["per_layer"]) / 1e3
            out.update({
                "eager_ms_per_step": round(r["eager_ms"], 4),
                # sums over the 53 layers of each call timed alone (warm caches), and of the packed-path kernels
                "api_call_ms_per_step": round(r["t_api"], 4),
                "packed_path_kernel_only_ms_per_step": round(r["t_conv"], 4),
                "packed_path_pack_act_ms_per_step": round(r["t_pack"], 4),
                "roofline_ms_per_step": round(t_roof, 5),
                "frac_of_per_layer_roofline": round(t_roof / r["event_ms"], 4),
            })
            if "cold_ms" in r:
                out["cold_ms_per_step"] = round(r["cold_ms"], 4)
                out["cold_note"] = (f"same step over {r['cold_sets']} rotating sets of layer buffers "
                                    f"({r['cold_sets'] * byts / 2 ** 20:.0f} MiB of operands and outputs per rotation)")
            out["per_layer"] = r["per_layer"]
    else:
        dtype = "i8" if "_i8" in wlname else "f16"
        if wlname.startswith("gemm"):
            size = int(wlname.rsplit("_", 1)[1])
            c = GemmCase(torch, unit, wl, size, size, size, dtype)
            fn, desc = c.run, f"GEMM {size}^3 {dtype}"
        else:
            c = ConvCase(torch, unit, wl, wl.LARGE_CONV, 32, dtype, 9, 0)
            fn, desc = c.api, f"conv N=32 C=K=256 56x56 3x3 {dtype} (pack_act + conv)"
        ms = wall_ms(torch, fn, args.steps, args.warmup)
        tops = 2.0 * c.macs / (ms * 1e-3) / 1e12
        kms = event_ms(torch, c.run if wlname.startswith("gemm") else c.conv, 50)
        out.update({"metric": f"{'int8' if dtype == 'i8' else 'fp16'} {'matmul' if wlname.startswith('gemm') else 'conv2d'} "
                              f"{'TOPS' if dtype == 'i8' else 'TFLOPS'}",
                    "value": round(tops, 2), "unit": "TOPS" if dtype == "i8" else "TFLOPS",
                    "ms_per_step": round(ms, 4), "dtype": dtype, "config": {"workload": desc, "tile": tile_str(c.info)},
                    "roofline": mfma_roofline(dtype, c.macs, kms, TRAFFIC.get(wlname))})
        out["roofline"]["algorithmic_bytes"] = c.bytes
        out["roofline"]["kernel_us"] = round(kms * 1e3, 2)

    if not args.no_others and not args.step_only:
        def add(name, dtype, macs, byts, ms, info, extra=None):
            tops = 2.0 * macs / (ms * 1e-3) / 1e12
            e = {"workload": name, "dtype": dtype, "us": round(ms * 1e3, 2), "value": round(tops, 2),
                 "unit": "TOPS" if dtype in ("i8", "u8i8") else "TFLOPS",
                 "frac_mfma_peak": round(tops / PEAK[dtype], 4),
                 "GBps": round(byts / (ms * 1e-3) / 1e9, 1), "tile": tile_str(info)}
            if extra:
                e.update(extra)
            others.append(e)

        for dtype in ("i8", "f16"):
            g = GemmCase(torch, unit, wl, 4096, 4096, 4096, dtype)
            add("gemm 4096^3", dtype, g.macs, g.bytes, event_ms(torch, g.run, 30), g.info)
            # the same launch on constant operands (all ones): what the kernel does when the operands' switching
            # activity does not pull the clock down (the benchmark's operands are the uniformly random ones above)
            g.A.fill_(1 if dtype == "i8" else 0x3c00)
            g.B.fill_(1 if dtype == "i8" else 0x3c00)
            add("gemm 4096^3, constant operands (all ones)", dtype, g.macs, g.bytes, event_ms(torch, g.run, 30), g.info)
            del g
            c = ConvCase(torch, unit, wl, wl.LARGE_CONV, 32, dtype, 9, 0)
            add("large conv N=32 C=K=256 56x56 3x3, kernel only", dtype, c.macs, c.bytes, event_ms(torch, c.conv, 20), c.info)
            add("large conv N=32 C=K=256 56x56 3x3, pack_act + conv", dtype, c.macs, c.bytes, event_ms(torch, c.api, 20), c.info)
            del c
            torch.cuda.empty_cache()
        for dtype in ("i8", "f16"):                # the same kernel on a problem of four workgroup rounds
            g = GemmCase(torch, unit, wl, 8192, 8192, 8192, dtype)
            add("gemm 8192^3", dtype, g.macs, g.bytes, event_ms(torch, g.run, 5), g.info)
            del g
            torch.cuda.empty_cache()
        for dtype in ("u8i8", "bf16", "fp8"):      # further operand types through the same kernel
            g = GemmCase(torch, unit, wl, 4096, 4096, 4096, dtype)
            add("gemm 4096^3", dtype, g.macs, g.bytes, event_ms(torch, g.run, 30), g.info)
            del g
        c = ConvCase(torch, unit, wl, wl.CONFIG1, 1, "i8", 1, 0)
        add("config 1: conv 1x64x56x56 * 64x64x3x3, kernel only", "i8", c.macs, c.bytes, event_ms(torch, c.conv, 200), c.info)
        add("config 1, pack_act + conv", "i8", c.macs, c.bytes, event_ms(torch, c.api, 200), c.info)
        g = GemmCase(torch, unit, wl, 1, 1000, 2048, "i8")
        add("gemm FC 1x1000x2048", "i8", g.macs, g.bytes, event_ms(torch, g.run, 200), g.info)
        if wlname != "resnet50_f16_b16":
            r = run_conv_set("f16", 16, 4, 20, 3, cold=False)
            t_roof = sum(l["roof_us"] * l["x"] for l in r["per_layer"]) / 1e3
            others.append({"workload": "53 ResNet-50-shaped conv layers, batch 16, fp16->fp32, one unit_conv2d_wpacked_f16 call per layer",
                           "dtype": "f16", "ms": round(r["ms"], 3), "event_ms": round(r["event_ms"], 3),
                           "value": round(2.0 * r["macs"] / (r["ms"] * 1e-3) / 1e12, 2), "unit": "TFLOPS",
                           "GBps": round(r["bytes"] / (r["event_ms"] * 1e-3) / 1e9, 1),
                           "roofline_ms": round(t_roof, 4), "frac_of_per_layer_roofline": round(t_roof / r["event_ms"], 4),
                           "packed_path_kernel_only_ms": round(r["t_conv"], 3), "packed_path_pack_act_ms": round(r["t_pack"], 3)})
        from paper_2101_08458_amd.resnet18_int8 import ResNet18Int8, random_params
        for batch in (1, 8):
            net = ResNet18Int8(batch, random_params(wl.rng(5, batch)))
            xin = torch.from_numpy(wl.int8_activations(wl.rng(5, 100 + batch), (batch, 3, 224, 224))).to("cuda:0")
            ms = wall_ms(torch, lambda: net.forward(xin), 50, 5)
            others.append({"workload": f"ResNet-18-shaped chained int8 inference, batch {batch} (HIP graph replay)",
                           "dtype": "i8", "ms": round(ms, 4), "images_per_s": round(batch / ms * 1e3, 1),
                           "value": round(2.0 * 1.8136e9 * batch / (ms * 1e-3) / 1e12, 2), "unit": "TOPS"})
            del net
        out["others"] = others
        # register-resident MFMA loop: the rate the matrix units sustain on this machine, on this kind of data
        out["mfma_ceiling"] = mfma_ceiling(torch, unit)
        ceil = {c["dtype"]: c["value"] for c in out["mfma_ceiling"] if c["operands"] == "random" and c["steps"] < 1000}
        for e in others:
            if e.get("workload", "") == "gemm 4096^3" and e["dtype"] in ceil:
                e["frac_of_measured_mfma_ceiling"] = round(e["value"] / ceil[e["dtype"]], 4)

    if not args.no_cpu and not args.step_only:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
