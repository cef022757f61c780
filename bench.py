#!/usr/bin/env python3
"""Benchmark of the VISTA hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--calibrate] [--legs a,b,...]
    (defaults: K = 200, W = 20, every leg)

One step = one pass of the hot path over one synthetic batch.  The headline leg is
  stage 1  vista_summarize on the jagged-batch workload (64 users, lognormal
           lengths with median 8k clipped to [1k, 100k], d=128, 4 heads, S=256, bf16),
`value` = history items summarized per second.  The same JSON line carries, under keys of
their own, the other legs (each timed over its own K steps, K scaled down for the long ones):
  stage2     vista_target_attend on the serving workload (1024 users x 512 candidates over
             S=256 cached bf16 summaries, d=128, 4 heads): candidate scores per second;
  lifelong   stage 1 on 8 users x 1,000,000 items (split-L merge);
  end_to_end 256 users, lengths U[10k,100k], two stacked layers (d=256, 8 heads, S=512) with
             the gated block between, then 256 candidates per user: per call and end to end;
  silu, qla  stage 1 with the SiLU score form / quasi-linear attention on the jagged batch;
  qla_backward  gradients of quasi-linear attention on the jagged batch (dQ, dK, dV);
  stage2_q8  stage 2 on int8-quantized summaries (the cache codec), serving workload.
`calibration` holds what this machine sustains, measured in the same run with the instructions
the kernels are made of (matrix-pipe rate and the shader clock it implies, HBM read
bandwidth, issue cost of v_exp_f32 / v_cvt_pk / v_add / MFMA, LDS operand reads, and the
register-only body of the stage-1 tile loop): every roofline gets `peak_measured` beside
the datasheet `peak`.  --calibrate prints the full table to stderr.
Inputs are resident in HBM before the timed region; times are medians over per-step HIP
event pairs recorded on the stream the kernels are launched on (`ms_per_step`), the headline
value divides by the mean over exactly K steps.  Prints ONE JSON line.
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

import numpy as np
import torch

from paper_2510_22049_amd import binding as V
from paper_2510_22049_amd import inputs as I

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA (datasheet)
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E (datasheet)
SIMDS = 256 * 4
CAL_LIB = os.path.join(ROOT, "paper_2510_22049_amd", "libvista_calibrate.so")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.txt")


def traffic_from_profiles(path: str = TRAFFIC_FILE):
    """HBM bytes per launch of the dominant kernels on the default workloads, from the committed
    rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each scaled by what the
    same counter reads for a copy of known size: the factors are in that file).  Returns
    {kernel: bytes} or {} when the file is missing."""
    out = {}
    try:
        text = open(path).read()
    except OSError:
        return out
    ff = re.search(r"FETCH_SIZE [\d.]+ \(true [\d.]+\) -> factor ([\d.]+)", text)
    wf = re.search(r"WRITE_SIZE [\d.]+ -> factor ([\d.]+)", text)
    if not ff or not wf:
        return out
    ffac, wfac = float(ff.group(1)), float(wf.group(1))
    for m in re.finditer(r"^(\w+)\s+([\d.]+)\s+[\d.]+\s+([\d.]+)\s+[\d.]+\s", text, re.M):
        out[m.group(1)] = (float(m.group(2)) * ffac + float(m.group(3)) * wfac) * 1024
    return out


def bf16_dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(x).cuda().to(torch.bfloat16)


SETTLE_S = 0.3   # untimed run-in per leg, see time_steps


def time_steps(fn, steps: int, warmup: int):
    """(mean, median) milliseconds per step over exactly `steps` launches; HIP events on the launch stream.

    Coming out of idle the chip runs through a power-management transient: the first hundred or so
    launches of these kernels take up to 25 % longer than the sustained rate they settle at.  The
    number of interest is the sustained one, so the step is first run untimed for SETTLE_S seconds,
    then come the `warmup` untimed steps and the `steps` timed ones."""
    t0 = time.perf_counter()
    while SETTLE_S > 0 and time.perf_counter() - t0 < SETTLE_S:
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    s = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record(s)
    for i in range(steps):
        fn()
        ev[i + 1].record(s)
    torch.cuda.synchronize()
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])
    return ev[0].elapsed_time(ev[steps]) / steps, float(np.median(per))


# ----------------------------------------------------------------- calibration

CAL_MODES = {"exp16": 0, "add16": 1, "cvt8_add8": 2, "exp16_add16": 3, "mfma4": 4, "mfma4_add16": 5, "mfma4_add32": 6,
             "mfma4_add48": 7, "mfma4_add64": 8, "mfma4_exp16": 9, "mfma16x4": 10, "mfma16x4_add32": 11,
             "mfma4_agpr_add32": 12, "mfma4x4x4_16": 13, "mfma4x4x4_16_add32": 14, "tile_body2": 15,
             "tile_body2_no_small": 16, "tile_body2_no_proj": 17, "tile_body2_loose_deps": 18,
             "tile_body2_lds": 19, "tile_body2_lds_barrier": 20, "tile_body2_lds_barrier_publish": 21}


def calibrate(full: bool):
    """Runs the calibration kernels (include/vista_calibrate.h); clocks are per SIMD at two waves each."""
    L = C.CDLL(CAL_LIB)
    L.vista_calibrate_issue.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    L.vista_calibrate_lds_read.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    L.vista_calibrate_stream_read.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    sink = torch.zeros(4096, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    iters = 20000

    def best(f, reps=4):
        if f() != 0:
            raise RuntimeError("calibration launch failed")
        torch.cuda.synchronize()
        t = 1e9
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            f()
            e1.record()
            torch.cuda.synchronize()
            t = min(t, e0.elapsed_time(e1))
        return t * 1e-3

    def issue(mode, w=2):
        return best(lambda: L.vista_calibrate_issue(CAL_MODES[mode], w, iters, sink.data_ptr(), st)) / iters

    for _ in range(20):                                   # bring the clocks up
        issue("mfma4")
    t_mfma = issue("mfma4")                               # 2 waves x 4 MFMAs of 32 clocks per SIMD and iteration
    clock = 2 * 4 * 32 / t_mfma / 1e9
    cal = {"mfma_tflops": 2 * 4 * 32768 * SIMDS / t_mfma / 1e12, "clock_ghz_from_mfma": clock,
           "note": "issue costs in shader clocks per wave-instruction with two waves per SIMD; the clock is the one "
                   "the MFMA-only loop implies (32 clocks per 32x32x16 MFMA); under the hot kernels' mix of MFMA and "
                   "vector work the part sustains less (see profiles/)"}
    clk = lambda t: t * clock * 1e9                       # seconds -> clocks
    add = clk(issue("add16")) / 32
    cal["v_add_f32"] = add
    cal["v_exp_f32"] = clk(issue("exp16")) / 32
    cal["v_exp_f32_beside_adds"] = (clk(issue("exp16_add16")) - 32 * add) / 32
    cal["v_cvt_pk_bf16_f32"] = (clk(issue("cvt8_add8")) - 16 * add) / 16
    a32, a64 = clk(issue("mfma4_add32")), clk(issue("mfma4_add64"))
    per_add = (a64 - a32) / 64
    cal["mfma_32x32x16_issue"] = (a64 - 128 * per_add) / 8
    cal["mfma_4x4x4_issue"] = (clk(issue("mfma4x4x4_16_add32")) - 64 * per_add) / 32
    # per iteration each of the SIMD's two waves works through two query blocks
    cal["stage1_block_clocks_per_simd"] = clk(issue("tile_body2")) / 4
    cal["lds_read_bytes_per_clock_cu"] = 8 * 16 * 1024 / clk(
        best(lambda: L.vista_calibrate_lds_read(0, 2, iters, sink.data_ptr(), st)) / iters)
    x = torch.empty(1 << 31, dtype=torch.uint8, device="cuda")
    x.fill_(1)
    t_rd = best(lambda: L.vista_calibrate_stream_read(x.data_ptr(), x.numel(), sink.data_ptr(), st), reps=6)
    cal["hbm_read_gbs"] = x.numel() / t_rd / 1e9
    del x
    if full:
        for w in (1, 2, 3, 4):
            for name in CAL_MODES:
                sys.stderr.write(f"calibrate: {name:22s} {w} waves/SIMD: {clk(issue(name, w)):8.1f} clocks per SIMD-iteration\n")
    return cal


# ----------------------------------------------------------------- workloads

def stage1_workload(sets: int):
    c = I.CONFIGS[2]
    lens = I.lengths(c)
    off = I.offsets_from_lengths(lens)
    N = int(off[-1])
    Q, Wk, Wv = I.virtual_queries(c), I.projection(c, "W_k"), I.projection(c, "W_v")
    X = I.history(c, lens)
    dev = dict(off=torch.from_numpy(off).cuda(), off_host=torch.from_numpy(off), Q=bf16_dev(Q),
               Wk=bf16_dev(Wk), Wv=bf16_dev(Wv))
    # distinct copies of the history so consecutive steps do not re-read a cache-resident buffer
    xs = [bf16_dev(X)]
    for _ in range(sets - 1):
        xs.append(xs[0].clone())
    outs = [torch.empty((c.B, c.S, c.d), device="cuda", dtype=torch.bfloat16) for _ in range(sets)]
    host = dict(X=X, off=off, Q=Q, Wk=Wk, Wv=Wv, lens=lens)
    return c, N, dev, xs, outs, host


def device_history(c, lens, seed):
    """Packed bf16 history drawn on the device (~N(0,1)); the long workloads are not built on the host."""
    off = I.offsets_from_lengths(lens)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    X = torch.empty((int(off[-1]), c.d), device="cuda", dtype=torch.bfloat16)
    step = 1 << 20
    for i in range(0, X.shape[0], step):
        X[i:i + step] = torch.randn((min(step, X.shape[0] - i), c.d), device="cuda", generator=g)
    return X, off


def cpu_baseline(host, c, budget_s: float = 12.0):
    """The numpy oracle, as it stands, on a bounded sample of the stage-1 workload."""
    from oracle import vista_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    order = np.argsort(host["lens"])            # shortest users first so the sample is bounded
    items, users, t0 = 0, 0, time.perf_counter()
    while time.perf_counter() - t0 < budget_s:  # whole passes over the users until the budget is spent
        for b in order:
            lo, hi = host["off"][b], host["off"][b + 1]
            O.summarize(host["X"][lo:hi], [0, hi - lo], host["Q"], host["Wk"], host["Wv"], c.H)
            items += int(hi - lo)
            users += 1
            if time.perf_counter() - t0 > budget_s:
                break
    dt = time.perf_counter() - t0
    return {"value": items / dt, "unit": "items/s", "cores": int(cores), "kind": "oracle",
            "sample": f"stage 1, {users} user histories of the jagged-batch workload (passes over the 64 users, "
                      f"shortest first), {items} items in {dt:.1f} s (fp64 numpy oracle)"}


def mfma_roofline(flop_item, items_per_s, cal, **extra):
    tf = flop_item * items_per_s / 1e12
    r = {"bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS,
         "flop_per_item": flop_item}
    if cal:
        r["peak_measured"] = cal["mfma_tflops"]
        r["frac_of_measured"] = tf / cal["mfma_tflops"]
    r.update(extra)
    return r


def hbm_roofline(bytes_unit, units_per_s, cal, **extra):
    gbs = bytes_unit * units_per_s / 1e9
    r = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
    if cal:
        r["peak_measured"] = cal["hbm_read_gbs"]
        r["frac_of_measured"] = gbs / cal["hbm_read_gbs"]
    r.update(extra)
    return r


def main() -> None:
    global SETTLE_S
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--settle-seconds", type=float, default=SETTLE_S,
                    help="untimed run-in per leg before the warm-up steps (0 for counter-collection runs)")
    ap.add_argument("--segment-items", type=int, default=0)
    ap.add_argument("--calibrate", action="store_true", help="print the full calibration table to stderr")
    ap.add_argument("--no-calibration", action="store_true", help="skip the calibration kernels")
    ap.add_argument("--legs", default="stage1,stage2,stage2_q8,lifelong,end_to_end,silu,qla,qla_backward",
                    help="comma-separated legs to run (stage1 always runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known traffic for scaling HBM counters)")
    a = ap.parse_args()
    SETTLE_S = a.settle_seconds
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    V.lib()
    torch.cuda.set_device(0)
    legs = set(a.legs.split(","))
    SETS = 4
    if a.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    cal = None if a.no_calibration else calibrate(a.calibrate)
    traffic = traffic_from_profiles()
    few = max(5, a.steps // 10)            # steps of the long legs (a step there takes milliseconds)

    # ------------------------------------------------------------- stage 1 (headline)
    c1, N, dev, xs, outs, host = stage1_workload(SETS)
    desc1 = V.summarize_desc(c1.B, c1.S, c1.d, c1.H, V.VISTA_BF16, N, segment_items=a.segment_items)
    ws = torch.empty(V.vista_summarize_workspace_bytes(desc1), dtype=torch.uint8, device="cuda")
    it = {"i": 0}

    def step1(attn=V.VISTA_ATTN_SOFTMAX, wsp=None):
        k = it["i"] % SETS
        it["i"] += 1
        V.vista_summarize(xs[k], dev["off"], dev["Q"], dev["Wk"], dev["Wv"], outs[k], H=c1.H,
                          offsets_host=dev["off_host"], workspace=wsp if wsp is not None else ws,
                          segment_items=a.segment_items, attn=attn)

    ms1, med1 = time_steps(step1, a.steps, a.warmup)
    items_per_s = N / (ms1 * 1e-3)
    flop_item = 4 * c1.d * c1.d + 4 * c1.S * c1.d          # K,V projection + QK^T + PV, per item
    ceiling = None
    if cal:   # what the tile loop's own instructions allow: 8 query blocks per SIMD and 32-item tile
        ceiling = 32 * 256 / (8 * cal["stage1_block_clocks_per_simd"]) * cal["clock_ghz_from_mfma"] * 1e9
    res = {
        "metric": "history items summarized/sec (stage 1, S=256) + candidate scores/sec (stage 2)",
        "value": items_per_s, "unit": "items/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms1, "ms_per_step_median": med1, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "stage-1 jagged batch: 64 users, lognormal lengths (median 8k, [1k,100k]), "
                               "d=128, 4 heads, S=256, bf16", "total_items": N,
                   "segment_items": V.vista_summarize_segment_items(desc1)},
        "roofline": mfma_roofline(
            flop_item, items_per_s, cal, traffic=traffic.get("summarize_mfma"),
            traffic_source="profiles/hbm_traffic_pmc.txt (default segment size)" if traffic else None,
            kernel="summarize_mfma_kernel<128,4,4,softmax>", algorithmic_bytes=N * c1.d * 2,
            note="duration = one whole vista_summarize call (summarize_mfma + merge kernels, HIP events on the "
                 "launch stream); the kernel-only average is in profiles/",
            co_bound={"bound": "alu", "what": "the tile loop's own instruction mix, registers only (per query block "
                                             "6 MFMAs, 16 v_exp_f32, 8 v_cvt_pk_bf16_f32, 4 4x4x4 MFMAs), measured "
                                             "by the calibration kernel at the MFMA-loop clock",
                      "achieved": items_per_s, "peak": ceiling, "unit": "items/s",
                      "frac": items_per_s / ceiling if ceiling else None, "exp_per_item": c1.S * c1.H}),
    }
    if cal:
        res["calibration"] = cal

    # ------------------------------------------------------------- SiLU score form / quasi-linear attention
    for leg, attn in (("silu", V.VISTA_ATTN_SILU), ("qla", V.VISTA_ATTN_QLA)):
        if leg not in legs:
            continue
        d_ = V.summarize_desc(c1.B, c1.S, c1.d, c1.H, V.VISTA_BF16, N, attn=attn, segment_items=a.segment_items)
        w_ = torch.empty(V.vista_summarize_workspace_bytes(d_), dtype=torch.uint8, device="cuda")
        ms, med = time_steps(lambda: step1(attn, w_), a.steps, a.warmup)
        ips = N / (ms * 1e-3)
        if leg == "silu":
            roof = mfma_roofline(flop_item, ips, cal, kernel="summarize_mfma_kernel<128,4,4,silu>",
                                 note="same flop count as the softmax form; two transcendentals per score (2^t, 1/x)")
        else:
            fl = 4 * c1.d * c1.d + 4 * c1.d * (c1.d // c1.H)       # projections + SiLU(K)^T V per head
            roof = hbm_roofline(2 * c1.d, ips, cal, kernel="qla_state_mfma_kernel<128>", bytes_per_item=2 * c1.d,
                                flop_per_item=fl, mfma_tflops=fl * ips / 1e12,
                                note="state stream: X read once (2d bytes per item); the finishing kernel is O(B S d)")
        res[leg] = {"value": ips, "unit": "items/s", "ms_per_step": ms, "ms_per_step_median": med,
                    "config": {"workload": f"stage-1 jagged batch, attn={leg}"}, "roofline": roof}
    if "qla_backward" in legs:
        dO = torch.randn((c1.B, c1.S, c1.d), device="cuda").to(torch.bfloat16)
        dQ = torch.empty_like(dO)
        dK, dV = torch.empty_like(xs[0]), torch.empty_like(xs[0])
        wb = V.vista_qla_backward(xs[0], dev["off"], dev["Q"], dev["Wk"], dev["Wv"], dO, dQ, dK, dV, H=c1.H,
                                  offsets_host=dev["off_host"])
        kb = {"i": 0}

        def stepb():
            k = kb["i"] % SETS
            kb["i"] += 1
            V.vista_qla_backward(xs[k], dev["off"], dev["Q"], dev["Wk"], dev["Wv"], dO, dQ, dK, dV, H=c1.H,
                                 offsets_host=dev["off_host"], workspace=wb)

        ms, med = time_steps(stepb, a.steps, a.warmup)
        ips = N / (ms * 1e-3)
        res["qla_backward"] = {"value": ips, "unit": "items/s", "ms_per_step": ms, "ms_per_step_median": med,
                               "config": {"workload": "stage-1 jagged batch, gradients of attn=qla (dQ, dK, dV)"},
                               "roofline": hbm_roofline(6 * c1.d, ips, cal, kernel="qla_bwd_items_mfma_kernel<128>",
                                                        bytes_per_item=6 * c1.d,
                                                        note="X read twice (state pass, item pass) would be 4d; the "
                                                             "algorithmic count is X once + dK and dV written = 6d bytes per item")}
        del dO, dQ, dK, dV, wb
    del xs, outs, ws
    torch.cuda.empty_cache()

    # ------------------------------------------------------------- stage 2
    if "stage2" in legs:
        c2 = I.CONFIGS[4]
        g = torch.Generator(device="cuda")
        g.manual_seed(0)
        cands, summs, outs2 = [], [], []
        for _ in range(SETS):
            cands.append(torch.randn((c2.B, c2.C, c2.d), device="cuda", generator=g).to(torch.bfloat16))
            summs.append(torch.randn((c2.B, c2.S, c2.d), device="cuda", generator=g).to(torch.bfloat16))
            outs2.append(torch.empty((c2.B, c2.C, c2.d), device="cuda", dtype=torch.bfloat16))
        jt = {"i": 0}

        def step2():
            k = jt["i"] % SETS
            jt["i"] += 1
            V.vista_target_attend(cands[k], summs[k], outs2[k], H=c2.H)

        ms2, med2 = time_steps(step2, a.steps, a.warmup)
        cand_per_s = c2.B * c2.C / (ms2 * 1e-3)
        bytes_cand = 2 * c2.d * 2 + c2.S * c2.d * 2 / c2.C       # candidate in + out + summaries amortised
        res["stage2"] = {"value": cand_per_s, "unit": "candidate scores/s", "ms_per_step": ms2, "ms_per_step_median": med2,
                         "config": {"workload": "stage-2 serving: 1024 users x 512 candidates, S=256, d=128, 4 heads, bf16"},
                         "roofline": hbm_roofline(bytes_cand, cand_per_s, cal, traffic=traffic.get("attend_mfma"),
                                                  kernel="attend_mfma_kernel<8>", bytes_per_candidate=bytes_cand,
                                                  exp_per_candidate=c2.S * c2.H)}
        if "stage2_q8" in legs:
            codes = [torch.empty((c2.B, c2.S, c2.d), device="cuda", dtype=torch.int8) for _ in range(SETS)]
            scl = [torch.empty((c2.B, c2.S, c2.H), device="cuda", dtype=torch.float32) for _ in range(SETS)]
            for k in range(SETS):
                V.vista_quantize_summaries(summs[k], codes[k], scl[k], H=c2.H)
            qt = {"i": 0}

            def stepq():
                k = qt["i"] % SETS
                qt["i"] += 1
                V.vista_target_attend_q8(cands[k], codes[k], scl[k], outs2[k], H=c2.H)

            msq, medq = time_steps(stepq, a.steps, a.warmup)
            cps = c2.B * c2.C / (msq * 1e-3)
            bq = 2 * c2.d * 2 + (c2.S * c2.d + 4 * c2.S * c2.H) / c2.C
            res["stage2_q8"] = {"value": cps, "unit": "candidate scores/s", "ms_per_step": msq, "ms_per_step_median": medq,
                                "config": {"workload": "stage-2 serving on int8 summaries (one scale per token and head)"},
                                "roofline": hbm_roofline(bq, cps, cal, kernel="attend_mfma_kernel<8> (int8 slab)",
                                                         bytes_per_candidate=bq)}
            del codes, scl
        del cands, summs, outs2
        torch.cuda.empty_cache()

    # ------------------------------------------------------------- lifelong (8 x 1M items)
    if "lifelong" in legs:
        c3 = I.CONFIGS[3]
        X3, off3 = device_history(c3, I.lengths(c3), 3)
        N3 = int(off3[-1])
        o3 = torch.empty((c3.B, c3.S, c3.d), device="cuda", dtype=torch.bfloat16)
        d3 = V.summarize_desc(c3.B, c3.S, c3.d, c3.H, V.VISTA_BF16, N3)
        w3 = torch.empty(V.vista_summarize_workspace_bytes(d3), dtype=torch.uint8, device="cuda")
        offd3, offh3 = torch.from_numpy(off3).cuda(), torch.from_numpy(off3)
        ms3, med3 = time_steps(lambda: V.vista_summarize(X3, offd3, dev["Q"], dev["Wk"], dev["Wv"], o3, H=c3.H,
                                                        offsets_host=offh3, workspace=w3), few, 3)
        ips3 = N3 / (ms3 * 1e-3)
        res["lifelong"] = {"value": ips3, "unit": "items/s", "ms_per_step": ms3, "ms_per_step_median": med3, "steps": few,
                           "config": {"workload": "stage-1 lifelong: 8 users x 1,000,000 items, d=128, 4 heads, S=256, bf16",
                                      "total_items": N3, "segment_items": V.vista_summarize_segment_items(d3)},
                           "roofline": mfma_roofline(flop_item, ips3, cal)}
        del X3, o3, w3
        torch.cuda.empty_cache()

    # ------------------------------------------------------------- end to end (two layers + gated block + stage 2)
    if "end_to_end" in legs:
        c5 = I.CONFIGS[5]
        X5, off5 = device_history(c5, I.lengths(c5), 5)
        N5 = int(off5[-1])
        offd5, offh5 = torch.from_numpy(off5).cuda(), torch.from_numpy(off5)
        Q0 = bf16_dev(I.virtual_queries(c5))
        W = {k: bf16_dev(I.projection(c5, k[:3], int(k[3]))) for k in ("W_k0", "W_v0", "W_k1", "W_v1")}
        Wg, Wu, Wo = (bf16_dev(w) for w in I.ffn_weights(c5))
        y1 = torch.empty((c5.B, c5.S, c5.d), device="cuda", dtype=torch.bfloat16)
        q1, y2 = torch.empty_like(y1), torch.empty_like(y1)
        g = torch.Generator(device="cuda")
        g.manual_seed(6)
        cand5 = torch.randn((c5.B, c5.C, c5.d), device="cuda", generator=g).to(torch.bfloat16)
        out5 = torch.empty_like(cand5)
        da = V.summarize_desc(c5.B, c5.S, c5.d, c5.H, V.VISTA_BF16, N5)
        db = V.summarize_desc(c5.B, c5.S, c5.d, c5.H, V.VISTA_BF16, N5, per_user_q=True)
        w5 = torch.empty(max(V.vista_summarize_workspace_bytes(da), V.vista_summarize_workspace_bytes(db)),
                         dtype=torch.uint8, device="cuda")
        layer1 = lambda: V.vista_summarize(X5, offd5, Q0, W["W_k0"], W["W_v0"], y1, H=c5.H, offsets_host=offh5, workspace=w5)
        block = lambda: V.vista_sglu_ffn(y1, Wg, Wu, Wo, q1)
        layer2 = lambda: V.vista_summarize(X5, offd5, q1, W["W_k1"], W["W_v1"], y2, H=c5.H, offsets_host=offh5, workspace=w5)
        stage2 = lambda: V.vista_target_attend(cand5, y2, out5, H=c5.H)

        def chain():
            layer1()
            block()
            layer2()
            stage2()

        chain()
        torch.cuda.synchronize()
        fl5 = 4 * c5.d * c5.d + 4 * c5.S * c5.d
        e2e = {"config": {"workload": "end to end: 256 users, lengths U[10k,100k], 2 layers (d=256, 8 heads, S=512) + "
                                      "SiLU-gated block (d_ff=512), then 256 candidates per user; bf16",
                          "total_items": N5}, "steps": few}
        for name, fn in (("layer1", layer1), ("gated_block", block), ("layer2", layer2), ("stage2", stage2), ("chain", chain)):
            ms, med = time_steps(fn, few, 2)
            e2e[name] = {"ms_per_step": ms, "ms_per_step_median": med}
        for name in ("layer1", "layer2"):
            ips = N5 / (e2e[name]["ms_per_step"] * 1e-3)
            e2e[name].update(value=ips, unit="items/s", roofline=mfma_roofline(fl5, ips, cal))
        e2e["value"] = N5 / (e2e["chain"]["ms_per_step"] * 1e-3)
        e2e["unit"] = "items/s through the whole chain"
        e2e["stage2"].update(value=c5.B * c5.C / (e2e["stage2"]["ms_per_step"] * 1e-3), unit="candidate scores/s")
        res["end_to_end"] = e2e
        del X5, y1, y2, q1, cand5, out5, w5
        torch.cuda.empty_cache()

    if not a.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(host, c1)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
