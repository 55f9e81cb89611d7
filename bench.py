#!/usr/bin/env python3
"""Benchmark of the partitioned FFN/MoE layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]                      all five workload shapes, one JSON line
    python bench.py --config mixtral_8x7b [--split r_gg,r_cg,r_cc] ...       one shape at one split (profiling runs)

A *step* is one pass of the whole hot path over one batch of synthetic input: one prompt-phase
call (T = the config's prefill length) followed by ``--decode-calls`` generation-phase calls of
the config's decode batch, each on different tokens (so that decode calls touch different experts
and no weight byte is served from the 256 MB Infinity Cache).  Inputs are resident in HBM before
the timed region.

Without --config the run covers every workload shape at full size in one process.  The headline
(``value``, ``ms_per_step``, ``roofline``, ``cpu_baseline``) is the largest one, the Mixtral-8x22B-shaped
layer with all weights resident, timed over exactly K steps after W warm-up steps; ``configs`` holds one
entry per shape and quoted split (the PhiMoE- and Mixtral-8x22B-shaped layers: all seven splits of the
sweep 100/0/0 ... 20/60/20) with the step time, tokens/s per phase, every weight kernel against its
roofline, host-link rate, overlap and the Eq. 6 prediction next to the measured call time; those
entries are timed over min(K, 3) steps of min(decode calls, 4) decode calls each.

The printed JSON line carries
  value / ms_per_step   whole-step throughput of the headline workload
  roofline              its dominant kernel (most GPU time in the step) against its roofline; kernel
                        time from HIP events recorded by the library around every launch
  configs               see above
  cpu_baseline          the CPU oracle timed on this machine's host cores on a bounded token sample
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
MFMA_BF16_PEAK_TF = 2500.0  # dense bf16
HEADLINE = "mixtral_8x22b"
TIMER_NOTE = ("kernel time = HIP events recorded by the library on the launch stream around each launch, in a repeat of "
              "the timed region (an event pair adds about 3 us of launch gap to a kernel's rocprofv3 duration)")


def load_pmc_traffic():
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE, each scaled by what the same
    counter reads for a plain copy of known size): the table rows of profiles/hbm_traffic_table.md, keyed by
    (config, split, kernel class).  Kernels that were not profiled report traffic = null."""
    out = {}
    path = os.path.join(ROOT, "profiles", "hbm_traffic_table.md")
    if not os.path.exists(path):
        return out
    for ln in open(path):
        m = re.match(r"\|\s*(\w+)\s*\|\s*([\d.]+)/([\d.]+)/([\d.]+)\s*\|\s*(\w+)\s*\|\s*([\d.]+)\s*\|\s*([\d.]+)\s*\|", ln)
        if m:
            split = tuple(round(float(m.group(i)) / 100.0, 4) for i in (2, 3, 4))
            # FETCH_SIZE counts half the bytes of a plain copy (factor 2.0), WRITE_SIZE all of them (factor 1.0)
            out[(m.group(1), split, m.group(5))] = (2.0 * float(m.group(6)) + float(m.group(7))) * 1024.0
    return out


PMC_TRAFFIC = load_pmc_traffic()


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default=None,
                    help="one workload shape only (tiny_dense, mixtral_8x7b, llama2_70b, qwen_moe, phimoe, mixtral_8x22b); "
                         "default: all five full-size shapes, headline on the Mixtral-8x22B-shaped layer")
    ap.add_argument("--split", default=None, help="r_gg,r_cg,r_cc (default: the config's)")
    ap.add_argument("--decode-calls", type=int, default=16)
    ap.add_argument("--n-g", type=int, default=-1, help="prefill tokens on CG' (default: all when r_cc > 0)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measurement of this machine's own HBM / MFMA / link peaks")
    ap.add_argument("--no-gg-only", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--q4", action="store_true",
                    help="4-bit weights (codes + bf16 group scales) instead of bf16: same step, same metric")
    ap.add_argument("--deq-mib", type=int, default=0,
                    help="with --q4: 0 = prompt-phase GEMMs convert the codes themselves; > 0 = two passes through a "
                         "bf16 scratch of this many MiB")
    ap.add_argument("--solve", action="store_true",
                    help="instead of the throughput line: profile this machine (Eq. 3), solve r_CG* for the config's "
                         "r_GG and n_g* for its prompt length (Section IV), and measure the layer over a sweep of "
                         "r_CG and of n_g next to the solved values")
    ap.add_argument("--place", action="store_true",
                    help="instead of the throughput line: whole-expert placement against uniform slicing at equal GPU "
                         "memory (MoE configs), decode calls of the config, bytes streamed and call time")
    ap.add_argument("--stack", type=int, default=0,
                    help="instead of the throughput line: a stack of this many layers of the config's shape under GPU-memory "
                         "budgets of 25/50/75 %% of its weights; greedy per-layer r_GG (Section IV-A.4) against the same "
                         "r_GG for every layer, decode step measured with and without cross-layer prefetch")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the throughput line: the config's layer moved through the GG/CG/CC sweep of the "
                         "PhiMoE / Mixtral-8x22B workloads (100/0/0 ... 20/60/20) with si_layer_resplit; per split the "
                         "prompt-phase and generation-phase call times, link rate and overlap")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run a plain elementwise copy of 1 GiB (reads 1 GiB, writes 1 GiB) three times: "
                         "the reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


class Workload:
    """Device-resident inputs of one step and the per-call routing facts needed for byte counts."""

    def __init__(self, cfg, n_decode, oracle_route=None):
        import torch
        import synth
        self.cfg = cfg
        dev = torch.device("cuda:0")
        self.xp_bits = synth.make_tokens(cfg, cfg.t_prefill)
        self.lp = synth.make_router_logits(cfg, self.xp_bits)
        self.xp = torch.from_numpy(self.xp_bits.view(np.int16)).to(dev)
        self.lp_dev = torch.from_numpy(self.lp).to(dev) if self.lp is not None else None
        self.yp = torch.empty((cfg.t_prefill, cfg.d_model), dtype=torch.float32, device=dev)
        self.dec = []
        for i in range(n_decode):
            xb = synth.make_tokens(cfg, cfg.t_decode, stream=100 + i)
            lg = synth.make_router_logits(cfg, xb)
            self.dec.append((torch.from_numpy(xb.view(np.int16)).to(dev),
                             torch.from_numpy(lg).to(dev) if lg is not None else None, lg))
        self.yd = torch.empty((cfg.t_decode, cfg.d_model), dtype=torch.float32, device=dev)

    @staticmethod
    def touched(cfg, logits):
        """Number of routed experts with at least one token (host arithmetic on the inputs only)."""
        if logits is None:
            return 1
        order = np.argsort(-logits, axis=1, kind="stable")[:, :cfg.top_k]
        return len(np.unique(order))


def run_steps(si, layer, wl, n_steps, n_g, stream, collect=None):
    cfg = wl.cfg
    for _ in range(n_steps):
        si.si_layer_forward(layer, wl.xp.data_ptr(), wl.lp_dev.data_ptr() if wl.lp_dev is not None else None,
                            cfg.t_prefill, n_g, si.SI_PREFILL, wl.yp.data_ptr(), stream=stream)
        if collect is not None:
            collect.append(("prefill", si.si_layer_stats(layer)))
        for xd, ld, _ in wl.dec:
            si.si_layer_forward(layer, xd.data_ptr(), ld.data_ptr() if ld is not None else None, cfg.t_decode, 0,
                                si.SI_DECODE, wl.yd.data_ptr(), stream=stream)
            if collect is not None:
                collect.append(("decode", si.si_layer_stats(layer)))


def create_layer(si, cfg, w, split):
    if "q_gate" in w:
        return si.si_layer_create_q4(cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k, w, split[0], split[1], split[2],
                                     max(cfg.t_prefill, cfg.t_decode), d_ff_shared=cfg.d_ff_shared, deq_mib=DEQ_MIB)
    shared = tuple(w[k] for k in ("s_gate", "s_up", "s_down")) if cfg.d_ff_shared else None
    return si.si_layer_create(cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k, w["w_gate"], w["w_up"], w["w_down"],
                              split[0], split[1], split[2], max(cfg.t_prefill, cfg.t_decode),
                              d_ff_shared=cfg.d_ff_shared, shared=shared)


def measure_layer(si, torch, layer, wl, steps, warmup, n_g):
    """Time `steps` steps (profiling off), then repeat them with per-launch events for kernel times."""
    cfg = wl.cfg
    info = si.si_layer_split_info(layer)
    stream = torch.cuda.current_stream().cuda_stream
    run_steps(si, layer, wl, warmup, n_g, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(si, layer, wl, steps, n_g, stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # per-phase call time without any event inside the library (back-to-back calls, one sync)
    reps = max(2, steps)
    t1 = time.perf_counter()
    for _ in range(reps):
        for xd, ld, _lg in wl.dec:
            si.si_layer_forward(layer, xd.data_ptr(), ld.data_ptr() if ld is not None else None, cfg.t_decode, 0,
                                si.SI_DECODE, wl.yd.data_ptr(), stream=stream)
    torch.cuda.synchronize()
    t_dec = (time.perf_counter() - t1) / (reps * len(wl.dec))
    t1 = time.perf_counter()
    for _ in range(reps):
        si.si_layer_forward(layer, wl.xp.data_ptr(), wl.lp_dev.data_ptr() if wl.lp_dev is not None else None,
                            cfg.t_prefill, n_g, si.SI_PREFILL, wl.yp.data_ptr(), stream=stream)
    torch.cuda.synchronize()
    t_pre = (time.perf_counter() - t1) / reps
    # same region again with HIP events around every launch (stream-ordered, on the launch stream)
    si.si_layer_set_profiling(layer, 1)
    stats = []
    run_steps(si, layer, wl, steps, n_g, stream, collect=stats)
    torch.cuda.synchronize()
    si.si_layer_set_profiling(layer, 0)
    return elapsed, stats, info, {"decode_call_us": 1e6 * t_dec, "prefill_call_us": 1e6 * t_pre}


def measure(si, torch, cfg, w, split, wl, steps, warmup, n_g):
    layer = create_layer(si, cfg, w, split)
    try:
        return measure_layer(si, torch, layer, wl, steps, warmup, n_g)
    finally:
        si.si_layer_destroy(layer)


def kernel_table(si, cfg, info, wl, stats, steps, n_g, q4=False):
    """Per kernel class: launches, mean duration, algorithmic bytes / flops per step, achieved rates.

    Algorithmic work (weight bytes are read once per call, bf16):
      decode gateup : touched experts x part columns x M x 2 matrices x 2 B
      decode down   : touched experts x part columns x M x 2 B
      prefill gateup: (token, expert) pairs x part columns x M x 4 flop ; weight bytes as above
      prefill down  : pairs x part columns x M x 2 flop
    Columns of the CC part count only when they run on the GPU (CG', the n_g tokens of X2).
    4-bit weights: every kernel reads 0.5 B of codes + 2/64 B of scales per weight; with --deq-mib > 0 the prefill
    GEMMs read the bf16 copies made by the dequantisation kernel instead (whose time is in the "fill" class)."""
    wb_dec = 0.5 + 2.0 / 64 if q4 else 2.0
    wb_pre = wb_dec if (q4 and DEQ_MIB == 0) else 2.0
    M, H, Hs, k = cfg.d_model, cfg.d_ff, cfg.d_ff_shared, cfg.top_k
    gpu_cols = info["n_gg"] + info["n_cg"]
    gpu_cols_s = info["s_gg"] + info["s_cg"]
    T = cfg.t_prefill
    # decode: per call, touched experts
    dec_bytes_gu = dec_bytes_dn = 0.0
    for _, _, lg in wl.dec:
        nt = Workload.touched(cfg, lg)
        dec_bytes_gu += (nt * gpu_cols + gpu_cols_s) * M * 2 * wb_dec
        dec_bytes_dn += (nt * gpu_cols + gpu_cols_s) * M * wb_dec
    ntp = Workload.touched(cfg, wl.lp)
    cc_cols_gpu = info["n_cc"] if n_g > 0 else 0
    cc_cols_gpu_s = info["s_cc"] if n_g > 0 else 0
    pre_w_gu = (ntp * (gpu_cols + cc_cols_gpu) + gpu_cols_s + cc_cols_gpu_s) * M * 2 * wb_pre
    pre_w_dn = pre_w_gu / 2
    pairs = T * k
    flop_gu = (pairs * gpu_cols + T * gpu_cols_s + n_g * k * info["n_cc"] + n_g * info["s_cc"]) * M * 4.0
    flop_dn = flop_gu / 2
    work = {"decode_gateup": ("hbm", dec_bytes_gu, 0.0), "decode_down": ("hbm", dec_bytes_dn, 0.0),
            "prefill_gateup": ("mfma", pre_w_gu, flop_gu), "prefill_down": ("mfma", pre_w_dn, flop_dn)}
    # activations a prompt-phase GEMM reads and writes once: x rows in (bf16), Hact out (bf16); Hact in, per-row outputs (fp32) out
    rows_cols = flop_gu / (4.0 * M)  # sum over launches of rows x hidden columns
    n_rows = pairs + (T if Hs else 0)
    act = {"prefill_gateup": n_rows * M * 2.0 + rows_cols * 2.0, "prefill_down": rows_cols * 2.0 + n_rows * M * 4.0}
    ms = np.zeros(8)
    launches = np.zeros(8, dtype=np.int64)
    for _, st in stats:
        ms += np.array(st["kernel_ms"])
        launches += np.array(st["kernel_launches"])
    out = {}
    for i, name in enumerate(si.SI_K_NAMES):
        if launches[i] == 0:
            continue
        ent = {"launches_per_step": float(launches[i]) / steps, "ms_per_step": float(ms[i]) / steps,
               "avg_launch_us": 1e3 * float(ms[i]) / float(launches[i])}
        if name in work:
            bound, nbytes, nflop = work[name]
            sec = ms[i] / steps / 1e3
            ent["bytes_per_step"] = nbytes
            if name in act:
                ent["act_bytes_per_step"] = act[name]
            ent["GBps"] = nbytes / sec / 1e9
            if nflop:
                ent["flop_per_step"] = nflop
                ent["TFLOPs"] = nflop / sec / 1e12
                # a GEMM whose arithmetic intensity is below the machine balance is bandwidth bound
                ai = nflop / nbytes
                bound = "mfma" if ai >= MFMA_BF16_PEAK_TF * 1e12 / (HBM_PEAK_GBS * 1e9) else "hbm"
            ent["bound"] = bound
        out[name] = ent
    return out


def eq6_prediction(st):
    """Layer time predicted by the timestamp recurrence of Section IV-A.2 (Eq. 6) from the separately measured
    per-resource times of one call: for the n staged pieces
        tau_L^i   = tau_L^(i-1) + t_L
        tau_C2G^i = max(tau_L^i, tau_C2G^(i-1)) + t_C2G
        tau_G^i   = max(tau_C2G^i, tau_G^(i-1)) + t_G
    with tau^0 = the hand-off wait, tau_G^0 additionally the assignment kernels and the resident (GG) part, which
    are enqueued before the first copy is waited for; t_fin = max(tau_G^n + merge, tau_C)."""
    n = st["n_copies"]
    t0 = st["handoff_ms"]
    merge = st["kernel_ms"][3] + st["kernel_ms"][6]
    gg = st["gpu_ms"] - st["staged_ms"] - merge
    tau_c = t0 + st["cc_ms"]
    if n == 0:
        return max(t0 + gg + merge, tau_c)
    t_c2g, t_g = st["copy_ms"] / n, st["staged_ms"] / n
    t_l = max(0.0, st["enqueue_ms"] - st["handoff_ms"] - st["cc_ms"]) / (n + 1)
    tau_l = tau_c2g = t0
    tau_g = t0 + gg
    for _ in range(n):
        tau_l += t_l
        tau_c2g = max(tau_l, tau_c2g) + t_c2g
        tau_g = max(tau_c2g, tau_g) + t_g
    return max(tau_g + merge, tau_c)


DEQ_MIB = 0  # set by main() from --deq-mib
MEASURED_PEAKS = None  # filled by main() from si_measure_peaks(): what the simplest kernels reach on this machine


def roofline_of(name, ent, cfg_name=None, split=None):
    traffic = PMC_TRAFFIC.get((cfg_name, tuple(split) if split is not None else None, name))
    if ent["bound"] == "hbm":
        a, p, unit = ent["GBps"], HBM_PEAK_GBS, "GB/s"
        measured = MEASURED_PEAKS["hbm_read_gbs"] if MEASURED_PEAKS else None
    else:
        a, p, unit = ent["TFLOPs"], MFMA_BF16_PEAK_TF, "TFLOP/s"
        measured = MEASURED_PEAKS["mfma_bf16_tflops"] if MEASURED_PEAKS else None
    out = {"kernel": name, "bound": ent["bound"], "achieved": round(a, 2), "peak": p, "unit": unit,
           "frac": round(a / p, 4), "traffic": traffic, "avg_launch_us": round(ent["avg_launch_us"], 2),
           "launches_per_step": ent["launches_per_step"]}
    if traffic:
        # weight bytes of the launch plus the activations it reads and the outputs it writes once
        algo = (ent["bytes_per_step"] + ent.get("act_bytes_per_step", 0.0)) / ent["launches_per_step"]
        out["algorithmic_bytes_per_launch"] = round(algo, 1)
        out["traffic_over_algorithmic"] = round(traffic / algo, 4)
        out["traffic_note"] = ("FETCH_SIZE counts what the L2 asks of the fabric: re-reads of activation rows that have left the "
                               "L2 are in it although the Infinity Cache, not HBM, serves them")
    if measured:
        out["measured_peak"] = round(measured, 1)
        out["frac_of_measured_peak"] = round(a / measured, 4)
    if ent["bound"] != "hbm" and MEASURED_PEAKS and MEASURED_PEAKS.get("mfma_bf16_random_tflops"):
        # the register-resident matrix loop on operands that look like data (the chip clocks lower on them)
        out["measured_peak_random_operands"] = round(MEASURED_PEAKS["mfma_bf16_random_tflops"], 1)
        out["frac_of_measured_peak_random_operands"] = round(a / MEASURED_PEAKS["mfma_bf16_random_tflops"], 4)
    return out


def cpu_baseline(cfg, w, wl, seconds):
    """The oracle, as it stands, on a bounded sample of the step's tokens (prefill tokens, all routed)."""
    import oracle
    shared = tuple(w[k] for k in ("s_gate", "s_up", "s_down")) if cfg.d_ff_shared and "s_gate" in w else None
    threads = oracle.get_threads()

    def run(n):
        sel = np.linspace(0, cfg.t_prefill - 1, n).astype(np.int32)
        t0 = time.perf_counter()
        if "q_gate" in w:
            oracle.layer_forward_q4(wl.xp_bits, w, logits=wl.lp, top_k=cfg.top_k, sel=sel)
        else:
            oracle.layer_forward(wl.xp_bits, w["w_gate"], w["w_up"], w["w_down"], logits=wl.lp, top_k=cfg.top_k,
                                 shared=shared, sel=sel)
        return time.perf_counter() - t0

    t1 = run(2)
    n = int(max(2, min(cfg.t_prefill, seconds / max(t1 / 2, 1e-6))))
    t = run(n)
    # the same oracle on one thread, on a sample a tenth as long
    oracle.set_threads(1)
    try:
        t_one = run(2)
        n_one = int(max(2, min(n, 0.2 * seconds / max(t_one / 2, 1e-6))))
        t_one = run(n_one)
    finally:
        oracle.set_threads(threads)
    return {"value": round(n / t, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d of the %d prefill tokens of the step (routing for all tokens, full fp64 layer output for "
                      "the sampled ones), %.1f s" % (n, cfg.t_prefill, t),
            "single_thread": {"value": round(n_one / t_one, 3), "unit": "tokens/s", "cores": 1,
                              "sample": "%d tokens, %.1f s" % (n_one, t_one)}}


def solver_study(args, si, torch, cfg, w, r_gg):
    """Profiler & Solver end to end on this machine: fit Eq. 3 from measurements of the library's own kernels,
    workers and copies; solve the generation-phase r_CG* for the given r_GG (Section IV-A.3) and, with the rates
    fixed there, the prompt-phase n_g* (Section IV-B); then measure the real layer at the solved values and on a
    sweep around them (the shape of the paper's slicing-rate ablation, Section V-E.2)."""
    M, H, E, k = cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k
    shared = tuple(w[kk] for kk in ("s_gate", "s_up", "s_down")) if cfg.d_ff_shared and "s_gate" in w else None
    stream = torch.cuda.current_stream().cuda_stream
    wl = Workload(cfg, args.decode_calls)
    R = 1.0 - r_gg

    def touched_mean(calls):
        return float(np.mean([Workload.touched(cfg, lg) for _, _, lg in calls]))

    q4 = "q_gate" in w

    def layer_times(split, n_g, reps):
        if q4:
            layer = si.si_layer_create_q4(M, H, E, k, w, split[0], split[1], split[2], max(cfg.t_prefill, cfg.t_decode),
                                          d_ff_shared=cfg.d_ff_shared)
        else:
            layer = si.si_layer_create(M, H, E, k, w["w_gate"], w["w_up"], w["w_down"], split[0], split[1], split[2],
                                       max(cfg.t_prefill, cfg.t_decode), d_ff_shared=cfg.d_ff_shared, shared=shared)
        try:
            info = si.si_layer_split_info(layer)
            dec, pre = [], []
            for r in range(reps + 1):
                for xd, ld, _ in wl.dec:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    si.si_layer_forward(layer, xd.data_ptr(), ld.data_ptr() if ld is not None else None, cfg.t_decode, 0,
                                        si.SI_DECODE, wl.yd.data_ptr(), stream=stream)
                    torch.cuda.synchronize()
                    if r:
                        dec.append(time.perf_counter() - t0)
            for r in range(reps + 1):
                for ng in n_g:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    si.si_layer_forward(layer, wl.xp.data_ptr(), wl.lp_dev.data_ptr() if wl.lp_dev is not None else None,
                                        cfg.t_prefill, ng, si.SI_PREFILL, wl.yp.data_ptr(), stream=stream)
                    torch.cuda.synchronize()
                    if r:
                        pre.append((ng, time.perf_counter() - t0))
        finally:
            si.si_layer_destroy(layer)
        return info, float(np.median(dec)), {ng: float(np.median([t for g, t in pre if g == ng])) for ng in n_g}

    # --- Profiler: one model per phase (rows of one expert's GEMM in that phase)
    rows_dec = max(1, -(-cfg.t_decode * k // E)) if E > 1 else cfg.t_decode
    e_dec = touched_mean(wl.dec) if E > 1 else 1.0
    if E > 1:
        rows_dec = max(1, int(round(cfg.t_decode * k / e_dec)))
    rows_pre = max(1, cfg.t_prefill * k // E)
    t0 = time.perf_counter()
    prof_dec = si.si_profile(M, H, rows_dec, mode=si.SI_DECODE, n_sizes=6, reps=5, q4=q4)
    prof_pre = si.si_profile(M, H, rows_pre, mode=si.SI_PREFILL, n_sizes=5, reps=3, q4=q4)
    # The token assignment moves along the token axis at full hidden size, so the prompt-phase GEMM models are
    # fitted along that axis: full-size GEMMs at several row counts (the start-up term then carries the cost of
    # streaming the weights once, which a fit over the hidden size at a fixed row count cannot see).
    rows_axis = sorted({r for r in (8, 64, 256, rows_pre) if r <= rows_pre})
    pts = [si.si_profile(M, H, r, mode=si.SI_PREFILL, n_sizes=2, reps=2, q4=q4) for r in rows_axis]
    n_ax = [p["n_gemm"][-1] for p in pts]
    model_pre = dict(prof_pre["model"])
    if len(rows_axis) >= 2:
        a, b, r2_gt = si.si_fit_linear(n_ax, [p["t_g"][-1] for p in pts], nonneg=True)
        model_pre["alpha_g"], model_pre["beta_g"] = a, b
        a, b, r2_ct = si.si_fit_linear(n_ax, [p["t_c"][-1] for p in pts], nonneg=True)
        model_pre["alpha_c"], model_pre["beta_c"] = a, b
    t_prof = time.perf_counter() - t0

    # --- Solver, generation phase: n_l = 3 GEMMs (gate, up, down) per expert that received tokens
    n_w = (0.5 + 2.0 / 64 if q4 else 2.0) * M * H   # bytes of one GEMM's weights on the link
    n_l_dec = int(round(3 * e_dec))
    sol = si.si_solve_split(prof_dec["model"], float(rows_dec) * M * H, n_w, n_l_dec, r_gg, r_step=64.0 / H)
    sweep = sorted({round(f * R, 6) for f in (0.0, 0.25, 0.5, 0.75, 1.0)} | {round(sol["r_cg"], 6)})
    e_pre = float(Workload.touched(cfg, wl.lp)) if E > 1 else 1.0
    n_l_pre = int(round(3 * e_pre))
    T = cfg.t_prefill
    rows = []
    best_split = None
    for r_cg in sweep:
        split = (r_gg, r_cg, max(0.0, 1.0 - r_gg - r_cg))
        is_star = abs(r_cg - sol["r_cg"]) < 1e-6
        ngs = [0]
        sol_ng = None
        if is_star:
            # --- Solver, prompt phase, rates fixed at the generation-phase optimum
            sol_ng = si.si_solve_ng(model_pre, rows_pre, M, H, n_w, n_l_pre, split[0], split[1])
            # the model counts rows of one expert's GEMM; the layer takes n_g in tokens
            ng_tokens = int(round(sol_ng["n_g"] * T / rows_pre))
            ngs = sorted({0, T // 4, T // 2, 3 * T // 4, T, min(T, ng_tokens)})
        info, t_dec, t_pre = layer_times(split, ngs, 3)
        pred = si.si_simulate(si.si_model_times(prof_dec["model"], float(rows_dec) * M * H, n_w, n_l_dec, split[0], split[1]),
                              n_l_dec)["t_fin"]
        row = {"r_cg": r_cg, "r_cc": round(split[2], 6), "columns": info, "solved": is_star,
               "decode_ms_measured": round(1e3 * t_dec, 4), "decode_ms_model": round(1e3 * pred, 4)}
        if is_star:
            row["prefill"] = {"n_g_solved_tokens": min(T, ng_tokens), "n_g_solved_rows": sol_ng["n_g"],
                              "model_ms_at_solved": round(1e3 * sol_ng["t_fin"], 4),
                              "measured_ms_by_n_g": {str(g): round(1e3 * t, 4) for g, t in t_pre.items()}}
        rows.append(row)
    best = min(rows, key=lambda r: r["decode_ms_measured"])
    star = [r for r in rows if r["solved"]][0]
    fixed = [r for r in rows if not r["solved"]]
    out = {
        "solver_study": cfg.name, "weights": "4-bit" if q4 else "bf16", "r_gg": r_gg, "profile_seconds": round(t_prof, 1),
        "model_decode": prof_dec["model"], "r2_decode": [prof_dec["r2_g"], prof_dec["r2_c"], prof_dec["r2_c2g"]],
        "model_prefill": model_pre, "model_prefill_rows_fitted": rows_axis,
        "r2_prefill": [prof_pre["r2_g"], prof_pre["r2_c"], prof_pre["r2_c2g"]],
        "sigma_launch": prof_dec["sigma_launch"], "rows_decode": rows_dec, "rows_prefill": rows_pre,
        "n_l_decode": n_l_dec, "n_l_prefill": n_l_pre,
        "r_cg_solved": sol["r_cg"], "case": sol["case"], "t_fin_model_ms": round(1e3 * sol["t_fin"], 4),
        "sweep": rows,
        "solved_vs_best_measured": round(star["decode_ms_measured"] / best["decode_ms_measured"], 4),
        "speedup_over_fixed": {str(r["r_cg"]): round(r["decode_ms_measured"] / star["decode_ms_measured"], 3) for r in fixed},
    }
    print(json.dumps(out))


def stack_study(args, si, torch, cfg, w):
    """Section IV-A.4 end to end: profile, t_fin*(r_GG = i/n_G) from the slicing-rate solve, greedy assignment of
    a GPU-memory budget over the layers of a stack, and the measured generation step of the stack against the
    uniform assignment of the same budget (the paper's memory-assignment ablation, Section V-E.3)."""
    M, H, E, k = cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k
    if E > 1:
        return stack_study_moe(args, si, torch, cfg, w)
    assert not cfg.d_ff_shared
    n_layers, n_G = args.stack, 8
    T = cfg.t_decode
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    prof = si.si_profile(M, H, T, mode=si.SI_DECODE, n_sizes=6, reps=5)
    n_gemm, n_w, n_l, step = float(T) * M * H, 2.0 * M * H, 3, 64.0 / H
    sols = [si.si_solve_split(prof["model"], n_gemm, n_w, n_l, i / n_G, r_step=step) for i in range(n_G + 1)]
    t_star = [s["t_fin"] for s in sols]
    n_m = 3.0 * n_w
    x = torch.from_numpy(synth_tokens(cfg, T).view(np.int16)).to(dev)
    out = torch.empty((T, M), dtype=torch.float32, device=dev)

    def run(r_ggs):
        layers = []
        try:
            for r_gg in r_ggs:
                sol = si.si_solve_split(prof["model"], n_gemm, n_w, n_l, r_gg, r_step=step)
                r_cg = sol["r_cg"]
                layers.append(si.si_layer_create(M, H, 1, 1, w["w_gate"], w["w_up"], w["w_down"], r_gg, r_cg,
                                                 max(0.0, 1.0 - r_gg - r_cg), T))
            st = si.si_stack_create(layers)
            res = {}
            for name, pf in (("prefetch", 3), ("no_prefetch", 0)):
                ts = []
                for i in range(8):
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    si.si_stack_forward(st, x.data_ptr(), None, T, 0, si.SI_DECODE, out.data_ptr(), prefetch=pf, stream=stream)
                    torch.cuda.synchronize()
                    if i >= 2:
                        ts.append(time.perf_counter() - t0)
                res[name] = float(np.median(ts))
            si.si_stack_destroy(st)
            return res
        finally:
            for l in layers:
                si.si_layer_destroy(l)

    rows = []
    for frac in (0.25, 0.5, 0.75):
        budget = frac * n_layers * n_m
        pick = si.si_assign_gpu_memory([t_star] * n_layers, [n_m] * n_layers, budget)
        greedy = [p / n_G for p in pick]
        uniform = [frac] * n_layers
        model_greedy = sum(t_star[p] for p in pick)
        model_uniform = n_layers * si.si_solve_split(prof["model"], n_gemm, n_w, n_l, frac, r_step=step)["t_fin"]
        mg, mu = run(greedy), run(uniform)
        rows.append({"budget_fraction": frac, "greedy_r_gg": greedy,
                     "greedy_ms": round(1e3 * mg["prefetch"], 3), "greedy_no_prefetch_ms": round(1e3 * mg["no_prefetch"], 3),
                     "uniform_ms": round(1e3 * mu["prefetch"], 3), "uniform_no_prefetch_ms": round(1e3 * mu["no_prefetch"], 3),
                     "model_greedy_ms": round(1e3 * model_greedy, 3), "model_uniform_ms": round(1e3 * model_uniform, 3),
                     "speedup_greedy_over_uniform": round(mu["prefetch"] / mg["prefetch"], 3),
                     "speedup_prefetch": round(mg["no_prefetch"] / mg["prefetch"], 3)})
    print(json.dumps({"stack_study": cfg.name, "layers": n_layers, "n_G": n_G, "tokens": T, "model": prof["model"],
                      "t_star_ms_by_r_gg": [round(1e3 * t, 4) for t in t_star],
                      "r_cg_star_by_r_gg": [round(s["r_cg"], 4) for s in sols], "budgets": rows}))


def stack_study_moe(args, si, torch, cfg, w):
    """A stack of MoE layers of the config's shape at one split (--split, default 50/50/0): generation step with and
    without cross-layer prefetch.  What can travel ahead of a layer's own token assignment is its shared expert's CG
    part; reported per setting: step time, busy time of the host link (sum of the layers' copy times) and the time
    the link idles per layer."""
    import synth
    split = tuple(float(v) for v in args.split.split(",")) if args.split else (0.5, 0.5, 0.0)
    n_layers = args.stack
    T = cfg.t_decode
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    layers = [create_layer(si, cfg, w, split) for _ in range(n_layers)]
    rows = []
    try:
        st = si.si_stack_create(layers)
        xb = synth.make_tokens(cfg, T, stream=7)
        lg = synth.make_router_logits(cfg, xb)
        x = torch.from_numpy(xb.view(np.int16)).to(dev)
        lgd = torch.from_numpy(lg).to(dev)
        out = torch.empty((T, cfg.d_model), dtype=torch.float32, device=dev)
        ptrs = [lgd.data_ptr()] * n_layers
        for name, pf in (("no_prefetch", 0), ("prefetch", 3)):
            for l in layers:
                si.si_layer_set_profiling(l, 0)
            ts = []
            for i in range(10):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                si.si_stack_forward(st, x.data_ptr(), ptrs, T, 0, si.SI_DECODE, out.data_ptr(), prefetch=pf, stream=stream)
                torch.cuda.synchronize()
                if i >= 2:
                    ts.append(time.perf_counter() - t0)
            for l in layers:
                si.si_layer_set_profiling(l, 1)
            busy = []
            for i in range(4):
                torch.cuda.synchronize()
                si.si_stack_forward(st, x.data_ptr(), ptrs, T, 0, si.SI_DECODE, out.data_ptr(), prefetch=pf, stream=stream)
                torch.cuda.synchronize()
                stats = [si.si_layer_stats(l) for l in layers]
                if i >= 1:
                    busy.append(sum(s_["copy_ms"] for s_ in stats))
            step_ms = 1e3 * float(np.median(ts))
            rows.append({"setting": name, "step_ms": round(step_ms, 3), "link_busy_ms": round(float(np.mean(busy)), 3),
                         "link_idle_ms_per_layer": round((step_ms - float(np.mean(busy))) / n_layers, 4),
                         "streamed_MB_per_step": round(sum(s_["bytes_streamed"] for s_ in stats) / 1e6, 1)})
        si.si_stack_destroy(st)
    finally:
        for l in layers:
            si.si_layer_destroy(l)
    print(json.dumps({"stack_study": cfg.name, "layers": n_layers, "tokens": T, "split": list(split), "rows": rows}))


def placement_study(args, si, torch, cfg, w):
    """Whole-expert placement against uniform slicing at the same GPU-memory budget: with a skewed router the
    most frequently chosen experts are kept resident, so fewer bytes cross the host link per call."""
    assert cfg.n_experts > 1, "--place needs an MoE config"
    M, H, E, k = cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k
    shared = tuple(w[kk] for kk in ("s_gate", "s_up", "s_down")) if cfg.d_ff_shared else None
    stream = torch.cuda.current_stream().cuda_stream
    wl = Workload(cfg, args.decode_calls)
    # expert frequencies from the prompt batch (host arithmetic on the router logits, an input)
    order = np.argsort(-wl.lp, axis=1, kind="stable")[:, :k]
    freq = np.bincount(order.ravel(), minlength=E).astype(np.float64)

    def run(split, placement):
        layer = si.si_layer_create(M, H, E, k, w["w_gate"], w["w_up"], w["w_down"], split[0], split[1], split[2],
                                   cfg.t_decode, d_ff_shared=cfg.d_ff_shared, shared=shared, placement=placement)
        try:
            ts, streamed = [], []
            si.si_layer_set_profiling(layer, 1)
            for r in range(4):
                for xd, ld, _ in wl.dec:
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    si.si_layer_forward(layer, xd.data_ptr(), ld.data_ptr(), cfg.t_decode, 0, si.SI_DECODE, wl.yd.data_ptr(), stream=stream)
                    torch.cuda.synchronize()
                    if r:
                        ts.append(time.perf_counter() - t0)
                        streamed.append(si.si_layer_stats(layer)["bytes_streamed"])
            return float(np.mean(ts)), float(np.mean(streamed))
        finally:
            si.si_layer_destroy(layer)

    rows = []
    for frac in (0.125, 0.25, 0.5):
        n_gg = int(round(frac * E))
        t_u, b_u = run((frac, 1.0 - frac, 0.0), None)
        place = si.si_place_experts(freq, n_gg, 1.0)
        t_p, b_p = run((1.0, 0.0, 0.0), place)
        mass = float(sum(freq[e] for e in range(E) if place[e] == 0) / freq.sum())
        rows.append({"gpu_fraction_of_routed_weights": frac, "resident_experts": n_gg, "routing_mass_resident": round(mass, 3),
                     "uniform_ms": round(1e3 * t_u, 4), "uniform_streamed_MB": round(b_u / 1e6, 2),
                     "placed_ms": round(1e3 * t_p, 4), "placed_streamed_MB": round(b_p / 1e6, 2),
                     "speedup": round(t_u / t_p, 3)})
    print(json.dumps({"placement_study": cfg.name, "tokens_per_call": cfg.t_decode, "experts": E, "top_k": k,
                      "decode_calls": len(wl.dec), "rows": rows}))


def sweep_study(args, si, torch, cfg, w):
    """One layer, re-sliced through the split sweep: call times per phase, streamed bytes, link rate, overlap."""
    import synth
    wl = Workload(cfg, args.decode_calls)
    stream = torch.cuda.current_stream().cuda_stream
    first = synth.SPLIT_SWEEP[0]
    shared = tuple(w[k] for k in ("s_gate", "s_up", "s_down")) if cfg.d_ff_shared else None
    layer = si.si_layer_create(cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k, w["w_gate"], w["w_up"], w["w_down"],
                               first[0], first[1], first[2], max(cfg.t_prefill, cfg.t_decode),
                               d_ff_shared=cfg.d_ff_shared, shared=shared)
    rows = []
    try:
        for split in synth.SPLIT_SWEEP:
            t0 = time.perf_counter()
            si.si_layer_resplit(layer, *split)
            t_resplit = time.perf_counter() - t0
            n_g = cfg.t_prefill if split[2] > 0 else 0
            run_steps(si, layer, wl, max(1, args.warmup), n_g, stream)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                for xd, ld, _lg in wl.dec:
                    si.si_layer_forward(layer, xd.data_ptr(), ld.data_ptr() if ld is not None else None, cfg.t_decode, 0,
                                        si.SI_DECODE, wl.yd.data_ptr(), stream=stream)
            torch.cuda.synchronize()
            t_dec = (time.perf_counter() - t1) / (args.steps * len(wl.dec))
            t1 = time.perf_counter()
            for _ in range(args.steps):
                si.si_layer_forward(layer, wl.xp.data_ptr(), wl.lp_dev.data_ptr() if wl.lp_dev is not None else None,
                                    cfg.t_prefill, n_g, si.SI_PREFILL, wl.yp.data_ptr(), stream=stream)
            torch.cuda.synchronize()
            t_pre = (time.perf_counter() - t1) / args.steps
            si.si_layer_set_profiling(layer, 1)
            stats = []
            run_steps(si, layer, wl, 1, n_g, stream, collect=stats)
            torch.cuda.synchronize()
            si.si_layer_set_profiling(layer, 0)
            pre = [st for kind, st in stats if kind == "prefill"]
            dec = [st for kind, st in stats if kind == "decode"]
            copied = sum(st["bytes_streamed"] for _, st in stats)
            copy_ms = sum(st["copy_ms"] for _, st in stats)
            rows.append({"split": list(split), "columns": si.si_layer_split_info(layer), "n_g": n_g,
                         "resplit_s": round(t_resplit, 3),
                         "prefill_call_ms": round(1e3 * t_pre, 3), "decode_call_ms": round(1e3 * t_dec, 4),
                         "prefill_tokens_per_s": round(cfg.t_prefill / t_pre, 1),
                         "decode_tokens_per_s": round(cfg.t_decode / t_dec, 1),
                         "streamed_MB_prefill": round(sum(st["bytes_streamed"] for st in pre) / 1e6, 1),
                         "streamed_MB_decode_call": round(float(np.mean([st["bytes_streamed"] for st in dec])) / 1e6, 1),
                         "link_GBps": round(copied / (copy_ms / 1e3) / 1e9, 2) if copy_ms > 0 else None,
                         "overlap_prefill": round(float(np.mean([st["overlap"] for st in pre])), 3),
                         "overlap_decode": round(float(np.mean([st["overlap"] for st in dec])), 3),
                         "cc_ms_decode_call": round(float(np.mean([st["cc_ms"] for st in dec])), 3)})
            print("sweep %s done" % (split,), file=sys.stderr, flush=True)
    finally:
        si.si_layer_destroy(layer)
    print(json.dumps({"study": "split sweep", "config": {"workload": "%s-shaped layer: E=%d top-%d M=%d H=%d, prefill %d tokens, "
                      "decode %d token(s) per call" % (cfg.name, cfg.n_experts, cfg.top_k, cfg.d_model, cfg.d_ff,
                                                        cfg.t_prefill, cfg.t_decode)},
                      "dtype": "bf16", "data": "synthetic", "rows": rows}))


def synth_tokens(cfg, T):
    import synth
    return synth.make_tokens(cfg, T, stream=7)


def workload_text(cfg, decode_calls):
    return ("%s-shaped layer: E=%d top-%d M=%d H=%d%s, step = 1 prefill call of %d tokens + %d decode calls of %d token(s)"
            % (cfg.name, cfg.n_experts, cfg.top_k, cfg.d_model, cfg.d_ff,
               (" + shared H=%d" % cfg.d_ff_shared) if cfg.d_ff_shared else "", cfg.t_prefill, decode_calls, cfg.t_decode))


def link_of(stats, steps):
    pre = [st for kind, st in stats if kind == "prefill"]
    dec = [st for kind, st in stats if kind == "decode"]
    copied = sum(s["bytes_streamed"] for _, s in stats)
    copy_ms = sum(s["copy_ms"] for _, s in stats)
    if copied <= 0:
        return None
    return {"GBps": round(copied / (copy_ms / 1e3) / 1e9, 2), "bytes_per_step": copied / steps,
            "copy_ms_per_step": copy_ms / steps,
            "overlap_prefill": float(np.mean([s["overlap"] for s in pre])),
            "overlap_decode": float(np.mean([s["overlap"] for s in dec])),
            "gg_kernel_time_under_copies_prefill": float(np.mean([s["gg_in_copy"] for s in pre])),
            "gg_kernel_time_under_copies_decode": float(np.mean([s["gg_in_copy"] for s in dec])),
            "cc_ms_per_step": sum(s["cc_ms"] for _, s in stats) / steps,
            "eq6_predicted_prefill_ms": float(np.mean([eq6_prediction(s) for s in pre])),
            "eq6_predicted_decode_ms": float(np.mean([eq6_prediction(s) for s in dec])),
            "measured_prefill_ms": float(np.mean([s["total_ms"] for s in pre])),
            "measured_decode_ms": float(np.mean([s["total_ms"] for s in dec]))}


def split_entry(si, cfg, split, n_g, wl, steps, elapsed, stats, info, calls, q4=False):
    """One row of the `configs` array: a workload shape at one GG/CG/CC split."""
    ktab = kernel_table(si, cfg, info, wl, stats, steps, n_g, q4=q4)
    tokens_per_step = cfg.t_prefill + len(wl.dec) * cfg.t_decode
    ms_per_step = 1e3 * elapsed / steps
    ent = {"config": cfg.name, "split_gg_cg_cc": [round(v, 4) for v in split], "columns": info, "n_g": n_g,
           "steps": steps, "decode_calls": len(wl.dec), "ms_per_step": round(ms_per_step, 4),
           "tokens_per_s": round(tokens_per_step / (ms_per_step / 1e3), 1),
           "prefill_call_ms": round(calls["prefill_call_us"] / 1e3, 4), "decode_call_us": round(calls["decode_call_us"], 2),
           "prefill_tokens_per_s": round(cfg.t_prefill / (calls["prefill_call_us"] / 1e6), 1),
           "decode_tokens_per_s": round(cfg.t_decode / (calls["decode_call_us"] / 1e6), 1)}
    # the generation-phase call as a whole against the HBM bound of the weight bytes its kernels read
    if "decode_gateup" in ktab and tuple(split)[0] == 1.0:
        call_bytes = (ktab["decode_gateup"]["bytes_per_step"] + ktab["decode_down"]["bytes_per_step"]) / len(wl.dec)
        ent["decode_call_frac_of_hbm_bound"] = round(call_bytes / (calls["decode_call_us"] / 1e6) / (HBM_PEAK_GBS * 1e9), 4)
    ent["rooflines"] = [roofline_of(k, ktab[k], None if q4 else cfg.name, split) for k in ktab if "bound" in ktab[k]]
    ent["other_kernels_us"] = {k: round(v["avg_launch_us"], 2) for k, v in ktab.items() if "bound" not in v}
    link = link_of(stats, steps)
    if link:
        ent["host_link"] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in link.items()}
    return ent, ktab


def all_configs_line(args, si, torch, synth):
    """Default run: every workload shape at full size; headline on the Mixtral-8x22B-shaped layer."""
    plan = [("mixtral_8x7b", [(1.0, 0.0, 0.0), (0.5, 0.5, 0.0)]),
            ("llama2_70b", [(1.0, 0.0, 0.0), (0.3, 0.5, 0.2)]),
            ("qwen_moe", [(1.0, 0.0, 0.0), (0.5, 0.5, 0.0)]),
            ("phimoe", list(synth.SPLIT_SWEEP)),
            (HEADLINE, list(synth.SPLIT_SWEEP))]
    entries = []
    head = None
    t_all = time.perf_counter()
    for name, splits in plan:
        cfg = synth.CONFIGS[name]
        t0 = time.perf_counter()
        w = synth.make_weights(cfg, threads=min(16, os.cpu_count() or 8))
        wl_full = Workload(cfg, args.decode_calls)
        wl_short = Workload(cfg, min(args.decode_calls, 4))
        t_gen = time.perf_counter() - t0
        layer = create_layer(si, cfg, w, splits[0])
        try:
            for split in splits:
                if split != splits[0]:
                    si.si_layer_resplit(layer, *split)
                n_g = cfg.t_prefill if split[2] > 0 else 0
                is_head = name == HEADLINE and split == (1.0, 0.0, 0.0)
                # resident-only splits take microseconds to milliseconds per step: full step count; the link-bound
                # ones take up to 0.3 s per step and are timed over a few steps of fewer decode calls
                full = is_head or split == (1.0, 0.0, 0.0)
                steps = args.steps if full else max(1, min(args.steps, 3))
                warmup = args.warmup if full else 1
                wl = wl_full if full else wl_short
                elapsed, stats, info, calls = measure_layer(si, torch, layer, wl, steps, warmup, n_g)
                ent, ktab = split_entry(si, cfg, split, n_g, wl, steps, elapsed, stats, info, calls)
                entries.append(ent)
                print("bench: %s %s done (%.1f s since start)" % (name, split, time.perf_counter() - t_all), file=sys.stderr, flush=True)
                if is_head:
                    weight_kernels = [k for k in ktab if "bound" in ktab[k]]
                    dominant = max(weight_kernels, key=lambda k: ktab[k]["ms_per_step"])
                    roof = roofline_of(dominant, ktab[dominant], cfg.name, split)
                    roof["timer"] = TIMER_NOTE
                    head = {"ent": ent, "roofline": roof, "elapsed": elapsed, "t_gen": t_gen, "info": info}
        finally:
            si.si_layer_destroy(layer)
        if name == HEADLINE and not args.no_cpu_baseline:
            head["cpu_baseline"] = cpu_baseline(cfg, w, wl_full, args.cpu_seconds)
        del w, wl_full, wl_short
    cfg = synth.CONFIGS[HEADLINE]
    ms_per_step = 1e3 * head["elapsed"] / args.steps
    tokens_per_step = cfg.t_prefill + args.decode_calls * cfg.t_decode
    out = {
        "metric": "FFN/MoE layer tokens/s (decode+prefill)", "value": round(tokens_per_step / (ms_per_step / 1e3), 2),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload_text(cfg, args.decode_calls), "split_gg_cg_cc": [1.0, 0.0, 0.0],
                   "columns": head["info"], "n_g": 0, "tokens_per_step": tokens_per_step},
        "roofline": head["roofline"],
        "configs": entries,
        "measured_peaks": {k: (round(v, 1) if isinstance(v, float) else v) for k, v in MEASURED_PEAKS.items()} if MEASURED_PEAKS else None,
        "bench_wall_s": round(time.perf_counter() - t_all, 1),
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    print(json.dumps(out))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported. "
              "The printed value is one GPU's throughput." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import synth
    import paper_2411_15715_amd as si
    si.lib()  # fail loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    global MEASURED_PEAKS, DEQ_MIB
    DEQ_MIB = args.deq_mib
    if not args.no_peaks:
        MEASURED_PEAKS = si.si_measure_peaks(0)
    if args.config is None:
        if args.q4 or args.solve or args.stack or args.place or args.sweep or args.split:
            print("bench.py: --q4 / --split / --solve / --stack / --place / --sweep need --config", file=sys.stderr)
            sys.exit(2)
        all_configs_line(args, si, torch, synth)
        return
    cfg = synth.CONFIGS[args.config]
    split = tuple(float(v) for v in args.split.split(",")) if args.split else cfg.split
    n_g = args.n_g if args.n_g >= 0 else (cfg.t_prefill if split[2] > 0 else 0)
    t0 = time.perf_counter()
    if args.q4:
        w = synth.make_weights_q4(cfg, threads=min(16, os.cpu_count() or 8))
    else:
        w = synth.make_weights(cfg, threads=min(16, os.cpu_count() or 8))
    if args.solve:
        solver_study(args, si, torch, cfg, w, split[0])
        return
    if args.stack:
        stack_study(args, si, torch, cfg, w)
        return
    if args.place:
        placement_study(args, si, torch, cfg, w)
        return
    if args.sweep:
        sweep_study(args, si, torch, cfg, w)
        return
    wl = Workload(cfg, args.decode_calls)
    t_gen = time.perf_counter() - t0
    tokens_per_step = cfg.t_prefill + args.decode_calls * cfg.t_decode

    elapsed, stats, info, calls = measure(si, torch, cfg, w, split, wl, args.steps, args.warmup, n_g)
    ms_per_step = 1e3 * elapsed / args.steps
    ktab = kernel_table(si, cfg, info, wl, stats, args.steps, n_g, q4=args.q4)
    weight_kernels = [k for k in ktab if "bound" in ktab[k]]
    dominant = max(weight_kernels, key=lambda k: ktab[k]["ms_per_step"])
    pre = [st for kind, st in stats if kind == "prefill"]
    dec = [st for kind, st in stats if kind == "decode"]
    phase = {
        "decode_call_us": calls["decode_call_us"], "prefill_call_us": calls["prefill_call_us"],
        "prefill_ms": float(np.mean([s["total_ms"] for s in pre])), "decode_ms": float(np.mean([s["total_ms"] for s in dec])),
        "prefill_tokens_per_s": cfg.t_prefill / (np.mean([s["total_ms"] for s in pre]) / 1e3),
        "decode_tokens_per_s": cfg.t_decode / (np.mean([s["total_ms"] for s in dec]) / 1e3),
    }
    link = link_of(stats, args.steps)
    roof = roofline_of(dominant, ktab[dominant], None if args.q4 else cfg.name, split)
    roof["timer"] = TIMER_NOTE
    out = {
        "metric": "FFN/MoE layer tokens/s (decode+prefill)", "value": round(tokens_per_step / (ms_per_step / 1e3), 2),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 weights x bf16 activations, f32 accumulate" if args.q4 else "bf16", "data": "synthetic",
        "config": {"workload": workload_text(cfg, args.decode_calls),
                   "split_gg_cg_cc": list(split), "columns": info, "n_g": n_g, "tokens_per_step": tokens_per_step},
        "roofline": roof,
        "phases": {k: round(v, 4) for k, v in phase.items()},
        "kernels": {k: {kk: (round(vv, 4) if isinstance(vv, float) else vv) for kk, vv in v.items()} for k, v in ktab.items()},
        "host_link": link,
        "input_generation_s": round(t_gen, 1),
        "measured_peaks": {k: (round(v, 1) if isinstance(v, float) else v) for k, v in MEASURED_PEAKS.items()} if MEASURED_PEAKS else None,
    }
    if not args.no_gg_only and tuple(split) != (1.0, 0.0, 0.0):
        e2, stats2, info2, calls2 = measure(si, torch, cfg, w, (1.0, 0.0, 0.0), wl, args.steps, args.warmup, 0)
        k2 = kernel_table(si, cfg, info2, wl, stats2, args.steps, 0, q4=args.q4)
        pre2 = [st for kind, st in stats2 if kind == "prefill"]
        dec2 = [st for kind, st in stats2 if kind == "decode"]
        out["gg_only"] = {
            "split_gg_cg_cc": [1.0, 0.0, 0.0], "ms_per_step": round(1e3 * e2 / args.steps, 4),
            "tokens_per_s": round(tokens_per_step / (e2 / args.steps), 2),
            "decode_call_us": round(calls2["decode_call_us"], 2), "prefill_call_us": round(calls2["prefill_call_us"], 2),
            "prefill_ms": round(float(np.mean([s["total_ms"] for s in pre2])), 4),
            "decode_ms": round(float(np.mean([s["total_ms"] for s in dec2])), 4),
            "rooflines": [roofline_of(k, k2[k], None if args.q4 else cfg.name, (1.0, 0.0, 0.0)) for k in k2 if "bound" in k2[k]],
        }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, w, wl, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
