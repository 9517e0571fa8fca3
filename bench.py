#!/usr/bin/env python3
"""Benchmark of the HPSGD hot path on one MI355X.

One "step" is one round of the overlapped schedule (Sec. 3.1): batch gather and local step of
all K workers (forward, BPTT, SGD commit) on the training stream, merge of the previous round's
replica changes and the clone of the global model on the synchronising stream.  The default
workload is the GRU language model (config 3: V10000 E256 H1024 L2 T35 B32, K=8, bf16 GEMM
operands / fp32 accumulate), the largest configuration that runs on one GPU; `--workload`
selects configs 1, 2, 4.  Inputs (shards, parameters) are resident in HBM before the timed
region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

# Kernels whose work is counted in bytes (HBM roofline); every other timed kernel is a contraction.
STREAMING_KERNELS = {"cvt2_kernel", "cvt2_pack_kernel", "softmax_ce_bf16_rows_kernel", "commit_kernel", "commit_acc4_kernel"}

# HBM bytes per launch of a kernel, from two `rocprofv3 --pmc` runs of this file (FETCH_SIZE, then
# WRITE_SIZE, in KiB per dispatch; FETCH_SIZE scaled by 2.0 and WRITE_SIZE by 1.0: the config-5
# kernels of the same run are the copy kernels of known size), averaged over the kernel's launches
# of a round.  Summaries with the full commands: profiles/bench_*.md.  Kernels not collected: null.
KIB = 1024.0
MEASURED_TRAFFIC_BYTES = {
    "gru_cls": {"gru_bwd_persist_kernel": (2.0 * 91903.0 + 150171.0) * KIB,
                "gru_fwd_persist_kernel": (2.0 * 26935.9 + 107529.2) * KIB},
    # the 192 x 256 form runs three products per round: the logits (679 MB) and two input gradients
    # (head and top layer; both launch 192 tiles and average 262 MB)
    "gru_lm": {"gemm_bf16_dlx_kernel<false, 2, 4, 3, 2, 2>":
                   ((2.0 * 153894.5 + 355321.4) + 2 * (2.0 * 109983.5 + 35879.3)) * KIB / 3,
               "gru_bwd_persist_bf16_kernel": (2.0 * 161238.2 + 240383.4) * KIB,
               "gru_fwd_persist_bf16_kernel": (2.0 * 89352.9 + 238874.5) * KIB,
               "gemm_bf16_dlx_kernel<true, 2, 4, 4, 2, 2>": (2.0 * 296087.8 + 325485.9) * KIB,
               "gemm_bf16_dlx_kernel<true, 2, 4, 3, 2, 2>": (2.0 * 95253.1 + 100010.3) * KIB,
               "softmax_ce_bf16_rows_kernel": (2.0 * 177839.5 + 194819.1) * KIB},
    "mlp": {},
}


WORKLOAD_TEXT = {
    "gru_cls": "config 2: GRU classifier I128 H512 T35 B64 C10, K=4 workers, fp32, merge every local step "
               "(overlapped on a second stream)",
    "gru_lm": "config 3: GRU language model V10000 E256 H1024 L2 T35 B32, K=8 workers, bf16 GEMM operands / "
              "fp32 accumulate, merge every local step (overlapped)",
    "mlp": "config 4: MLP 784-1024-1024-10, B128, K=16 workers, fp32, merge every local step (overlapped)",
    "tiny_gru": "config 1: tiny GRU I16 H32 T8 B4, K=2 (launch-bound, parity case)",
}


def mfma_probe(hb, torch, dev, prec):
    """Sustained rate of a pure-MFMA loop (no memory traffic) on every CU, with all-zero and with
    random operands: the operand data decides the power the matrix cores draw and with it the
    clock the chip holds, so this is the ceiling any real contraction of that type sees."""
    out = {}
    sink = torch.empty(256 * 256, dtype=torch.float32, device=dev)
    res = torch.zeros(4, dtype=torch.float64, device=dev)
    iters = 4000
    for kind in ("zeros", "random"):
        if kind == "zeros":
            ops = torch.zeros(16384, dtype=torch.uint8, device=dev)
        else:
            g = torch.Generator(device=dev).manual_seed(7)
            vals = torch.rand(4096, device=dev, generator=g) * 2 - 1
            ops = (vals.to(torch.bfloat16).view(torch.uint8).repeat(2) if prec == "bf16"
                   else vals.view(torch.uint8)).contiguous()
        for _ in range(2):
            hb.probe_mfma_rate(prec, ops, iters, res, sink)
        torch.cuda.synchronize()
        clk, wall, n, flops = res.cpu().tolist()
        seconds = wall / 100e6
        # one wave on every SIMD: 256 workgroups x 4 waves
        out[kind] = {"TFLOP/s": 256 * 4 * n * flops / seconds / 1e12, "shader_MHz": clk / wall * 100.0}
    return out


def samples_per_round(cfg):
    return cfg["K"] * cfg["batch"] * (cfg["seq_len"] if cfg["kind"] == "gru_lm" else 1)


def make_trainer(wl, harness, name, dev, prepare=False, implicit_clone=True):
    cfg = wl.CONFIGS[name]
    K = cfg["K"]
    init = wl.init_params(cfg)
    shards = [wl.make_shard(cfg, k) for k in range(K)]
    orders = [wl.batch_order(cfg, k) for k in range(K)]
    return cfg, init, shards, harness.Trainer(cfg, init, shards, orders, device=dev, prepare=prepare,
                                              implicit_clone=implicit_clone)


def timed_rounds(torch, tr, lr, step, n):
    """n overlapped rounds bracketed by device synchronisation; returns (seconds, next step)."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        tr.ovl_round(step, lr)
        step += 1
    torch.cuda.synchronize()
    return time.perf_counter() - t0, step


def quick_workload(torch, wl, harness, name, dev, rounds=100, warmup=10, **trainer_args):
    """Throughput of another configuration in the same overlapped schedule (an extra key of the line)."""
    cfg, _, _, tr = make_trainer(wl, harness, name, dev, **trainer_args)
    tr.ovl_begin()
    _, step = timed_rounds(torch, tr, cfg["lr"], 0, warmup)
    el, step = timed_rounds(torch, tr, cfg["lr"], step, rounds)
    tr.ovl_drain()
    unit = "tokens/s" if cfg["kind"] == "gru_lm" else "samples/s"
    return {"workload": WORKLOAD_TEXT[name], "value": samples_per_round(cfg) * rounds / el, "unit": unit,
            "ms_per_step": 1e3 * el / rounds, "steps": rounds}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-merge-stress", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the other configurations, the schedule comparisons and the matrix-core probe")
    ap.add_argument("--prepare", default="clones_a", choices=["off", "replicas_b", "clones_b", "clones_a"],
                    help="where the bf16 weight copies of a round's freshly cloned replicas are made: by the local "
                         "step itself from the K replicas (off), ahead on the synchronising stream from the replicas "
                         "or from the clone's source, or on the training stream from the clone's source (default)")
    ap.add_argument("--workload", default="gru_lm", choices=["gru_cls", "gru_lm", "mlp", "tiny_gru"],
                    help="default: config 3, the largest configuration that fits one GPU")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (K workers are a group dimension on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2009_02701_amd import binding as hb
    from paper_2009_02701_amd import harness, workloads as wl

    dev = "cuda:0"
    cfg, init, shards, tr = make_trainer(wl, harness, args.workload, dev, False if args.prepare == "off" else args.prepare)
    K, B, lr = cfg["K"], cfg["batch"], cfg["lr"]
    knames = tr.ctx.kernel_names()
    per_round = samples_per_round(cfg)
    unit = "tokens/s" if cfg["kind"] == "gru_lm" else "samples/s"
    mfma_peak = (PEAK_BF16_MFMA_TFLOPS if cfg.get("prec") == "bf16" else PEAK_FP32_MFMA_TFLOPS) * 1e12

    # ---- pass 0: every timed kernel with an event pair of its own, a few rounds: which single
    # kernel takes the most time of a round
    tr.ovl_begin()
    _, step = timed_rounds(torch, tr, lr, 0, 3)
    tr.ctx.kernel_timer_enable(range(1, hb.KERNEL_COUNT))
    probe_rounds = 5
    _, step = timed_rounds(torch, tr, lr, step, probe_rounds)
    kernels = {}
    for kid in range(1, hb.KERNEL_COUNT):
        n, ms, work = tr.ctx.kernel_timer_read(kid)
        if n:
            streaming = knames[kid] in STREAMING_KERNELS
            peak = PEAK_HBM_GBS * 1e9 if streaming else mfma_peak
            kernels[knames[kid]] = {"id": kid, "launches_per_step": n / probe_rounds, "avg_us": 1e3 * ms / n,
                                    "us_per_step": 1e3 * ms / probe_rounds, "bound": "hbm" if streaming else "mfma",
                                    "frac_of_peak": work / (ms * 1e-3) / peak}
    tr.ctx.kernel_timer_enable([])
    dominant = max(kernels, key=lambda k: kernels[k]["us_per_step"])
    dom_id = kernels[dominant]["id"]
    fused = tr.ctx.recurrence_info()

    # ---- warm-up, then the timed region: `value` comes from K rounds with no instrumentation
    _, step = timed_rounds(torch, tr, lr, step, args.warmup)
    elapsed, step = timed_rounds(torch, tr, lr, step, args.steps)
    ms_per_step = 1e3 * elapsed / args.steps
    value = per_round / (ms_per_step * 1e-3)

    # ---- the spread: every round of a second pass between two events on the training stream
    n_spread = max(20, min(args.steps, 100))
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_spread + 1)]
    torch.cuda.synchronize()
    evs[0].record(tr.stream_a)
    for i in range(n_spread):
        tr.ovl_round(step, lr)
        step += 1
        evs[i + 1].record(tr.stream_a)
    torch.cuda.synchronize()
    per_round_ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(n_spread)]
    spread = {"rounds": n_spread, "median_ms": statistics.median(per_round_ms), "min_ms": min(per_round_ms),
              "max_ms": max(per_round_ms), "mean_ms": sum(per_round_ms) / n_spread}

    # ---- the same rounds replayed from a HIP graph (one graph = `period` rounds; extra key, the
    # headline stays the eagerly issued schedule): what is left of the host's share
    graph_replay = None
    if not args.no_extras:
        graph = tr.ovl_capture(step, lr)
        period = tr.ovl_replay(graph)   # the capture itself ran nothing: this replay issues the captured rounds
        step += period
        n_rep = max(1, args.steps // period)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(n_rep):
            step += tr.ovl_replay(graph)
        torch.cuda.synchronize()
        el_g = time.perf_counter() - c0
        graph_replay = {"rounds_per_graph": period, "replays": n_rep, "ms_per_step": 1e3 * el_g / (n_rep * period),
                        "value": per_round * n_rep * period / el_g, "unit": unit}
        del graph

    # ---- the same region once more with a HIP event pair around every launch of the dominant
    # kernel only (recorded by its launcher on the stream the launch goes to): the roofline's
    # launch duration, and the kernel's algorithmic work as its launcher counts it
    tr.ctx.kernel_timer_enable([dom_id])
    el_i, step = timed_rounds(torch, tr, lr, step, args.steps)
    n_dom, ms_dom, work_dom = tr.ctx.kernel_timer_read(dom_id)
    tr.ctx.kernel_timer_enable([])
    tr.ovl_drain()
    streaming = dominant in STREAMING_KERNELS
    peak = PEAK_HBM_GBS * 1e9 if streaming else mfma_peak
    scale = 1e9 if streaming else 1e12
    dur = ms_dom * 1e-3 / n_dom
    ach = work_dom / n_dom / dur
    roofline = {"kernel": dominant, "bound": "hbm" if streaming else "mfma", "achieved": ach / scale,
                "peak": peak / scale, "unit": "GB/s" if streaming else "TFLOP/s", "frac": ach / peak,
                "avg_launch_us": dur * 1e6, "launches_timed": n_dom, "launches_per_step": n_dom / args.steps,
                "work_per_launch": work_dom / n_dom,
                "ms_per_step_with_event_pairs": 1e3 * el_i / args.steps,
                "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload, {}).get(dominant)}

    # ---- overlap (Sec. 3.1 / 3.2): the training side alone (gather + local step, no exchange), the
    # synchronising side alone (merge + clone), the blocking order of the two, and the overlapped
    # round - each side in the form the overlapped round runs it (the clone is the snapshot alone,
    # the local step reads its parameters from it).  efficiency = (t_A + t_B) / t_overlapped: 1 = nothing hidden, (t_A + t_B) / max(t_A, t_B)
    # = everything hidden (what Sec. 3.2's count gives for gamma = 1 and t_sync = k t_train, k < 1).
    n_ov = max(20, min(args.steps, 60))
    tr.s_train_side(lr, 5)
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    tr.s_train_side(lr, n_ov)
    t_a = (time.perf_counter() - c0) / n_ov
    sb = tr.stream_b
    def sync_side():
        if tr.implicit_clone:
            tr.merge_snapshot(0, sb)
        else:
            tr.merge(0, sb)
            tr.sync_all(0, sb)
    for _ in range(3):
        sync_side()
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    for _ in range(n_ov):
        sync_side()
    torch.cuda.synchronize()
    t_b = (time.perf_counter() - c0) / n_ov
    tr.s_seq(lr, 1, 5, record_loss=False)
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    tr.s_seq(lr, 1, n_ov, record_loss=False)
    t_blocking = (time.perf_counter() - c0) / n_ov
    t_ovl = ms_per_step * 1e-3
    overlap = {"t_train_ms": 1e3 * t_a, "t_sync_ms": 1e3 * t_b, "t_blocking_round_ms": 1e3 * t_blocking,
               "t_overlapped_round_ms": 1e3 * t_ovl, "overlap_efficiency": (t_a + t_b) / t_ovl,
               "all_hidden_would_be": (t_a + t_b) / max(t_a, t_b),
               "hidden_fraction_of_sync": max(0.0, min(1.0, (t_a + t_b - t_ovl) / t_b)), "rounds": n_ov}

    async_driver, compare, forms, others, probe, written_out = None, None, None, None, None, None
    if not args.no_extras:
        # ---- the asynchronous driver (Alg. 2 + Alg. 3 with the status check at run time): the same
        # kernels, the number of local steps per synchronisation decided by whether stream B is idle;
        # once as is, once with a synthetic synchronisation latency of about 2.5 local steps
        async_driver = []
        for delay in (0, int(2.5e3 * ms_per_step)):
            torch.cuda.synchronize()
            a0 = time.perf_counter()
            counts = tr.s_async(lr, 60, sync_delay_us=delay)
            a1 = time.perf_counter()
            async_driver.append({"sync_delay_us": delay, "local_steps": 60, "rounds": len(counts),
                                 "max_steps_per_round": max(counts), "value": 60 * per_round / (a1 - a0),
                                 "unit": unit})

        # ---- the paper's comparison in shape (Sec. 4.3): the same 64 local steps under the same
        # synthetic synchronisation latency with the blocking schedules (synchronous SGD, Local SGD
        # with gamma = 8, Sec. 4.1) and with the overlapped asynchronous one
        delay = int(2.5e3 * ms_per_step)
        compare = {"sync_delay_us": delay, "local_steps": 64, "unit": unit}
        for name, run in (("ssgd_blocking", lambda: tr.s_seq(lr, 1, 64, record_loss=False, sync_delay_us=delay)),
                          ("local_sgd_gamma8_blocking", lambda: tr.s_seq(lr, 8, 8, record_loss=False, sync_delay_us=delay)),
                          ("hpsgd_async", lambda: tr.s_async(lr, 64, sync_delay_us=delay)),
                          ("psgd_no_sync", lambda: tr.s_psgd(lr, 64, record_loss=False))):
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            run()
            compare[name] = 64 * per_round / (time.perf_counter() - c0)

        # gradient-form synchronisation (Eq. 1 as printed): blocking rounds of one local step, for the
        # cost of accumulating gradients (no update in GEMM epilogues) next to the delta form
        forms = {"unit": unit}
        for name, run in (("delta_form_s_seq", lambda: tr.s_seq(lr, 1, 32, record_loss=False)),
                          ("gradient_form_s_seq_grad", lambda: tr.s_seq_grad(lr, 1, 32, record_loss=False))):
            run()
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            run()
            forms[name] = 32 * per_round / (time.perf_counter() - c0)
        # the commit kernels of the two forms against HBM (update: 12 B per parameter it touches;
        # update + accumulate: 20 B per parameter), one event pair per launch
        commit_ids = [knames.index("commit_kernel"), knames.index("commit_acc4_kernel")]
        tr.ctx.kernel_timer_enable(commit_ids)
        tr.s_seq(lr, 1, 8, record_loss=False)
        tr.s_seq_grad(lr, 1, 8, record_loss=False)
        torch.cuda.synchronize()
        for kid in commit_ids:
            n, ms, work = tr.ctx.kernel_timer_read(kid)
            if n:
                forms[knames[kid]] = {"avg_us": 1e3 * ms / n, "bytes_per_launch": work / n,
                                      "GBps": work / (ms * 1e-3) / 1e9,
                                      "frac_hbm_peak": work / (ms * 1e-3) / (PEAK_HBM_GBS * 1e9)}
        tr.ctx.kernel_timer_enable([])
        # what a pure-MFMA loop of this workload's operand type sustains on this chip right now
        prec = "bf16" if cfg.get("prec") == "bf16" else "fp32"
        probe = {"dtype": prec, **mfma_probe(hb, torch, dev, prec)}

    del tr
    torch.cuda.empty_cache()
    if not args.no_extras:
        # ---- the other single-GPU configurations in the same schedule (parity cases; extra keys)
        others = {name: quick_workload(torch, wl, harness, name, dev)
                  for name in ("gru_cls", "mlp", "gru_lm") if name != args.workload}
        torch.cuda.empty_cache()
        # ---- this workload with "make replica" as a copy of its own (hpsgd_sync_all writes the K clones,
        # the local step runs in place): the same bits as the headline's schedule, more bytes
        written_out = quick_workload(torch, wl, harness, args.workload, dev, implicit_clone=False,
                                     prepare=False if args.prepare == "off" else args.prepare)
        written_out.pop("workload")
        torch.cuda.empty_cache()

    # ---- merge-only stress (config 5): merge + sync of 100M floats, K = 8, pure HBM streaming
    merge_stress = None
    if not args.no_merge_stress:
        c5 = wl.CONFIGS["merge_stress"]
        P5, K5, iters = c5["P"], c5["K"], c5["iters"]
        gen = torch.Generator(device=dev).manual_seed(wl.BASE_SEED)
        G = torch.rand(P5, device=dev, generator=gen) * 2 - 1
        S = torch.empty_like(G)
        R = torch.empty(K5, P5, device=dev)
        reps = list(R)
        hb.sync_all(G, reps, S)
        for k in range(K5):
            R[k].add_(torch.randn(P5, device=dev, generator=gen) * 1e-3)
        st = torch.cuda.current_stream()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * iters + 1)]
        for _ in range(3):
            hb.merge(G, reps, S)
            hb.sync_all(G, reps, S)
        torch.cuda.synchronize()
        ev[0].record(st)
        for i in range(iters):
            hb.merge(G, reps, S)
            ev[2 * i + 1].record(st)
            hb.sync_all(G, reps, S)
            ev[2 * i + 2].record(st)
        torch.cuda.synchronize()
        tm = [ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(iters)]
        ts = [ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(iters)]
        t_merge, t_sync = sum(tm) / iters, sum(ts) / iters
        bm, bs = 4.0 * (K5 + 3) * P5, 4.0 * (K5 + 2) * P5
        # merge and clone of the same generation as one pass (hpsgd_merge_sync, 4 (2K + 4) B/param)
        fe = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        for _ in range(3):
            hb.merge_sync(G, reps, S)
        fe[0].record(st)
        for i in range(iters):
            hb.merge_sync(G, reps, S)
            fe[i + 1].record(st)
        torch.cuda.synchronize()
        tf = [fe[i].elapsed_time(fe[i + 1]) for i in range(iters)]
        t_fused = sum(tf) / iters
        bf_ = 4.0 * (2 * K5 + 4) * P5
        # the gradient-form merge (Eq. 1 as printed) on the same buffers taken as accumulators
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            hb.merge_grad(G, reps, 1e-3)
        g0.record(st)
        for _ in range(iters):
            hb.merge_grad(G, reps, 1e-3)
        g1.record(st)
        torch.cuda.synchronize()
        t_mg = g0.elapsed_time(g1) / iters
        merge_stress = {
            "workload": "config 5: flat fp32 vector P=1e8, K=8, merge+sync x50",
            "merge_ms": t_merge, "merge_ms_median": statistics.median(tm), "merge_ms_min": min(tm),
            "merge_GBps": bm / t_merge / 1e6, "merge_frac_hbm": bm / t_merge / 1e6 / PEAK_HBM_GBS,
            "sync_ms": t_sync, "sync_ms_median": statistics.median(ts), "sync_ms_min": min(ts),
            "sync_GBps": bs / t_sync / 1e6, "sync_frac_hbm": bs / t_sync / 1e6 / PEAK_HBM_GBS,
            "merge_plus_sync_ms": t_merge + t_sync,
            "merge_plus_sync_GBps": (bm + bs) / (t_merge + t_sync) / 1e6,
            "merge_plus_sync_frac_hbm": (bm + bs) / (t_merge + t_sync) / 1e6 / PEAK_HBM_GBS,
            "merge_sync_one_pass_ms": t_fused, "merge_sync_one_pass_ms_median": statistics.median(tf),
            "merge_sync_one_pass_ms_min": min(tf), "merge_sync_one_pass_GBps": bf_ / t_fused / 1e6,
            "merge_sync_one_pass_frac_hbm": bf_ / t_fused / 1e6 / PEAK_HBM_GBS,
            "merge_grad_ms": t_mg, "merge_grad_GBps": bs / t_mg / 1e6, "merge_grad_frac_hbm": bs / t_mg / 1e6 / PEAK_HBM_GBS,
        }
        del G, S, R, reps
        torch.cuda.empty_cache()

    # ---- CPU baseline: the float64 oracle on the host cores, same workload, bounded sample
    cpu, cpu_1t = None, None
    if not args.no_cpu_baseline:
        from oracle import hpsgd_oracle as oc
        try:
            from threadpoolctl import threadpool_info, threadpool_limits
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threadpool_limits = None
            cores = os.cpu_count()

        def oracle_rate(name, min_rounds, min_seconds):
            c = wl.CONFIGS[name]
            ini = init if name == args.workload else wl.init_params(c)
            shs = shards if name == args.workload else [wl.make_shard(c, k) for k in range(c["K"])]
            bf = lambda k, s: oc.gather_batch(c["kind"], shs[k][0], shs[k][1], wl.batch_indices(c, k, s))
            rounds, el = 0, 0.0
            c0 = time.perf_counter()
            while rounds < min_rounds or el < min_seconds:
                oc.s_seq(ini, bf, c["K"], c["lr"], gamma=1, rounds=1)
                rounds += 1
                el = time.perf_counter() - c0
            return samples_per_round(c) * rounds / el, rounds, el

        # the headline workload: 2 rounds at least (config 3 is about 1.1 TFLOP of float64 per round)
        v, rounds, el = oracle_rate(args.workload, 2, 10.0 if cfg["kind"] != "gru_lm" else 0.0)
        cpu = {"value": v, "unit": unit, "cores": int(cores), "kind": "oracle",
               "sample": f"{rounds} rounds of (local step of all {K} workers + merge + sync) on the same "
                         f"{args.workload} inputs, float64 numpy, {el:.1f} s"}
        # one thread, configs 1, 2 and 4
        if threadpool_limits is not None and not args.no_extras:
            cpu_1t = {}
            with threadpool_limits(limits=1):
                for name in ("tiny_gru", "gru_cls", "mlp"):
                    v, rounds, el = oracle_rate(name, 1, 2.0)
                    cpu_1t[name] = {"value": v, "unit": "samples/s", "cores": 1, "kind": "oracle",
                                    "sample": f"{rounds} rounds, {el:.1f} s"}

    out = {
        "metric": "local-step samples/sec (overlapped HPSGD round: gather + local step + merge + sync)",
        "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.get("prec") == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload], "global_batch": K * B,
                   "seq_len": cfg.get("seq_len"), "parallelism": f"1 GPU, K={K} simulated workers",
                   "make_replica": "part of the local step: it reads the one model the replicas are clones of and "
                                   "writes all K updated replicas (hpsgd_local_step_all_cloned; bit-identical to "
                                   "hpsgd_sync_all + the step in place, which `written_out_clones` times)"},
        "roofline": roofline, "cpu_baseline": cpu, "ms_per_step_spread": spread, "overlap": overlap,
        "kernels": kernels, "hip_graph_replay": graph_replay, "merge_stress": merge_stress, "other_workloads": others,
        "written_out_clones": written_out,
        "cpu_baseline_one_thread": cpu_1t,
        "recurrence_launches": {"resident_weight_layers": fused[0], "with_input_projection": fused[1],
                                "with_dW_hh_and_bias_gradients": fused[2]},
        "mfma_probe": probe, "async_driver": async_driver, "schedules_under_sync_latency": compare,
        "synchronisation_forms": forms,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
