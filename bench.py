#!/usr/bin/env python3
"""Benchmark of the HPSGD hot path on one MI355X.

One "step" is one round of the overlapped schedule on the GRU classifier workload
(config 2: I128 H512 T35 B64, K=4 workers, fp32): batch gather, local step of all K workers
(forward, BPTT, SGD commit) on stream A, merge of the previous round on stream B, and the
replica sync at the round boundary.  Inputs (shards, parameters) are resident in HBM before
the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of a role's kernel on the default workload (one launch = the recurrence of
# all 35 time steps of the layer, all 4 workers), from two rocprofv3 --pmc runs
# (FETCH_SIZE scaled by 2.0, WRITE_SIZE by 1.0 after calibration with a plain 1 GiB copy kernel;
# summary in profiles/pmc_hbm_traffic_gru_cls_and_merge.md).  Configs 3 and 4: the role's launches of one
# step added up and divided by the launches the role's timer counts, like `achieved`
# (profiles/pmc_hbm_traffic_gru_lm_and_mlp.md).  Other roles: not collected (null).
MEASURED_TRAFFIC_BYTES = {
    "gru_cls": {"gemm_recurrent_bwd": (2.0 * 84280.5 + 133496.3) * 1024, "gemm_recurrent_fwd": (2.0 * 27504.8 + 89880.0) * 1024},
    # logits GEMM + head dX + head dW with update + bias-gradient reduction, 5 timed launches
    "gru_lm": {"gemm_head": ((2.0 * 185896.3 + 351619.4) + (2.0 * 168394.5 + 35840.0) + (2.0 * 296277.5 + 320924.6)
                             + (2.0 * 22242.0 + 312.5)) * 1024 / 5},
    # dX and dW GEMMs of layers 3 and 2, dW of layer 1, the bias/loss column sums: 6 launches
    "mlp": {"mlp_bwd": ((2.0 * 4942.5 + 8192.0) + (2.0 * 5017.5 + 710.3) + (2.0 * 41198.8 + 8192.0)
                        + (2.0 * 37054.7 + 65536.4) + (2.0 * 29373.9 + 50233.4) + (2.0 * 8337.2 + 136.3)) * 1024 / 6},
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


def role_work_per_step(cfg, role_name, commit_params=None, fused=(0, 0, 0)):
    """Algorithmic work of ALL launches of a role in one local step of all K workers:
    (bound, flops or bytes per step, peak in the same unit per second).  commit_params: how many
    parameters per worker the commit kernel handled (the rest are updated in GEMM epilogues).
    fused = (resident, xproj, dw) from Context.recurrence_info(): the bottom `xproj` layers' input
    projections are part of the forward recurrence launches and the top-to-bottom first `dw`
    layers' dW_hh products part of the backward ones (every layer when dw == layers), so their
    flops are counted with those roles."""
    kind, K, B = cfg["kind"], cfg["K"], cfg["batch"]
    mfma_peak = (PEAK_BF16_MFMA_TFLOPS if cfg.get("prec") == "bf16" else PEAK_FP32_MFMA_TFLOPS) * 1e12
    hbm = PEAK_HBM_GBS * 1e9
    if kind == "mlp":
        d = cfg["dims"]
        fwd = sum(2.0 * B * d[i] * d[i + 1] for i in range(len(d) - 1)) * K
        bwd = (sum(2.0 * B * d[i] * d[i + 1] for i in range(len(d) - 1))
               + sum(2.0 * B * d[i] * d[i + 1] for i in range(1, len(d) - 1))) * K
        P = sum(d[i] * d[i + 1] + d[i + 1] for i in range(len(d) - 1))
        if commit_params is not None:
            P = commit_params
        return {"mlp_fwd": ("mfma", fwd, mfma_peak), "mlp_bwd": ("mfma", bwd, mfma_peak),
                "commit": ("hbm", 12.0 * P * K, hbm)}.get(role_name, (None, None, None))
    T, H, L = cfg["seq_len"], cfg["hidden"], cfg["layers"]
    TB = T * B
    lm = kind == "gru_lm"
    widths = [cfg["embed"] if lm else cfg["input"]] + [H] * (L - 1)
    classes = cfg["vocab"] if lm else cfg["classes"]
    nrows = TB if lm else B
    P = sum(3 * H * w + 3 * H * H + 6 * H for w in widths) + classes * H + classes + (cfg["vocab"] * cfg["embed"] if lm else 0)
    if commit_params is not None:
        P = commit_params
    _, n_xproj, n_dw = fused
    # a layer's input projection is fused only where its input is narrow: the narrowest first
    xproj_flops = sum(sorted(2.0 * TB * 3 * H * w for w in widths)[:n_xproj]) * K
    dw_flops = n_dw * 2.0 * 3 * H * H * TB * K
    table = {
        "gemm_input_projection": ("mfma", sum(2.0 * TB * 3 * H * w for w in widths) * K - xproj_flops, mfma_peak),
        "gemm_recurrent_fwd": ("mfma", 2.0 * B * 3 * H * H * T * L * K + xproj_flops, mfma_peak),
        "gemm_recurrent_bwd": ("mfma", 2.0 * B * 3 * H * H * T * L * K + dw_flops, mfma_peak),
        "gemm_weight_grad": ("mfma", sum(2.0 * 3 * H * w * TB + 2.0 * 3 * H * H * TB for w in widths) * K - dw_flops,
                             mfma_peak),
        "gemm_input_grad": ("mfma", sum(2.0 * TB * 3 * H * w for w in (widths if lm else widths[1:])) * K, mfma_peak),
        "gemm_head": ("mfma", 3 * 2.0 * nrows * classes * H * K, mfma_peak),
        "gru_cell_fwd": ("hbm", 48.0 * B * H * T * L * K, hbm),
        "gru_cell_bwd": ("hbm", 56.0 * B * H * T * L * K, hbm),
        "softmax_ce": ("hbm", 8.0 * nrows * classes * K, hbm),
        "commit": ("hbm", 12.0 * P * K, hbm),
    }
    return table.get(role_name, (None, None, None))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-merge-stress", action="store_true")
    ap.add_argument("--prepare", action="store_true",
                    help="make the next step's bf16 weight copies on the synchronising stream (measured slower)")
    ap.add_argument("--workload", default="gru_cls", choices=["gru_cls", "gru_lm", "mlp", "tiny_gru"],
                    help="default: config 2, the one the headline metric is quoted on")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (K workers are a group dimension on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2009_02701_amd import binding as hb
    from paper_2009_02701_amd import harness, workloads as wl

    dev = "cuda:0"
    cfg = wl.CONFIGS[args.workload]
    K, B, lr = cfg["K"], cfg["batch"], cfg["lr"]
    init = wl.init_params(cfg)
    shards = [wl.make_shard(cfg, k) for k in range(K)]
    orders = [wl.batch_order(cfg, k) for k in range(K)]
    tr = harness.Trainer(cfg, init, shards, orders, device=dev, prepare=args.prepare)
    names = tr.ctx.role_names()

    # ---- pass 0: which role dominates the local step (all roles timed, a few rounds)
    tr.ovl_begin()
    for t in range(3):
        tr.ovl_round(t, lr)
    torch.cuda.synchronize()
    tr.ctx.timer_enable(range(hb.ROLE_COUNT))
    probe_rounds = 5
    for t in range(probe_rounds):
        tr.ovl_round(3 + t, lr)
    torch.cuda.synchronize()
    breakdown = {}
    for r, nm in enumerate(names):
        n, ms = tr.ctx.timer_read(r)
        if n:
            breakdown[nm] = {"launches_per_step": n / probe_rounds, "avg_us": 1e3 * ms / n,
                             "us_per_step": 1e3 * ms / probe_rounds}
    commit_params = tr.ctx.commit_kernel_params()
    fused = tr.ctx.recurrence_info()
    dominant = max(breakdown, key=lambda k: breakdown[k]["us_per_step"])
    dom_role = names.index(dominant)
    tr.ctx.timer_enable([dom_role])

    # ---- warm-up, then the timed region: `value` comes from K rounds with no instrumentation
    tr.ctx.timer_enable([])
    step = 3 + probe_rounds
    for t in range(args.warmup):
        tr.ovl_round(step, lr)
        step += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.steps):
        tr.ovl_round(step, lr)
        step += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = 1e3 * (t1 - t0) / args.steps
    samples_per_step = K * B * (cfg["seq_len"] if cfg["kind"] == "gru_lm" else 1)
    unit = "tokens/s" if cfg["kind"] == "gru_lm" else "samples/s"
    value = samples_per_step / (ms_per_step * 1e-3)

    # ---- the same region once more with HIP event pairs around every launch of the dominant
    # role (on the stream the kernels run on): the roofline's launch duration
    tr.ctx.timer_enable([dom_role])
    tr.ctx.timer_read(dom_role)
    t2 = time.perf_counter()
    for t in range(args.steps):
        tr.ovl_round(step, lr)
        step += 1
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    n_dom, ms_dom = tr.ctx.timer_read(dom_role)
    tr.ctx.timer_enable([])
    tr.ovl_drain()
    ms_per_step_instrumented = 1e3 * (t3 - t2) / args.steps

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
                             "max_steps_per_round": max(counts), "value": 60 * samples_per_step / (a1 - a0),
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
        compare[name] = 64 * samples_per_step / (time.perf_counter() - c0)

    # gradient-form synchronisation (Eq. 1 as printed): blocking rounds of one local step, for the
    # cost of accumulating gradients (no update in GEMM epilogues) next to the delta form
    forms = {"unit": unit}
    for name, run in (("delta_form_s_seq", lambda: tr.s_seq(lr, 1, 32, record_loss=False)),
                      ("gradient_form_s_seq_grad", lambda: tr.s_seq_grad(lr, 1, 32, record_loss=False))):
        run()
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        run()
        forms[name] = 32 * samples_per_step / (time.perf_counter() - c0)

    bound, work, peak = role_work_per_step(cfg, dominant, commit_params, fused)
    roofline = None
    if bound is not None and n_dom:
        dur = ms_dom * 1e-3 / n_dom
        ach = work / breakdown[dominant]["launches_per_step"] / dur
        scale = 1e12 if bound == "mfma" else 1e9
        roofline = {"kernel": dominant, "bound": bound, "achieved": ach / scale, "peak": peak / scale,
                    "unit": "TFLOP/s" if bound == "mfma" else "GB/s", "frac": ach / peak,
                    "avg_launch_us": dur * 1e6, "launches_timed": n_dom,
                    "ms_per_step_with_event_pairs": ms_per_step_instrumented,
                    "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload, {}).get(dominant)}
    for nm, v in breakdown.items():
        b_, w_, p_ = role_work_per_step(cfg, nm, commit_params, fused)
        if b_ is not None:
            v["frac_of_peak"] = w_ / (v["us_per_step"] * 1e-6) / p_
            v["bound"] = b_

    # ---- merge-only stress (config 5): merge + sync of 100M floats, K = 8, pure HBM streaming
    merge_stress = None
    if not args.no_merge_stress:
        c5 = wl.CONFIGS["merge_stress"]
        P5, K5, iters = c5["P"], c5["K"], c5["iters"]
        del tr
        torch.cuda.empty_cache()
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
        t_merge = sum(ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(iters)) / iters
        t_sync = sum(ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(iters)) / iters
        bm, bs = 4.0 * (K5 + 3) * P5, 4.0 * (K5 + 2) * P5
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
            "workload": "flat fp32 vector P=1e8, K=8, merge+sync x50",
            "merge_ms": t_merge, "merge_GBps": bm / t_merge / 1e6, "merge_frac_hbm": bm / t_merge / 1e6 / PEAK_HBM_GBS,
            "sync_ms": t_sync, "sync_GBps": bs / t_sync / 1e6, "sync_frac_hbm": bs / t_sync / 1e6 / PEAK_HBM_GBS,
            "merge_plus_sync_GBps": (bm + bs) / (t_merge + t_sync) / 1e6,
            "merge_grad_ms": t_mg, "merge_grad_GBps": bs / t_mg / 1e6, "merge_grad_frac_hbm": bs / t_mg / 1e6 / PEAK_HBM_GBS,
        }
        del G, S, R, reps
        torch.cuda.empty_cache()

    # ---- CPU baseline: the float64 oracle on the host cores, same workload, bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import hpsgd_oracle as oc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        bf = lambda k, s: wl.host_batch(cfg, shards[k], wl.batch_indices(cfg, k, s))
        oc.s_seq(init, bf, K, lr, gamma=1, rounds=1)   # warm
        rounds, el = 0, 0.0
        c0 = time.perf_counter()
        while el < 10.0 or rounds < 2:
            oc.s_seq(init, bf, K, lr, gamma=1, rounds=1)
            rounds += 1
            el = time.perf_counter() - c0
        cpu = {"value": samples_per_step * rounds / el, "unit": unit, "cores": int(cores), "kind": "oracle",
               "sample": f"{rounds} rounds of (local step of all {K} workers + merge + sync) on the same "
                         f"{args.workload} inputs, float64 numpy, {el:.1f} s"}

    # what a pure-MFMA loop of this workload's operand type sustains on this chip right now
    prec = "bf16" if cfg.get("prec") == "bf16" else "fp32"
    probe = {"dtype": prec, **mfma_probe(hb, torch, dev, prec)}
    out = {
        "metric": "local-step samples/sec (overlapped HPSGD round: gather + local step + merge + sync)",
        "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.get("prec") == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload], "global_batch": K * B,
                   "seq_len": cfg.get("seq_len"), "parallelism": f"1 GPU, K={K} simulated workers"},
        "roofline": roofline, "cpu_baseline": cpu, "kernels": breakdown, "merge_stress": merge_stress,
        "recurrence_launches": {"resident_weight_layers": fused[0], "with_input_projection": fused[1],
                                "with_dW_hh_and_bias_gradients": fused[2]},
        "mfma_probe": probe, "async_driver": async_driver, "schedules_under_sync_latency": compare,
        "synchronisation_forms": forms,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
