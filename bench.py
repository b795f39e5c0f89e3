#!/usr/bin/env python3
"""Benchmark of the freeze-aware stage backward + masked AdamW + APF EMAs on
one MI355X.

A "step" is one pass of the whole hot path over one synthetic microbatch:
  tf_stage_backward (dX for every layer, dW for unfrozen layers only)
  -> tf_masked_adamw fused with the stability EMAs and per-tensor score sums
  -> score sums to host -> tf_stability_scores -> tf_select_lowest.
The default run times the largest single-GPU configuration, the LLaMA-8B-shaped
stage (8 blocks, d=4096, GQA kv=1024, ffn=14336, 4096 tokens, bf16 with fp32
master weights and Adam states; the mask freezes the first ceil(r*L) tensors of
a seeded permutation): `value` is its tokens/s at r = 0.5, "sweep" its sweep
over r.  On the same tensors it then times the elementwise pass alone with
per-element Bernoulli masks ("elementwise_8b") and eight microbatches of 1024
tokens with fp32 accumulation ("microbatches_8b"), and finally the
LLaMA-1B-shaped stage with its five-point sweep ("llama1b_stage": lowest APF
scores after 5 seeded warm-up steps).  --workload N runs one of them alone.
Inputs are seeded and synthetic (workloads.py) and are resident in HBM before
the timed region starts.

One JSON line is printed on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E
HEADLINE_R = 0.5
PAPER_CONTEXT = ("paper: LLaMA-3-8B fine-tuning throughput +36..40% at average freeze ratio ~0.33-0.36, "
                 "4xH200 NVLink, PP=4, 8 microbatches (Table llama8b) - other hardware, context only")


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=0, choices=[0, 2, 3, 4, 5, 6, 7, 8],
                    help="0 = the benchmark line (LLaMA-8B stage, then the elementwise pass and the 8 microbatches on "
                         "its tensors, then the LLaMA-1B stage); config id: 2 = LLaMA-1B-shaped stage; 3 = LLaMA-8B stage; "
                         "4 = elementwise pass only, Bernoulli element masks; 5 = 8 microbatches with fp32 dW accumulation; "
                         "6 = selection steps on the 8B stage's tensors (AutoFreeze norms, Alg. 2 budget reconciliation); "
                         "7 = the benchmark stage with sub-tensor freezing (256-row blocks drawn under the parameter budget r P); "
                         "8 = the benchmark stage with q/k/v and gate/up sharing their input (one dX per group)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    return ap.parse_args()


class Stage:
    """All device buffers of one stage, filled from the seeded generators."""

    def __init__(self, cfg, wl, tf, torch):
        def dev(a, dtype):
            if dtype == "bf16":
                bits = wl.f32_to_bf16_bits(a).view(np.int16)
                return torch.from_numpy(bits).cuda().view(torch.bfloat16).reshape(a.shape)
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()

        self.cfg, self.tf, self.torch = cfg, tf, torch
        self.shapes = cfg.shapes
        self.L = cfg.n_layers
        self.T = cfg.T
        self.sizes = [k * n for k, n in self.shapes]
        t0 = time.time()

        def make(l):
            p = wl.gen_weight(cfg, l)
            _, X, dY = wl.gen_layer(cfg, l)
            return p, X, dY

        with ThreadPoolExecutor(max_workers=8) as ex:
            host = list(ex.map(make, range(self.L)))
        log(f"generated inputs for {self.L} layers in {time.time() - t0:.1f}s")
        bf, f32 = torch.bfloat16, torch.float32
        self.p = [dev(h[0].reshape(-1), "f32") for h in host]
        self.W = [dev(h[0], "bf16") for h in host]                 # stored bf16 copy of the master weights
        self.X = [dev(h[1], "bf16") for h in host]
        self.dY = [dev(h[2], "bf16") for h in host]
        del host
        z = lambda dt: [torch.zeros(n, dtype=dt, device="cuda") for n in self.sizes]
        self.m, self.v, self.E, self.A = z(f32), z(f32), z(f32), z(f32)
        self.dX = [torch.empty((self.T, k), dtype=bf, device="cuda") for k, n in self.shapes]
        self.dW = [torch.zeros((k, n), dtype=bf, device="cuda") for k, n in self.shapes]
        self.sums = torch.zeros(2 * self.L, dtype=torch.float64, device="cuda")
        self.sums_host = torch.zeros(2 * self.L, dtype=torch.float64, pin_memory=True)
        # the same buffers go to the library step after step: marshal their pointers once
        for name in ("p", "W", "X", "dY", "m", "v", "E", "A", "dX", "dW"):
            setattr(self, name, tf.PtrTable(getattr(self, name)))
        self.steps = [1] * self.L
        self.hp = {k: float(np.float32(getattr(cfg, k))) for k in ("lr", "beta1", "beta2", "eps", "weight_decay")}
        self.decay = float(np.float32(cfg.ema_decay))
        torch.cuda.synchronize()
        log(f"device buffers ready, {torch.cuda.memory_allocated() / 2**30:.1f} GiB")

    def adamw(self, ctx, grads, mask):
        hp = self.hp
        self.tf.tf_masked_adamw(ctx, self.sizes, self.p, self.m, self.v, grads, self.tf.TF_BF16, self.steps,
                                hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"],
                                p_lowp=self.W, tensor_freeze_mask=mask, ema=self.E, ema_abs=self.A,
                                ema_decay=self.decay, score_sums=self.sums)
        for l in range(self.L):
            if mask is None or not mask[l]:
                self.steps[l] += 1

    def step(self, ctx, mask, n_freeze):
        """One pass of the hot path; returns the mask the scores would pick next."""
        tf = self.tf
        tf.tf_stage_backward(ctx, self.shapes, self.T, tf.TF_BF16, self.W, self.X, self.dY, mask,
                             self.dX, self.dW, tf.TF_BF16)
        self.adamw(ctx, self.dW, mask)
        self.sums_host.copy_(self.sums, non_blocking=True)       # into pinned memory: no staging copy
        self.torch.cuda.current_stream().synchronize()           # the step ends here: the scores pick the next mask
        scores = tf.tf_stability_scores(self.sums_host.numpy())
        return tf.tf_select_lowest(scores, n_freeze)


def cpu_baseline(cfg, wl, r):
    """Time the fp64 oracle on a bounded sample of the same workload: block 0's
    seven layers, the first Ts tokens, backward at ratio r + AdamW/EMA step."""
    import oracle
    Ts = 2048 if cfg.d <= 2048 else 768          # about 10-20 s of host work either way
    sub = wl.scaled(cfg, blocks=1)
    sh = sub.shapes
    mask = wl.permutation_mask(sub, r)
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    W, X, dY = zip(*[wl.gen_layer(sub, l, T=Ts) for l in range(7)])
    W, X, dY = [f64(a) for a in W], [f64(a) for a in X], [f64(a) for a in dY]
    dX = [np.zeros((Ts, k)) for k, n in sh]
    dW = [None if mask[l] else np.zeros(sh[l]) for l in range(7)]
    t0 = time.perf_counter()
    oracle.stage_backward(sh, Ts, W, X, dY, mask, dX, dW)
    t_bwd = time.perf_counter() - t0
    hp = {k: getattr(cfg, k) for k in ("lr", "beta1", "beta2", "eps", "weight_decay")}
    t_opt = 0.0
    for l in range(7):
        if mask[l]:
            continue
        n = sh[l][0] * sh[l][1]
        st = [np.ones(n) * 1e-3 for _ in range(5)]               # touched pages: time the arithmetic, not the faults
        g = dW[l].reshape(-1)
        t0 = time.perf_counter()
        oracle.masked_adamw(st[0], st[1], st[2], g, step=1, ema=st[3], ema_abs=st[4], ema_decay=cfg.ema_decay, **hp)
        t_opt += time.perf_counter() - t0
    # one full step = backward over T tokens of all blocks + optimizer over all blocks
    t_full = t_bwd * (cfg.T / Ts) * cfg.blocks + t_opt * cfg.blocks
    return {
        "value": cfg.T / t_full, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": f"block 0 of {cfg.blocks} (7 layers), first {Ts} of {cfg.T} tokens, r={r} "
                  f"({int(mask.sum())}/7 tensors frozen): backward {t_bwd:.2f}s + AdamW/EMA {t_opt:.2f}s measured, "
                  f"scaled by tokens and blocks to a full step of {t_full:.0f}s",
    }


TRAFFIC_NOTE = ("HBM bytes per launch from separate rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this workload, "
                "calibrated on a 1 GiB copy and recorded in profiles/hbm_traffic.txt; not counted in this run")


def warmup_scores(cfg, st, ctx, wl, tf, torch):
    """cfg 2's mask source: 5 seeded optimizer steps with nothing frozen, then the APF scores."""
    t0 = time.time()
    for s in range(1, 6):
        with ThreadPoolExecutor(max_workers=8) as ex:
            grads = list(ex.map(lambda l: wl.f32_to_bf16_bits(wl.gen_grad(cfg, l, s)).view(np.int16), range(st.L)))
        gd = [torch.from_numpy(g).cuda().view(torch.bfloat16) for g in grads]
        st.adamw(ctx, gd, None)
        torch.cuda.synchronize()
        del gd, grads
    scores = tf.tf_stability_scores(st.sums.cpu().numpy())
    log(f"warm-up optimizer steps done in {time.time() - t0:.1f}s; score range {scores.min():.4f}..{scores.max():.4f}")
    return scores


def stage_report(args, cfg, st, ctx, wl, tf, torch, headline_r, sweep_rs, zero_operands):
    """Times the whole step of one stage configuration at headline_r and over sweep_rs; returns
    (head, sweep, rooflines) with the per-kernel event times of the launches of the timed steps."""
    L, T, P = st.L, st.T, cfg.n_params
    # cfg 2: lowest APF scores after the warm-up steps; cfg 3: first ceil(r L) of a seeded permutation
    scores = warmup_scores(cfg, st, ctx, wl, tf, torch) if cfg.cfg_id == 2 else None

    def run(r, steps, warmup):
        n = tf.tf_num_frozen(r, L)
        mask = tf.tf_select_lowest(scores, n) if scores is not None else wl.permutation_mask(cfg, r)
        phi = wl.frozen_param_fraction(cfg, mask)
        for _ in range(warmup):
            st.step(ctx, mask, n)
        torch.cuda.synchronize()
        ctx.profile_enable(True)
        ctx.profile_collect()
        gc.collect()
        gc.disable()            # a generational collection of the interpreter costs tens of ms
        t0 = time.perf_counter()
        for _ in range(steps):
            st.step(ctx, mask, n)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        gc.enable()
        prof = ctx.profile_collect()
        ctx.profile_enable(False)
        per_kind = {}
        for k, ms in prof:
            per_kind.setdefault(k, []).append(ms)
        kern = {k: {"launches_per_step": len(v) / steps, "avg_ms": float(np.mean(v))} for k, v in per_kind.items()}
        ms_step = dt / steps * 1e3
        flops = 2.0 * T * P * (2.0 - phi)
        unfrozen = sum(st.sizes[l] for l in range(L) if not mask[l])
        out = {"r": r, "n_frozen": int(n), "phi": phi, "ms_per_step": ms_step, "tokens_per_s": T / (ms_step / 1e3),
               "tflops": flops / (ms_step / 1e3) / 1e12, "kernels": kern}
        g_ms = sum(v["avg_ms"] * v["launches_per_step"] for k, v in kern.items() if k.startswith("d"))
        out["backward_ms"] = g_ms
        out["backward_tflops"] = flops / (g_ms / 1e3) / 1e12 if g_ms > 0 else None
        out["backward_pct_mfma_peak"] = 100.0 * out["backward_tflops"] / PEAK_BF16_TFLOPS if g_ms > 0 else None
        if "adamw" in kern:
            a_ms = kern["adamw"]["avg_ms"] * kern["adamw"]["launches_per_step"]
            out["adamw_ms"] = a_ms
            out["adamw_gbps"] = 44.0 * unfrozen / (a_ms / 1e3) / 1e9
            out["adamw_pct_hbm_peak"] = 100.0 * out["adamw_gbps"] / PEAK_HBM_GBPS
        return out

    head = run(headline_r, args.steps, args.warmup)
    head["mask"] = ("ceil(r*L) lowest APF scores after 5 seeded warm-up steps" if scores is not None
                    else "first ceil(r*L) entries of a seeded permutation")
    log(f"cfg{cfg.cfg_id} r={headline_r}: {head['ms_per_step']:.3f} ms/step, {head['tokens_per_s']:.0f} tok/s, "
        f"backward {head['backward_tflops']:.0f} TFLOP/s")
    sweep = []
    for r in sweep_rs:
        s = run(r, args.steps, 2) if r != headline_r else head
        sweep.append(s)
        log(f"cfg{cfg.cfg_id} sweep r={r}: phi={s['phi']:.3f} {s['ms_per_step']:.3f} ms/step, backward {s['backward_ms']:.3f} ms")
    t_by_r = {s["r"]: s for s in sweep}
    if 0.0 in t_by_r and 1.0 in t_by_r:
        b0, b1 = t_by_r[0.0]["backward_ms"], t_by_r[1.0]["backward_ms"]
        for s in sweep:
            if 0.0 < s["r"] < 1.0 and s["phi"] > 0:
                # time saved relative to what the skipped dW FLOP fraction would ideally save
                s["eta_backward"] = (b0 - s["backward_ms"]) / (s["phi"] * (b0 - b1))
                d0 = t_by_r[0.0]["kernels"].get("dw_mfma", {}).get("avg_ms")
                dr = s["kernels"].get("dw_mfma", {}).get("avg_ms")
                if d0 and dr:   # the same slope on the dW kernel alone (dX does not depend on r)
                    s["eta_dw_kernel"] = (d0 - dr) / (s["phi"] * d0)

    # ---- roofline of the dominant kernel: the grouped input-gradient GEMM ----
    roof = {}
    dx = head["kernels"].get("dx_mfma")
    if dx:
        fl = 2.0 * T * P / dx["launches_per_step"]
        ach = fl / (dx["avg_ms"] / 1e3) / 1e12
        roof["roofline"] = {"kernel": "gemm_mfma_kernel<NT> (dX = dY W^T, all layers, one grouped launch)",
                            "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                            "frac": ach / PEAK_BF16_TFLOPS, "traffic": read_traffic("dx_mfma", cfg.cfg_id),
                            "traffic_source": TRAFFIC_NOTE, "avg_launch_ms": dx["avg_ms"], "flop_per_launch": fl}
    if dx and zero_operands:
        # The same launch on all-zero operands.  Data decides how far the chip can clock under its
        # power limit: with nothing toggling in the matrix cores the clock stays near its maximum
        # and the figure shows what the instruction stream itself delivers.  Context for `frac`,
        # which is measured on the seeded inputs above.
        zW = [torch.zeros_like(st.W[l]) for l in range(L)]
        zdY = [torch.zeros_like(st.dY[l]) for l in range(L)]
        all_frozen = np.ones(L, dtype=np.uint8)

        def dx_only():
            tf.tf_stage_backward(ctx, st.shapes, st.T, tf.TF_BF16, zW, st.X, zdY, all_frozen, st.dX, st.dW, tf.TF_BF16)

        n_warm = max(4, int(120.0 / dx["avg_ms"]))              # the clock settles over the first 100 ms of load
        for _ in range(n_warm):
            dx_only()
        torch.cuda.synchronize()
        ctx.profile_enable(True)
        ctx.profile_collect()
        for _ in range(20):
            dx_only()
        torch.cuda.synchronize()
        ms0 = [ms for k, ms in ctx.profile_collect() if k == "dx_mfma"]
        ctx.profile_enable(False)
        del zW, zdY
        if ms0:
            ach0 = 2.0 * T * P / (float(np.sum(ms0)) / 20 / 1e3) / 1e12
            roof["roofline"]["achieved_zero_operands"] = ach0
            roof["roofline"]["frac_zero_operands"] = ach0 / PEAK_BF16_TFLOPS
            log(f"cfg{cfg.cfg_id} dX launch on all-zero operands: {ach0:.0f} TFLOP/s")
    dw = head["kernels"].get("dw_mfma")
    if dw:
        fl = 2.0 * T * P * (1.0 - head["phi"]) / dw["launches_per_step"]
        ach = fl / (dw["avg_ms"] / 1e3) / 1e12
        roof["roofline_dw"] = {"kernel": "gemm_mfma_kernel<TN> (dW = X^T dY, unfrozen layers only)", "bound": "mfma",
                               "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                               "frac": ach / PEAK_BF16_TFLOPS, "traffic": read_traffic("dw_mfma", cfg.cfg_id),
                               "traffic_source": TRAFFIC_NOTE, "avg_launch_ms": dw["avg_ms"]}
    if "adamw_gbps" in head:
        roof["roofline_adamw"] = {"kernel": "ew_kernel (masked AdamW + APF EMAs + score sums)", "bound": "hbm",
                                  "achieved": head["adamw_gbps"], "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                  "frac": head["adamw_gbps"] / PEAK_HBM_GBPS,
                                  "traffic": read_traffic("adamw", cfg.cfg_id), "traffic_source": TRAFFIC_NOTE,
                                  "avg_launch_ms": head["adamw_ms"]}
    return head, sweep, roof


def lp_example(sweep, tf):
    """What the measured times mean for the method (context, not a metric): a 4-stage, 8-microbatch
    pipeline of such stages, every backward action between the measured r = 1 and r = 0 times,
    forward = the r = 1 backward (same GEMM FLOPs as dX), through the freeze-ratio linear program."""
    t_by_r = {x["r"]: x for x in sweep}
    if 0.0 not in t_by_r or 1.0 not in t_by_r:
        return None
    S_, M_ = 4, 8
    hi, lo = t_by_r[0.0]["backward_ms"], t_by_r[1.0]["backward_ms"]
    w_max = np.r_[np.full(S_ * M_, lo), np.full(S_ * M_, hi)]
    w_min = np.r_[np.full(S_ * M_, lo), np.full(S_ * M_, lo)]
    ex = {}
    for name, sched, per_rank in (("gpipe", tf.TF_SCHEDULE_GPIPE, 1), ("1f1b", tf.TF_SCHEDULE_1F1B, 1),
                                  ("interleaved_1f1b", tf.TF_SCHEDULE_INTERLEAVED_1F1B, 2), ("zbv", tf.TF_SCHEDULE_ZBV, 2)):
        # two stages per rank: the same four ranks, every stage half of a measured one
        n = S_ * per_rank * M_
        lo_, hi_ = np.r_[w_min[:S_ * M_], w_min[S_ * M_:]] / per_rank, np.r_[w_max[:S_ * M_], w_max[S_ * M_:]] / per_rank
        sol = tf.tf_freeze_ratio_lp(S_ * per_rank, M_, sched, np.r_[np.full(n, lo_[0]), np.full(n, lo_[-1])],
                                    np.r_[np.full(n, hi_[0]), np.full(n, hi_[-1])], 0.8, 1e-4)
        ex[name] = {"batch_ms_no_freezing": sol["P_d_max"], "batch_ms_at_r_star": sol["P_d"],
                    "mean_r_star": float(np.mean(sol["r"][n:])),
                    "throughput_gain_pct": 100.0 * (sol["P_d_max"] / sol["P_d"] - 1.0)}
    return {"stages": S_, "microbatches": M_, "r_max": 0.8, "lambda": 1e-4, "backward_ms_r0": hi, "backward_ms_r1": lo, **ex}


def workload_name(cfg, L, P):
    return (f"cfg{cfg.cfg_id} {cfg.name}: {cfg.blocks} blocks, d={cfg.d}, kv={cfg.kv}, ffn={cfg.ffn}, "
            f"T={cfg.T} tokens, L={L} tensors, P={P} params")


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU's stage; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of this library).", file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads as wl
    import paper_2602_05754_amd as tf

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(tf.library_path()):
        raise RuntimeError("libtf.so has not been built (python -c 'import __graft_entry__ as g; g.build()')")
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = 1 << 30
        a = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n,
                          "GBps": 2 * n / dt / 1e9}), flush=True)
        return
    ctx = tf.Context(0)
    if args.workload in (4, 5, 6, 7, 8):
        cfg = wl.CONFIGS[{6: 3, 7: 2, 8: 2}.get(args.workload, args.workload)]
        fn = {4: bench_elementwise, 5: bench_microbatches, 6: bench_selection, 7: bench_row_blocks, 8: bench_shared_inputs}
        out = fn[args.workload](args, cfg, ctx, wl, tf, torch)
        ctx.close()
        print(json.dumps(out), flush=True)
        return

    # ---- the headline stage: cfg 3 by default (the largest configuration one GPU holds) ----
    cfg = wl.CONFIGS[2 if args.workload == 2 else 3]
    st = Stage(cfg, wl, tf, torch)
    L, P = st.L, cfg.n_params
    sweep_rs = [] if args.no_sweep else wl.R_SWEEP[cfg.cfg_id] + [1.0]
    head, sweep, roof = stage_report(args, cfg, st, ctx, wl, tf, torch, HEADLINE_R, sweep_rs, zero_operands=not args.no_sweep)
    line = {
        "metric": f"stage-backward tokens/s (freeze-aware backward + masked AdamW + APF EMAs), r={HEADLINE_R}",
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload_name(cfg, L, P), "r": HEADLINE_R, "n_frozen": head["n_frozen"],
                   "phi": head["phi"], "mask": head["mask"]},
        "tflops": head["tflops"], "roofline": roof.get("roofline"), "cpu_baseline": None, "sweep": sweep,
        "paper_context": PAPER_CONTEXT,
    }
    line.update({k: v for k, v in roof.items() if k != "roofline"})
    ex = lp_example(sweep, tf)
    if ex:
        line["schedule_lp_example"] = ex
    if args.workload == 0:
        # the other configurations, each with its own workload name and rooflines
        line["elementwise_8b"] = bench_elementwise(args, wl.CONFIGS[4], ctx, wl, tf, torch, st=st)
        line["microbatches_8b"] = bench_microbatches(args, wl.CONFIGS[5], ctx, wl, tf, torch, st=st)
        del st
        gc.collect()
        torch.cuda.empty_cache()
        cfg2 = wl.CONFIGS[2]
        st2 = Stage(cfg2, wl, tf, torch)
        h2, sw2, roof2 = stage_report(args, cfg2, st2, ctx, wl, tf, torch, HEADLINE_R, wl.R_SWEEP[2] + [1.0], zero_operands=False)
        line["llama1b_stage"] = {"workload": workload_name(cfg2, st2.L, cfg2.n_params), "r": HEADLINE_R, "mask": h2["mask"],
                                 "ms_per_step": h2["ms_per_step"], "tokens_per_s": h2["tokens_per_s"], "sweep": sw2, **roof2}
        ex2 = lp_example(sw2, tf)
        if ex2:
            line["llama1b_stage"]["schedule_lp_example"] = ex2
        del st2
    if not args.no_cpu_baseline:
        log("timing the fp64 oracle on a bounded sample (host cores)...")
        line["cpu_baseline"] = cpu_baseline(cfg, wl, HEADLINE_R)
        log(f"oracle: {line['cpu_baseline']['value']:.2f} tokens/s on {line['cpu_baseline']['cores']} threads")
    ctx.close()
    print(json.dumps(line), flush=True)


def _timed(ctx, torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    ctx.profile_collect()
    gc.collect()
    gc.disable()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    gc.enable()
    prof = ctx.profile_collect()
    ctx.profile_enable(False)
    return dt, prof


def bench_elementwise(args, cfg, ctx, wl, tf, torch, st=None):
    """cfg 4: masked AdamW + APF EMAs over the 8B stage's 1.74e9 parameters, dense and with per-element
    Bernoulli(r) masks.  Timing-only inputs: same distributions as workloads.py but drawn on the
    device (a seeded torch generator), because 3.5e9 host draws would take minutes; parity of this
    pass is covered by the tests at one block of the same tensors.  With `st` (a Stage of the same
    tensors) its master weights and states are used as they stand after the stage's steps."""
    sizes = [k * n for k, n in cfg.shapes]
    L, P = len(sizes), sum(sizes)
    g = torch.Generator(device="cuda").manual_seed(wl.SEED_BASE + 4)
    rn = lambda n, std, dt=torch.float32: (torch.randn(n, generator=g, device="cuda") * std).to(dt)
    if st is not None:
        p, m, v, E, A, low = st.p, st.m, st.v, st.E, st.A, st.W
    else:
        p = [rn(n, cfg.w_std) for n in sizes]
        m = [rn(n, 3e-4) for n in sizes]; v = [rn(n, 1e-3).square_() for n in sizes]
        E = [rn(n, 1e-5) for n in sizes]; A = [rn(n, 1e-4).abs_() for n in sizes]
        low = [x.to(torch.bfloat16) for x in p]
    grad = tf.PtrTable([rn(n, cfg.g_std, torch.bfloat16) for n in sizes])
    hp = {k: float(np.float32(getattr(cfg, k))) for k in ("lr", "beta1", "beta2", "eps", "weight_decay")}
    log(f"cfg 4 buffers ready, {torch.cuda.memory_allocated() / 2**30:.1f} GiB")
    rows = []
    # each ratio in the default mode (the stored bf16 copy of frozen elements is read back) and under
    # the promise that the copy is the rounding of the master weights (true for these buffers)
    for r, promise in [(0.0, False)] + [(r, pr) for r in wl.R_SWEEP[4] for pr in (False, True)]:
        bits = None
        if r > 0:
            gb = torch.Generator(device="cuda").manual_seed(wl.SEED_BASE + 40 + int(100 * r))
            bits = [(torch.rand((n + 31) // 32 * 32, generator=gb, device="cuda") < r).view(-1, 32).to(torch.int64)
                    .mul_(2 ** torch.arange(32, device="cuda", dtype=torch.int64)).sum(1).to(torch.int32) for n in sizes]
        ctx.assume_lowp_is_rounded_master(promise)
        fn = lambda: tf.tf_masked_adamw(ctx, sizes, p, m, v, grad, tf.TF_BF16, [2] * L, hp["lr"], hp["beta1"], hp["beta2"],
                                        hp["eps"], hp["weight_decay"], p_lowp=low, elem_freeze_bits=bits, ema=E, ema_abs=A,
                                        ema_decay=float(np.float32(cfg.ema_decay)))
        dt, prof = _timed(ctx, torch, fn, args.steps, args.warmup)
        ctx.assume_lowp_is_rounded_master(False)
        kms = sum(t for k, t in prof if k == "adamw") / args.steps
        alg = P * ((1 - r) * 44 + (0.125 if r > 0 else 0))
        rows.append({"r": r, "lowp_is_rounded_master": promise, "ms_kernels": kms, "ms_per_call": dt * 1e3,
                     "algorithmic_GBps": alg / kms / 1e6, "dense_equivalent_GBps": P * 44 / kms / 1e6,
                     "pct_hbm_peak_dense_equivalent": P * 44 / kms / 1e6 / 80.0})
        log(f"cfg4 r={r}{' (copy = rounded master promised)' if promise else ''}: {kms:.3f} ms, algorithmic "
            f"{rows[-1]['algorithmic_GBps']:.0f} GB/s, dense-equivalent {rows[-1]['dense_equivalent_GBps']:.0f} GB/s")
        del bits
    dense = rows[0]
    return {"workload": f"cfg4 {cfg.name}: {L} tensors, {P} elements, fp32 p/m/v/E/A + bf16 grad and copy, Bernoulli element masks",
            "rows": rows,
            "roofline": {"kernel": "ew_kernel (masked AdamW + APF EMAs), dense (r = 0)", "bound": "hbm",
                         "achieved": dense["algorithmic_GBps"], "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                         "frac": dense["algorithmic_GBps"] / PEAK_HBM_GBPS, "traffic": read_traffic("adamw", 4),
                         "traffic_source": TRAFFIC_NOTE, "avg_launch_ms": dense["ms_kernels"] / 2.0,
                         "launches_per_call": 2, "bytes_per_call": P * 44.0}}


def bench_row_blocks(args, cfg, ctx, wl, tf, torch):
    """The benchmark stage (cfg 2) with sub-tensor freezing: 256-row blocks of the weight tensors are
    drawn under the budget floor(r P) (tf_select_row_blocks), the backward skips their dW rows
    (tf_stage_backward_blocks) and the optimizer skips their elements (element masks made by
    tf_row_blocks_to_bits).  The frozen parameter fraction phi then equals r to within one block."""
    st = Stage(cfg, wl, tf, torch)
    L, T, P = st.L, st.T, cfg.n_params
    bits = [torch.zeros((n + 31) // 32, dtype=torch.int32, device="cuda") for n in st.sizes]
    hp = st.hp
    rows = []
    for r in (0.0, 0.1, 0.25, 0.5, 0.75, 0.9, 1.0):
        masks, frozen = tf.tf_select_row_blocks(st.shapes, 256, r, 20260205754)
        phi = frozen / P
        tf.tf_row_blocks_to_bits(ctx, st.shapes, masks, 256, bits)
        tmask = np.array([int(m.all()) for m in masks], dtype=np.uint8)        # wholly frozen tensors need no optimizer blocks
        def step():
            tf.tf_stage_backward_blocks(ctx, st.shapes, T, tf.TF_BF16, st.W, st.X, st.dY, None, masks, 256,
                                        st.dX, st.dW, tf.TF_BF16)
            tf.tf_masked_adamw(ctx, st.sizes, st.p, st.m, st.v, st.dW, tf.TF_BF16, st.steps, hp["lr"], hp["beta1"],
                               hp["beta2"], hp["eps"], hp["weight_decay"], p_lowp=st.W, tensor_freeze_mask=tmask,
                               elem_freeze_bits=bits, ema=st.E, ema_abs=st.A, ema_decay=st.decay)
        dt, prof = _timed(ctx, torch, step, args.steps, 2)
        k = {}
        for name, ms in prof:
            k.setdefault(name, []).append(ms)
        per = {n: float(np.sum(v)) / args.steps for n, v in k.items()}
        launches = {n: len(v) / args.steps for n, v in k.items()}
        bwd = sum(v for n, v in per.items() if n.startswith("d"))
        rows.append({"r": r, "phi": phi, "frozen_blocks": int(sum(int(m.sum()) for m in masks)), "ms_per_step": dt * 1e3,
                     "backward_ms": bwd, "backward_tflops": 2.0 * T * P * (2.0 - phi) / bwd / 1e9,
                     "dw_ms": per.get("dw_mfma", 0.0), "dw_launches": launches.get("dw_mfma", 0.0),
                     "adamw_ms": per.get("adamw", 0.0),
                     "adamw_algorithmic_GBps": (44.0 * (P - frozen) + P / 8.0) / per["adamw"] / 1e6 if per.get("adamw") else None})
        log(f"row blocks r={r}: phi={phi:.4f} {dt * 1e3:.3f} ms/step, backward {bwd:.3f} ms "
            f"(dW {rows[-1]['dw_ms']:.3f} ms in {rows[-1]['dw_launches']:.0f} launches), AdamW {rows[-1]['adamw_ms']:.3f} ms")
    b0, b1 = rows[0]["backward_ms"], rows[-1]["backward_ms"]
    for x in rows[1:-1]:
        x["eta_backward"] = (b0 - x["backward_ms"]) / (x["phi"] * (b0 - b1))
    return {"workload": f"cfg2 stage with 256-row-block freezing, L={L} tensors, P={P} params, T={T}", "rows": rows}


def bench_shared_inputs(args, cfg, ctx, wl, tf, torch):
    """The benchmark stage (cfg 2) with q/k/v and gate/up of every block sharing their input: one dX
    per group (the members are contraction segments of one problem), against the plain backward in
    which every layer writes its own dX.  Same FLOPs; 16 instead of 28 dX outputs."""
    st = Stage(cfg, wl, tf, torch)
    L, T, P = st.L, st.T, cfg.n_params
    groups = []
    for b in range(cfg.blocks):
        groups += [2 * b, 2 * b, 2 * b, -1, 2 * b + 1, 2 * b + 1, -1]
    shared = {}
    dX = []
    for l in range(L):
        key = groups[l] if groups[l] >= 0 else -(l + 1)
        shared.setdefault(key, st.dX[l])
        dX.append(shared[key])
    frozen = np.ones(L, np.uint8)
    out = {}
    for name, fn in (("plain", lambda: tf.tf_stage_backward(ctx, st.shapes, T, tf.TF_BF16, st.W, None, st.dY, frozen, st.dX, None, tf.TF_BF16)),
                     ("shared", lambda: tf.tf_stage_backward_shared(ctx, st.shapes, T, tf.TF_BF16, st.W, None, st.dY, frozen, None, 0,
                                                                    groups, dX, None, tf.TF_BF16))):
        dt, prof = _timed(ctx, torch, fn, args.steps, args.warmup)
        ms = float(np.mean([t for k, t in prof if k == "dx_mfma"]))
        out[name] = {"dx_ms": ms, "dx_tflops": 2.0 * T * P / ms / 1e9}
        log(f"dX {name}: {ms:.3f} ms, {out[name]['dx_tflops']:.0f} TFLOP/s")
    return {"workload": f"cfg2 stage, input gradients with and without shared-input groups, T={T}", **out}


def bench_selection(args, cfg, ctx, wl, tf, torch):
    """The selection steps beside the hot path at the 8B stage's size (56 tensors, 1.74e9 elements):
    the AutoFreeze norm pass (12 B per element: p and snapshot read, snapshot written) and the Alg. 2
    budget reconciliation of Bernoulli(0.3) base masks to r = 0.5 (add) and r = 0.1 (remove)."""
    sizes = [k * n for k, n in cfg.shapes]
    L, P = len(sizes), sum(sizes)
    g = torch.Generator(device="cuda").manual_seed(wl.SEED_BASE + 6)
    p = [torch.randn(n, generator=g, device="cuda") * cfg.w_std for n in sizes]
    snap = [x + torch.randn(x.numel(), generator=g, device="cuda") * 1e-4 for x in p]
    norms = torch.zeros(L, dtype=torch.float64, device="cuda")
    dt, prof = _timed(ctx, torch, lambda: tf.tf_autofreeze_norms(ctx, sizes, p, snap, norms), args.steps, args.warmup)
    kms = sum(t for k, t in prof if k == "autofreeze") / args.steps
    out = {"workload": f"selection steps, {L} tensors, {P} elements",
           "autofreeze_norms": {"ms_kernels": kms, "GBps": P * 12 / kms / 1e6, "pct_hbm_peak": P * 12 / kms / 1e6 / 80.0,
                                "bytes_per_element": 12}}
    log(f"autofreeze norms: {kms:.3f} ms, {out['autofreeze_norms']['GBps']:.0f} GB/s")
    del snap
    base = [(torch.rand((n + 31) // 32 * 32, generator=g, device="cuda") < 0.3).view(-1, 32).to(torch.int64)
            .mul_(2 ** torch.arange(32, device="cuda", dtype=torch.int64)).sum(1).to(torch.int32) for n in sizes]
    stats = torch.zeros(3, dtype=torch.int64, device="cuda")
    rows = []
    for r in (0.5, 0.1):
        work = [b.clone() for b in base]
        def fn():
            for w, b in zip(work, base):
                w.copy_(b)
            tf.tf_reconcile_mask(ctx, sizes, work, int(r * P), 20260205754, stats=stats)
        dt, prof = _timed(ctx, torch, fn, max(args.steps // 4, 3), 1)
        kms = float(np.mean([t for k, t in prof if k == "reconcile"]))
        st = stats.cpu().numpy()
        rows.append({"r": r, "n_freeze": int(r * P), "base_ones": int(st[0]), "case": int(st[1]), "ms": kms,
                     "Gelements_per_s": P / kms / 1e6})
        log(f"reconcile r={r}: {kms:.3f} ms ({rows[-1]['Gelements_per_s']:.1f} G elements/s), case {int(st[1])}")
    out["reconcile"] = rows
    return out


def bench_microbatches(args, cfg, ctx, wl, tf, torch, st=None):
    """cfg 5: 8 sequential backward calls of 1 x 1024 tokens on the 8B stage, dW accumulated in fp32
    for unfrozen tensors only, a different freeze ratio per call.  One microbatch's seeded inputs are
    used for all 8 calls (timing only; the accumulation parity test draws fresh ones): its own draw,
    or with `st` (a Stage of the same tensors at more tokens) the first 1024 tokens of that stage's."""
    T = cfg.T
    if st is None:
        st = Stage(cfg, wl, tf, torch)
        X, dY = st.X, st.dY
    else:
        X = tf.PtrTable([st.X[l][:T] for l in range(st.L)])
        dY = tf.PtrTable([st.dY[l][:T] for l in range(st.L)])
    L, P = st.L, cfg.n_params
    dX = tf.PtrTable([st.dX[l][:T] for l in range(L)])
    acc_t = [torch.zeros((k, n), device="cuda") for k, n in st.shapes]
    acc = tf.PtrTable(acc_t)
    ratios = wl.microbatch_ratios(cfg)
    masks = [wl.permutation_mask(cfg, r, microbatch=i) for i, r in enumerate(ratios)]
    # a layer's first unfrozen microbatch of the step overwrites its accumulator, the later ones add
    adds, never = tf.tf_microbatch_plan(np.stack(masks))
    seen = 1 - never                        # unfrozen in at least one microbatch: these accumulators are live
    def one_step():
        for mk, am in zip(masks, adds):
            tf.tf_stage_backward_microbatch(ctx, st.shapes, T, tf.TF_BF16, st.W, X, dY, mk, dX, acc, tf.TF_F32, am)
    def one_step_all_adding():      # one flag per call: every call adds, so the step starts by clearing the accumulators
        for l in range(L):
            if seen[l]:
                acc_t[l].zero_()
        for mk in masks:
            tf.tf_stage_backward(ctx, st.shapes, T, tf.TF_BF16, st.W, X, dY, mk, dX, acc, tf.TF_F32, accumulate=True)
    dt_add, _ = _timed(ctx, torch, one_step_all_adding, args.steps, args.warmup)
    dt, prof = _timed(ctx, torch, one_step, args.steps, args.warmup)
    # per call: one dX launch, then one or two dW launches (the overwriting layers, the adding layers)
    calls = []
    for k, t in prof:
        if k == "dx_mfma":
            calls.append([t, 0.0])
        elif k == "dw_mfma" and calls:
            calls[-1][1] += t
    per_call = []
    for i, (r, mk, am) in enumerate(zip(ratios, masks, adds)):
        phi = wl.frozen_param_fraction(cfg, mk)
        tdx = float(np.mean([c[0] for c in calls[i::len(masks)]])); tdw = float(np.mean([c[1] for c in calls[i::len(masks)]]))
        # minimum traffic of the dW launches: X and dY read once, the fp32 gradient written, and read where it is added to
        grad_bytes = sum(k * n * (8 if am[l] else 4) for l, (k, n) in enumerate(st.shapes) if not mk[l])
        unfrozen_bytes = grad_bytes + 2 * T * sum((k + n) * (0 if mk[l] else 1) for l, (k, n) in enumerate(st.shapes))
        dw_flop = 2.0 * T * P * (1 - phi)
        t_roof_ms = max(dw_flop / (PEAK_BF16_TFLOPS * 1e12), unfrozen_bytes / (PEAK_HBM_GBPS * 1e9)) * 1e3
        per_call.append({"r": r, "n_frozen": int(mk.sum()), "phi": phi, "layers_overwriting": int(((1 - mk) * (1 - am)).sum()),
                         "dx_ms": tdx, "dw_ms": tdw,
                         "dx_tflops": 2.0 * T * P / tdx / 1e9, "dw_tflops": dw_flop / tdw / 1e9,
                         "dw_GBps_min_traffic": unfrozen_bytes / tdw / 1e6, "dw_frac_of_its_roof": t_roof_ms / tdw})
        log(f"cfg5 call {i}: r={r} phi={phi:.3f} dX {tdx:.3f} ms ({per_call[-1]['dx_tflops']:.0f} TFLOP/s), "
            f"dW {tdw:.3f} ms ({per_call[-1]['dw_tflops']:.0f} TFLOP/s, {per_call[-1]['dw_GBps_min_traffic']:.0f} GB/s of its minimum traffic, "
            f"{100 * per_call[-1]['dw_frac_of_its_roof']:.0f} % of max(MFMA, HBM) roof; {per_call[-1]['layers_overwriting']} layers overwrite)")
    log(f"cfg5: {dt * 1e3:.2f} ms per 8 calls ({dt_add * 1e3:.2f} ms with one flag per call: the accumulators cleared, then every call adding)")
    tot_bytes = sum(c["dw_GBps_min_traffic"] * c["dw_ms"] * 1e6 for c in per_call)
    tot_ms = sum(c["dw_ms"] for c in per_call)
    return {"workload": f"cfg5 {cfg.name}: 8 calls of T={T}, fp32 dW accumulation, {L} tensors, P={P} params",
            "ms_per_8_calls": dt * 1e3, "tokens_per_s": 8 * T / dt, "calls": per_call,
            "ms_per_8_calls_cleared_then_every_call_adding": dt_add * 1e3,
            "roofline_dw": {"kernel": "gemm_mfma_kernel<TN, fp32 out> (dW = / += X^T dY per layer, unfrozen layers only), mean over the 8 calls",
                            "bound": "hbm", "achieved": tot_bytes / tot_ms / 1e6, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": tot_bytes / tot_ms / 1e6 / PEAK_HBM_GBPS, "traffic": read_traffic("dw_mfma", 5),
                            "traffic_source": TRAFFIC_NOTE, "avg_launch_ms": tot_ms / len(per_call),
                            "frac_of_max_mfma_hbm_roof": float(np.mean([c["dw_frac_of_its_roof"] for c in per_call])),
                            # the calls in which every unfrozen layer adds (read-modify-write only: HBM is their roof)
                            "frac_of_max_mfma_hbm_roof_calls_that_only_add": float(np.mean(
                                [c["dw_frac_of_its_roof"] for c in per_call if c["layers_overwriting"] == 0] or [0.0]))},
            "roofline_dx": {"kernel": "gemm_mfma_kernel<NT> at T=1024", "bound": "mfma",
                            "achieved": float(np.mean([c["dx_tflops"] for c in per_call])), "peak": PEAK_BF16_TFLOPS,
                            "unit": "TFLOP/s", "frac": float(np.mean([c["dx_tflops"] for c in per_call])) / PEAK_BF16_TFLOPS,
                            "avg_launch_ms": float(np.mean([c["dx_ms"] for c in per_call]))}}


def read_traffic(kernel: str, cfg_id: int):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), as
    recorded in profiles/hbm_traffic.txt ("<kernel> cfg<id> <bytes>"), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for ln in open(path):
        f = ln.split()
        if len(f) >= 3 and not ln.startswith("#") and f[0] == kernel and f[1] == f"cfg{cfg_id}":
            return float(f[2])
    return None


if __name__ == "__main__":
    main()
