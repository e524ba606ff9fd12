"""Benchmark of the freeze-boundary training step on one MI355X.

A step is one pass of the whole hot path: pt_frozen_forward (front end, frozen
blocks or a cache gather), pt_active_fwd_bwd, pt_layer_grad_norms (its begin
half before and its end half, the host's wait, after the enqueue of
pt_optimizer_step) and pt_optimizer_step, on a synthetic batch already resident
in HBM.  The default
workload is ViT-B/16, bf16 with fp32 accumulation, micro-batch 64, AdamW, k = 0.

Prints ONE JSON line (see the keys below).  `roofline` describes the dominant
kernel (the weight-gradient matrix-core GEMM) from HIP-event timings taken inside
this run; `cpu_baseline` is the CPU checker timed on a small batch of the same
shapes.  `--gpus N` with N > 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of each GEMM class (mean over the launches of one step), from rocprofv3
# --pmc FETCH_SIZE and --pmc WRITE_SIZE runs of this script, scaled by what the same counters
# read for the --calibrate-copy kernel; the figures and commands are in profiles/.
MEASURED_TRAFFIC = {
    ("vit_b16", 0, "gemm_nn"): 115097149 + 57009860,    # fetched + written, forward products
    ("vit_b16", 0, "gemm_nt"): 150142135 + 30901561,    # input-gradient products
    ("vit_b16", 0, "gemm_tn"): 422498938 + 71133510,    # weight gradients (one grouped launch per block) incl. their split-K reductions
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vit_b16",
                    help="vit_b16 | vit_b16_b128 | bert_base_qa | bert_large_qa | bert_base_cls")
    ap.add_argument("--micro-batches", type=int, default=1,
                    help="M > 1: a step is M micro-batches of the workload's batch accumulated into one optimizer step")
    ap.add_argument("--k", type=int, default=0, help="freeze boundary of the timed run")
    ap.add_argument("--no-sweep", action="store_true", help="skip the extra measurements at other boundaries")
    ap.add_argument("--sweep", default="", help="comma-separated boundaries of the sweep (default 1, L/4, L/2, 3L/4)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline")
    ap.add_argument("--host-tier", action="store_true",
                    help="keep every cached row in pinned host memory (window of 4 batches in HBM, next batch prefetched)")
    ap.add_argument("--schedule", default="",
                    help="comma-separated boundaries, e.g. 0,3,6,9: after the main measurement, run --phase-steps steps "
                         "at each boundary in turn (the boundary only moves up) and report samples/s per phase and the "
                         "cost of each pt_set_freeze_boundary call")
    ap.add_argument("--phase-steps", type=int, default=50)
    ap.add_argument("--profile-steps", type=int, default=3)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy four times (a kernel of known HBM traffic, for scaling "
                         "the memory counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def flops_per_sample(w, k, cached):
    """Algorithmic FLOPs of one step per sample: e + k f + 3 (L-k) f, minus e + k f on a cache hit."""
    D, F, S, L = w["D"], w["F"], w["S"], w["L"]
    f = 2.0 * S * (D * 3 * D + D * D + 2 * D * F) + 4.0 * S * S * D
    e = 2.0 * (S - 1) * (w["chans"] * w["patch"] ** 2) * D if w["arch"] == "vit" else 0.0
    return (0.0 if cached else e + k * f) + 3.0 * (L - k) * f


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {a.gpus}); no multi-GPU path exists",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2102_03161_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    w = synth.workload(a.workload)
    B = w["B"]
    n_ids = 4 * B
    M = a.micro_batches
    if a.host_tier:
        ctx = binding.Context(binding.make_config(w, cache_slots=0, host_slots=n_ids, window_slots=4 * B, grad_accum=M > 1))
    else:
        ctx = binding.Context(binding.make_config(w, cache_slots=n_ids, grad_accum=M > 1))
    seed = 2
    for tid, name, shape, _, _ in ctx.tensors():
        ctx.write_tensor(tid, binding.KIND_PARAM, synth.round_bf16(synth.gen_param(seed, name, shape)))
    batches = []
    for i in range(4):   # four seeded batches with distinct sample ids, resident in HBM
        x, y = synth.gen_inputs(w, seed, B, tag=f"b{i}")
        batches.append((torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev), np.arange(i * B, (i + 1) * B)))
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)

    def step(i, use_cache=False):
        for j in range(M):
            x, y, ids = batches[(i * M + j) % len(batches)]
            hk = ctx.frozen_forward(x, ids if use_cache else None)
            if use_cache and a.host_tier:   # stage the next batch's rows while this one trains
                ctx.cache_prefetch(batches[(i * M + j + 1) % len(batches)][2])
            ctx.active_fwd_bwd(hk, y, want_loss=False)
            if M > 1:
                ctx.accumulate_grads(first=(j == 0))
        if M > 1:
            ctx.finish_accumulation(want_loss=False)
        ctx.layer_grad_norms_begin()          # asks for the norms of the gradients as they are now
        ctx.optimizer_step(**hp)              # its pass over the gradient also leaves the sums of squares
        return ctx.layer_grad_norms_end()     # synchronises: the freeze rule reads these on the host

    def timed(n_warm, n_steps, use_cache=False):
        for i in range(n_warm):
            step(i, use_cache)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_steps):
            step(i, use_cache)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n_steps

    if a.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if a.k:
        ctx.set_freeze_boundary(a.k)
    sec = timed(a.warmup, a.steps)
    sps = M * B / sec
    fl = flops_per_sample(w, a.k, False) * B * M
    result = {
        "metric": "train samples/sec on 1 GPU vs frozen prefix k; % bf16 MFMA peak",
        "value": round(sps, 2), "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {w['arch']} L={w['L']} D={w['D']} H={w['H']} F={w['F']} S={w['S']} "
                               f"micro-batch {B}" + (f" x {M} accumulated" if M > 1 else "") +
                               f", AdamW, freeze boundary k={a.k}, no cache",
                   "global_batch": B * M, "seq_len": w["S"], "k": a.k},
        "step_tflops": round(fl / sec / 1e12, 2),
        "step_frac_of_bf16_peak": round(fl / sec / 1e12 / PEAK_BF16_TFLOPS, 4),
    }

    # ---- per-kernel timing with HIP events (extra steps, not part of the timed region above) ----
    ctx.profile_reset()
    ctx.profile_enable(True)
    for i in range(a.profile_steps):
        step(i)
    ctx.profile_enable(False)
    prof = ctx.profile_read()
    breakdown = {}
    for name, (ms, n, wk) in prof.items():
        if n:
            breakdown[name] = {"ms_per_step": round(ms / a.profile_steps, 4), "launches_per_step": n // a.profile_steps,
                               "avg_us": round(1e3 * ms / n, 2)}
            if name.startswith("gemm") or name.startswith("attn"):
                breakdown[name]["tflops"] = round(wk / (ms * 1e-3) / 1e12, 2)
                breakdown[name]["frac_of_bf16_peak"] = round(wk / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
                if name.startswith("attn"):
                    # attention sits below the ridge (98 FLOP/B at S = 197): also its compulsory bytes against
                    # HBM.  Forward reads qkv and writes ctx (8 D bytes per token), backward reads qkv, ctx, dctx
                    # and writes dqkv (16 D); the top block under a first-token head moves less than this.
                    per_tok = (8 if name == "attn_fwd" else 16) * w["D"]
                    blocks = (w["L"] - a.k) * M * a.profile_steps
                    byts = float(per_tok) * B * w["S"] * blocks
                    breakdown[name]["gbs"] = round(byts / (ms * 1e-3) / 1e9, 1)
                    breakdown[name]["frac_of_hbm_peak"] = round(byts / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
            elif wk:
                breakdown[name]["gbs"] = round(wk / (ms * 1e-3) / 1e9, 1)
                breakdown[name]["frac_of_hbm_peak"] = round(wk / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
    result["breakdown"] = breakdown
    gemm_names = [n for n in ("gemm_tn", "gemm_nn", "gemm_nt") if prof[n][1]]
    dom = max(gemm_names, key=lambda n: prof[n][0])
    ms, n, wk = prof[dom]
    ach = wk / (ms * 1e-3) / 1e12
    result["roofline"] = {"kernel": {"gemm_tn": "weight-gradient GEMMs dW = x^T dy (gemm_wgrad_group_kernel + splitk_reduce_kernel)",
                                     "gemm_nn": "forward GEMMs y = x W (gemm_pp_kernel / gemm_dma_kernel, TA=false TB=false)",
                                     "gemm_nt": "input-gradient GEMMs dx = dy W^T (gemm_pp_kernel / gemm_dma_kernel, TB=true)"}[dom],
                          "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                          "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                          "traffic": MEASURED_TRAFFIC.get((a.workload, a.k, dom)),
                          "avg_launch_us": round(1e3 * ms / n, 2), "launches_per_step": n // a.profile_steps,
                          "flops_per_launch": wk / n}

    # ---- freeze schedule: fixed step counts per boundary, switch cost measured around the call ----
    if a.schedule and a.k == 0:
        phases = []
        for k in [int(v) for v in a.schedule.split(",")]:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ctx.set_freeze_boundary(k)
            torch.cuda.synchronize()
            t_switch = time.perf_counter() - t0
            s_phase = timed(0, a.phase_steps)
            phases.append({"k": k, "steps": a.phase_steps, "samples_per_s": round(M * B / s_phase, 1),
                           "step_tflops": round(flops_per_sample(w, k, False) * B * M / s_phase / 1e12, 1),
                           "switch_ms": round(t_switch * 1e3, 3)})
        result["schedule"] = phases
        a.no_sweep = True   # the boundary has moved: the sweep below would start from the last phase

    # ---- samples/s versus k (the boundary only moves up): uncached and cached ----
    if not a.no_sweep and a.k == 0:
        sweep = {"k0": round(sps, 1)}
        ks = [int(v) for v in a.sweep.split(",")] if a.sweep else [1, w["L"] // 4, w["L"] // 2, 3 * w["L"] // 4]
        for k in sorted(set(ks)):
            ctx.set_freeze_boundary(k)
            s_unc = timed(2, 8, use_cache=False)
            step(0, True); step(1, True); step(2, True); step(3, True)     # fill / advance the cache rows
            s_hit = timed(2, 8, use_cache=True)
            ms_re, ms_hit = ctx.time_frozen_forward(batches[0][0], batches[0][2], 3)
            sweep[f"k{k}_prefix_ms"] = {"recompute": round(ms_re, 4), "cached": round(ms_hit, 4)}
            sweep[f"k{k}"] = round(M * B / s_unc, 1)
            sweep[f"k{k}_cached"] = round(M * B / s_hit, 1)
        result["samples_per_s_vs_k"] = sweep
        if a.host_tier:
            result["cache_tier"] = "host-pinned rows, 4-batch HBM window, next batch prefetched"
            result["host_tier_stats"] = ctx.host_tier_stats()
    ctx.close()

    # ---- the CPU checker timed on a small batch of the same shapes ----
    if not a.no_cpu:
        from oracle import encoder as orc
        from threadpoolctl import threadpool_info
        Bo = 32
        cfg = orc.Config(**synth.model_fields(w))
        p = {n: synth.gen_param(seed, n, s).astype(np.float64) for n, s in orc.param_shapes(cfg).items()}
        x, y = synth.gen_inputs(w, seed, Bo)
        x = x.astype(np.float64) if x.dtype.kind == 'f' else x
        st = orc.new_opt_state(p)
        t0 = time.perf_counter()
        hk, fs = orc.frozen_forward(cfg, p, x, a.k)
        loss, grads, _ = orc.active_fwd_bwd(cfg, p, hk, y, a.k, fs)
        orc.layer_grad_norms(cfg, grads, a.k)
        orc.adamw_step(cfg, p, grads, st, a.k, 1e-3, 0.9, 0.999, 1e-8, 0.01)
        dt = time.perf_counter() - t0
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        result["cpu_baseline"] = {"value": round(Bo / dt, 3), "unit": "samples/s", "cores": threads, "kind": "oracle",
                                  "sample": f"one full step (frozen forward, forward+backward, grad norms, AdamW) of the "
                                            f"numpy oracle in fp64 at batch {Bo}, same shapes, k={a.k}; {dt:.1f} s"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
