"""Benchmark of the freeze-boundary training step on one MI355X.

A step is one pass of the whole hot path: pt_frozen_forward (front end, frozen
blocks or a cache gather), pt_active_fwd_bwd, pt_layer_grad_norms (its begin
half before and its end half, the host's wait, after the enqueue of
pt_optimizer_step) and pt_optimizer_step, on a synthetic batch already resident
in HBM.  The default workload is ViT-B/16, bf16 with fp32 accumulation,
micro-batch 64, AdamW, k = 0.

Prints ONE JSON line.  `value` is the samples/s of the timed steps.  `roofline`
describes the dominant kernel, gemm_wgrad_group_kernel (the four weight
gradients of an encoder block as one launch), from HIP-event timings taken
inside this run around that kernel alone; `breakdown` gives every kernel class;
`step_tflops` counts the work that was launched (sum over the timed launches),
not a dense equivalent.  Beside the main figure the default run reports
samples/s against the boundary k with and without the cache (`samples_per_s_vs_k`),
the cached-prefix configuration over four epochs of repeated batches plus a
permuted one (`epochs`), the freeze rule of Eq. 1 driving the boundary per epoch
(`auto_freeze`), the freeze schedule 0 -> 3 -> 6 -> 9 at micro-batch 128 with
the per-phase utilisation (`schedule_b128`), and the CPU checker timed on
the same shapes (`cpu_baseline`).  `--gpus N` with N > 1 is refused: this build
is single-GPU.
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

# HBM bytes per launch of gemm_wgrad_group_kernel over one encoder block (its four weight gradients), from the
# two rocprofv3 --pmc runs in profiles/*_hbm_traffic.md (FETCH_SIZE, then WRITE_SIZE), each scaled by what the
# same counter reads for the plain copy of --calibrate-copy: fetched + written.
# A launch also carries, on the workgroups it adds for otherwise idle CUs, the summation of the previous block's
# split-K slabs (56.6 MB read, 28.3 MB written) and one LayerNorm backward pass over the tokens (136 MB at
# 12608 tokens); those bytes are in the figures.
MEASURED_TRAFFIC = {
    ("vit_b16", 0): 769_487_200,                     # profiles/vit_b16_b64_k0_hbm_traffic.md
    ("bert_base_qa", 0): 741_764_665,                # profiles/bert_base_b32_s384_k0_hbm_traffic.md
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
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the epochs / schedule measurements that the default ViT-B/16 run appends")
    ap.add_argument("--host-tier", action="store_true",
                    help="keep every cached row in pinned host memory (window of 4 batches in HBM, next batch prefetched)")
    ap.add_argument("--schedule", default="",
                    help="comma-separated boundaries, e.g. 0,3,6,9: after the main measurement, run --phase-steps steps "
                         "at each boundary in turn (the boundary only moves up) and report samples/s, the kernel "
                         "classes' utilisation and the cost of each pt_set_freeze_boundary call per phase")
    ap.add_argument("--phase-steps", type=int, default=50)
    ap.add_argument("--epochs", type=int, default=0,
                    help="N > 0: the cached-prefix configuration: --epoch-batches seeded batches replayed N times at "
                         "boundary --epoch-k (epoch 1 misses and fills the cache, the others hit), then once more "
                         "with the samples permuted over the batches; samples/s per epoch and the norms are reported")
    ap.add_argument("--epoch-batches", type=int, default=16)
    ap.add_argument("--epoch-k", type=int, default=6)
    ap.add_argument("--auto-freeze", type=float, default=0.0,
                    help="alpha of the freeze rule (Eq. 1): after every --epoch-steps steps the norms of the last step "
                         "go through pt_next_boundary and the result through pt_set_freeze_boundary; the boundary "
                         "trajectory and samples/s per epoch are reported (--auto-epochs epochs)")
    ap.add_argument("--epoch-steps", type=int, default=20)
    ap.add_argument("--auto-epochs", type=int, default=8)
    ap.add_argument("--profile-steps", type=int, default=3)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy four times (a kernel of known HBM traffic, for scaling "
                         "the memory counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def flops_per_sample(w, k, cached):
    """Algorithmic FLOPs of one step per sample as a dense network: e + k f + 3 (L-k) f, minus e + k f on a cache hit."""
    D, F, S, L = w["D"], w["F"], w["S"], w["L"]
    f = 2.0 * S * (D * 3 * D + D * D + 2 * D * F) + 4.0 * S * S * D
    e = 2.0 * (S - 1) * (w["chans"] * w["patch"] ** 2) * D if w["arch"] == "vit" else 0.0
    return (0.0 if cached else e + k * f) + 3.0 * (L - k) * f


GEMM_CLASSES = ("gemm_nn", "gemm_nt", "gemm_tn", "wgrad_block")


class Runner:
    """One context with its resident batches; `step` is the whole hot path once."""

    def __init__(self, torch, np, binding, synth, workload, M=1, host_tier=False, n_batches=4, cache_batches=None, seed=2):
        self.torch, self.np, self.binding = torch, np, binding
        self.w = w = synth.workload(workload)
        self.B, self.M, self.host_tier = w["B"], M, host_tier
        B = self.B
        n_ids = (cache_batches or n_batches) * B
        if host_tier:
            cfg = binding.make_config(w, cache_slots=0, host_slots=n_ids, window_slots=4 * B, grad_accum=M > 1)
        else:
            cfg = binding.make_config(w, cache_slots=n_ids, grad_accum=M > 1)
        self.ctx = binding.Context(cfg)
        for tid, name, shape, _, _ in self.ctx.tensors():
            self.ctx.write_tensor(tid, binding.KIND_PARAM, synth.round_bf16(synth.gen_param(seed, name, shape)))
        self.batches = []
        for i in range(n_batches):   # seeded batches with distinct sample ids, resident in HBM
            x, y = synth.gen_inputs(w, seed, B, tag=f"b{i}")
            self.batches.append((torch.from_numpy(x).to("cuda:0"), torch.from_numpy(y).to("cuda:0"),
                                 np.arange(i * B, (i + 1) * B)))
        self.hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)

    def step(self, i, use_cache=False, batches=None):
        ctx, M = self.ctx, self.M
        batches = batches or self.batches
        for j in range(M):
            x, y, ids = batches[(i * M + j) % len(batches)]
            hk = ctx.frozen_forward(x, ids if use_cache else None)
            if use_cache and self.host_tier:   # stage the next batch's rows while this one trains
                ctx.cache_prefetch(batches[(i * M + j + 1) % len(batches)][2])
            ctx.active_fwd_bwd(hk, y, want_loss=False)
            if M > 1:
                ctx.accumulate_grads(first=(j == 0))
        if M > 1:
            ctx.finish_accumulation(want_loss=False)
        ctx.layer_grad_norms_begin()          # asks for the norms of the gradients as they are now
        ctx.optimizer_step(**self.hp)         # its pass over the gradient also leaves the sums of squares
        return ctx.layer_grad_norms_end()     # synchronises: the freeze rule reads these on the host

    def timed(self, n_warm, n_steps, use_cache=False, batches=None, first=0):
        for i in range(n_warm):
            self.step(first + i, use_cache, batches)
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_steps):
            self.step(first + n_warm + i, use_cache, batches)
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n_steps

    def profile(self, n_steps, k, use_cache=False):
        """Per-class kernel timing with HIP events the library records around every launch on its own stream
        (extra steps, never part of a timed region).  Returns (breakdown, raw, launched FLOPs per step)."""
        ctx, w = self.ctx, self.w
        ctx.profile_reset()
        ctx.profile_enable(True)
        for i in range(n_steps):
            self.step(i, use_cache)
        ctx.profile_enable(False)
        prof = ctx.profile_read()
        out = {}
        launched = 0.0
        for name, (ms, n, wk) in prof.items():
            if not n:
                continue
            e = {"ms_per_step": round(ms / n_steps, 4), "launches_per_step": round(n / n_steps, 2), "avg_us": round(1e3 * ms / n, 2)}
            if name in GEMM_CLASSES or name.startswith("attn"):
                launched += wk / n_steps
                e["tflops"] = round(wk / (ms * 1e-3) / 1e12, 2)
                e["frac_of_bf16_peak"] = round(wk / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
                if name.startswith("attn"):
                    # attention sits below the ridge (98 FLOP/B at S = 197): also its compulsory bytes against
                    # HBM.  Forward reads qkv and writes ctx (8 D bytes per token), backward reads qkv, ctx, dctx
                    # and writes dqkv (16 D); the top block under a first-token head moves less than this.
                    per_tok = (8 if name == "attn_fwd" else 16) * w["D"]
                    blocks = (w["L"] - k) * self.M * n_steps
                    byts = float(per_tok) * self.B * w["S"] * blocks
                    e["gbs"] = round(byts / (ms * 1e-3) / 1e9, 1)
                    e["frac_of_hbm_peak"] = round(byts / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
            elif wk:
                e["gbs"] = round(wk / (ms * 1e-3) / 1e9, 1)
                e["frac_of_hbm_peak"] = round(wk / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
            out[name] = e
        return out, prof, launched

    def utilisation(self, n_steps, k):
        """Condensed per-phase figures: matrix-core utilisation of the GEMM and attention classes (launched
        FLOPs over their kernel time, as a fraction of the bf16 peak) and HBM GB/s of the memory-bound classes."""
        bd, prof, launched = self.profile(n_steps, k)
        gemm_ms = sum(prof[n][0] for n in GEMM_CLASSES) + prof["splitk_reduce"][0]
        gemm_fl = sum(prof[n][2] for n in GEMM_CLASSES)
        attn_ms = prof["attn_fwd"][0] + prof["attn_bwd"][0]
        attn_fl = prof["attn_fwd"][2] + prof["attn_bwd"][2]
        out = {"gemm_tflops": round(gemm_fl / (gemm_ms * 1e-3) / 1e12, 1) if gemm_ms else None,
               "gemm_frac_of_bf16_peak": round(gemm_fl / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4) if gemm_ms else None,
               "attn_tflops": round(attn_fl / (attn_ms * 1e-3) / 1e12, 1) if attn_ms else None,
               "launched_tflop_per_step": round(launched / 1e12, 4)}
        for name in ("ln_fwd", "ln_bwd", "opt", "cache"):
            if name in bd and "gbs" in bd[name]:
                out[name + "_gbs"] = bd[name]["gbs"]
        return out

    def close(self):
        self.ctx.close()


def run_schedule(r, ks, phase_steps, profile_steps):
    """Fixed step counts per boundary; the switch cost is measured around the pt_set_freeze_boundary call."""
    torch = r.torch
    phases = []
    for k in ks:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r.ctx.set_freeze_boundary(k)
        torch.cuda.synchronize()
        t_switch = time.perf_counter() - t0
        s_phase = r.timed(0, phase_steps)
        ph = {"k": k, "steps": phase_steps, "samples_per_s": round(r.M * r.B / s_phase, 1),
              "ms_per_step": round(s_phase * 1e3, 3), "switch_ms": round(t_switch * 1e3, 3)}
        ph.update(r.utilisation(profile_steps, k))
        ph["step_tflops"] = round(ph["launched_tflop_per_step"] / s_phase, 1)
        phases.append(ph)
    return phases


def run_epochs(r, n_epochs, k):
    """The cached-prefix configuration: the resident batches replayed n_epochs times at boundary k (epoch 1
    misses and writes the cache, later epochs hit), then one epoch with the samples permuted over the batches
    (every batch then gathers rows that were written by other batches)."""
    torch, np = r.torch, r.np
    r.ctx.set_freeze_boundary(k)
    nb = len(r.batches)
    out = []
    norms = None

    def epoch(batches, label):
        nonlocal norms
        before = r.ctx.cache_stats()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(nb):
            norms = r.step(i, True, batches)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        after = r.ctx.cache_stats()
        out.append({"epoch": label, "samples_per_s": round(nb * r.B / dt, 1), "ms_per_step": round(1e3 * dt / nb, 3),
                    **{key: int(after[key] - before[key]) for key in ("hits", "advances", "misses", "block_runs")}})

    for e in range(n_epochs):
        epoch(r.batches, str(e + 1))
    # permuted epoch: the same samples, dealt to the batches in another order
    perm = np.random.default_rng(3).permutation(nb * r.B)
    xs = torch.cat([b[0] for b in r.batches]); ys = torch.cat([b[1] for b in r.batches])
    shuffled = []
    for i in range(nb):
        sel = perm[i * r.B:(i + 1) * r.B]
        idx = torch.from_numpy(sel).to("cuda:0")
        shuffled.append((xs[idx].contiguous(), ys[idx].contiguous(), sel.astype(np.int64)))
    del xs, ys
    epoch(shuffled, "permuted")
    return {"k": k, "batches": nb, "samples": nb * r.B, "epochs": out,
            "layer_grad_norms_last_step": [round(float(v), 6) for v in norms]}


def run_auto_freeze(r, alpha, epoch_steps, n_epochs):
    """Eq. 1 closed on the library: per epoch, the norms of the last step -> pt_next_boundary -> pt_set_freeze_boundary."""
    L = r.w["L"]
    out = []
    k = r.ctx.get_freeze_boundary()
    for e in range(n_epochs):
        r.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(epoch_steps):
            norms = r.step(e * epoch_steps + i, k > 0)
        r.torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        k_next = r.binding.next_boundary(norms, L, k, alpha)
        out.append({"epoch": e + 1, "k": k, "samples_per_s": round(epoch_steps * r.M * r.B / dt, 1), "k_next": k_next})
        r.ctx.set_freeze_boundary(k_next)
        k = k_next
    return {"alpha": alpha, "epoch_steps": epoch_steps, "trajectory": out}


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
    default_run = a.workload == "vit_b16" and a.k == 0 and a.micro_batches == 1 and not a.host_tier and not a.schedule \
        and not a.epochs and not a.auto_freeze and not a.no_extra and not a.no_sweep
    r = Runner(torch, np, binding, synth, a.workload, a.micro_batches, a.host_tier,
               n_batches=a.epoch_batches if a.epochs else 4)
    w, B, M = r.w, r.B, r.M

    if a.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if a.k:
        r.ctx.set_freeze_boundary(a.k)
    sec = r.timed(a.warmup, a.steps)
    sps = M * B / sec
    result = {
        "metric": "train samples/sec on 1 GPU vs frozen prefix k; % bf16 MFMA peak",
        "value": round(sps, 2), "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {w['arch']} L={w['L']} D={w['D']} H={w['H']} F={w['F']} S={w['S']} "
                               f"micro-batch {B}" + (f" x {M} accumulated" if M > 1 else "") +
                               f", AdamW, freeze boundary k={a.k}, no cache",
                   "global_batch": B * M, "seq_len": w["S"], "k": a.k},
    }

    # ---- per-kernel timing with HIP events (extra steps, not part of the timed region above) ----
    breakdown, prof, launched = r.profile(a.profile_steps, a.k)
    # FLOPs actually launched per step (GEMM and attention launches, summed by the library as it launches them):
    # under a first-token head the top block works on one row per sample behind its attention, so this is less
    # than the dense-network formula
    result["step_tflops"] = round(launched / sec / 1e12, 2)
    result["step_frac_of_bf16_peak"] = round(launched / sec / 1e12 / PEAK_BF16_TFLOPS, 4)
    result["step_tflop_launched"] = round(launched / 1e12, 4)
    result["step_tflop_dense_equivalent"] = round(flops_per_sample(w, a.k, False) * B * M / 1e12, 4)
    result["breakdown"] = breakdown
    ms, n, wk = prof["wgrad_block"]
    if n:
        ach = wk / (ms * 1e-3) / 1e12
        traffic = MEASURED_TRAFFIC.get((a.workload, a.k))
        result["roofline"] = {"kernel": "gemm_wgrad_group_kernel (the four weight gradients dW = x^T dy of one encoder block, "
                                        "one launch, two-way split over the tokens; on 40 workgroups added for idle CUs the launch also sums "
                                        "the previous block's slabs and runs one LayerNorm backward pass, whose bytes are in "
                                        "traffic and whose time is in avg_launch_us; flops_per_launch counts the weight gradients only)",
                              "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                              "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                              "avg_launch_us": round(1e3 * ms / n, 2), "launches_per_step": round(n / a.profile_steps, 2),
                              "flops_per_launch": wk / n}
    else:   # no whole block is active (k = L, or fp32 mode): the largest GEMM class stands in
        dom = max((c for c in GEMM_CLASSES if prof[c][1]), key=lambda c: prof[c][0], default=None)
        if dom:
            ms, n, wk = prof[dom]
            ach = wk / (ms * 1e-3) / 1e12
            result["roofline"] = {"kernel": dom, "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS,
                                  "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": None,
                                  "avg_launch_us": round(1e3 * ms / n, 2), "launches_per_step": round(n / a.profile_steps, 2),
                                  "flops_per_launch": wk / n}

    moved = False
    if a.schedule and a.k == 0:
        result["schedule"] = run_schedule(r, [int(v) for v in a.schedule.split(",")], a.phase_steps, a.profile_steps)
        moved = True
    if a.epochs and not moved:
        result["epochs"] = run_epochs(r, a.epochs, a.epoch_k)
        moved = True
    if a.auto_freeze and not moved:
        result["auto_freeze"] = run_auto_freeze(r, a.auto_freeze, a.epoch_steps, a.auto_epochs)
        moved = True

    # ---- samples/s versus k (the boundary only moves up): uncached and cached ----
    if not a.no_sweep and not moved and a.k == 0:
        sweep = {"k0": round(sps, 1)}
        ks = [int(v) for v in a.sweep.split(",")] if a.sweep else [1, w["L"] // 4, w["L"] // 3, w["L"] // 2, 2 * w["L"] // 3, 3 * w["L"] // 4] \
            if w["arch"] == "bert" else [1, w["L"] // 4, w["L"] // 2, 3 * w["L"] // 4]
        for k in sorted(set(ks)):
            r.ctx.set_freeze_boundary(k)
            s_unc = r.timed(2, 8, use_cache=False)
            for i in range(4):
                r.step(i, True)     # fill / advance the cache rows
            s_hit = r.timed(2, 8, use_cache=True)
            ms_re, ms_hit = r.ctx.time_frozen_forward(r.batches[0][0], r.batches[0][2], 3)
            sweep[f"k{k}_prefix_ms"] = {"recompute": round(ms_re, 4), "cached": round(ms_hit, 4)}
            sweep[f"k{k}"] = round(M * B / s_unc, 1)
            sweep[f"k{k}_cached"] = round(M * B / s_hit, 1)
        result["samples_per_s_vs_k"] = sweep
        if a.host_tier:
            result["cache_tier"] = "host-pinned rows, 4-batch HBM window, next batch prefetched"
            result["host_tier_stats"] = r.ctx.host_tier_stats()
    r.close()
    del r
    torch.cuda.empty_cache()

    if default_run:
        # the cached-prefix configuration: 16 seeded batches (1024 sample ids, 310 MB of cache rows), k = 6,
        # four epochs and a permuted one
        r3 = Runner(torch, np, binding, synth, "vit_b16", n_batches=16)
        result["epochs"] = run_epochs(r3, 4, 6)
        r3.close()
        del r3
        torch.cuda.empty_cache()
        # Eq. 1 closed on the library: per epoch of 10 steps the norms of the last step decide the next boundary
        r4 = Runner(torch, np, binding, synth, "vit_b16")
        result["auto_freeze"] = run_auto_freeze(r4, 1.0 / 3.0, 10, 6)
        r4.close()
        del r4
        torch.cuda.empty_cache()
        # the freeze schedule at micro-batch 128: 200 steps, the boundary moving 0 -> 3 -> 6 -> 9 every 50 steps
        r5 = Runner(torch, np, binding, synth, "vit_b16_b128")
        result["schedule_b128"] = run_schedule(r5, [0, 3, 6, 9], 50, 2)
        r5.close()
        del r5
        torch.cuda.empty_cache()

    # ---- the CPU checker timed on a bounded sample of the same workload ----
    if not a.no_cpu:
        from oracle import encoder as orc
        from threadpoolctl import threadpool_info
        Bo = 32
        cfg = orc.Config(**synth.model_fields(w))
        seed = 2
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
