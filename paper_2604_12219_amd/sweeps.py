#!/usr/bin/env python3
"""Method variants as runtime switches, measured on one MI355X with synthetic Wan-shaped inputs:

  python -m paper_2604_12219_amd.sweeps groups     # first-order group size: time and error against dense attention
  python -m paper_2604_12219_amd.sweeps noise      # routing noise amplitude: how much of the selection it changes
  python -m paper_2604_12219_amd.sweeps histogram  # selection counts of key blocks over a 50-step budget schedule

Everything runs through the HIP library (the dense kernel is the accuracy reference); nothing here is
needed by the forward path itself.  Prints markdown tables.

groups:    group = 0 drops the unselected blocks, 1 is the per-block first-order term (Eq.13), N_B the single
           global matrix of PISA (Eq.6/Eq.7), 32 the paper's choice (Sec. "Grouped First-Order Approximation").
histogram: the experiment behind the paper's selection-count figure (Sec. "Stochastic Routing"): with a
           deterministic top-k the same blocks are selected at every step; the seeded bias spreads the exact
           computation over more blocks.
"""
from __future__ import annotations

import argparse
import sys

import torch

import workloads

from . import pasa as P


def _time_ms(fn, reps=3):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _errors(out, ref):
    """per-head max|d|/max|ref| and mean|d|/mean|ref|, worst head"""
    d = (out.float() - ref.float()).abs()
    r = ref.float().abs()
    mx = (d.amax(dim=(2, 3)) / r.amax(dim=(2, 3))).max().item()
    mean = (d.mean(dim=(2, 3)) / r.mean(dim=(2, 3))).max().item()
    return mx, mean


def sweep_groups(workload: str, noise_amp: float, input_noise: float):
    w = workloads.WORKLOADS[workload]
    q, k, v = workloads.make_workload_qkv(w, device="cuda", noise_amplitude=input_noise)
    base = P.Shape.of(q, block=w.block)
    nb = P.num_blocks(base)
    k_sel = P.topk_count(nb, w.keep_ratio)
    dense = P.attn_dense_ref(q, k, v, base)
    t_dense = _time_ms(lambda: P.attn_dense_ref(q, k, v, base, out=dense))
    scores = P.block_score(q, k, base)
    idx, mask = P.route(scores, k_sel, w.seed, noise_amp)
    print(f"workload {w.name}: n={w.n} H={w.heads} d={w.d} block={w.block} k={k_sel}/{nb}, white-noise amplitude of the inputs "
          f"{input_noise}, dense kernel {t_dense:.2f} ms\n")
    print("| group | kv_stats ms | attention ms | speed-up over dense | max rel. error vs dense | mean rel. error vs dense |")
    print("|---|---|---|---|---|---|")
    out = torch.empty_like(q)
    for group in (0, 1, 16, 32, 64, nb):
        shape = P.Shape.of(q, block=w.block, group=group)
        ws = torch.empty(P.attn_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
        t_stats = _time_ms(lambda: P.kv_stats(k, v, shape, ws=ws))
        t_attn = _time_ms(lambda: P.sparse_attn_fwd(q, k, v, shape, idx, mask, out=out, ws=ws, prepared=True))
        mx, mean = _errors(out, dense)
        name = {0: "0 (drop)", 1: "1 (per block)", nb: f"{nb} (global)"}.get(group, str(group))
        print(f"| {name} | {t_stats:.2f} | {t_attn:.2f} | {t_dense / (t_stats + t_attn):.2f}x | {mx:.3e} | {mean:.3e} |")


def sweep_noise(workload: str):
    w = workloads.WORKLOADS[workload]
    q, k, _ = workloads.make_workload_qkv(w, device="cuda")
    shape = P.Shape.of(q, block=w.block)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, w.keep_ratio)
    scores = P.block_score(q, k, shape)
    _, m0 = P.route(scores, k_sel, w.seed, 0.0)
    print(f"workload {w.name}: k={k_sel}/{nb}; logit spread (std over key blocks, mean over rows) "
          f"{scores.std(dim=-1).mean().item():.3f}\n")
    print("| noise amplitude | selected blocks that differ from the deterministic top-k |")
    print("|---|---|")
    bits = torch.arange(32, device="cuda", dtype=torch.int32)
    for amp in (0.0, 0.03, 0.06, 0.125, 0.25, 0.5, 1.0):
        _, m = P.route(scores, k_sel, w.seed + 1, amp)
        changed = (((m & ~m0)[..., None] >> bits) & 1).sum().item()
        print(f"| {amp} | {changed / (m.shape[0] * nb * k_sel):.1%} |")


def selection_histogram(workload: str, n_steps: int, noise_amp: float):
    w = workloads.WORKLOADS[workload]
    bits = torch.arange(32, device="cuda", dtype=torch.int32)
    counts = {}
    for label, amp, kind in (("deterministic", 0.0, "uniform"), ("stochastic, uniform bias", noise_amp, "uniform"),
                             ("stochastic, Gumbel bias", noise_amp / 2, "gumbel")):
        total = None
        for step in range(n_steps):
            a = workloads.budget_schedule_noise_amplitude(step, n_steps)
            q, k, _ = workloads.make_workload_qkv(w, device="cuda", noise_amplitude=a, seed=w.seed)
            shape = P.Shape.of(q, block=w.block)
            nb = P.num_blocks(shape)
            k_sel = P.topk_count(nb, workloads.budget_schedule_keep_ratio(step, n_steps))
            scores = P.block_score(q, k, shape)
            _, m = P.route(scores, k_sel, w.seed + step, amp, noise=kind)
            sel = ((m[..., None] >> bits) & 1).reshape(m.shape[0], nb, -1)[..., :nb]  # [BH, query block, key block]
            total = sel.to(torch.int32) if total is None else total + sel
        counts[label] = total.float()
    print(f"workload {w.name}, {n_steps} steps of the budget schedule (keep ratio 0.1..0.4, input noise 1.0 -> 0.2), "
          f"per (head, query block, key block) pair: in how many steps was the pair computed exactly?\n")
    print("| routing | never | 1-5 steps | 6-25 steps | more than 25 | pairs ever selected | mean steps of a selected pair |")
    print("|---|---|---|---|---|---|---|")
    for label, c in counts.items():
        n = c.numel()
        ever = (c > 0).sum().item()
        print(f"| {label} | {(c == 0).sum().item() / n:.1%} | {((c >= 1) & (c <= 5)).sum().item() / n:.1%} | "
              f"{((c >= 6) & (c <= 25)).sum().item() / n:.1%} | {(c > 25).sum().item() / n:.1%} | {ever / n:.1%} | "
              f"{c.sum().item() / max(ever, 1):.1f} |")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=("groups", "noise", "histogram"))
    ap.add_argument("--workload", default=None)
    ap.add_argument("--noise-amp", type=float, default=0.125)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--input-noise", type=float, default=1.0,
                    help="white-noise amplitude of the synthetic inputs (1.0 = the benchmark's; smaller = smoother, more video-like)")
    args = ap.parse_args()
    P.load_library()
    assert torch.cuda.is_available(), "no GPU visible"
    if args.what == "groups":
        sweep_groups(args.workload or "wan14b-720p", args.noise_amp, args.input_noise)
    elif args.what == "noise":
        sweep_noise(args.workload or "wan1.3b-480p")
    else:
        selection_histogram(args.workload or "wan1.3b-480p", args.steps, args.noise_amp)
    return 0


if __name__ == "__main__":
    sys.exit(main())
