#!/usr/bin/env python3
"""Benchmark of the PASA sparse-attention forward on one MI355X.

One "step" = one pass of the whole hot path over one synthetic batch already resident in HBM:
  pasa_kv_stats -> pasa_block_score_with_stats -> pasa_route (fresh seed per step) -> pasa_sparse_attn_fwd_prepared
(the statistics do not depend on the queries, so they run first and scoring takes the block-mean keys from them instead of
reading K again; statistics + prepared attention are exactly what pasa_sparse_attn_fwd runs, issued separately so that HIP
events can bracket the attention kernel for the roofline figure).

Prints ONE JSON line: dense-equivalent TFLOP/s (4*B*H*n^2*d / time) as `value`, ms per call, the roofline
of the dominant kernel, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
HBM_PEAK_BYTES_PER_S = 8.0e12   # MI355X HBM3E
# HBM-side bytes per launch of the dominant kernel are MEASURED, not computed here: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this command, scaled by a plain copy of known size.  The summaries under profiles/ carry one line per
# measurement, "bench.traffic: workload=<name> group=<g> bytes_per_launch=<float> kernel_sha=<digest> measured=<date>",
# where the digest names the attention kernel's sources at the time of the run: a figure measured on other sources is
# not reported (roofline.traffic = null and roofline.traffic_source says why).
KERNEL_SOURCES = ("pasa_attn.hip", "pasa_mfma_pipes.hpp", "pasa_device.hpp", "pasa_kernels.hpp")


def kernel_source_digest():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2604_12219_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, group):
    """-> (bytes per launch or None, where the figure comes from / why there is none)"""
    digest = kernel_source_digest()
    stale = None
    pdir = os.path.join(ROOT, "profiles")
    for fn in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not fn.endswith(".txt"):
            continue
        for line in open(os.path.join(pdir, fn)):
            if not line.startswith("bench.traffic:"):
                continue
            kv = dict(item.split("=", 1) for item in line.split()[1:])
            if kv.get("workload") != workload or int(kv.get("group", -1)) != group:
                continue
            if kv.get("kernel_sha") == digest:
                return float(kv["bytes_per_launch"]), f"profiles/{fn} (rocprofv3 --pmc FETCH_SIZE x2 + WRITE_SIZE, measured {kv.get('measured')}, kernel sources {digest})"
            stale = f"profiles/{fn} was measured on other kernel sources ({kv.get('kernel_sha')}, now {digest}): not reported"
    return None, stale or f"no counter run committed for workload {workload}, group {group}"


NOISE_AMP_DEFAULT = 0.125       # logit units: calibrated once on the 480p workload (~15 % of selections change)


def algorithmic_flops(B, H, n, d, block, group, k_sel):
    nb = (n + block - 1) // block
    ng = (nb + min(group, nb) - 1) // min(group, nb) if group > 0 else 0
    bh = B * H
    exact = bh * nb * k_sel * 4 * block * block * d
    zeroth = bh * nb * 4 * block * nb * d if group > 0 else 0
    first = bh * nb * ng * 2 * block * d * d
    stats = bh * nb * 2 * block * d * d if group > 0 else 0
    scores = bh * nb * nb * 2 * d
    return dict(exact=exact, zeroth=zeroth, first=first, stats=stats, scores=scores,
                attn=exact + zeroth + first, total=exact + zeroth + first + stats + scores,
                dense=4 * bh * n * n * d)


def cpu_baseline(w, q, k, v, k_sel, noise_amp, group, target_seconds=20.0):
    """Time the fp64 oracle (its own scoring, routing, statistics and attention) on a sample sized for roughly
    `target_seconds`: a strided subset of the query blocks of head 0 if a whole head takes longer than that,
    otherwise as many whole heads as fit."""
    import numpy as np
    import oracle
    nb = w.n_blocks

    def head(h):
        return tuple(t[0, h:h + 1].float().cpu().numpy().astype(np.float64) for t in (q, k, v))

    q0, k0, v0 = head(0)
    t0 = time.perf_counter()
    s = oracle.block_scores(q0, k0, w.block).astype(np.float32)
    idx = oracle.route(s, k_sel, w.seed, noise_amp, bh_ids=[0])
    t_route = time.perf_counter() - t0
    # time the head's statistics alone, probe a few query blocks, then size the sample to the time target
    t0 = time.perf_counter()
    oracle.kv_stats(k0, v0, w.block, group)
    t_stats = time.perf_counter() - t0
    probe = list(range(0, nb, max(1, nb // 16)))[:16]
    t0 = time.perf_counter()
    oracle.pasa_attention(q0, k0, v0, idx, w.block, group=group, q_blocks=probe)
    per_block = max((time.perf_counter() - t0 - t_stats) / len(probe), 1e-4)
    n_sample = int(max(2, min(nb, (target_seconds - t_stats) / per_block)))
    stride = max(1, -(-nb // n_sample))
    blocks = list(range(0, nb, stride))
    if blocks[-1] != nb - 1:
        blocks.append(nb - 1)  # always include the ragged tail block
    t0 = time.perf_counter()
    oracle.pasa_attention(q0, k0, v0, idx, w.block, group=group, q_blocks=blocks)
    t_attn = time.perf_counter() - t0
    rows = sum(min(w.block, w.n - j * w.block) for j in blocks)
    frac = rows / w.n
    total = t_route * frac + t_attn  # scoring/routing cost scaled to the sampled share of the head
    per_head = t_route + t_stats + (t_attn - t_stats) / frac
    heads_done = frac
    sample = (f"head 0 of {w.heads}, {len(blocks)} of {nb} query blocks (stride {stride}, tail block included), "
              f"full-head statistics and routing")
    if stride == 1:  # a whole head fits the budget: add whole heads (each with its own scoring and routing)
        extra = int(min(w.heads - 1, max(0, round((target_seconds - total) / per_head))))
        for h in range(1, 1 + extra):
            qh, kh, vh = head(h)
            t0 = time.perf_counter()
            sh = oracle.block_scores(qh, kh, w.block).astype(np.float32)
            ih = oracle.route(sh, k_sel, w.seed, noise_amp, bh_ids=[h])
            oracle.pasa_attention(qh, kh, vh, ih, w.block, group=group)
            total += time.perf_counter() - t0
        heads_done = 1 + extra
        sample = f"heads 0..{extra} of {w.heads}, every query block, each head with its own scoring, routing and statistics"
    dense_equiv = 4.0 * w.n * w.n * w.d * heads_done / total / 1e12
    return dict(value=dense_equiv, unit="TFLOP/s (dense-equivalent)", cores=oracle.num_threads(), kind="oracle",
                sample=f"{sample}; {total:.1f} s", seconds=total, seconds_per_head_extrapolated=per_head)


def run_budget_schedule(args):
    """The budget-schedule workload: the Wan-1.3B 480p shape run for 50 denoising steps, keep ratio per step from
    workloads.budget_schedule_keep_ratio (k from 51 to 205 of 512 blocks), a fresh routing seed and freshly drawn
    inputs (white-noise amplitude 1.0 -> 0.2) per step.  The inputs of all 50 steps are generated first and stay
    resident in HBM (15 GB); scores, index lists, bitmaps, workspaces and the output are allocated ONCE, sized for the
    largest k, and every step runs in them: k is a runtime argument, nothing is recompiled or re-allocated.
    One bench "step" is one denoising step (one call of the whole hot path); --steps is fixed at the schedule length and
    --warmup runs that many leading steps of the schedule once, untimed, beforehand."""
    import torch
    import paper_2604_12219_amd as P
    import workloads

    P.load_library()
    assert torch.cuda.is_available(), "no GPU visible"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = workloads.WORKLOADS["wan1.3b-480p"]
    n_steps = 50
    nb, bh = w.n_blocks, w.batch * w.heads
    keeps = [workloads.budget_schedule_keep_ratio(s, n_steps) for s in range(n_steps)]
    ks = [P.topk_count(nb, r) for r in keeps]
    k_max = max(ks)
    inputs = [workloads.make_workload_qkv(w, device=dev, noise_amplitude=workloads.budget_schedule_noise_amplitude(s, n_steps),
                                          seed=w.seed + s) for s in range(n_steps)]
    shape = P.Shape.of(inputs[0][0], block=w.block, group=args.group)
    scores = torch.empty((bh, nb, nb), dtype=torch.float32, device=dev)
    idx_buf = torch.empty(bh * nb * k_max, dtype=torch.int32, device=dev)
    mask = torch.empty((bh, nb, P.mask_words(nb)), dtype=torch.int32, device=dev)
    ws_score = torch.empty(P.score_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    ws_attn = torch.empty(P.attn_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    out = torch.empty_like(inputs[0][0])
    allocated_before = torch.cuda.memory_allocated()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(n_steps)]

    def step(s, events=None):
        q, k, v = inputs[s]
        idx = idx_buf[: bh * nb * ks[s]].view(bh, nb, ks[s])
        if events: events[0].record()
        P.kv_stats(k, v, shape, ws=ws_attn)
        if events: events[1].record()
        P.block_score(q, None, shape, scores=scores, ws=ws_score, stats_ws=ws_attn)
        if events: events[2].record()
        P.route(scores, ks[s], w.seed + s, args.noise_amp, idx=idx, mask=mask)
        if events: events[3].record()
        P.sparse_attn_fwd(q, k, v, shape, idx, mask, out=out, ws=ws_attn, prepared=True)
        if events: events[4].record()

    for s in range(min(args.warmup, n_steps)):
        step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(n_steps):
        step(s, ev[s])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert torch.cuda.memory_allocated() == allocated_before, "a step allocated device memory"
    per_step_ms = [e[0].elapsed_time(e[4]) for e in ev]
    attn_ms = [e[3].elapsed_time(e[4]) for e in ev]
    stage_ms = [sum(e[i].elapsed_time(e[i + 1]) for e in ev) / n_steps for i in range(4)]
    fl = [algorithmic_flops(w.batch, w.heads, w.n, w.d, w.block, args.group, k_sel) for k_sel in ks]
    attn_flops, dense_flops = sum(f["attn"] for f in fl), sum(f["dense"] for f in fl)
    attn_total_s = sum(attn_ms) * 1e-3
    attn_tflops = attn_flops / attn_total_s / 1e12
    dense_ms = None
    if not args.no_dense:
        q, k, v = inputs[0]
        P.attn_dense_ref(q, k, v, shape, out=out, ws=ws_attn)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            P.attn_dense_ref(q, k, v, shape, out=out, ws=ws_attn)
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / 3
    result = {
        "metric": "dense-equivalent TFLOP/s over the 50-step budget schedule (sum of 4*B*H*n^2*d / total time); ms per denoising step in ms_per_step",
        "value": dense_flops / elapsed / 1e12,
        "unit": "TFLOP/s (dense-equivalent)",
        "n_gpus": 1, "steps": n_steps, "warmup": min(args.warmup, n_steps), "ms_per_step": elapsed / n_steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "budget-schedule", "shape": w.name, "B": w.batch, "H": w.heads, "n": w.n, "d": w.d, "block": w.block,
                   "n_blocks": nb, "group": args.group, "noise_amp": args.noise_amp, "seed": "seed + step",
                   "keep_ratio": "0.1 + 0.3*exp(-((t-0.3)/0.1)^2), t = step/50", "k_sel_min": min(ks), "k_sel_max": k_max,
                   "k_sel_mean": sum(ks) / n_steps, "input_noise_amplitude": "1.0 -> 0.2, linear"},
        "total_ms": elapsed * 1e3,
        "per_step": {"k_sel": ks, "ms": [round(x, 4) for x in per_step_ms], "attn_ms": [round(x, 4) for x in attn_ms]},
        "stage_ms_mean": {"kv_stats": stage_ms[0], "block_score": stage_ms[1], "route": stage_ms[2], "sparse_attn": stage_ms[3]},
        "buffers_allocated_once": True,
        "dense_ref_ms": dense_ms,
        "speedup_vs_dense_ref": (dense_ms * n_steps / (elapsed * 1e3)) if dense_ms else None,
        "roofline": {"kernel": "attn_kernel (sparse: exact tiles + grouped approximation), all 50 launches", "bound": "mfma",
                     "achieved": attn_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "avg_launch_ms": sum(attn_ms) / n_steps, "flops_per_launch": attn_flops / n_steps},
    }
    if not args.no_cpu_baseline:
        q, k, v = inputs[15]  # the step with the largest k
        result["cpu_baseline"] = cpu_baseline(w, q, k, v, ks[15], args.noise_amp, args.group, args.cpu_seconds)
        result["cpu_baseline"]["sample"] = "schedule step 15 (k = %d): " % ks[15] + result["cpu_baseline"]["sample"]
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="wan14b-720p",
                    help="a name of workloads.WORKLOADS, or budget-schedule (50 denoising steps of the 480p shape with a per-step keep ratio)")
    ap.add_argument("--noise-amp", type=float, default=NOISE_AMP_DEFAULT)
    ap.add_argument("--group", type=int, default=32)
    ap.add_argument("--kv-slices", type=int, default=0, help="key-range slices of the attention kernel (0 = the library's choice)")
    ap.add_argument("--with-prior", action="store_true",
                    help="route on the full logit of Eq.8: statistics first, then the covariance prior as key bias (not the default path)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-mfma-probe", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--token-major", action="store_true",
                    help="Q, K, V and O as [B,H,n,d] views of token-major storage [B,n,H,d] (what a transformer block hands over) "
                         "instead of head-major storage (not the default path)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain device copy of Q (known size) so that hardware byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (heads would shard across GPUs with no collective); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.workload == "budget-schedule":
        return run_budget_schedule(args)

    import torch
    import paper_2604_12219_amd as P
    import workloads

    P.load_library()  # fails loudly when the HIP library is missing
    assert torch.cuda.is_available(), "no GPU visible"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = workloads.WORKLOADS[args.workload]
    q, k, v = workloads.make_workload_qkv(w, device=dev)
    if args.token_major:  # the same values, rows of one head H*d elements apart
        q, k, v = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))
    shape = P.Shape.of(q, block=w.block, group=args.group, kv_slices=args.kv_slices)
    nb = P.num_blocks(shape)
    k_sel = P.topk_count(nb, w.keep_ratio)
    bh = w.batch * w.heads

    scores = torch.empty((bh, nb, nb), dtype=torch.float32, device=dev)
    idx = torch.empty((bh, nb, k_sel), dtype=torch.int32, device=dev)
    mask = torch.empty((bh, nb, P.mask_words(nb)), dtype=torch.int32, device=dev)
    ws_score = torch.empty(P.score_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    ws_attn = torch.empty(P.attn_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    out = torch.empty_like(q)
    n_ev = args.steps
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(n_ev)]

    beta = torch.empty((bh, nb), dtype=torch.float32, device=dev) if args.with_prior else None

    def step(i, events=None):
        if args.with_prior:  # statistics first: the prior needs them; its time is booked under block_score
            P.kv_stats(k, v, shape, ws=ws_attn)
            if events: events[0].record()
            P.key_prior(k, v, shape, ws_attn, beta=beta)
            P.block_score(q, k, shape, key_bias=beta, scores=scores, ws=ws_score)
            if events: events[1].record()
            P.route(scores, k_sel, w.seed + i, args.noise_amp, idx=idx, mask=mask)
            if events: events[2].record()
            if events: events[3].record()
        elif args.group > 0:  # statistics first (they do not depend on the queries): scoring takes the block-mean keys from them
            if events: events[0].record()
            P.kv_stats(k, v, shape, ws=ws_attn)
            if events: events[1].record()
            P.block_score(q, None, shape, scores=scores, ws=ws_score, stats_ws=ws_attn)
            if events: events[2].record()
            P.route(scores, k_sel, w.seed + i, args.noise_amp, idx=idx, mask=mask)
            if events: events[3].record()
        else:  # approximation off: no statistics
            if events: events[0].record()
            if events: events[1].record()
            P.block_score(q, k, shape, scores=scores, ws=ws_score)
            if events: events[2].record()
            P.route(scores, k_sel, w.seed + i, args.noise_amp, idx=idx, mask=mask)
            if events: events[3].record()
        P.sparse_attn_fwd(q, k, v, shape, idx, mask, out=out, ws=ws_attn, prepared=True)
        if events: events[4].record()

    if args.copy_probe:  # 2 * q.numel() * 2 bytes of traffic: read Q, write a copy
        probe = torch.empty_like(q)
        probe.copy_(q)
        del probe
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, ev[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    stage_ms = [sum(e[s].elapsed_time(e[s + 1]) for e in ev) / n_ev for s in range(4)]
    call_ms = sorted(e[0].elapsed_time(e[4]) for e in ev)  # per call, events on the stream
    attn_ms = stage_ms[3]

    fl = algorithmic_flops(w.batch, w.heads, w.n, w.d, w.block, args.group, k_sel)
    dense_equiv_tflops = fl["dense"] / (ms_per_step * 1e-3) / 1e12
    computed_tflops = fl["total"] / (ms_per_step * 1e-3) / 1e12
    attn_tflops = fl["attn"] / (attn_ms * 1e-3) / 1e12

    dense_ms = None
    if not args.no_dense:
        P.attn_dense_ref(q, k, v, shape, out=out, ws=ws_attn)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 2
        e0.record()
        for _ in range(reps):
            P.attn_dense_ref(q, k, v, shape, out=out, ws=ws_attn)
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / reps

    qkv_bytes = w.batch * w.heads * w.n * w.d * 2
    score_bytes = bh * nb * nb * 4
    means_bytes = bh * nb * w.d * 4  # pooled means of one tensor (split bf16 pairs)
    # which timed interval holds which stage (the covariance-prior path books the prior under block_score and runs the
    # statistics before the first event)
    slot = {"block_score": 0, "route": 1, "kv_stats": 2} if args.with_prior else {"kv_stats": 0, "block_score": 1, "route": 2}
    stage = {name: stage_ms[i] for name, i in slot.items()}
    reads_k = args.with_prior or args.group == 0  # otherwise scoring takes the block-mean keys from the statistics
    stage_bytes = {"block_score": (2 if reads_k else 1) * qkv_bytes + score_bytes + 3 * means_bytes,
                   "route": score_bytes + bh * nb * (k_sel + P.mask_words(nb)) * 4,
                   "kv_stats": 2 * qkv_bytes + (bh * ((nb + 31) // 32) * 64 * w.d * 2 + means_bytes if args.group else 0)}
    stage_hbm = {name: {"algorithmic_GB": stage_bytes[name] / 1e9,
                        "achieved_TBps": stage_bytes[name] / (stage[name] * 1e-3) / 1e12,
                        "frac_of_8TBps": stage_bytes[name] / (stage[name] * 1e-3) / HBM_PEAK_BYTES_PER_S}
                 for name in ("block_score", "route", "kv_stats")} if not args.with_prior and args.group > 0 else None
    # bytes of K/V tiles the attention kernel asks for if no tile were reused between query blocks
    tile_bytes = bh * nb * k_sel * 2 * w.block * w.d * 2
    traffic, traffic_source = (measured_traffic(w.name, args.group) if args.kv_slices in (0, 1) and not args.with_prior and not args.token_major
                               else (None, "not the default path"))
    # what a loop of nothing but MFMAs reaches on this device right now (the published peak assumes 2.4 GHz)
    mfma_loop = None if args.no_mfma_probe else P.mfma_probe()
    # ... and with N(0,1)-like operands in the registers: the matrix cores draw more power and the clock drops
    mfma_loop_data = None if args.no_mfma_probe else P.mfma_probe(random_operands=True)
    result = {
        "metric": "dense-equivalent TFLOP/s of one PASA sparse-attention call (4*B*H*n^2*d / time); ms per call in ms_per_step",
        "value": dense_equiv_tflops,
        "unit": "TFLOP/s (dense-equivalent)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.batch, "H": w.heads, "n": w.n, "d": w.d, "block": w.block,
                   "keep_ratio": w.keep_ratio, "k_sel": k_sel, "n_blocks": nb, "group": args.group,
                   "noise_amp": args.noise_amp, "seed": w.seed, "kv_slices": args.kv_slices, "covariance_prior": args.with_prior,
                   "layout": "token-major [B,n,H,d] storage" if args.token_major else "head-major [B,H,n,d] storage"},
        "ms_per_call_median": call_ms[len(call_ms) // 2], "ms_per_call_min": call_ms[0],
        "stage_ms": {"kv_stats": stage["kv_stats"], "block_score": stage["block_score"], "route": stage["route"], "sparse_attn": attn_ms},
        # the HBM-bound stages against the 8 TB/s peak: algorithmic bytes (inputs read once, outputs written once) / time
        "stage_hbm": stage_hbm,
        "computed_tflops": computed_tflops,
        "algorithmic_tflop": {kk: vv / 1e12 for kk, vv in fl.items()},
        "dense_ref_ms": dense_ms,
        "dense_ref_tflops": (fl["dense"] / (dense_ms * 1e-3) / 1e12) if dense_ms else None,
        "speedup_vs_dense_ref": (dense_ms / ms_per_step) if dense_ms else None,
        "roofline": {"kernel": "attn_kernel (sparse: exact tiles + grouped approximation)", "bound": "mfma",
                     "achieved": attn_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     # what the launch is limited by, from the counters: K/V tile reads that miss the L2 and cross the fabric
                     "limiter": "reads through the fabric (L2 misses of K/V tiles)" if traffic else None,
                     "traffic_rate_TBps": (traffic / (attn_ms * 1e-3) / 1e12) if traffic else None,
                     "avg_launch_ms": attn_ms, "flops_per_launch": fl["attn"],
                     "unshared_tile_TBps": tile_bytes / (attn_ms * 1e-3) / 1e12,
                     "mfma_loop_tflops": mfma_loop, "mfma_loop_random_operands_tflops": mfma_loop_data},
        "paper_context": "paper reports end-to-end video latency only (8x H800): PASA 2.19x over dense at Wan 2.1-14B 720p",
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, q, k, v, k_sel, args.noise_amp, args.group, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
