#!/usr/bin/env python3
"""Benchmark of the policy-gradient head on one MI355X.

A step is one pass of the whole path over one synthetic packed microbatch that is already
resident in device memory: trloo_advantage (returns + leave-one-out advantages of the whole
rollout batch) followed by pg_loss_fwd_bwd (mismatch pre-pass, fused LM-head forward, clipped
surrogate, backward to dH and dW).  The workload is the Qwen3-14B head shape (hidden 5120,
vocab 151936) with 32768 loss tokens: entry [2] of the benchmark's configuration list.

Prints ONE JSON line (see README / DESIGN for the fields).  The oracle is imported only for the
`cpu_baseline` leg, which times it on a bounded row sample of the same shape.
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

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak (published)
TRAFFIC_SOURCE = "profiles/gemm_store_kernel_hbm_traffic.md"


def measured_mfma_only_tflops():
    """What the MFMA instruction alone sustains on THIS box right now, with operands and accumulators in
    registers and random operands: tile_bench's register-only loop, run as a child process (context for the
    roofline fraction, which divides by the published peak).  None when the tool is not built or fails."""
    import re
    import subprocess
    exe = os.path.join(ROOT, "paper_2602_05885_amd", "tile_bench")
    if not os.path.exists(exe):
        return None
    try:
        out = subprocess.run([exe, "1", "3"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=60).stdout
    except Exception:
        return None
    rates = [float(m.group(1)) for m in re.finditer(r"random operands, 1 workgroup.*?([0-9.]+) TFLOP/s", out)]
    return rates[-1] if rates else None

# L2<->fabric bytes per gemm_store_kernel launch from the FETCH_SIZE / WRITE_SIZE counter runs
# summarised in profiles/gemm_store_kernel_hbm_traffic.md (mean over a step's 14 launches, each
# counter scaled by what it reads for a plain 1 GiB copy).  Valid only for the kernel sources the
# counters were taken with: the digest below is of csrc/gemm_core.h + csrc/kernels_gemm.hip.
TRAFFIC_GEMM_STORE = {"read_bytes": 5873740.1 * 1024 * 2.000, "write_bytes": 547145.8 * 1024 * 1.000,
                      "sources_sha256": "b723ddea9561855eacbc87e3419af6609ef3501b8bad89cd1a341ee4c90ba681"}


def kernel_sources_digest() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in ("gemm_core.h", "kernels_gemm.hip"):
        with open(os.path.join(ROOT, "paper_2602_05885_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(kernel: str):
    """L2<->fabric bytes per launch of the dominant kernel from the stored counter runs, or None when they
    do not describe the kernel that is about to run (another kernel dominates, or the sources changed)."""
    if kernel != "gemm_store_kernel" or kernel_sources_digest() != TRAFFIC_GEMM_STORE["sources_sha256"]:
        return None
    return TRAFFIC_GEMM_STORE["read_bytes"] + TRAFFIC_GEMM_STORE["write_bytes"]


def cpu_baseline(spec, rows: int):
    """Times the fp64 oracle (as it stands) on `rows` active rows at the full d and V."""
    import numpy as np
    import torch
    from oracle import pg_oracle as O
    from paper_2602_05885_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    H, W, y = synth.make_head(rows, spec.d, spec.V, spec.dtype, spec.seed + 1000, "cpu", spec.unit_rms)
    Hn, Wn, yn = H.double().numpy(), W.double().numpy(), y.numpy()
    del H, W
    n_seg = 4
    cu = np.linspace(0, rows, n_seg + 1).astype(np.int32)
    mask = np.ones(rows, np.uint8)
    R = np.random.default_rng(0).random((2, 2, 1)).astype(np.float32)
    t0 = time.perf_counter()
    _, A, _ = O.trloo_advantage(R, np.ones_like(R, dtype=np.uint8), 1.0)
    out = O.pg_loss_fwd_bwd(Hn, Wn, yn, mask, cu, A.reshape(-1), None, None, O.Params(temperature=spec.temperature))
    dt = time.perf_counter() - t0
    assert np.isfinite(out["loss"])
    return {"value": rows / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{rows} active rows at d={spec.d}, V={spec.V}, fp64 numpy, fwd+bwd, {dt:.1f} s"}


def aux_stage_times(B, torch, dev, rewards, valid, out, loss_mask, old_logp, rollout_logp, dW, H, reps: int = 20):
    """Microseconds per call of the small stages around the path (outside the timed region): rewards
    and PRS on the rollout batch's samples, both advantage baselines, the monitors on the step's outputs."""
    n = rewards.numel()
    g = torch.Generator(device="cpu").manual_seed(1)
    correct = (torch.rand(n, generator=g) < 0.5).to(torch.uint8).to(dev)
    t_ref = torch.rand(n, generator=g).add(0.5).to(dev)
    t_ker = torch.rand(n, generator=g).add(0.25).to(dev)
    t_tot = torch.rand(n, generator=g).add(0.5).to(dev)
    t_gen = (t_tot * 0.5).contiguous()
    vflat = valid.reshape(-1).contiguous()
    calls = {
        "turn_reward": lambda: B.turn_reward(correct, t_ref, t_ker, t_gen, t_tot, 3.0),
        "prs_retain": lambda: B.prs_retain(t_gen, vflat, 1234, 0.3, 0.1),
        "trloo_advantage": lambda: B.trloo_advantage(rewards, valid, 1.0),
        "grpo_advantage": lambda: B.grpo_advantage(rewards, valid, 1.0),
        "pg_monitors": lambda: B.pg_monitors(out["logp"], rollout_logp if rollout_logp is not None else old_logp,
                                             out["entropy"], loss_mask, out["dH"], dW),
    }
    gamma = torch.ones(H.shape[1], dtype=H.dtype, device=dev)
    h_buf, dx_buf = torch.empty_like(H), torch.empty_like(H)
    calls["pg_rmsnorm_fwd"] = lambda: B.pg_rmsnorm_fwd(H, gamma, 1e-6, want_rstd=False, out=h_buf)
    calls["pg_rmsnorm_bwd"] = lambda: B.pg_rmsnorm_bwd(H, gamma, out["dH"], 1e-6, out=dx_buf)
    res = {}
    for name, fn in calls.items():
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name] = e0.elapsed_time(e1) / reps * 1e3
    # what a plain device-to-device copy of the same [T, d] sustains on this machine (the practical ceiling of a
    # streaming kernel: read + write)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    dx_buf.copy_(H)
    e0.record()
    for _ in range(reps):
        dx_buf.copy_(H)
    e1.record()
    torch.cuda.synchronize()
    res["plain_copy_GBps"] = 2 * H.numel() * H.element_size() / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9
    nbytes = H.numel() * H.element_size()
    res["pg_rmsnorm_fwd_GBps"] = 2 * nbytes / (res["pg_rmsnorm_fwd"] * 1e-6) / 1e9       # x read, h written
    res["pg_rmsnorm_bwd_GBps"] = 3 * nbytes / (res["pg_rmsnorm_bwd"] * 1e-6) / 1e9       # x, dh read, dx written
    res["pg_monitors_GBps"] = ((dW.numel() * dW.element_size() + nbytes) / (res["pg_monitors"] * 1e-6) / 1e9)
    return res


def timed(torch, B, fn, steps, warmup):
    """ms per step (host clock around a synchronised region) and the per-kernel-class event times."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    B.pg_profile_enable(True, 64 * max(steps, 1))
    t0 = time.perf_counter()
    for _ in range(steps):
        out = fn()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = B.pg_profile_read()
    B.pg_profile_enable(False)
    kern = {k: {"launches_per_step": n / steps, "ms_per_step": ms / steps} for k, (ms, n) in prof.items() if n}
    return dt / steps * 1e3, kern, out


def forward_only_workload(torch, B, synth, dev, config, steps, warmup, scale_rows=1.0):
    """pg_logprob_fwd over all rows of a configuration: ms per step, rows/s, % of peak on 2dV."""
    spec = synth.SPECS[config]
    batch = synth.make_batch(spec, scale_rows)
    T, d, V = batch.T, spec.d, spec.V
    H, W, y = synth.make_head(T, d, V, spec.dtype, spec.seed, dev, spec.unit_rms)
    prm = B.Params(dtype=0 if spec.dtype == "bf16" else 1, temperature=spec.temperature)
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
    outbuf = tuple(torch.empty(T, dtype=torch.float32, device=dev) for _ in range(3))
    ms, kern, _ = timed(torch, B, lambda: B.pg_logprob_fwd(H, W, y, None, prm, ws, out=outbuf), steps, warmup)
    flops = 2.0 * d * V * T
    return {"workload": f"configs[{config}] {spec.name}: d={d}, V={V}, {T} rows, forward only, temperature {spec.temperature}",
            "step": "pg_logprob_fwd", "steps": steps, "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3),
            "flops_per_token": "2dV", "pct_mfma_peak": 100.0 * flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "kernels": kern}


def bench_forward_only(args, torch, B, synth, dev):
    """pg_logprob_fwd (log-prob, entropy, logsumexp) over all rows of the chosen configuration."""
    spec = synth.SPECS[args.config]
    batch = synth.make_batch(spec, args.scale_rows)
    T, d, V = batch.T, spec.d, spec.V
    H, W, y = synth.make_head(T, d, V, spec.dtype, spec.seed, dev, spec.unit_rms)
    prm = B.Params(dtype=0 if spec.dtype == "bf16" else 1, temperature=spec.temperature)
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
    outbuf = tuple(torch.empty(T, dtype=torch.float32, device=dev) for _ in range(3))
    for _ in range(args.warmup):
        B.pg_logprob_fwd(H, W, y, None, prm, ws, out=outbuf)
    torch.cuda.synchronize()
    B.pg_profile_enable(True, 8 * max(args.steps, 1))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        B.pg_logprob_fwd(H, W, y, None, prm, ws, out=outbuf)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = B.pg_profile_read()
    B.pg_profile_enable(False)
    ms_step = dt / args.steps * 1e3
    flops = 2.0 * d * V * T
    k_ms = prof["fwd"][0] / max(prof["fwd"][1], 1)
    ach = flops / (k_ms * 1e-3) / 1e12
    line = {"metric": "LM-head log-prob forward tokens/sec (old-policy recompute); % bf16 MFMA peak",
            "value": T * args.steps / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16" if spec.dtype == "bf16" else "f32", "data": "synthetic",
            "config": {"workload": f"configs[{args.config}] {spec.name}: d={d}, V={V}, {T} rows, forward only",
                       "temperature": spec.temperature, "step": "pg_logprob_fwd"},
            "pct_mfma_peak_2dV": 100.0 * flops / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "roofline": {"bound": "mfma", "kernel": "lmhead_fwd_kernel", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                         "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                         "flops_per_launch": flops, "avg_launch_ms": k_ms, "launches_per_step": 1.0},
            "cpu_baseline": None}
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="index into the workload list (default: 14B head, 32k loss tokens)")
    ap.add_argument("--mismatch-mode", type=int, default=2)
    ap.add_argument("--cpu-rows", type=int, default=2048, help="rows of the oracle's timed sample (0 = skip)")
    ap.add_argument("--scale-rows", type=float, default=1.0, help="shrink the packed microbatch (debugging)")
    ap.add_argument("--workload", choices=["pg", "sft", "fwd", "shard", "bwd"], default="pg",
                    help="pg: trloo_advantage + pg_loss_fwd_bwd (the headline); sft: pg_sft_fwd_bwd at the same shape; "
                         "fwd: pg_logprob_fwd over every row (the old-policy recompute); shard: one vocab shard's "
                         "share of the step (pg_head_shard_fwd + pg_head_partials_merge + pg_loss_shard_bwd); "
                         "bwd: pg_loss_shard_bwd on the whole head from the softmax states the old-policy "
                         "recompute left behind (valid while the weights are those of that recompute: the "
                         "forward contraction is not repeated, 6dV instead of 8dV flops per token)")
    ap.add_argument("--vocab-shards", type=int, default=2, help="number of vocab shards for --workload shard")
    ap.add_argument("--no-others", dest="others", action="store_false",
                    help="skip the secondary workloads that the default run times after the headline "
                         "(other_workloads: Sec. 5.1's rejection rule, backward from states, fused RMS normalisation, forward-only 128k rows)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run three plain device-to-device copies of this size (the known-size reference "
                         "that hardware-counter byte counts are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 "
              "(the path shards by token rows; no multi-GPU figure is produced)", file=sys.stderr)
        sys.exit(2)

    mfma_only = measured_mfma_only_tflops() if args.workload == "pg" else None

    import torch
    from paper_2602_05885_amd import binding as B
    from paper_2602_05885_amd import synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "fwd":
        return bench_forward_only(args, torch, B, synth, dev)
    spec = synth.SPECS[args.config]
    batch = synth.make_batch(spec, args.scale_rows)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    H, W, y = synth.make_head(T, d, V, spec.dtype, spec.seed, dev, spec.unit_rms)
    loss_mask = torch.from_numpy(batch.loss_mask).to(dev)
    cu = torch.from_numpy(batch.cu_seqlens).to(dev)
    seg_sample = torch.from_numpy(batch.seg_sample).to(dev)
    rewards = torch.from_numpy(batch.rewards).to(dev)
    valid = torch.from_numpy(batch.valid).to(dev)
    n_loss = int(batch.loss_mask.sum())

    dtype_id = 0 if spec.dtype == "bf16" else 1
    prm = B.Params(dtype=dtype_id, temperature=spec.temperature, mismatch_mode=args.mismatch_mode)

    # old-policy log-probs come from the forward call of the library itself (the RL step's
    # "recompute" stage); the rollout engine's log-probs are those plus noise and outliers.
    ws_f = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
    old_logp, _, _ = B.pg_logprob_fwd(H, W, y, loss_mask, prm, ws_f, want_entropy=False, want_lse=False)
    torch.cuda.synchronize()
    del ws_f
    rollout_logp = synth.perturb_logp(old_logp, spec.logp_noise, spec.outlier_frac, spec.seed + 1)
    if args.mismatch_mode == 0:
        rollout_logp = None

    V_full = V
    if args.workload == "shard":
        # this process plays shard 0 of --vocab-shards equal shards; the other shards' softmax states
        # (what the exchange would deliver) are prepared once, outside the timed region
        g = args.vocab_shards
        assert g >= 2 and V // g >= 1
        Vs = V // g
        others = None
        for k in range(1, g):
            a, b = k * Vs, (V if k == g - 1 else (k + 1) * Vs)
            wsk = B.alloc_workspace(T, d, b - a, 0, prm, B.CALL_LOGPROB_FWD, dev)
            pk = B.pg_head_shard_fwd(H, W[a:b], y, loss_mask, a, prm, wsk)
            others = pk if others is None else B.pg_head_partials_merge(others, pk, out=others)
            torch.cuda.synchronize()
            del wsk
        W = W[:Vs]
        V = Vs
        part = torch.empty((T, 4), dtype=torch.float32, device=dev)
        merged = torch.empty_like(part)
    if args.workload == "bwd":
        # the recompute stage, run once outside the timed region, keeps the rows' softmax states
        wsk = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
        merged = B.pg_head_shard_fwd(H, W, y, loss_mask, 0, prm, wsk)
        torch.cuda.synchronize()
        del wsk
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    dW = torch.empty((V, d), dtype=torch.float32, device=dev)
    outbuf = (torch.empty(1, dtype=torch.float32, device=dev),
              torch.empty((T, d), dtype=torch.float32, device=dev) if args.workload in ("shard", "bwd") else torch.empty_like(H),
              torch.empty(T, dtype=torch.float32, device=dev), torch.empty(T, dtype=torch.float32, device=dev),
              torch.empty(8, dtype=torch.int64, device=dev))

    def step():
        if args.workload == "sft":
            return B.pg_sft_fwd_bwd(H, W, y, loss_mask, prm, ws, dW=dW, out=outbuf)
        adv, _, _ = B.trloo_advantage(rewards, valid, 1.0, want_returns=False, want_group_n=False)
        if args.workload == "shard":
            B.pg_head_shard_fwd(H, W, y, loss_mask, 0, prm, ws, out=part)
            B.pg_head_partials_merge(part, others, out=merged)
            return B.pg_loss_shard_bwd(H, W, y, loss_mask, cu, adv.reshape(-1), seg_sample, old_logp, rollout_logp,
                                       merged, 0, prm, ws, dH_f32=True, dW=dW, out=outbuf)
        if args.workload == "bwd":
            return B.pg_loss_shard_bwd(H, W, y, loss_mask, cu, adv.reshape(-1), seg_sample, old_logp, rollout_logp,
                                       merged, 0, prm, ws, dH_f32=True, dW=dW, out=outbuf)
        return B.pg_loss_fwd_bwd(H, W, y, loss_mask, cu, adv.reshape(-1), seg_sample, old_logp, rollout_logp, prm, ws,
                                 dW=dW, out=outbuf)

    if args.calib_copy_mib > 0:
        src = torch.zeros(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        out = step()
    torch.cuda.synchronize()
    B.pg_profile_enable(True, 64 * max(args.steps, 1))
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # step boundaries, same stream
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()
        out = step()
    marks[args.steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = B.pg_profile_read()
    B.pg_profile_enable(False)
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))

    # the same step once more with dW += (gradient accumulation over microbatches), outside the timed region
    acc_ms = None
    if args.workload == "pg" and args.steps > 0:
        prm_acc = B.Params(dtype=dtype_id, temperature=spec.temperature, mismatch_mode=args.mismatch_mode,
                           accumulate_dW=1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        adv0, _, _ = B.trloo_advantage(rewards, valid, 1.0, want_returns=False, want_group_n=False)
        n_acc = 3
        e0.record()
        for _ in range(n_acc):
            B.pg_loss_fwd_bwd(H, W, y, loss_mask, cu, adv0.reshape(-1), seg_sample, old_logp, rollout_logp, prm_acc, ws,
                              dW=dW, out=outbuf)
        e1.record()
        torch.cuda.synchronize()
        acc_ms = e0.elapsed_time(e1) / n_acc
        out = step()                       # leave dW and the outputs as one overwrite step produces them
        torch.cuda.synchronize()

    counters = out["counters"].cpu().numpy()
    n_active = int(counters[0])
    loss = float(out["loss"][0])
    assert loss == loss, "loss is NaN"
    ms_step = dt / args.steps * 1e3
    tokens_per_s = n_active * args.steps / dt

    # ---- roofline of the dominant kernel ----
    # Algorithmic flops of each launch class per step: every class is one contraction over the whole
    # vocabulary, 2 d V flops per active token.
    rows_of = {"fwd": V, "dlogits": V, "dw": V, "dh": V}
    kernel_of = {"fwd": "lmhead_fwd_kernel", "dlogits": "lmhead_dlogits_kernel", "dw": "gemm_store_kernel",
                 "dh": "gemm_store_kernel"}
    kern = {}
    for k, (ms, n) in prof.items():
        if n:
            fl = 2.0 * d * rows_of[k] * n_active                      # per step
            kern[k] = {"kernel": kernel_of[k], "launches_per_step": n / args.steps, "ms_per_step": ms / args.steps,
                       "avg_launch_ms": ms / n, "flop_per_step": fl, "tflops": fl * args.steps / (ms * 1e-3) / 1e12}
    by_kernel = {}
    for k, v in kern.items():
        b = by_kernel.setdefault(v["kernel"], {"ms": 0.0, "launches": 0.0, "flop": 0.0})
        b["ms"] += v["ms_per_step"]
        b["launches"] += v["launches_per_step"]
        b["flop"] += v["flop_per_step"]
    dom = max(by_kernel, key=lambda k: by_kernel[k]["ms"])
    b = by_kernel[dom]
    achieved = b["flop"] / (b["ms"] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_TFLOPS,
                "measured_mfma_only_tflops": mfma_only,          # tile_bench's register-only loop, this run, this box
                "frac_of_measured_mfma_rate": achieved / mfma_only if mfma_only else None,
                "traffic": measured_traffic(dom),
                "traffic_source": TRAFFIC_SOURCE if measured_traffic(dom) is not None else None,
                "flops_per_launch": b["flop"] / b["launches"], "avg_launch_ms": b["ms"] / b["launches"],
                "launches_per_step": b["launches"]}
    n_contractions = 3.0 if args.workload == "bwd" else 4.0       # logits (twice unless the forward is not repeated), dH, dW
    executed = 2.0 * n_contractions * d * V * n_active / (ms_step * 1e-3) / 1e12
    useful = 6.0 * d * V * n_active / (ms_step * 1e-3) / 1e12

    # ---- the secondary workloads, timed after the headline in the same process (shorter runs) ----
    others = None
    if args.workload == "pg" and args.others and args.steps > 0:
        others = {}
        n_steps = max(3, args.steps // 2)

        def loss_entry(name, what, fn, n_contr):
            ms, kern_o, out_o = timed(torch, B, fn, n_steps, 2)
            na = int(out_o["counters"][0])
            fl = 2.0 * n_contr * d * V * na
            others[name] = {"workload": what, "steps": n_steps, "ms_per_step": ms, "active_tokens": na,
                            "tokens_per_s": na / (ms * 1e-3), "flops_per_token": f"{int(2 * n_contr)}dV",
                            "pct_mfma_peak": 100.0 * fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "kernels": kern_o}

        # the paper's own mismatch rule (Sec. 5.1: geometric rejection) on the headline microbatch
        prm1 = B.Params(dtype=dtype_id, temperature=spec.temperature, mismatch_mode=1)
        adv_flat = B.trloo_advantage(rewards, valid, 1.0, want_returns=False, want_group_n=False)[0].reshape(-1)
        rollout1 = rollout_logp if rollout_logp is not None else synth.perturb_logp(old_logp, spec.logp_noise, spec.outlier_frac, spec.seed + 1)

        def step_mode1():
            B.trloo_advantage(rewards, valid, 1.0, want_returns=False, want_group_n=False)
            return B.pg_loss_fwd_bwd(H, W, y, loss_mask, cu, adv_flat, seg_sample, old_logp, rollout1, prm1, ws, dW=dW, out=outbuf)
        loss_entry("geometric_rejection", f"configs[{args.config}], mismatch_mode 1 (Sec. 5.1's rejection rule): "
                   "trloo_advantage + pg_loss_fwd_bwd; tokens/s and % of peak count the tokens that stay active", step_mode1, 4.0)

        # the same with the W^T cache a trainer can keep while W is unchanged (further microbatches of one step)
        wt = B.alloc_w_transposed(d, V, dev)
        prm1c = B.Params(dtype=dtype_id, temperature=spec.temperature, mismatch_mode=1, w_transposed=wt)
        B.pg_loss_fwd_bwd(H, W, y, loss_mask, cu, adv_flat, seg_sample, old_logp, rollout1, prm1c, ws, dW=dW, out=outbuf)   # fills it
        prm1c.w_transposed_valid = 1

        def step_mode1_cached():
            B.trloo_advantage(rewards, valid, 1.0, want_returns=False, want_group_n=False)
            return B.pg_loss_fwd_bwd(H, W, y, loss_mask, cu, adv_flat, seg_sample, old_logp, rollout1, prm1c, ws, dW=dW, out=outbuf)
        loss_entry("geometric_rejection_wt_cached", "as geometric_rejection, with pg_params.w_transposed filled by an earlier "
                   "call on the same W (a microbatch after the first of an optimizer step)", step_mode1_cached, 4.0)
        del wt

        # loss + backward from the recompute stage's softmax states (the forward contraction is not repeated)
        states = B.pg_head_shard_fwd(H, W, y, loss_mask, 0, prm, ws)
        dH32 = torch.empty((T, d), dtype=torch.float32, device=dev)
        out_b = (outbuf[0], dH32, outbuf[2], outbuf[3], outbuf[4])

        def step_bwd():
            B.trloo_advantage(rewards, valid, 1.0, want_returns=False, want_group_n=False)
            return B.pg_loss_shard_bwd(H, W, y, loss_mask, cu, adv_flat, seg_sample, old_logp, rollout_logp, states, 0, prm,
                                       ws, dH_f32=True, dW=dW, out=out_b)
        loss_entry("backward_from_states", f"configs[{args.config}], trloo_advantage + pg_loss_shard_bwd on the whole head from the "
                   "softmax states of pg_head_shard_fwd (valid while the weights are those of the recompute)", step_bwd, 3.0)
        del states, dH32, out_b

        # RMS normalisation in front of the head: fused into the loss call against the three separate calls
        gamma = torch.ones(d, dtype=H.dtype, device=dev)
        ws_n = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD_NORMED, dev)
        Hn, dXn = torch.empty_like(H), torch.empty_like(H)

        def step_fused():
            B.trloo_advantage(rewards, valid, 1.0, want_returns=False, want_group_n=False)
            return B.pg_loss_fwd_bwd_normed(H, gamma, 1e-6, W, y, loss_mask, cu, adv_flat, seg_sample, old_logp, rollout_logp,
                                            prm, ws_n, dW=dW, out=outbuf)

        def step_separate():
            B.trloo_advantage(rewards, valid, 1.0, want_returns=False, want_group_n=False)
            B.pg_rmsnorm_fwd(H, gamma, 1e-6, want_rstd=False, out=Hn)
            o = B.pg_loss_fwd_bwd(Hn, W, y, loss_mask, cu, adv_flat, seg_sample, old_logp, rollout_logp, prm, ws, dW=dW, out=outbuf)
            B.pg_rmsnorm_bwd(H, gamma, o["dH"], 1e-6, out=dXn)
            return o
        loss_entry("with_rmsnorm_fused", f"configs[{args.config}] with the RMS normalisation of the hidden states in front of the head: "
                   "trloo_advantage + pg_loss_fwd_bwd_normed (normalisation and its backward inside the call)", step_fused, 4.0)
        loss_entry("with_rmsnorm_separate_calls", "the same as trloo_advantage + pg_rmsnorm_fwd + pg_loss_fwd_bwd + pg_rmsnorm_bwd",
                   step_separate, 4.0)
        del ws_n, Hn, dXn, gamma

    cpu = cpu_baseline(spec, args.cpu_rows) if args.cpu_rows > 0 and args.workload == "pg" else None
    aux = (aux_stage_times(B, torch, dev, rewards, valid, out, loss_mask, old_logp, rollout_logp, dW, H)
           if args.workload not in ("shard", "bwd") else None)

    line = {
        "metric": {"pg": "loss fwd+bwd tokens/sec at 14B shape (h5120,V151936); % bf16 MFMA peak",
                   "sft": "SFT cross-entropy fwd+bwd tokens/sec at 14B shape (h5120,V151936); % bf16 MFMA peak",
                   "shard": f"loss fwd+bwd tokens/sec of one of {args.vocab_shards} vocab shards of the head; % bf16 MFMA peak",
                   "bwd": "loss + backward tokens/sec at 14B shape from the recompute stage's softmax states "
                          "(forward contraction not repeated); % bf16 MFMA peak",
                   }[args.workload],
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_per_step_median": step_ms[len(step_ms) // 2] if step_ms else None,
        "ms_per_step_min": step_ms[0] if step_ms else None, "ms_per_step_accumulate_dW": acc_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype_id == 0 else "f32", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {spec.name}: d={d}, V={V}, {batch.P}x{batch.K}x{batch.Tmax} rollout batch, "
                               f"packed microbatch of {S} segments, {T} rows, {n_loss} loss tokens",
                   "loss_tokens": n_loss, "active_tokens": n_active, "packed_rows": T, "segments": S,
                   "mismatch_mode": args.mismatch_mode, "temperature": spec.temperature,
                   "dW": "fp32 overwrite",
                   "step": {"pg": "trloo_advantage + pg_loss_fwd_bwd", "sft": "pg_sft_fwd_bwd",
                            "shard": "trloo_advantage + pg_head_shard_fwd + pg_head_partials_merge + pg_loss_shard_bwd",
                            "bwd": "trloo_advantage + pg_loss_shard_bwd (states from pg_head_shard_fwd, outside the timed region)"
                            }[args.workload],
                   **({"vocab_shards": args.vocab_shards, "V_shard": V, "V": V_full} if args.workload == "shard" else {})},
        "packed_rows_per_s": T * args.steps / dt,          # value counts active (loss, not rejected) rows only
        "pct_mfma_peak_executed_8dV": 100.0 * executed / PEAK_BF16_TFLOPS,      # of 6dV for --workload bwd
        "executed_contractions_per_token": n_contractions,
        "pct_mfma_peak_useful_6dV": 100.0 * useful / PEAK_BF16_TFLOPS,
        "loss": loss, "counters": {n: int(c) for n, c in zip(B.COUNTER_NAMES, counters)},
        "kernels": kern, "roofline": roofline, "cpu_baseline": cpu, "aux_stages_us": aux,      # per call; the *_GBps entries are algorithmic bytes / time
    }
    if others is not None:
        # the forward-only recompute workload needs the memory of the step's buffers
        del H, W, y, ws, dW, outbuf, out
        torch.cuda.empty_cache()
        others["forward_only_128k"] = forward_only_workload(torch, B, synth, dev, 4, max(3, args.steps // 2), 2, args.scale_rows)
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
