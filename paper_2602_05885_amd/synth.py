"""Seeded synthetic workloads shaped like the paper's RL training batches.

This module only *draws inputs* (hidden states, head weights, token ids, batch
structure, rewards, log-prob noise).  It contains none of the method's
arithmetic and is the one piece shared by the tests of the CPU oracle and of
the HIP library: both sides receive exactly the same bits.

The real workload (Sec. 6.1: Qwen3-8B/14B policies, 16 prompts x 16 rollouts,
up to 3 turns, at most 8192 generated tokens per turn, every turn a training
sample) needs datasets and trained weights that are not available; only the
shapes, length mix and value distributions are reproduced here.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass
class WorkloadSpec:
    name: str
    d: int
    V: int
    P: int                       # prompts
    K: int                       # rollouts per prompt
    Tmax: int                    # turns
    len_lo: int                  # response length range (inclusive)
    len_hi: int
    ctx_frac: float              # masked context rows per response row
    pack_rows: int = 0           # stop packing at this many rows (0 = no limit)
    pack_loss_rows: int = 0      # ... or at this many loss rows
    dtype: str = "bf16"          # "bf16" or "f32"
    stop_prob: float = 0.15      # a rollout ends after a turn with this probability
    reward: str = "eq1"          # "eq1": C + C*min(lognormal,3); "binary": {0,1}
    logp_noise: float = 0.05     # rollout log-prob = trainer log-prob + N(0, noise)
    outlier_frac: float = 0.0    # fraction of tokens with an extra +-3
    temperature: float = 1.0
    unit_rms: bool = True
    seed: int = 0


# The five configurations of the benchmark definition (index = position in its list).
SPECS = {
    0: WorkloadSpec("tiny-f32", d=64, V=1000, P=4, K=4, Tmax=2, len_lo=32, len_hi=32,
                    ctx_frac=0.0, dtype="f32", stop_prob=0.0, reward="binary",
                    unit_rms=False, seed=58851),
    1: WorkloadSpec("qwen3-8b-head-16k", d=4096, V=151936, P=8, K=8, Tmax=3, len_lo=256,
                    len_hi=1024, ctx_frac=1.0 / 3.0, pack_rows=16384, seed=58852),
    2: WorkloadSpec("qwen3-14b-head-32k", d=5120, V=151936, P=16, K=8, Tmax=3, len_lo=256,
                    len_hi=1024, ctx_frac=1.0 / 3.0, pack_loss_rows=32768, logp_noise=0.1,
                    outlier_frac=0.01, seed=58853),
    3: WorkloadSpec("qwen3-14b-long-64k", d=5120, V=151936, P=4, K=16, Tmax=4, len_lo=1024,
                    len_hi=8192, ctx_frac=2.0 / 3.0, pack_rows=65536, seed=58854),
    4: WorkloadSpec("qwen3-14b-fwd-128k", d=5120, V=151936, P=32, K=16, Tmax=2, len_lo=128,
                    len_hi=128, ctx_frac=0.0, stop_prob=0.0, temperature=0.7, seed=58855),
}


@dataclass
class Batch:
    """Rollout-batch structure: rewards/validity for all samples, and one packed microbatch."""
    P: int
    K: int
    Tmax: int
    rewards: np.ndarray          # [P,K,Tmax] float32, 0 where the turn was never generated
    valid: np.ndarray            # [P,K,Tmax] uint8
    cu_seqlens: np.ndarray       # [S+1] int32, packed-row offsets of the microbatch's segments
    seg_sample: np.ndarray       # [S] int32, flat (p*K+k)*Tmax+t index of each segment
    loss_mask: np.ndarray        # [T] uint8, 1 on response rows
    T: int = 0
    S: int = 0


def _np_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=seed))


def make_batch(spec: WorkloadSpec, scale_rows: float = 1.0) -> Batch:
    """Draw validity, rewards, segment lengths; pack the first samples in (p,k,t) order."""
    rng = _np_rng(spec.seed)
    P, K, Tm = spec.P, spec.K, spec.Tmax
    valid = np.zeros((P, K, Tm), np.uint8)
    stop = rng.random((P, K, Tm)) < spec.stop_prob
    for p in range(P):
        for k in range(K):
            for t in range(Tm):
                valid[p, k, t] = 1
                if stop[p, k, t]:
                    break
    correct = (rng.random((P, K, Tm)) < 0.5)
    if spec.reward == "binary":
        rewards = correct.astype(np.float32)
    else:
        speed = np.minimum(rng.lognormal(0.0, 0.5, (P, K, Tm)), 3.0)
        rewards = np.where(correct, 1.0 + speed, 0.0).astype(np.float32)
    rewards = rewards * valid
    resp = rng.integers(spec.len_lo, spec.len_hi + 1, (P, K, Tm))

    pack_rows = int(spec.pack_rows * scale_rows)
    pack_loss = int(spec.pack_loss_rows * scale_rows)
    cu = [0]
    seg = []
    mask = []
    loss_rows = 0
    done = False
    for p in range(P):
        for k in range(K):
            for t in range(Tm):
                if not valid[p, k, t] or done:
                    continue
                n_resp = int(resp[p, k, t])
                n_ctx = int(round(n_resp * spec.ctx_frac))
                if pack_loss and loss_rows + n_resp >= pack_loss:
                    n_resp = pack_loss - loss_rows
                    done = True
                if pack_rows and cu[-1] + n_ctx + n_resp > pack_rows:
                    done = True
                    continue
                if n_resp <= 0:
                    continue
                cu.append(cu[-1] + n_ctx + n_resp)
                seg.append((p * K + k) * Tm + t)
                mask.append(np.concatenate([np.zeros(n_ctx, np.uint8), np.ones(n_resp, np.uint8)]))
                loss_rows += n_resp
    loss_mask = np.concatenate(mask) if mask else np.zeros(0, np.uint8)
    return Batch(P, K, Tm, rewards, valid, np.asarray(cu, np.int32), np.asarray(seg, np.int32),
                 loss_mask, T=int(cu[-1]), S=len(seg))


def make_head(T: int, d: int, V: int, dtype: str, seed: int, device="cpu", unit_rms=True,
              w_std: float = 0.02):
    """H [T,d], W [V,d], y [T]: hidden states, head weight, sampled token ids."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    H = torch.empty((T, d), dtype=tdt, device=dev)
    step = max(1, (1 << 26) // max(d, 1))
    for a in range(0, T, step):
        h = torch.randn((min(step, T - a), d), generator=g, device=dev, dtype=torch.float32)
        if unit_rms:
            h = h * torch.rsqrt((h * h).mean(dim=1, keepdim=True))
        H[a:a + h.shape[0]] = h.to(tdt)
    W = torch.empty((V, d), dtype=tdt, device=dev)
    for a in range(0, V, step):
        w = torch.randn((min(step, V - a), d), generator=g, device=dev, dtype=torch.float32)
        W[a:a + w.shape[0]] = (w * w_std).to(tdt)
    y = torch.randint(0, V, (T,), generator=g, device=dev, dtype=torch.int32)
    return H, W, y


def perturb_logp(base: torch.Tensor, noise: float, outlier_frac: float, seed: int) -> torch.Tensor:
    """base + N(0, noise), plus +-3 on a random `outlier_frac` of the entries (float32)."""
    g = torch.Generator(device=base.device)
    g.manual_seed(seed)
    out = base.float() + noise * torch.randn(base.shape, generator=g, device=base.device)
    if outlier_frac > 0:
        u = torch.rand(base.shape, generator=g, device=base.device)
        sign = torch.where(torch.rand(base.shape, generator=g, device=base.device) < 0.5, -3.0, 3.0)
        out = out + torch.where(u < outlier_frac, sign, torch.zeros_like(sign))
    return out.float()


def small_spec(name="small", d=128, V=2500, P=3, K=4, Tmax=3, len_lo=20, len_hi=90, ctx_frac=0.4,
               dtype="bf16", seed=1234, **kw) -> WorkloadSpec:
    """A ragged miniature of the packed multi-turn batch for parity tests."""
    return WorkloadSpec(name, d=d, V=V, P=P, K=K, Tmax=Tmax, len_lo=len_lo, len_hi=len_hi,
                        ctx_frac=ctx_frac, dtype=dtype, seed=seed, **kw)
