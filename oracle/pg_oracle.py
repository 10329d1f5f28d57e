"""fp64 CPU oracle for the multi-turn policy-gradient head (TEST INFRASTRUCTURE).

This file is the yardstick the HIP library is measured against.  It is plain
numpy in float64, written from the paper's statement of the method, and shares
no code, table or helper with the GPU path.  Nothing outside tests/, the smoke
check and the benchmark's CPU-baseline leg may import it.

What follows the paper directly
  * turn returns            -- Sec. 4.2, Eq. (2)  (reward-to-go, discount gamma)
  * GRPO mean baseline      -- Sec. 4.2, Eq. (3)  (kept as a cross-check)
  * TRLOO advantages        -- Sec. 4.2, Eq. (5)  (leave-one-out over the valid
                               rollouts of one prompt at one turn)
  * mismatch rejection      -- Sec. 5.1 (geometric-mean ratio window and the
                               token-level veto)
  * gradient direction      -- App. A: grad of log pi(y|s) times the advantage;
                               for a softmax head d log pi(y) / d z = onehot - p.

Stages around the path (Sec. 3.3, 4.2, 5.1, 5.2 and App. ablations)
  * cold-start SFT loss     -- Sec. 3.3: token-mean cross-entropy of the same head
                               (the paper names the stage, the loss is the textbook one)
  * rewards                 -- Eq. (1) speedup reward with the cap of 3, Eq. (7) with the
                               profiling ratio PR = T_generated / T_total added
  * PRS                     -- Eq. (8): keep with probability clip((PR - tau) / s, 0, 1),
                               and the hard-threshold variant of the PRS ablation
  * monitors                -- Sec. 5.1: entropy, gradient norm and the perplexities of the
                               trainer's and the rollout engine's log-probs
  * final RMSNorm           -- the trainer's step in front of the head (the policies of Sec. 6.1
                               are Qwen3 models, whose last layer before the head is an RMSNorm);
                               the paper does not mention it, the definition is the textbook one

  * vocab-sharded head      -- the same head with W split by vocabulary rows (how a head is
                               spread over devices); the paper does not mention it.  Each
                               shard's per-row softmax state, the merge of two states, and a
                               shard's share of the gradients, all by direct definition

What the paper does not write down and is fixed here by definition (each is a
stated reading, "parity unpinned" beyond self-consistency): the PPO-style
clipped surrogate and its epsilon, token-mean normalisation, the truncated
importance weight of mode 2, the temperature, and A = 0 for groups of fewer
than two valid rollouts.  Everything else in this file is pinned by the tests
under tests/ that do not need a GPU (closed forms, brute force, a library
log-softmax, autograd cross-entropy, finite differences, exact enumeration).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


# --------------------------------------------------------------------------
# parameters (names follow the C header; values follow the paper where given)
# --------------------------------------------------------------------------
@dataclass
class Params:
    temperature: float = 1.0
    clip_eps_lo: float = 0.2
    clip_eps_hi: float = 0.2
    mismatch_mode: int = 0        # 0 none, 1 geometric rejection (Sec. 5.1), 2 token truncation
    geo_lo: float = 0.999         # Sec. 5.1: keep iff w in [0.999, 1.001]
    geo_hi: float = 1.001
    veto_ratio: float = 1e-4      # Sec. 5.1: reject the sample if any token ratio < 1e-4
    trunc_c: float = 2.0
    norm_override: float = 0.0


def _f32(x: float) -> float:
    """Thresholds cross the C boundary as float32; use the same value here."""
    return float(np.float32(x))


# --------------------------------------------------------------------------
# Sec. 4.2, Eq. (1): R = C + C * min(T_reference / T_kernel, 3)
# (the stage before the path; here so the paper's worked example can be replayed)
# --------------------------------------------------------------------------
def reward_eq1(correct, speedup, cap: float = 3.0) -> np.ndarray:
    C = np.asarray(correct, dtype=np.float64)
    return C + C * np.minimum(np.asarray(speedup, dtype=np.float64), cap)


# --------------------------------------------------------------------------
# Sec. 4.2, Eq. (2): G_{i,t} = sum_{t' >= t} gamma^(t'-t) R_{i,t'}
# --------------------------------------------------------------------------
def returns(rewards: np.ndarray, gamma: float = 1.0) -> np.ndarray:
    R = np.asarray(rewards, dtype=np.float64)
    P, K, Tm = R.shape
    g = float(np.float32(gamma))
    G = np.zeros_like(R)
    for p in range(P):
        for k in range(K):
            for t in range(Tm):
                acc = 0.0
                for tp in range(t, Tm):
                    acc += (g ** (tp - t)) * R[p, k, tp]
                G[p, k, t] = acc
    return G


# --------------------------------------------------------------------------
# Sec. 4.2, Eq. (3): A = G - mean over the valid rollouts of the turn group
# --------------------------------------------------------------------------
def grpo_advantage(rewards, valid, gamma: float = 1.0) -> np.ndarray:
    G = returns(rewards, gamma)
    valid = np.asarray(valid).astype(bool)
    P, K, Tm = G.shape
    A = np.zeros_like(G)
    for p in range(P):
        for t in range(Tm):
            members = [k for k in range(K) if valid[p, k, t]]
            if not members:
                continue
            mean = sum(G[p, j, t] for j in members) / len(members)
            for k in members:
                A[p, k, t] = G[p, k, t] - mean
    return A


# --------------------------------------------------------------------------
# Sec. 4.2, Eq. (5): A_{i,t} = G_{i,t} - 1/(N_t-1) * sum_{j in group, j != i} G_{j,t}
# Groups with fewer than two valid rollouts have no leave-one-out baseline:
# their advantages are 0 (a reading; the equation is stated for N_t > 1 only).
# --------------------------------------------------------------------------
def trloo_advantage(rewards, valid, gamma: float = 1.0):
    G = returns(rewards, gamma)
    valid = np.asarray(valid).astype(bool)
    P, K, Tm = G.shape
    A = np.zeros_like(G)
    N = np.zeros((P, Tm), dtype=np.int32)
    for p in range(P):
        for t in range(Tm):
            members = [k for k in range(K) if valid[p, k, t]]
            N[p, t] = len(members)
            if len(members) < 2:
                continue
            for i in members:
                others = 0.0
                for j in members:
                    if j != i:
                        others += G[p, j, t]
                A[p, i, t] = G[p, i, t] - others / (len(members) - 1)
    return G, A, N


# --------------------------------------------------------------------------
# LM head: z = H W^T / tau, log-softmax, sampled-token log-prob, entropy.
# pi_train(a_t | s_t) of Sec. 5.1 is softmax(z)[y_t]; entropy is the monitor
# the paper plots (nats, of the temperature-scaled distribution).
# --------------------------------------------------------------------------
def logits(H, W, tau: float = 1.0) -> np.ndarray:
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    return (H @ W.T) / _f32(tau)


def logprob_entropy_from_logits(z: np.ndarray, y: np.ndarray):
    M = z.max(axis=1, keepdims=True)
    e = np.exp(z - M)
    s = e.sum(axis=1, keepdims=True)
    lse = (M + np.log(s))[:, 0]
    p = e / s
    logp = z[np.arange(z.shape[0]), y] - lse
    ent = lse - (p * z).sum(axis=1)
    return logp, ent, lse, p


def lm_head_logprob(H, W, y, tau: float = 1.0, row_mask=None, block: int = 512):
    """Per-row log-prob of y, entropy and logsumexp; masked rows give 0."""
    H = np.asarray(H, dtype=np.float64)
    y = np.asarray(y, dtype=np.int64)
    T = H.shape[0]
    act = np.ones(T, bool) if row_mask is None else np.asarray(row_mask).astype(bool)
    logp = np.zeros(T)
    ent = np.zeros(T)
    lse = np.zeros(T)
    rows = np.nonzero(act)[0]
    for a in range(0, len(rows), block):
        r = rows[a:a + block]
        z = logits(H[r], W, tau)
        lp, en, ls, _ = logprob_entropy_from_logits(z, y[r])
        logp[r], ent[r], lse[r] = lp, en, ls
    return logp, ent, lse


def merge_softmax_partials(parts):
    """Combine partial (m, s, u) states of a row, s = sum e^(z-m), u = sum e^(z-m)(z-m).

    Not used by the oracle itself (which takes the whole row at once); it states
    the algebra a blocked implementation must obey and is unit-tested against the
    direct formula.  Returns (lse, entropy).
    """
    m, s, u = parts[0]
    for (m2, s2, u2) in parts[1:]:
        mm = max(m, m2)
        a1, a2 = np.exp(m - mm), np.exp(m2 - mm)
        u = a1 * (u + (m - mm) * s) + a2 * (u2 + (m2 - mm) * s2)
        s = a1 * s + a2 * s2
        m = mm
    lse = m + np.log(s)
    ent = np.log(s) - u / s
    return lse, ent


# --------------------------------------------------------------------------
# Vocab-sharded head.  A shard holds W[v0:v1]; its state of row t is
#   m = max_v z_v,  s = sum_v e^(z_v - m),  u = sum_v e^(z_v - m)(z_v - m)   over v0 <= v < v1,
#   z_y = z at y_t if the shard holds row y_t of W, else 0,
# with z = H_t W^T / tau.  Rows that are masked out carry the empty state (0, 0, 0, 0).
# --------------------------------------------------------------------------
def head_shard_partials(H, W_shard, y, v_offset: int, tau: float = 1.0, row_mask=None) -> np.ndarray:
    H = np.asarray(H, dtype=np.float64)
    y = np.asarray(y, dtype=np.int64)
    T = H.shape[0]
    Vs = np.asarray(W_shard).shape[0]
    act = np.ones(T, bool) if row_mask is None else np.asarray(row_mask).astype(bool)
    out = np.zeros((T, 4))
    for t in np.nonzero(act)[0]:
        z = logits(H[t:t + 1], W_shard, tau)[0]
        m = z.max()
        e = np.exp(z - m)
        yl = y[t] - v_offset
        out[t] = (m, e.sum(), (e * (z - m)).sum(), z[yl] if 0 <= yl < Vs else 0.0)
    return out


def merge_shard_partials(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """State of the union of two disjoint vocab ranges, row by row; the empty state is neutral."""
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    out = np.zeros_like(a)
    for t in range(a.shape[0]):
        (m1, s1, u1, z1), (m2, s2, u2, z2) = a[t], b[t]
        if s1 == 0.0:
            out[t] = (m2, s2, u2, z1 + z2)
        elif s2 == 0.0:
            out[t] = (m1, s1, u1, z1 + z2)
        else:
            m = max(m1, m2)
            a1, a2 = np.exp(m1 - m), np.exp(m2 - m)          # re-reference both sums to the common max
            out[t] = (m, a1 * s1 + a2 * s2,
                      a1 * (u1 + (m1 - m) * s1) + a2 * (u2 + (m2 - m) * s2), z1 + z2)
    return out


def finish_shard_partials(parts: np.ndarray):
    """(log-prob, entropy, logsumexp) per row from states merged over the whole vocabulary; 0 on empty rows."""
    parts = np.asarray(parts, np.float64)
    T = parts.shape[0]
    logp, ent, lse = np.zeros(T), np.zeros(T), np.zeros(T)
    live = parts[:, 1] > 0
    m, s_, u, zy = (parts[live, k] for k in range(4))
    lse[live] = m + np.log(s_)
    logp[live] = zy - lse[live]
    ent[live] = np.log(s_) - u / s_
    return logp, ent, lse


# --------------------------------------------------------------------------
# Sec. 5.1: mismatch correction from trainer-vs-rollout log-probs of the sampled
# tokens.  One segment = one training sample = one (prompt, rollout, turn); |T|
# is the number of its loss (response) tokens.  No gradient flows through it.
# --------------------------------------------------------------------------
def drop_filtered_segments(loss_mask, cu_seqlens, seg_keep):
    """Sec. 5.2: samples filtered out before training (PRS keep flag 0) take no part in the update --
    their rows leave the loss mask.  Returns (mask, number of dropped segments that had loss rows)."""
    mask = np.array(loss_mask).astype(bool)
    if seg_keep is None:
        return mask, 0
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    dropped = 0
    for s in range(len(cu) - 1):
        if not seg_keep[s]:
            dropped += int(mask[cu[s]:cu[s + 1]].any())
            mask[cu[s]:cu[s + 1]] = False
    return mask, dropped


def mismatch_weights(old_logp, rollout_logp, loss_mask, cu_seqlens, prm: Params):
    """Returns c[T] (weight per token), active[T], seg_keep[S], counters dict."""
    loss_mask = np.asarray(loss_mask).astype(bool)
    T = loss_mask.shape[0]
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    S = len(cu) - 1
    c = np.zeros(T)
    keep = np.ones(S, bool)
    n_geo = n_veto = n_trunc = 0
    if prm.mismatch_mode == 0:
        c[loss_mask] = 1.0
        return c, loss_mask.copy(), keep, dict(geo=0, veto=0, trunc=0)
    delta = np.asarray(old_logp, np.float64) - np.asarray(rollout_logp, np.float64)
    veto = _f32(prm.veto_ratio)
    for s in range(S):
        idx = np.arange(cu[s], cu[s + 1])
        idx = idx[loss_mask[idx]]
        if len(idx) == 0:
            continue
        d = delta[idx]
        vetoed = veto > 0.0 and np.exp(d.min()) < veto          # strictly below the threshold
        if vetoed:
            n_veto += 1
        if prm.mismatch_mode == 1:
            w = np.exp(d.sum() / len(idx))                       # geometric-mean ratio
            in_window = (_f32(prm.geo_lo) <= w) and (w <= _f32(prm.geo_hi))
            if not in_window:
                n_geo += 1
            keep[s] = in_window and not vetoed
            if keep[s]:
                c[idx] = 1.0
        else:                                                    # mode 2: truncated token weight
            keep[s] = not vetoed
            if keep[s]:
                ratio = np.exp(d)
                n_trunc += int((ratio > _f32(prm.trunc_c)).sum())
                c[idx] = np.minimum(ratio, _f32(prm.trunc_c))
    active = np.zeros(T, bool)
    for s in range(S):
        if keep[s]:
            sl = slice(cu[s], cu[s + 1])
            active[sl] = loss_mask[sl]
    return c, active, keep, dict(geo=n_geo, veto=n_veto, trunc=n_trunc)


# --------------------------------------------------------------------------
# Clipped surrogate on r = pi_theta / pi_old with advantage A (per token).
#   l = -min(r A, clip(r, 1-eps_lo, 1+eps_hi) A);   g = dl / dlogp.
# With one update per rollout batch r = 1 and g = -A: App. A's estimator.
# --------------------------------------------------------------------------
def surrogate(logp, old_logp, A, prm: Params):
    r = np.ones_like(logp) if old_logp is None else np.exp(logp - old_logp)
    lo, hi = 1.0 - _f32(prm.clip_eps_lo), 1.0 + _f32(prm.clip_eps_hi)
    loss = -np.minimum(r * A, np.clip(r, lo, hi) * A)
    flows = ((A >= 0) & (r <= hi)) | ((A < 0) & (r >= lo))
    g = np.where(flows, -A * r, 0.0)
    clip_hi = (A >= 0) & (r > hi)
    clip_lo = (A < 0) & (r < lo)
    return loss, g, r, clip_hi, clip_lo


def pg_loss_fwd_bwd(H, W, y, loss_mask, cu_seqlens, adv_seg, old_logp, rollout_logp,
                    prm: Params, dW_prev=None, block: int = 256, vocab_slice=None, seg_keep=None):
    """Loss, dH, dW, per-token log-prob/entropy and counters, all float64.

    adv_seg[s] is the advantage of segment s, broadcast to its loss tokens.
    vocab_slice = (v0, v1): one vocab shard's share of the gradients -- the softmax still runs
    over all of W, but only the columns v0 <= v < v1 of dS are contracted: dW has the v1 - v0
    rows of that range and dH is that range's term of the sum over v (dW_prev likewise).
    seg_keep[s] = 0 drops segment s before anything else (drop_filtered_segments).
    """
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    y = np.asarray(y, dtype=np.int64)
    T, d = H.shape
    V = W.shape[0]
    tau = _f32(prm.temperature)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    S = len(cu) - 1
    loss_mask, n_dropped = drop_filtered_segments(loss_mask, cu, seg_keep)
    old = None if old_logp is None else np.asarray(old_logp, np.float64)

    c, active, keep, mm = mismatch_weights(old, rollout_logp, loss_mask, cu, prm)
    n_active = int(active.sum())
    norm = _f32(prm.norm_override) if prm.norm_override > 0 else float(max(1, n_active))

    A_tok = np.zeros(T)
    for s in range(S):
        A_tok[cu[s]:cu[s + 1]] = float(adv_seg[s])

    logp = np.zeros(T)
    ent = np.zeros(T)
    dH = np.zeros((T, d))
    v0, v1 = (0, V) if vocab_slice is None else vocab_slice
    dW = np.zeros((v1 - v0, d)) if dW_prev is None else np.array(dW_prev, dtype=np.float64)
    total = 0.0
    n_hi = n_lo = 0
    rows = np.nonzero(active)[0]
    for a in range(0, len(rows), block):
        r_ = rows[a:a + block]
        z = logits(H[r_], W, tau)
        lp, en, _, p = logprob_entropy_from_logits(z, y[r_])
        logp[r_], ent[r_] = lp, en
        l, g, _, chi, clo = surrogate(lp, None if old is None else old[r_], A_tok[r_], prm)
        total += float((c[r_] * l).sum())
        n_hi += int(chi.sum())
        n_lo += int(clo.sum())
        coef = c[r_] * g / norm                       # d(loss)/d(logp_t)
        dS = -p * (coef / tau)[:, None]               # (coef/tau) * (onehot - p)
        dS[np.arange(len(r_)), y[r_]] += coef / tau
        dS = dS[:, v0:v1]
        dH[r_] = dS @ W[v0:v1]
        dW += dS.T @ H[r_]
    counters = np.array([n_active, n_hi, n_lo, mm["geo"], mm["veto"], mm["trunc"],
                         int(loss_mask.sum()), n_dropped], dtype=np.int64)
    return dict(loss=total / norm, dH=dH, dW=dW, logp=logp, entropy=ent,
                counters=counters, active=active, c=c, norm=norm)


def loss_value_only(H, W, y, loss_mask, cu_seqlens, adv_seg, old_logp, rollout_logp, prm: Params):
    """The scalar loss as a function of (H, W) with everything else held fixed."""
    return pg_loss_fwd_bwd(H, W, y, loss_mask, cu_seqlens, adv_seg, old_logp,
                           rollout_logp, prm)["loss"]


# --------------------------------------------------------------------------
# Row-sampled variants for sizes where the whole problem is too slow in fp64:
# every per-row quantity (log-prob, entropy, dH row) depends on that row alone
# once the token weights c, the advantages and the normaliser are known.
# --------------------------------------------------------------------------
def dH_rows(H_rows, W, y_rows, coef_rows, tau: float):
    z = logits(H_rows, W, tau)
    _, _, _, p = logprob_entropy_from_logits(z, np.asarray(y_rows, np.int64))
    k = np.asarray(coef_rows, np.float64) / _f32(tau)
    dS = -p * k[:, None]
    dS[np.arange(len(k)), np.asarray(y_rows, np.int64)] += k
    return dS @ np.asarray(W, np.float64)


# --------------------------------------------------------------------------
# Sec. 3.3 (cold-start SFT): token-mean cross-entropy of the LM head on the loss
# tokens, L = -(1/norm) sum_t m_t log softmax(z_t)[y_t], and its gradients
# dS = (softmax - onehot) / (norm tau), dH = dS W, dW = dS^T H.
# --------------------------------------------------------------------------
def sft_ce_fwd_bwd(H, W, y, loss_mask, tau: float = 1.0, norm_override: float = 0.0,
                   dW_prev=None, block: int = 256):
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    y = np.asarray(y, dtype=np.int64)
    T, d = H.shape
    V = W.shape[0]
    tau = _f32(tau)
    act = np.asarray(loss_mask).astype(bool)
    n = int(act.sum())
    norm = _f32(norm_override) if norm_override > 0 else float(max(1, n))
    logp = np.zeros(T)
    ent = np.zeros(T)
    dH = np.zeros((T, d))
    dW = np.zeros((V, d)) if dW_prev is None else np.array(dW_prev, dtype=np.float64)
    total = 0.0
    rows = np.nonzero(act)[0]
    for a in range(0, len(rows), block):
        r_ = rows[a:a + block]
        z = logits(H[r_], W, tau)
        lp, en, _, p = logprob_entropy_from_logits(z, y[r_])
        logp[r_], ent[r_] = lp, en
        total += float(-lp.sum())
        dS = p / (norm * tau)
        dS[np.arange(len(r_)), y[r_]] -= 1.0 / (norm * tau)
        dH[r_] = dS @ W
        dW += dS.T @ H[r_]
    return dict(loss=total / norm, dH=dH, dW=dW, logp=logp, entropy=ent, n=n, norm=norm)


# --------------------------------------------------------------------------
# Sec. 5.2, Eq. (6)-(7): profiling ratio PR = T_generated / T_total and the reward
#   R = C + C * min(T_reference / T_kernel, cap) + C * PR      (PR term optional)
# Times of incorrect kernels are irrelevant (C = 0 zeroes every term).
# --------------------------------------------------------------------------
def profiling_ratio(t_generated, t_total) -> np.ndarray:
    return np.asarray(t_generated, np.float64) / np.asarray(t_total, np.float64)


def turn_reward(correct, t_reference, t_kernel, t_generated=None, t_total=None, cap: float = 3.0):
    C = (np.asarray(correct) != 0).astype(np.float64)
    speedup = np.minimum(np.asarray(t_reference, np.float64) / np.asarray(t_kernel, np.float64), _f32(cap))
    R = np.where(C > 0, 1.0 + speedup, 0.0)
    pr = np.zeros_like(R)
    if t_generated is not None:
        pr = np.where(C > 0, profiling_ratio(t_generated, t_total), 0.0)
        R = R + pr
    return R, pr


# --------------------------------------------------------------------------
# Sec. 5.2, Eq. (8): PRS retention probability, and the Bernoulli draw.
# The draw uses one Philox4x32-10 block per sample (Salmon et al., SC'11):
# counter = (index, 0, 0, 0), key = (seed_lo, seed_hi); u = (x0 + 0.5) / 2^32;
# keep iff u < p.  The hard-threshold variant of the PRS ablation keeps iff PR >= tau.
# --------------------------------------------------------------------------
def prs_probability(pr, tau: float = 0.3, s: float = 0.1) -> np.ndarray:
    pr = np.asarray(pr, np.float64)
    return np.clip((pr - _f32(tau)) / _f32(s), 0.0, 1.0)


_PHILOX_M0, _PHILOX_M1 = 0xD2511F53, 0xCD9E8D57
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key):
    """One block of Philox-4x32 with 10 rounds; counter: 4 words, key: 2 words (Python ints)."""
    c0, c1, c2, c3 = (int(x) & 0xFFFFFFFF for x in counter)
    k0, k1 = (int(x) & 0xFFFFFFFF for x in key)
    for _ in range(10):
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & 0xFFFFFFFF
        hi1, lo1 = p1 >> 32, p1 & 0xFFFFFFFF
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & 0xFFFFFFFF, lo1, (hi0 ^ c3 ^ k1) & 0xFFFFFFFF, lo0
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return c0, c1, c2, c3


def prs_uniform(index: int, seed: int) -> float:
    x0 = philox4x32_10((index & 0xFFFFFFFF, (index >> 32) & 0xFFFFFFFF, 0, 0),
                       (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))[0]
    return (x0 + 0.5) / 4294967296.0


def prs_retain(pr, valid, seed: int, tau: float = 0.3, s: float = 0.1, hard: bool = False):
    """keep[i] (uint8) and p[i]; invalid samples (turn never generated) are not kept."""
    pr = np.asarray(pr, np.float64).reshape(-1)
    valid = np.asarray(valid).reshape(-1).astype(bool)
    p = prs_probability(pr, tau, s)
    keep = np.zeros(pr.shape[0], np.uint8)
    for i in range(pr.shape[0]):
        if not valid[i]:
            continue
        if hard:
            keep[i] = 1 if pr[i] >= _f32(tau) else 0
        else:
            keep[i] = 1 if prs_uniform(i, seed) < p[i] else 0
    return keep, p


# --------------------------------------------------------------------------
# Sec. 5.1 monitors over the loss tokens of a microbatch: mean entropy, perplexity
# exp(-mean logp) of the trainer's and of the rollout engine's log-probs, and the
# Euclidean norms of the head's gradients.
# --------------------------------------------------------------------------
def monitors(logp_train, logp_rollout, entropy, loss_mask, dH=None, dW=None):
    m = np.asarray(loss_mask).astype(bool)
    n = int(m.sum())
    den = float(max(1, n))
    out = dict(n=n)
    out["entropy_mean"] = float(np.asarray(entropy, np.float64)[m].sum() / den) if entropy is not None else 0.0
    out["ppl_train"] = float(np.exp(-np.asarray(logp_train, np.float64)[m].sum() / den))
    out["ppl_rollout"] = (float(np.exp(-np.asarray(logp_rollout, np.float64)[m].sum() / den))
                          if logp_rollout is not None else 0.0)
    out["dH_norm"] = float(np.sqrt((np.asarray(dH, np.float64) ** 2).sum())) if dH is not None else 0.0
    out["dW_norm"] = float(np.sqrt((np.asarray(dW, np.float64) ** 2).sum())) if dW is not None else 0.0
    return out


# --------------------------------------------------------------------------
# The step in front of the head in the Qwen3 policies of Sec. 6.1: root-mean-square
# normalisation  h = x * rstd * gamma,  rstd = 1 / sqrt(mean_j x_j^2 + eps),  per row.
# Backward, with g = dL/dh:  xhat = x * rstd,
#   dx = rstd * (gamma g - xhat * mean_j(gamma_j g_j xhat_j)),   dgamma = sum_rows g * xhat.
# --------------------------------------------------------------------------
def rmsnorm_fwd(X, gamma, eps: float):
    X = np.asarray(X, np.float64)
    g = np.asarray(gamma, np.float64)
    rstd = 1.0 / np.sqrt((X * X).mean(axis=1) + _f32(eps))
    return X * rstd[:, None] * g[None, :], rstd


def rmsnorm_bwd(X, gamma, eps: float, dH):
    X = np.asarray(X, np.float64)
    g = np.asarray(gamma, np.float64)
    dH = np.asarray(dH, np.float64)
    d = X.shape[1]
    rstd = 1.0 / np.sqrt((X * X).mean(axis=1) + _f32(eps))
    xhat = X * rstd[:, None]
    gg = dH * g[None, :]
    dX = rstd[:, None] * (gg - xhat * ((gg * xhat).sum(axis=1) / d)[:, None])
    dgamma = (dH * xhat).sum(axis=0)
    return dX, dgamma
