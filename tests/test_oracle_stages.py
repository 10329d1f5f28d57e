"""Pins for the oracle's stages around the path: SFT cross-entropy (Sec. 3.3), rewards with the
profiling ratio (Sec. 4.2 Eq. 1, Sec. 5.2 Eq. 6-7), PRS (Eq. 8) and the monitors (Sec. 5.1).  CPU only."""
import os

import numpy as np
import pytest
import torch

from oracle import pg_oracle as O


def _rows(golden_dir, name):
    return [l.split() for l in open(os.path.join(golden_dir, name)) if l.strip() and not l.startswith("#")]


# ---------------------------------------------------------------- SFT cross-entropy
def _sft_problem(seed=0, T=37, d=24, V=53):
    rng = np.random.default_rng(seed)
    H = rng.normal(size=(T, d))
    W = rng.normal(size=(V, d)) * 0.3
    y = rng.integers(0, V, size=T)
    mask = (rng.random(T) < 0.7).astype(np.uint8)
    return H, W, y, mask


@pytest.mark.parametrize("tau", [1.0, 0.7])
def test_sft_matches_library_cross_entropy_autograd(tau):
    H, W, y, mask = _sft_problem()
    out = O.sft_ce_fwd_bwd(H, W, y, mask, tau)
    Ht = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    z = (Ht @ Wt.T) / float(np.float32(tau))
    m = torch.tensor(mask.astype(bool))
    loss = torch.nn.functional.cross_entropy(z[m], torch.tensor(y)[m], reduction="mean")
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-12
    np.testing.assert_allclose(out["dH"], Ht.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(out["dW"], Wt.grad.numpy(), atol=1e-13)
    assert np.all(out["dH"][mask == 0] == 0)
    assert np.all(out["logp"][mask == 0] == 0)


def test_sft_zero_weights_is_log_vocab():
    H, W, y, mask = _sft_problem(1)
    out = O.sft_ce_fwd_bwd(H, np.zeros_like(W), y, mask)
    assert abs(out["loss"] - np.log(W.shape[0])) < 1e-12
    np.testing.assert_allclose(out["entropy"][mask != 0], np.log(W.shape[0]), atol=1e-12)


def test_sft_norm_override_and_accumulate():
    H, W, y, mask = _sft_problem(2)
    a = O.sft_ce_fwd_bwd(H, W, y, mask)
    n = int(mask.sum())
    b = O.sft_ce_fwd_bwd(H, W, y, mask, norm_override=2.0 * n)
    np.testing.assert_allclose(b["dW"], a["dW"] / 2, atol=1e-14)
    assert abs(b["loss"] - a["loss"] / 2) < 1e-14
    prev = np.full_like(W, 0.25)
    c = O.sft_ce_fwd_bwd(H, W, y, mask, dW_prev=prev)
    np.testing.assert_allclose(c["dW"], a["dW"] + 0.25, atol=1e-14)


def test_sft_is_policy_gradient_with_unit_advantage():
    """App. A: with A = 1 on every token and r = 1 the estimator's gradient is that of -mean log pi."""
    H, W, y, mask = _sft_problem(3)
    T = H.shape[0]
    cu = np.array([0, T // 2, T], dtype=np.int32)
    pg = O.pg_loss_fwd_bwd(H, W, y, mask, cu, np.ones(2), None, None, O.Params())
    sft = O.sft_ce_fwd_bwd(H, W, y, mask)
    np.testing.assert_allclose(pg["dW"], sft["dW"], atol=1e-14)
    np.testing.assert_allclose(pg["dH"], sft["dH"], atol=1e-14)


def test_sft_all_masked():
    H, W, y, mask = _sft_problem(4)
    out = O.sft_ce_fwd_bwd(H, W, y, np.zeros_like(mask))
    assert out["loss"] == 0.0 and not out["dW"].any() and not out["dH"].any()


# ---------------------------------------------------------------- rewards with the profiling ratio
def test_turn_reward_reduces_to_eq1(golden_dir):
    rows = np.array(_rows(golden_dir, "layernorm_case_rewards.txt"), dtype=np.float64)
    speed, R_exp = rows[:, 1], rows[:, 2]
    # speedup = T_reference / T_kernel: take T_kernel = 1
    R, pr = O.turn_reward(np.ones(3), speed, np.ones(3))
    np.testing.assert_allclose(R, R_exp, atol=1e-12)
    assert not pr.any()


def test_turn_reward_cap_incorrect_and_pr(golden_dir):
    consts = {r[0]: float(r[1]) for r in _rows(golden_dir, "paper_constants.txt")}
    cap = consts["speedup_cap"]
    correct = np.array([1, 1, 0, 1])
    t_ref = np.array([10.0, 9.0, 5.0, 2.0])
    t_ker = np.array([1.0, 3.0, 1.0, 4.0])           # speedups 10 (capped), 3, -, 0.5
    t_gen = np.array([0.5, 0.25, 0.9, 1.0])
    t_tot = np.array([1.0, 1.0, 1.0, 1.0])
    R, pr = O.turn_reward(correct, t_ref, t_ker, t_gen, t_tot, cap)
    np.testing.assert_allclose(R, [1 + 3 + 0.5, 1 + 3 + 0.25, 0.0, 1 + 0.5 + 1.0], atol=1e-12)
    np.testing.assert_allclose(pr, [0.5, 0.25, 0.0, 1.0])
    # PR lies in [0, 1], so the capped speedup term (<= 3) dominates it (Sec. 5.2)
    R0, _ = O.turn_reward(correct, t_ref, t_ker, None, None, cap)
    assert np.all(R - R0 >= 0) and np.all(R - R0 <= 1)


# ---------------------------------------------------------------- PRS
def test_prs_probability_paper_values(golden_dir):
    consts = {r[0]: float(r[1]) for r in _rows(golden_dir, "paper_constants.txt")}
    tau, s = consts["prs_tau"], consts["prs_s"]
    for name, pr, p in _rows(golden_dir, "profiling_case.txt"):
        assert abs(O.prs_probability(float(pr), tau, s) - float(p)) < 1e-12
    # the soft band [0.3, 0.4): linear from 0 to 1
    np.testing.assert_allclose(O.prs_probability([0.3, 0.325, 0.35, 0.4, 0.41], tau, s), [0, 0.25, 0.5, 1, 1], atol=1e-6)


def test_philox_known_answers(golden_dir):
    for r in _rows(golden_dir, "philox4x32_10_kat.txt"):
        w = [int(x, 16) for x in r]
        assert list(O.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def test_prs_retain_extremes_and_hard_variant():
    # PR crosses the C boundary as float32, and so do tau and s: use those values here too
    pr = np.array([0.0, 0.29, 0.3, 0.35, 0.39999, 0.4, 0.9, 0.9], dtype=np.float32)
    valid = np.array([1, 1, 1, 1, 1, 1, 1, 0])
    keep, p = O.prs_retain(pr, valid, seed=1234)
    assert keep[0] == 0 and keep[1] == 0 and keep[2] == 0      # p = 0 is never kept
    assert keep[5] == 1 and keep[6] == 1                       # p = 1 is always kept
    assert keep[7] == 0                                        # never generated: not kept
    hard, _ = O.prs_retain(pr, valid, seed=1234, hard=True)
    np.testing.assert_array_equal(hard, [0, 0, 1, 1, 1, 1, 1, 0])


def test_prs_retain_rate_and_determinism():
    n = 20000
    pr = np.full(n, 0.35)                                       # p = 0.5
    keep, p = O.prs_retain(pr, np.ones(n), seed=7)
    assert abs(p[0] - 0.5) < 1e-6
    assert abs(keep.mean() - 0.5) < 0.015                       # 4 sigma of a fair coin over 20000
    keep2, _ = O.prs_retain(pr, np.ones(n), seed=7)
    np.testing.assert_array_equal(keep, keep2)
    keep3, _ = O.prs_retain(pr, np.ones(n), seed=8)
    assert (keep != keep3).mean() > 0.4                         # another seed, another draw
    # monotone coupling: the same uniform decides every threshold
    keep_hi, _ = O.prs_retain(np.full(n, 0.38), np.ones(n), seed=7)
    assert np.all(keep_hi >= keep)


# ---------------------------------------------------------------- monitors
def test_monitors_closed_forms():
    V, T = 1000, 64
    rng = np.random.default_rng(0)
    mask = (rng.random(T) < 0.6).astype(np.uint8)
    logp = np.full(T, -np.log(V))
    ent = np.full(T, np.log(V))
    dH = rng.normal(size=(T, 8))
    dW = rng.normal(size=(V, 8))
    m = O.monitors(logp, logp + np.log(2.0), ent, mask, dH, dW)
    assert abs(m["ppl_train"] - V) < 1e-9                       # uniform policy: perplexity = V
    assert abs(m["ppl_rollout"] - V / 2) < 1e-9
    assert abs(m["entropy_mean"] - np.log(V)) < 1e-12
    assert abs(m["dH_norm"] - np.linalg.norm(dH)) < 1e-12
    assert abs(m["dW_norm"] - np.linalg.norm(dW)) < 1e-12
    assert m["n"] == int(mask.sum())
    # masked tokens do not count
    logp2 = logp.copy(); logp2[mask == 0] = -50.0
    assert abs(O.monitors(logp2, None, None, mask)["ppl_train"] - V) < 1e-9


# ---------------------------------------------------------------- RMSNorm in front of the head
def test_rmsnorm_against_library_autograd():
    rng = np.random.default_rng(0)
    T, d, eps = 13, 48, 1e-6
    X = rng.normal(size=(T, d)) * rng.uniform(0.1, 5.0, size=(T, 1))
    gamma = rng.normal(1.0, 0.2, size=d)
    G = rng.normal(size=(T, d))
    Xt = torch.tensor(X, requires_grad=True)
    gt = torch.tensor(gamma, requires_grad=True)
    h = torch.nn.functional.rms_norm(Xt, (d,), gt, eps=float(np.float32(eps)))
    (h * torch.tensor(G)).sum().backward()
    H, rstd = O.rmsnorm_fwd(X, gamma, eps)
    dX, dg = O.rmsnorm_bwd(X, gamma, eps, G)
    np.testing.assert_allclose(H, h.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dX, Xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), atol=1e-12)


def test_rmsnorm_invariants():
    rng = np.random.default_rng(1)
    T, d = 7, 64
    X = rng.normal(size=(T, d))
    gamma = rng.normal(1.0, 0.3, size=d)
    G = rng.normal(size=(T, d))
    H, rstd = O.rmsnorm_fwd(X, gamma, 0.0)
    H2, _ = O.rmsnorm_fwd(3.7 * X, gamma, 0.0)
    np.testing.assert_allclose(H, H2, atol=1e-12)                       # scale invariance at eps = 0
    np.testing.assert_allclose(((H / gamma) ** 2).mean(axis=1), 1.0, atol=1e-12)   # unit RMS before the gain
    dX, dg = O.rmsnorm_bwd(X, gamma, 0.0, G)
    np.testing.assert_allclose((dX * X).sum(axis=1), 0.0, atol=1e-12)   # hence the gradient is orthogonal to x
    Xu = X / np.sqrt((X * X).mean(axis=1, keepdims=True))
    Hu, _ = O.rmsnorm_fwd(Xu, np.ones(d), 0.0)
    np.testing.assert_allclose(Hu, Xu, atol=1e-12)                      # unit-RMS rows, unit gain: identity
    # central finite difference of <G, h(x)> in one coordinate
    e = np.zeros_like(X); e[2, 5] = 1e-6
    f = lambda Z: (O.rmsnorm_fwd(Z, gamma, 1e-6)[0] * G).sum()
    fd = (f(X + e) - f(X - e)) / 2e-6
    assert abs(fd - O.rmsnorm_bwd(X, gamma, 1e-6, G)[0][2, 5]) < 1e-6


# ---------------------------------------------------------------- samples filtered out before training (Sec. 5.2)
def test_dropped_samples_equal_a_microbatch_packed_without_them():
    """Dropping a sample by its keep flag must give what a packer gives that never packed it: same loss,
    same dW, same dH rows for the rows that remain, and the normaliser counts kept loss rows only."""
    rng = np.random.default_rng(11)
    T, d, V = 60, 12, 31
    H = rng.normal(size=(T, d))
    W = rng.normal(size=(V, d)) * 0.4
    y = rng.integers(0, V, size=T)
    cu = np.array([0, 9, 22, 22, 40, 51, 60])               # one empty segment
    mask = (rng.random(T) < 0.7).astype(np.uint8)
    mask[40:51] = 0                                          # a segment without loss rows
    adv = rng.normal(size=6)
    lp, _, _ = O.lm_head_logprob(H, W, y, 1.0)
    old = lp + rng.normal(size=T) * 0.1
    roll = old + rng.normal(size=T) * 0.05
    keep = np.array([1, 0, 1, 1, 0, 0], np.uint8)            # drops segments 1, 4 (no loss rows) and 5
    prm = O.Params(mismatch_mode=2)
    a = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, old, roll, prm, seg_keep=keep)
    rows = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in range(6) if keep[s]])
    lens = [cu[s + 1] - cu[s] for s in range(6) if keep[s]]
    cu2 = np.concatenate([[0], np.cumsum(lens)])
    b = O.pg_loss_fwd_bwd(H[rows], W, y[rows], mask[rows], cu2, adv[keep.astype(bool)], old[rows], roll[rows], prm)
    assert abs(a["loss"] - b["loss"]) < 1e-15 and a["norm"] == b["norm"] == mask[rows].sum()
    np.testing.assert_allclose(a["dW"], b["dW"], atol=1e-15)
    np.testing.assert_allclose(a["dH"][rows], b["dH"], atol=1e-15)
    gone = np.setdiff1d(np.arange(T), rows)
    assert not a["dH"][gone].any() and not a["logp"][gone].any()
    assert a["counters"][7] == 2 and b["counters"][7] == 0       # segment 4 had no loss rows: not counted
    assert np.array_equal(a["counters"][:7], b["counters"][:7])
    # keep-all flags change nothing
    c = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, old, roll, prm, seg_keep=np.ones(6, np.uint8))
    e = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, old, roll, prm)
    assert c["loss"] == e["loss"] and np.array_equal(c["dW"], e["dW"])


def test_dropped_sample_is_not_examined_by_mismatch_rejection():
    """A dropped sample with a vetoed token raises neither the veto nor the window counter."""
    T = 20
    H = np.eye(T, 8)
    W = np.ones((5, 8)) * 0.1
    y = np.zeros(T, np.int64)
    cu = np.array([0, 10, 20])
    mask = np.ones(T, np.uint8)
    old = np.full(T, -1.0)
    roll = old.copy()
    roll[3] = old[3] + 12.0                                  # ratio e^-12 < 1e-4 in segment 0
    prm = O.Params(mismatch_mode=1)
    kept = O.pg_loss_fwd_bwd(H, W, y, mask, cu, [1.0, 1.0], old, roll, prm)
    drop = O.pg_loss_fwd_bwd(H, W, y, mask, cu, [1.0, 1.0], old, roll, prm, seg_keep=[0, 1])
    assert kept["counters"][4] == 1 and kept["counters"][3] == 1 and kept["counters"][6] == 20
    assert drop["counters"][4] == 0 and drop["counters"][3] == 0 and drop["counters"][7] == 1
    assert drop["counters"][6] == 10 and drop["counters"][0] == 10
