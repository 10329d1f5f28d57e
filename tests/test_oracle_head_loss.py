"""Pins for the oracle's LM head, mismatch rule, surrogate and gradients.  CPU only."""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp as scipy_lse

from oracle import pg_oracle as O


# ----------------------------------------------------------------------------- LM head
def test_logsumexp_brute_force_and_library():
    rng = np.random.default_rng(0)
    H = rng.normal(size=(6, 5))
    W = rng.normal(size=(11, 5))
    y = rng.integers(0, 11, 6)
    for tau in (1.0, 0.7, 2.0):
        logp, ent, lse = O.lm_head_logprob(H, W, y, tau)
        t32 = float(np.float32(tau))
        for t in range(6):
            z = [sum(H[t, k] * W[v, k] for k in range(5)) / t32 for v in range(11)]
            brute = math.log(sum(math.exp(v) for v in z))
            assert abs(lse[t] - brute) < 1e-12
            assert abs(logp[t] - (z[y[t]] - brute)) < 1e-12
            p = [math.exp(v - brute) for v in z]
            assert abs(ent[t] + sum(pi * math.log(pi) for pi in p)) < 1e-12
        z = (H @ W.T) / t32
        np.testing.assert_allclose(lse, scipy_lse(z, axis=1), atol=1e-12)
        ref = torch.log_softmax(torch.from_numpy(z), dim=1).numpy()
        np.testing.assert_allclose(logp, ref[np.arange(6), y], atol=1e-12)


def test_head_invariants():
    rng = np.random.default_rng(1)
    H = rng.normal(size=(9, 16))
    W = rng.normal(size=(40, 16)) * 0.3
    y = rng.integers(0, 40, 9)
    logp, ent, lse = O.lm_head_logprob(H, W, y, 1.0)
    assert np.all(ent >= 0) and np.all(ent <= math.log(40) + 1e-12)
    # probabilities of a row sum to one
    for t in range(9):
        allp = [O.lm_head_logprob(H[t:t + 1], W, np.array([v]), 1.0)[0][0] for v in range(40)]
        assert abs(np.exp(allp).sum() - 1.0) < 1e-12
    # temperature is a rescaling of the hidden state (0.5 is exact in float32)
    a = O.lm_head_logprob(H, W, y, 0.5)
    b = O.lm_head_logprob(H / 0.5, W, y, 1.0)
    for u, v in zip(a, b):
        np.testing.assert_allclose(u, v, atol=1e-12)
    # zero weights: uniform distribution
    lp0, en0, ls0 = O.lm_head_logprob(H, np.zeros_like(W), y, 1.0)
    np.testing.assert_allclose(lp0, -math.log(40), atol=1e-14)
    np.testing.assert_allclose(en0, math.log(40), atol=1e-14)
    # masked rows are zero
    m = np.array([1, 0, 1, 1, 0, 1, 1, 1, 0], np.uint8)
    lpm, enm, lsm = O.lm_head_logprob(H, W, y, 1.0, row_mask=m)
    assert np.all(lpm[m == 0] == 0) and np.all(enm[m == 0] == 0) and np.all(lsm[m == 0] == 0)
    np.testing.assert_allclose(lpm[m == 1], logp[m == 1], atol=1e-14)


def test_uniform_entropy_at_qwen_vocab():
    # ln V at V = 151936
    lp, en, _ = O.lm_head_logprob(np.ones((1, 4)), np.zeros((151936, 4)), np.array([7]), 1.0)
    assert abs(en[0] - 11.93121) < 1e-5 and abs(lp[0] + 11.93121) < 1e-5


def test_partial_merge_matches_direct():
    rng = np.random.default_rng(2)
    z = rng.normal(size=200) * 4
    p = np.exp(z - scipy_lse(z))
    lse_ref, ent_ref = scipy_lse(z), -(p * np.log(p)).sum()
    for trial in range(5):
        cuts = np.sort(rng.choice(np.arange(1, 200), size=7, replace=False))
        chunks = np.split(z, cuts)
        parts = []
        for ch in chunks:
            m = ch.max()
            e = np.exp(ch - m)
            parts.append((m, e.sum(), (e * (ch - m)).sum()))
        order = rng.permutation(len(parts))
        lse, ent = O.merge_softmax_partials([parts[i] for i in order])
        assert abs(lse - lse_ref) < 1e-12 and abs(ent - ent_ref) < 1e-12


# ----------------------------------------------------------------------------- mismatch rule
def _segs(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


def test_mrs_identity_and_paper_window():
    cu = _segs([5, 4, 6])
    mask = np.ones(15, np.uint8)
    old = np.linspace(-3, -1, 15).astype(np.float32)
    prm = O.Params(mismatch_mode=1)
    c, act, keep, cnt = O.mismatch_weights(old, old.copy(), mask, cu, prm)
    assert keep.all() and np.all(c == 1) and cnt == dict(geo=0, veto=0, trunc=0)
    # constant log-ratio: w = exp(delta); the paper keeps w in [0.999, 1.001]
    for delta, kept in ((math.log(1.0009), True), (math.log(1.0011), False),
                        (math.log(0.9991), True), (math.log(0.9989), False)):
        roll = (old.astype(np.float64) - delta)
        _, _, keep, _ = O.mismatch_weights(old.astype(np.float64), roll, mask, cu, prm)
        assert bool(keep.all()) == kept and bool(keep.any()) == kept


def test_mrs_closed_interval_and_strict_veto():
    cu = _segs([3, 3])
    mask = np.ones(6, np.uint8)
    old = np.full(6, -2.0)
    # w == 1 exactly with a degenerate window [1, 1]: the window is closed, so it is kept
    _, _, keep, _ = O.mismatch_weights(old, old, mask, cu, O.Params(mismatch_mode=1, geo_lo=1.0, geo_hi=1.0))
    assert keep.all()
    # a token ratio equal to the veto threshold does not "drop below" it
    _, _, keep, cnt = O.mismatch_weights(old, old, mask, cu, O.Params(mismatch_mode=1, veto_ratio=1.0))
    assert keep.all() and cnt["veto"] == 0


def test_mrs_geometric_mean_uses_loss_tokens_of_each_sample():
    cu = _segs([4, 4])
    mask = np.array([0, 1, 1, 1, 1, 1, 0, 0], np.uint8)
    old = np.zeros(8)
    roll = np.zeros(8)
    roll[0] = 5.0                 # masked token: ignored
    roll[6:] = -5.0               # masked tokens: ignored
    roll[1:4] = [0.0003, -0.0003, 0.0006]     # mean delta = -0.0002 -> w ~ 0.9998, kept
    roll[4:6] = [-0.004, 0.0]                 # mean delta = +0.002  -> w ~ 1.002, rejected
    c, act, keep, cnt = O.mismatch_weights(old, roll, mask, cu, O.Params(mismatch_mode=1))
    assert list(keep) == [True, False] and cnt["geo"] == 1
    assert list(act) == [False, True, True, True, False, False, False, False]


def test_token_veto_rejects_only_its_segment():
    cu = _segs([50, 50])
    mask = np.ones(100, np.uint8)
    old = np.zeros(100)
    roll = np.zeros(100)
    roll[10] = -math.log(0.9e-4)          # ratio 0.9e-4 < 1e-4; ln(1e-4) = -9.2103
    # compensate so that the geometric mean alone would pass
    roll[:10] -= -math.log(0.9e-4) / 10
    _, act, keep, cnt = O.mismatch_weights(old, roll, mask, cu, O.Params(mismatch_mode=1))
    assert list(keep) == [False, True] and cnt == dict(geo=0, veto=1, trunc=0)
    assert not act[:50].any() and act[50:].all()
    roll[10] = -math.log(1.1e-4)          # just above the threshold: no veto
    roll[:10] = (-math.log(1.1e-4)) / -10
    _, _, keep, cnt = O.mismatch_weights(old, roll, mask, cu, O.Params(mismatch_mode=1))
    assert cnt["veto"] == 0


def test_truncation_mode():
    cu = _segs([4])
    mask = np.ones(4, np.uint8)
    old = np.array([0.0, 1.0, -1.0, 0.1])
    roll = np.zeros(4)
    c, act, keep, cnt = O.mismatch_weights(old, roll, mask, cu, O.Params(mismatch_mode=2))
    np.testing.assert_allclose(c, [1.0, 2.0, math.exp(-1), math.exp(0.1)], atol=1e-12)
    assert cnt["trunc"] == 1 and act.all()


# ----------------------------------------------------------------------------- surrogate
def test_ppo_truth_table():
    prm = O.Params()
    A = np.array([1.0, 1.0, 1.0, -1.0, -1.0, -1.0, 0.0])
    r = np.array([1.5, 1.0, 0.5, 1.5, 1.0, 0.5, 1.3])
    loss, g, rr, chi, clo = O.surrogate(np.log(r), np.zeros(7), A, prm)
    np.testing.assert_allclose(rr, r)
    #            A>0,r>1+e  A>0,r=1  A>0,r<1-e  A<0,r>1+e  A<0,r=1  A<0,r<1-e
    np.testing.assert_allclose(loss[:6], [-1.2, -1.0, -0.5, 1.5, 1.0, 0.8], atol=1e-7)
    np.testing.assert_allclose(g[:6], [0.0, -1.0, -0.5, 1.5, 1.0, 0.0], atol=1e-12)
    assert list(chi[:6]) == [True, False, False, False, False, False]
    assert list(clo[:6]) == [False, False, False, False, False, True]
    # unequal ranges: the ratio is clipped to [1 - eps_lo, 1 + eps_hi] = [0.9, 1.3]
    asym = O.Params(clip_eps_lo=0.1, clip_eps_hi=0.3)
    ra = np.array([1.25, 1.35, 0.95, 0.85])
    Aa = np.array([1.0, 1.0, -1.0, -1.0])
    loss_a, g_a, _, chi_a, clo_a = O.surrogate(np.log(ra), np.zeros(4), Aa, asym)
    np.testing.assert_allclose(loss_a, [-1.25, -1.3, 0.95, 0.9], atol=1e-7)
    np.testing.assert_allclose(g_a, [-1.25, 0.0, 0.95, 0.0], atol=1e-12)
    assert list(chi_a) == [False, True, False, False] and list(clo_a) == [False, False, False, True]
    # on-policy: r = 1, l = -A, g = -A   (App. A estimator)
    loss, g, rr, _, _ = O.surrogate(np.log(r), None, A, prm)
    np.testing.assert_allclose(loss, -A)
    np.testing.assert_allclose(g, -A)


def _tiny_problem(seed, T=12, d=8, V=17, S=3):
    rng = np.random.default_rng(seed)
    H = rng.normal(size=(T, d))
    W = rng.normal(size=(V, d)) * 0.5
    y = rng.integers(0, V, T)
    cu = _segs([T // S] * S)
    mask = (rng.random(T) < 0.8).astype(np.uint8)
    mask[0] = 1
    adv = rng.normal(size=S) * 2
    return H, W, y, mask, cu, adv


def test_on_policy_loss_closed_form():
    H, W, y, mask, cu, adv = _tiny_problem(0)
    out = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, None, None, O.Params())
    A_tok = np.repeat(adv, 4)
    n = mask.sum()
    assert abs(out["loss"] - (-(A_tok * mask).sum() / n)) < 1e-12
    assert out["counters"][0] == n and out["counters"][6] == n
    assert np.all(out["dH"][mask == 0] == 0) and np.all(out["logp"][mask == 0] == 0)


def test_cross_entropy_special_case_matches_autograd():
    """A = 1, on-policy, no mismatch: dH, dW are the gradients of mean softmax cross-entropy."""
    H, W, y, mask, cu, _ = _tiny_problem(1)
    for tau in (1.0, 0.7):
        prm = O.Params(temperature=tau)
        out = O.pg_loss_fwd_bwd(H, W, y, mask, cu, np.ones(3), None, None, prm)
        Ht = torch.tensor(H, requires_grad=True)
        Wt = torch.tensor(W, requires_grad=True)
        z = (Ht @ Wt.T) / float(np.float32(tau))
        rows = torch.tensor(np.nonzero(mask)[0])
        ce = torch.nn.functional.cross_entropy(z[rows], torch.tensor(y)[rows], reduction="mean")
        ce.backward()
        np.testing.assert_allclose(out["dH"], Ht.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(out["dW"], Wt.grad.numpy(), atol=1e-12)
        assert abs(out["loss"] + 1.0) < 1e-12                 # value of the surrogate is -mean(A r)
        # A = -1 flips the sign; gradients are linear in A
        neg = O.pg_loss_fwd_bwd(H, W, y, mask, cu, -np.ones(3), None, None, prm)
        np.testing.assert_allclose(neg["dW"], -out["dW"], atol=1e-14)
        tri = O.pg_loss_fwd_bwd(H, W, y, mask, cu, 3 * np.ones(3), None, None, prm)
        np.testing.assert_allclose(tri["dH"], 3 * out["dH"], atol=1e-13)


def _fd_check(H, W, y, mask, cu, adv, old, roll, prm, eps=1e-6):
    out = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, old, roll, prm)
    rng = np.random.default_rng(5)
    f = lambda Hx, Wx: O.loss_value_only(Hx, Wx, y, mask, cu, adv, old, roll, prm)
    for _ in range(12):
        t, k = rng.integers(H.shape[0]), rng.integers(H.shape[1])
        Hp, Hm = H.copy(), H.copy()
        Hp[t, k] += eps
        Hm[t, k] -= eps
        fd = (f(Hp, W) - f(Hm, W)) / (2 * eps)
        assert abs(fd - out["dH"][t, k]) < 2e-8, ("dH", t, k, fd, out["dH"][t, k])
        v, k = rng.integers(W.shape[0]), rng.integers(W.shape[1])
        Wp, Wm = W.copy(), W.copy()
        Wp[v, k] += eps
        Wm[v, k] -= eps
        fd = (f(H, Wp) - f(H, Wm)) / (2 * eps)
        assert abs(fd - out["dW"][v, k]) < 2e-8, ("dW", v, k, fd, out["dW"][v, k])
    return out


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("tau", [1.0, 0.7])
def test_finite_differences_all_branches(mode, tau):
    H, W, y, mask, cu, adv = _tiny_problem(7 + mode)
    prm = O.Params(temperature=tau, mismatch_mode=mode, geo_lo=0.9, geo_hi=1.1)
    logp, _, _ = O.lm_head_logprob(H, W, y, tau)
    rng = np.random.default_rng(11)
    # ratios spread over all four clip quadrants, kept away from the thresholds
    r = rng.choice([0.6, 0.9, 1.0, 1.1, 1.4], size=len(y))
    old = logp - np.log(r)
    roll = old + rng.normal(size=len(y)) * 0.05
    roll[5] = old[5] + 12.0                # one vetoed segment in modes 1/2 (if token 5 is a loss token)
    out = _fd_check(H, W, y, mask, cu, adv, old, roll, prm)
    assert out["counters"][1] + out["counters"][2] > 0          # some rows are clipped
    # rows of dS sum to zero  =>  columns of dW sum to zero (score-function identity, App. A)
    np.testing.assert_allclose(out["dW"].sum(axis=0), 0, atol=1e-12)
    # <dW, W> = <dH, H>: both are sum_t sum_v dS[t,v] * (H W^T)[t,v]
    assert abs((out["dW"] * W).sum() - (out["dH"] * H).sum()) < 1e-12


def test_norm_override_and_all_rejected():
    H, W, y, mask, cu, adv = _tiny_problem(3)
    base = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, None, None, O.Params())
    ovr = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, None, None, O.Params(norm_override=100.0))
    np.testing.assert_allclose(ovr["dW"] * 100.0, base["dW"] * base["norm"], atol=1e-12)
    # every sample rejected: loss 0, gradients 0, normaliser clamps at 1
    old = np.zeros(len(y))
    roll = old - 1.0                        # w = e, far outside the window
    rej = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, old, roll, O.Params(mismatch_mode=1))
    assert rej["loss"] == 0 and not rej["dW"].any() and not rej["dH"].any() and rej["norm"] == 1.0
    assert rej["counters"][0] == 0 and rej["counters"][3] == 3


def test_accumulate_dW():
    H, W, y, mask, cu, adv = _tiny_problem(4)
    prev = np.full_like(W, 0.25)
    a = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, None, None, O.Params())
    b = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, None, None, O.Params(), dW_prev=prev)
    np.testing.assert_allclose(b["dW"], a["dW"] + 0.25, atol=1e-15)


def test_dH_rows_matches_full():
    H, W, y, mask, cu, adv = _tiny_problem(9)
    out = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, None, None, O.Params(temperature=0.7))
    rows = np.nonzero(mask)[0][:5]
    coef = -np.repeat(adv, 4)[rows] / out["norm"]
    np.testing.assert_allclose(O.dH_rows(H[rows], W, y[rows], coef, 0.7), out["dH"][rows], atol=1e-14)


def test_surrogate_propagates_nan_to_the_loss():
    """A NaN log-prob must not be swallowed by the min / clip of the surrogate."""
    l, g, r, _, _ = O.surrogate(np.array([np.nan, -1.0]), np.array([-1.0, -1.0]), np.array([1.0, 1.0]), O.Params())
    assert np.isnan(l[0]) and l[1] == -1.0
