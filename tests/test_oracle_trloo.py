"""Pins for the oracle's returns / GRPO / TRLOO (Sec. 4.2, Eq. 1-5; App. A).  CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import pg_oracle as O


def _load_case(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "layernorm_case_rewards.txt"))
            if l.strip() and not l.startswith("#")]
    a = np.array(rows, dtype=np.float64)
    return a[:, 1], a[:, 2], a[:, 3]


def test_paper_worked_example(golden_dir):
    """Speedups printed in the paper's LayerNorm case -> Eq. (1) rewards -> Eq. (2) returns."""
    speed, R_exp, G_exp = _load_case(golden_dir)
    R = O.reward_eq1(np.ones(3), speed)
    np.testing.assert_allclose(R, R_exp, atol=1e-12)
    G = O.returns(R.reshape(1, 1, 3), 1.0)[0, 0]
    np.testing.assert_allclose(G, G_exp, atol=1e-12)
    G0 = O.returns(R.reshape(1, 1, 3), 0.0)[0, 0]           # gamma = 0 ablation: G = R
    np.testing.assert_allclose(G0, R_exp, atol=1e-12)


def test_reward_clip_and_incorrect():
    # speedup beyond 3 is capped; an incorrect kernel earns nothing (Eq. 1)
    np.testing.assert_allclose(O.reward_eq1([1, 1, 0], [7.5, 3.0, 2.0]), [4.0, 4.0, 0.0])


def test_return_recurrence():
    rng = np.random.default_rng(0)
    R = rng.normal(size=(3, 4, 5))
    for gamma in (1.0, 0.5, 0.0):
        G = O.returns(R, gamma)
        np.testing.assert_allclose(G[:, :, -1], R[:, :, -1])
        np.testing.assert_allclose(G[:, :, :-1] - gamma * G[:, :, 1:], R[:, :, :-1], atol=1e-12)


def test_trloo_closed_forms():
    rng = np.random.default_rng(1)
    P, K, Tm = 5, 7, 3
    R = rng.normal(size=(P, K, Tm)).astype(np.float32)
    valid = (rng.random((P, K, Tm)) < 0.7).astype(np.uint8)
    valid[0, :, 0] = 0                       # empty group
    valid[1, :, 1] = 0
    valid[1, 3, 1] = 1                       # singleton group
    G, A, N = O.trloo_advantage(R, valid, 1.0)
    Agrpo = O.grpo_advantage(R, valid, 1.0)
    for p in range(P):
        for t in range(Tm):
            mem = np.nonzero(valid[p, :, t])[0]
            assert N[p, t] == len(mem)
            # invalid rollouts get nothing
            assert np.all(A[p, valid[p, :, t] == 0, t] == 0)
            if len(mem) < 2:
                assert np.all(A[p, :, t] == 0)
                continue
            n = len(mem)
            # leave-one-out advantages sum to zero over the group
            assert abs(A[p, mem, t].sum()) < 1e-12
            # the two printed forms of Eq. (5) agree: A = N/(N-1) (G - mean)
            np.testing.assert_allclose(A[p, mem, t], n / (n - 1) * (G[p, mem, t] - G[p, mem, t].mean()),
                                       atol=1e-12)
            # ... which is N/(N-1) times the GRPO advantage of Eq. (3)
            np.testing.assert_allclose(A[p, mem, t], n / (n - 1) * Agrpo[p, mem, t], atol=1e-12)


def test_trloo_two_rollouts():
    R = np.array([[[3.0], [1.25]]], dtype=np.float32)          # P=1, K=2, one turn
    _, A, N = O.trloo_advantage(R, np.ones_like(R, dtype=np.uint8))
    assert N[0, 0] == 2
    np.testing.assert_allclose(A[0, :, 0], [1.75, -1.75])


def test_trloo_shift_scale_invariance():
    rng = np.random.default_rng(2)
    R = rng.normal(size=(2, 6, 3))
    valid = np.ones_like(R, dtype=np.uint8)
    _, A, _ = O.trloo_advantage(R, valid)
    R2 = R.copy()
    R2[:, :, 2] += 5.0                        # same constant to every rollout at the last turn
    _, A2, _ = O.trloo_advantage(R2, valid)
    np.testing.assert_allclose(A2, A, atol=1e-12)
    _, A3, _ = O.trloo_advantage(3.0 * R, valid)
    np.testing.assert_allclose(A3, 3.0 * A, atol=1e-12)


def test_single_turn_is_textbook_rloo():
    rng = np.random.default_rng(3)
    R = rng.normal(size=(1, 9, 1))
    _, A, _ = O.trloo_advantage(R, np.ones_like(R, dtype=np.uint8))
    r = R[0, :, 0]
    expected = np.array([r[i] - np.delete(r, i).mean() for i in range(9)])
    np.testing.assert_allclose(A[0, :, 0], expected, atol=1e-12)


def test_early_termination_and_return_credit():
    # a rollout that stops after turn 0 still counts, with its own return, in turn 0's group;
    # later turns see a smaller group (N_t varies, Sec. 4.2)
    R = np.zeros((1, 3, 2), np.float32)
    R[0, :, 0] = [1.0, 2.0, 4.0]
    R[0, :2, 1] = [10.0, 20.0]
    valid = np.ones((1, 3, 2), np.uint8)
    valid[0, 2, 1] = 0
    G, A, N = O.trloo_advantage(R, valid)
    np.testing.assert_allclose(G[0, :, 0], [11.0, 22.0, 4.0])
    assert list(N[0]) == [3, 2]
    np.testing.assert_allclose(A[0, :, 0], [11 - 13, 22 - 7.5, 4 - 16.5])
    np.testing.assert_allclose(A[0, :, 1], [-10.0, 10.0, 0.0])


@pytest.mark.parametrize("N", [2, 3])
def test_exact_enumeration_unbiasedness(N):
    """App. A: E[g_GRPO] = (1 - 1/N) grad J, the leave-one-out estimator is unbiased.

    One prompt, one turn, one token per rollout, a categorical policy over V = 3
    tokens with logits theta; reward depends on the sampled token only.  All V^N
    joint samples are enumerated with their probabilities.  The per-sample gradient
    of log pi comes out of the oracle's own backward (dH with W = I), so this also
    pins the sign and shape of (onehot - softmax) and the token-mean normaliser.
    """
    V = 3
    theta = np.array([0.3, -0.5, 0.9])
    reward_of = np.array([1.0, 0.0, 2.5])
    pi = np.exp(theta) / np.exp(theta).sum()
    gradJ = sum(pi[yv] * reward_of[yv] * (np.eye(V)[yv] - pi) for yv in range(V))
    W = np.eye(V)
    H = np.tile(theta, (N, 1))
    cu = np.arange(N + 1, dtype=np.int32)
    mask = np.ones(N, np.uint8)
    prm = O.Params()
    exp_trloo = np.zeros(V)
    exp_grpo = np.zeros(V)
    for ys in itertools.product(range(V), repeat=N):
        prob = np.prod(pi[list(ys)])
        R = reward_of[list(ys)].reshape(1, N, 1)
        valid = np.ones_like(R, dtype=np.uint8)
        _, A, _ = O.trloo_advantage(R, valid)
        Ag = O.grpo_advantage(R, valid)
        for adv, acc in ((A, exp_trloo), (Ag, exp_grpo)):
            out = O.pg_loss_fwd_bwd(H, W, np.array(ys), mask, cu, adv[0, :, 0], None, None, prm)
            acc += prob * (-out["dH"].sum(axis=0))          # g_hat = -(d loss / d theta)
    np.testing.assert_allclose(exp_trloo, gradJ, atol=1e-12)
    np.testing.assert_allclose(exp_grpo, (1 - 1 / N) * gradJ, atol=1e-12)
