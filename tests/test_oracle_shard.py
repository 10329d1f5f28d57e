"""Pins for the oracle's vocab-sharded head: a shard's softmax state, the merge of two states and a
shard's share of the gradients are checked against the unsharded definitions (library
log-softmax, the whole-vocabulary loss) and against the algebra they must obey.  CPU only."""
import itertools

import numpy as np
import pytest
import torch

from oracle import pg_oracle as O


def _problem(seed=0, T=29, d=16, V=61):
    rng = np.random.default_rng(seed)
    H = rng.normal(size=(T, d))
    W = rng.normal(size=(V, d)) * 0.8
    y = rng.integers(0, V, size=T)
    mask = (rng.random(T) < 0.75).astype(np.uint8)
    return H, W, y, mask


def _shards(V, cuts):
    edges = [0] + list(cuts) + [V]
    return list(zip(edges[:-1], edges[1:]))


@pytest.mark.parametrize("cuts,tau", [((20,), 1.0), ((7, 40), 0.7), ((1, 2, 60), 1.3)])
def test_merged_shard_states_equal_library_log_softmax(cuts, tau):
    H, W, y, mask = _problem()
    parts = [O.head_shard_partials(H, W[a:b], y, a, tau, mask) for a, b in _shards(W.shape[0], cuts)]
    merged = parts[0]
    for p in parts[1:]:
        merged = O.merge_shard_partials(merged, p)
    logp, ent, lse = O.finish_shard_partials(merged)
    z = torch.tensor(H @ W.T / float(np.float32(tau)))
    ls = torch.log_softmax(z, dim=1)
    live = mask.astype(bool)
    ref_logp = ls[torch.arange(len(y)), torch.tensor(y)].numpy()
    ref_ent = -(ls.exp() * ls).sum(dim=1).numpy()
    np.testing.assert_allclose(logp[live], ref_logp[live], atol=1e-12)
    np.testing.assert_allclose(ent[live], ref_ent[live], atol=1e-12)
    np.testing.assert_allclose(lse[live], torch.logsumexp(z, dim=1).numpy()[live], atol=1e-12)
    assert np.all(merged[~live] == 0) and np.all(logp[~live] == 0) and np.all(ent[~live] == 0)


def test_shard_state_is_the_plain_definition():
    H, W, y, _ = _problem(1)
    a, b = 13, 40
    P = O.head_shard_partials(H, W[a:b], y, a, 1.0)
    z = H @ W[a:b].T
    for t in range(H.shape[0]):
        m = max(z[t])
        assert abs(P[t, 0] - m) < 1e-12
        assert abs(P[t, 1] - sum(np.exp(v - m) for v in z[t])) < 1e-12
        assert abs(P[t, 2] - sum(np.exp(v - m) * (v - m) for v in z[t])) < 1e-12
        assert abs(P[t, 3] - (z[t, y[t] - a] if a <= y[t] < b else 0.0)) < 1e-12
    # exactly one shard of a partition holds the sampled token's logit
    owners = sum((O.head_shard_partials(H, W[lo:hi], y, lo)[:, 3] != 0).astype(int)
                 for lo, hi in _shards(W.shape[0], (13, 40)))
    assert np.all(owners == 1)


def test_merge_is_commutative_associative_and_has_a_neutral_element():
    H, W, y, mask = _problem(2)
    sh = _shards(W.shape[0], (9, 30, 45))
    parts = [O.head_shard_partials(H, W[a:b], y, a, 1.0, mask) for a, b in sh]
    ref = None
    for order in itertools.permutations(range(4)):
        m = parts[order[0]]
        for k in order[1:]:
            m = O.merge_shard_partials(m, parts[k])
        if ref is None:
            ref = m
        np.testing.assert_allclose(m, ref, rtol=1e-13, atol=1e-13)
    tree = O.merge_shard_partials(O.merge_shard_partials(parts[0], parts[1]), O.merge_shard_partials(parts[2], parts[3]))
    np.testing.assert_allclose(tree, ref, rtol=1e-13, atol=1e-13)
    empty = np.zeros_like(parts[0])
    assert np.array_equal(O.merge_shard_partials(parts[0], empty), parts[0])
    assert np.array_equal(O.merge_shard_partials(empty, parts[0]), parts[0])


def test_merge_with_far_apart_maxima_does_not_overflow():
    a = np.array([[700.0, 3.0, -1.5, 700.0]])
    b = np.array([[-700.0, 5.0, -2.0, 0.0]])
    m = O.merge_shard_partials(a, b)
    assert np.all(np.isfinite(m)) and m[0, 0] == 700.0 and abs(m[0, 1] - 3.0) < 1e-12
    np.testing.assert_allclose(O.merge_shard_partials(b, a), m)


@pytest.mark.parametrize("mode", [0, 2])
def test_shard_gradients_tile_the_whole_vocabulary_gradients(mode):
    rng = np.random.default_rng(5)
    H, W, y, mask = _problem(3, T=40, V=50)
    cu = np.array([0, 11, 25, 40])
    adv = rng.normal(size=3)
    lp, _, _ = O.lm_head_logprob(H, W, y, 1.0)
    old = lp + rng.normal(size=len(lp)) * 0.15
    roll = old + rng.normal(size=len(lp)) * 0.1
    prm = O.Params(mismatch_mode=mode)
    full = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, old, roll, prm)
    dH_sum = np.zeros_like(full["dH"])
    for a, b in _shards(W.shape[0], (17, 33)):
        part = O.pg_loss_fwd_bwd(H, W, y, mask, cu, adv, old, roll, prm, vocab_slice=(a, b))
        assert part["dW"].shape == (b - a, W.shape[1])
        np.testing.assert_allclose(part["dW"], full["dW"][a:b], rtol=0, atol=1e-15)
        assert part["loss"] == full["loss"] and np.array_equal(part["logp"], full["logp"])
        dH_sum += part["dH"]
    np.testing.assert_allclose(dH_sum, full["dH"], atol=1e-14)
    # a shard that holds no sampled token still has a gradient: -coef/tau * p on its columns
    none = O.pg_loss_fwd_bwd(H, W, np.zeros_like(y), mask, cu, adv, None, None, O.Params(), vocab_slice=(17, 33))
    assert np.abs(none["dW"]).max() > 0


def test_shard_dW_accumulates_into_the_shards_rows():
    H, W, y, mask = _problem(4, T=24, V=30)
    cu = np.array([0, 24])
    prev = np.full((12, W.shape[1]), 0.5)
    a = O.pg_loss_fwd_bwd(H, W, y, mask, cu, [1.0], None, None, O.Params(), vocab_slice=(10, 22))
    b = O.pg_loss_fwd_bwd(H, W, y, mask, cu, [1.0], None, None, O.Params(), vocab_slice=(10, 22), dW_prev=prev)
    np.testing.assert_allclose(b["dW"], a["dW"] + 0.5, atol=1e-15)
