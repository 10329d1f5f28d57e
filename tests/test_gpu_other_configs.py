"""The other full-size workloads of the benchmark definition, each run once through the C ABI and
checked with the size-independent tools of the headline test: a library (torch fp32) log-prob for
every row, the fp64 oracle on sampled rows, exact integer outputs, and identities.

  configs[1]  Qwen3-8B head (d=4096), 16k packed rows, the paper's geometric rejection (mode 1)
  configs[3]  64k packed rows of long segments, K=16 rollouts x 4 turns, ~40 % rows masked, on-policy
  configs[4]  forward only, 128k rows, temperature 0.7
"""
import numpy as np
import pytest
import torch

from oracle import pg_oracle as O
from paper_2602_05885_amd import binding as B
from paper_2602_05885_amd import synth
from tests._cases import np64, rel_fro
from tests.test_gpu_fullsize import library_logp_lse

pytestmark = pytest.mark.gpu

N_ROWS = 24


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


def _check_rows_and_identities(spec, batch, H, W, y, out, active, coef_tok, lib_logp, dev, seed):
    """coef_tok[t] = d loss / d logp_t of every row (0 on inactive rows)."""
    T = H.shape[0]
    rng = np.random.default_rng(seed)
    act_idx = np.nonzero(active)[0]
    rows = np.sort(rng.choice(act_idx, N_ROWS, replace=False))
    Wn = np64(W)
    Hr = np64(H[torch.from_numpy(rows).to(dev)])
    yn = y.cpu().numpy().astype(np.int64)
    o_logp, o_ent, _ = O.lm_head_logprob(Hr, Wn, yn[rows], spec.temperature)
    got = out["logp"].cpu().numpy()
    assert np.abs(lib_logp.cpu().numpy()[rows] - o_logp).max() <= 2e-4         # the library reference itself
    assert np.abs(got[rows] - o_logp).max() <= 2e-3
    assert np.abs(out["entropy"].cpu().numpy()[rows] - o_ent).max() <= 2e-3
    assert np.abs(got[active] - lib_logp.cpu().numpy()[active]).max() <= 2e-3
    assert np.all(got[~active] == 0)
    ref = O.dH_rows(Hr, Wn, yn[rows], coef_tok[rows], spec.temperature)
    assert rel_fro(np64(out["dH"][torch.from_numpy(rows).to(dev)]), ref) <= 1e-2
    inactive = torch.from_numpy(np.nonzero(~active)[0]).to(dev)
    assert not out["dH"][inactive].any()
    dW, dH = out["dW"], out["dH"]
    col = dW.double().sum(dim=0)
    assert float((col.abs() / dW.double().abs().sum(dim=0)).max()) < 2e-3      # rows of dS sum to zero
    lhs = float((dW.double() * W.double()).sum())
    rhs = float((dH.double() * H.double()).sum())
    assert abs(lhs - rhs) <= 1e-2 * max(abs(lhs), abs(rhs)), (lhs, rhs)


def test_config1_8b_head_geometric_rejection(dev):
    spec = synth.SPECS[1]
    batch = synth.make_batch(spec)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    print(f"[config1] T={T} S={S} d={d} V={V}", flush=True)
    H, W, y = synth.make_head(T, d, V, spec.dtype, spec.seed, dev, spec.unit_rms)
    lib_logp, _ = library_logp_lse(H, W, y, spec.temperature)
    old = lib_logp.cpu().numpy().astype(np.float32)                            # on-policy: ratio 1
    # per-segment trainer-vs-rollout offsets: inside the paper's window, outside it, and one veto
    rng = np.random.Generator(np.random.Philox(key=spec.seed + 5))
    delta = np.zeros(T)
    choices = np.array([0.0, 4e-4, -5e-4, 2.5e-3, -3e-3])
    for s in range(S):
        a, b = batch.cu_seqlens[s], batch.cu_seqlens[s + 1]
        delta[a:b] = choices[s % len(choices)] + rng.uniform(-1e-5, 1e-5, size=b - a)
    a, b = batch.cu_seqlens[0], batch.cu_seqlens[1]
    delta[a + np.nonzero(batch.loss_mask[a:b])[0][3]] = -10.0                   # token veto in segment 0
    rollout = (old.astype(np.float64) - delta).astype(np.float32)
    prm = B.Params(mismatch_mode=1, temperature=spec.temperature)
    to = lambda x: torch.from_numpy(x).to(dev)
    adv, _, gn = B.trloo_advantage(to(batch.rewards), to(batch.valid), 1.0)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    out = B.pg_loss_fwd_bwd(H, W, y, to(batch.loss_mask), to(batch.cu_seqlens), adv.reshape(-1), to(batch.seg_sample),
                            to(old), to(rollout), prm, ws)
    torch.cuda.synchronize()
    del ws
    oprm = O.Params(mismatch_mode=1, temperature=spec.temperature)
    _, A, N = O.trloo_advantage(batch.rewards, batch.valid, 1.0)
    assert np.abs(adv.cpu().numpy() - A).max() <= 1e-6 and np.array_equal(gn.cpu().numpy(), N)
    c, active, keep, mm = O.mismatch_weights(old, rollout, batch.loss_mask, batch.cu_seqlens, oprm)
    cnt = out["counters"].cpu().numpy()
    assert cnt[0] == active.sum() and cnt[3] == mm["geo"] and cnt[4] == mm["veto"] and cnt[6] == batch.loss_mask.sum()
    assert 0 < active.sum() < batch.loss_mask.sum() and mm["geo"] > 0 and mm["veto"] == 1
    norm = float(max(1, int(active.sum())))
    A_tok = np.zeros(T)
    adv_seg = A.reshape(-1)[batch.seg_sample]
    for s in range(S):
        A_tok[batch.cu_seqlens[s]:batch.cu_seqlens[s + 1]] = adv_seg[s]
    coef = np.where(active, -A_tok * c / norm, 0.0)                             # r = 1: dl/dlogp = -A
    ref_loss = float((c[active] * -A_tok[active]).sum() / norm)
    assert abs(float(out["loss"][0]) - ref_loss) <= 1e-3 * abs(ref_loss)
    _check_rows_and_identities(spec, batch, H, W, y, out, active, coef, lib_logp, dev, 11)


def test_config3_long_segments_on_policy(dev):
    spec = synth.SPECS[3]
    batch = synth.make_batch(spec)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    print(f"[config3] T={T} S={S} loss rows={int(batch.loss_mask.sum())}", flush=True)
    H, W, y = synth.make_head(T, d, V, spec.dtype, spec.seed, dev, spec.unit_rms)
    lib_logp, _ = library_logp_lse(H, W, y, spec.temperature)
    prm = B.Params(mismatch_mode=0, temperature=spec.temperature)
    to = lambda x: torch.from_numpy(x).to(dev)
    adv, _, gn = B.trloo_advantage(to(batch.rewards), to(batch.valid), 1.0)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    out = B.pg_loss_fwd_bwd(H, W, y, to(batch.loss_mask), to(batch.cu_seqlens), adv.reshape(-1), to(batch.seg_sample),
                            None, None, prm, ws)
    torch.cuda.synchronize()
    del ws
    _, A, N = O.trloo_advantage(batch.rewards, batch.valid, 1.0)
    assert np.abs(adv.cpu().numpy() - A).max() <= 1e-6 and np.array_equal(gn.cpu().numpy(), N)
    assert N.max() <= 16 and N.min() >= 1
    active = batch.loss_mask.astype(bool)
    frac_masked = 1.0 - active.mean()
    assert 0.3 < frac_masked < 0.5
    n = int(active.sum())
    cnt = out["counters"].cpu().numpy()
    assert cnt[0] == n and cnt[6] == n and not cnt[1:6].any()
    A_tok = np.zeros(T)
    adv_seg = A.reshape(-1)[batch.seg_sample]
    for s in range(S):
        A_tok[batch.cu_seqlens[s]:batch.cu_seqlens[s + 1]] = adv_seg[s]
    ref_loss = float(-A_tok[active].sum() / n)                                  # on-policy closed form: -mean A
    assert abs(float(out["loss"][0]) - ref_loss) <= 1e-3 * max(abs(ref_loss), 1e-3)
    coef = np.where(active, -A_tok / n, 0.0)
    _check_rows_and_identities(spec, batch, H, W, y, out, active, coef, lib_logp, dev, 13)


def test_config4_forward_only_128k(dev):
    spec = synth.SPECS[4]
    batch = synth.make_batch(spec)
    T, d, V = batch.T, spec.d, spec.V
    assert T == 131072
    H, W, y = synth.make_head(T, d, V, spec.dtype, spec.seed, dev, spec.unit_rms)
    lib_logp, lib_lse = library_logp_lse(H, W, y, float(np.float32(spec.temperature)))
    prm = B.Params(temperature=spec.temperature)
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
    logp, ent, lse = B.pg_logprob_fwd(H, W, y, None, prm, ws)
    torch.cuda.synchronize()
    assert float((logp - lib_logp).abs().max()) <= 2e-3
    assert float((lse - lib_lse).abs().max()) <= 2e-3
    rows = np.sort(np.random.default_rng(17).choice(T, N_ROWS, replace=False))
    o_logp, o_ent, o_lse = O.lm_head_logprob(np64(H[torch.from_numpy(rows).to(dev)]), np64(W),
                                             y.cpu().numpy().astype(np.int64)[rows], spec.temperature)
    assert np.abs(logp.cpu().numpy()[rows] - o_logp).max() <= 2e-3
    assert np.abs(ent.cpu().numpy()[rows] - o_ent).max() <= 2e-3
    assert np.abs(lse.cpu().numpy()[rows] - o_lse).max() <= 2e-3
    to = lambda x: torch.from_numpy(x).to(dev)
    adv, ret, gn = B.trloo_advantage(to(batch.rewards), to(batch.valid), 1.0)
    torch.cuda.synchronize()
    G, A, N = O.trloo_advantage(batch.rewards, batch.valid, 1.0)
    assert np.abs(adv.cpu().numpy() - A).max() <= 1e-6 and np.array_equal(gn.cpu().numpy(), N)


def test_f32_head_at_full_vocabulary_operand_beyond_4_gib(dev):
    """fp32 H and W at the 14B head shape: the split weight operand is [151936, 3 x 5120] bf16 = 4.7 GB, beyond
    what one 32-bit buffer range covers, so every tile's resource must start at its own rows.  Target tokens
    are placed in the vocabulary rows beyond the 4 GiB mark; log-prob, entropy and logsumexp against the
    oracle on sampled rows (fp32 inputs: 2e-4), dH rows and dW rows of a small loss call likewise."""
    T, d, V = 1000, 5120, 151936
    H, W, y = synth.make_head(T, d, V, "f32", 4242, dev, unit_rms=True, w_std=0.02)
    first_beyond = (1 << 32) // (3 * d * 2) + 1
    y[::2] = torch.randint(first_beyond, V, (len(y[::2]),), generator=torch.Generator().manual_seed(1)).to(dev).to(y.dtype)
    prm = B.Params(dtype=1)
    ws = B.alloc_workspace(T, d, V, 1, prm, B.CALL_LOSS_FWD_BWD, dev)
    logp, ent, lse = B.pg_logprob_fwd(H, W, y, None, prm, ws)
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(3).choice(T, 24, replace=False))
    rt = torch.from_numpy(rows).to(dev)
    Wn, yn = np64(W), y.cpu().numpy().astype(np.int64)
    assert (yn[rows] >= first_beyond).any()
    o_logp, o_ent, o_lse = O.lm_head_logprob(np64(H[rt]), Wn, yn[rows], 1.0)
    assert np.abs(logp.cpu().numpy()[rows] - o_logp).max() <= 2e-4
    assert np.abs(ent.cpu().numpy()[rows] - o_ent).max() <= 2e-4
    assert np.abs(lse.cpu().numpy()[rows] - o_lse).max() <= 2e-4
    lib_logp, _ = library_logp_lse(H, W, y, 1.0)
    assert float((logp - lib_logp).abs().max()) <= 2e-4
    # backward through the same operand: SFT loss on all rows, sampled dH rows and dW rows beyond the mark
    out = B.pg_sft_fwd_bwd(H, W, y, torch.ones(T, dtype=torch.uint8, device=dev), prm, ws)
    torch.cuda.synchronize()
    ref_dH = O.dH_rows(np64(H[rt]), Wn, yn[rows], np.full(len(rows), -1.0 / T), 1.0)
    assert rel_fro(np64(out["dH"][rt]), ref_dH) <= 1e-2
    vs = np.unique(np.concatenate([yn[::2][:6], [V - 1, first_beyond, 0]]))
    Hn = np64(H)
    z = Hn @ Wn[vs].T
    lse_rows = (torch.logsumexp(H.double() @ W.double().T, dim=1)).cpu().numpy()
    k = -1.0 / T
    dS = -np.exp(z - lse_rows[:, None]) * k + (yn[:, None] == vs[None, :]) * k
    assert rel_fro(np64(out["dW"][torch.from_numpy(vs).to(dev)]), dS.T @ Hn) <= 1e-2
