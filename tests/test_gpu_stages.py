"""Parity of the stages around the path with the fp64 oracle, through the C ABI: SFT cross-entropy
(Sec. 3.3), GRPO baseline (Eq. 3), rewards with the profiling ratio (Eq. 1, 6-7), PRS (Eq. 8) and the
monitors (Sec. 5.1).  Integer / byte outputs are compared exactly."""
import numpy as np
import pytest
import torch

from oracle import pg_oracle as O
from paper_2602_05885_amd import binding as B
from paper_2602_05885_amd import synth
from tests._cases import np64, rel_fro

pytestmark = pytest.mark.gpu

TOL_ADV, TOL_LOGP, TOL_LOSS, TOL_GRAD = 1e-6, 2e-3, 1e-3, 1e-2


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


# ------------------------------------------------------------------------------------ SFT
@pytest.mark.parametrize("T,d,V,dtype,tau,seed,mask_frac", [
    (1024, 64, 1000, "f32", 1.0, 11, 0.0),        # the tiny fp32 configuration's head
    (700, 128, 3000, "bf16", 1.0, 12, 0.3),       # ragged rows and vocab, several tiles
    (1500, 256, 5000, "bf16", 0.7, 13, 0.5),
])
def test_sft_parity(dev, T, d, V, dtype, tau, seed, mask_frac, monkeypatch):
    monkeypatch.setenv("PG_HEAD_DS_BUDGET_BYTES", str(2 * 2048 * 1024))      # forces several vocab chunks
    H, W, y = synth.make_head(T, d, V, dtype, seed, dev, unit_rms=(dtype == "bf16"),
                              w_std=0.02 if dtype == "bf16" else 0.1)
    rng = np.random.default_rng(seed)
    mask = (rng.random(T) >= mask_frac).astype(np.uint8)
    prm = B.Params(dtype=0 if dtype == "bf16" else 1, temperature=tau)
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOSS_FWD_BWD, dev)
    out = B.pg_sft_fwd_bwd(H, W, y, torch.from_numpy(mask).to(dev), prm, ws)
    torch.cuda.synchronize()
    ref = O.sft_ce_fwd_bwd(np64(H), np64(W), y.cpu().numpy(), mask, tau)
    tol_logp = TOL_LOGP if dtype == "bf16" else 2e-4
    assert abs(float(out["loss"][0]) - ref["loss"]) <= TOL_LOSS * abs(ref["loss"])
    assert np.abs(out["logp"].cpu().numpy() - ref["logp"]).max() <= tol_logp
    assert np.abs(out["entropy"].cpu().numpy() - ref["entropy"]).max() <= tol_logp
    assert rel_fro(np64(out["dH"]), ref["dH"]) <= TOL_GRAD
    assert rel_fro(np64(out["dW"]), ref["dW"]) <= TOL_GRAD
    assert np.all(np64(out["dH"])[mask == 0] == 0)
    cnt = out["counters"].cpu().numpy()
    assert cnt[0] == ref["n"] and cnt[6] == ref["n"] and not cnt[1:6].any()
    # with the W^T cache (filled by the call, then trusted): the same bits
    prm.w_transposed = B.alloc_w_transposed(d, V, dev)
    for valid in (0, 1):
        prm.w_transposed_valid = valid
        again = B.pg_sft_fwd_bwd(H, W, y, torch.from_numpy(mask).to(dev), prm, ws)
        torch.cuda.synchronize()
        assert torch.equal(again["dH"], out["dH"]) and torch.equal(again["dW"], out["dW"]) and torch.equal(again["loss"], out["loss"])


def test_sft_accumulate_override_and_empty(dev):
    T, d, V = 300, 64, 777
    H, W, y = synth.make_head(T, d, V, "bf16", 21, dev, unit_rms=True)
    mask = np.ones(T, np.uint8)
    mask[::3] = 0
    prm = B.Params(norm_override=1000.0, accumulate_dW=1)
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOSS_FWD_BWD, dev)
    prev = torch.full((V, d), 0.125, dtype=torch.float32, device=dev)
    dW = prev.clone()
    out = B.pg_sft_fwd_bwd(H, W, y, torch.from_numpy(mask).to(dev), prm, ws, dW=dW)
    torch.cuda.synchronize()
    ref = O.sft_ce_fwd_bwd(np64(H), np64(W), y.cpu().numpy(), mask, 1.0, norm_override=1000.0, dW_prev=np64(prev))
    assert abs(float(out["loss"][0]) - ref["loss"]) <= TOL_LOSS * abs(ref["loss"])
    assert rel_fro(np64(out["dW"]) - 0.125, ref["dW"] - 0.125) <= TOL_GRAD
    # all rows masked: zero loss, zero gradients
    prm0 = B.Params()
    out0 = B.pg_sft_fwd_bwd(H, W, y, torch.zeros(T, dtype=torch.uint8, device=dev), prm0, ws)
    torch.cuda.synchronize()
    assert float(out0["loss"][0]) == 0.0 and not out0["dH"].any() and not out0["dW"].any()


# ------------------------------------------------------------------------------------ GRPO
@pytest.mark.parametrize("P,K,Tm,gamma,seed", [(4, 4, 2, 1.0, 0), (16, 8, 3, 1.0, 1), (3, 5, 7, 0.9, 4), (2, 1, 3, 0.0, 5),
                                                (2, 130, 2, 0.9, 6)])
def test_grpo_parity(dev, P, K, Tm, gamma, seed):
    rng = np.random.default_rng(seed)
    correct = rng.random((P, K, Tm)) < 0.5
    R = np.where(correct, 1.0 + np.minimum(rng.lognormal(0, 0.5, (P, K, Tm)), 3.0), 0.0).astype(np.float32)
    valid = (rng.random((P, K, Tm)) < 0.75).astype(np.uint8)
    valid[0, :, 0] = 0                          # empty group
    valid[-1, :, -1] = 0
    valid[-1, 0, -1] = 1                        # singleton group: A = G - G = 0
    adv, ret, gn = B.grpo_advantage(torch.from_numpy(R).to(dev), torch.from_numpy(valid).to(dev), gamma)
    torch.cuda.synchronize()
    A = O.grpo_advantage(R, valid, gamma)
    assert np.abs(adv.cpu().numpy() - A).max() <= TOL_ADV
    assert np.abs(ret.cpu().numpy() - O.returns(R, gamma)).max() <= TOL_ADV
    assert np.array_equal(gn.cpu().numpy(), valid.sum(axis=1).astype(np.int32))


# ------------------------------------------------------------------------------------ rewards, PRS
@pytest.mark.parametrize("n,seed,with_pr", [(1, 0, True), (384, 1, True), (1000, 2, False), (70001, 3, True)])
def test_turn_reward_parity(dev, n, seed, with_pr):
    rng = np.random.default_rng(seed)
    correct = (rng.random(n) < 0.5).astype(np.uint8)
    t_ref = rng.lognormal(0.0, 0.5, n).astype(np.float32)
    t_ker = (t_ref / np.maximum(rng.lognormal(0.0, 0.8, n), 0.05)).astype(np.float32)    # some speedups beyond the cap
    t_tot = rng.lognormal(0.0, 0.5, n).astype(np.float32)
    t_gen = (t_tot * rng.random(n)).astype(np.float32)
    to = lambda a: torch.from_numpy(a).to(dev)
    R, pr = B.turn_reward(to(correct), to(t_ref), to(t_ker), to(t_gen) if with_pr else None,
                          to(t_tot) if with_pr else None, 3.0)
    torch.cuda.synchronize()
    R_ref, pr_ref = O.turn_reward(correct, t_ref, t_ker, t_gen if with_pr else None, t_tot if with_pr else None, 3.0)
    assert np.abs(R.cpu().numpy() - R_ref).max() <= 1e-6 * 5
    assert np.abs(pr.cpu().numpy() - pr_ref).max() <= 1e-6
    assert (R_ref > 4.0 - 1e-9).any() or n < 100          # the cap is exercised
    R2, _ = B.turn_reward(to(correct), to(t_ref), to(t_ker), None, None, 1.5)            # another cap
    torch.cuda.synchronize()
    R2_ref, _ = O.turn_reward(correct, t_ref, t_ker, None, None, 1.5)
    assert np.abs(R2.cpu().numpy() - R2_ref).max() <= 1e-6 * 5 and (n < 100 or R2_ref.max() == 2.5)


@pytest.mark.parametrize("n,seed,hard", [(5, 7, False), (4096, 8, False), (70001, 9, False), (4096, 10, True)])
def test_prs_retain_parity(dev, n, seed, hard):
    rng = np.random.default_rng(seed)
    pr = rng.random(n).astype(np.float32)
    pr[: min(n, 4)] = np.float32([0.3, 0.4, 0.35, 0.29999])[: min(n, 4)]
    valid = (rng.random(n) < 0.9).astype(np.uint8)
    big_seed = (seed << 40) + 12345                       # exercises the high key word
    keep, p = B.prs_retain(torch.from_numpy(pr).to(dev), torch.from_numpy(valid).to(dev), big_seed, 0.3, 0.1, hard)
    torch.cuda.synchronize()
    keep_ref, p_ref = O.prs_retain(pr, valid, big_seed, 0.3, 0.1, hard)
    assert np.array_equal(keep.cpu().numpy(), keep_ref)                         # byte-exact decisions
    assert np.abs(p.cpu().numpy() - p_ref).max() <= 1e-6
    keep_nv, _ = B.prs_retain(torch.from_numpy(pr).to(dev), None, big_seed, 0.3, 0.1, hard)
    torch.cuda.synchronize()
    ref_nv, _ = O.prs_retain(pr, np.ones(n), big_seed, 0.3, 0.1, hard)
    assert np.array_equal(keep_nv.cpu().numpy(), ref_nv)
    keep2, p2 = B.prs_retain(torch.from_numpy(pr).to(dev), None, big_seed, 0.5, 0.25, hard)      # other threshold, softness
    torch.cuda.synchronize()
    ref2, p2_ref = O.prs_retain(pr, np.ones(n), big_seed, 0.5, 0.25, hard)
    assert np.array_equal(keep2.cpu().numpy(), ref2) and np.abs(p2.cpu().numpy() - p2_ref).max() <= 1e-6
    assert n < 100 or not np.array_equal(ref2, ref_nv)


# ------------------------------------------------------------------------------------ monitors
@pytest.mark.parametrize("T,d,V,gdtype,seed", [(1, 64, 100, torch.float32, 0), (5000, 64, 999, torch.float32, 1),
                                               (3001, 128, 1001, torch.bfloat16, 2)])
def test_monitors_parity(dev, T, d, V, gdtype, seed):
    rng = np.random.default_rng(seed)
    mask = (rng.random(T) < 0.7).astype(np.uint8)
    lt = (-rng.gamma(2.0, 1.5, T)).astype(np.float32)
    lr = (lt + rng.normal(0, 0.1, T)).astype(np.float32)
    ent = rng.gamma(2.0, 1.0, T).astype(np.float32)
    dH = torch.from_numpy(rng.normal(0, 1e-3, (T, d)).astype(np.float32)).to(dev).to(gdtype)
    dW = torch.from_numpy(rng.normal(0, 1e-3, (V, d)).astype(np.float32)).to(dev)      # fp32 dW, element count not a multiple of 8 * 1024
    to = lambda a: torch.from_numpy(a).to(dev)
    out = B.pg_monitors(to(lt), to(lr), to(ent), to(mask), dH, dW)
    torch.cuda.synchronize()
    got = dict(zip(B.MONITOR_NAMES, out.cpu().numpy()[:6]))
    ref = O.monitors(lt, lr, ent, mask, np64(dH), np64(dW))
    for k in ("entropy_mean", "ppl_train", "ppl_rollout", "dH_norm", "dW_norm"):
        assert abs(got[k] - ref[k]) <= 1e-9 * max(1.0, abs(ref[k])), (k, got[k], ref[k])
    assert int(got["n"]) == ref["n"]
    # optional inputs absent -> zeros; repeatable bit for bit
    out2 = B.pg_monitors(to(lt), None, None, to(mask))
    out3 = B.pg_monitors(to(lt), to(lr), to(ent), to(mask), dH, dW)
    torch.cuda.synchronize()
    o2 = out2.cpu().numpy()
    assert o2[0] == 0 and o2[2] == 0 and o2[3] == 0 and o2[4] == 0 and abs(o2[1] - ref["ppl_train"]) <= 1e-9 * ref["ppl_train"]
    assert torch.equal(out, out3)


# ------------------------------------------------------------------------------------ RMSNorm
@pytest.mark.parametrize("T,d,dtype,seed", [(1, 64, torch.float32, 0), (37, 520, torch.float32, 1),
                                            (1000, 5120, torch.bfloat16, 2), (4099, 4096, torch.bfloat16, 3),
                                            (513, 8192, torch.bfloat16, 4)])
def test_rmsnorm_parity(dev, T, d, dtype, seed):
    rng = np.random.default_rng(seed)
    eps = 1e-6 if seed % 2 == 0 else 0.05            # the larger one changes rstd by percents: it must be honoured
    X = torch.from_numpy((rng.normal(size=(T, d)) * rng.uniform(0.2, 4.0, size=(T, 1))).astype(np.float32)).to(dev).to(dtype)
    gamma = torch.from_numpy(rng.normal(1.0, 0.2, size=d).astype(np.float32)).to(dev).to(dtype)
    G = torch.from_numpy((rng.normal(size=(T, d)) * 1e-3).astype(np.float32)).to(dev).to(dtype)
    H, rstd = B.pg_rmsnorm_fwd(X, gamma, eps)
    dX, dg = B.pg_rmsnorm_bwd(X, gamma, G, eps)
    dX2, dg2 = B.pg_rmsnorm_bwd(X, gamma, G, eps)
    torch.cuda.synchronize()
    H_ref, rstd_ref = O.rmsnorm_fwd(np64(X), np64(gamma), eps)
    dX_ref, dg_ref = O.rmsnorm_bwd(np64(X), np64(gamma), eps, np64(G))
    tol = 1e-5 if dtype == torch.float32 else 3e-3          # output rounding to bf16: 2^-9 per element
    assert rel_fro(np64(H), H_ref) <= tol
    assert np.abs(rstd.cpu().numpy() / rstd_ref - 1).max() <= 1e-5
    assert rel_fro(np64(dX), dX_ref) <= tol
    assert rel_fro(dg.double().cpu().numpy(), dg_ref) <= 1e-4
    assert torch.equal(dX, dX2) and torch.equal(dg, dg2)      # fixed reduction order
    # in place on the incoming gradient
    Gc = G.clone()
    dX3, _ = B.pg_rmsnorm_bwd(X, gamma, Gc, eps, out=Gc)
    torch.cuda.synchronize()
    assert torch.equal(dX3, dX)


def test_rmsnorm_feeds_the_head(dev):
    """x -> RMSNorm -> fused head loss -> dH -> RMSNorm backward: the chain against the oracle's chain."""
    T, d, V = 600, 256, 3000
    rng = np.random.default_rng(5)
    X = torch.from_numpy((rng.normal(size=(T, d)) * 3.0).astype(np.float32)).to(dev).bfloat16()
    gamma = torch.from_numpy(rng.normal(1.0, 0.1, size=d).astype(np.float32)).to(dev).bfloat16()
    _, W, y = synth.make_head(T, d, V, "bf16", 31, dev, unit_rms=True)
    mask = (rng.random(T) < 0.8).astype(np.uint8)
    H, _ = B.pg_rmsnorm_fwd(X, gamma, 1e-6, want_rstd=False)
    prm = B.Params()
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOSS_FWD_BWD, dev)
    out = B.pg_sft_fwd_bwd(H, W, y, torch.from_numpy(mask).to(dev), prm, ws)
    dX, dg = B.pg_rmsnorm_bwd(X, gamma, out["dH"], 1e-6)
    torch.cuda.synchronize()
    H_ref, _ = O.rmsnorm_fwd(np64(X), np64(gamma), 1e-6)
    H_bits = torch.from_numpy(H_ref).bfloat16().double().numpy()          # the head sees bf16 hidden states
    ref = O.sft_ce_fwd_bwd(H_bits, np64(W), y.cpu().numpy(), mask)
    dX_ref, dg_ref = O.rmsnorm_bwd(np64(X), np64(gamma), 1e-6, ref["dH"])
    assert abs(float(out["loss"][0]) - ref["loss"]) <= TOL_LOSS * abs(ref["loss"])
    assert rel_fro(np64(dX), dX_ref) <= TOL_GRAD
    assert rel_fro(dg.double().cpu().numpy(), dg_ref) <= TOL_GRAD


@pytest.mark.parametrize("dtype,mode,kind,seed,few", [("bf16", 2, "token", 71, False), ("bf16", 1, "window", 72, False),
                                                      ("f32", 0, "none", 73, False), ("bf16", 1, "window", 8080, True)])
def test_loss_with_fused_rmsnorm(dev, monkeypatch, dtype, mode, kind, seed, few):
    """pg_loss_fwd_bwd_normed (normalisation applied while the rows are compacted, its backward while dH is
    scattered) against the oracle's chain rmsnorm_fwd -> pg_loss_fwd_bwd -> rmsnorm_bwd, several vocab chunks,
    masked and rejected rows; and against the separate calls of the library (same kernels around the head)."""
    from tests._cases import segment_offsets, ratio_targets, block_rel_fro
    if few:     # most samples rejected: the dH accumulator holds several split-K slabs that the fused backward adds up
        spec = synth.small_spec(seed=seed, d=128, V=4200, dtype=dtype, P=4, K=6, Tmax=3, len_lo=40, len_hi=120)
    else:
        spec = synth.small_spec(seed=seed, d=192, V=2300, dtype=dtype, P=3, K=4, Tmax=3)
    batch = synth.make_batch(spec)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    monkeypatch.setenv("PG_HEAD_DS_BUDGET_BYTES", str(((T + 255) // 256 * 256) * 2 * 256 * 3))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(seed)
    eps = 1e-5
    X = torch.from_numpy((rng.normal(size=(T, d)) * rng.uniform(0.3, 3.0, size=(T, 1))).astype(np.float32)).to(dev).to(tdt)
    gamma = torch.from_numpy(rng.normal(1.0, 0.2, size=d).astype(np.float32)).to(dev).to(tdt)
    _, W, y = synth.make_head(T, d, V, dtype, spec.seed, dev, unit_rms=True, w_std=0.02 if dtype == "bf16" else 0.1)
    # oracle chain; the head sees h rounded to the storage dtype
    H_ref, _ = O.rmsnorm_fwd(np64(X), np64(gamma), eps)
    H_bits = torch.from_numpy(H_ref).to(tdt).double().numpy()
    Wn, yn = np64(W), y.cpu().numpy().astype(np.int64)
    base = O.lm_head_logprob(H_bits, Wn, yn, 1.0)[0]
    old = (base - np.log(ratio_targets(T, seed))).astype(np.float32)
    rollout = (old.astype(np.float64) - segment_offsets(batch, seed, kind)).astype(np.float32)
    _, A, _ = O.trloo_advantage(batch.rewards, batch.valid, 1.0)
    ref = O.pg_loss_fwd_bwd(H_bits, Wn, yn, batch.loss_mask, batch.cu_seqlens, A.reshape(-1)[batch.seg_sample],
                            old, rollout if mode else None, O.Params(mismatch_mode=mode))
    dX_ref, dg_ref = O.rmsnorm_bwd(np64(X), np64(gamma), eps, ref["dH"])
    # library, fused
    to = lambda a: torch.from_numpy(a).to(dev)
    prm = B.Params(dtype=0 if dtype == "bf16" else 1, mismatch_mode=mode)
    adv, _, _ = B.trloo_advantage(to(batch.rewards), to(batch.valid), 1.0)
    args = (to(batch.loss_mask), to(batch.cu_seqlens), adv.reshape(-1), to(batch.seg_sample), to(old),
            to(rollout) if mode else None)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD_NORMED, dev)
    out = B.pg_loss_fwd_bwd_normed(X, gamma, eps, W, y, *args, prm, ws)
    out2 = B.pg_loss_fwd_bwd_normed(X, gamma, eps, W, y, *args, prm, ws)
    torch.cuda.synchronize()
    tol_lp = TOL_LOGP if dtype == "bf16" else 2e-4
    assert np.array_equal(out["counters"].cpu().numpy(), ref["counters"])
    assert 0 < ref["counters"][0] < T
    if few:
        assert 2 * ((int(ref["counters"][0]) + 255) // 256 * 256) <= (T + 255) // 256 * 256      # room for two parts
    assert np.abs(out["logp"].cpu().numpy() - ref["logp"]).max() <= tol_lp
    assert np.abs(out["entropy"].cpu().numpy() - ref["entropy"]).max() <= tol_lp
    assert abs(float(out["loss"][0]) - ref["loss"]) <= TOL_LOSS * abs(ref["loss"])
    e_dx, e_dg, e_dw = rel_fro(np64(out["dX"]), dX_ref), rel_fro(out["dgamma"].double().cpu().numpy(), dg_ref), rel_fro(np64(out["dW"]), ref["dW"])
    print(f"[fused norm {dtype} mode {mode}] dX {e_dx:.2e} (worst block {block_rel_fro(np64(out['dX']), dX_ref):.2e}) dgamma {e_dg:.2e} dW {e_dw:.2e}")
    tol_g = TOL_GRAD if dtype == "bf16" else 5e-5            # split operands throughout for fp32 (achieved 1e-5)
    assert e_dx <= tol_g and e_dg <= tol_g and e_dw <= tol_g
    assert block_rel_fro(np64(out["dX"]), dX_ref) <= tol_g
    assert np.all(np64(out["dX"])[~ref["active"]] == 0)
    for k in ("loss", "dX", "dgamma", "dW", "logp"):
        assert torch.equal(out[k], out2[k]), k                                      # fixed reduction orders
    # the separate calls (normalise every row, head, backward of the normalisation) agree with the fused one
    H, _ = B.pg_rmsnorm_fwd(X, gamma, eps, want_rstd=False)
    ws1 = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    sep = B.pg_loss_fwd_bwd(H, W, y, *args, prm, ws1)
    dX_sep, dg_sep = B.pg_rmsnorm_bwd(X, gamma, sep["dH"], eps)
    torch.cuda.synchronize()
    assert torch.equal(sep["logp"], out["logp"]) and torch.equal(sep["dW"], out["dW"]) and torch.equal(sep["loss"], out["loss"])
    assert rel_fro(np64(dX_sep), np64(out["dX"])) <= 5e-3 and rel_fro(dg_sep.double().cpu().numpy(), out["dgamma"].double().cpu().numpy()) <= 5e-3


# ------------------------------------------------------------------------------------ the whole recipe
@pytest.mark.parametrize("mode,kind,seed", [(1, "window", 41), (2, "token", 42)])
def test_recipe_reward_prs_trloo_loss(dev, monkeypatch, mode, kind, seed):
    """Rewards with the profiling ratio (Eq. 1, 6-7) -> PRS keep flags (Eq. 8) -> TRLOO (Eq. 5) -> loss with
    mismatch correction (Sec. 5.1), chained on the device with no host step between the calls: the keep
    flags and the advantage table go straight into pg_loss_fwd_bwd."""
    from tests._cases import build_loss_case
    spec = synth.small_spec(seed=seed, P=4, K=5, Tmax=3)
    batch, tin, nin = build_loss_case(spec, dev, lambda H, W, y, tau: O.lm_head_logprob(H, W, y, tau)[0], kind,
                                      on_policy=False)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    monkeypatch.setenv("PG_HEAD_DS_BUDGET_BYTES", str(((T + 255) // 256 * 256) * 2 * 256 * 4))
    n = spec.P * spec.K * spec.Tmax
    rng = np.random.default_rng(seed)
    correct = (rng.random(n) < 0.7).astype(np.uint8)
    t_ref = rng.lognormal(0.0, 0.5, n).astype(np.float32)
    t_ker = (t_ref / np.maximum(rng.lognormal(0.0, 0.8, n), 0.05)).astype(np.float32)
    t_tot = rng.lognormal(0.0, 0.5, n).astype(np.float32)
    t_gen = (t_tot * rng.random(n)).astype(np.float32)
    valid = nin["valid"]
    to = lambda a: torch.from_numpy(a).to(dev)
    prm = B.Params(mismatch_mode=mode)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    R, pr = B.turn_reward(to(correct), to(t_ref), to(t_ker), to(t_gen), to(t_tot), 3.0)
    keep, _ = B.prs_retain(pr, tin["valid"].reshape(-1), 2602, 0.3, 0.1, False)
    adv, _, _ = B.trloo_advantage(R.reshape(spec.P, spec.K, spec.Tmax), tin["valid"], 1.0)
    out = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                            tin["old"], tin["rollout"], prm, ws, sample_keep=keep)
    torch.cuda.synchronize()

    R_ref, pr_ref = O.turn_reward(correct, t_ref, t_ker, t_gen, t_tot, 3.0)
    R32, pr32 = R_ref.astype(np.float32), pr_ref.astype(np.float32)          # what the ABI hands from stage to stage
    keep_ref, _ = O.prs_retain(pr32, valid.reshape(-1), 2602, 0.3, 0.1, False)
    assert np.array_equal(keep.cpu().numpy(), keep_ref)
    _, A, _ = O.trloo_advantage(R32.reshape(spec.P, spec.K, spec.Tmax), valid, 1.0)
    assert np.abs(adv.cpu().numpy() - A).max() <= TOL_ADV
    oprm = O.Params(mismatch_mode=mode)
    seg = nin["seg_sample"]
    ref = O.pg_loss_fwd_bwd(nin["H"], nin["W"], nin["y"], nin["loss_mask"], nin["cu"], A.reshape(-1)[seg], nin["old"],
                            nin["rollout"], oprm, seg_keep=keep_ref[seg])
    cnt = out["counters"].cpu().numpy()
    assert np.array_equal(cnt, ref["counters"]), (cnt, ref["counters"])
    assert 0 < cnt[7] < S and 0 < cnt[0] < batch.loss_mask.sum()              # some samples dropped, some kept
    assert abs(float(out["loss"][0]) - ref["loss"]) <= TOL_LOSS * max(abs(ref["loss"]), 1e-6)
    assert np.abs(out["logp"].cpu().numpy() - ref["logp"]).max() <= TOL_LOGP
    dH = np64(out["dH"])
    assert np.all(dH[~ref["active"]] == 0)
    assert rel_fro(dH, ref["dH"]) <= TOL_GRAD and rel_fro(np64(out["dW"]), ref["dW"]) <= TOL_GRAD
    # the same flags as a zeroed loss mask: bitwise the same gradients
    lm = tin["loss_mask"].clone()
    cu = batch.cu_seqlens
    for s in range(S):
        if not keep_ref[seg[s]]:
            lm[cu[s]:cu[s + 1]] = 0
    out2 = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], lm, tin["cu"], adv.reshape(-1), tin["seg_sample"],
                             tin["old"], tin["rollout"], prm, ws)
    torch.cuda.synchronize()
    assert torch.equal(out2["dW"], out["dW"]) and torch.equal(out2["dH"], out["dH"]) and torch.equal(out2["loss"], out["loss"])
