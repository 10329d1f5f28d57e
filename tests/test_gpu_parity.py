"""Parity of the HIP library (through the C ABI) with the fp64 oracle on the same seeded inputs.

Tolerances are the stated ones: advantages 1e-6 abs, log-probs 2e-3 abs (bf16 inputs), loss 1e-3
relative, dH / dW 1e-2 relative Frobenius norm.  Integer outputs (counters, group sizes) must match
exactly; test inputs keep ratios and sample weights away from the decision thresholds.
"""
import numpy as np
import pytest
import torch

from oracle import pg_oracle as O
from paper_2602_05885_amd import binding as B
from paper_2602_05885_amd import synth
from tests._cases import block_rel_fro, build_loss_case, np64, rel_fro

pytestmark = pytest.mark.gpu

TOL_ADV, TOL_LOGP, TOL_LOSS, TOL_GRAD = 1e-6, 2e-3, 1e-3, 1e-2


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


def oracle_logp(Hn, Wn, yn, tau):
    return O.lm_head_logprob(Hn, Wn, yn, tau)[0]


# ------------------------------------------------------------------------------------ TRLOO
@pytest.mark.parametrize("P,K,Tm,gamma,seed", [(4, 4, 2, 1.0, 0), (16, 8, 3, 1.0, 1), (4, 16, 4, 1.0, 2),
                                                (32, 16, 2, 1.0, 3), (3, 5, 7, 0.9, 4), (2, 1, 3, 1.0, 5),
                                                (1, 2, 1, 0.0, 6),
                                                (2, 100, 3, 0.9, 7),      # rollouts beyond one wavefront's 64 lanes
                                                (2, 300, 2, 1.0, 8)])     # ... and beyond the returns a lane holds
def test_trloo_parity(dev, P, K, Tm, gamma, seed):
    rng = np.random.default_rng(seed)
    correct = rng.random((P, K, Tm)) < 0.5
    R = np.where(correct, 1.0 + np.minimum(rng.lognormal(0, 0.5, (P, K, Tm)), 3.0), 0.0).astype(np.float32)
    valid = (rng.random((P, K, Tm)) < 0.75).astype(np.uint8)
    if P > 1:
        valid[0, :, 0] = 0                      # empty group
        valid[1, :, -1] = 0
        valid[1, 0, -1] = 1                     # singleton group
    adv, ret, gn = B.trloo_advantage(torch.from_numpy(R).to(dev), torch.from_numpy(valid).to(dev), gamma)
    torch.cuda.synchronize()
    G, A, N = O.trloo_advantage(R, valid, gamma)
    assert np.abs(adv.cpu().numpy() - A).max() <= TOL_ADV
    assert np.abs(ret.cpu().numpy() - G).max() <= TOL_ADV
    assert np.array_equal(gn.cpu().numpy(), N)


# ------------------------------------------------------------------------------------ forward
def _fwd_case(dev, T, d, V, dtype, tau, seed, mask_frac):
    H, W, y = synth.make_head(T, d, V, dtype, seed, dev, unit_rms=(dtype == "bf16"),
                              w_std=0.02 if dtype == "bf16" else 0.1)
    rng = np.random.default_rng(seed)
    mask = None
    if mask_frac > 0:
        mask = (rng.random(T) >= mask_frac).astype(np.uint8)
    prm = B.Params(dtype=0 if dtype == "bf16" else 1, temperature=tau)
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
    tm = None if mask is None else torch.from_numpy(mask).to(dev)
    logp, ent, lse = B.pg_logprob_fwd(H, W, y, tm, prm, ws)
    torch.cuda.synchronize()
    rl, re, rs = O.lm_head_logprob(np64(H), np64(W), y.cpu().numpy(), tau, row_mask=mask)
    return (logp.cpu().numpy(), ent.cpu().numpy(), lse.cpu().numpy()), (rl, re, rs), mask


@pytest.mark.parametrize("T,d,V,tau,mask_frac", [(700, 128, 2500, 1.0, 0.3), (1024, 64, 1000, 1.0, 0.0),
                                                  (513, 320, 5000, 0.7, 0.5), (255, 64, 257, 1.0, 0.0),
                                                  (1, 64, 1, 1.0, 0.0), (300, 64, 300, 2.0, 1.0)])
def test_logprob_fwd_bf16(dev, T, d, V, tau, mask_frac):
    got, ref, mask = _fwd_case(dev, T, d, V, "bf16", tau, 100 + T, mask_frac)
    for g, r in zip(got, ref):
        assert np.abs(g - r).max() <= TOL_LOGP
    if mask is not None:
        for g in got:
            assert np.all(g[mask == 0] == 0)


@pytest.mark.parametrize("T,d,V,tau", [(1024, 64, 1000, 1.0), (300, 128, 777, 0.7)])
def test_logprob_fwd_f32(dev, T, d, V, tau):
    got, ref, _ = _fwd_case(dev, T, d, V, "f32", tau, 7, 0.2)
    for g, r in zip(got, ref):
        assert np.abs(g - r).max() <= 2e-4          # split-bf16 products keep ~16 mantissa bits


def test_logprob_fwd_optional_outputs_and_bad_token(dev):
    T, d, V = 300, 64, 500
    H, W, y = synth.make_head(T, d, V, "bf16", 3, dev)
    y[5] = V + 10                                # out of range: no one-hot hit, log-prob = -lse
    prm = B.Params()
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
    logp, ent, lse = B.pg_logprob_fwd(H, W, y, None, prm, ws, want_entropy=False, want_lse=True)
    torch.cuda.synchronize()
    assert ent is None
    assert abs(float(logp[5]) + float(lse[5])) < 1e-5


def test_peaked_distributions_large_logits(dev):
    """Logits with a standard deviation of about 40 (nearly one-hot softmax, log-probs down to -300, entropies
    near 0): the online maximum must keep every exponent in range, forward and backward."""
    T, d, V = 520, 128, 3000
    H, W, y = synth.make_head(T, d, V, "bf16", 909, dev, unit_rms=True, w_std=3.5)
    Hn, Wn, yn = np64(H), np64(W), y.cpu().numpy()
    z = Hn @ Wn.T
    y[::3] = torch.from_numpy(z.argmax(axis=1)[::3].astype(np.int32)).to(dev)       # a third of the targets are the mode
    yn = y.cpu().numpy()
    assert z.std() > 30
    prm = B.Params(mismatch_mode=0)
    ws = B.alloc_workspace(T, d, V, 1, prm, B.CALL_LOSS_FWD_BWD, dev)
    logp, ent, lse = B.pg_logprob_fwd(H, W, y, None, prm, ws)
    torch.cuda.synchronize()
    rl, re, rs = O.lm_head_logprob(Hn, Wn, yn, 1.0)
    assert rl.min() < -100 and re.min() < 1e-3
    e_logp, e_ent, e_lse = (np.abs(logp.cpu().numpy() - rl).max(), np.abs(ent.cpu().numpy() - re).max(),
                            np.abs(lse.cpu().numpy() - rs).max())
    print(f"[peaked] max|dlogp| {e_logp:.2e} (|logp| up to {np.abs(rl).max():.0f}) max|dentropy| {e_ent:.2e} "
          f"max|dlse| {e_lse:.2e}")
    assert e_logp <= TOL_LOGP and e_ent <= TOL_LOGP and e_lse <= TOL_LOGP
    cu = torch.tensor([0, T], dtype=torch.int32, device=dev)
    adv = torch.tensor([1.5], dtype=torch.float64, device=dev)
    out = B.pg_loss_fwd_bwd(H, W, y, torch.ones(T, dtype=torch.uint8, device=dev), cu, adv, None, None, None, prm, ws)
    torch.cuda.synchronize()
    ref = O.pg_loss_fwd_bwd(Hn, Wn, yn, np.ones(T, np.uint8), np.array([0, T]), [1.5], None, None, O.Params())
    assert torch.isfinite(out["dW"]).all() and torch.isfinite(out["dH"].float()).all()
    assert abs(float(out["loss"][0]) - ref["loss"]) <= TOL_LOSS * abs(ref["loss"])
    assert rel_fro(np64(out["dH"]), ref["dH"]) <= TOL_GRAD and rel_fro(np64(out["dW"]), ref["dW"]) <= TOL_GRAD


def test_non_finite_inputs_propagate_and_stay_local(dev):
    """A NaN or an infinity in the inputs must come out as NaN in what depends on it and nowhere else; no
    kernel takes a data-dependent branch or address from H or W, so the call returns as always."""
    T, d, V = 600, 64, 900
    H, W, y = synth.make_head(T, d, V, "bf16", 17, dev)
    prm = B.Params(mismatch_mode=0)
    ws = B.alloc_workspace(T, d, V, 1, prm, B.CALL_LOSS_FWD_BWD, dev)
    clean = B.pg_logprob_fwd(H, W, y, None, prm, ws)[0].clone()
    Hn = H.clone()
    Hn[7, 3] = float("nan")
    Hn[300, 5] = float("inf")
    logp, ent, lse = B.pg_logprob_fwd(Hn, W, y, None, prm, ws)
    torch.cuda.synchronize()
    bad = torch.zeros(T, dtype=torch.bool, device=dev)
    bad[7] = bad[300] = True
    assert torch.isnan(logp[bad]).all() and torch.isnan(lse[bad]).all()
    assert torch.equal(logp[~bad], clean[~bad])                     # every other row is untouched, bit for bit
    ones = torch.ones(T, dtype=torch.uint8, device=dev)
    cu = torch.tensor([0, T], dtype=torch.int32, device=dev)
    adv = torch.ones(1, dtype=torch.float64, device=dev)
    out = B.pg_loss_fwd_bwd(Hn, W, y, ones, cu, adv, None, clean, None, prm, ws)     # ratio exp(logp - old)
    torch.cuda.synchronize()
    assert torch.isnan(out["loss"]).all() and torch.isnan(out["dH"][7].float()).all()
    ok = out["dH"][~bad].float()
    assert torch.isfinite(ok).all()                                 # other rows' gradients do not see it
    assert int(out["counters"][0]) == T
    # a masked-out row may hold anything: it is never read
    mask = ones.clone()
    mask[7] = mask[300] = 0
    out2 = B.pg_loss_fwd_bwd(Hn, W, y, mask, cu, adv, None, clean, None, prm, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(out2["loss"]).all() and torch.isfinite(out2["dW"]).all() and torch.isfinite(out2["dH"].float()).all()


# ------------------------------------------------------------------------------------ loss fwd + bwd
def _run_loss(dev, spec, prm, mismatch_kind, on_policy, monkeypatch=None, budget_tiles=None, accumulate=False):
    batch, tin, nin = build_loss_case(spec, dev, oracle_logp, mismatch_kind, on_policy)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    if budget_tiles is not None:
        t_cap = (T + 255) // 256 * 256
        monkeypatch.setenv("PG_HEAD_DS_BUDGET_BYTES", str(t_cap * 2 * 256 * budget_tiles))
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    dW = dW_prev = None
    if accumulate:
        g = torch.Generator(device=dev)
        g.manual_seed(5)
        dW = (torch.randn((V, d), generator=g, device=dev) * 1e-3).to(torch.bfloat16 if prm.dW_dtype else torch.float32)
        dW_prev = np64(dW)
    out = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1),
                            tin["seg_sample"], tin["old"], tin["rollout"], prm, ws, dW=dW)
    torch.cuda.synchronize()
    _, A, _ = O.trloo_advantage(nin["rewards"], nin["valid"], 1.0)
    oprm = O.Params(temperature=prm.temperature, clip_eps_lo=prm.clip_eps_lo, clip_eps_hi=prm.clip_eps_hi,
                    mismatch_mode=prm.mismatch_mode, geo_lo=prm.geo_lo, geo_hi=prm.geo_hi,
                    veto_ratio=prm.veto_ratio, trunc_c=prm.trunc_c, norm_override=prm.norm_override)
    ref = O.pg_loss_fwd_bwd(nin["H"], nin["W"], nin["y"], nin["loss_mask"], nin["cu"],
                            A.reshape(-1)[nin["seg_sample"]], nin["old"], nin["rollout"], oprm, dW_prev=dW_prev)
    return out, ref, batch


def _compare(out, ref, logp_tol=TOL_LOGP, grad_tol=TOL_GRAD):
    assert np.array_equal(out["counters"].cpu().numpy(), ref["counters"]), \
        (out["counters"].cpu().numpy(), ref["counters"])
    e_logp = np.abs(out["logp"].cpu().numpy() - ref["logp"]).max()
    e_ent = np.abs(out["entropy"].cpu().numpy() - ref["entropy"]).max()
    loss = float(out["loss"][0])
    e_loss = abs(loss - ref["loss"]) / max(abs(ref["loss"]), 1e-6)
    dH, dW = np64(out["dH"]), np64(out["dW"])
    e_dH, e_dW = rel_fro(dH, ref["dH"]), rel_fro(dW, ref["dW"])
    b_dH, b_dW = block_rel_fro(dH, ref["dH"]), block_rel_fro(dW, ref["dW"])
    # achieved errors (shown with pytest -s, and in the failure report)
    print(f"[parity] logp {e_logp:.2e} entropy {e_ent:.2e} loss(rel) {e_loss:.2e} dH {e_dH:.2e} (worst 256-row block "
          f"{b_dH:.2e}) dW {e_dW:.2e} (worst block {b_dW:.2e})")
    assert e_logp <= logp_tol and e_ent <= logp_tol, (e_logp, e_ent)
    assert e_loss <= TOL_LOSS, (loss, ref["loss"])
    assert np.all(dH[~ref["active"]] == 0)
    assert e_dH <= grad_tol and e_dW <= grad_tol, (e_dH, e_dW)
    # no 256-row block of either gradient may be off by more than the whole-matrix bound either
    assert b_dH <= grad_tol and b_dW <= grad_tol, (b_dH, b_dW)


def test_loss_config0_tiny_f32(dev):
    """The tiny fp32 configuration: d=64, V=1000, 4x4x2 samples of 32 tokens, eps 0.2, tau 1."""
    spec = synth.SPECS[0]
    prm = B.Params(dtype=1, mismatch_mode=0)
    out, ref, batch = _run_loss(dev, spec, prm, "none", on_policy=False)
    assert batch.T == 1024 and batch.S == 32
    # fp32 inputs: every contraction (logits, dW, dH) runs on operands split into a bf16 value and a bf16
    # remainder, dS included, with the product of two remainders dropped: ~2^-16 per product.  Achieved
    # (printed by _compare): log-probs 3e-6 absolute, gradients 4e-6 relative.
    _compare(out, ref, logp_tol=2e-4, grad_tol=5e-5)
    assert ref["counters"][1] > 0 and ref["counters"][2] > 0       # both clip branches occur


@pytest.mark.parametrize("mode,kind", [(0, "none"), (1, "window"), (2, "token")])
@pytest.mark.parametrize("tau", [1.0, 0.7])
def test_loss_small_bf16_modes(dev, monkeypatch, mode, kind, tau):
    """Ragged packed batch spanning several token and vocab tiles, backward in 4 vocab chunks."""
    spec = synth.small_spec(temperature=tau, seed=4321 + mode)
    prm = B.Params(mismatch_mode=mode, temperature=tau)
    out, ref, batch = _run_loss(dev, spec, prm, kind, on_policy=False, monkeypatch=monkeypatch, budget_tiles=3)
    assert batch.T > 1024 and 0 < ref["counters"][0] < batch.T
    if mode == 1:
        assert ref["counters"][3] > 0 and ref["counters"][4] > 0
    if mode == 2:
        assert ref["counters"][5] > 0 and ref["counters"][4] > 0
    _compare(out, ref)


def test_loss_unequal_clip_ranges(dev):
    """eps_lo != eps_hi (ratio clipped to [0.65, 1.05]): both clip counters and the gradients must follow."""
    spec = synth.small_spec(d=64, V=900, seed=98)
    prm = B.Params(clip_eps_lo=0.35, clip_eps_hi=0.05, mismatch_mode=0)
    out, ref, _ = _run_loss(dev, spec, prm, "none", on_policy=False)
    _compare(out, ref)
    # the same inputs under the default symmetric range give different counters
    assert ref["counters"][1] > 0 and ref["counters"][2] > 0
    out_s, ref_s, _ = _run_loss(dev, spec, B.Params(mismatch_mode=0), "none", on_policy=False)
    assert ref["counters"][1] != ref_s["counters"][1] and ref["counters"][2] != ref_s["counters"][2]


def test_loss_non_default_mismatch_parameters(dev):
    """The window, the veto threshold and the truncation cap come from the parameters, not from the paper's
    defaults: a wider, off-centre window keeps a sample the default rejects; a veto threshold of 0 switches
    the veto off; a lower threshold lets the e^-10 token through; a cap of 1.2 truncates more tokens."""
    spec = synth.small_spec(d=64, V=900, seed=4322, P=3, K=5, Tmax=3)
    base, ref_base, _ = _run_loss(dev, spec, B.Params(mismatch_mode=1), "window", on_policy=False)
    prm = B.Params(mismatch_mode=1, geo_lo=0.9965, geo_hi=1.0015, veto_ratio=0.0)
    out, ref, _ = _run_loss(dev, spec, prm, "window", on_policy=False)
    _compare(out, ref)
    assert ref["counters"][4] == 0 and ref_base["counters"][4] == 1                  # veto switched off
    assert 0 < ref["counters"][3] < ref_base["counters"][3]                          # fewer samples outside the window
    assert ref["counters"][0] > ref_base["counters"][0]
    base2, ref_base2, _ = _run_loss(dev, spec, B.Params(mismatch_mode=2), "token", on_policy=False)
    prm2 = B.Params(mismatch_mode=2, trunc_c=1.2, veto_ratio=1e-6)
    out2, ref2, _ = _run_loss(dev, spec, prm2, "token", on_policy=False)
    _compare(out2, ref2)
    assert ref2["counters"][4] == 0 and ref_base2["counters"][4] == 1                # e^-10 = 4.5e-5 is above 1e-6
    assert ref2["counters"][5] > ref_base2["counters"][5] > 0                        # more tokens hit the lower cap


def test_loss_on_policy_no_old_logp(dev):
    spec = synth.small_spec(d=64, V=900, seed=99)
    out, ref, _ = _run_loss(dev, spec, B.Params(), "none", on_policy=True)
    _compare(out, ref)


def test_loss_accumulate_bf16_dW_and_norm_override(dev, monkeypatch):
    spec = synth.small_spec(d=192, V=1300, seed=77)
    prm = B.Params(accumulate_dW=1, dW_dtype=0, norm_override=5000.0)
    out, ref, _ = _run_loss(dev, spec, prm, "none", on_policy=False, monkeypatch=monkeypatch, budget_tiles=2,
                            accumulate=True)
    _compare(out, ref)
    prm = B.Params(accumulate_dW=0, dW_dtype=1)
    out, ref, _ = _run_loss(dev, spec, prm, "none", on_policy=False)
    _compare(out, ref)                            # bf16 dW: rounding 2^-9 per element, inside 1e-2
    prm = B.Params(accumulate_dW=1, dW_dtype=1)   # read-modify-write of a bf16 dW, several chunks
    out, ref, _ = _run_loss(dev, spec, prm, "none", on_policy=False, monkeypatch=monkeypatch, budget_tiles=2,
                            accumulate=True)
    assert out["dW"].dtype == torch.bfloat16
    _compare(out, ref)


def test_loss_f32_multichunk_with_truncation(dev, monkeypatch):
    spec = synth.small_spec(d=64, V=1500, dtype="f32", seed=55, unit_rms=False)
    prm = B.Params(dtype=1, mismatch_mode=2)
    out, ref, _ = _run_loss(dev, spec, prm, "token", on_policy=False, monkeypatch=monkeypatch, budget_tiles=2)
    _compare(out, ref, logp_tol=2e-4, grad_tol=5e-5)


@pytest.mark.parametrize("budget_tiles,d,dtype", [(None, 128, "bf16"), (4, 128, "bf16"), (None, 512, "bf16"), (4, 128, "f32")])
def test_loss_few_active_rows_split_contraction(dev, monkeypatch, budget_tiles, d, dtype):
    """Most samples rejected by the geometric window: the active rows fill a fraction of the padded row
    capacity, so the dH contraction is cut along the vocabulary into parts that accumulate side by side
    (one chunk; several chunks whose last one is too short to be cut; several column tiles; an fp32 head,
    whose parts each add their two remainder terms)."""
    spec = synth.small_spec(seed=8080, d=d, V=4200, P=4, K=6, Tmax=3, len_lo=40, len_hi=120, dtype=dtype,
                            unit_rms=(dtype == "bf16"))
    prm = B.Params(dtype=0 if dtype == "bf16" else 1, mismatch_mode=1)
    out, ref, batch = _run_loss(dev, spec, prm, "window", on_policy=False, monkeypatch=monkeypatch,
                                budget_tiles=budget_tiles)
    n_active = int(ref["counters"][0])
    t_cap = (batch.T + 255) // 256 * 256
    n_pad = (n_active + 255) // 256 * 256
    assert 0 < n_active and 2 * n_pad <= t_cap, (n_active, t_cap)       # room for at least two parts
    if dtype == "bf16":
        _compare(out, ref)
    else:
        _compare(out, ref, logp_tol=2e-4, grad_tol=5e-5)
    out2, _, _ = _run_loss(dev, spec, prm, "window", on_policy=False, monkeypatch=monkeypatch, budget_tiles=budget_tiles)
    assert torch.equal(out["dH"], out2["dH"]) and torch.equal(out["dW"], out2["dW"])      # fixed summation order


@pytest.mark.parametrize("budget_tiles,dtype", [(None, "bf16"), (3, "bf16"), (5, "f32")])
def test_loss_very_few_active_rows(dev, monkeypatch, budget_tiles, dtype):
    """Four samples of 58 kept by their keep flags.  In one vocab chunk the dH contraction runs in its maximum of
    eight parts; planned in several chunks, the rows are so few that the recompute of the whole vocabulary runs in
    the first chunk's launch and dW / dH read the wide layout of dS (bf16 and fp32 heads)."""
    from tests._cases import recompute_covers_vocabulary
    spec = synth.small_spec(seed=8081, d=128, V=4200, P=4, K=6, Tmax=3, len_lo=40, len_hi=120, dtype=dtype,
                            unit_rms=(dtype == "bf16"))
    prm = B.Params(dtype=0 if dtype == "bf16" else 1, mismatch_mode=2)
    batch, tin, nin = build_loss_case(spec, dev, oracle_logp, "token", on_policy=False)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    if budget_tiles is not None:
        monkeypatch.setenv("PG_HEAD_DS_BUDGET_BYTES", str((T + 255) // 256 * 256 * 2 * 256 * budget_tiles))
    keep = np.zeros(spec.P * spec.K * spec.Tmax, np.uint8)
    keep[nin["seg_sample"][[3, 17, 30, 44]]] = 1
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    out = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                            tin["old"], tin["rollout"], prm, ws, sample_keep=torch.from_numpy(keep).to(dev))
    torch.cuda.synchronize()
    _, A, _ = O.trloo_advantage(nin["rewards"], nin["valid"], 1.0)
    ref = O.pg_loss_fwd_bwd(nin["H"], nin["W"], nin["y"], nin["loss_mask"], nin["cu"], A.reshape(-1)[nin["seg_sample"]],
                            nin["old"], nin["rollout"], O.Params(mismatch_mode=2), seg_keep=keep[nin["seg_sample"]])
    n_pad = (int(ref["counters"][0]) + 255) // 256 * 256
    assert 0 < n_pad and 8 * n_pad <= (T + 255) // 256 * 256
    chunk_rows = B.pg_backward_chunk_rows(T, d, V, S, prm)
    if budget_tiles is None:
        assert chunk_rows >= V
    else:
        assert chunk_rows == 256 * budget_tiles and recompute_covers_vocabulary(T, V, n_pad, chunk_rows)
    if dtype == "bf16":
        _compare(out, ref)
    else:
        _compare(out, ref, logp_tol=2e-4, grad_tol=5e-5)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_loss_w_transposed_cache(dev, monkeypatch, dtype):
    """The optional W^T cache: a call that fills it and a call that trusts it give the bits of a call without it
    (several vocab chunks, ragged vocabulary); a stale cache is really what the dH contraction reads.  For an
    fp32 head the cache holds the bf16 values of W^T and the remainders are rebuilt on every call."""
    spec = synth.small_spec(d=192, V=2100, seed=611, dtype=dtype, unit_rms=(dtype == "bf16"))
    dt = 0 if dtype == "bf16" else 1
    batch, tin, nin = build_loss_case(spec, dev, oracle_logp, "token", on_policy=False)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    monkeypatch.setenv("PG_HEAD_DS_BUDGET_BYTES", str((T + 255) // 256 * 256 * 2 * 256 * 3))
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    cache = B.alloc_w_transposed(d, V, dev)
    cache.random_(0, 255)

    def run(prm):
        ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
        out = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1),
                                tin["seg_sample"], tin["old"], tin["rollout"], prm, ws)
        torch.cuda.synchronize()
        return out
    plain = run(B.Params(dtype=dt, mismatch_mode=2))
    fill = run(B.Params(dtype=dt, mismatch_mode=2, w_transposed=cache, w_transposed_valid=0))
    trust = run(B.Params(dtype=dt, mismatch_mode=2, w_transposed=cache, w_transposed_valid=1))
    for k in ("loss", "dH", "dW", "logp", "entropy", "counters"):
        assert torch.equal(fill[k], plain[k]) and torch.equal(trust[k], plain[k]), k
    cache.zero_()                                   # a cache that does not hold W^T: dH = dS 0 = 0, dW untouched
    stale = run(B.Params(dtype=dt, mismatch_mode=2, w_transposed=cache, w_transposed_valid=1))
    assert torch.equal(stale["dW"], plain["dW"])
    if dtype == "bf16":
        assert not stale["dH"].any()
    else:                                           # what is left is dS times the remainders W - bf16(W)
        assert 0 < np.linalg.norm(np64(stale["dH"])) < 2e-2 * np.linalg.norm(np64(plain["dH"]))
    with pytest.raises(ValueError):
        B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                          tin["old"], tin["rollout"], B.Params(dtype=dt, mismatch_mode=2, w_transposed=cache[:64]),
                          B.alloc_workspace(T, d, V, S, B.Params(dtype=dt), B.CALL_LOSS_FWD_BWD, dev))


def test_loss_all_masked_and_all_rejected(dev):
    spec = synth.small_spec(d=64, V=600, seed=31)
    batch, tin, nin = build_loss_case(spec, dev, oracle_logp, "window", on_policy=False)
    T, S = batch.T, batch.S
    adv = torch.ones(batch.P * batch.K * batch.Tmax, dtype=torch.float64, device=dev)
    for prm, mask, roll in ((B.Params(), torch.zeros(T, dtype=torch.uint8, device=dev), tin["rollout"]),
                            (B.Params(mismatch_mode=1), tin["loss_mask"], tin["old"] - 1.0)):
        ws = B.alloc_workspace(T, spec.d, spec.V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
        out = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], mask, tin["cu"], adv, tin["seg_sample"], tin["old"],
                                roll, prm, ws)
        torch.cuda.synchronize()
        assert float(out["loss"][0]) == 0.0
        assert not out["dW"].any() and not out["dH"].any() and not out["logp"].any()
        assert int(out["counters"][0]) == 0


def test_loss_empty_microbatch(dev):
    d, V = 64, 300
    prm = B.Params()
    ws = torch.empty(max(256, B.pg_workspace_bytes(0, d, V, 0, prm, B.CALL_LOSS_FWD_BWD)), dtype=torch.uint8, device=dev)
    H = torch.empty((0, d), dtype=torch.bfloat16, device=dev)
    W = torch.randn((V, d), device=dev).to(torch.bfloat16)
    y = torch.empty(0, dtype=torch.int32, device=dev)
    cu = torch.zeros(1, dtype=torch.int32, device=dev)
    adv = torch.zeros(1, dtype=torch.float64, device=dev)
    dW = torch.full((V, d), 3.0, dtype=torch.float32, device=dev)
    out = B.pg_loss_fwd_bwd(H, W, y, torch.empty(0, dtype=torch.uint8, device=dev), cu, adv, None, None, None, prm,
                            ws, dW=dW)
    torch.cuda.synchronize()
    assert float(out["loss"][0]) == 0.0 and not dW.any() and not out["counters"].any()


def test_repeatable_bitwise(dev):
    """Fixed reduction orders everywhere: two runs give identical bits."""
    spec = synth.small_spec(d=128, V=1100, seed=8)
    a, _, _ = _run_loss(dev, spec, B.Params(mismatch_mode=2), "token", on_policy=False)
    b, _, _ = _run_loss(dev, spec, B.Params(mismatch_mode=2), "token", on_policy=False)
    for k in ("loss", "dH", "dW", "logp", "entropy", "counters"):
        assert torch.equal(a[k], b[k]), k


def test_two_streams_and_two_threads_do_not_interfere(dev):
    """The library keeps no device state between calls: the same step issued on two streams from two host threads
    at once, each with its own workspace and outputs, gives on both the bits of a single call."""
    import threading
    spec = synth.small_spec(d=128, V=2100, seed=9)
    prm = B.Params(mismatch_mode=2)
    batch, tin, _ = build_loss_case(spec, dev, oracle_logp, "token", on_policy=False)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    call = lambda ws, st: B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1),
                                            tin["seg_sample"], tin["old"], tin["rollout"], prm, ws, stream=st)
    ref = call(B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev), None)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)]        # default priority
    wss = [B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev) for _ in streams]
    results, errors = [None, None], []

    def worker(i):
        try:
            torch.cuda.set_device(dev)
            for _ in range(3):
                results[i] = call(wss[i], streams[i])
        except Exception as e:          # surfaced below: a thread must not die silently
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=60)
    torch.cuda.synchronize()
    assert not errors and all(not t.is_alive() for t in threads), errors
    for r in results:
        for k in ("loss", "dH", "dW", "logp", "entropy", "counters"):
            assert torch.equal(r[k], ref[k]), k


def test_hip_graph_replay_matches_eager(dev):
    """The whole step (advantages + loss forward/backward) captured in a HIP graph: the library enqueues
    only kernels on the caller's stream, so a replay must reproduce the eager result bit for bit, also
    after other work has run in between."""
    spec = synth.small_spec(seed=4321)
    batch, tin, nin = build_loss_case(spec, dev, oracle_logp, mismatch_kind="token")
    prm = B.Params(mismatch_mode=2)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    adv = torch.empty((batch.P, batch.K, batch.Tmax), dtype=torch.float64, device=dev)
    dW = torch.empty((V, d), dtype=torch.float32, device=dev)
    outbuf = (torch.empty(1, dtype=torch.float32, device=dev), torch.empty_like(tin["H"]),
              torch.empty(T, dtype=torch.float32, device=dev), torch.empty(T, dtype=torch.float32, device=dev),
              torch.empty(8, dtype=torch.int64, device=dev))

    def step(stream=None):
        B._check(B.lib().trloo_advantage(B._ptr(tin["rewards"]), B._ptr(tin["valid"]), batch.P, batch.K, batch.Tmax, 1.0,
                                         None, B._ptr(adv), None, B._stream(stream)))
        return B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1),
                                 tin["seg_sample"], tin["old"], tin["rollout"], prm, ws, dW=dW, out=outbuf, stream=stream)

    out = step()                                   # eager (also initialises the kernel attributes)
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in out.items()}
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(side)
    for rep in range(3):
        for t in outbuf:
            t.zero_()
        dW.zero_()
        ws.random_(0, 255)                         # the workspace holds nothing between calls
        graph.replay()
        torch.cuda.synchronize()
        for k in ("loss", "dH", "dW", "logp", "entropy", "counters"):
            assert torch.equal(out[k], eager[k]), (rep, k)
        _ = (tin["H"].float() @ tin["W"].float().T).sum()      # unrelated work between replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("seed", list(range(12)))
def test_loss_random_shapes(dev, seed, monkeypatch):
    """Seeded sweep over ragged shapes, modes and parameters (sizes the oracle finishes in a second)."""
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.choice([64, 128, 192, 320, 448]))
    V = int(rng.integers(257, 3500))
    spec = synth.small_spec(name=f"rand{seed}", d=d, V=V, P=int(rng.integers(1, 5)), K=int(rng.integers(2, 7)),
                            Tmax=int(rng.integers(1, 5)), len_lo=int(rng.integers(1, 30)), len_hi=int(rng.integers(30, 140)),
                            ctx_frac=float(rng.choice([0.0, 0.3, 1.0])), dtype=str(rng.choice(["bf16", "bf16", "f32"])),
                            seed=700 + seed, stop_prob=float(rng.choice([0.0, 0.2, 0.5])),
                            temperature=float(rng.choice([1.0, 0.7, 1.3])))
    mode = int(rng.integers(0, 3))
    kind = {0: "none", 1: "window", 2: "token"}[mode]
    prm = B.Params(dtype=0 if spec.dtype == "bf16" else 1, temperature=spec.temperature, mismatch_mode=mode,
                   clip_eps_lo=0.2, clip_eps_hi=0.2, dW_dtype=int(rng.integers(0, 2)),
                   norm_override=float(rng.choice([0.0, 0.0, 777.0])))
    on_policy, budget, accumulate = bool(rng.integers(0, 2)), int(rng.integers(1, 6)), bool(rng.integers(0, 2))
    prm.accumulate_dW = int(accumulate)
    out, ref, batch = _run_loss(dev, spec, prm, kind, on_policy=on_policy, monkeypatch=monkeypatch, budget_tiles=budget,
                                accumulate=accumulate)
    if spec.dtype == "bf16" or prm.dW_dtype:       # (a bf16 dW rounds an fp32 head's gradient like any other)
        _compare(out, ref, TOL_LOGP if spec.dtype == "bf16" else 2e-4)
    else:
        _compare(out, ref, 2e-4, grad_tol=5e-5)
    # the same call with the W^T cache, filled by it and then trusted, gives the same bits
    cache = B.alloc_w_transposed(spec.d, spec.V, dev)
    for valid in (0, 1):
        prm.w_transposed, prm.w_transposed_valid = cache, valid
        again, _, _ = _run_loss(dev, spec, prm, kind, on_policy=on_policy, monkeypatch=monkeypatch, budget_tiles=budget,
                                accumulate=accumulate)
        for k in ("loss", "dH", "dW", "logp", "entropy", "counters"):
            assert torch.equal(again[k], out[k]), (valid, k)
