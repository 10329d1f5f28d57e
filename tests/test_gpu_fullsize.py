"""Parity at the benchmark's full size (Qwen3-14B head, d=5120, V=151936, 32768 loss tokens), in the
launch configuration bench.py times (mismatch mode 2, fp32 dW overwrite, default chunking).

The fp64 oracle cannot run the whole problem in test time, so:
  * per-row outputs (log-prob, entropy, dH rows) are compared with the oracle on sampled rows;
  * every row's log-prob is also compared with a plain library computation (torch fp32 matmul +
    log_softmax on the GPU), which is itself checked against the oracle on the sampled rows;
  * sampled rows of dW are compared with an fp64 evaluation of dS^T H whose logsumexp comes from
    that library computation;
  * size-independent identities: columns of dW sum to zero (rows of dS do), <dW,W> = <dH,H>,
    inactive rows of dH are zero, the loss equals the surrogate formula applied to the log-probs.
Inputs: H, W, y and the batch structure are seeded draws; old_logp is the library log-prob divided
by a policy ratio drawn away from the clip thresholds; rollout_logp adds N(0, 0.1) and 1 % outliers
of +-3.  No input or expected value comes from the HIP path.
"""
import numpy as np
import pytest
import torch

from oracle import pg_oracle as O
from paper_2602_05885_amd import binding as B
from paper_2602_05885_amd import synth
from tests._cases import block_rel_fro, np64, ratio_targets, rel_fro

pytestmark = pytest.mark.gpu

N_ROWS = 48          # sampled token rows
N_VOCAB = 24         # sampled vocab rows of dW


def library_logp_lse(H, W, y, tau, chunk=2048):
    """torch fp32 reference for all rows (library GEMM + log_softmax), chunked over rows."""
    T = H.shape[0]
    Wf = W.float()
    logp = torch.empty(T, dtype=torch.float32, device=H.device)
    lse = torch.empty_like(logp)
    for a in range(0, T, chunk):
        z = (H[a:a + chunk].float() @ Wf.T) / tau
        l = torch.logsumexp(z, dim=1)
        logp[a:a + chunk] = z.gather(1, y[a:a + chunk].long()[:, None])[:, 0] - l
        lse[a:a + chunk] = l
    return logp, lse


@pytest.fixture(scope="module")
def full_case():
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    spec = synth.SPECS[2]
    batch = synth.make_batch(spec)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    print(f"[fullsize] T={T} S={S} d={d} V={V}", flush=True)
    H, W, y = synth.make_head(T, d, V, spec.dtype, spec.seed, dev, spec.unit_rms)
    lib_logp, lib_lse = library_logp_lse(H, W, y, spec.temperature)
    r = ratio_targets(T, spec.seed)
    old = (lib_logp.double().cpu().numpy() - np.log(r)).astype(np.float32)
    old_t = torch.from_numpy(old).to(dev)
    rollout_t = synth.perturb_logp(old_t, spec.logp_noise, spec.outlier_frac, spec.seed + 1)
    tin = dict(H=H, W=W, y=y, loss_mask=torch.from_numpy(batch.loss_mask).to(dev),
               cu=torch.from_numpy(batch.cu_seqlens).to(dev), seg_sample=torch.from_numpy(batch.seg_sample).to(dev),
               rewards=torch.from_numpy(batch.rewards).to(dev), valid=torch.from_numpy(batch.valid).to(dev),
               old=old_t, rollout=rollout_t)
    prm = B.Params(mismatch_mode=2, temperature=spec.temperature)
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    print("[fullsize] launching pg_loss_fwd_bwd", flush=True)
    out = B.pg_loss_fwd_bwd(H, W, y, tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"], old_t, rollout_t,
                            prm, ws)
    torch.cuda.synchronize()
    del ws
    print("[fullsize] GPU done; oracle on sampled rows", flush=True)

    # ---- oracle side (fp64, sampled) ----
    oprm = O.Params(mismatch_mode=2, temperature=spec.temperature)
    _, A, _ = O.trloo_advantage(batch.rewards, batch.valid, 1.0)
    adv_seg = A.reshape(-1)[batch.seg_sample]
    rollout = rollout_t.cpu().numpy()
    c, active, keep, mm = O.mismatch_weights(old, rollout, batch.loss_mask, batch.cu_seqlens, oprm)
    norm = float(max(1, int(active.sum())))
    A_tok = np.zeros(T)
    for s in range(S):
        A_tok[batch.cu_seqlens[s]:batch.cu_seqlens[s + 1]] = adv_seg[s]
    rng = np.random.default_rng(2)
    rows = np.sort(rng.choice(np.nonzero(active)[0], N_ROWS, replace=False))
    Wn = np64(W)
    Hr = np64(H[torch.from_numpy(rows).to(dev)])
    yn = y.cpu().numpy().astype(np.int64)
    o_logp, o_ent, o_lse = O.lm_head_logprob(Hr, Wn, yn[rows], spec.temperature)
    return dict(spec=spec, batch=batch, tin=tin, out=out, adv=adv, A=A, c=c, active=active, norm=norm, A_tok=A_tok,
                rows=rows, Wn=Wn, Hr=Hr, yn=yn, o_logp=o_logp, o_ent=o_ent, o_lse=o_lse, lib_logp=lib_logp,
                lib_lse=lib_lse, old=old, mm=mm, oprm=oprm)


def test_full_advantages(full_case):
    assert np.abs(full_case["adv"].cpu().numpy() - full_case["A"]).max() <= 1e-6


def test_full_logprob_rows(full_case):
    fc = full_case
    rows = fc["rows"]
    # the library reference agrees with the oracle where the oracle can be evaluated
    assert np.abs(fc["lib_logp"].cpu().numpy()[rows] - fc["o_logp"]).max() <= 2e-4
    got = fc["out"]["logp"].cpu().numpy()
    assert np.abs(got[rows] - fc["o_logp"]).max() <= 2e-3
    assert np.abs(fc["out"]["entropy"].cpu().numpy()[rows] - fc["o_ent"]).max() <= 2e-3
    # every active row against the library reference; inactive rows are zero
    act = fc["active"]
    assert np.abs(got[act] - fc["lib_logp"].cpu().numpy()[act]).max() <= 2e-3
    assert np.all(got[~act] == 0)


def test_full_counters_and_loss(full_case):
    fc = full_case
    cnt = fc["out"]["counters"].cpu().numpy()
    assert cnt[0] == fc["active"].sum() and cnt[6] == fc["batch"].loss_mask.sum()
    assert cnt[4] == fc["mm"]["veto"] and cnt[5] == fc["mm"]["trunc"] and cnt[3] == 0
    # the loss is the surrogate formula over all active rows; evaluate it in fp64 on the library
    # log-probs (verified above on sampled rows), and check the clip counters the same way
    act = fc["active"]
    lp = fc["lib_logp"].double().cpu().numpy()
    l, g, r, chi, clo = O.surrogate(lp[act], fc["old"].astype(np.float64)[act], fc["A_tok"][act], fc["oprm"])
    ref_loss = float((fc["c"][act] * l).sum() / fc["norm"])
    loss = float(fc["out"]["loss"][0])
    assert abs(loss - ref_loss) <= 1e-3 * abs(ref_loss), (loss, ref_loss)
    assert cnt[1] == chi.sum() and cnt[2] == clo.sum()
    assert chi.sum() > 1000 and clo.sum() > 1000


def test_full_dH_rows(full_case):
    fc = full_case
    rows = fc["rows"]
    l, g, r, _, _ = O.surrogate(fc["o_logp"], fc["old"].astype(np.float64)[rows], fc["A_tok"][rows], fc["oprm"])
    coef = fc["c"][rows] * g / fc["norm"]
    ref = O.dH_rows(fc["Hr"], fc["Wn"], fc["yn"][rows], coef, fc["spec"].temperature)
    dev = fc["out"]["dH"].device
    got = np64(fc["out"]["dH"][torch.from_numpy(rows).to(dev)])
    assert rel_fro(got, ref) <= 1e-2, rel_fro(got, ref)
    inactive = torch.from_numpy(np.nonzero(~fc["active"])[0]).to(dev)
    assert not fc["out"]["dH"][inactive].any()


def test_full_dW_sampled_rows_and_identities(full_case):
    fc = full_case
    act = np.nonzero(fc["active"])[0]
    dev = fc["out"]["dW"].device
    spec = fc["spec"]
    tau = float(np.float32(spec.temperature))
    rng = np.random.default_rng(3)
    # half of the sampled vocab rows are tokens that occur as targets (one-hot term present)
    vs = np.unique(np.concatenate([rng.choice(fc["yn"][act], N_VOCAB // 2), rng.integers(0, spec.V, N_VOCAB // 2),
                                   [spec.V - 1, 0]]))
    Ha = np64(fc["tin"]["H"][torch.from_numpy(act).to(dev)])                  # [T_a, d] fp64
    lp = fc["lib_logp"].double().cpu().numpy()[act]
    lse = fc["lib_lse"].double().cpu().numpy()[act]
    l, g, r, _, _ = O.surrogate(lp, fc["old"].astype(np.float64)[act], fc["A_tok"][act], fc["oprm"])
    k = fc["c"][act] * g / fc["norm"] / tau
    z = (Ha @ fc["Wn"][vs].T) / tau                                          # [T_a, n_v]
    dS = -np.exp(z - lse[:, None]) * k[:, None]
    onehot = (fc["yn"][act][:, None] == vs[None, :])
    dS += onehot * k[:, None]
    ref = dS.T @ Ha
    got = np64(fc["out"]["dW"][torch.from_numpy(vs).to(dev)])
    assert rel_fro(got, ref) <= 1e-2, rel_fro(got, ref)
    # identities that hold at any size
    dW = fc["out"]["dW"]
    dH = fc["out"]["dH"]
    col = dW.double().sum(dim=0)
    scale = dW.double().abs().sum(dim=0)
    assert float((col.abs() / scale).max()) < 2e-3          # rows of dS sum to zero (up to bf16 rounding of dS)
    lhs = float((dW.double() * fc["tin"]["W"].double()).sum())
    rhs = float((dH.double() * fc["tin"]["H"].double()).sum())
    assert abs(lhs - rhs) <= 1e-2 * max(abs(lhs), abs(rhs)), (lhs, rhs)


def _library_gradients(H, W, y, act_rows, lse_a, k_a, tau, T, vocab_step=4096):
    """torch fp32 reference for ALL of dW and dH (library GEMMs, chunked over the vocabulary): for a vocab
    slice, z = H_a W_s^T / tau, dS = k (onehot - exp(z - lse)), dW_s = dS^T H_a, dH_a += dS W_s."""
    dev = H.device
    Ha = H[act_rows].float()
    ya = y[act_rows].long()
    V, d = W.shape
    dW = torch.empty((V, d), dtype=torch.float32, device=dev)
    dHa = torch.zeros((Ha.shape[0], d), dtype=torch.float32, device=dev)
    for a in range(0, V, vocab_step):
        Ws = W[a:a + vocab_step].float()
        dS = torch.exp((Ha @ Ws.T) / tau - lse_a[:, None]).mul_(-k_a[:, None])
        hit = (ya >= a) & (ya < a + Ws.shape[0])
        idx = torch.nonzero(hit)[:, 0]
        dS[idx, ya[idx] - a] += k_a[idx]
        dW[a:a + Ws.shape[0]] = dS.T @ Ha
        dHa += dS @ Ws
    dH = torch.zeros((T, d), dtype=torch.float32, device=dev)
    dH[act_rows] = dHa
    return dW, dH


def test_full_all_rows_against_library_gradients(full_case):
    """Every row of dW and dH at the benchmark's size against a torch fp32 computation (library GEMMs), in
    blocks of 256 rows - a misplaced or wrong MFMA tile cannot hide in a block - with the library result
    itself checked against fp64 on sampled rows, among them the first and last vocabulary row of every
    backward chunk (where one launch's tiles end and the next one's begin)."""
    fc = full_case
    tin, spec, batch = fc["tin"], fc["spec"], fc["batch"]
    dev = tin["H"].device
    T, d, V, S = tin["H"].shape[0], spec.d, spec.V, batch.S
    tau = float(np.float32(spec.temperature))
    act = np.nonzero(fc["active"])[0]
    act_t = torch.from_numpy(act).to(dev)
    lp = fc["lib_logp"].double().cpu().numpy()[act]
    _, g, _, _, _ = O.surrogate(lp, fc["old"].astype(np.float64)[act], fc["A_tok"][act], fc["oprm"])
    k = fc["c"][act] * g / fc["norm"] / tau                                   # fp64 coefficients
    k_t = torch.from_numpy(k.astype(np.float32)).to(dev)
    lib_dW, lib_dH = _library_gradients(tin["H"], tin["W"], tin["y"], act_t, fc["lib_lse"][act_t], k_t, tau, T)
    torch.cuda.synchronize()

    # chunk boundaries of the launch configuration under test
    prm = B.Params(mismatch_mode=2, temperature=spec.temperature)
    vc = B.pg_backward_chunk_rows(T, d, V, S, prm)
    assert 0 < vc < V and vc % 256 == 0, vc
    edges = sorted({v for c in range((V + vc - 1) // vc) for v in (c * vc, min(V, (c + 1) * vc) - 1)})
    print(f"[fullsize] backward chunks of {vc} vocabulary rows; boundary rows {edges}", flush=True)
    assert len(edges) >= 4

    # the library reference against fp64 on the chunk-boundary rows and a few more
    rng = np.random.default_rng(11)
    vs = np.unique(np.concatenate([edges, rng.choice(fc["yn"][act], 6), rng.integers(0, V, 6)]))
    Ha = np64(tin["H"][act_t])
    lse = fc["lib_lse"].double().cpu().numpy()[act]
    z = (Ha @ fc["Wn"][vs].T) / tau
    dS = -np.exp(z - lse[:, None]) * k[:, None] + (fc["yn"][act][:, None] == vs[None, :]) * k[:, None]
    ref_rows = dS.T @ Ha
    vs_t = torch.from_numpy(vs).to(dev)
    e_lib = rel_fro(np64(lib_dW[vs_t]), ref_rows)
    e_got = max(rel_fro(np64(fc["out"]["dW"][v:v + 1]), ref_rows[i:i + 1]) for i, v in enumerate(vs))
    print(f"[fullsize] dW rows vs fp64: library {e_lib:.2e}, kernels (worst single row of {len(vs)}) {e_got:.2e}", flush=True)
    assert e_lib <= 1e-4, e_lib
    assert e_got <= 1e-2, e_got
    rows = fc["rows"]
    l, g_r, r, _, _ = O.surrogate(fc["o_logp"], fc["old"].astype(np.float64)[rows], fc["A_tok"][rows], fc["oprm"])
    ref_dH = O.dH_rows(fc["Hr"], fc["Wn"], fc["yn"][rows], fc["c"][rows] * g_r / fc["norm"], spec.temperature)
    e_lib_h = rel_fro(np64(lib_dH[torch.from_numpy(rows).to(dev)]), ref_dH)
    assert e_lib_h <= 2e-4, e_lib_h           # the library side uses fp32 log-probs for the coefficients

    # all rows, block by block
    got_dW, got_dH = fc["out"]["dW"], fc["out"]["dH"].float()
    def blocks(a, b):
        n = (a.shape[0] + 255) // 256 * 256
        pad = lambda t: torch.nn.functional.pad(t, (0, 0, 0, n - t.shape[0])).reshape(n // 256, -1)
        err = (pad(a) - pad(b)).double().norm(dim=1)
        den = pad(b).double().norm(dim=1)
        return (err / torch.clamp(den, min=1e-3 * float(den.mean()))).cpu().numpy(), float((pad(a) - pad(b)).double().norm() / pad(b).double().norm())
    bw, ew = blocks(got_dW, lib_dW)
    bh, eh = blocks(got_dH, lib_dH)
    print(f"[fullsize] all rows vs library fp32: dW {ew:.2e} (worst of {len(bw)} blocks {bw.max():.2e} at block {int(bw.argmax())}), "
          f"dH {eh:.2e} (worst of {len(bh)} blocks {bh.max():.2e})", flush=True)
    assert ew <= 1e-2 and eh <= 1e-2
    assert bw.max() <= 1e-2 and bh.max() <= 1e-2
    del lib_dW, lib_dH


def dh_split_parts(n_pad, t_cap, tiles_n, k_stages):
    """The device's choice of how many parts the dH contraction is cut into (restated from the header's
    description: enough parts to fill 256 compute units, at most 8, at least 8 stages each, and the parts'
    accumulator slabs must fit into the [t_cap, d] accumulator)."""
    if n_pad <= 0:
        return 1
    tiles = (n_pad // 256) * tiles_n
    ks = 256 // max(tiles, 1)
    ks = min(ks, t_cap // n_pad, k_stages // 8, 8)
    return max(ks, 1)


def test_full_geometric_rejection_few_rows_split_contraction(full_case):
    """Sec. 5.1's rule at the benchmark's size with most samples rejected: two samples' log-ratios sit inside
    [0.999, 1.001] by construction, all others 5e-3 outside, so about 1.3 k of 32768 loss tokens stay active
    and the dH contraction runs cut into parts along the vocabulary (asserted from the counters)."""
    fc = full_case
    tin, spec, batch = fc["tin"], fc["spec"], fc["batch"]
    dev = tin["H"].device
    T, d, V, S = tin["H"].shape[0], spec.d, spec.V, batch.S
    tau = float(np.float32(spec.temperature))
    seg_loss = np.array([batch.loss_mask[batch.cu_seqlens[s]:batch.cu_seqlens[s + 1]].sum() for s in range(S)])
    seg_adv = np.array([fc["A_tok"][batch.cu_seqlens[s]] for s in range(S)])
    cand = [s for s in range(S) if abs(seg_adv[s]) > 0.1 and seg_loss[s] > 128]      # samples that carry a gradient
    keep_segs = next([a, b] for i, a in enumerate(cand) for b in cand[i + 1:] if 1024 < seg_loss[a] + seg_loss[b] <= 1536)
    assert seg_adv[keep_segs[0]] != seg_adv[keep_segs[1]]
    rng = np.random.default_rng(77)
    delta = np.empty(T)
    for s in range(S):
        a, b = batch.cu_seqlens[s], batch.cu_seqlens[s + 1]
        delta[a:b] = (2e-4 if s in keep_segs else 5e-3) + rng.uniform(-1e-5, 1e-5, b - a)
    rollout = (fc["old"].astype(np.float64) - delta).astype(np.float32)
    rollout_t = torch.from_numpy(rollout).to(dev)
    prm = B.Params(mismatch_mode=1, temperature=spec.temperature)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    out = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], fc["adv"].reshape(-1),
                            tin["seg_sample"], tin["old"], rollout_t, prm, ws)
    torch.cuda.synchronize()
    del ws
    oprm = O.Params(mismatch_mode=1, temperature=spec.temperature)
    c, active, keep, mm = O.mismatch_weights(fc["old"], rollout, batch.loss_mask, batch.cu_seqlens, oprm)
    cnt = out["counters"].cpu().numpy()
    n_act = int(active.sum())
    assert cnt[0] == n_act == seg_loss[keep_segs].sum() and cnt[6] == batch.loss_mask.sum()
    assert cnt[3] == mm["geo"] == S - 2 and cnt[4] == mm["veto"] == 0 and cnt[5] == 0
    # the launch really is the split one
    vc = B.pg_backward_chunk_rows(T, d, V, S, prm)
    t_cap, n_pad = (T + 255) // 256 * 256, (n_act + 255) // 256 * 256
    parts = dh_split_parts(n_pad, t_cap, (d + 255) // 256, vc // 64)
    print(f"[fullsize] geometric rejection keeps {n_act} rows (padded {n_pad}): dH contraction in {parts} parts", flush=True)
    assert parts >= 2
    # ... and the recompute of the whole vocabulary runs in the first chunk's launch
    from tests._cases import recompute_covers_vocabulary
    assert vc < V and recompute_covers_vocabulary(T, V, n_pad, vc)
    # per-row outputs against the oracle on sampled active rows; inactive rows are zero
    act = np.nonzero(active)[0]
    rows = np.sort(rng.choice(act, 24, replace=False))
    Hr = np64(tin["H"][torch.from_numpy(rows).to(dev)])
    o_logp, o_ent, _ = O.lm_head_logprob(Hr, fc["Wn"], fc["yn"][rows], spec.temperature)
    got_lp, got_ent = out["logp"].cpu().numpy(), out["entropy"].cpu().numpy()
    assert np.abs(got_lp[rows] - o_logp).max() <= 2e-3 and np.abs(got_ent[rows] - o_ent).max() <= 2e-3
    assert np.all(got_lp[~active] == 0) and np.abs(got_lp[act] - fc["lib_logp"].cpu().numpy()[act]).max() <= 2e-3
    norm = float(max(1, n_act))
    l, g, r, chi, clo = O.surrogate(fc["lib_logp"].double().cpu().numpy()[act], fc["old"].astype(np.float64)[act],
                                    fc["A_tok"][act], oprm)
    ref_loss = float(l.sum() / norm)
    assert abs(ref_loss) > 1e-3 and abs(float(out["loss"][0]) - ref_loss) <= 1e-3 * abs(ref_loss), (float(out["loss"][0]), ref_loss)
    assert cnt[1] == chi.sum() and cnt[2] == clo.sum()
    l_r, g_r, _, _, _ = O.surrogate(o_logp, fc["old"].astype(np.float64)[rows], fc["A_tok"][rows], oprm)
    ref_dH = O.dH_rows(Hr, fc["Wn"], fc["yn"][rows], g_r / norm, spec.temperature)
    got_dH = np64(out["dH"][torch.from_numpy(rows).to(dev)])
    assert rel_fro(got_dH, ref_dH) <= 1e-2, rel_fro(got_dH, ref_dH)
    assert not out["dH"][torch.from_numpy(np.nonzero(~active)[0]).to(dev)].any()
    # sampled dW rows in fp64 over all active rows (chunk boundaries included)
    edges = [0, vc - 1, vc, V - 1]
    vs = np.unique(np.concatenate([edges, rng.choice(fc["yn"][act], 8), rng.integers(0, V, 8)]))
    Ha = np64(tin["H"][torch.from_numpy(act).to(dev)])
    lse = fc["lib_lse"].double().cpu().numpy()[act]
    k = g / norm / tau
    z = (Ha @ fc["Wn"][vs].T) / tau
    dS = -np.exp(z - lse[:, None]) * k[:, None] + (fc["yn"][act][:, None] == vs[None, :]) * k[:, None]
    got_w = np64(out["dW"][torch.from_numpy(vs).to(dev)])
    assert rel_fro(got_w, dS.T @ Ha) <= 1e-2, rel_fro(got_w, dS.T @ Ha)
    # all of dW and dH, block by block, against the library gradients for this active set
    act_t = torch.from_numpy(act).to(dev)
    lib_dW, lib_dH = _library_gradients(tin["H"], tin["W"], tin["y"], act_t, fc["lib_lse"][act_t],
                                        torch.from_numpy(k.astype(np.float32)).to(dev), tau, T)
    assert block_rel_fro(np64(out["dH"]), np64(lib_dH)) <= 1e-2
    e = float((out["dW"] - lib_dW).double().norm() / lib_dW.double().norm())
    assert e <= 1e-2, e


def test_full_logprob_fwd_call(full_case):
    """The forward-only entry point at the same size, all loss rows, against the library reference
    and the oracle's sampled rows."""
    fc = full_case
    tin, spec = fc["tin"], fc["spec"]
    T = tin["H"].shape[0]
    prm = B.Params(temperature=spec.temperature)
    ws = B.alloc_workspace(T, spec.d, spec.V, 0, prm, B.CALL_LOGPROB_FWD, tin["H"].device)
    logp, ent, lse = B.pg_logprob_fwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], prm, ws)
    torch.cuda.synchronize()
    m = fc["batch"].loss_mask.astype(bool)
    assert np.abs(logp.cpu().numpy()[m] - fc["lib_logp"].cpu().numpy()[m]).max() <= 2e-3
    assert np.abs(lse.cpu().numpy()[m] - fc["lib_lse"].cpu().numpy()[m]).max() <= 2e-3
    rows = fc["rows"]
    assert np.abs(lse.cpu().numpy()[rows] - fc["o_lse"]).max() <= 2e-3
    assert np.abs(ent.cpu().numpy()[rows] - fc["o_ent"]).max() <= 2e-3
    assert not logp[torch.from_numpy(~m).to(logp.device)].any()


def test_full_sft_and_monitors(full_case):
    """The SFT cross-entropy entry point (Sec. 3.3) at the same size and launch configuration, and the
    monitors (Sec. 5.1) on its outputs: loss against the library log-probs, sampled dH and dW rows
    against fp64 evaluations, norms against fp64 reductions of the same outputs."""
    fc = full_case
    tin, spec = fc["tin"], fc["spec"]
    dev = tin["H"].device
    T = tin["H"].shape[0]
    tau = float(np.float32(spec.temperature))
    prm = B.Params(temperature=spec.temperature)
    ws = B.alloc_workspace(T, spec.d, spec.V, 0, prm, B.CALL_LOSS_FWD_BWD, dev)
    out = B.pg_sft_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], prm, ws)
    torch.cuda.synchronize()
    del ws
    m = fc["batch"].loss_mask.astype(bool)
    n = int(m.sum())
    lp = fc["lib_logp"].double().cpu().numpy()
    ref_loss = float(-lp[m].sum() / n)
    assert abs(float(out["loss"][0]) - ref_loss) <= 1e-3 * abs(ref_loss)
    cnt = out["counters"].cpu().numpy()
    assert cnt[0] == n and cnt[6] == n
    # sampled rows of dH: coefficient -1/n on every loss row (fc["rows"] are loss rows)
    rows = fc["rows"]
    ref = O.dH_rows(fc["Hr"], fc["Wn"], fc["yn"][rows], np.full(len(rows), -1.0 / n), spec.temperature)
    got = np64(out["dH"][torch.from_numpy(rows).to(dev)])
    assert rel_fro(got, ref) <= 1e-2, rel_fro(got, ref)
    assert not out["dH"][torch.from_numpy(np.nonzero(~m)[0]).to(dev)].any()
    # sampled vocab rows of dW
    act = np.nonzero(m)[0]
    rng = np.random.default_rng(5)
    vs = np.unique(np.concatenate([rng.choice(fc["yn"][act], N_VOCAB // 2), rng.integers(0, spec.V, N_VOCAB // 2),
                                   [spec.V - 1, 0]]))
    Ha = np64(tin["H"][torch.from_numpy(act).to(dev)])
    lse = fc["lib_lse"].double().cpu().numpy()[act]
    k = -1.0 / n / tau
    z = (Ha @ fc["Wn"][vs].T) / tau
    dS = -np.exp(z - lse[:, None]) * k
    dS += (fc["yn"][act][:, None] == vs[None, :]) * k
    got = np64(out["dW"][torch.from_numpy(vs).to(dev)])
    assert rel_fro(got, dS.T @ Ha) <= 1e-2
    # monitors on these outputs
    mon = B.pg_monitors(out["logp"], fc["lib_logp"], out["entropy"], tin["loss_mask"], out["dH"], out["dW"])
    torch.cuda.synchronize()
    g = dict(zip(B.MONITOR_NAMES, mon.cpu().numpy()[:6]))
    mt = torch.from_numpy(m).to(dev)
    assert int(g["n"]) == n
    assert abs(g["dW_norm"] - float(out["dW"].double().pow(2).sum().sqrt())) <= 1e-9 * g["dW_norm"]
    assert abs(g["dH_norm"] - float(out["dH"].double().pow(2).sum().sqrt())) <= 1e-9 * g["dH_norm"]
    assert abs(g["ppl_train"] - float(torch.exp(-out["logp"].double()[mt].sum() / n))) <= 1e-9 * g["ppl_train"]
    assert abs(g["ppl_rollout"] - float(np.exp(-lp[m].sum() / n))) <= 1e-6 * g["ppl_rollout"]
    assert abs(g["entropy_mean"] - float(out["entropy"].double()[mt].sum() / n)) <= 1e-9 * g["entropy_mean"]
    assert abs(np.log(g["ppl_train"]) - ref_loss) <= 1e-3 * abs(ref_loss)          # perplexity = exp(cross-entropy)


def test_full_vocab_shards(full_case):
    """The head split in two vocab shards of 75968 rows (not a multiple of the 256-row tile), each at the
    full token count: merged forward states against the library reference and the oracle's sampled
    rows; each shard's dH term on sampled rows and dW on sampled vocab rows against fp64; the two dH
    terms together and the two dW blocks against the unsharded call."""
    fc = full_case
    tin, spec, batch = fc["tin"], fc["spec"], fc["batch"]
    dev = tin["H"].device
    T, d, V, S = tin["H"].shape[0], spec.d, spec.V, batch.S
    tau = float(np.float32(spec.temperature))
    prm = B.Params(mismatch_mode=2, temperature=spec.temperature)
    half = V // 2
    shards = [(0, half), (half, V)]
    parts = []
    for a, b in shards:
        ws = B.alloc_workspace(T, d, b - a, 0, prm, B.CALL_LOGPROB_FWD, dev)
        parts.append(B.pg_head_shard_fwd(tin["H"], tin["W"][a:b], tin["y"], tin["loss_mask"], a, prm, ws))
        torch.cuda.synchronize()
        del ws
    merged = B.pg_head_partials_merge(parts[0], parts[1])
    torch.cuda.synchronize()
    logp, ent, lse = O.finish_shard_partials(merged.cpu().numpy())
    m = batch.loss_mask.astype(bool)
    rows = fc["rows"]
    assert np.abs(logp[m] - fc["lib_logp"].cpu().numpy()[m]).max() <= 2e-3
    assert np.abs(lse[m] - fc["lib_lse"].cpu().numpy()[m]).max() <= 2e-3
    assert np.abs(logp[rows] - fc["o_logp"]).max() <= 2e-3 and np.abs(ent[rows] - fc["o_ent"]).max() <= 2e-3
    assert not merged[torch.from_numpy(~m).to(dev)].any()
    owner = (parts[0][:, 3] != 0).cpu().numpy().astype(int) + (parts[1][:, 3] != 0).cpu().numpy().astype(int)
    assert np.all(owner[m] <= 1) and owner[m].mean() > 0.999          # a logit of exactly 0 is possible, not likely

    # oracle on the sampled rows as a sub-problem: one-token segments carrying the full problem's
    # advantage, weights and normaliser (the sampled rows are active, so none of them is vetoed)
    n_r = len(rows)
    rollout = tin["rollout"].cpu().numpy()
    sub_prm = O.Params(mismatch_mode=2, temperature=spec.temperature, norm_override=fc["norm"])
    act = np.nonzero(fc["active"])[0]
    Ha = np64(tin["H"][torch.from_numpy(act).to(dev)])
    lp_a = fc["lib_logp"].double().cpu().numpy()[act]
    lse_a = fc["lib_lse"].double().cpu().numpy()[act]
    _, g, _, _, _ = O.surrogate(lp_a, fc["old"].astype(np.float64)[act], fc["A_tok"][act], fc["oprm"])
    k = fc["c"][act] * g / fc["norm"] / tau
    rng = np.random.default_rng(9)
    dH_sum = None
    ws = B.alloc_workspace(T, d, V - half, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    for a, b in shards:
        out = B.pg_loss_shard_bwd(tin["H"], tin["W"][a:b], tin["y"], tin["loss_mask"], tin["cu"], fc["adv"].reshape(-1),
                                  tin["seg_sample"], tin["old"], tin["rollout"], merged, a, prm, ws, dH_f32=True)
        torch.cuda.synchronize()
        assert torch.equal(out["counters"], fc["out"]["counters"])
        assert abs(float(out["loss"][0]) - float(fc["out"]["loss"][0])) <= 1e-5 * abs(float(fc["out"]["loss"][0]))
        assert (out["logp"] - fc["out"]["logp"]).abs().max().item() <= 1e-4
        ref = O.pg_loss_fwd_bwd(fc["Hr"], fc["Wn"], fc["yn"][rows], np.ones(n_r, np.uint8), np.arange(n_r + 1),
                                fc["A_tok"][rows], fc["old"][rows], rollout[rows], sub_prm, vocab_slice=(a, b))
        got = np64(out["dH"][torch.from_numpy(rows).to(dev)])
        assert rel_fro(got, ref["dH"]) <= 1e-2, ((a, b), rel_fro(got, ref["dH"]))
        # sampled vocab rows of this shard's dW (fp64 dS^T H over all active rows, logsumexp from the library reference)
        vs = np.unique(np.concatenate([rng.choice(fc["yn"][act][(fc["yn"][act] >= a) & (fc["yn"][act] < b)], N_VOCAB // 2),
                                       rng.integers(a, b, N_VOCAB // 2), [a, b - 1]]))
        z = (Ha @ fc["Wn"][vs].T) / tau
        dS = -np.exp(z - lse_a[:, None]) * k[:, None] + (fc["yn"][act][:, None] == vs[None, :]) * k[:, None]
        got_w = np64(out["dW"][torch.from_numpy(vs - a).to(dev)])
        assert rel_fro(got_w, dS.T @ Ha) <= 1e-2, ((a, b), rel_fro(got_w, dS.T @ Ha))
        # against the unsharded call (same kernels; the states crossed the boundary in natural-log units)
        blk = fc["out"]["dW"][a:b]
        assert float((out["dW"] - blk).double().norm() / blk.double().norm()) <= 2e-3
        dH_sum = out["dH"].double() if dH_sum is None else dH_sum + out["dH"].double()
        del out
    full = fc["out"]["dH"].double()
    assert float((dH_sum - full).norm() / full.norm()) <= 1e-2
