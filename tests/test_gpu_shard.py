"""Parity of the vocab-sharded head with the fp64 oracle, through the C ABI: every shard's softmax
state, the merge operator, and each shard's loss / dW rows / dH term, for ragged shard sizes, both
dtypes and every mismatch mode; the shards together must also reproduce the unsharded call."""
import numpy as np
import pytest
import torch

from oracle import pg_oracle as O
from paper_2602_05885_amd import binding as B
from paper_2602_05885_amd import synth
from tests._cases import build_loss_case, np64, rel_fro

pytestmark = pytest.mark.gpu

TOL_LOGP, TOL_LOSS, TOL_GRAD = 2e-3, 1e-3, 1e-2


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


def oracle_logp(Hn, Wn, yn, tau):
    return O.lm_head_logprob(Hn, Wn, yn, tau)[0]


def _edges(V, cuts):
    e = [0] + list(cuts) + [V]
    return list(zip(e[:-1], e[1:]))


def _check_partials(got, ref, tol):
    """m and z_y to the log-prob tolerance; s and u relative to the size of s."""
    assert np.abs(got[:, 0] - ref[:, 0]).max() <= tol
    assert np.abs(got[:, 3] - ref[:, 3]).max() <= tol
    scale = np.maximum(ref[:, 1], 1.0)
    assert (np.abs(got[:, 1] - ref[:, 1]) / scale).max() <= 2 * tol
    assert (np.abs(got[:, 2] - ref[:, 2]) / (scale * np.maximum(1.0, np.abs(ref[:, 2]) / scale))).max() <= 4 * tol


@pytest.mark.parametrize("T,d,V,dtype,tau,cuts,mask_frac,seed", [
    (700, 128, 2500, "bf16", 1.0, (1000,), 0.3, 31),            # two ragged shards
    (513, 64, 1000, "bf16", 0.7, (1, 300, 999), 0.0, 32),       # one-row shards at both ends
    (300, 64, 777, "f32", 1.0, (256, 512), 0.2, 33),            # shards that are whole tiles
])
def test_shard_forward_states_and_merge(dev, T, d, V, dtype, tau, cuts, mask_frac, seed):
    H, W, y = synth.make_head(T, d, V, dtype, seed, dev, unit_rms=(dtype == "bf16"),
                              w_std=0.05 if dtype == "bf16" else 0.1)
    rng = np.random.default_rng(seed)
    mask = (rng.random(T) >= mask_frac).astype(np.uint8)
    mask_t = torch.from_numpy(mask).to(dev)
    prm = B.Params(dtype=0 if dtype == "bf16" else 1, temperature=tau)
    Hn, Wn, yn = np64(H), np64(W), y.cpu().numpy()
    tol = TOL_LOGP if dtype == "bf16" else 2e-4
    merged = ref_merged = None
    for a, b in _edges(V, cuts):
        Ws = W[a:b].contiguous()
        ws = B.alloc_workspace(T, d, b - a, 0, prm, B.CALL_LOGPROB_FWD, dev)
        part = B.pg_head_shard_fwd(H, Ws, y, mask_t, a, prm, ws)
        torch.cuda.synchronize()
        ref = O.head_shard_partials(Hn, Wn[a:b], yn, a, tau, mask)
        got = part.cpu().numpy().astype(np.float64)
        assert np.all(got[mask == 0] == 0)
        _check_partials(got, ref, tol)
        # the merge operator on the oracle's own states (isolates the operator from the contraction)
        if merged is None:
            merged, ref_merged, ref_dev = part, ref, torch.from_numpy(ref.astype(np.float32)).to(dev)
        else:
            merged = B.pg_head_partials_merge(merged, part, out=merged)        # in place
            nxt = torch.from_numpy(ref.astype(np.float32)).to(dev)
            ref_dev = B.pg_head_partials_merge(ref_dev, nxt)
            ref_merged = O.merge_shard_partials(ref_merged, ref)
            torch.cuda.synchronize()
            _check_partials(ref_dev.cpu().numpy().astype(np.float64), ref_merged, 1e-5)
    logp, ent, lse = O.finish_shard_partials(merged.cpu().numpy())
    g_logp, g_ent, g_lse = B.pg_head_partials_finish(merged)                  # the same step on the device
    torch.cuda.synchronize()
    for g, r in ((g_logp, logp), (g_ent, ent), (g_lse, lse)):
        assert np.abs(g.cpu().numpy() - r).max() <= 1e-5 and not g[torch.from_numpy(mask == 0).to(dev)].any()
    only_logp = B.pg_head_partials_finish(merged, want_entropy=False, want_lse=False)
    assert only_logp[1] is None and only_logp[2] is None and torch.equal(only_logp[0], g_logp)
    rl, re, rs = O.lm_head_logprob(Hn, Wn, yn, tau, mask)
    assert np.abs(logp - rl).max() <= tol and np.abs(ent - re).max() <= tol and np.abs(lse - rs).max() <= tol
    # and the unsharded call gives the same numbers
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
    lp, en, ls = B.pg_logprob_fwd(H, W, y, mask_t, prm, ws)
    torch.cuda.synchronize()
    assert np.abs(lp.cpu().numpy() - logp).max() <= 1e-4 and np.abs(en.cpu().numpy() - ent).max() <= 1e-4


def _oracle_params(prm):
    return O.Params(temperature=prm.temperature, clip_eps_lo=prm.clip_eps_lo, clip_eps_hi=prm.clip_eps_hi,
                    mismatch_mode=prm.mismatch_mode, geo_lo=prm.geo_lo, geo_hi=prm.geo_hi,
                    veto_ratio=prm.veto_ratio, trunc_c=prm.trunc_c, norm_override=prm.norm_override)


@pytest.mark.parametrize("mode,kind,tau,cuts,dtype", [
    (0, "none", 1.0, (1200,), "bf16"),
    (1, "window", 0.7, (700, 1900), "bf16"),
    (2, "token", 1.0, (256, 257, 2000), "bf16"),
    (2, "token", 1.0, (400,), "f32"),
])
def test_shard_loss_backward(dev, monkeypatch, mode, kind, tau, cuts, dtype):
    """Forward on every shard, merge, backward on every shard: loss, log-probs, counters, each shard's
    dW rows and dH term against the oracle; the dH terms together against the whole-vocabulary dH."""
    if dtype == "bf16":
        spec = synth.small_spec(temperature=tau, seed=977 + mode)
    else:
        spec = synth.small_spec(temperature=tau, seed=977 + mode, d=64, V=1000, dtype="f32", unit_rms=False)
    prm = B.Params(dtype=0 if dtype == "bf16" else 1, mismatch_mode=mode, temperature=tau)
    batch, tin, nin = build_loss_case(spec, dev, oracle_logp, kind, on_policy=False)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    t_cap = (T + 255) // 256 * 256
    monkeypatch.setenv("PG_HEAD_DS_BUDGET_BYTES", str(t_cap * 2 * 256 * 3))        # several backward chunks per shard
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    _, A, _ = O.trloo_advantage(nin["rewards"], nin["valid"], 1.0)
    A_seg = A.reshape(-1)[nin["seg_sample"]]
    oprm = _oracle_params(prm)
    full = O.pg_loss_fwd_bwd(nin["H"], nin["W"], nin["y"], nin["loss_mask"], nin["cu"], A_seg, nin["old"], nin["rollout"], oprm)

    shards = _edges(V, cuts)
    Ws = [tin["W"][a:b].contiguous() for a, b in shards]
    merged = None
    for (a, b), Wsh in zip(shards, Ws):
        ws = B.alloc_workspace(T, d, b - a, 0, prm, B.CALL_LOGPROB_FWD, dev)
        part = B.pg_head_shard_fwd(tin["H"], Wsh, tin["y"], tin["loss_mask"], a, prm, ws)
        merged = part if merged is None else B.pg_head_partials_merge(merged, part)
    dH_sum = np.zeros((T, d))
    tol_logp = TOL_LOGP if dtype == "bf16" else 2e-4
    for (a, b), Wsh in zip(shards, Ws):
        ws = B.alloc_workspace(T, d, b - a, S, prm, B.CALL_LOSS_FWD_BWD, dev)
        out = B.pg_loss_shard_bwd(tin["H"], Wsh, tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                                  tin["old"], tin["rollout"], merged, a, prm, ws, dH_f32=True)
        torch.cuda.synchronize()
        ref = O.pg_loss_fwd_bwd(nin["H"], nin["W"], nin["y"], nin["loss_mask"], nin["cu"], A_seg, nin["old"],
                                nin["rollout"], oprm, vocab_slice=(a, b))
        assert np.array_equal(out["counters"].cpu().numpy(), ref["counters"])
        assert np.abs(out["logp"].cpu().numpy() - ref["logp"]).max() <= tol_logp
        assert np.abs(out["entropy"].cpu().numpy() - ref["entropy"]).max() <= tol_logp
        assert abs(float(out["loss"][0]) - ref["loss"]) <= TOL_LOSS * max(abs(ref["loss"]), 1e-6)
        assert out["dH"].dtype == torch.float32 and tuple(out["dW"].shape) == (b - a, d)
        dH = np64(out["dH"])
        assert np.all(dH[~ref["active"]] == 0)
        if b - a > 1:
            assert rel_fro(np64(out["dW"]), ref["dW"]) <= TOL_GRAD, ((a, b), rel_fro(np64(out["dW"]), ref["dW"]))
            assert rel_fro(dH, ref["dH"]) <= TOL_GRAD, ((a, b), rel_fro(dH, ref["dH"]))
        else:       # a single vocab row: compare on the scale of the whole gradient
            assert np.linalg.norm(np64(out["dW"]) - ref["dW"]) <= TOL_GRAD * np.linalg.norm(full["dW"]) / np.sqrt(V)
            assert np.linalg.norm(dH - ref["dH"]) <= TOL_GRAD * np.linalg.norm(full["dH"])
        dH_sum += dH
        # the shard's own W^T cache (filled by the call, then trusted): the same bits
        prm_c = B.Params(dtype=prm.dtype, mismatch_mode=mode, temperature=tau, w_transposed=B.alloc_w_transposed(d, b - a, dev))
        for valid in (0, 1):
            prm_c.w_transposed_valid = valid
            again = B.pg_loss_shard_bwd(tin["H"], Wsh, tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                                        tin["old"], tin["rollout"], merged, a, prm_c, ws, dH_f32=True)
            torch.cuda.synchronize()
            assert torch.equal(again["dH"], out["dH"]) and torch.equal(again["dW"], out["dW"]), ((a, b), valid)
    assert rel_fro(dH_sum, full["dH"]) <= TOL_GRAD


def test_shard_backward_bf16_dH_accumulate_and_one_shard_equals_unsharded(dev):
    """A single shard covering the whole vocabulary must reproduce pg_loss_fwd_bwd bit for bit (same kernels,
    same order), with dH in the dtype of H and dW accumulated."""
    spec = synth.small_spec(seed=555)
    prm = B.Params(mismatch_mode=2, accumulate_dW=1)
    batch, tin, nin = build_loss_case(spec, dev, oracle_logp, "token", on_policy=False)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)
    base = torch.full((V, d), 0.25, dtype=torch.float32, device=dev)
    a = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                          tin["old"], tin["rollout"], prm, ws, dW=base.clone())
    wsf = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOGPROB_FWD, dev)
    part = B.pg_head_shard_fwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], 0, prm, wsf)
    b = B.pg_loss_shard_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                            tin["old"], tin["rollout"], part, 0, prm, ws, dH_f32=False, dW=base.clone())
    torch.cuda.synchronize()
    assert b["dH"].dtype == tin["H"].dtype
    assert torch.equal(a["counters"], b["counters"])
    # the state crosses the boundary in natural-log units (one extra rounding): not bitwise, but far inside tolerance
    assert (a["logp"] - b["logp"]).abs().max().item() <= 2e-5
    assert abs(float(a["loss"][0]) - float(b["loss"][0])) <= 1e-5 * max(abs(float(a["loss"][0])), 1e-6)
    assert rel_fro(np64(b["dW"]) - 0.25, np64(a["dW"]) - 0.25) <= 1e-3
    assert rel_fro(np64(b["dH"]), np64(a["dH"])) <= 1e-2        # bf16 outputs: one ulp flips


def test_shard_empty_and_all_masked(dev):
    T, d, Vs = 300, 64, 500
    H, W, y = synth.make_head(T, d, Vs, "bf16", 71, dev, unit_rms=True)
    prm = B.Params(mismatch_mode=0)
    ws = B.alloc_workspace(T, d, Vs, 1, prm, B.CALL_LOSS_FWD_BWD, dev)
    zeros = torch.zeros(T, dtype=torch.uint8, device=dev)
    part = B.pg_head_shard_fwd(H, W, y + 4000, zeros, 4000, prm, ws)
    torch.cuda.synchronize()
    assert not part.any()
    cu = torch.tensor([0, T], dtype=torch.int32, device=dev)
    adv = torch.ones(1, dtype=torch.float64, device=dev)
    seg = torch.zeros(1, dtype=torch.int32, device=dev)
    out = B.pg_loss_shard_bwd(H, W, y + 4000, zeros, cu, adv, seg, None, None, part, 4000, prm, ws)
    torch.cuda.synchronize()
    assert float(out["loss"][0]) == 0.0 and not out["dH"].any() and not out["dW"].any()
    # T = 0
    e = torch.empty((0, d), dtype=torch.bfloat16, device=dev)
    part0 = B.pg_head_shard_fwd(e, W, y[:0], None, 0, prm, ws)
    assert part0.shape == (0, 4)
    assert B.pg_head_partials_merge(part0, part0).shape == (0, 4)


def test_shard_sequence_in_a_hip_graph(dev):
    """Forward on two shards, merge, finish and the backward of one shard captured in one HIP graph: replays
    reproduce the eager results bit for bit with a scrambled workspace (kernels only, no state between calls)."""
    spec = synth.small_spec(seed=4323)
    prm = B.Params(mismatch_mode=2)
    batch, tin, _ = build_loss_case(spec, dev, oracle_logp, "token", on_policy=False)
    T, d, V, S = batch.T, spec.d, spec.V, batch.S
    cut = 1100
    Wa, Wb = tin["W"][:cut].contiguous(), tin["W"][cut:].contiguous()
    ws = B.alloc_workspace(T, d, V, S, prm, B.CALL_LOSS_FWD_BWD, dev)          # large enough for every call below
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    pa = torch.empty((T, 4), dtype=torch.float32, device=dev)
    pb = torch.empty_like(pa)
    merged = torch.empty_like(pa)
    dW = torch.empty((V - cut, d), dtype=torch.float32, device=dev)
    outbuf = (torch.empty(1, dtype=torch.float32, device=dev), torch.empty((T, d), dtype=torch.float32, device=dev),
              torch.empty(T, dtype=torch.float32, device=dev), torch.empty(T, dtype=torch.float32, device=dev),
              torch.empty(8, dtype=torch.int64, device=dev))

    def step(stream=None):
        B.pg_head_shard_fwd(tin["H"], Wa, tin["y"], tin["loss_mask"], 0, prm, ws, out=pa, stream=stream)
        B.pg_head_shard_fwd(tin["H"], Wb, tin["y"], tin["loss_mask"], cut, prm, ws, out=pb, stream=stream)
        B.pg_head_partials_merge(pa, pb, out=merged, stream=stream)
        return B.pg_loss_shard_bwd(tin["H"], Wb, tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                                   tin["old"], tin["rollout"], merged, cut, prm, ws, dH_f32=True, dW=dW, out=outbuf,
                                   stream=stream)

    out = step()
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in out.items()}
    eager_merged = merged.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(side)
    for rep in range(3):
        for t in outbuf + (pa, pb, merged, dW):
            t.zero_()
        ws.random_(0, 255)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(merged, eager_merged), rep
        for k in ("loss", "dH", "dW", "logp", "entropy", "counters"):
            assert torch.equal(out[k], eager[k]), (rep, k)
        _ = (tin["H"].float() @ Wa.float().T).sum()
        torch.cuda.synchronize()
