"""Builds seeded test cases: the same arrays go to the oracle (numpy fp64) and to the HIP library (torch)."""
import numpy as np
import torch

from paper_2602_05885_amd import synth


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def ratio_targets(n, seed, lo=0.8, hi=1.2, margin=0.03):
    """Policy ratios spread over all clip branches, never within `margin` of a threshold."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    base = rng.choice([0.55, 0.7, 0.9, 1.0, 1.0, 1.1, 1.3, 1.6], size=n)
    r = base * (1.0 + rng.uniform(-0.02, 0.02, size=n))
    assert np.all(np.abs(r - lo) > margin) and np.all(np.abs(r - hi) > margin)
    return r


def segment_offsets(batch, seed, kind):
    """Per-token log-ratio old - rollout: a per-segment constant (well inside or well outside the
    paper's [0.999, 1.001] window) plus tiny zero-centred noise; one segment gets a vetoed token."""
    rng = np.random.Generator(np.random.Philox(key=seed + 77))
    T, S = batch.T, batch.S
    delta = np.zeros(T)
    if kind == "none":
        return delta
    seg_choices = np.array([0.0, 4e-4, -5e-4, 2.5e-3, -3e-3]) if kind == "window" else np.array([0.0, 0.3, -0.4, 0.9, -0.1])
    for s in range(S):
        a, b = batch.cu_seqlens[s], batch.cu_seqlens[s + 1]
        delta[a:b] = seg_choices[s % len(seg_choices)] + rng.uniform(-1e-5, 1e-5, size=b - a) * (kind == "window") \
            + rng.normal(0, 0.2, size=b - a) * (kind == "token")
    if S >= 2:                                   # token veto in segment 1: ratio e^-10 < 1e-4
        a, b = batch.cu_seqlens[1], batch.cu_seqlens[2]
        loss_rows = np.nonzero(batch.loss_mask[a:b])[0]
        if len(loss_rows):
            delta[a + loss_rows[len(loss_rows) // 2]] = -10.0
    return delta


def build_loss_case(spec, device, oracle_logp_fn, mismatch_kind="none", on_policy=False, scale_rows=1.0):
    """Returns (torch inputs on `device`, numpy inputs for the oracle)."""
    batch = synth.make_batch(spec, scale_rows)
    H, W, y = synth.make_head(batch.T, spec.d, spec.V, spec.dtype, spec.seed, device, spec.unit_rms)
    Hn, Wn, yn = np64(H), np64(W), y.cpu().numpy().astype(np.int64)
    old = rollout = None
    if not on_policy or mismatch_kind != "none":
        base = oracle_logp_fn(Hn, Wn, yn, spec.temperature)              # oracle log-probs: inputs only
        r = np.ones(batch.T) if on_policy else ratio_targets(batch.T, spec.seed)
        old = (base - np.log(r)).astype(np.float32)
        rollout = (old.astype(np.float64) - segment_offsets(batch, spec.seed, mismatch_kind)).astype(np.float32)
    tin = dict(
        H=H, W=W, y=y,
        loss_mask=torch.from_numpy(batch.loss_mask).to(device),
        cu=torch.from_numpy(batch.cu_seqlens).to(device),
        seg_sample=torch.from_numpy(batch.seg_sample).to(device),
        rewards=torch.from_numpy(batch.rewards).to(device),
        valid=torch.from_numpy(batch.valid).to(device),
        old=None if old is None else torch.from_numpy(old).to(device),
        rollout=None if rollout is None else torch.from_numpy(rollout).to(device),
    )
    nin = dict(H=Hn, W=Wn, y=yn, loss_mask=batch.loss_mask, cu=batch.cu_seqlens, seg_sample=batch.seg_sample,
               rewards=batch.rewards, valid=batch.valid, old=old, rollout=rollout)
    return batch, tin, nin


def rel_fro(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return np.linalg.norm(a - b) / den if den > 0 else np.linalg.norm(a)


def block_rel_fro(a, b, rows=256):
    """Largest relative Frobenius error over consecutive blocks of `rows` rows (a wrong 16 x 16 MFMA tile
    moves a whole-matrix norm by almost nothing; it cannot hide in a 256-row block).  A block's error is
    taken relative to its own reference norm, or, where that is below 1e-3 of the mean block norm (rows
    of inactive tokens, vocabulary rows nobody's distribution touches), relative to the mean block norm."""
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    n = (a.shape[0] + rows - 1) // rows
    den = np.array([np.linalg.norm(b[i * rows:(i + 1) * rows]) for i in range(n)])
    err = np.array([np.linalg.norm(a[i * rows:(i + 1) * rows] - b[i * rows:(i + 1) * rows]) for i in range(n)])
    floor = 1e-3 * (den.mean() if den.size and den.mean() > 0 else 1.0)
    return float((err / np.maximum(den, floor)).max()) if n else 0.0


def pad_ld(n: int) -> int:
    """Leading dimension the library gives a scratch matrix with n columns (an odd number of 128-byte lines)."""
    return n + 64 if (n // 64) % 2 == 0 else n


def recompute_covers_vocabulary(T: int, V: int, n_pad: int, chunk_rows: int) -> bool:
    """The library's device-side rule for few active rows, restated for the tests: dS of the whole vocabulary fits
    the chunk scratch (sized for t_cap rows and chunk_rows columns) at n_pad rows, in both orientations."""
    t_cap, v_pad = (T + 255) // 256 * 256, (V + 255) // 256 * 256
    if chunk_rows >= v_pad or n_pad <= 0:
        return False                                  # one chunk anyway / nothing to do
    return n_pad * pad_ld(v_pad) <= t_cap * pad_ld(chunk_rows) and v_pad * pad_ld(n_pad) <= chunk_rows * pad_ld(t_cap)
