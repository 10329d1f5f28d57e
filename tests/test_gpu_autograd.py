"""The torch.autograd glue hands out exactly what the C ABI computed: loss.backward() leaves the library's dH in
H.grad and its dW in W.grad (fp32 head: bit for bit; bf16 head: dW in W's dtype), and the loss matches the oracle."""
import numpy as np
import pytest
import torch

from oracle import pg_oracle as O
from paper_2602_05885_amd import autograd as A
from paper_2602_05885_amd import binding as B
from paper_2602_05885_amd import synth
from tests._cases import build_loss_case, np64, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


def oracle_logp(Hn, Wn, yn, tau):
    return O.lm_head_logprob(Hn, Wn, yn, tau)[0]


def test_pg_head_loss_backward_f32(dev):
    spec = synth.small_spec(seed=606, d=64, V=900, dtype="f32", unit_rms=False)
    prm = B.Params(dtype=1, mismatch_mode=2)
    batch, tin, nin = build_loss_case(spec, dev, oracle_logp, "token", on_policy=False)
    adv, _, _ = B.trloo_advantage(tin["rewards"], tin["valid"], 1.0)
    ws = B.alloc_workspace(batch.T, spec.d, spec.V, batch.S, prm, B.CALL_LOSS_FWD_BWD, dev)
    ref = B.pg_loss_fwd_bwd(tin["H"], tin["W"], tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                            tin["old"], tin["rollout"], prm, ws)
    H = tin["H"].clone().requires_grad_(True)
    W = tin["W"].clone().requires_grad_(True)
    loss, aux = A.pg_head_loss(H, W, tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                               tin["old"], tin["rollout"], prm)
    assert loss.dim() == 0 and loss.requires_grad
    loss.backward()
    torch.cuda.synchronize()
    assert torch.equal(H.grad, ref["dH"]) and torch.equal(W.grad, ref["dW"])
    assert torch.equal(loss.detach().reshape(1), ref["loss"]) and torch.equal(aux["logp"], ref["logp"])
    _, Aor, _ = O.trloo_advantage(nin["rewards"], nin["valid"], 1.0)
    o = O.pg_loss_fwd_bwd(nin["H"], nin["W"], nin["y"], nin["loss_mask"], nin["cu"], Aor.reshape(-1)[nin["seg_sample"]],
                          nin["old"], nin["rollout"], O.Params(mismatch_mode=2))
    assert abs(float(loss.detach()) - o["loss"]) <= 1e-3 * abs(o["loss"])
    assert rel_fro(np64(H.grad), o["dH"]) <= 1e-2 and rel_fro(np64(W.grad), o["dW"]) <= 1e-2
    # an upstream factor, applied on request
    H2 = tin["H"].clone().requires_grad_(True)
    W2 = tin["W"].clone().requires_grad_(True)
    loss2, _ = A.pg_head_loss(H2, W2, tin["y"], tin["loss_mask"], tin["cu"], adv.reshape(-1), tin["seg_sample"],
                              tin["old"], tin["rollout"], prm, workspace=ws, scale_by_upstream=True)
    (loss2 * 0.5).backward()
    torch.cuda.synchronize()
    assert torch.allclose(H2.grad, ref["dH"] * 0.5) and torch.allclose(W2.grad, ref["dW"] * 0.5)


def test_sft_head_loss_bf16_with_external_accumulator(dev):
    T, d, V = 700, 128, 3000
    H0, W0, y = synth.make_head(T, d, V, "bf16", 12, dev, unit_rms=True)
    mask = torch.from_numpy((np.random.default_rng(12).random(T) >= 0.3).astype(np.uint8)).to(dev)
    prm = B.Params(accumulate_dW=1)
    ws = B.alloc_workspace(T, d, V, 0, prm, B.CALL_LOSS_FWD_BWD, dev)
    acc_ref = torch.full((V, d), 0.5, dtype=torch.float32, device=dev)
    ref = B.pg_sft_fwd_bwd(H0, W0, y, mask, prm, ws, dW=acc_ref)
    H = H0.clone().requires_grad_(True)
    W = W0.clone().requires_grad_(True)
    acc = torch.full((V, d), 0.5, dtype=torch.float32, device=dev)
    loss, aux = A.sft_head_loss(H, W, y, mask, prm, workspace=ws, dW_accum=acc)
    loss.backward()
    torch.cuda.synchronize()
    assert torch.equal(H.grad, ref["dH"]) and W.grad is None and torch.equal(acc, acc_ref)
    o = O.sft_ce_fwd_bwd(np64(H0), np64(W0), y.cpu().numpy(), mask.cpu().numpy(), 1.0)
    assert abs(float(loss.detach()) - o["loss"]) <= 1e-3 * abs(o["loss"])
    # without an accumulator W.grad arrives in W's dtype
    prm0 = B.Params()
    H3 = H0.clone().requires_grad_(True)
    W3 = W0.clone().requires_grad_(True)
    loss3, _ = A.sft_head_loss(H3, W3, y, mask, prm0, workspace=ws)
    loss3.backward()
    torch.cuda.synchronize()
    assert W3.grad.dtype == torch.bfloat16 and rel_fro(np64(W3.grad), o["dW"]) <= 1e-2
