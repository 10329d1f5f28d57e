"""pg_monitors_static, the entry point that allocates nothing (its partial sums live in a static device
array inside the library), against pg_monitors with a caller-owned workspace: same kernels, same fixed
summation order, so the eight outputs must agree bit for bit.  Two calls in a row, the second on a
smaller input (the array keeps the first call's contents), each also checked against the fp64 oracle's
monitors.  Runs last (file name), alone or after the other tests."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import pg_oracle as O
from paper_2602_05885_amd import binding as B

pytestmark = pytest.mark.gpu


def _inputs(dev, T, n_h, n_w, seed, w_dtype):
    g = torch.Generator(device="cpu").manual_seed(seed)
    logp = -torch.rand(T, generator=g) * 5.0
    roll = logp + 0.1 * torch.randn(T, generator=g)
    ent = torch.rand(T, generator=g) * 3.0
    mask = (torch.rand(T, generator=g) < 0.7).to(torch.uint8)
    dH = (torch.randn(n_h, generator=g) * 1e-3).to(torch.bfloat16)
    dW = (torch.randn(n_w, generator=g) * 1e-4).to(w_dtype)
    return [t.to(dev) for t in (logp, roll, ent, mask, dH, dW)]


def _oracle(logp, roll, ent, mask, dH, dW):
    f = lambda t: t.double().cpu().numpy()
    return O.monitors(f(logp), f(roll), f(ent), mask.cpu().numpy(), f(dH), f(dW))


def test_monitors_static_matches_workspace_variant_twice():
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    B.pg_init()
    out_static = torch.empty(8, dtype=torch.float64, device=dev)
    # first call: larger input; second call: smaller input (odd sizes: ragged tail of the 8-element units)
    for T, n_h, n_w, seed, w_dtype in ((50_000, 1_000_003, 2_500_001, 1, torch.float32),
                                       (777, 4_099, 12_345, 2, torch.bfloat16)):
        logp, roll, ent, mask, dH, dW = _inputs(dev, T, n_h, n_w, seed, w_dtype)
        ref = B.pg_monitors(logp, roll, ent, mask, dH, dW)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(dev)
        got = B.pg_monitors_static(logp, roll, ent, mask, dH, dW, out=out_static)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(dev) == before
        assert torch.equal(got, ref), (got.cpu().numpy(), ref.cpu().numpy())
        want = _oracle(logp, roll, ent, mask, dH, dW)
        g = dict(zip(B.MONITOR_NAMES, got.cpu().numpy()[:6]))
        for k in B.MONITOR_NAMES:
            assert abs(g[k] - want[k]) <= 1e-9 * max(1.0, abs(want[k])), (k, g[k], want[k])
    # optional inputs absent; T = 0
    logp, roll, ent, mask, dH, dW = _inputs(dev, 300, 64, 64, 3, torch.float32)
    assert torch.equal(B.pg_monitors_static(logp, None, None, mask), B.pg_monitors(logp, None, None, mask))
    empty = torch.empty(0, device=dev)
    got = B.pg_monitors_static(empty, None, None, torch.empty(0, dtype=torch.uint8, device=dev), dH, None)
    torch.cuda.synchronize()
    assert float(got[5]) == 0.0 and float(got[1]) == 1.0 and float(got[3]) > 0.0


def test_monitors_static_rejects_sizes_beyond_its_maximum():
    lib = B.lib()
    one = C.c_void_p(16)          # never dereferenced: validation fails first
    rc = lib.pg_monitors_static(one, None, None, one, (1 << 31) + 1, None, 0, 0, None, 0, 0, one, None)
    assert rc == -2 and "at most" in B.pg_last_error()
    rc = lib.pg_monitors_static(one, None, None, one, 4, one, 0, (1 << 40) + 8, None, 0, 0, one, None)
    assert rc == -2
    rc = lib.pg_monitors_static(one, None, None, one, 4, None, 0, 0, None, 0, 0, None, None)
    assert rc == -1
