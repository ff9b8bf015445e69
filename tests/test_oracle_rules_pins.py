"""Pins for the oracle's other update rules: momentum SGD and the combined (synchronous) mode."""
import numpy as np
import pytest
import torch

import oracle

F32 = np.float32


def _one(e0, s0, lr, eps, mu, opt, comb, gs, k=2, S=3):
    E = np.array([[e0]] + [[0.0]] * (k - 1), F32)
    A = np.array([[s0]] + [[0.0]] * (k - 1), F32)
    PE, PA = oracle.encode(E, k), oracle.encode(A, k)
    ld, lp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
    oracle.update_rule(E, A, PE, PA, k, S, lr, eps, mu, opt, comb, np.zeros(len(gs), np.uint64),
                       np.array(gs, F32).reshape(-1, 1), ld, lp)
    return E[0, 0], A[0, 0], PE[0, 0], PA[0, 0], int(ld.sum()), int(lp.sum())


@pytest.mark.parametrize("name", ["mom1", "mom2"])
def test_golden_momentum(golden, name):
    g = golden("momentum_and_combined.txt")
    e, v, pe, pa, nd, np_ = _one(g[f"{name}.e0"][0], g[f"{name}.v0"][0], g[f"{name}.lr"][0], 0.0,
                                 g[f"{name}.mu"][0], 1, 0, g[f"{name}.g"])
    assert e == g[f"{name}.e"][0] and v == g[f"{name}.v"][0]
    assert pe == e and pa == v                 # the other member is zero: parity = entry / state
    assert nd == np_ == len(g[f"{name}.g"])


def test_golden_combined(golden):
    g = golden("momentum_and_combined.txt")
    e, G, pe, pa, nd, np_ = _one(g["comb1.e0"][0], g["comb1.G0"][0], g["comb1.lr"][0], 0.0, 0.0, 0, 1, g["comb1.g"])
    assert e == pytest.approx(g["comb1.e"][0], abs=1e-7) and G == g["comb1.G"][0]
    assert nd == np_ == 1                      # one update per modified entry
    e, v, pe, pa, nd, np_ = _one(g["comb2.e0"][0], g["comb2.v0"][0], g["comb2.lr"][0], 0.0, g["comb2.mu"][0], 1, 1,
                                 g["comb2.g"])
    assert e == g["comb2.e"][0] and v == g["comb2.v"][0] and nd == 1


def test_rule_adagrad_sequential_equals_the_pinned_oracle():
    rng = np.random.default_rng(0)
    R, D, k, S, n = 24, 8, 4, 5, 300
    E = ((rng.random((R, D)) - 0.5) / 8).astype(F32)
    A = (rng.random((R, D)) * 1e-3).astype(F32)
    PE, PA = oracle.encode(E, k), oracle.encode(A, k)
    keys = rng.integers(0, R, n).astype(np.uint64)
    grads = ((rng.random((n, D)) - 0.5) / 64).astype(F32)
    a = [x.copy() for x in (E, A, PE, PA)]
    b = [x.copy() for x in (E, A, PE, PA)]
    oracle.update(*a, k, S, 0.01, 1e-8, keys, grads)
    oracle.update_rule(*b, k, S, 0.01, 1e-8, 0.0, 0, 0, keys, grads)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_momentum_matches_torch_sgd():
    rng = np.random.default_rng(5)
    R, D, k, S, lr, mu, n = 8, 4, 2, 3, 0.05, 0.9, 60
    E = (rng.random((R, D)) - 0.5).astype(F32)
    V = ((rng.random((R, D)) - 0.5) / 4).astype(F32)
    PE, PV = oracle.encode(E, k), oracle.encode(V, k)
    keys = rng.integers(0, R, n).astype(np.uint64)
    grads = (rng.random((n, D)) - 0.5).astype(F32)
    # torch applies the optimizer to every row each step; rows without a gradient must not move, so
    # each row gets its own parameter and only the addressed one is stepped
    params = [torch.tensor(E[r], dtype=torch.float64, requires_grad=True) for r in range(R)]
    opts = [torch.optim.SGD([p], lr=float(F32(lr)), momentum=float(F32(mu)), dampening=0.0) for p in params]
    for r in range(R):
        opts[r].state[params[r]]["momentum_buffer"] = torch.tensor(V[r], dtype=torch.float64)
    for i in range(n):
        r = int(keys[i])
        params[r].grad = torch.tensor(grads[i], dtype=torch.float64)
        opts[r].step()
    oracle.update_rule(E, V, PE, PV, k, S, lr, 0.0, mu, 1, 0, keys, grads)
    ref_e = np.stack([p.detach().numpy() for p in params])
    ref_v = np.stack([opts[r].state[params[r]]["momentum_buffer"].numpy() for r in range(R)])
    np.testing.assert_allclose(E, ref_e.astype(F32), rtol=2e-7, atol=1e-9)
    np.testing.assert_allclose(V, ref_v.astype(F32), rtol=2e-7, atol=1e-9)
    # the parity of the velocities stays the sum of the velocities (the rule is linear in v)
    np.testing.assert_allclose(PV, V.astype(np.float64).reshape(R // k, k, D).sum(1), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(PE, E.astype(np.float64).reshape(R // k, k, D).sum(1), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("m", [1, 5, 300])
def test_momentum_chain_closed_form(m):
    """v_t = mu^t v_0 + sum_s mu^(t-s) g_s ; e_m = e_0 - lr * sum_t v_t."""
    rng = np.random.default_rng(m)
    D, k, S, lr, mu = 8, 2, 3, 0.01, 0.9
    E = (rng.random((2, D)) - 0.5).astype(F32)
    V = ((rng.random((2, D)) - 0.5) / 4).astype(F32)
    E0, V0 = E.copy(), V.copy()
    PE, PV = oracle.encode(E, k), oracle.encode(V, k)
    grads = ((rng.random((m, D)) - 0.5) / 8).astype(F32)
    oracle.update_rule(E, V, PE, PV, k, S, lr, 0.0, mu, 1, 0, np.ones(m, np.uint64), grads)
    mu64, lr64 = float(F32(mu)), float(F32(lr))
    t = np.arange(1, m + 1)
    vt = np.stack([mu64 ** tt * V0[1].astype(np.float64) +
                   (mu64 ** (tt - 1 - np.arange(tt))[:, None] * grads[:tt].astype(np.float64)).sum(0) for tt in t])
    np.testing.assert_allclose(V[1], vt[-1], rtol=3e-7, atol=1e-9)
    np.testing.assert_allclose(E[1], E0[1] - lr64 * vt.sum(0), rtol=3e-7, atol=1e-8)
    np.testing.assert_array_equal(E[0], E0[0])


@pytest.mark.parametrize("opt", [0, 1])
def test_combined_equals_sequential_on_presummed_gradients(opt):
    rng = np.random.default_rng(9 + opt)
    R, D, k, S, n = 20, 8, 4, 5, 200
    E = ((rng.random((R, D)) - 0.5) / 8).astype(F32)
    A = (rng.random((R, D)) * 1e-3).astype(F32)
    PE, PA = oracle.encode(E, k), oracle.encode(A, k)
    keys = rng.integers(0, R, n).astype(np.uint64)
    # dyadic gradients with few bits, so that every per-entry sum is exactly representable in fp32
    grads = (rng.integers(-64, 64, (n, D)) / 4096.0).astype(F32)
    a = [x.copy() for x in (E, A, PE, PA)]
    ld, lp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
    oracle.update_rule(*a, k, S, 0.01, 1e-8, 0.9, opt, 1, keys, grads, ld, lp)
    uk = np.unique(keys)
    summed = np.stack([grads[keys == x].astype(np.float64).sum(0) for x in uk]).astype(F32)
    b = [x.copy() for x in (E, A, PE, PA)]
    ld2, lp2 = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
    oracle.update_rule(*b, k, S, 0.01, 1e-8, 0.9, opt, 0, uk, summed, ld2, lp2)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    np.testing.assert_array_equal(ld, ld2)
    np.testing.assert_array_equal(lp, lp2)
    assert int(ld.sum()) == len(uk) == int(lp.sum())          # one update per modified entry, and one parity update
