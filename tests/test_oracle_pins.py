"""Pins for the CPU oracle: it is checked against what the paper and the mathematics fix, never
against itself.  Citations are to the ECRM paper (arXiv 2104.01981)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import brute

F32 = np.float32


def _tables(R, D, k, rng, a_scale=1e-3):
    E = ((rng.random((R, D)) - 0.5) / 8).astype(F32)
    A = (rng.random((R, D)) * a_scale).astype(F32)
    return E, A, oracle.encode(E, k), oracle.encode(A, k)


def _one_param_chain(e0, G0, lr, eps, gs, k=2, S=3):
    """Run the oracle on one parameter (row 0 of a 1-stripe table), return (e, G, pe, pa)."""
    E = np.array([[e0]] + [[0.0]] * (k - 1), F32)
    A = np.array([[G0]] + [[0.0]] * (k - 1), F32)
    PE, PA = oracle.encode(E, k), oracle.encode(A, k)
    keys = np.zeros(len(gs), np.uint64)
    grads = np.array(gs, F32).reshape(-1, 1)
    oracle.update(E, A, PE, PA, k, S, lr, eps, keys, grads)
    return E[0, 0], A[0, 0], PE[0, 0], PA[0, 0]


# ---- Sec. 3.3.1: the printed Adagrad rule, hand-computed chains ----------------------------------

@pytest.mark.parametrize("name", ["chain1", "chain2", "chain3", "chain4"])
def test_golden_adagrad_chains(golden, name):
    g = golden("adagrad_chains.txt")
    e, G, pe, pa = _one_param_chain(g[f"{name}.e0"][0], g[f"{name}.G0"][0], g[f"{name}.lr"][0],
                                    g[f"{name}.eps"][0], g[f"{name}.g"])
    assert e == pytest.approx(g[f"{name}.e"][0], abs=1e-7)
    assert G == pytest.approx(g[f"{name}.G"][0], abs=0)
    # the other member of the stripe is zero, so the parity must equal the entry / accumulator
    assert pe == pytest.approx(g[f"{name}.e"][0], abs=1e-7)
    assert pa == g[f"{name}.G"][0]


def _mutant_chain(e0, G0, lr, eps, gs, mistake):
    e, G = e0, G0
    for g in gs:
        if mistake == "stale_accumulator":      # uses G_{t-1}
            e -= lr / np.sqrt(G + eps) * g if G + eps > 0 else 0.0
            G += g * g
            continue
        G += g * g if mistake != "abs_not_square" else abs(g)
        if mistake == "eps_outside_root":
            e -= lr / (np.sqrt(G) + eps) * g
        elif mistake == "wrong_sign":
            e += lr / np.sqrt(G + eps) * g
        elif mistake == "no_root":
            e -= lr / (G + eps) * g
        else:
            e -= lr / np.sqrt(G + eps) * g
    return e, G


@pytest.mark.parametrize("mistake", ["stale_accumulator", "eps_outside_root", "wrong_sign", "no_root",
                                     "abs_not_square"])
def test_golden_chains_have_teeth(golden, mistake):
    """Each plausible slip in the rule misses at least one of the hand-computed chains."""
    g = golden("adagrad_chains.txt")
    missed = False
    for name in ["chain1", "chain2", "chain3", "chain4"]:
        e, G = _mutant_chain(g[f"{name}.e0"][0], g[f"{name}.G0"][0], g[f"{name}.lr"][0],
                             g[f"{name}.eps"][0], g[f"{name}.g"], mistake)
        if abs(e - g[f"{name}.e"][0]) > 1e-6 or abs(G - g[f"{name}.G"][0]) > 1e-6:
            missed = True
    assert missed
    # and the unmutated transcription hits all of them
    for name in ["chain1", "chain2", "chain3", "chain4"]:
        e, G = _mutant_chain(g[f"{name}.e0"][0], g[f"{name}.G0"][0], g[f"{name}.lr"][0],
                             g[f"{name}.eps"][0], g[f"{name}.g"], None)
        assert abs(e - g[f"{name}.e"][0]) < 1e-12 and G == g[f"{name}.G"][0]


# ---- Sec. 3.3.2: difference propagation keeps the parity current -------------------------------

def test_golden_parity_chain_k2(golden):
    g = golden("parity_chain_k2.txt")
    E = np.array(g["e0"], F32).reshape(2, 1)
    A = np.array(g["G0"], F32).reshape(2, 1)
    PE = np.array(g["pe0"], F32).reshape(1, 1)
    PA = np.array(g["pa0"], F32).reshape(1, 1)
    keys = np.array(g["keys"], np.uint64)
    grads = np.array(g["g"], F32).reshape(-1, 1)
    oracle.update(E, A, PE, PA, 2, 3, 1.0, 0.0, keys, grads)
    np.testing.assert_allclose(E[:, 0], g["e"], rtol=0, atol=1e-7)
    np.testing.assert_array_equal(A[:, 0], g["G"])
    assert PE[0, 0] == pytest.approx(g["pe"][0], abs=1e-7)
    assert PA[0, 0] == g["pa"][0]


def test_golden_strawman_breaks_parity(golden):
    """Sec. 3.3.1: applying the optimizer at the parity with the parity accumulator is wrong."""
    g = golden("parity_chain_k2.txt")
    E = np.array(g["e0"], F32).reshape(2, 1)
    A = np.array(g["G0"], F32).reshape(2, 1)
    PE = np.array(g["pe0"], F32).reshape(1, 1)
    PA = np.array(g["pa0"], F32).reshape(1, 1)
    keys = np.array(g["keys"][:1], np.uint64)
    grads = np.array(g["g"][:1], F32).reshape(-1, 1)
    oracle.update_gradient_propagation(E, A, PE, PA, 2, 1.0, 0.0, keys, grads)
    assert PE[0, 0] == pytest.approx(g["strawman.pe_after_item0"][0], abs=1e-7)
    assert abs(PE[0, 0] - (E[0, 0] + E[1, 0])) > 0.1       # the invariant is broken
    assert PA[0, 0] == A[0, 0] + A[1, 0]                   # while the accumulator parity is fine


def test_strawman_fails_invariant_random():
    rng = np.random.default_rng(5)
    R, D, k = 64, 8, 4
    E, A, PE, PA = _tables(R, D, k, rng)
    keys = rng.integers(0, R, 200).astype(np.uint64)
    grads = ((rng.random((200, D)) - 0.5) / 64).astype(F32)
    oracle.update_gradient_propagation(E, A, PE, PA, k, 0.01, 1e-8, keys, grads)
    resid = np.abs(PE.astype(np.float64) - E.astype(np.float64).reshape(R // k, k, D).sum(1)).max()
    assert resid > 1e-3


# ---- Sec. 1 / 2.4 / 3.2: sum encoder, subtraction decoder ---------------------------------------

def test_golden_sum_code_k3(golden):
    g = golden("sum_code_k3.txt")
    T = np.array([g["e1"], g["e2"], g["e3"]], F32)
    P = oracle.encode(T, 3)
    np.testing.assert_array_equal(P[0], np.array(g["p"], F32))
    for lost, name in enumerate(["e1", "e2", "e3"]):
        rec = oracle.decode_member(T, P, 3, lost)
        np.testing.assert_array_equal(rec[0], np.array(g[name], F32))


@pytest.mark.parametrize("k", [2, 3, 4, 10])
def test_any_k_of_k_plus_1(k):
    """Sec. 2.4: any k of the k+1 units recover the rest (exact on dyadic values)."""
    rng = np.random.default_rng(k)
    R, D = 8 * k, 16
    T = (rng.integers(-512, 512, (R, D)) / 64.0).astype(F32)
    P = oracle.encode(T, k)
    np.testing.assert_array_equal(P, T.reshape(R // k, k, D).sum(1))
    for lost in range(k):
        rec = oracle.decode_member(T, P, k, lost)
        np.testing.assert_array_equal(rec, T[lost::k])


# ---- special case: eps = 0 reduces to the library's Adagrad --------------------------------------

def test_eps0_matches_torch_adagrad():
    rng = np.random.default_rng(11)
    R, D, k, S, lr = 8, 4, 2, 3, 0.05
    E, A, PE, PA = _tables(R, D, k, rng, a_scale=1.0)
    A += F32(0.5)                      # torch with a zero sum and zero gradient would give 0/0
    PA = oracle.encode(A, k)
    n = 40
    keys = rng.integers(0, R, n).astype(np.uint64)
    grads = (rng.random((n, D)) - 0.5).astype(F32)

    p = torch.tensor(E, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adagrad([p], lr=float(F32(lr)), eps=0.0, lr_decay=0.0, weight_decay=0.0)
    opt.state[p]["sum"] = torch.tensor(A, dtype=torch.float64)
    opt.state[p]["step"] = torch.tensor(0.0)
    for i in range(n):
        gfull = torch.zeros(R, D, dtype=torch.float64)
        gfull[int(keys[i])] = torch.tensor(grads[i], dtype=torch.float64)
        p.grad = gfull
        opt.step()
    oracle.update(E, A, PE, PA, k, S, lr, 0.0, keys, grads)
    np.testing.assert_allclose(E, p.detach().numpy().astype(F32), rtol=2e-7, atol=1e-9)
    np.testing.assert_allclose(A, opt.state[p]["sum"].numpy().astype(F32), rtol=2e-7, atol=0)


# ---- closed form of a run of updates on one entry ------------------------------------------------

@pytest.mark.parametrize("m", [1, 2, 7, 64, 1000])
def test_single_row_chain_closed_form(m):
    """G_t = G_0 + prefix sum of g^2 ; e_m = e_0 - lr * sum_t g_t / sqrt(G_t + eps)."""
    rng = np.random.default_rng(m)
    R, D, k, S, lr, eps = 8, 16, 4, 5, 0.01, 1e-8
    E, A, PE, PA = _tables(R, D, k, rng)
    E0, A0, PE0, PA0 = E.copy(), A.copy(), PE.copy(), PA.copy()
    row = 5
    keys = np.full(m, row, np.uint64)
    grads = ((rng.random((m, D)) - 0.5) / 64).astype(F32)
    oracle.update(E, A, PE, PA, k, S, lr, eps, keys, grads)
    g64 = grads.astype(np.float64)
    Gt = A0[row].astype(np.float64) + np.cumsum(g64 * g64, axis=0)
    lr64, eps64 = float(F32(lr)), float(F32(eps))
    e_ref = E0[row].astype(np.float64) - lr64 * (g64 / np.sqrt(Gt + eps64)).sum(0)
    np.testing.assert_allclose(E[row], e_ref, rtol=2e-7, atol=1e-9)
    np.testing.assert_allclose(A[row], Gt[-1], rtol=2e-7, atol=0)
    # the stripe's parity moved by exactly the same amounts; everything else is untouched
    np.testing.assert_allclose(PE[1], PE0[1].astype(np.float64) + (e_ref - E0[row]), rtol=3e-7, atol=1e-8)
    np.testing.assert_allclose(PA[1], PA0[1].astype(np.float64) + (Gt[-1] - A0[row]), rtol=3e-7, atol=0)
    mask = np.ones(R, bool); mask[row] = False
    np.testing.assert_array_equal(E[mask], E0[mask])
    np.testing.assert_array_equal(A[mask], A0[mask])
    np.testing.assert_array_equal(PE[0], PE0[0])


# ---- independent transcription (NumPy brute force) ----------------------------------------------

@pytest.mark.parametrize("R,D,k,S,n,seed", [(16, 4, 2, 3, 100, 0), (40, 8, 4, 5, 500, 1),
                                            (30, 12, 10, 11, 300, 2), (12, 4, 3, 7, 64, 3)])
def test_brute_force_small(R, D, k, S, n, seed):
    rng = np.random.default_rng(seed)
    E, A, PE, PA = _tables(R, D, k, rng)
    keys = rng.integers(0, R, n).astype(np.uint64)
    grads = ((rng.random((n, D)) - 0.5) / 64).astype(F32)
    bE, bA, bPE, bPA, bld, blp = brute.update(E, A, PE, PA, k, S, 0.01, 1e-8, keys, grads)
    ld, lp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
    oracle.update(E, A, PE, PA, k, S, 0.01, 1e-8, keys, grads, ld, lp)
    for x, y in [(E, bE), (A, bA), (PE, bPE), (PA, bPA)]:
        np.testing.assert_allclose(x, y, rtol=2e-7, atol=1e-10)
    np.testing.assert_array_equal(ld, bld)
    np.testing.assert_array_equal(lp, blp)


def test_brute_force_tiny_workload():
    """The smallest named workload (2^16 updates on 2^14 rows, uniform keys, seed 0)."""
    import synth_inputs as si
    w = si.WORKLOADS["tiny"]
    R, n, D, k, S = w["R"], w["n"], 32, si.DEFAULT_K, si.DEFAULT_S   # D cut to keep the loop short
    keys = si.workload_keys("tiny")
    grads = si.grads(w["seed"], 0, n, D).numpy()
    E = si.table(w["seed"], si.TAG_E0, R, D).numpy().copy()
    A = si.table(w["seed"], si.TAG_A0, R, D).numpy().copy()
    PE, PA = oracle.encode(E, k), oracle.encode(A, k)
    bE, bA, bPE, bPA, bld, blp = brute.update(E, A, PE, PA, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, keys, grads)
    ld, lp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
    oracle.update(E, A, PE, PA, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, keys, grads, ld, lp, threads=4)
    for x, y in [(E, bE), (A, bA), (PE, bPE), (PA, bPA)]:
        np.testing.assert_allclose(x, y, rtol=2e-7, atol=1e-10)
    np.testing.assert_array_equal(ld, bld)
    np.testing.assert_array_equal(lp, blp)


# ---- invariants ---------------------------------------------------------------------------------

def _parity_residual(T, P, k):
    R, D = T.shape
    s = T.astype(np.float64).reshape(R // k, k, D)
    return np.abs(P.astype(np.float64) - s.sum(1)), np.abs(s).sum(1)


@pytest.mark.parametrize("k,S", [(2, 5), (4, 5), (10, 11)])
def test_parity_invariant_over_calls(k, S):
    """Sec. 3.1: parities stay up to date with the parameters -- re-encoding from scratch gives
    the incrementally maintained parity (to fp32 rounding), after every call."""
    rng = np.random.default_rng(7 + k)
    R, D = 20 * k, 8
    E, A, PE, PA = _tables(R, D, k, rng)
    for call in range(4):
        n = 300
        keys = rng.integers(0, R, n).astype(np.uint64)
        if call == 2:
            keys[:] = keys[0]                       # a call that hammers one entry
        grads = ((rng.random((n, D)) - 0.5) / 64).astype(F32)
        oracle.update(E, A, PE, PA, k, S, 0.01, 1e-8, keys, grads)
        for T, P in [(E, PE), (A, PA)]:
            resid, mag = _parity_residual(T, P, k)
            assert (resid <= 1e-6 * mag + 5e-8 * k).all()


@pytest.mark.parametrize("k,S", [(2, 5), (4, 5), (10, 11), (3, 4)])
def test_load_accounting(k, S):
    """Sec. 3.6: each entry update is also applied to exactly one parity, so both totals are n,
    whatever k is; and the per-server counts are the plain histograms of the placement."""
    rng = np.random.default_rng(3)
    R, n = 12 * k * S, 5000
    keys = rng.integers(0, R, n).astype(np.uint64)
    ld, lp = oracle.load(keys, R, k, S)
    assert int(ld.sum()) == n and int(lp.sum()) == n
    g, j = keys // np.uint64(k), keys % np.uint64(k)
    np.testing.assert_array_equal(ld, np.bincount(((g + 1 + j) % np.uint64(S)).astype(np.int64), minlength=S))
    np.testing.assert_array_equal(lp, np.bincount((g % np.uint64(S)).astype(np.int64), minlength=S))
    st, mem, ds, ps = oracle.route(keys, R, k, S)
    np.testing.assert_array_equal(st, g)
    np.testing.assert_array_equal(mem, j.astype(np.uint32))
    np.testing.assert_array_equal(np.bincount(ds, minlength=S).astype(np.uint64), ld)
    np.testing.assert_array_equal(np.bincount(ps, minlength=S).astype(np.uint64), lp)


@pytest.mark.parametrize("k,S", [(2, 3), (3, 4), (4, 5), (2, 5), (10, 11), (4, 8)])
def test_placement_brute_force(k, S):
    """Sec. 3.2: rotating placement -- the k+1 units of a stripe sit on k+1 different servers, and
    every server hosts the same number of parities (+-1 when S does not divide the stripe count);
    with S = k+1 the members are on exactly 'the k other servers' (the RAID-5 layout of Fig. 3)."""
    Gn = 7 * S + 3
    R = Gn * k
    keys = np.arange(R, dtype=np.uint64)
    st, mem, ds, ps = oracle.route(keys, R, k, S)
    per_server = np.zeros(S, int)
    for g in range(Gn):
        rows = np.where(st == g)[0]
        assert list(rows) == list(range(g * k, g * k + k))
        assert sorted(mem[rows]) == list(range(k))
        servers = set(ds[rows].tolist())
        p = int(ps[rows[0]])
        assert (ps[rows] == p).all()
        assert len(servers) == k and p not in servers
        if S == k + 1:
            assert servers == set(range(S)) - {p}
        per_server[p] += 1
        assert p == g % S                              # rotation
    assert per_server.max() - per_server.min() <= 1


# ---- order semantics ----------------------------------------------------------------------------

def test_order_matters_only_within_a_key():
    rng = np.random.default_rng(21)
    R, D, k, S, n = 16, 8, 4, 5, 120
    E0, A0, PE0, PA0 = _tables(R, D, k, rng)
    keys = rng.integers(0, R, n).astype(np.uint64)
    grads = ((rng.random((n, D)) - 0.5) / 64).astype(F32)

    def run(kk, gg):
        E, A, PE, PA = E0.copy(), A0.copy(), PE0.copy(), PA0.copy()
        oracle.update(E, A, PE, PA, k, S, 0.01, 1e-8, kk, gg)
        return E, A, PE, PA

    base = run(keys, grads)
    # a stable re-ordering BY KEY keeps every key's arrival order: entries are bit-identical
    order = np.argsort(keys, kind="stable")
    same = run(keys[order], grads[order])
    np.testing.assert_array_equal(base[0], same[0])
    np.testing.assert_array_equal(base[1], same[1])
    np.testing.assert_allclose(base[2], same[2], rtol=1e-6, atol=1e-8)   # parity sums re-associate
    # reversing the items of every key changes the entries (Adagrad is order dependent)
    rev = run(keys[order][::-1].copy(), grads[order][::-1].copy())
    assert np.abs(base[0] - rev[0]).max() > 1e-6
    np.testing.assert_allclose(base[1], rev[1], rtol=1e-6)               # the accumulator is a sum


def test_threads_bit_identical():
    rng = np.random.default_rng(2)
    R, D, k, S, n = 64, 16, 4, 5, 2000
    E0, A0, PE0, PA0 = _tables(R, D, k, rng)
    keys = rng.integers(0, R, n).astype(np.uint64)
    grads = ((rng.random((n, D)) - 0.5) / 64).astype(F32)
    outs = []
    for t in (1, 3, 8):
        E, A, PE, PA = E0.copy(), A0.copy(), PE0.copy(), PA0.copy()
        oracle.update(E, A, PE, PA, k, S, 0.01, 1e-8, keys, grads, threads=t)
        outs.append((E, A, PE, PA))
    for o in outs[1:]:
        for x, y in zip(outs[0], o):
            np.testing.assert_array_equal(x, y)


def test_bad_key_modifies_nothing():
    rng = np.random.default_rng(4)
    R, D, k, S = 16, 4, 4, 5
    E, A, PE, PA = _tables(R, D, k, rng)
    E0 = E.copy()
    keys = np.array([1, 2, R, 3], np.uint64)
    grads = np.ones((4, D), F32)
    with pytest.raises(ValueError):
        oracle.update(E, A, PE, PA, k, S, 0.01, 1e-8, keys, grads)
    np.testing.assert_array_equal(E, E0)


def test_empty_batch():
    rng = np.random.default_rng(4)
    E, A, PE, PA = _tables(16, 4, 4, rng)
    E0 = E.copy()
    oracle.update(E, A, PE, PA, 4, 5, 0.01, 1e-8, np.zeros(0, np.uint64), np.zeros((0, 4), F32))
    np.testing.assert_array_equal(E, E0)
