"""Pins for the oracle's recovery functions (Sec. 3.4 of the ECRM paper; decoder of Sec. 3.2)."""
import numpy as np
import pytest

import oracle

F32 = np.float32


def _dyadic_tables(R, D, k, rng):
    E = (rng.integers(-512, 512, (R, D)) / 64.0).astype(F32)
    A = (rng.integers(0, 1024, (R, D)) / 128.0).astype(F32)
    return E, A, oracle.encode(E, k), oracle.encode(A, k)


def test_golden_k3_lose_each_server(golden):
    """The paper's example: p = e1 + e2 + e3 on four servers; whichever server fails, what it held
    comes back exactly (dyadic values)."""
    g = golden("sum_code_k3.txt")
    E0 = np.array([g["e1"], g["e2"], g["e3"]], F32)
    A0 = np.abs(E0) * F32(2)
    PE0, PA0 = oracle.encode(E0, 3), oracle.encode(A0, 3)
    np.testing.assert_array_equal(PE0[0], np.array(g["p"], F32))
    for server in range(4):
        E, A, PE, PA = E0.copy(), A0.copy(), PE0.copy(), PA0.copy()
        oracle.fail_server(E, A, PE, PA, 3, 4, server)
        lost = np.isnan(E).any(1).sum() + np.isnan(PE).any(1).sum()
        assert lost == 1                                   # stripe 0 has one unit on every one of the 4 servers
        oracle.recover_server(E, A, PE, PA, 3, 4, server)
        for x, y in ((E, E0), (A, A0), (PE, PE0), (PA, PA0)):
            np.testing.assert_array_equal(x, y)
    # the layout itself: parity of stripe 0 on server 0, e1, e2, e3 on servers 1, 2, 3
    E, A, PE, PA = E0.copy(), A0.copy(), PE0.copy(), PA0.copy()
    oracle.fail_server(E, A, PE, PA, 3, 4, 2)
    assert np.isnan(E[1]).all() and not np.isnan(E[[0, 2]]).any() and not np.isnan(PE).any()


@pytest.mark.parametrize("k,S", [(2, 3), (2, 5), (4, 5), (10, 11), (3, 7)])
def test_any_single_server_loss_is_recovered_exactly(k, S):
    """Sec. 2.4: any k of the k+1 units of a stripe suffice -- for every server, on dyadic values."""
    rng = np.random.default_rng(k * 100 + S)
    R, D = k * (3 * S + 2), 8
    E0, A0, PE0, PA0 = _dyadic_tables(R, D, k, rng)
    for server in range(S):
        E, A, PE, PA = E0.copy(), A0.copy(), PE0.copy(), PA0.copy()
        oracle.fail_server(E, A, PE, PA, k, S, server)
        # what is lost is exactly what the placement puts on that server
        st, mem, ds, ps = oracle.route(np.arange(R, dtype=np.uint64), R, k, S)
        np.testing.assert_array_equal(np.isnan(E).all(1), ds == server)
        np.testing.assert_array_equal(np.isnan(PE).all(1), (np.arange(R // k) % S) == server)
        oracle.recover_server(E, A, PE, PA, k, S, server)
        for x, y in ((E, E0), (A, A0), (PE, PE0), (PA, PA0)):
            np.testing.assert_array_equal(x, y)


def test_recovery_after_updates_is_within_rounding():
    """After training steps the stored parity and the stored entries are each rounded to fp32 once per
    call, so a decoded entry equals the lost one up to those roundings: after c calls
    |err| <= (c+1) * 2^-24 * (|parity| + sum of |entries| of the stripe)."""
    rng = np.random.default_rng(8)
    R, D, k, S = 4 * 50, 16, 4, 5
    E = ((rng.random((R, D)) - 0.5) / 8).astype(F32)
    A = (rng.random((R, D)) * 1e-3).astype(F32)
    PE, PA = oracle.encode(E, k), oracle.encode(A, k)
    for _ in range(3):
        keys = rng.integers(0, R, 400).astype(np.uint64)
        grads = ((rng.random((400, D)) - 0.5) / 64).astype(F32)
        oracle.update(E, A, PE, PA, k, S, 0.01, 1e-8, keys, grads)
    E0, A0, PE0, PA0 = E.copy(), A.copy(), PE.copy(), PA.copy()
    for server in range(S):
        E, A, PE, PA = E0.copy(), A0.copy(), PE0.copy(), PA0.copy()
        oracle.fail_server(E, A, PE, PA, k, S, server)
        oracle.recover_server(E, A, PE, PA, k, S, server)
        assert not np.isnan(E).any() and not np.isnan(PA).any()
        calls = 3
        for T, T0, P0 in ((E, E0, PE0), (A, A0, PA0)):
            mag = np.abs(P0) + np.abs(T0).reshape(R // k, k, D).sum(1)
            bound = (calls + 1) * 2.0 ** -24 * mag + 1e-12
            assert (np.abs(T - T0) <= np.repeat(bound, k, axis=0)).all()
        assert (np.abs(PE - PE0) <= (calls + 1) * 2.0 ** -24 * (np.abs(PE0) + np.abs(E0).reshape(R // k, k, D).sum(1)) + 1e-12).all()


def test_degraded_read_equals_plain_read_on_dyadic_values():
    rng = np.random.default_rng(3)
    R, D, k, S = 4 * 30, 8, 4, 5
    E, A, PE, PA = _dyadic_tables(R, D, k, rng)
    keys = rng.integers(0, R, 500).astype(np.uint64)
    plain_e, plain_a = oracle.degraded_read(E, A, PE, PA, k, S, keys, S + 7)      # nobody down
    np.testing.assert_array_equal(plain_e, E[keys.astype(np.int64)])
    for lost in range(S):
        Ef, Af, PEf, PAf = E.copy(), A.copy(), PE.copy(), PA.copy()
        oracle.fail_server(Ef, Af, PEf, PAf, k, S, lost)
        de, da = oracle.degraded_read(Ef, Af, PEf, PAf, k, S, keys, lost)
        np.testing.assert_array_equal(de, plain_e)           # never touches the NaN rows, decodes exactly
        np.testing.assert_array_equal(da, plain_a)


def test_stale_parity_decodes_the_old_value():
    """Appendix, Table 1: if the difference of an update has not reached the parity when the server
    fails, decoding gives back the entry as of the last difference the parity has seen."""
    E = np.array([[1.0], [2.0], [4.0]], F32)
    A = np.array([[0.5], [0.25], [0.125]], F32)
    PE, PA = oracle.encode(E, 3), oracle.encode(A, 3)
    E_new = E.copy()
    E_new[0, 0] = 0.75                       # entry updated on its server, parity not yet
    oracle.fail_server(E_new, A, PE, PA, 3, 4, 1)          # server 1 holds member 0 of stripe 0
    oracle.recover_server(E_new, A, PE, PA, 3, 4, 1)
    assert E_new[0, 0] == 1.0                # x_t, not x_{t+1}
