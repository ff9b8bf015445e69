"""Pins for the oracle's gradient-propagation strawman (Sec. 3.3.1) under both update rules."""
import numpy as np
import pytest

import oracle

F32 = np.float32


def _tables(rng, R, D, k):
    E = ((rng.random((R, D)) - 0.5) / 8).astype(F32)
    A = (rng.random((R, D)) * 1e-3).astype(F32)
    return E, A, oracle.encode(E, k), oracle.encode(A, k)


def test_momentum_hand_chain():
    # k = 2, one stripe, mu = 1/2, lr = 1/4; all values dyadic, so every step is exact.
    # items: (row 0, g = 1), (row 1, g = 2), (row 0, g = -1/2)
    E = np.array([[1.0], [2.0]], F32)
    V = np.array([[0.5], [0.25]], F32)
    PE, PV = np.array([[3.0]], F32), np.array([[0.75]], F32)
    keys = np.array([0, 1, 0], np.uint64)
    grads = np.array([[1.0], [2.0], [-0.5]], F32)
    oracle.update_gradient_propagation_rule(E, V, PE, PV, 2, 0.25, 0.0, keys, grads, optimizer=1, momentum=0.5)
    # entry 0: v = .5*.5+1 = 1.25, e = 1-.3125 = .6875; then v = .625-.5 = .125, e = .6875-.03125 = .65625
    # entry 1: v = .125+2 = 2.125, e = 2-.53125 = 1.46875
    # parity : v = .375+1 = 1.375, e = 3-.34375 = 2.65625; v = .6875+2 = 2.6875, e = 2.65625-.671875 = 1.984375;
    #          v = 1.34375-.5 = .84375, e = 1.984375-.2109375 = 1.7734375
    assert E[0, 0] == 0.65625 and V[0, 0] == 0.125
    assert E[1, 0] == 1.46875 and V[1, 0] == 2.125
    assert PE[0, 0] == 1.7734375 and PV[0, 0] == 0.84375
    # the parity is no longer the sum of its entries (2.125), nor its state the sum of theirs (2.25)
    assert PE[0, 0] != E[0, 0] + E[1, 0] and PV[0, 0] != V[0, 0] + V[1, 0]


def test_adagrad_hand_chain():
    # k = 2, lr = 1, eps = 0; accumulators chosen so that every square root is exact.
    # items: (row 0, g = 3), (row 1, g = 4)
    E = np.array([[10.0], [20.0]], F32)
    A = np.array([[16.0], [9.0]], F32)
    PE, PA = np.array([[30.0]], F32), np.array([[25.0]], F32)
    oracle.update_gradient_propagation_rule(E, A, PE, PA, 2, 1.0, 0.0, np.array([0, 1], np.uint64),
                                            np.array([[3.0], [4.0]], F32))
    # entry 0: A = 25, e = 10 - 3/5 = 9.4;  entry 1: A = 25, e = 20 - 4/5 = 19.2
    # parity : A = 34, e = 30 - 3/sqrt(34);  A = 50, e -= 4/sqrt(50)
    assert A[0, 0] == 25.0 and A[1, 0] == 25.0 and PA[0, 0] == 50.0
    assert E[0, 0] == F32(9.4) and E[1, 0] == F32(19.2)
    assert PE[0, 0] == pytest.approx(30.0 - 3.0 / np.sqrt(34.0) - 4.0 / np.sqrt(50.0), abs=2e-6)
    assert abs(float(PE[0, 0]) - (9.4 + 19.2)) > 0.3          # far from the sum of the entries


def test_rule_version_equals_the_pinned_strawman_for_adagrad():
    rng = np.random.default_rng(3)
    R, D, k, n = 24, 8, 4, 400
    E, A, PE, PA = _tables(rng, R, D, k)
    keys = rng.integers(0, R, n).astype(np.uint64)
    grads = ((rng.random((n, D)) - 0.5) / 64).astype(F32)
    a = [x.copy() for x in (E, A, PE, PA)]
    b = [x.copy() for x in (E, A, PE, PA)]
    oracle.update_gradient_propagation(*a, k, 0.01, 1e-8, keys, grads)
    oracle.update_gradient_propagation_rule(*b, k, 0.01, 1e-8, keys, grads, optimizer=0)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("opt", [0, 1])
def test_entries_follow_the_ordinary_rule_and_parities_break(opt):
    rng = np.random.default_rng(4 + opt)
    R, D, k, S, n = 40, 4, 4, 5, 600
    E, A, PE, PA = _tables(rng, R, D, k)
    keys = rng.integers(0, R, n).astype(np.uint64)
    grads = ((rng.random((n, D)) - 0.5) / 4).astype(F32)
    ref = [x.copy() for x in (E, A, PE, PA)]
    oracle.update_rule(*ref, k, S, 0.05, 1e-8, 0.9, opt, 0, keys, grads, np.zeros(S, np.uint64), np.zeros(S, np.uint64))
    got = [x.copy() for x in (E, A, PE, PA)]
    oracle.update_gradient_propagation_rule(*got, k, 0.05, 1e-8, keys, grads, optimizer=opt, momentum=0.9)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])     # entries and state: same training
    def resid(T, P):
        return np.abs(P.astype(np.float64) - T.astype(np.float64).reshape(R // k, k, D).sum(1)).max()
    assert resid(ref[0], ref[2]) < 1e-5 and resid(ref[1], ref[3]) < 1e-5         # difference propagation keeps the code
    assert resid(got[0], got[2]) > 1e-3                                          # the strawman does not


def test_key_out_of_range_is_refused():
    E, A, PE, PA = _tables(np.random.default_rng(0), 8, 4, 2)
    with pytest.raises(ValueError):
        oracle.update_gradient_propagation_rule(E, A, PE, PA, 2, 0.1, 0.0, np.array([8], np.uint64), np.zeros((1, 4), F32))
