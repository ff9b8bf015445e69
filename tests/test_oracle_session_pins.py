"""Pins for the recovery-under-load protocol oracle (Sec. 3.4 "Training during recovery")."""
import numpy as np
import pytest

import oracle
from oracle.recovery_session import RecoverySession

F32 = np.float32


def _setup(R, D, k, S, seed):
    rng = np.random.default_rng(seed)
    E = ((rng.random((R, D)) - 0.5) / 8).astype(F32)
    A = (rng.random((R, D)) * 1e-3).astype(F32)
    return rng, E, A, oracle.encode(E, k), oracle.encode(A, k)


def _batch(rng, R, D, n, hot=None):
    keys = rng.integers(0, R, n).astype(np.uint64)
    if hot is not None:
        keys[::3] = hot
    return keys, ((rng.random((n, D)) - 0.5) / 64).astype(F32)


@pytest.mark.parametrize("chunks", [1, 3, 10])
@pytest.mark.parametrize("k,S", [(4, 5), (2, 5)])
def test_training_through_a_recovery_equals_instant_recovery(chunks, k, S):
    """Whatever the chunking, once everything is rebuilt and replayed the model is the one an instant
    recovery at the moment of the failure would have led to -- up to the roundings of the stored sums
    (the decoder runs at different moments, on parities that have been rounded a different number of
    times).  No update is lost, none is applied twice (the load counters say so exactly)."""
    R, D, server = k * 60, 8, 2
    rng, E, A, PE, PA = _setup(R, D, k, S, seed=chunks * 10 + k)
    batches = [_batch(rng, R, D, 400, hot=np.uint64((server + S - 1) % S if k > 1 else 0)) for _ in range(3 * chunks + 2)]
    # reference: fail, recover everything at once, then train
    rE, rA, rPE, rPA = E.copy(), A.copy(), PE.copy(), PA.copy()
    rld, rlp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
    oracle.fail_server(rE, rA, rPE, rPA, k, S, server)
    oracle.recover_server(rE, rA, rPE, rPA, k, S, server)
    for kk, gg in batches:
        oracle.update(rE, rA, rPE, rPA, k, S, 0.01, 1e-8, kk, gg, rld, rlp)
    # the protocol
    ld, lp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
    oracle.fail_server(E, A, PE, PA, k, S, server)
    ses = RecoverySession(E, A, PE, PA, k, S, 0.01, 1e-8, server, chunks, capacity=10000, load_data=ld, load_parity=lp)
    it = iter(batches)
    waiting_seen = 0
    for c in range(ses.chunks):
        assert ses.update(*next(it))
        ses.lock()
        assert ses.update(*next(it))
        ses.decode()
        assert ses.update(*next(it))
        waiting_seen = max(waiting_seen, len(ses.buf_keys))
        ses.unlock()
    assert not ses.active and len(ses.buf_keys) == 0 and waiting_seen > 0
    for b in it:
        assert ses.update(*b)
    assert not np.isnan(E).any() and not np.isnan(PA).any()
    np.testing.assert_array_equal(ld, rld)
    np.testing.assert_array_equal(lp, rlp)
    # a decoded accumulator carries the rounding of its parity (absolute ~1e-10), which is a large
    # RELATIVE change when the accumulator itself is tiny, and Adagrad's step depends on it
    for x, y, atol in ((E, rE, 5e-6), (A, rA, 2e-9), (PE, rPE, 1e-5), (PA, rPA, 4e-9)):
        np.testing.assert_allclose(x, y, rtol=1e-4, atol=atol)
    # and the parity invariant holds at the end
    np.testing.assert_allclose(PE, E.astype(np.float64).reshape(R // k, k, D).sum(1), rtol=1e-5, atol=1e-6)


def test_what_waits_is_exactly_what_the_paper_says():
    k, S, R, server = 4, 5, 4 * 50, 3
    rng, E, A, PE, PA = _setup(R, 4, k, S, seed=1)
    ses = RecoverySession(E, A, PE, PA, k, S, 0.01, 1e-8, server, chunks=5, capacity=10 ** 6)
    keys = np.arange(R, dtype=np.uint64)
    st, mem, ds, ps = oracle.route(keys, R, k, S)
    # nothing locked: only the lost entries themselves wait
    np.testing.assert_array_equal(ses.held(keys), ds == server)
    ses.lock()                                              # chunk 0 = stripes [0, 10)
    h = ses.held(keys)
    in_chunk = st < 10
    affected = (ds.reshape(-1, k) == server).any(1) | (ps.reshape(-1, k)[:, 0] == server)
    np.testing.assert_array_equal(h, (in_chunk & np.repeat(affected, k)) | (ds == server))
    ses.decode()
    ses.unlock()                                            # chunk 0 rebuilt: its entries are free again
    h = ses.held(keys)
    assert not h[in_chunk].any()
    np.testing.assert_array_equal(h[~in_chunk], (ds == server)[~in_chunk])


def test_full_buffer_rejects_the_batch():
    k, S, R, server = 4, 5, 4 * 20, 1
    rng, E, A, PE, PA = _setup(R, 4, k, S, seed=2)
    ses = RecoverySession(E, A, PE, PA, k, S, 0.01, 1e-8, server, chunks=1, capacity=5)
    ses.lock()
    E0 = E.copy()
    keys, grads = _batch(rng, R, 4, 200)
    assert not ses.update(keys, grads)
    np.testing.assert_array_equal(E, E0)
    assert len(ses.buf_keys) == 0
