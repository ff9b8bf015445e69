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


# ---- reads during the recovery (Sec. 3.4: a locked entry updated meanwhile is served from the buffer) ----

def _reference_after(E0, A0, PE0, PA0, k, S, server, batches):
    """fail, rebuild everything at once, then apply the batches: what a worker should see"""
    rE, rA, rPE, rPA = E0.copy(), A0.copy(), PE0.copy(), PA0.copy()
    oracle.fail_server(rE, rA, rPE, rPA, k, S, server)
    oracle.recover_server(rE, rA, rPE, rPA, k, S, server)
    for kk, gg in batches:
        oracle.update(rE, rA, rPE, rPA, k, S, 0.01, 1e-8, kk, gg)
    return rE, rA


@pytest.mark.parametrize("chunks", [1, 4])
def test_a_reader_never_notices_the_recovery(chunks):
    """At every point of the protocol -- before a lock, under it, after the decode, after the unlock --
    reading all entries gives what training without a failure would have given (to the roundings of
    the stored sums): waiting updates are seen, lost entries are decoded, nothing is seen twice."""
    k, S, R, D, server = 4, 5, 4 * 40, 8, 2
    rng, E, A, PE, PA = _setup(R, D, k, S, seed=77 + chunks)
    E0, A0, PE0, PA0 = E.copy(), A.copy(), PE.copy(), PA.copy()
    oracle.fail_server(E, A, PE, PA, k, S, server)
    ses = RecoverySession(E, A, PE, PA, k, S, 0.01, 1e-8, server, chunks, capacity=10 ** 6)
    allkeys = np.arange(R, dtype=np.uint64)
    done, saw_waiting = [], False

    def check():
        rE, rA = _reference_after(E0, A0, PE0, PA0, k, S, server, done)
        gE, gA = ses.read(allkeys)
        np.testing.assert_allclose(gE, rE, rtol=1e-4, atol=5e-6)
        np.testing.assert_allclose(gA, rA, rtol=1e-4, atol=2e-9)

    check()
    for c in range(ses.chunks):
        for stage in ("before", "locked", "decoded"):
            if stage == "locked":
                ses.lock()
            if stage == "decoded":
                ses.decode()
            b = _batch(rng, R, D, 300, hot=np.uint64(5))
            assert ses.update(*b)
            done.append(b)
            saw_waiting |= len(ses.buf_keys) > 0
            check()
        ses.unlock()
        check()
    assert saw_waiting and not ses.active


def test_read_before_unlock_is_the_entry_after_unlock():
    """The value read from the buffer is bit for bit the one the replay writes."""
    k, S, R, D, server = 4, 5, 4 * 30, 4, 0
    rng, E, A, PE, PA = _setup(R, D, k, S, seed=5)
    oracle.fail_server(E, A, PE, PA, k, S, server)
    ses = RecoverySession(E, A, PE, PA, k, S, 0.01, 1e-8, server, chunks=3, capacity=10 ** 6)
    allkeys = np.arange(R, dtype=np.uint64)
    for c in range(ses.chunks):
        ses.lock()
        assert ses.update(*_batch(rng, R, D, 500))
        ses.decode()
        assert ses.update(*_batch(rng, R, D, 500))
        before_E, before_A = ses.read(allkeys)
        ses.unlock()
        after_E, after_A = ses.read(allkeys)
        np.testing.assert_array_equal(before_E, after_E)
        np.testing.assert_array_equal(before_A, after_A)
        lo, hi = c * ses.spc * k, min((c + 1) * ses.spc * k, R)       # the released chunk is now in the tables
        np.testing.assert_array_equal(E[lo:hi], after_E[lo:hi])
        np.testing.assert_array_equal(A[lo:hi], after_A[lo:hi])


def test_read_without_waiting_updates_is_the_table_or_the_decoded_entry():
    k, S, R, D, server = 2, 5, 2 * 40, 4, 3
    rng, E, A, PE, PA = _setup(R, D, k, S, seed=6)
    E0 = E.copy()
    oracle.fail_server(E, A, PE, PA, k, S, server)
    ses = RecoverySession(E, A, PE, PA, k, S, 0.01, 1e-8, server, chunks=2, capacity=10)
    allkeys = np.arange(R, dtype=np.uint64)
    gE, _ = ses.read(allkeys)
    _, _, ds, _ = oracle.route(allkeys, R, k, S)
    lost = ds == server
    assert lost.any() and np.isnan(E[lost]).all()
    np.testing.assert_array_equal(gE[~lost], E0[~lost])                   # survivors: the table itself
    np.testing.assert_allclose(gE[lost], E0[lost], rtol=0, atol=2e-7)     # lost ones: decoded, to one rounding of the sum
    with pytest.raises(ValueError):                                       # synchronous training: steps must not be merged
        RecoverySession(E.copy(), A.copy(), PE.copy(), PA.copy(), k, S, 0.01, 1e-8, server, 2, 100, combine=1)
    for m in ("optimizer",):                                              # momentum SGD goes through the same door
        ses2 = RecoverySession(E.copy(), A.copy(), PE.copy(), PA.copy(), k, S, 0.01, 1e-8, server, 2, 100,
                               optimizer=1, momentum=0.9, combine=0)
        ses2.lock()
        kk, gg = _batch(rng, R, D, 50)
        assert ses2.update(kk, gg)
        rE, rA = ses2.read(allkeys)
        ses2.decode()
        ses2.unlock()
        r2E, r2A = ses2.read(allkeys)
        np.testing.assert_array_equal(rE, r2E)
