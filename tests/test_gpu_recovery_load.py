"""Training while a server is rebuilt chunk by chunk (Sec. 3.4): libecrm against the protocol oracle,
with the decoder on a second stream."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from ecrm_case import Case, grads_for, log
from oracle.recovery_session import RecoverySession

pytestmark = pytest.mark.gpu


def _batch(seed, first, n, R, D, hot_rows):
    keys = si.uniform_keys(seed, first, n, R)
    for i, h in enumerate(hot_rows):                  # a few hot entries, some of them on the failed server
        keys[i::11] = h
    return keys, grads_for(seed, first, n, D)


@pytest.mark.parametrize("chunks", [1, 4, 10])
@pytest.mark.parametrize("R,D,k,S,server,opt,comb", [(4 * 3000, 128, 4, 5, 2, 0, 0), (2 * 2500, 128, 2, 5, 0, 0, 0),
                                                      (10 * 400, 256, 10, 11, 7, 0, 0), (4 * 3000, 128, 4, 5, 4, 1, 0),
                                                      (4 * 3000, 128, 4, 5, 1, 1, 0)])
def test_training_during_recovery(chunks, R, D, k, S, server, opt, comb):
    n, seed = 20000, 83
    cap = 8 * n                                       # hot lost entries of the last chunk wait through the whole recovery
    c = Case(R, D, k, S, max_batch=cap, seed=seed, optimizer=opt, momentum=0.9, combine=comb)
    st, mem, ds, ps = oracle.route(np.arange(R, dtype=np.uint64), R, k, S)
    lost_rows = np.nonzero(ds == server)[0]
    hot = [int(lost_rows[3]), int(lost_rows[len(lost_rows) // 2]), 5, int(lost_rows[-1]), R - 1]
    first = 0
    for _ in range(2):                                # some training before the failure
        keys, g = _batch(seed, first, n, R, D, hot)
        c.update(keys, g)
        first += n
    c.ctx.fail_server(server)
    oracle.fail_server(c.hE, c.hA, c.hPE, c.hPA, k, S, server)
    buf_keys = torch.empty(2 * cap, dtype=torch.int64, device="cuda")
    buf_grads = torch.empty(2 * cap, D, device="cuda")
    c.ctx.recovery_begin(server, chunks, buf_keys, buf_grads, cap)
    ses = RecoverySession(c.hE, c.hA, c.hPE, c.hPA, k, S, c.lr, c.eps, server, chunks, cap, c.hld, c.hlp,
                          optimizer=opt, momentum=0.9, combine=comb, threads=8)
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()

    def both_update():
        nonlocal first
        keys, g = _batch(seed, first, n, R, D, hot)
        first += n
        c.ctx.update(torch.from_numpy(keys.view(np.int64)).cuda(), g)
        assert ses.update(keys, g.cpu().numpy())

    max_waiting = 0
    for ch in range(ses.chunks):
        both_update()
        c.ctx.recovery_lock()
        ses.lock()
        both_update()                                  # enqueued after the lock: its chunk items wait
        ev = torch.cuda.Event()
        ev.record(main)
        side.wait_event(ev)                            # decode after everything enqueued before it ...
        c.ctx.recovery_decode(stream=side)
        done = torch.cuda.Event()
        done.record(side)
        ses.decode()
        both_update()                                  # ... and concurrently with this one
        stt = c.ctx.recovery_state()
        assert stt["active"] and stt["next_chunk"] == ch and stt["buffered"] == len(ses.buf_keys)
        max_waiting = max(max_waiting, stt["buffered"])
        main.wait_event(done)
        c.ctx.recovery_unlock()
        ses.unlock()
    stt = c.ctx.recovery_state()
    assert not stt["active"] and stt["buffered"] == 0 and max_waiting > 0
    both_update()
    log("recovery under load", (chunks, R, D, k, S, server, opt, comb), "max waiting", max_waiting, c.compare("session"))
    assert not bool(torch.isnan(c.E).any()) and not bool(torch.isnan(c.PA).any())
    c.check_invariant()


def test_recovery_buffer_overflow_and_state_errors():
    R, D, k, S, n, server = 4 * 1000, 128, 4, 5, 8000, 3
    c = Case(R, D, k, S, max_batch=n, seed=89)
    keys = si.uniform_keys(89, 0, n, R)
    g = grads_for(89, 0, n, D)
    kt = torch.from_numpy(keys.view(np.int64)).cuda()
    cap = 64
    buf_keys = torch.empty(2 * cap, dtype=torch.int64, device="cuda")
    buf_grads = torch.empty(2 * cap, D, device="cuda")
    assert c.ctx.recovery_lock(check=False) == -8                  # no recovery in progress
    assert c.ctx.recovery_begin(9, 2, buf_keys, buf_grads, cap, check=False) == -1
    assert c.ctx.recovery_begin(server, 0, buf_keys, buf_grads, cap, check=False) == -1
    assert c.ctx.recovery_begin(server, 2, buf_keys, buf_grads, n + 1, check=False) == -1
    c.ctx.recovery_begin(server, 2, buf_keys, buf_grads, cap)
    assert c.ctx.recovery_begin(server, 2, buf_keys, buf_grads, cap, check=False) == -8
    assert c.ctx.recovery_decode(check=False) == -8                 # nothing locked
    lib, raw = c.ctx._lib, c.ctx._ctx
    assert lib.ecrm_encode(raw, None) == -8                         # no second loss, full rebuild or re-encoding
    assert lib.ecrm_fail_server(raw, 1, None) == -8                 # while the chunked protocol runs
    assert lib.ecrm_recover_server(raw, server, None) == -8
    assert c.ctx.recovery_unlock(check=False) == -8
    c.ctx.recovery_lock()
    assert c.ctx.recovery_lock(check=False) == -8
    assert c.ctx.recovery_unlock(check=False) == -8                 # nothing has been decoded under this lock
    assert c.ctx.bind_raw(c.E.data_ptr(), c.A.data_ptr(), c.PE.data_ptr(), c.PA.data_ptr(), c.ld.data_ptr(),
                          c.lp.data_ptr(), c.scratch.data_ptr(), c.scratch.numel()) == -8   # would drop the buffer
    before = [t.clone() for t in (c.E, c.A, c.PE, c.PA, c.ld, c.lp)]
    c.ctx.update(kt, g)                                             # far more than 64 items have to wait
    assert c.ctx.status() == -7                                     # ECRM_EBUFFER
    assert c.ctx.batch_stats()["rejected"] == 1
    for t, b in zip((c.E, c.A, c.PE, c.PA, c.ld, c.lp), before):
        assert torch.equal(t, b)
    assert c.ctx.recovery_state()["buffered"] == 0
    c.ctx.clear_status()
    # a batch that fits: 10 items of the locked chunk
    st = keys // np.uint64(k)
    small = keys[st < 100][:10].copy()
    c.ctx.update(torch.from_numpy(small.view(np.int64)).cuda(), g[:10].contiguous())
    assert c.ctx.status() == 0
    assert 0 < c.ctx.recovery_state()["buffered"] <= 10


@pytest.mark.parametrize("chunks", [1, 4])
@pytest.mark.parametrize("R,D,k,S,server,opt,comb", [(4 * 3000, 128, 4, 5, 2, 0, 0), (10 * 400, 256, 10, 11, 7, 1, 0),
                                                      (2 * 2500, 36, 2, 5, 0, 1, 0)])
def test_reads_during_recovery(chunks, R, D, k, S, server, opt, comb):
    """ecrm_recovery_read against the protocol oracle's read at every stage (before a lock, under it,
    after the decode, after the unlock), and against the tables the replay leaves behind."""
    n, seed = 12000, 97
    cap = 8 * n
    c = Case(R, D, k, S, max_batch=cap, seed=seed, optimizer=opt, momentum=0.9, combine=comb)
    st, mem, ds, ps = oracle.route(np.arange(R, dtype=np.uint64), R, k, S)
    lost_rows = np.nonzero(ds == server)[0]
    hot = [int(lost_rows[3]), int(lost_rows[len(lost_rows) // 2]), 5, int(lost_rows[-1]), R - 1]
    first = 0
    keys, g = _batch(seed, first, n, R, D, hot)
    c.update(keys, g)
    first += n
    c.ctx.fail_server(server)
    oracle.fail_server(c.hE, c.hA, c.hPE, c.hPA, k, S, server)
    buf_keys = torch.empty(2 * cap, dtype=torch.int64, device="cuda")
    buf_grads = torch.empty(2 * cap, D, device="cuda")
    c.ctx.recovery_begin(server, chunks, buf_keys, buf_grads, cap)
    ses = RecoverySession(c.hE, c.hA, c.hPE, c.hPA, k, S, c.lr, c.eps, server, chunks, cap, c.hld, c.hlp,
                          optimizer=opt, momentum=0.9, combine=comb, threads=8)
    rng = np.random.default_rng(1)
    sample = np.unique(np.concatenate([np.array(hot), rng.integers(0, R, 120), rng.choice(lost_rows, 80),
                                       np.arange(0, min(R, 40 * k))])).astype(np.uint64)
    sample_t = torch.from_numpy(sample.view(np.int64)).cuda()
    oe = torch.empty(len(sample), D, device="cuda")
    oa = torch.empty(len(sample), D, device="cuda")

    def both_update():
        nonlocal first
        keys, g = _batch(seed, first, n, R, D, hot)
        first += n
        c.ctx.update(torch.from_numpy(keys.view(np.int64)).cuda(), g)
        assert ses.update(keys, g.cpu().numpy())

    def both_read(stage):
        c.ctx.recovery_read(sample_t, oe, oa)
        hE, hA = ses.read(sample)
        assert c.ctx.status() == 0
        assert not bool(torch.isnan(oe).any())
        np.testing.assert_allclose(oe.cpu().numpy(), hE, rtol=1e-4, atol=5e-6, err_msg=stage)
        np.testing.assert_allclose(oa.cpu().numpy(), hA, rtol=1e-4, atol=2e-9, err_msg=stage)

    both_read("right after the failure")
    for ch in range(ses.chunks):
        both_update()
        both_read(f"chunk {ch}: before the lock")
        c.ctx.recovery_lock()
        ses.lock()
        both_update()
        both_read(f"chunk {ch}: locked")
        c.ctx.recovery_decode()
        ses.decode()
        both_update()
        both_read(f"chunk {ch}: decoded")
        seen_e, seen_a = oe.clone(), oa.clone()
        c.ctx.recovery_unlock()
        ses.unlock()
        both_read(f"chunk {ch}: released")
        # what was read from the buffer is what the replay wrote (a long chain is summed piecewise there)
        assert torch.allclose(seen_e, oe, rtol=1e-6, atol=1e-9) and torch.allclose(seen_a, oa, rtol=1e-6, atol=1e-12)
        assert int((seen_e != oe).sum()) <= 1e-3 * oe.numel()
        lo, hi = ch * ses.spc * k, min((ch + 1) * ses.spc * k, R)
        inside = torch.from_numpy(((sample >= lo) & (sample < hi))).cuda()
        rows = sample_t[inside]
        assert torch.equal(c.E[rows], oe[inside]) and torch.equal(c.A[rows], oa[inside])
    assert not c.ctx.recovery_state()["active"]
    both_update()
    both_read("after the recovery")                     # a plain gather again
    assert torch.equal(c.E[sample_t], oe)
    log("reads during recovery", (chunks, R, D, k, S, server, opt, comb), c.compare("session reads"))


def test_no_recovery_protocol_for_combined_training():
    """Synchronous training takes one step per entry and training step (Sec. 4.4); a replayed buffer would
    merge several steps into one, so the library refuses to start the protocol in that mode."""
    c = Case(4 * 100, 128, 4, 5, max_batch=100, seed=3, combine=1)
    bk = torch.empty(200, dtype=torch.int64, device="cuda")
    bg = torch.empty(200, 128, device="cuda")
    assert c.ctx.recovery_begin(1, 2, bk, bg, 100, check=False) == -1


def test_recovery_read_errors():
    c = Case(4 * 100, 128, 4, 5, max_batch=100, seed=3)
    kt = torch.tensor([1, 2, 400], dtype=torch.int64, device="cuda")
    oe = torch.full((3, 128), 7.0, device="cuda")
    c.ctx.recovery_read(kt, oe)
    assert c.ctx.status() == -5                          # a key >= rows
    assert torch.equal(oe[0], c.E[1]) and torch.equal(oe[1], c.E[2]) and bool((oe[2] == 7.0).all())
    c.ctx.clear_status()
