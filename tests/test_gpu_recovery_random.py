"""Seeded random recovery-under-load protocols (Sec. 3.4): random geometry, failed server, number of
chunks, rule, and a random number of update batches and reads between the protocol's steps -- libecrm
against the protocol oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from ecrm_case import Case, grads_for, log
from oracle.recovery_session import RecoverySession

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", range(10))
def test_random_protocol(case):
    rng = np.random.default_rng(777 + case)
    k = int(rng.choice([1, 2, 3, 4, 10]))
    S = k + 1 + int(rng.integers(0, 3))
    D = int(rng.choice([36, 128, 256]))
    R = k * int(rng.integers(50, 2500))
    chunks, server = int(rng.integers(1, 13)), int(rng.integers(0, S))
    opt, comb = int(rng.integers(0, 2)), int(rng.integers(0, 2)) * 0     # the draw is kept so that the cases stay what they were; combined training has no recovery protocol
    n, seed = int(rng.choice([1, 700, 5000, 6145, 20000])), 3000 + case
    cap = 40 * n + 64
    c = Case(R, D, k, S, max_batch=cap, seed=seed, optimizer=opt, momentum=0.9, combine=comb)
    _, _, ds, _ = oracle.route(np.arange(R, dtype=np.uint64), R, k, S)
    lost = np.nonzero(ds == server)[0]
    hot = [int(lost[0]), int(lost[-1]), int(rng.integers(0, R))] if len(lost) else [0, 1, 2]
    first = 0

    def batch():
        nonlocal first
        keys = si.uniform_keys(seed, first, n, R)
        for i, h in enumerate(hot):
            keys[i::9] = h
        g = grads_for(seed, first, n, D)
        first += n
        return keys, g

    c.update(*batch())
    c.ctx.fail_server(server)
    oracle.fail_server(c.hE, c.hA, c.hPE, c.hPA, k, S, server)
    bk = torch.empty(2 * cap, dtype=torch.int64, device="cuda")
    bg = torch.empty(2 * cap, D, device="cuda")
    c.ctx.recovery_begin(server, chunks, bk, bg, cap)
    ses = RecoverySession(c.hE, c.hA, c.hPE, c.hPA, k, S, c.lr, c.eps, server, chunks, cap, c.hld, c.hlp,
                          optimizer=opt, momentum=0.9, combine=comb, threads=8)
    side, main = torch.cuda.Stream(), torch.cuda.current_stream()
    sample = np.unique(np.concatenate([np.array(hot), rng.integers(0, R, 60), lost[:40]])).astype(np.uint64)
    sample_t = torch.from_numpy(sample.view(np.int64)).cuda()
    oe = torch.empty(len(sample), D, device="cuda")
    oa = torch.empty(len(sample), D, device="cuda")

    def upd():
        keys, g = batch()
        c.ctx.update(torch.from_numpy(keys.view(np.int64)).cuda(), g)
        assert ses.update(keys, g.cpu().numpy())

    def read(tag):
        c.ctx.recovery_read(sample_t, oe, oa)
        hE, hA = ses.read(sample)
        np.testing.assert_allclose(oe.cpu().numpy(), hE, rtol=1e-4, atol=5e-6, err_msg=tag)
        np.testing.assert_allclose(oa.cpu().numpy(), hA, rtol=1e-4, atol=2e-9, err_msg=tag)

    for ch in range(ses.chunks):
        for _ in range(int(rng.integers(0, 3))):
            upd()
        c.ctx.recovery_lock()
        ses.lock()
        for _ in range(int(rng.integers(0, 3))):
            upd()
        if rng.random() < 0.5:
            read(f"chunk {ch} locked")
        if rng.random() < 0.5:                       # the decoder on a second stream, updates beside it
            ev = torch.cuda.Event()
            ev.record(main)
            side.wait_event(ev)
            c.ctx.recovery_decode(stream=side)
            done = torch.cuda.Event()
            done.record(side)
            ses.decode()
            for _ in range(int(rng.integers(0, 3))):
                upd()
            main.wait_event(done)
        else:
            c.ctx.recovery_decode()
            ses.decode()
            for _ in range(int(rng.integers(0, 3))):
                upd()
            if rng.random() < 0.5:
                read(f"chunk {ch} decoded")
        assert c.ctx.recovery_state()["buffered"] == len(ses.buf_keys)
        c.ctx.recovery_unlock()
        ses.unlock()
        if rng.random() < 0.3:
            read(f"chunk {ch} released")
    assert not c.ctx.recovery_state()["active"]
    upd()
    log("random protocol", case, (R, D, k, S, server, ses.chunks, n, opt, comb), c.compare(f"protocol {case}"))
    assert not bool(torch.isnan(c.E).any()) and not bool(torch.isnan(c.PA).any())
