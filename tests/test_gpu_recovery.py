"""GPU parity of the recovery entry points against the oracle (bit-exact: both sides take the sums
in fp64 in the same order and round once)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from ecrm_case import Case, grads_for, log

pytestmark = pytest.mark.gpu


def _trained_case(R, D, k, S, n, seed):
    c = Case(R, D, k, S, max_batch=n, seed=seed)
    for call in range(2):
        c.update(si.uniform_keys(seed, call * n, n, R), grads_for(seed, call * n, n, D))
    c.compare("trained")
    return c


@pytest.mark.parametrize("R,D,k,S", [(4 * 2000, 128, 4, 5), (2 * 1500, 128, 2, 5), (10 * 300, 256, 10, 11),
                                     (3 * 700, 36, 3, 4), (64 * 20, 1024, 64, 65), (4 * 100, 4, 4, 9),
                                     (500, 128, 1, 2)])
def test_fail_and_recover_every_server(R, D, k, S):
    c = _trained_case(R, D, k, S, 20000, seed=51)
    for server in range(S):
        before = [t.clone() for t in (c.E, c.A, c.PE, c.PA)]
        c.ctx.fail_server(server)
        oracle.fail_server(c.hE, c.hA, c.hPE, c.hPA, k, S, server)
        # the same units are lost on both sides
        for dev, host in ((c.E, c.hE), (c.A, c.hA), (c.PE, c.hPE), (c.PA, c.hPA)):
            np.testing.assert_array_equal(torch.isnan(dev).cpu().numpy(), np.isnan(host))
        assert bool(torch.isnan(c.E).any()) or bool(torch.isnan(c.PE).any())
        c.ctx.recover_server(server)
        oracle.recover_server(c.hE, c.hA, c.hPE, c.hPA, k, S, server)
        assert c.ctx.status() == 0
        for dev, host in ((c.E, c.hE), (c.A, c.hA), (c.PE, c.hPE), (c.PA, c.hPA)):
            np.testing.assert_array_equal(dev.cpu().numpy(), host)
        # and what came back is the lost data up to the roundings of the stored sums
        for new, old in zip((c.E, c.A, c.PE, c.PA), before):
            assert torch.allclose(new, old, rtol=2e-6, atol=2e-7)
    c.check_invariant()


def test_training_continues_after_recovery():
    R, D, k, S, n = 4 * 3000, 128, 4, 5, 30000
    c = _trained_case(R, D, k, S, n, seed=53)
    c.ctx.fail_server(3)
    c.ctx.recover_server(3)
    oracle.fail_server(c.hE, c.hA, c.hPE, c.hPA, k, S, 3)
    oracle.recover_server(c.hE, c.hA, c.hPE, c.hPA, k, S, 3)
    c.update(si.uniform_keys(53, 5 * n, n, R), grads_for(53, 5 * n, n, D))
    log("after recovery", c.compare("after recovery"))
    c.check_invariant()


@pytest.mark.parametrize("R,D,k,S", [(4 * 2000, 128, 4, 5), (10 * 300, 256, 10, 11), (2 * 999, 36, 2, 5)])
def test_degraded_read(R, D, k, S):
    c = _trained_case(R, D, k, S, 20000, seed=57)
    n = 30011
    keys = si.uniform_keys(58, 0, n, R)
    kt = torch.from_numpy(keys.view(np.int64)).cuda()
    oe, oa = torch.empty(n, D, device="cuda"), torch.empty(n, D, device="cuda")
    # nobody down: a plain gather
    c.ctx.degraded_read(kt, None, oe, oa)
    assert torch.equal(oe, c.E[kt]) and torch.equal(oa, c.A[kt])
    plain = oe.clone()
    for lost in range(S):
        c.ctx.fail_server(lost)
        oracle.fail_server(c.hE, c.hA, c.hPE, c.hPA, k, S, lost)
        oe.fill_(-7.0)
        oa.fill_(-7.0)
        c.ctx.degraded_read(kt, lost, oe, oa)
        he, ha = oracle.degraded_read(c.hE, c.hA, c.hPE, c.hPA, k, S, keys, lost)
        np.testing.assert_array_equal(oe.cpu().numpy(), he)
        np.testing.assert_array_equal(oa.cpu().numpy(), ha)
        assert not bool(torch.isnan(oe).any())
        assert torch.allclose(oe, plain, rtol=2e-6, atol=2e-7)
        # only E, no accumulators
        oe2 = torch.empty_like(oe)
        c.ctx.degraded_read(kt, lost, oe2, None)
        assert torch.equal(oe2, oe)
        c.ctx.recover_server(lost)
        oracle.recover_server(c.hE, c.hA, c.hPE, c.hPA, k, S, lost)
    assert c.ctx.status() == 0


def test_recovery_argument_errors():
    R, D, k, S = 4 * 100, 128, 4, 5
    c = Case(R, D, k, S, max_batch=16, seed=1)
    lib, ctx = c.ctx._lib, c.ctx._ctx
    assert lib.ecrm_fail_server(ctx, 5, None) == -1
    assert lib.ecrm_recover_server(ctx, 99, None) == -1
    keys = torch.tensor([1, 2, R, 3], dtype=torch.int64, device="cuda")
    out = torch.full((4, D), -1.0, device="cuda")
    assert c.ctx.degraded_read(keys, 7, out, check=False) == -1
    c.ctx.degraded_read(keys, 2, out)
    assert c.ctx.status() == -5                      # the bad key is reported, its row left alone
    assert bool((out[2] == -1.0).all()) and not bool((out[[0, 1, 3]] == -1.0).all())
    assert c.ctx.degraded_read(keys[:0], None, out, check=False) == 0
