"""ecrm_update_static (the entry point for callers that cannot allocate: its scratch buffer is a fixed
array inside the library) against ecrm_update on the same inputs, through the C ABI: two calls in a row,
the second with a smaller batch, so that what the first call left in the shared array is there when the
second one runs."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from ecrm_case import ATOL_A, ATOL_E, RTOL, log
from paper_2104_01981_amd import Ecrm

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _tables(R, D, k, S, seed):
    E = si.table(seed, si.TAG_E0, R, D, DEV)
    A = si.table(seed, si.TAG_A0, R, D, DEV)
    PE, PA = torch.zeros(R // k, D, device=DEV), torch.zeros(R // k, D, device=DEV)
    ld = torch.zeros(S, dtype=torch.int64, device=DEV)
    lp = torch.zeros(S, dtype=torch.int64, device=DEV)
    return E, A, PE, PA, ld, lp


def _batches(R, D, seed, sizes):
    out, first = [], 0
    for n in sizes:
        keys = si.uniform_keys(seed, first, n, R)
        keys[1::3] = 77                      # one hot entry: the split-chain buffers of the array are used too
        keys[2::7] = R - 1
        out.append((torch.from_numpy(keys.view(np.int64)).to(DEV), si.grads(seed, first, n, D, DEV)))
        first += n
    return out


@pytest.mark.parametrize("R,D,k,S,opt,prop", [(4 * 4096, 128, 4, 5, 0, 0), (2 * 3000, 256, 2, 5, 1, 0),
                                              (10 * 500, 36, 10, 11, 0, 0), (4 * 2048, 128, 4, 5, 0, 2)])
def test_static_scratch_matches_bound_scratch(R, D, k, S, opt, prop):
    seed, sizes = 41, [1 << 16, 20011]       # the largest batch the array serves, then a smaller one
    ref = _tables(R, D, k, S, seed)
    got = _tables(R, D, k, S, seed)
    ctx = Ecrm(R, D, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, max(sizes), optimizer=opt, momentum=0.9, propagation=prop)
    scratch = torch.empty(ctx.scratch_bytes(), dtype=torch.uint8, device=DEV)
    ctx.bind(*ref, scratch)
    ctx.encode()
    got[2].copy_(ref[2])
    got[3].copy_(ref[3])
    rejected = torch.full((1,), 7, dtype=torch.int32, device=DEV)
    for keys, g in _batches(R, D, seed, sizes):
        ctx.update(keys, g)
        ctx.update_static(*got, keys, g, rejected=rejected)
        assert int(rejected.item()) == 0
        for name, a, b, atol in (("E", got[0], ref[0], ATOL_E), ("A", got[1], ref[1], ATOL_A),
                                 ("PE", got[2], ref[2], ATOL_E), ("PA", got[3], ref[3], ATOL_A)):
            err = (a.double() - b.double()).abs()
            assert bool((err <= RTOL * b.double().abs() + atol).all()), f"{name}: max err {float(err.max())}"
            log(f"  n={keys.numel()} {name}: {int((a != b).sum())} of {a.numel()} elements differ")
        assert torch.equal(got[4], ref[4]) and torch.equal(got[5], ref[5])
    assert ctx.status() == 0
    # a bad key: nothing applied, reported through `rejected`, and the next call starts clean
    keys, g = _batches(R, D, seed, [4096])[0]
    before = [t.clone() for t in got]
    bad = keys.clone()
    bad[100] = R
    ctx.update_static(*got, bad, g, rejected=rejected)
    assert int(rejected.item()) == 1
    for t, b in zip(got, before):
        assert torch.equal(t, b)
    ctx.update_static(*got, keys, g, rejected=rejected)
    assert int(rejected.item()) == 0 and not torch.equal(got[0], before[0])
    # limits
    big = torch.zeros((1 << 16) + 1, dtype=torch.int64, device=DEV)
    assert ctx.update_static(*got, big, g, check=False) == -4            # more than the array serves
    ctx.destroy()


def test_static_scratch_refuses_what_does_not_fit():
    R, D, k, S = 4 * 256, 1024, 4, 5         # momentum SGD at D = 1024 needs two sets of chain partials
    ctx = Ecrm(R, D, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, 1024, optimizer=1, momentum=0.9)
    t = _tables(R, D, k, S, 5)
    keys = torch.zeros(16, dtype=torch.int64, device=DEV)
    g = torch.zeros(16, D, device=DEV)
    assert ctx.update_static(*t, keys, g, check=False) == -3
    ctx.destroy()
