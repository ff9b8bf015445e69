"""The three large workloads at their full sizes, in the launch configuration bench.py times (one
ecrm_update per batch, batches resident in HBM, one stream).  The oracle cannot run 2^26..2^28
updates of 128 lanes in seconds, so it is run on SAMPLED stripes -- the hottest ones, random touched
ones and random untouched ones -- with all their updates in arrival order; stripes never interact, so
each sampled stripe sees exactly the sequence it sees in the full run.  On top of that: per-server
counters against the oracle over all keys (bit-exact), the parity invariant over the whole tables,
and untouched rows bit-identical to their initial values."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from ecrm_case import ATOL_A, ATOL_E, RTOL, log
from paper_2104_01981_amd import Ecrm

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
D, K, S = si.DEFAULT_D, si.DEFAULT_K, si.DEFAULT_S


def _fill(t, seed, tag, first_elem):
    CH = 1 << 22
    rows = t.shape[0]
    for r0 in range(0, rows, CH):
        r1 = min(rows, r0 + CH)
        t[r0:r1] = si.values(seed, tag, first_elem + r0 * D, (r1 - r0) * D, DEV).view(r1 - r0, D)


def _invariant(T, P, atol):
    CH = 1 << 20                                   # stripes per slice
    G = P.shape[0]
    for g0 in range(0, G, CH):
        g1 = min(G, g0 + CH)
        s = T[g0 * K:g1 * K].double().view(g1 - g0, K, D)
        resid = (P[g0:g1].double() - s.sum(1)).abs()
        bound = RTOL * s.abs().sum(1) + atol * K
        assert bool((resid <= bound).all())


@pytest.mark.parametrize("name", ["large_uniform", "large_skewed", "hbm_scale"])
def test_full_size_sampled(name):
    w = si.WORKLOADS[name]
    R, nb, seed = w["R"], w["batches"], w["seed"]
    per = w["n"] // nb
    G = R // K
    log(f"{name}: R={R} batches={nb}x{per}")

    E = torch.empty(R, D, device=DEV)
    A = torch.empty(R, D, device=DEV)
    _fill(E, seed, si.TAG_E0, 0)
    _fill(A, seed, si.TAG_A0, 0)
    PE, PA = torch.empty(G, D, device=DEV), torch.empty(G, D, device=DEV)
    ld = torch.zeros(S, dtype=torch.int64, device=DEV)
    lp = torch.zeros(S, dtype=torch.int64, device=DEV)
    ctx = Ecrm(R, D, K, S, si.DEFAULT_LR, si.DEFAULT_EPS, per)
    scratch = torch.empty(ctx.scratch_bytes(), dtype=torch.uint8, device=DEV)
    ctx.bind(E, A, PE, PA, ld, lp, scratch)
    ctx.encode()

    keys = [si.workload_keys_t(name, b, 0, DEV) for b in range(nb)]

    # ---- choose the sampled stripes from the first batch's keys (measurement-side, torch only)
    uk, cnt = torch.unique(keys[0], return_counts=True)
    hot_rows = uk[torch.argsort(cnt, descending=True)[:6]]
    gen = torch.Generator(device="cpu").manual_seed(1234)
    touched = uk[torch.randint(0, uk.numel(), (40,), generator=gen).to(DEV)]
    anyrow = torch.randint(0, R, (18,), generator=gen).to(DEV)
    stripes = torch.unique(torch.cat([hot_rows, touched, anyrow]) // K)
    stripes_h = stripes.cpu().numpy()
    m = len(stripes_h)
    rows_h = (stripes_h[:, None] * K + np.arange(K)[None, :]).reshape(-1)
    rows_t = torch.from_numpy(rows_h).to(DEV)
    log(f"  {m} sampled stripes, hottest row has {int(cnt.max())} updates in batch 0")
    del uk, cnt

    # ---- oracle side: compact tables of the sampled stripes, from the generator
    hE = si.table_rows(seed, si.TAG_E0, rows_h, D).copy()
    hA = si.table_rows(seed, si.TAG_A0, rows_h, D).copy()
    hPE, hPA = oracle.encode(hE, K), oracle.encode(hA, K)
    np.testing.assert_array_equal(PE[stripes].cpu().numpy(), hPE)          # encode, sampled
    np.testing.assert_array_equal(PA[stripes].cpu().numpy(), hPA)
    hld, hlp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)

    for b in range(nb):
        g = si.grads(seed, b * per, per, D, DEV)
        ctx.update(keys[b], g)
        # the sampled stripes' items of this batch, in arrival order, re-keyed to the compact tables
        gk = keys[b] // K
        pos = torch.searchsorted(stripes, gk).clamp(max=m - 1)
        sel = torch.nonzero(stripes[pos] == gk).squeeze(1)
        ck = (pos[sel] * K + keys[b][sel] % K).cpu().numpy().view(np.uint64)
        cg = g[sel].cpu().numpy()
        oracle.update(hE, hA, hPE, hPA, K, S, si.DEFAULT_LR, si.DEFAULT_EPS, ck, cg, threads=8)
        l1, l2 = oracle.load(keys[b].cpu().numpy().view(np.uint64), R, K, S)
        hld += l1
        hlp += l2
        log(f"  batch {b}: {len(ck)} sampled items, stats {ctx.batch_stats()}")
        del g, gk, pos, sel
    assert ctx.status() == 0

    # ---- sampled rows against the oracle
    for nm, dev_t, idx, host, atol in (("E", E, rows_t, hE, ATOL_E), ("A", A, rows_t, hA, ATOL_A),
                                       ("PE", PE, stripes, hPE, ATOL_E), ("PA", PA, stripes, hPA, ATOL_A)):
        got = dev_t[idx].cpu().numpy()
        err = np.abs(got.astype(np.float64) - host.astype(np.float64))
        bound = RTOL * np.abs(host.astype(np.float64)) + atol
        assert (err <= bound).all(), f"{name} {nm}: max err {err.max()}, worst ratio {(err / bound).max()}"
        log(f"  {nm}: max err {err.max():.3e}, {int((got != host).sum())} of {got.size} differ in the last bit")
    # ---- integer side over ALL items, invariant over ALL stripes
    np.testing.assert_array_equal(ld.cpu().numpy().view(np.uint64), hld)
    np.testing.assert_array_equal(lp.cpu().numpy().view(np.uint64), hlp)
    assert int(hld.sum()) == w["n"] and int(hlp.sum()) == w["n"]
    _invariant(E, PE, ATOL_E)
    _invariant(A, PA, ATOL_A)
    # ---- rows no batch touched keep their initial bits
    touched_mask = torch.zeros(R, dtype=torch.bool, device=DEV)
    for b in range(nb):
        touched_mask[keys[b]] = True
    untouched = torch.nonzero(~touched_mask).squeeze(1)
    if untouched.numel():
        pick = untouched[torch.randint(0, untouched.numel(), (4096,), generator=gen).to(DEV)]
        ref = torch.from_numpy(si.table_rows(seed, si.TAG_E0, pick.cpu().numpy(), D)).to(DEV)
        assert torch.equal(E[pick], ref)
    ctx.destroy()
