"""The three large workloads at their full sizes, in the launch configuration bench.py times (one
ecrm_update per batch, batches resident in HBM, one stream), plus the largest one in the two other
shapes of the paper's evaluation: 256 floats per entry with k = 2 (Sec. 4.1, the doubled-dimension
data set) and k = 10 on 11 servers (Sec. 4.3).  The oracle cannot run 2^26..2^28 updates of 128 lanes in
seconds, so it is run on
  * a CONTIGUOUS SHARD of 1/16 of the stripes (at least 2 M rows), placed so that it contains the
    hottest row, with all the updates of its rows from every batch in arrival order -- every element
    of every row of the shard is compared; and
  * SAMPLED stripes anywhere in the tables -- the other hottest rows, random touched ones and random
    ones -- likewise with all their updates.
Stripes never interact, so each of them sees exactly the sequence it sees in the full run.  On top of
that: per-server counters against the oracle over all keys (bit-exact), the parity invariant over the
whole tables, and untouched rows bit-identical to their initial values."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from ecrm_case import ATOL_A, ATOL_E, RTOL, log
from paper_2104_01981_amd import Ecrm

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _fill(t, seed, tag, first_elem):
    rows, D = t.shape
    CH = (1 << 29) // D
    for r0 in range(0, rows, CH):
        r1 = min(rows, r0 + CH)
        t[r0:r1] = si.values(seed, tag, first_elem + r0 * D, (r1 - r0) * D, DEV).view(r1 - r0, D)


def _invariant(T, P, atol, K):
    D = T.shape[1]
    CH = (1 << 27) // D                            # stripes per slice
    G = P.shape[0]
    for g0 in range(0, G, CH):
        g1 = min(G, g0 + CH)
        s = T[g0 * K:g1 * K].double().view(g1 - g0, K, D)
        resid = (P[g0:g1].double() - s.sum(1)).abs()
        bound = RTOL * s.abs().sum(1) + atol * K
        assert bool((resid <= bound).all())


def _compare(what, nm, got, host, atol):
    err = np.abs(got.astype(np.float64) - host.astype(np.float64))
    bound = RTOL * np.abs(host.astype(np.float64)) + atol
    assert (err <= bound).all(), f"{what} {nm}: max err {err.max()}, worst ratio {(err / bound).max()}"
    mism = int((got != host).sum())
    assert mism <= 1e-4 * got.size + 2, f"{what} {nm}: {mism} of {got.size} elements differ in the last bit"
    log(f"  {what} {nm}: {got.shape[0]} rows, max err {err.max():.3e}, {mism} of {got.size} differ in the last bit")


# name, D, k, S, batches run (0 = all of the workload's)
CASES = [("large_uniform", 128, 4, 5, 0), ("large_skewed", 128, 4, 5, 0), ("hbm_scale", 128, 4, 5, 0),
         ("hbm_scale", 256, 2, 5, 3), ("hbm_scale", 128, 10, 11, 3)]


@pytest.mark.parametrize("name,D,K,S,nbatch", CASES, ids=[f"{c[0]}-D{c[1]}-k{c[2]}-S{c[3]}" for c in CASES])
def test_full_size(name, D, K, S, nbatch):
    w = si.WORKLOADS[name]
    nb, seed = nbatch or w["batches"], w["seed"]
    R = w["R"] // K * K                            # the largest multiple of k (k = 10 does not divide 2^25)
    per = w["n"] // w["batches"]
    G = R // K
    log(f"{name}: R={R} D={D} k={K} S={S} batches={nb}x{per}")
    torch.cuda.empty_cache()

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

    keys = []
    for b in range(nb):
        kg = si.workload_keys_t(name, b, 0, DEV)
        keys.append(torch.where(kg >= R, kg - R, kg))       # differs only when k does not divide the generator's 2^m rows

    # ---- choose the sampled stripes from the first batch's keys (measurement-side, torch only)
    uk, cnt = torch.unique(keys[0], return_counts=True)
    hot_rows = uk[torch.argsort(cnt, descending=True)[:6]]
    gen = torch.Generator(device="cpu").manual_seed(1234)
    touched = uk[torch.randint(0, uk.numel(), (40,), generator=gen).to(DEV)]
    anyrow = torch.randint(0, R, (18,), generator=gen).to(DEV)
    # ---- the contiguous shard: 1/16 of the stripes, around the hottest row
    Gs = max(G // 16, -(-(2 << 20) // K))
    g_hot = int(hot_rows[0]) // K
    sg0 = min(max(0, g_hot - Gs // 2), G - Gs)
    r0, r1 = sg0 * K, (sg0 + Gs) * K
    sE, sA = E[r0:r1].cpu().numpy(), A[r0:r1].cpu().numpy()       # the generator's values: nothing has been updated yet
    sPE, sPA = oracle.encode(sE, K), oracle.encode(sA, K)
    np.testing.assert_array_equal(PE[sg0:sg0 + Gs].cpu().numpy(), sPE)      # encode, every stripe of the shard
    np.testing.assert_array_equal(PA[sg0:sg0 + Gs].cpu().numpy(), sPA)
    log(f"  shard: stripes [{sg0}, {sg0 + Gs}) = rows [{r0}, {r1})")
    stripes = torch.unique(torch.cat([hot_rows, touched, anyrow]) // K)
    stripes = stripes[(stripes < sg0) | (stripes >= sg0 + Gs)]            # the shard covers its own
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
        # the shard's items of this batch, in arrival order, re-keyed to the shard's tables
        ssel = torch.nonzero((keys[b] >= r0) & (keys[b] < r1)).squeeze(1)
        sk_ = (keys[b][ssel] - r0).cpu().numpy().view(np.uint64)
        sg_ = g[ssel].cpu().numpy()
        oracle.update(sE, sA, sPE, sPA, K, S, si.DEFAULT_LR, si.DEFAULT_EPS, sk_, sg_,
                      threads=min(16, oracle.max_threads()))
        stats = ctx.batch_stats()
        log(f"  batch {b}: {len(ck)} sampled items, {len(sk_)} shard items, stats {stats}")
        if name == "large_skewed":     # thousands of long rows: those of moderate length are walked by one workgroup each
            assert stats["one_workgroup_rows"] > 3000 and stats["pieces"] > 0
        del g, gk, pos, sel, ssel, sg_
    assert ctx.status() == 0

    # ---- every row of the shard, and the sampled rows, against the oracle
    for nm, dev_t, lo, hi, host, atol in (("E", E, r0, r1, sE, ATOL_E), ("A", A, r0, r1, sA, ATOL_A),
                                          ("PE", PE, sg0, sg0 + Gs, sPE, ATOL_E), ("PA", PA, sg0, sg0 + Gs, sPA, ATOL_A)):
        _compare("shard", nm, dev_t[lo:hi].cpu().numpy(), host, atol)
    for nm, dev_t, idx, host, atol in (("E", E, rows_t, hE, ATOL_E), ("A", A, rows_t, hA, ATOL_A),
                                       ("PE", PE, stripes, hPE, ATOL_E), ("PA", PA, stripes, hPA, ATOL_A)):
        _compare("sampled", nm, dev_t[idx].cpu().numpy(), host, atol)
    # ---- integer side over ALL items, invariant over ALL stripes
    np.testing.assert_array_equal(ld.cpu().numpy().view(np.uint64), hld)
    np.testing.assert_array_equal(lp.cpu().numpy().view(np.uint64), hlp)
    assert int(hld.sum()) == nb * per and int(hlp.sum()) == nb * per
    _invariant(E, PE, ATOL_E, K)
    _invariant(A, PA, ATOL_A, K)
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
