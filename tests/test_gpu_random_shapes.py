"""Seeded random shapes, rules and batch sizes -- the sizes drawn mostly from around the kernels'
internal boundaries (sort tile, wave window, hand-out tickets of the apply kernel) -- against the oracle."""
import numpy as np
import pytest

import synth_inputs as si
from ecrm_case import Case, grads_for, log

pytestmark = pytest.mark.gpu

WAVES = 5120                      # resident waves of the apply kernel on 256 compute units
BOUNDARY_N = [1, 2, 63, 64, 65, 6143, 6144, 6145, 12287, 12288, 12289, 16 * WAVES - 1, 16 * WAVES, 16 * WAVES + 1,
              64 * WAVES - 5, 64 * WAVES + 5, 655359, 655360, 655377, 1310723]


def _draw(case):
    rng = np.random.default_rng(4242 + case)
    k = int(rng.choice([1, 2, 3, 4, 5, 7, 10, 16, 64]))
    S = k + 1 + int(rng.integers(0, 4)) * int(rng.integers(0, 2))
    D = int(rng.choice([4, 8, 36, 64, 100, 128, 132, 200, 256, 384, 512, 1024]))
    n = int(rng.choice(BOUNDARY_N)) if rng.random() < 0.6 else int(rng.integers(1, 300000))
    n = min(n, (1 << 29) // (D * 4))
    R = int(rng.integers(1, max(2, min(1 << 17, (128 << 20) // (D * 4)) // k))) * k
    opt, comb = int(rng.integers(0, 2)), int(rng.integers(0, 2))
    prop = int(rng.choice([0, 0, 0, 1, 2])) if comb == 0 else int(rng.choice([0, 2]))
    return rng, R, D, k, S, n, opt, comb, prop


@pytest.mark.parametrize("case", range(24))
def test_random_shape(case):
    rng, R, D, k, S, n, opt, comb, prop = _draw(case)
    c = Case(R, D, k, S, max_batch=n, seed=2000 + case, optimizer=opt, momentum=0.9, combine=comb, propagation=prop)
    keys = si.uniform_keys(2000 + case, 0, n, R)
    skew = rng.random()
    if skew < 0.4 and n > 8:                       # a few hot rows, one of them very hot
        hot = rng.integers(0, R, 3).astype(np.uint64)
        keys[::2], keys[1::7], keys[3::11] = hot[0], hot[1], hot[2]
    elif skew < 0.6:
        keys = (keys % np.uint64(max(1, R // 50))).astype(np.uint64)
    for call in range(2):
        c.update(keys if call == 0 else np.roll(keys, 3), grads_for(2000 + case, call * n, n, D))
    log("random shape", case, (R, D, k, S, n, opt, comb, prop), c.compare(f"random {case}"))
    if prop == 0:
        c.check_invariant()


@pytest.mark.parametrize("case", range(8))
def test_random_run_lengths(case):
    """Batches made of runs of many lengths around the boundaries of the chain tiers (1024: out of the apply kernel;
    up to 32768: one workgroup per run if the batch has enough long rows -- forced with the tuning knob in every other
    case; beyond: pieces), on the Adagrad rule in all three propagation modes."""
    rng = np.random.default_rng(777 + case)
    k = int(rng.choice([1, 2, 4, 10]))
    S = k + 1 + int(rng.integers(0, 3))
    D = int(rng.choice([36, 128, 128, 256, 512]))
    n = int(rng.integers(150000, 420000))
    n = min(n, (1 << 29) // (D * 4))
    R = int(rng.integers(8, 4000)) * k
    prop = int(rng.choice([0, 0, 1, 2]))
    c = Case(R, D, k, S, max_batch=n, seed=3000 + case, propagation=prop)
    if case % 2:
        c.ctx.tune(1, 1)                           # ECRM_TUNE_MID_MIN_ROWS
    keys = si.uniform_keys(3000 + case, 0, n, R)
    pos = 0
    for r in rng.permutation(R)[:14]:
        m = int(rng.choice([1024, 1025, 1300, 2048, 2049, 5000, 8193, 20000, 32768, 32769, 70000]))
        if pos + m > n:
            break
        keys[pos:pos + m] = r
        pos += m
    keys = rng.permutation(keys)
    for call in range(2):
        c.update(keys if call == 0 else np.roll(keys, 5), grads_for(3000 + case, call * n, n, D))
    stats = c.ctx.batch_stats()
    # what the call's LAST pass found: grouped by stripe for the parity half of gradient propagation, else by row
    counts = np.bincount((keys // np.uint64(k) if prop == 1 else keys).astype(np.int64))
    assert stats["long_rows"] == int((counts > 1024).sum())
    assert stats["one_workgroup_rows"] == (int(((counts > 1024) & (counts <= 32768)).sum()) if case % 2 else 0)
    log("random run lengths", case, (R, D, k, S, n, prop), stats, c.compare(f"runs {case}"))
    if prop == 0:
        c.check_invariant()
