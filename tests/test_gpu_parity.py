"""GPU parity: libecrm (through its C ABI) against the CPU oracle on the same seeded inputs.
Integer outputs (routing, per-server counts) bit-exact; tables within rtol 1e-5 (+ 5e-7 / 1e-9
absolute for entry-like / accumulator-like values)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from ecrm_case import Case, grads_for, log

pytestmark = pytest.mark.gpu

LONG_RUN = 1024      # ECRM_LONG_RUN of include/ecrm.h
MID_RUN = 32768      # ECRM_MID_RUN
TUNE_MID_MIN_ROWS = 1


def test_generator_matches_on_device():
    a = si.grads(5, 1000, 4096, 128, "cuda:0").cpu()
    b = si.grads(5, 1000, 4096, 128)
    assert torch.equal(a, b)
    assert torch.equal(si.table(5, si.TAG_A0, 512, 128, "cuda:0").cpu(), si.table(5, si.TAG_A0, 512, 128))


def test_encode_matches_oracle():
    c = Case(R=4 * 1000, D=128, k=4, S=5, max_batch=16, seed=9)
    np.testing.assert_array_equal(c.PE.cpu().numpy(), c.hPE)
    np.testing.assert_array_equal(c.PA.cpu().numpy(), c.hPA)


@pytest.mark.parametrize("k,S", [(4, 5), (2, 5), (10, 11), (3, 4)])
def test_route_bit_exact(k, S):
    R, n = k * 5000, 100003
    c = Case(R=R, D=4, k=k, S=S, max_batch=16)
    keys = si.uniform_keys(1, 0, n, R)
    kt = torch.from_numpy(keys.view(np.int64)).cuda()
    st = torch.empty(n, dtype=torch.int64, device="cuda")
    mem, ds, ps = (torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(3))
    c.ctx.route(kt, st, mem, ds, ps)
    assert c.ctx.status() == 0
    ost, omem, ods, ops = oracle.route(keys, R, k, S)
    np.testing.assert_array_equal(st.cpu().numpy().view(np.uint64), ost)
    np.testing.assert_array_equal(mem.cpu().numpy().view(np.uint32), omem)
    np.testing.assert_array_equal(ds.cpu().numpy().view(np.uint32), ods)
    np.testing.assert_array_equal(ps.cpu().numpy().view(np.uint32), ops)


def test_tiny_workload():
    w = si.WORKLOADS["tiny"]
    c = Case(w["R"], si.DEFAULT_D, si.DEFAULT_K, si.DEFAULT_S, w["n"], seed=w["seed"])
    c.update(si.workload_keys("tiny"), grads_for(w["seed"], 0, w["n"], si.DEFAULT_D))
    log("tiny", c.compare("tiny"))
    c.check_invariant()


def test_medium_workload():
    w = si.WORKLOADS["medium"]
    c = Case(w["R"], si.DEFAULT_D, si.DEFAULT_K, si.DEFAULT_S, w["n"], seed=w["seed"])
    c.update(si.workload_keys("medium"), grads_for(w["seed"], 0, w["n"], si.DEFAULT_D))
    log("medium", c.compare("medium"))
    c.check_invariant()


@pytest.mark.parametrize("R,D,k,S,n", [
    (4 * 251, 128, 4, 5, 10007),        # ragged tail of the sort tile
    (2 * 1000, 4, 2, 5, 8193),          # smallest entry, one item past a tile
    (10 * 300, 36, 10, 11, 5000),       # D not a multiple of 128, k = 10
    (3 * 999, 256, 3, 4, 20000),        # the paper's larger entry size
    (4 * 500, 512, 4, 5, 3000),         # two column blocks
    (64 * 20, 1024, 64, 65, 2000),      # maximum D and k
    (4 * 64, 200, 4, 8, 70000),         # few rows, many duplicates per row (runs of ~270)
    (1 << 16, 128, 4, 5, 1),            # a single update
    (1000, 128, 1, 2, 5000),            # k = 1: the parity is a mirror of the entry
    (4 * 700, 128, 4, 1024, 9000),      # the largest number of servers
    (2 * 333, 8, 2, 3, 40000),          # very short rows, long runs (~60 updates per entry)
    (4 * 300, 16, 4, 5, 1025),          # one item past a small sort tile
    (4 * 40000, 8, 4, 5, 1 << 19),      # the largest batch that is sorted in small tiles
    (4 * 40000, 8, 4, 5, (1 << 19) + 1),  # the smallest one that is sorted in large tiles
])
def test_shapes(R, D, k, S, n):
    c = Case(R, D, k, S, max_batch=n, seed=17)
    c.update(si.uniform_keys(17, 0, n, R), grads_for(17, 0, n, D))
    log((R, D, k, S, n), c.compare(str((R, D, k, S, n))))
    c.check_invariant()


HOT_ROW_LENGTHS = [1, 2, 255, 256, 257, 1023, 1024, 1025, 1026, 1280, 1281, 5000, 32768, 32769, 300000]


@pytest.mark.parametrize("m,one_workgroup", [(m, False) for m in HOT_ROW_LENGTHS] +
                         [(m, True) for m in HOT_ROW_LENGTHS if LONG_RUN < m <= 2 * MID_RUN])
def test_one_hot_row(m, one_workgroup):
    """All updates on one entry: the run goes through the split-chain path once it is longer than
    1024 (the two lengths around the threshold take different paths and must agree with the oracle).  Up to 32768
    updates the run can be walked by one workgroup; a batch with a single long row does that only when told to."""
    R, D, k, S = 1 << 10, 128, 4, 5
    c = Case(R, D, k, S, max_batch=m, seed=23)
    if one_workgroup:
        c.ctx.tune(TUNE_MID_MIN_ROWS, 1)
    keys = np.full(m, 777, np.uint64)
    c.update(keys, grads_for(23, 0, m, D))
    stats = c.ctx.batch_stats()
    assert stats["long_rows"] == (1 if m > LONG_RUN else 0)
    assert stats["long_items"] == (m if m > LONG_RUN else 0)
    assert stats["one_workgroup_rows"] == (1 if one_workgroup and LONG_RUN < m <= MID_RUN else 0)
    log("hot row", m, stats, c.compare(f"hot{m}"))
    c.check_invariant()


@pytest.mark.parametrize("one_workgroup", [False, True])
def test_hot_rows_share_a_stripe(one_workgroup):
    """Two long runs and one short run in the same stripe, plus a long run at the very end."""
    R, D, k, S = 64, 128, 4, 5
    rng = np.random.default_rng(0)
    keys = np.concatenate([np.full(3000, 8), np.full(1700, 9), np.full(5, 11), np.full(1500, 63),
                           rng.integers(0, R, 2000)]).astype(np.uint64)
    rng.shuffle(keys)
    c = Case(R, D, k, S, max_batch=len(keys), seed=29)
    if one_workgroup:
        c.ctx.tune(TUNE_MID_MIN_ROWS, 1)
    c.update(keys, grads_for(29, 0, len(keys), D))
    stats = c.ctx.batch_stats()
    assert stats["long_rows"] == 3 and stats["one_workgroup_rows"] == (3 if one_workgroup else 0)
    log("shared stripe", stats, c.compare("shared"))
    c.check_invariant()


@pytest.mark.parametrize("one_workgroup", [True, False])
@pytest.mark.parametrize("D,k,S", [(128, 4, 5), (256, 2, 5), (36, 10, 11), (512, 4, 5)])
def test_rows_of_every_length_class(D, k, S, one_workgroup):
    """Runs on both sides of every boundary of the split-chain path in one batch: the 1024 above which a run
    leaves the apply kernel, the lengths that one workgroup walks with one read of the gradients (up to 32768,
    listed in classes that double in length, 256 or 128 updates per round), and beyond that the pieces.  A batch
    with this few long rows would cut all of them into pieces; the tuning knob sends them to the workgroups."""
    lens = [1024, 1025, 1279, 1281, 2048, 2049, 3000, 4096, 4097, 8192, 8193, 9000, 16384, 16385, 20000, 32767,
            32768, 32769, 40000, 50000]     # more than 2^18 updates in all: the apply kernel works from its list of groups
    R = k * 64
    rng = np.random.default_rng(5)
    rows = rng.permutation(R)[:len(lens)]
    keys = np.concatenate([np.full(m, r) for m, r in zip(lens, rows)] + [rng.integers(0, R, 3000)]).astype(np.uint64)
    rng.shuffle(keys)
    c = Case(R, D, k, S, max_batch=len(keys), seed=31)
    if one_workgroup:
        c.ctx.tune(TUNE_MID_MIN_ROWS, 1)
    c.update(keys, grads_for(31, 0, len(keys), D))
    stats = c.ctx.batch_stats()
    counts = np.bincount(keys.astype(np.int64), minlength=R)
    assert stats["long_rows"] == int((counts > LONG_RUN).sum())
    assert stats["long_items"] == int(counts[counts > LONG_RUN].sum())
    assert stats["one_workgroup_rows"] == (int(((counts > LONG_RUN) & (counts <= MID_RUN)).sum()) if one_workgroup else 0)
    log("length classes", (D, k, S), stats, c.compare(f"classes D={D}"))
    c.check_invariant()
    c.update(keys[::-1].copy(), grads_for(31, len(keys), len(keys), D))      # once more, on accumulators that are not small
    log("length classes, second call", (D, k, S), c.compare(f"classes D={D} again"))
    c.check_invariant()


@pytest.mark.parametrize("name,shift", [("large_skewed", 6), ("hbm_scale", 8), ("large_uniform", 6)])
def test_scaled_workloads(name, shift):
    """The large workloads' recipes at reduced size (same skew, same interleave)."""
    w = si.WORKLOADS[name]
    R, per = w["R"] >> shift, (w["n"] >> shift) // w["batches"]
    c = Case(R, si.DEFAULT_D, si.DEFAULT_K, si.DEFAULT_S, per, seed=w["seed"])
    for b in range(min(2, w["batches"])):
        keys = si.workload_keys(name, batch=b, scale_shift=shift)
        c.update(keys, grads_for(w["seed"], b * per, per, si.DEFAULT_D))
        log(name, b, c.ctx.batch_stats(), c.compare(f"{name}[{b}]"))
    c.check_invariant()


def test_calls_in_a_row_carry_state():
    R, D, k, S = 4 * 3000, 128, 4, 5
    c = Case(R, D, k, S, max_batch=50000, seed=31)
    first = 0
    for n in (50000, 1, 777, 0, 20000):
        if n:
            c.update(si.uniform_keys(31, first, n, R), grads_for(31, first, n, D))
        else:
            assert c.ctx.update(torch.empty(0, dtype=torch.int64, device="cuda"),
                                torch.empty(0, D, device="cuda"), n=0) == 0
        first += n
    log("calls", c.compare("calls"))
    c.check_invariant()


def test_two_runs_are_bit_identical():
    w = si.WORKLOADS["large_skewed"]
    shift = 8
    R, n = w["R"] >> shift, w["n"] >> shift
    keys = si.workload_keys("large_skewed", scale_shift=shift)
    outs = []
    for _ in range(2):
        c = Case(R, 128, 4, 5, n, seed=3)
        kt = torch.from_numpy(keys.view(np.int64)).cuda()
        c.ctx.update(kt, grads_for(3, 0, n, 128))
        assert c.ctx.status() == 0
        outs.append([t.clone() for t in (c.E, c.A, c.PE, c.PA, c.ld, c.lp)])
    for x, y in zip(*outs):
        assert torch.equal(x, y)


def test_bad_key_rejects_the_whole_batch():
    R, D, k, S, n = 4 * 1000, 128, 4, 5, 30000
    c = Case(R, D, k, S, max_batch=n, seed=37)
    before = [t.clone() for t in (c.E, c.A, c.PE, c.PA, c.ld, c.lp)]
    keys = si.uniform_keys(37, 0, n, R)
    bad = keys.copy()
    bad[12345] = R                      # first invalid id
    g = grads_for(37, 0, n, D)
    c.ctx.update(torch.from_numpy(bad.view(np.int64)).cuda(), g)
    assert c.ctx.status() == -5         # ECRM_EKEYRANGE
    assert c.ctx.batch_stats()["rejected"] == 1
    for t, b in zip((c.E, c.A, c.PE, c.PA, c.ld, c.lp), before):
        assert torch.equal(t, b)
    bad[12345] = 2 ** 63 + 5            # a huge id whose low 32 bits look valid
    c.ctx.update(torch.from_numpy(bad.view(np.int64)).cuda(), g)
    assert c.ctx.status() == -5
    for t, b in zip((c.E, c.A, c.PE, c.PA, c.ld, c.lp), before):
        assert torch.equal(t, b)
    # the status is sticky until cleared; a good batch afterwards is applied normally
    c.ctx.clear_status()
    assert c.ctx.status() == 0
    c.update(keys, g)
    c.compare("after bad")


def test_argument_errors():
    R, D, k, S = 4 * 100, 128, 4, 5
    c = Case(R, D, k, S, max_batch=100, seed=1)
    keys = torch.zeros(200, dtype=torch.int64, device="cuda")
    g = torch.zeros(200, D, device="cuda")
    assert c.ctx.update(keys, g, n=101, check=False) == -4       # ECRM_EBATCH
    assert c.ctx.update(keys[1:], g, n=10, check=False) == 0     # 8-byte aligned keys are fine
    assert c.ctx.update(keys, g.view(-1)[1:], n=10, check=False) == -1   # misaligned gradients
    from paper_2104_01981_amd import Ecrm
    e = Ecrm(R, D, k, S, 0.01, 1e-8, 100)
    need = e.scratch_bytes()
    sc = torch.empty(need, dtype=torch.uint8, device="cuda")
    p = c.E.data_ptr()
    assert e.bind_raw(p, p, p, p, c.ld.data_ptr(), c.lp.data_ptr(), sc.data_ptr(), need - 1) == -3
    assert e.bind_raw(p, p, p, p, c.ld.data_ptr(), c.lp.data_ptr(), sc.data_ptr() + 16, need) == -3
    assert e.bind_raw(p + 4, p, p, p, c.ld.data_ptr(), c.lp.data_ptr(), sc.data_ptr(), need) == -1
    assert e.bind_raw(0, p, p, p, c.ld.data_ptr(), c.lp.data_ptr(), sc.data_ptr(), need) == -1


def test_profile_hooks():
    R, D, k, S, n = 4 * 1000, 128, 4, 5, 20000
    c = Case(R, D, k, S, max_batch=n, seed=41)
    c.ctx.profile(True)
    kt = torch.from_numpy(si.uniform_keys(41, 0, n, R).view(np.int64)).cuda()
    g = grads_for(41, 0, n, D)
    for _ in range(3):
        c.ctx.update(kt, g)
    ms, calls = c.ctx.profile_read()
    assert calls == 3 and all(m >= 0 for m in ms) and ms[0] > 0 and ms[2] > 0
    c.ctx.profile(False)
    c.ctx.update(kt, g)
    assert c.ctx.profile_read()[1] == 0


@pytest.mark.parametrize("n", [20000, 300000])
def test_update_inside_a_hip_graph(n):
    """ecrm_update only enqueues kernels (no memsets, no synchronisation), so a caller may capture it.
    Replays are checked one by one against eager calls on a twin, with eager work in between.  The larger batch
    brings the kernels of large batches into the graph: the list of groups, and (tuned in) the one-workgroup chains."""
    R, D, k, S = 4 * 2000, 128, 4, 5
    a = Case(R, D, k, S, max_batch=n, seed=71)
    b = Case(R, D, k, S, max_batch=n, seed=71)
    keys = si.uniform_keys(71, 0, n, R)
    keys[::7] = 4321                                   # a long run as well (42 857 updates in the larger batch: pieces)
    if n > 100000:
        keys[1::61] = 999                              # ~4 900 updates: one workgroup
        a.ctx.tune(TUNE_MID_MIN_ROWS, 1)
        b.ctx.tune(TUNE_MID_MIN_ROWS, 1)
    kt = torch.from_numpy(keys.view(np.int64)).cuda()
    g = grads_for(71, 0, n, D)
    a.ctx.update(kt, g)                                # warm-up outside the capture (first-call set-up)
    b.ctx.update(kt, g)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        a.ctx.update(kt, g, stream=side)
    b.ctx.update(kt, g)                                # the capture itself ran nothing on a; this call belongs to
    graph.replay()                                     # ... the first replay
    for rep in range(4):
        torch.cuda.synchronize()
        for x, y in zip((a.E, a.A, a.PE, a.PA, a.ld, a.lp), (b.E, b.A, b.PE, b.PA, b.ld, b.lp)):
            assert torch.equal(x, y), f"replay {rep}"
        (a.E.sum() + b.E.sum()).item()                 # unrelated eager work and a sync between replays
        graph.replay()
        b.ctx.update(kt, g)
    torch.cuda.synchronize()
    assert torch.equal(a.E, b.E) and torch.equal(a.PA, b.PA)
    assert a.ctx.status() == 0
    if n > 100000:
        stats = a.ctx.batch_stats()
        assert stats["long_rows"] == 2 and stats["one_workgroup_rows"] == 1 and stats["pieces"] > 0


def test_row_traffic_probe():
    """The measurement aid behind the bench line's row-traffic figures: rows at even positions of the list come from
    the first table, rows at odd positions from the second; with `write` each of them is written back plus one."""
    from paper_2104_01981_amd import probe_row_traffic
    table_rows, n = 5000, 4096
    ta = torch.zeros(table_rows, 128, device="cuda")
    tb = torch.zeros(table_rows, 128, device="cuda")
    rows = torch.randperm(table_rows, device="cuda")[:n].to(torch.int32)
    sink = torch.zeros(1, device="cuda")
    probe_row_traffic(ta, tb, table_rows, rows, 0, sink)
    assert float(ta.abs().sum()) == 0.0 and float(tb.abs().sum()) == 0.0 and float(sink) == 0.0
    probe_row_traffic(ta, tb, table_rows, rows, 1, sink)
    probe_row_traffic(ta, tb, table_rows, rows, 1, sink)
    want_a = torch.zeros(table_rows, device="cuda")
    want_b = torch.zeros(table_rows, device="cuda")
    want_a[rows[0::2].long()] = 2.0
    want_b[rows[1::2].long()] = 2.0
    assert torch.equal(ta, want_a[:, None].expand(-1, 128)) and torch.equal(tb, want_b[:, None].expand(-1, 128))
