"""Host-side checks of libecrm that need no GPU: the library loads, exports every symbol the
header declares, validates configurations, and reports the sizes the paper's overhead formula
gives (Sec. 2.4 / 3.1: a (k+r)/k code with r = 1)."""
import ctypes as C
import os
import re

import pytest

from paper_2104_01981_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        from paper_2104_01981_amd import build
        build.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "ecrm.h")).read()
    declared = set(re.findall(r"\b(ecrm_[a-z_]+)\s*\(", header))
    assert declared == set(binding.SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def _create(lib, **kw):
    base = dict(rows=1 << 14, dim=128, k=4, servers=5, optimizer=0, lr=0.01, eps=1e-8, max_batch=1 << 16,
                momentum=0.0, combine=0)
    base.update(kw)
    cfg = binding.EcrmConfig(**base)
    ctx = C.c_void_p(0)
    rc = lib.ecrm_create(C.byref(cfg), C.byref(ctx))
    return rc, ctx


@pytest.mark.parametrize("kw", [dict(rows=10), dict(rows=3), dict(dim=130), dict(dim=0), dict(dim=2048),
                                dict(k=0), dict(k=65, rows=65 * 4, servers=70), dict(servers=4),
                                dict(servers=2000), dict(optimizer=2), dict(optimizer=1, momentum=1.0), dict(combine=2),
                                dict(lr=float("nan")), dict(eps=-1.0),
                                dict(max_batch=0), dict(max_batch=(1 << 31) + 1), dict(rows=1 << 32)])
def test_create_rejects_bad_config(lib, kw):
    rc, ctx = _create(lib, **kw)
    assert rc == binding.ECRM_EINVAL and not ctx.value


@pytest.mark.parametrize("k,R,D", [(2, 1 << 12, 128), (4, 1 << 12, 128), (10, 10 * 400, 256)])
def test_memory_overhead_is_k_plus_1_over_k(lib, k, R, D):
    rc, ctx = _create(lib, rows=R, dim=D, k=k, servers=k + 1)
    assert rc == 0
    data, par = lib.ecrm_data_bytes(ctx), lib.ecrm_parity_bytes(ctx)
    assert data == R * D * 4 and par * k == data          # 50 %, 25 %, 10 % for k = 2, 4, 10
    assert lib.ecrm_scratch_bytes(ctx) % 256 == 0 and lib.ecrm_scratch_bytes(ctx) > 0
    lib.ecrm_destroy(ctx)


def test_unbound_context_refuses_work(lib):
    rc, ctx = _create(lib)
    assert rc == 0
    assert lib.ecrm_encode(ctx, None) == binding.ECRM_ENOTBOUND
    assert lib.ecrm_update(ctx, None, None, 1, None) == binding.ECRM_ENOTBOUND
    assert lib.ecrm_status(ctx, None) == binding.ECRM_ENOTBOUND
    lib.ecrm_destroy(ctx)
    lib.ecrm_destroy(None)


def test_tuning_knob_and_probe_validate_their_arguments(lib):
    rc, ctx = _create(lib)
    assert rc == 0
    assert lib.ecrm_tune(ctx, 1, C.c_uint64(7)) == 0                       # ECRM_TUNE_MID_MIN_ROWS
    assert lib.ecrm_tune(ctx, 1, C.c_uint64(0)) == 0                       # back to the default
    assert lib.ecrm_tune(ctx, 1, C.c_uint64(1 << 32)) == binding.ECRM_EINVAL
    assert lib.ecrm_tune(ctx, 99, C.c_uint64(1)) == binding.ECRM_EINVAL    # no such knob
    assert lib.ecrm_tune(None, 1, C.c_uint64(1)) == binding.ECRM_EINVAL
    lib.ecrm_destroy(ctx)
    # the probe refuses null pointers and empty or oversized lists before it touches the device
    assert lib.ecrm_probe_row_traffic(None, None, C.c_uint64(16), None, C.c_uint64(8), 0, None, None) == binding.ECRM_EINVAL


def test_strerror(lib):
    for code in range(-6, 1):
        assert len(lib.ecrm_strerror(code)) > 1
    assert b"unknown" in lib.ecrm_strerror(-99)


def test_scratch_grows_with_batch(lib):
    sizes = []
    for mb in (1 << 10, 1 << 16, 1 << 20):
        rc, ctx = _create(lib, max_batch=mb)
        sizes.append(lib.ecrm_scratch_bytes(ctx))
        lib.ecrm_destroy(ctx)
    assert sizes[0] < sizes[1] < sizes[2]
    assert sizes[2] < (1 << 20) * 64          # well under 64 B per item


def _placement_ref(x, R, k, S, server, chunks, nxt, locked):
    """Placement (Sec. 3.2) and the hold-back rule (Sec. 3.4) in unbounded Python integers."""
    g, j = x // k, x % k
    ds, ps = (g + 1 + j) % S, g % S
    stripes = R // k
    spc = -(-stripes // chunks)
    if ps == server:
        unit = k
    else:
        unit = next((m for m in range(k) if (g + 1 + m) % S == server), -1)
    c = g // spc
    held = unit >= 0 and c >= nxt and ((c == nxt and locked) or unit == j)
    return [g, j, ds, ps, int(held), unit & 0xFFFFFFFF]


@pytest.mark.parametrize("R,k,S", [((1 << 32) - 4096, 1, 2), ((1 << 32) - 4096, 4, 5), ((1 << 32) - 4096 - 64, 64, 65),
                                   ((1 << 31) + 4096, 1, 3), (((1 << 32) - 4096) // 10 * 10, 10, 11),
                                   ((1 << 32) - 4096 - 3, 3, 1024), (1 << 25, 4, 5)])
def test_index_arithmetic_at_the_top_of_the_row_range(lib, R, k, S):
    """The kernels divide by k, S and the chunk size with 32-bit multiply-and-shift; rows go up to
    2^32 - 4096.  Same answers as unbounded integer arithmetic at both ends of the range, around 2^31,
    around multiples of k*S, and on a spread of other rows."""
    import random
    rc, ctx = _create(lib, rows=R, k=k, servers=S, dim=4)
    assert rc == 0
    rnd = random.Random(R ^ k ^ S)
    xs = set()
    for base in (0, k * S, 1 << 31, (1 << 31) // (k * S) * (k * S), R - 1, R // 2, R - k * S):
        for d in range(-3 * k - 2, 3 * k + 3):
            if 0 <= base + d < R:
                xs.add(base + d)
    xs.update(rnd.randrange(R) for _ in range(1500))
    xs.update(rnd.randrange(max(0, R - (1 << 20)), R) for _ in range(500))
    out = (C.c_uint32 * 6)()
    stripes = R // k
    for chunks in (1, 7, 1000, min(stripes, 5000)):
        spc = -(-stripes // chunks)
        nchunks = -(-stripes // spc)
        for x in xs:
            server = rnd.randrange(S)
            nxt = rnd.choice([0, nchunks - 1, rnd.randrange(nchunks), (x // k) // spc])
            locked = rnd.random() < 0.5
            assert lib.ecrm_host_placement(ctx, x, server, chunks, nxt, 1 if locked else 0, out) == 0
            assert list(out) == _placement_ref(x, R, k, S, server, chunks, nxt, locked), (x, server, chunks, nxt, locked)
    assert lib.ecrm_host_placement(ctx, R, 0, 1, 0, 0, out) == binding.ECRM_EINVAL
    lib.ecrm_destroy(ctx)
