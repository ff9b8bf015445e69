"""Thin ctypes binding of libecrm.so: argument marshalling only.

Every step of the update path runs in the library's HIP kernels; torch is used for device memory
and streams.  The library must have been built (paper_2104_01981_amd/build.py); there is no CPU
fallback, and a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os

ECRM_OK, ECRM_EINVAL, ECRM_ENOTBOUND, ECRM_ESCRATCH, ECRM_EBATCH, ECRM_EKEYRANGE, ECRM_EHIP = 0, -1, -2, -3, -4, -5, -6
ECRM_EBUFFER, ECRM_ESTATE = -7, -8
ECRM_PHASES = 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("ECRM_LIBRARY") or os.path.join(_HERE, "libecrm.so")
_lib = None

SYMBOLS = ["ecrm_create", "ecrm_destroy", "ecrm_data_bytes", "ecrm_parity_bytes", "ecrm_scratch_bytes",
           "ecrm_bind", "ecrm_encode", "ecrm_route", "ecrm_update", "ecrm_update_static", "ecrm_status", "ecrm_clear_status",
           "ecrm_tune", "ecrm_probe_row_traffic", "ecrm_profile", "ecrm_profile_read", "ecrm_batch_stats", "ecrm_host_placement", "ecrm_strerror",
           "ecrm_fail_server", "ecrm_recover_server", "ecrm_degraded_read",
           "ecrm_recovery_begin", "ecrm_recovery_lock", "ecrm_recovery_decode", "ecrm_recovery_unlock",
           "ecrm_recovery_state", "ecrm_recovery_read"]


class EcrmConfig(C.Structure):
    _fields_ = [("rows", C.c_uint64), ("dim", C.c_uint32), ("k", C.c_uint32), ("servers", C.c_uint32),
                ("optimizer", C.c_uint32), ("lr", C.c_float), ("eps", C.c_float), ("max_batch", C.c_uint64),
                ("momentum", C.c_float), ("combine", C.c_uint32), ("propagation", C.c_uint32)]


class EcrmError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libecrm.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2104_01981_amd/build.py`")
        lib = C.CDLL(_LIB_PATH)
        vp, u64p, u32p, f32p = C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p
        lib.ecrm_create.argtypes = [C.POINTER(EcrmConfig), C.POINTER(C.c_void_p)]
        lib.ecrm_destroy.argtypes = [vp]
        lib.ecrm_destroy.restype = None
        for name in ("ecrm_data_bytes", "ecrm_parity_bytes", "ecrm_scratch_bytes"):
            getattr(lib, name).argtypes = [vp]
            getattr(lib, name).restype = C.c_size_t
        lib.ecrm_bind.argtypes = [vp, f32p, f32p, f32p, f32p, u64p, u64p, vp, C.c_size_t]
        lib.ecrm_encode.argtypes = [vp, vp]
        lib.ecrm_route.argtypes = [vp, u64p, C.c_uint64, u64p, u32p, u32p, u32p, vp]
        lib.ecrm_update.argtypes = [vp, u64p, f32p, C.c_uint64, vp]
        lib.ecrm_update_static.argtypes = [vp, f32p, f32p, f32p, f32p, u64p, u64p, u64p, f32p, C.c_uint64, u32p, vp]
        lib.ecrm_fail_server.argtypes = [vp, C.c_uint32, vp]
        lib.ecrm_recover_server.argtypes = [vp, C.c_uint32, vp]
        lib.ecrm_degraded_read.argtypes = [vp, u64p, C.c_uint64, C.c_uint32, f32p, f32p, vp]
        lib.ecrm_recovery_begin.argtypes = [vp, C.c_uint32, C.c_uint32, u64p, f32p, C.c_uint64, vp]
        lib.ecrm_recovery_read.argtypes = [vp, u64p, C.c_uint64, f32p, f32p, vp]
        lib.ecrm_recovery_lock.argtypes = [vp]
        lib.ecrm_recovery_decode.argtypes = [vp, vp]
        lib.ecrm_recovery_unlock.argtypes = [vp, vp]
        lib.ecrm_recovery_state.argtypes = [vp, vp, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                            C.POINTER(C.c_uint32), C.POINTER(C.c_uint64)]
        lib.ecrm_status.argtypes = [vp, vp]
        lib.ecrm_clear_status.argtypes = [vp, vp]
        lib.ecrm_tune.argtypes = [vp, C.c_int, C.c_uint64]
        lib.ecrm_probe_row_traffic.argtypes = [vp, vp, C.c_uint64, vp, C.c_uint64, C.c_int, vp, vp]
        lib.ecrm_profile.argtypes = [vp, C.c_int]
        lib.ecrm_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
        lib.ecrm_batch_stats.argtypes = [vp, vp, C.POINTER(C.c_uint64)]
        lib.ecrm_host_placement.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                            C.POINTER(C.c_uint32)]
        lib.ecrm_strerror.argtypes = [C.c_int]
        lib.ecrm_strerror.restype = C.c_char_p
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load_library().ecrm_strerror(code).decode()


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def probe_row_traffic(table_a, table_b, table_rows, rows, write, sink, stream=None):
    """ecrm_probe_row_traffic (measurement aid): rows of 128 floats at rows[i], alternately from the two tables."""
    rc = load_library().ecrm_probe_row_traffic(_ptr(table_a), _ptr(table_b), C.c_uint64(table_rows), _ptr(rows),
                                               C.c_uint64(rows.numel()), C.c_int(1 if write else 0), _ptr(sink),
                                               _stream(stream))
    if rc != ECRM_OK:
        raise EcrmError(rc, "ecrm_probe_row_traffic")


class Ecrm:
    """One context of the library.  Method names mirror the C entry points (ecrm_<name>)."""

    def __init__(self, rows, dim=128, k=4, servers=5, lr=0.01, eps=1e-8, max_batch=1 << 20, optimizer=0,
                 momentum=0.0, combine=0, propagation=0):
        self._lib = load_library()
        self.cfg = EcrmConfig(rows, dim, k, servers, optimizer, lr, eps, max_batch, momentum, combine, propagation)
        self._ctx = C.c_void_p(0)
        rc = self._lib.ecrm_create(C.byref(self.cfg), C.byref(self._ctx))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_create")
        self._keep = None

    def destroy(self):
        if self._ctx:
            self._lib.ecrm_destroy(self._ctx)
            self._ctx = C.c_void_p(0)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def data_bytes(self):
        return self._lib.ecrm_data_bytes(self._ctx)

    def parity_bytes(self):
        return self._lib.ecrm_parity_bytes(self._ctx)

    def scratch_bytes(self):
        return self._lib.ecrm_scratch_bytes(self._ctx)

    def bind_raw(self, E, A, PE, PA, load_data, load_parity, scratch, scratch_bytes):
        """ecrm_bind with raw integer addresses (for error-path tests)."""
        return self._lib.ecrm_bind(self._ctx, C.c_void_p(E), C.c_void_p(A), C.c_void_p(PE), C.c_void_p(PA),
                                   C.c_void_p(load_data), C.c_void_p(load_parity), C.c_void_p(scratch),
                                   C.c_size_t(scratch_bytes))

    def bind(self, E, A, PE, PA, load_data, load_parity, scratch):
        import torch
        R, D, k, S = self.cfg.rows, self.cfg.dim, self.cfg.k, self.cfg.servers
        for t, shape in ((E, (R, D)), (A, (R, D)), (PE, (R // k, D)), (PA, (R // k, D))):
            assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == shape
        for t in (load_data, load_parity):
            assert t.is_cuda and t.dtype in (torch.int64, torch.uint64) and t.numel() == S and t.is_contiguous()
        assert scratch.is_cuda and scratch.dtype == torch.uint8 and scratch.is_contiguous()
        rc = self._lib.ecrm_bind(self._ctx, _ptr(E), _ptr(A), _ptr(PE), _ptr(PA), _ptr(load_data),
                                 _ptr(load_parity), _ptr(scratch), C.c_size_t(scratch.numel()))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_bind")
        self._keep = (E, A, PE, PA, load_data, load_parity, scratch)

    def drop_buffers(self):
        """Python side only: stop keeping the bound tensors alive (bind again before any further call)."""
        self._keep = None

    def encode(self, stream=None):
        rc = self._lib.ecrm_encode(self._ctx, _stream(stream))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_encode")

    def route(self, keys, stripe=None, member=None, data_srv=None, parity_srv=None, stream=None):
        rc = self._lib.ecrm_route(self._ctx, _ptr(keys), C.c_uint64(keys.numel()), _ptr(stripe), _ptr(member),
                                  _ptr(data_srv), _ptr(parity_srv), _stream(stream))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_route")

    def update(self, keys, grads, n=None, stream=None, check=True):
        n = keys.numel() if n is None else n
        rc = self._lib.ecrm_update(self._ctx, _ptr(keys), _ptr(grads), C.c_uint64(n), _stream(stream))
        if check and rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_update")
        return rc

    def update_static(self, E, A, PE, PA, load_data, load_parity, keys, grads, n=None, rejected=None, stream=None,
                      check=True):
        """ecrm_update_static: the library's own fixed scratch array, tables passed per call."""
        n = keys.numel() if n is None else n
        rc = self._lib.ecrm_update_static(self._ctx, _ptr(E), _ptr(A), _ptr(PE), _ptr(PA), _ptr(load_data),
                                          _ptr(load_parity), _ptr(keys), _ptr(grads), C.c_uint64(n), _ptr(rejected),
                                          _stream(stream))
        if check and rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_update_static")
        return rc

    def fail_server(self, server, stream=None):
        rc = self._lib.ecrm_fail_server(self._ctx, C.c_uint32(server), _stream(stream))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_fail_server")

    def recover_server(self, server, stream=None):
        rc = self._lib.ecrm_recover_server(self._ctx, C.c_uint32(server), _stream(stream))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_recover_server")

    def degraded_read(self, keys, lost_server, out_E, out_A=None, stream=None, check=True):
        lost = 0xFFFFFFFF if lost_server is None else lost_server
        rc = self._lib.ecrm_degraded_read(self._ctx, _ptr(keys), C.c_uint64(keys.numel()), C.c_uint32(lost),
                                          _ptr(out_E), _ptr(out_A), _stream(stream))
        if check and rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_degraded_read")
        return rc

    def recovery_read(self, keys, out_E, out_A=None, stream=None, check=True):
        rc = self._lib.ecrm_recovery_read(self._ctx, _ptr(keys), C.c_uint64(keys.numel()), _ptr(out_E), _ptr(out_A),
                                          _stream(stream))
        if check and rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_recovery_read")
        return rc

    def recovery_begin(self, server, chunks, buf_keys, buf_grads, capacity, stream=None, check=True):
        rc = self._lib.ecrm_recovery_begin(self._ctx, C.c_uint32(server), C.c_uint32(chunks), _ptr(buf_keys),
                                           _ptr(buf_grads), C.c_uint64(capacity), _stream(stream))
        if check and rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_recovery_begin")
        self._keep_rec = (buf_keys, buf_grads)
        return rc

    def recovery_lock(self, check=True):
        rc = self._lib.ecrm_recovery_lock(self._ctx)
        if check and rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_recovery_lock")
        return rc

    def recovery_decode(self, stream=None, check=True):
        rc = self._lib.ecrm_recovery_decode(self._ctx, _stream(stream))
        if check and rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_recovery_decode")
        return rc

    def recovery_unlock(self, stream=None, check=True):
        rc = self._lib.ecrm_recovery_unlock(self._ctx, _stream(stream))
        if check and rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_recovery_unlock")
        return rc

    def recovery_state(self, stream=None):
        a, nx, ch, bf = C.c_uint32(0), C.c_uint32(0), C.c_uint32(0), C.c_uint64(0)
        rc = self._lib.ecrm_recovery_state(self._ctx, _stream(stream), C.byref(a), C.byref(nx), C.byref(ch), C.byref(bf))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_recovery_state")
        return dict(active=bool(a.value), next_chunk=int(nx.value), chunks=int(ch.value), buffered=int(bf.value))

    def status(self, stream=None):
        return self._lib.ecrm_status(self._ctx, _stream(stream))

    def clear_status(self, stream=None):
        rc = self._lib.ecrm_clear_status(self._ctx, _stream(stream))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_clear_status")

    def profile(self, enable=True):
        rc = self._lib.ecrm_profile(self._ctx, 1 if enable else 0)
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_profile")

    def profile_read(self):
        ms = (C.c_double * ECRM_PHASES)()
        calls = C.c_uint64(0)
        rc = self._lib.ecrm_profile_read(self._ctx, ms, C.byref(calls))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_profile_read")
        return list(ms), int(calls.value)

    def host_placement(self, key, failed_server, chunks, next_chunk, locked):
        out = (C.c_uint32 * 6)()
        rc = self._lib.ecrm_host_placement(self._ctx, C.c_uint64(key), C.c_uint32(failed_server), C.c_uint32(chunks),
                                           C.c_uint32(next_chunk), C.c_uint32(1 if locked else 0), out)
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_host_placement")
        return [int(v) for v in out]

    def batch_stats(self, stream=None):
        out = (C.c_uint64 * 5)()
        rc = self._lib.ecrm_batch_stats(self._ctx, _stream(stream), out)
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_batch_stats")
        return dict(long_rows=int(out[0]), pieces=int(out[1]), long_items=int(out[2]), rejected=int(out[3]),
                    one_workgroup_rows=int(out[4]))

    def tune(self, what, value):
        rc = self._lib.ecrm_tune(self._ctx, C.c_int(what), C.c_uint64(value))
        if rc != ECRM_OK:
            raise EcrmError(rc, "ecrm_tune")
