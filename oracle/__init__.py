"""ctypes front end of the CPU oracle (test infrastructure; see ecrm_oracle.c for what it states).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ecrm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC",
                               "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.ecrm_oracle_update.restype = C.c_int
        _lib.ecrm_oracle_update_gradient_propagation.restype = C.c_int
        _lib.ecrm_oracle_update_gradient_propagation_rule.restype = C.c_int
        _lib.ecrm_oracle_route.restype = C.c_int
        _lib.ecrm_oracle_load.restype = C.c_int
        _lib.ecrm_oracle_max_threads.restype = C.c_int
        _lib.ecrm_oracle_recover_server.restype = C.c_int
        _lib.ecrm_oracle_recover_range.restype = C.c_int
        _lib.ecrm_oracle_update_rule.restype = C.c_int
        _lib.ecrm_oracle_fail_server.restype = C.c_int
        _lib.ecrm_oracle_degraded_read.restype = C.c_int
    return _lib


def _p(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _f32(a):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return _p(a, C.c_float)


def _u64(a):
    assert a.dtype == np.uint64 and a.flags.c_contiguous
    return _p(a, C.c_uint64)


def max_threads() -> int:
    return int(lib().ecrm_oracle_max_threads())


def route(keys: np.ndarray, R: int, k: int, S: int):
    n = len(keys)
    stripe = np.empty(n, np.uint64)
    member = np.empty(n, np.uint32)
    ds = np.empty(n, np.uint32)
    ps = np.empty(n, np.uint32)
    rc = lib().ecrm_oracle_route(_u64(keys), C.c_uint64(n), C.c_uint64(R), C.c_uint32(k), C.c_uint32(S),
                                 _u64(stripe), _p(member, C.c_uint32), _p(ds, C.c_uint32), _p(ps, C.c_uint32))
    if rc != 0:
        raise ValueError("key out of range")
    return stripe, member, ds, ps


def load(keys: np.ndarray, R: int, k: int, S: int):
    ld = np.zeros(S, np.uint64)
    lp = np.zeros(S, np.uint64)
    rc = lib().ecrm_oracle_load(_u64(keys), C.c_uint64(len(keys)), C.c_uint64(R), C.c_uint32(k), C.c_uint32(S),
                                _u64(ld), _u64(lp))
    if rc != 0:
        raise ValueError("key out of range")
    return ld, lp


def encode(T: np.ndarray, k: int) -> np.ndarray:
    R, D = T.shape
    P = np.empty((R // k, D), np.float32)
    lib().ecrm_oracle_encode(_f32(T), C.c_uint64(R), C.c_uint32(D), C.c_uint32(k), _f32(P))
    return P


def decode_member(T: np.ndarray, P: np.ndarray, k: int, lost: int) -> np.ndarray:
    R, D = T.shape
    out = np.empty((R // k, D), np.float32)
    lib().ecrm_oracle_decode_member(_f32(T), _f32(P), C.c_uint64(R), C.c_uint32(D), C.c_uint32(k),
                                    C.c_uint32(lost), _f32(out))
    return out


def recover_server(E, A, PE, PA, k: int, S: int, server: int) -> None:
    R, D = E.shape
    rc = lib().ecrm_oracle_recover_server(_f32(E), _f32(A), _f32(PE), _f32(PA), C.c_uint64(R), C.c_uint32(D),
                                          C.c_uint32(k), C.c_uint32(S), C.c_uint32(server))
    if rc != 0:
        raise ValueError("bad server")


def recover_range(E, A, PE, PA, k: int, S: int, server: int, g_lo: int, g_hi: int) -> None:
    R, D = E.shape
    rc = lib().ecrm_oracle_recover_range(_f32(E), _f32(A), _f32(PE), _f32(PA), C.c_uint64(R), C.c_uint32(D),
                                         C.c_uint32(k), C.c_uint32(S), C.c_uint32(server), C.c_uint64(g_lo),
                                         C.c_uint64(g_hi))
    if rc != 0:
        raise ValueError("bad server or range")


def fail_server(E, A, PE, PA, k: int, S: int, server: int) -> None:
    R, D = E.shape
    rc = lib().ecrm_oracle_fail_server(_f32(E), _f32(A), _f32(PE), _f32(PA), C.c_uint64(R), C.c_uint32(D),
                                       C.c_uint32(k), C.c_uint32(S), C.c_uint32(server))
    if rc != 0:
        raise ValueError("bad server")


def degraded_read(E, A, PE, PA, k: int, S: int, keys, lost: int):
    R, D = E.shape
    n = len(keys)
    oe, oa = np.empty((n, D), np.float32), np.empty((n, D), np.float32)
    rc = lib().ecrm_oracle_degraded_read(_f32(E), _f32(A), _f32(PE), _f32(PA), C.c_uint64(R), C.c_uint32(D),
                                         C.c_uint32(k), C.c_uint32(S), _u64(keys), C.c_uint64(n),
                                         C.c_uint32(lost), _f32(oe), _f32(oa))
    if rc != 0:
        raise ValueError("key out of range")
    return oe, oa


def update(E, A, PE, PA, k: int, S: int, lr: float, eps: float, keys, grads,
           load_data=None, load_parity=None, threads: int = 1) -> None:
    """In-place update of the four fp32 tables (and, if given, the u64 load counters)."""
    R, D = E.shape
    n = len(keys)
    assert grads.shape == (n, D) and A.shape == (R, D) and PE.shape == (R // k, D) == PA.shape
    ld = _u64(load_data) if load_data is not None else None
    lp = _u64(load_parity) if load_parity is not None else None
    rc = lib().ecrm_oracle_update(_f32(E), _f32(A), _f32(PE), _f32(PA), C.c_uint64(R), C.c_uint32(D),
                                  C.c_uint32(k), C.c_uint32(S), C.c_float(lr), C.c_float(eps),
                                  _u64(keys), _f32(grads), C.c_uint64(n), ld, lp, C.c_int(threads))
    if rc == -1:
        raise ValueError("key out of range")
    if rc != 0:
        raise RuntimeError(f"oracle update failed ({rc})")


def update_rule(E, A, PE, PA, k: int, S: int, lr: float, eps: float, momentum: float, optimizer: int,
                combine: int, keys, grads, load_data=None, load_parity=None) -> None:
    """Adagrad (0) or momentum SGD (1), updates applied one by one (combine 0) or summed per entry (1)."""
    R, D = E.shape
    n = len(keys)
    assert grads.shape == (n, D)
    ld = _u64(load_data) if load_data is not None else None
    lp = _u64(load_parity) if load_parity is not None else None
    rc = lib().ecrm_oracle_update_rule(_f32(E), _f32(A), _f32(PE), _f32(PA), C.c_uint64(R), C.c_uint32(D),
                                       C.c_uint32(k), C.c_uint32(S), C.c_float(lr), C.c_float(eps),
                                       C.c_float(momentum), C.c_uint32(optimizer), C.c_uint32(combine),
                                       _u64(keys), _f32(grads), C.c_uint64(n), ld, lp)
    if rc == -1:
        raise ValueError("key out of range")
    if rc != 0:
        raise RuntimeError(f"oracle update_rule failed ({rc})")


def update_gradient_propagation(E, A, PE, PA, k: int, lr: float, eps: float, keys, grads) -> None:
    R, D = E.shape
    rc = lib().ecrm_oracle_update_gradient_propagation(
        _f32(E), _f32(A), _f32(PE), _f32(PA), C.c_uint64(R), C.c_uint32(D), C.c_uint32(k),
        C.c_float(lr), C.c_float(eps), _u64(keys), _f32(grads), C.c_uint64(len(keys)))
    if rc != 0:
        raise RuntimeError(f"oracle strawman failed ({rc})")


def update_gradient_propagation_rule(E, A, PE, PA, k: int, lr: float, eps: float, keys, grads,
                                     optimizer: int = 0, momentum: float = 0.0) -> None:
    """Gradient propagation (Sec. 3.3.1) under Adagrad (optimizer 0) or momentum SGD (optimizer 1)."""
    R, D = E.shape
    rc = lib().ecrm_oracle_update_gradient_propagation_rule(
        _f32(E), _f32(A), _f32(PE), _f32(PA), C.c_uint64(R), C.c_uint32(D), C.c_uint32(k),
        C.c_float(lr), C.c_float(eps), C.c_float(momentum), C.c_uint32(optimizer),
        _u64(keys), _f32(grads), C.c_uint64(len(keys)))
    if rc == -1:
        raise ValueError("key out of range")
    if rc != 0:
        raise RuntimeError(f"oracle strawman failed ({rc})")
