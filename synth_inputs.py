"""Seeded synthetic inputs for the ECRM sparse-update path.

This module only *produces inputs*: keys, gradients and initial table values.  It holds none of
the method's arithmetic (no routing, optimizer or parity code) and is the one module that both
the test oracle's callers and the GPU path's callers draw their inputs from.

Everything is a pure function of (seed, tag, index) through one counter-based 64-bit mixer (the
SplitMix64 output function of Steele, Lea & Flood applied to ``stream + (index+1)*GOLDEN``), so
any element can be produced in isolation, on the host or on the device, bit-identically: the mixer
is written once with wrapping int64 torch ops that behave the same on both.

Values are small dyadic rationals, exactly representable in fp32:

    u     = top 24 bits of the hash                    (integer in [0, 2^24))
    grad  = (u - 2^23) * 2^-30        in [-2^-7, 2^-7)
    E0    = (u - 2^23) * 2^-27        in [-2^-4, 2^-4)
    A0    =  u         * 2^-34        in [0, 2^-10)

Keys stand in for the sparse-feature ids of a click-log data set (the paper trains on Criteo
Terabyte, which is not available here): either uniform over the R rows, or Zipf(theta) over a
number of ranks by exact inverse-CDF sampling, the ranks scattered injectively over the rows so
that hot rows fall on different stripes and servers.
"""
from __future__ import annotations

import numpy as np
import torch

GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1

TAG_KEY_UNIFORM = 1
TAG_KEY_ZIPF = 2
TAG_GRAD = 3
TAG_E0 = 4
TAG_A0 = 5
TAG_SCATTER = 6


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 holds for the same bits."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def mix64_py(z: int) -> int:
    """SplitMix64 output function on Python ints (reference for the tensor version)."""
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _M1) & _MASK64
    z = ((z ^ (z >> 27)) * _M2) & _MASK64
    return z ^ (z >> 31)


def stream_key(seed: int, tag: int) -> int:
    return mix64_py(seed * GOLDEN + tag)


def hash_py(seed: int, tag: int, index: int) -> int:
    return mix64_py(stream_key(seed, tag) + (index + 1) * GOLDEN)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    # logical shift right on int64: arithmetic shift, then clear the sign-extended bits
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix64(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_M1)
    z = (z ^ _lsr(z, 27)) * _s64(_M2)
    return z ^ _lsr(z, 31)


def hash_tensor(seed: int, tag: int, index: torch.Tensor) -> torch.Tensor:
    """h(seed, tag, index) for an int64 tensor of indices; int64 result (bits of the u64 hash)."""
    assert index.dtype == torch.int64
    z = (index + 1) * _s64(GOLDEN) + _s64(stream_key(seed, tag))
    return _mix64(z)


def _u24(seed: int, tag: int, index: torch.Tensor) -> torch.Tensor:
    return _lsr(hash_tensor(seed, tag, index), 40)


def values(seed: int, tag: int, start: int, count: int, device="cpu",
           chunk: int = 1 << 26) -> torch.Tensor:
    """fp32 values for flat element indices [start, start+count) of stream (seed, tag)."""
    out = torch.empty(count, dtype=torch.float32, device=device)
    for c0 in range(0, count, chunk):
        c1 = min(count, c0 + chunk)
        idx = torch.arange(start + c0, start + c1, dtype=torch.int64, device=device)
        u = _u24(seed, tag, idx)
        if tag == TAG_GRAD:
            v = (u - (1 << 23)).to(torch.float32) * (2.0 ** -30)
        elif tag == TAG_E0:
            v = (u - (1 << 23)).to(torch.float32) * (2.0 ** -27)
        elif tag == TAG_A0:
            v = u.to(torch.float32) * (2.0 ** -34)
        else:
            raise ValueError("not a value stream")
        out[c0:c1] = v
    return out


def grads(seed: int, first_item: int, n_items: int, D: int, device="cpu") -> torch.Tensor:
    """Gradient rows for items [first_item, first_item+n_items): shape [n_items, D] fp32."""
    return values(seed, TAG_GRAD, first_item * D, n_items * D, device).view(n_items, D)


def grad_rows(seed: int, items: np.ndarray, D: int) -> np.ndarray:
    """Gradient rows for an arbitrary list of item indices (host, for sampled checks)."""
    it = torch.from_numpy(np.asarray(items, dtype=np.int64))
    idx = (it[:, None] * D + torch.arange(D, dtype=torch.int64)[None, :]).reshape(-1)
    u = _u24(seed, TAG_GRAD, idx)
    v = (u - (1 << 23)).to(torch.float32) * (2.0 ** -30)
    return v.view(len(items), D).numpy()


def table_rows(seed: int, tag: int, rows: np.ndarray, D: int) -> np.ndarray:
    """Initial table rows (TAG_E0 or TAG_A0) for an arbitrary list of row ids (host)."""
    r = torch.from_numpy(np.asarray(rows, dtype=np.int64))
    idx = (r[:, None] * D + torch.arange(D, dtype=torch.int64)[None, :]).reshape(-1)
    u = _u24(seed, tag, idx)
    if tag == TAG_E0:
        v = (u - (1 << 23)).to(torch.float32) * (2.0 ** -27)
    elif tag == TAG_A0:
        v = u.to(torch.float32) * (2.0 ** -34)
    else:
        raise ValueError("not a table stream")
    return v.view(len(rows), D).numpy()


def table(seed: int, tag: int, R: int, D: int, device="cpu") -> torch.Tensor:
    return values(seed, tag, 0, R * D, device).view(R, D)


# ----------------------------------------------------------------------------------------------
# keys (torch int64 tensors on `device`; the *_keys wrappers return host u64 arrays)
# ----------------------------------------------------------------------------------------------

def uniform_keys_t(seed: int, start: int, count: int, R: int, device="cpu") -> torch.Tensor:
    """Uniform row ids in [0, R): (hash >> 1) mod R."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _lsr(hash_tensor(seed, TAG_KEY_UNIFORM, idx), 1) % R


_zipf_cache: dict = {}


def zipf_cdf(n_ranks: int, theta: float) -> np.ndarray:
    """Normalised fp64 prefix table of the weights r^-theta, r = 1..n_ranks (always summed on the
    host, sequentially, so that every device sees the same table)."""
    key = (n_ranks, theta)
    if key not in _zipf_cache:
        w = np.arange(1, n_ranks + 1, dtype=np.float64) ** (-theta)
        c = np.cumsum(w)
        c /= c[-1]
        _zipf_cache.clear()
        _zipf_cache[key] = {"cpu": torch.from_numpy(c)}
    return _zipf_cache[key]["cpu"].numpy()


def _zipf_cdf_t(n_ranks: int, theta: float, device) -> torch.Tensor:
    zipf_cdf(n_ranks, theta)
    slot = _zipf_cache[(n_ranks, theta)]
    dev = str(torch.device(device))
    if dev not in slot:
        slot[dev] = slot["cpu"].to(device)
    return slot[dev]


def _scatter_ranks_t(seed: int, rank: torch.Tensor, n_ranks: int, R: int) -> torch.Tensor:
    """Injective map rank -> row: an odd-multiplier bijection of [0, n_ranks) (n_ranks a power of
    two), spread over R >= n_ranks rows by a per-rank hashed offset inside R // n_ranks."""
    assert n_ranks & (n_ranks - 1) == 0 and R >= n_ranks and R % n_ranks == 0
    perm = (rank * 0x9E3779B1) & (n_ranks - 1)
    spread = R // n_ranks
    if spread == 1:
        return perm
    return perm * spread + _lsr(hash_tensor(seed, TAG_SCATTER, rank), 1) % spread


def _scatter_ranks(seed: int, rank: np.ndarray, n_ranks: int, R: int) -> np.ndarray:
    r = torch.from_numpy(np.asarray(rank, dtype=np.int64))
    return _scatter_ranks_t(seed, r, n_ranks, R).numpy().view(np.uint64)


def zipf_keys_t(seed: int, start: int, count: int, R: int, n_ranks: int, theta: float = 0.99,
                device="cpu") -> torch.Tensor:
    """Row ids whose popularity rank follows Zipf(theta) over n_ranks ranks (exact inverse CDF:
    binary search of a 53-bit uniform in the prefix table)."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    u = _lsr(hash_tensor(seed, TAG_KEY_ZIPF, idx), 11).to(torch.float64) * (2.0 ** -53)
    rank = torch.searchsorted(_zipf_cdf_t(n_ranks, theta, device), u, right=True)
    rank = torch.clamp(rank, max=n_ranks - 1)
    return _scatter_ranks_t(seed, rank, n_ranks, R)


def mixed_keys_t(seed: int, start: int, count: int, R: int, n_ranks: int, theta: float = 0.99,
                 device="cpu") -> torch.Tensor:
    """Even item indices uniform, odd item indices Zipf (the interleaved HBM-scale stream)."""
    assert start % 2 == 0
    out = uniform_keys_t(seed, start, count, R, device)
    out[1::2] = zipf_keys_t(seed, start, count, R, n_ranks, theta, device)[1::2]
    return out


def _host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def uniform_keys(seed, start, count, R):
    return _host(uniform_keys_t(seed, start, count, R))


def zipf_keys(seed, start, count, R, n_ranks, theta=0.99):
    return _host(zipf_keys_t(seed, start, count, R, n_ranks, theta))


def mixed_keys(seed, start, count, R, n_ranks, theta=0.99):
    return _host(mixed_keys_t(seed, start, count, R, n_ranks, theta))


# ----------------------------------------------------------------------------------------------
# the five workloads (sizes, seeds and skew are this repository's own choice; D, k, S from the
# paper's evaluation setup: 128 features per entry, k = 4, five servers)
# ----------------------------------------------------------------------------------------------

WORKLOADS = {
    #  name            n        R        seed  kind       batches
    "tiny":          dict(n=1 << 16, R=1 << 14, seed=0, kind="uniform", batches=1),
    "medium":        dict(n=1 << 22, R=1 << 20, seed=1, kind="uniform", batches=1),
    "large_uniform": dict(n=1 << 26, R=1 << 24, seed=2, kind="uniform", batches=1),
    "large_skewed":  dict(n=1 << 26, R=1 << 24, seed=3, kind="zipf", batches=1, n_ranks=1 << 24),
    "hbm_scale":     dict(n=1 << 28, R=1 << 25, seed=4, kind="mixed", batches=16, n_ranks=1 << 24),
}
DEFAULT_D = 128
DEFAULT_K = 4
DEFAULT_S = 5
DEFAULT_LR = 0.01
DEFAULT_EPS = 1e-8


def workload_keys_t(name: str, batch: int = 0, scale_shift: int = 0, device="cpu") -> torch.Tensor:
    """Keys (int64 tensor on `device`) of one batch of a named workload.  ``scale_shift`` halves n,
    R and the rank count that many times (same recipe, smaller)."""
    w = WORKLOADS[name]
    n = w["n"] >> scale_shift
    R = w["R"] >> scale_shift
    per = n // w["batches"]
    start = batch * per
    if w["kind"] == "uniform":
        return uniform_keys_t(w["seed"], start, per, R, device)
    nr = w["n_ranks"] >> scale_shift
    if w["kind"] == "zipf":
        return zipf_keys_t(w["seed"], start, per, R, nr, device=device)
    return mixed_keys_t(w["seed"], start, per, R, nr, device=device)


def workload_keys(name: str, batch: int = 0, scale_shift: int = 0) -> np.ndarray:
    return _host(workload_keys_t(name, batch, scale_shift))
