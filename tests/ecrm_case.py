"""Shared driver of the GPU parity tests: runs one configuration through libecrm (via the C ABI
binding) and through the CPU oracle on the same seeded inputs and compares them."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import synth_inputs as si
from paper_2104_01981_amd import Ecrm

RTOL = 1e-5
ATOL_E = 5e-7     # entries and parity entries (values ~1e-1)
ATOL_A = 1e-9     # accumulators and parity accumulators (values ~1e-3)


def log(*a):
    print(*a, flush=True)


class Case:
    def __init__(self, R, D, k, S, max_batch, seed=0, lr=si.DEFAULT_LR, eps=si.DEFAULT_EPS, optimizer=0,
                 momentum=0.0, combine=0, propagation=0):
        self.propagation = propagation
        self.R, self.D, self.k, self.S, self.seed, self.lr, self.eps = R, D, k, S, seed, lr, eps
        self.optimizer, self.momentum, self.combine = optimizer, momentum, combine
        dev = "cuda:0"
        self.E = si.table(seed, si.TAG_E0, R, D, dev)
        self.A = si.table(seed, si.TAG_A0, R, D, dev)
        self.PE = torch.zeros(R // k, D, device=dev)
        self.PA = torch.zeros(R // k, D, device=dev)
        self.ld = torch.zeros(S, dtype=torch.int64, device=dev)
        self.lp = torch.zeros(S, dtype=torch.int64, device=dev)
        self.ctx = Ecrm(R, D, k, S, lr, eps, max_batch, optimizer, momentum, combine, propagation)
        self.scratch = torch.empty(self.ctx.scratch_bytes(), dtype=torch.uint8, device=dev)
        self.ctx.bind(self.E, self.A, self.PE, self.PA, self.ld, self.lp, self.scratch)
        self.ctx.encode()
        # host mirror for the oracle
        self.hE = si.table(seed, si.TAG_E0, R, D).numpy().copy()
        self.hA = si.table(seed, si.TAG_A0, R, D).numpy().copy()
        self.hPE = oracle.encode(self.hE, k)
        self.hPA = oracle.encode(self.hA, k)
        self.hld = np.zeros(S, np.uint64)
        self.hlp = np.zeros(S, np.uint64)

    def update(self, keys_np, grads_t):
        """keys_np: u64 host array; grads_t: [n, D] fp32 device tensor.  Runs both sides."""
        keys_t = torch.from_numpy(keys_np.view(np.int64)).to("cuda:0")
        self.ctx.update(keys_t, grads_t, n=len(keys_np))
        self.oracle_update(keys_np, grads_t)

    def oracle_update(self, keys_np, grads_t):
        """The oracle's side of update() alone."""
        if self.propagation == 1:       # gradient propagation: the strawman, counted like the real thing
            oracle.update_gradient_propagation_rule(self.hE, self.hA, self.hPE, self.hPA, self.k, self.lr, self.eps,
                                                    keys_np, grads_t.cpu().numpy(), self.optimizer, self.momentum)
            ld, lp = oracle.load(keys_np, self.R, self.k, self.S)
            self.hld += ld
            self.hlp += lp
        elif self.propagation == 2:     # no redundancy: parities and their counters stay as they are
            oracle.update_rule(self.hE, self.hA, self.hPE.copy(), self.hPA.copy(), self.k, self.S, self.lr, self.eps,
                               self.momentum, self.optimizer, self.combine, keys_np, grads_t.cpu().numpy(),
                               self.hld, np.zeros(self.S, np.uint64))
        elif self.optimizer == 0 and self.combine == 0:
            oracle.update(self.hE, self.hA, self.hPE, self.hPA, self.k, self.S, self.lr, self.eps, keys_np,
                          grads_t.cpu().numpy(), self.hld, self.hlp, threads=min(16, oracle.max_threads()))
        else:
            oracle.update_rule(self.hE, self.hA, self.hPE, self.hPA, self.k, self.S, self.lr, self.eps,
                               self.momentum, self.optimizer, self.combine, keys_np, grads_t.cpu().numpy(),
                               self.hld, self.hlp)

    def compare(self, what=""):
        assert self.ctx.status() == 0
        report = {}
        for name, dev, host, atol in (("E", self.E, self.hE, ATOL_E), ("A", self.A, self.hA, ATOL_A),
                                      ("PE", self.PE, self.hPE, ATOL_E), ("PA", self.PA, self.hPA, ATOL_A)):
            got = dev.cpu().numpy()
            err = np.abs(got.astype(np.float64) - host.astype(np.float64))
            bound = RTOL * np.abs(host.astype(np.float64)) + atol
            mism = int((got != host).sum())
            report[name] = (float(err.max()), mism)
            assert (err <= bound).all(), f"{what} {name}: max err {err.max()} (worst ratio {(err / bound).max()})"
            assert mism <= 1e-4 * got.size + 2, f"{what} {name}: {mism} of {got.size} elements differ in the last bit"
        np.testing.assert_array_equal(self.ld.cpu().numpy().view(np.uint64), self.hld)
        np.testing.assert_array_equal(self.lp.cpu().numpy().view(np.uint64), self.hlp)
        return report

    def check_invariant(self):
        """Parity rows equal the re-encoded sums of the GPU's own output (to fp32 rounding)."""
        k, D = self.k, self.D
        for T, P, atol in ((self.E, self.PE, ATOL_E), (self.A, self.PA, ATOL_A)):
            s = T.double().view(-1, k, D)
            resid = (P.double() - s.sum(1)).abs()
            bound = RTOL * s.abs().sum(1) + atol * k
            assert bool((resid <= bound).all())


def grads_for(seed, first_item, n, D):
    return si.grads(seed, first_item, n, D, "cuda:0")
