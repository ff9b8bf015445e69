"""Training while a failed server is rebuilt -- the protocol of Sec. 3.4 ("Training during
recovery") of the ECRM paper, stated plainly on the CPU (test infrastructure).

What Sec. 3.4 prescribes, in short: recovery proceeds chunk by chunk; the chunk being decoded is
locked, updates that would change anything the decoder reads for that chunk are set aside in a
buffer instead of being applied, and they are applied as soon as the chunk is done, when the lock
moves on to the next chunk.  Training does not stop at any point.
Readings taken here (the paper does not spell them out):
  * a chunk is a contiguous range of stripes; what the decoder reads for a chunk are all entries
    (and the parity) of the chunk's stripes that have a unit on the failed server;
  * an update to an entry that the failed server held cannot be applied before that entry has been
    rebuilt: it is buffered until its chunk is released, whether or not the chunk is locked;
  * buffered updates are replayed in arrival order; their load is counted when they are applied;
  * a batch whose buffered part does not fit the buffer is rejected as a whole;
  * the protocol is stated for asynchronous training (one update at a time, Sec. 2.1, 3.3.2) only.
    The synchronous variant sketched in Sec. 4.4 takes ONE step per modified entry and training step;
    a buffer that is replayed in one go would merge the waiting updates of several steps into a single
    step, which is not the training that would have happened without the failure.  combine=1 is refused.
All arithmetic is the oracle's (oracle.update / oracle.update_rule / oracle.recover_range).
"""
from __future__ import annotations

import numpy as np

import oracle


class RecoverySession:
    def __init__(self, E, A, PE, PA, k, S, lr, eps, server, chunks, capacity, load_data=None, load_parity=None,
                 optimizer=0, momentum=0.0, combine=0, threads=1):
        if combine:
            raise ValueError("recovery under load is defined for asynchronous training only (combine=0)")
        self.E, self.A, self.PE, self.PA = E, A, PE, PA
        self.k, self.S, self.lr, self.eps = k, S, lr, eps
        self.optimizer, self.momentum, self.combine, self.threads = optimizer, momentum, combine, threads
        self.ld, self.lp = load_data, load_parity
        self.server, self.capacity = server, capacity
        stripes = E.shape[0] // k
        self.spc = -(-stripes // chunks)                    # stripes per chunk
        self.chunks = -(-stripes // self.spc)
        self.next, self.locked, self.active = 0, False, True
        self.buf_keys, self.buf_grads = np.zeros(0, np.uint64), np.zeros((0, E.shape[1]), np.float32)

    # -- which updates have to wait ---------------------------------------------------------------
    def held(self, keys):
        if not self.active:
            return np.zeros(len(keys), bool)
        k, S, s = np.uint64(self.k), np.uint64(self.S), np.uint64(self.server)
        g, j = keys // k, keys % k
        parity_here = g % S == s
        member_here = (s + S - (g + np.uint64(1)) % S) % S          # the j with (g+1+j) mod S == s, if < k
        affected = parity_here | (member_here < k)
        chunk = g // np.uint64(self.spc)
        own_entry_lost = (~parity_here) & (member_here == j)
        in_locked = (chunk == np.uint64(self.next)) & self.locked
        return affected & (chunk >= np.uint64(self.next)) & (in_locked | own_entry_lost)

    def _apply(self, keys, grads):
        if len(keys) == 0:
            return
        if self.optimizer == 0 and self.combine == 0:
            oracle.update(self.E, self.A, self.PE, self.PA, self.k, self.S, self.lr, self.eps, keys, grads,
                          self.ld, self.lp, threads=self.threads)
        else:
            oracle.update_rule(self.E, self.A, self.PE, self.PA, self.k, self.S, self.lr, self.eps, self.momentum,
                               self.optimizer, self.combine, keys, grads, self.ld, self.lp)

    def update(self, keys, grads):
        """Returns False (and changes nothing) if the part that has to wait does not fit the buffer."""
        h = self.held(keys)
        if len(self.buf_keys) + int(h.sum()) > self.capacity:
            return False
        self.buf_keys = np.concatenate([self.buf_keys, keys[h]])
        self.buf_grads = np.concatenate([self.buf_grads, grads[h]])
        self._apply(np.ascontiguousarray(keys[~h]), np.ascontiguousarray(grads[~h]))
        return True

    # -- what a worker reads meanwhile ------------------------------------------------------------
    def read(self, keys):
        """Entries and their state as a worker sees them during the recovery (Sec. 3.4 serves a locked
        entry that has been updated meanwhile out of the buffer).  Reading taken here: the value
        is the one the entry will have once its waiting updates have been replayed, i.e. the stored
        entry with the buffered updates of that entry applied in arrival order; an entry that the
        failed server held and that is not rebuilt yet is first decoded from its stripe.  Nothing is
        modified."""
        keys = np.asarray(keys, np.uint64)
        D = self.E.shape[1]
        outE, outA = np.empty((len(keys), D), np.float32), np.empty((len(keys), D), np.float32)
        held = self.held(keys)
        k, S, s = np.uint64(self.k), np.uint64(self.S), np.uint64(self.server)
        for i, x in enumerate(keys):
            g, j = x // k, x % k
            member_here = (s + S - (g + np.uint64(1)) % S) % S
            lost_unbuilt = (self.active and g % S != s and member_here == j
                            and g // np.uint64(self.spc) >= np.uint64(self.next))
            if lost_unbuilt:
                e, a = oracle.degraded_read(self.E, self.A, self.PE, self.PA, self.k, self.S,
                                            np.array([x], np.uint64), self.server)
                e, a = e.copy(), a.copy()
            else:
                e, a = self.E[int(x):int(x) + 1].copy(), self.A[int(x):int(x) + 1].copy()
            if held[i]:
                sel = self.buf_keys == x
                if sel.any():
                    # the entry alone in a table of its own: the oracle's update rule on its waiting updates
                    pe, pa = e.copy(), a.copy()
                    oracle.update_rule(e, a, pe, pa, 1, 2, self.lr, self.eps, self.momentum, self.optimizer,
                                       self.combine, np.zeros(int(sel.sum()), np.uint64),
                                       np.ascontiguousarray(self.buf_grads[sel]), np.zeros(2, np.uint64),
                                       np.zeros(2, np.uint64))
            outE[i], outA[i] = e[0], a[0]
        return outE, outA

    # -- the recovery process ---------------------------------------------------------------------
    def lock(self):
        assert self.active and not self.locked and self.next < self.chunks
        self.locked = True

    def decode(self):
        assert self.locked
        stripes = self.E.shape[0] // self.k
        lo = self.next * self.spc
        oracle.recover_range(self.E, self.A, self.PE, self.PA, self.k, self.S, self.server, lo,
                             min(lo + self.spc, stripes))

    def unlock(self):
        assert self.locked
        self.locked = False
        self.next += 1
        keys, grads = self.buf_keys, self.buf_grads
        self.buf_keys, self.buf_grads = keys[:0], grads[:0]
        ok = self.update(keys, grads)                       # what still has to wait goes back into the buffer
        assert ok
        if self.next >= self.chunks:
            self.active = False
            assert len(self.buf_keys) == 0
