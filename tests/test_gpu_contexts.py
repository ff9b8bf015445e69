"""Two contexts at once: different shapes and update rules, their calls interleaved on two streams.
A context's state (geometry, grid sizes, scratch) must be its own."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from ecrm_case import Case, grads_for, log

pytestmark = pytest.mark.gpu


def test_two_contexts_interleaved_on_two_streams():
    a = Case(4 * 3000, 128, 4, 5, max_batch=30000, seed=101)                              # Adagrad, D = 128
    b = Case(2 * 2500, 256, 2, 5, max_batch=30000, seed=103, optimizer=1, momentum=0.9)   # momentum SGD, D = 256
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    first = 0
    for step in range(4):
        n = [30000, 7001, 12289, 1][step]
        batches = []
        for c in (a, b):
            keys = si.uniform_keys(c.seed, first, n, c.R)
            keys[1::3] = 5                                  # a hot entry in each (split-chain path when n is large)
            g = grads_for(c.seed, first, n, c.D)
            batches.append((keys, torch.from_numpy(keys.view(np.int64)).cuda(), g))
        torch.cuda.synchronize()                            # inputs are ready; from here on only the two streams
        a.ctx.update(batches[0][1], batches[0][2], stream=sa)
        b.ctx.update(batches[1][1], batches[1][2], stream=sb)
        a.ctx.update(batches[0][1], batches[0][2], stream=sa)      # the same batch once more on each, crossing over
        b.ctx.update(batches[1][1], batches[1][2], stream=sb)
        torch.cuda.synchronize()
        for c, (keys, _, g) in zip((a, b), batches):       # oracle side, twice as well
            for _ in range(2):
                c.oracle_update(keys, g)
        first += n
    assert a.ctx.status(sa) == 0 and b.ctx.status(sb) == 0
    log("context A", a.compare("context A"))
    log("context B", b.compare("context B"))
    a.check_invariant()
    b.check_invariant()
