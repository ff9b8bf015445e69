"""Per-item NumPy transcription of the ECRM update, for tiny inputs (test infrastructure).

Independent of ecrm_oracle.c: one Python loop over the items in arrival order, float64 row
arithmetic, no grouping, no shadows of untouched rows.  It follows Sec. 3.3.1 (the Adagrad step:
accumulator first, epsilon under the root) and Sec. 3.3.2 (the data server sends the differences
in entry and in optimizer state; the parity server adds them), with the rotating placement of
Sec. 3.2 for the per-server counts.
"""
from __future__ import annotations

import numpy as np


def update(E, A, PE, PA, k, S, lr, eps, keys, grads):
    """Returns new (E, A, PE, PA) as fp32 and (load_data, load_parity) as u64; inputs untouched."""
    lr = float(np.float32(lr))
    eps = float(np.float32(eps))
    e64 = {}
    a64 = {}
    pe64 = {}
    pa64 = {}
    load_data = np.zeros(S, np.uint64)
    load_parity = np.zeros(S, np.uint64)
    for i, x in enumerate(np.asarray(keys).tolist()):
        g, j = divmod(x, k)
        if x not in e64:
            e64[x] = E[x].astype(np.float64)
            a64[x] = A[x].astype(np.float64)
        if g not in pe64:
            pe64[g] = PE[g].astype(np.float64)
            pa64[g] = PA[g].astype(np.float64)
        grad = grads[i].astype(np.float64)
        a_new = a64[x] + grad * grad
        e_new = e64[x] - lr / np.sqrt(a_new + eps) * grad
        pe64[g] = pe64[g] + (e_new - e64[x])
        pa64[g] = pa64[g] + (a_new - a64[x])
        e64[x], a64[x] = e_new, a_new
        load_data[(g + 1 + j) % S] += 1
        load_parity[g % S] += 1
    En, An, PEn, PAn = E.copy(), A.copy(), PE.copy(), PA.copy()
    for x in e64:
        En[x] = e64[x].astype(np.float32)
        An[x] = a64[x].astype(np.float32)
    for g in pe64:
        PEn[g] = pe64[g].astype(np.float32)
        PAn[g] = pa64[g].astype(np.float32)
    return En, An, PEn, PAn, load_data, load_parity
