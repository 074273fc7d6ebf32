"""Oracle: the iteration gradient by its definition (test infrastructure only).

Sec. 4.3 property (i) and the proof-sketch appendix: the gradient an iteration commits is
(1/B) * sum of g(x) over the multiset A(t) of microbatches inside the contributing
survivors' buffers, whichever replica computed each term.  No replicas, no protocol, no
order: `exact_mean` sums each element with math.fsum (exactly rounded), `mean64` is the
same sum in float64 for inputs too large for a Python loop.
"""
import math

import numpy as np


def exact_mean(grads, B):
    """grads: list of equal-length 1-D arrays (one per committed microbatch).  Returns the
    float64 array whose element i is fsum(g[i] for g in grads) / B, the sum exactly rounded."""
    n = len(grads[0])
    cols = [np.asarray(g, np.float64) for g in grads]
    out = np.empty(n, np.float64)
    for i in range(n):
        out[i] = math.fsum(float(c[i]) for c in cols) / B
    return out


def mean64(grads, B):
    total = np.zeros(len(grads[0]), np.float64)
    for g in grads:
        total += np.asarray(g, np.float64)
    return total / float(B)
