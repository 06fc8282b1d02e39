"""Oracle of the in-place backward of the log-softmax loss (Sec. 4.2.2 "Memory-Efficient Gradient
Computation", Alg. 3 "In-place Backward for Log-Softmax Loss").  TEST INFRASTRUCTURE: plain numpy in
fp64, the algorithm's steps in the paper's order and notation; only tests, the smoke check and the
benchmarks' cpu_baseline legs may use it.

Per row (one token position): logits z[V], target distribution p[V], upstream gradient g.
    s  = sum(p * g)
    pi = softmax(z)
    z <- -(p * g - pi * s)
which is d/dz of  L = -sum_v g_v p_v log softmax(z)_v.

Reading of what the paper leaves open: g is the gradient arriving at the per-position loss, i.e.
one number per row (loss weight / position mask times the upstream scalar); the formula is written
so that a per-element g of shape [N, V] works too, and the oracle accepts both.  The "masked"
softmax loss of the text has no mask in Alg. 3: masked positions are rows with g = 0 (their
gradient row is exactly zero).  p need not sum to one.
"""
import numpy as np


def logsoftmax_loss_bwd(z, p, g):
    """z, p: [N, V]; g: [N] or [N, V].  Returns the new contents of z as fp64 [N, V]."""
    z = np.asarray(z, dtype=np.float64)
    p = np.asarray(p, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    if g.ndim == 1:
        g = g[:, None]
    s = np.sum(p * g, axis=1, keepdims=True)
    e = np.exp(z - np.max(z, axis=1, keepdims=True))
    pi = e / np.sum(e, axis=1, keepdims=True)
    return -(p * g - pi * s)
