"""Oracle of the in-place backward of the log-softmax loss (Sec. 4.2.2 "Memory-Efficient Gradient
Computation", Alg. 3).  TEST INFRASTRUCTURE: plain numpy in fp64; only tests, the smoke check and the
benchmarks' cpu_baseline legs may use it.

Definition.  Per row (one token position) with logits z[V], target weights p[V] and upstream
gradient g, the loss is  L = -sum_v w_v * log softmax(z)_v  with  w = p * g.  Since
d log softmax(z)_v / d z_u = [u == v] - softmax(z)_u, its gradient with respect to the logits is
    dL/dz_u = softmax(z)_u * sum_v w_v - w_u,
and that is what the operation leaves in place of the logits.  The oracle evaluates this
expression with log softmax taken through a log-sum-exp.

Reading of what the paper leaves open: g is the gradient arriving at the per-position loss, i.e.
one number per row (loss weight / position mask times the upstream scalar); a per-element g of
shape [N, V] is accepted too.  The "masked" softmax loss of the text shows no mask in Alg. 3:
masked positions are rows with g = 0 (their gradient row is exactly zero).  p need not sum to one.
"""
import numpy as np


def logsoftmax_loss_bwd(z, p, g):
    """z, p: [N, V]; g: [N] or [N, V].  Returns dL/dz, the new contents of z, as fp64 [N, V]."""
    z = np.asarray(z, dtype=np.float64)
    w = np.asarray(p, dtype=np.float64) * (np.asarray(g, dtype=np.float64)[:, None] if np.ndim(g) == 1 else np.asarray(g, dtype=np.float64))
    zmax = np.max(z, axis=1, keepdims=True)
    log_softmax = z - (zmax + np.log(np.sum(np.exp(z - zmax), axis=1, keepdims=True)))
    return np.exp(log_softmax) * np.sum(w, axis=1, keepdims=True) - w
