"""Sec. 3.3 step 3: the update rule applied with the combined gradient on the
flat parameter array.  The paper names the rule (momentum) without a formula;
the reading taken: g = G + wd * p ; v' = m * v - lr * g ; p' = p + v'
(coupled L2 weight decay on every element of the flat array)."""
import numpy as np


def sgd_momentum(p, v, G, lr, momentum, weight_decay=0.0):
    p = np.asarray(p, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    g = G + weight_decay * p
    v_new = momentum * v - lr * g
    return p + v_new, v_new


def reduce_and_update(p, v, worker_grads, lr, momentum, weight_decay=0.0,
                      weights=None, worker_losses=None):
    """Steps 2 and 3 of Sec. 3.3 back to back: average the N per-worker flat
    gradients, then update.  Also the mean of the per-worker scalar losses
    (Sec. 3.2 step 3) when given.  Returns (p', v', G, loss or None)."""
    from .reduce import reduce_buffers
    G = reduce_buffers(list(worker_grads), "mean", weights)
    loss = None
    if worker_losses is not None:
        loss = float(reduce_buffers([np.atleast_1d(np.float64(x)) for x in worker_losses],
                                    "mean", weights)[0])
    p2, v2 = sgd_momentum(p, v, G, lr, momentum, weight_decay)
    return p2, v2, G, loss
