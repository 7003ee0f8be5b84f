"""Sec. 3.3 step 3: the update rule applied with the combined gradient on the
flat parameter array.  The paper names the rules (momentum, Nesterov momentum,
RMSProp, Adam) by reference to the Lasagne library, without formulas; the readings
taken are the published forms of those rules as that library states them, with
g = G + wd * p (coupled L2 weight decay on every element of the flat array):

  momentum   v' = m v - lr g ;            p' = p + v'
  nesterov   v' = m v - lr g ;            p' = p + m v' - lr g
  rmsprop    a' = rho a + (1-rho) g^2 ;   p' = p - lr g / sqrt(a' + eps)
  adam       m' = b1 m + (1-b1) g ; v' = b2 v + (1-b2) g^2 ;
             p' = p - lr sqrt(1-b2^t)/(1-b1^t) * m' / (sqrt(v') + eps),  t = 1, 2, ...
"""
import numpy as np


def sgd_momentum(p, v, G, lr, momentum, weight_decay=0.0):
    p = np.asarray(p, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    g = G + weight_decay * p
    v_new = momentum * v - lr * g
    return p + v_new, v_new


def nesterov_momentum(p, v, G, lr, momentum, weight_decay=0.0):
    p = np.asarray(p, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(G, dtype=np.float64) + weight_decay * p
    v_new = momentum * v - lr * g
    return p + momentum * v_new - lr * g, v_new


def rmsprop(p, a, G, lr, rho, eps, weight_decay=0.0):
    p = np.asarray(p, dtype=np.float64)
    a = np.asarray(a, dtype=np.float64)
    g = np.asarray(G, dtype=np.float64) + weight_decay * p
    a_new = rho * a + (1.0 - rho) * g * g
    return p - lr * g / np.sqrt(a_new + eps), a_new


def adam(p, m, v, G, lr, beta1, beta2, eps, t, weight_decay=0.0):
    """t is the number of this update (1 for the first)."""
    p = np.asarray(p, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(G, dtype=np.float64) + weight_decay * p
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    a_t = lr * np.sqrt(1.0 - beta2 ** t) / (1.0 - beta1 ** t)
    return p - a_t * m_new / (np.sqrt(v_new) + eps), m_new, v_new


def apply_rule(rule, p, s1, s2, G, h):
    """One update with rule in {"momentum","nesterov","rmsprop","adam"}; h is a
    dict of hyper-parameters (lr, momentum, rho, beta1, beta2, eps, t,
    weight_decay).  Returns (p', s1', s2') with s2' = None where unused."""
    wd = h.get("weight_decay", 0.0)
    if rule == "momentum":
        p2, v2 = sgd_momentum(p, s1, G, h["lr"], h["momentum"], wd)
        return p2, v2, None
    if rule == "nesterov":
        p2, v2 = nesterov_momentum(p, s1, G, h["lr"], h["momentum"], wd)
        return p2, v2, None
    if rule == "rmsprop":
        p2, a2 = rmsprop(p, s1, G, h["lr"], h["rho"], h["eps"], wd)
        return p2, a2, None
    if rule == "adam":
        return adam(p, s1, s2, G, h["lr"], h["beta1"], h["beta2"], h["eps"], h["t"], wd)
    raise ValueError(rule)


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
