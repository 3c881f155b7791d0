"""Oracle optimizer updates (numpy float64).  TEST INFRASTRUCTURE ONLY.

Section 8 names the optimizers (Adam for ViT; SGD with momentum and decoupled
weight decay for the others) without formulas.  Readings:
  Adam:  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
         w <- w - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps),  t = global step >= 1
  SGDW:  m <- mu m + g;  w <- w - lr * m - lr * wd * w   (decay uses the old w)
Only selected tensors are touched; the state of an unselected tensor is frozen.
"""
import numpy as np


def adam(w, m, v, g, lr, beta1, beta2, eps, step):
    w, m, v, g = (np.asarray(a, dtype=np.float64) for a in (w, m, v, g))
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return w - lr * mhat / (np.sqrt(vhat) + eps), m, v


def sgdw(w, m, g, lr, momentum, wd):
    w, m, g = (np.asarray(a, dtype=np.float64) for a in (w, m, g))
    m = momentum * m + g
    return w - lr * m - lr * wd * w, m


def masked_update(kind, mask, weights, state, grads, **hp):
    """Apply the update to the selected tensors; return new (weights, state) lists.

    state[k] is (m, v) for Adam and (m,) for SGDW.  Unselected entries are
    returned as the very same objects.
    """
    new_w, new_s = list(weights), list(state)
    for k, sel in enumerate(mask):
        if not sel:
            continue
        if kind == "adam":
            w, m, v = adam(weights[k], state[k][0], state[k][1], grads[k],
                           hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["step"])
            new_w[k], new_s[k] = w, (m, v)
        elif kind == "sgdw":
            w, m = sgdw(weights[k], state[k][0], grads[k], hp["lr"], hp["momentum"], hp["wd"])
            new_w[k], new_s[k] = w, (m,)
        else:
            raise ValueError(kind)
    return new_w, new_s
