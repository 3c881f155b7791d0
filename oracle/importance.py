"""Oracle tensor importance (numpy float64).  TEST INFRASTRUCTURE ONLY.

Eq. 2: the importance of tensor k is the sum over its weights of
(dL/dw_i) * (delta w_i); by Eq. 5 at c = 0 the gradient is taken at the
current weights.  Reading of the sign (Section 4 describes the evaluation as
undoing a recent update): delta w = w_snapshot - w_current, the snapshot being
the weights the undo would restore, so that an update which lowered the loss
gets a positive importance, I_k ~ L(w_snapshot) - L(w_current) restricted to
tensor k (Eq. 6).
"""
import numpy as np

from . import nets


def importance_from_grads(grads, weights, snapshot):
    """Per-tensor sum of g * (w_snapshot - w); float64, one value per tensor."""
    out = np.zeros(len(grads), dtype=np.float64)
    for k, (g, w, s) in enumerate(zip(grads, weights, snapshot)):
        dw = np.asarray(s, dtype=np.float64) - np.asarray(w, dtype=np.float64)
        out[k] = np.sum(np.asarray(g, dtype=np.float64) * dw)
    return out


def abs_importance_from_grads(grads, weights, snapshot):
    """Per-tensor sum of |g * delta w|: the scale against which rounding error is judged."""
    out = np.zeros(len(grads), dtype=np.float64)
    for k, (g, w, s) in enumerate(zip(grads, weights, snapshot)):
        dw = np.asarray(s, dtype=np.float64) - np.asarray(w, dtype=np.float64)
        out[k] = np.sum(np.abs(np.asarray(g, dtype=np.float64) * dw))
    return out


def importance(cfg, weights, snapshot, x, y):
    """Full backward pass at the current weights (all tensors selected), then Eq. 2."""
    r = nets.step(cfg, weights, x, y, [1] * len(weights))
    return importance_from_grads(r["grads"], weights, snapshot), r


# ----------------------------------------------------------------------------
# the two metrics the ablation of Section 8 compares Eq. 2 with ("Weight", "Grad.")
# ----------------------------------------------------------------------------
# The paper names them only.  Reading: the L1 norm of the tensor's weights, and the L1 norm of its
# gradient on the batch.  Neither is additive in the sense of Section 4 (summing magnitudes does not
# estimate a loss change), which is the point of the ablation.
def weight_magnitude(weights):
    return np.array([np.abs(np.asarray(w, dtype=np.float64)).sum() for w in weights])


def grad_magnitude(grads):
    return np.array([np.abs(np.asarray(g, dtype=np.float64)).sum() for g in grads])
