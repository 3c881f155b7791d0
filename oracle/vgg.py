"""Oracle forward pass and masked backward pass of a plain convolution stack (VGG family; numpy
float64).  TEST INFRASTRUCTURE ONLY.

Same contract as oracle/nets.py and oracle/resnet.py: the gradient of the mean softmax
cross-entropy w.r.t. every selected tensor, on the tensor-level chain of Sections 2.3 and 5 with
the loop
    for j = N-1 .. j*:  if M[j]: dw(j);   if j > j*: dy(j)
Every convolution and linear layer is two tensors, Kernel and Bias (Section 5.1): the bias has
t_dy = 0 (its dy() is the identity), the kernel's dy() passes the gradient to the layer input and
on through the operations without weights in front of it (ReLU, 2x2 max pooling, flattening), up
to the pre-activation of the previous layer.

Layout NHWC; convolution weights [out, kh, kw, in] with zero padding 1; the linear layers read the
pooled features flattened in (h, w, c) order.  `store` is the storage-precision hook described in
oracle/resnet.py: applied to every tensor a bf16 evaluation keeps in memory (activations after
bias + ReLU, pooled features, error gradients); a layer's pre-activation is not such a tensor
here (bias and ReLU are applied to the unrounded sum), and neither is the column gradient of a
3x3 convolution (d @ W, before the adjoint of im2col sums it into the input gradient, which is
rounded once).
"""
import numpy as np

from .nets import _Tiny, _run_chain, softmax_xent
from .resnet import Conv, _same

_F = np.float64


def maxpool_2x2(x):
    """2x2 window, stride 2; returns the output and the chosen tap (first maximum in (dy, dx) order)."""
    B, H, W, C = x.shape
    assert H % 2 == 0 and W % 2 == 0
    taps = np.stack([x[:, dy::2, dx::2, :] for dy in range(2) for dx in range(2)], axis=0)
    arg = np.argmax(taps, axis=0)
    return np.take_along_axis(taps, arg[None], axis=0)[0], arg


def maxpool_2x2_backward(d, arg, shape):
    dx = np.zeros(shape, dtype=_F)
    for dy_ in range(2):
        for dx_ in range(2):
            dx[:, dy_::2, dx_::2, :] = d * (arg == dy_ * 2 + dx_)
    return dx


def layout(cfg):
    """[(tensor index of the kernel, stage, first of its stage)] per convolution, and the index of fc0.W."""
    convs, t = [], 0
    for s, n in enumerate(cfg.convs):
        for k in range(n):
            convs.append((t, s, k == 0))
            t += 2
    return convs, t


def vgg_forward(cfg, weights, x, y, store=None):
    q = store if store is not None else _same
    W = [np.asarray(w, dtype=_F) for w in weights]
    h = np.asarray(x, dtype=_F)
    convs, t_fc = layout(cfg)
    units, pools = [], []
    for i, (t, s, first) in enumerate(convs):
        cv = Conv(h, W[t], 1)                                  # pre-activation: not a stored tensor
        yv = q(np.maximum(cv.out + W[t + 1], 0.0))
        units.append({"t": t, "conv": cv, "y": yv, "stage": s})
        h = yv
        last_of_stage = i + 1 == len(convs) or convs[i + 1][2]
        if last_of_stage:
            p, arg = maxpool_2x2(yv)                           # values are already rounded: p needs no rounding
            pools.append({"arg": arg, "in_shape": yv.shape})
            h = p
    feat = h.reshape(h.shape[0], -1)
    acts = [feat]                                              # input of fc j
    n_fc = len(cfg.fc) + 1
    a = feat
    for j in range(n_fc):
        z = a @ W[t_fc + 2 * j].T + W[t_fc + 2 * j + 1]
        if j + 1 < n_fc:
            a = q(np.maximum(z, 0.0))
            acts.append(a)
    logits = z
    loss, dlogits = softmax_xent(logits, np.asarray(y))
    c = dict(W=W, q=q, units=units, pools=pools, acts=acts, pooled_shape=h.shape, logits=logits, dlogits=dlogits,
             t_fc=t_fc, n_fc=n_fc)
    return loss, c


def vgg_step(cfg, weights, x, y, mask, store=None):
    loss, c = vgg_forward(cfg, weights, x, y, store)
    W, q, units, pools, acts = c["W"], c["q"], c["units"], c["pools"], c["acts"]
    t_fc, n_fc = c["t_fc"], c["n_fc"]
    N = len(W)
    # d: gradient w.r.t. the pre-activation of the layer being visited; dl: the logit gradient as
    # the matrix products read it
    state = {"d": c["dlogits"], "dl": q(c["dlogits"])}

    def identity(s):
        pass

    def through_last_pool(dfeat):
        """Gradient of the flattened features -> pre-activation of the last convolution."""
        dp = dfeat.reshape(c["pooled_shape"])
        u = units[-1]
        return maxpool_2x2_backward(dp, pools[-1]["arg"], pools[-1]["in_shape"]) * (u["y"] > 0.0)

    chain = [None] * N
    # ---- linear layers
    for j in range(n_fc):
        tw = t_fc + 2 * j
        key = "dl" if j == n_fc - 1 else "d"                   # the last layer multiplies the rounded copy

        def fc_dw(s, j=j, key=key):
            return s[key].T @ acts[j]

        def fc_dy(s, j=j, tw=tw, key=key):
            dx = q(s[key] @ W[tw])                             # stored GEMM result
            if j > 0:
                s["d"] = q(dx * (acts[j] > 0.0))               # ReLU of the previous linear layer
            else:
                s["d"] = q(through_last_pool(dx))
        chain[tw] = _Tiny(fc_dw, fc_dy)
        chain[tw + 1] = _Tiny(lambda s: s["d"].sum(axis=0), identity)
    # ---- convolutions
    for i, u in enumerate(units):
        t = u["t"]

        def conv_dy(s, i=i, u=u):
            dx = u["conv"].dx(s["d"])
            prev = units[i - 1]
            if prev["stage"] != u["stage"]:                    # a pooling layer sits in between
                pl = pools[prev["stage"]]
                dx = maxpool_2x2_backward(q(dx), pl["arg"], pl["in_shape"])
            s["d"] = q(dx * (prev["y"] > 0.0))
        chain[t] = _Tiny(lambda s, u=u: u["conv"].dw(s["d"]), conv_dy if i > 0 else None)
        chain[t + 1] = _Tiny(lambda s: s["d"].reshape(-1, s["d"].shape[-1]).sum(axis=0), identity)
    grads, work = _run_chain(chain, mask, state)
    return dict(loss=loss, grads=grads, work=work, logits=c["logits"])
