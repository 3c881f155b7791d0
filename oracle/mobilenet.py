"""Oracle forward pass and masked backward pass of an inverted-residual network (MobileNetV2 family;
numpy float64).  TEST INFRASTRUCTURE ONLY.

Same contract as oracle/nets.py and oracle/resnet.py: the gradient of the mean softmax
cross-entropy w.r.t. every selected tensor, on the tensor-level chain of Sections 2.3 and 5 with
the loop
    for j = N-1 .. j*:  if M[j]: dw(j);   if j > j*: dy(j)
Every convolution is followed by a folded BatchNorm, a per-channel affine y = gain * z + shift, so
it contributes three tensors W, g, b (the tiny layers of Section 5.1); ReLU6 follows the stem, the
expansion, the depthwise convolution and the last convolution, nothing follows the projection.  A
block of stride 1 whose input and output widths agree adds its input to its output.  From the
output side the gradient of such a block's output goes both into the projection's affine and,
untouched, to the block input; the two meet again in dy() of the block's first weight (the
expansion), which is needed exactly when something before the block is selected.

The derivative of ReLU6 is taken as one strictly inside (0, 6) and zero elsewhere, decided on the
stored activation.  Layout NHWC; dense convolution weights [out, kh, kw, in], depthwise ones
[channels, 3, 3, 1]; zero padding 1 for the 3x3 kernels.  `store` is the storage-precision hook
described in oracle/resnet.py (applied to convolution outputs, activations, block outputs, pooled
features, error gradients handed from one backward operation to the next).
"""
import numpy as np

from .nets import _Tiny, _run_chain, softmax_xent
from .resnet import Conv, _same, _sum_channels

_F = np.float64


def relu6(a):
    return np.minimum(np.maximum(a, 0.0), 6.0)


def relu6_mask(y):
    return (y > 0.0) & (y < 6.0)


class Depthwise:
    """3x3 depthwise convolution, zero padding 1: out[b,ho,wo,c] = sum_taps x[b, ho*s+ky-1, wo*s+kx-1, c] * w[c,ky,kx]."""

    def __init__(self, x, w, stride, q=_same):
        B, H, W, C = x.shape
        self.x_shape, self.stride = x.shape, stride
        self.w = w.reshape(C, 3, 3)
        self.Ho, self.Wo = (H + 2 - 3) // stride + 1, (W + 2 - 3) // stride + 1
        self.xp = np.zeros((B, H + 2, W + 2, C), dtype=_F)
        self.xp[:, 1:1 + H, 1:1 + W, :] = x
        out = np.zeros((B, self.Ho, self.Wo, C), dtype=_F)
        for ky in range(3):
            for kx in range(3):
                out += self._tap(ky, kx) * self.w[:, ky, kx]
        self.out = q(out)

    def _tap(self, ky, kx):
        s = self.stride
        return self.xp[:, ky:ky + s * self.Ho:s, kx:kx + s * self.Wo:s, :]

    def dw(self, d):
        g = np.empty((self.w.shape[0], 3, 3, 1), dtype=_F)
        for ky in range(3):
            for kx in range(3):
                g[:, ky, kx, 0] = _sum_channels(d * self._tap(ky, kx))
        return g

    def dx(self, d):
        B, H, W, C = self.x_shape
        s = self.stride
        dxp = np.zeros((B, H + 2, W + 2, C), dtype=_F)
        for ky in range(3):
            for kx in range(3):
                dxp[:, ky:ky + s * self.Ho:s, kx:kx + s * self.Wo:s, :] += d * self.w[:, ky, kx]
        return dxp[:, 1:1 + H, 1:1 + W, :]


def block_layout(cfg):
    """[(c_in, hidden, c_out, stride, has_expansion, has_shortcut, first tensor index)] and the index of last.W."""
    out, t, cin = [], 3, cfg.stem
    for (tf, c, n, s) in cfg.settings:
        for i in range(n):
            stride = s if i == 0 else 1
            expand = tf != 1
            out.append((cin, cin * tf, c, stride, expand, stride == 1 and cin == c, t))
            t += 9 if expand else 6
            cin = c
    return out, t


def mobilenet_forward(cfg, weights, x, y, store=None):
    q = store if store is not None else _same
    W = [np.asarray(w, dtype=_F) for w in weights]
    x = np.asarray(x, dtype=_F)
    stem = Conv(x, W[0], 2, q)
    h = q(relu6(stem.out * W[1] + W[2]))
    c = {"W": W, "q": q, "stem": stem, "stem_y": h}
    blocks = []
    layout, t_last = block_layout(cfg)
    for (cin, hid, cout, stride, expand, shortcut, t) in layout:
        b = {"x": h, "t": t, "expand": expand, "shortcut": shortcut}
        a = h
        if expand:
            b["exp"] = Conv(h, W[t], 1, q)
            a = q(relu6(b["exp"].out * W[t + 1] + W[t + 2]))
            b["y_exp"] = a
            t += 3
        b["t_dw"] = t
        b["dw"] = Depthwise(a, W[t], stride, q)
        a = q(relu6(b["dw"].out * W[t + 1] + W[t + 2]))
        b["y_dw"] = a
        b["proj"] = Conv(a, W[t + 3], 1, q)
        p = b["proj"].out * W[t + 4] + W[t + 5]
        h = q(p + h) if shortcut else q(p)
        b["y"] = h
        blocks.append(b)
    last = Conv(h, W[t_last], 1, q)
    last_y = q(relu6(last.out * W[t_last + 1] + W[t_last + 2]))
    p = q(last_y.mean(axis=(1, 2)))
    logits = p @ W[t_last + 3].T + W[t_last + 4]
    loss, dlogits = softmax_xent(logits, np.asarray(y))
    c.update(blocks=blocks, last=last, last_y=last_y, p=p, logits=logits, dlogits=dlogits, t_last=t_last)
    return loss, c


def mobilenet_step(cfg, weights, x, y, mask, store=None):
    loss, c = mobilenet_forward(cfg, weights, x, y, store)
    q, W, blocks, t_last = c["q"], c["W"], c["blocks"], c["t_last"]
    N = len(W)
    # state: d    = gradient w.r.t. the output of the tiny layer being visited
    #        dsum = gradient w.r.t. the output of the current block (what a shortcut hands to the block input)
    #        dl   = the logit gradient as the matrix products read it
    state = {"d": c["dlogits"], "dl": q(c["dlogits"]), "dsum": None}

    def identity(s):
        pass

    def gain(conv_out, gidx):
        def dy(s):
            s["d"] = q(s["d"] * W[gidx])
        return _Tiny(lambda s: _sum_channels(s["d"] * conv_out), dy)

    shift = lambda: _Tiny(lambda s: _sum_channels(s["d"]), identity)
    chain = [None] * N

    # ---- head: linear layer, average pooling, ReLU6 of the last convolution
    def head_dy(s):
        ly = c["last_y"]
        dp = q(s["dl"] @ W[t_last + 3])
        d = np.broadcast_to(dp[:, None, None, :] / (ly.shape[1] * ly.shape[2]), ly.shape)
        s["d"] = q(d * relu6_mask(ly))
    chain[t_last + 4] = _Tiny(lambda s: s["d"].sum(axis=0), identity)
    chain[t_last + 3] = _Tiny(lambda s: s["dl"].T @ c["p"], head_dy)
    chain[t_last + 2] = shift()
    chain[t_last + 1] = gain(c["last"].out, t_last + 1)

    def last_dy(s):
        s["d"] = q(c["last"].dx(s["d"]))           # the block output in front of it has no activation
        s["dsum"] = s["d"]
    chain[t_last] = _Tiny(lambda s: c["last"].dw(s["d"]), last_dy)

    # ---- blocks, each entered with d = dsum = gradient of its output
    for bi, b in enumerate(blocks):
        t, td = b["t"], b["t_dw"]
        chain[td + 5] = shift()
        chain[td + 4] = gain(b["proj"].out, td + 4)

        def proj_dy(s, b=b):
            s["d"] = q(b["proj"].dx(s["d"]) * relu6_mask(b["y_dw"]))
        chain[td + 3] = _Tiny(lambda s, b=b: b["proj"].dw(s["d"]), proj_dy)
        chain[td + 2] = shift()
        chain[td + 1] = gain(b["dw"].out, td + 1)

        def to_block_input(s, dx, b=b, bi=bi):
            """dx: gradient reaching the block input through the main branch."""
            if b["shortcut"]:
                dx = dx + s["dsum"]
            if bi == 0:
                s["d"] = q(dx * relu6_mask(c["stem_y"]))   # ReLU6 of the stem
            else:
                s["d"] = q(dx)                             # the previous block ends without an activation
            s["dsum"] = s["d"]

        if b["expand"]:
            def dw_dy(s, b=b):
                s["d"] = q(b["dw"].dx(s["d"]) * relu6_mask(b["y_exp"]))
            chain[td] = _Tiny(lambda s, b=b: b["dw"].dw(s["d"]), dw_dy)
            chain[t + 2] = shift()
            chain[t + 1] = gain(b["exp"].out, t + 1)
            chain[t] = _Tiny(lambda s, b=b: b["exp"].dw(s["d"]),
                             lambda s, b=b, f=to_block_input: f(s, b["exp"].dx(s["d"])))
        else:
            chain[td] = _Tiny(lambda s, b=b: b["dw"].dw(s["d"]),
                              lambda s, b=b, f=to_block_input: f(s, b["dw"].dx(s["d"])))

    # ---- stem
    chain[2] = shift()
    chain[1] = gain(c["stem"].out, 1)
    chain[0] = _Tiny(lambda s: c["stem"].dw(s["d"]), None)

    grads, work = _run_chain(chain, mask, state)
    return dict(loss=loss, grads=grads, work=work, logits=c["logits"])
