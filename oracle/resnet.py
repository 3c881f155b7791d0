"""Oracle forward pass and masked backward pass of the bottleneck ResNet (numpy float64).
TEST INFRASTRUCTURE ONLY.

Same contract as oracle/nets.py: the gradient of the mean softmax cross-entropy w.r.t. every
selected tensor, computed on the tensor-level chain of Sections 2.3 and 5 with the loop
    for j = N-1 .. j*:  if M[j]: dw(j);   if j > j*: dy(j)
A branched network is unrolled into a sequence by execution order (Section 5).  Reading for the
projection shortcut of a block: its three tensors (convolution, gain, shift) come after the main
branch in the chain; passing the gradient through the shortcut convolution to the block input is
needed exactly when something before the block is selected, so it is part of dy() of the block's
first main convolution, where the two branches are summed.  Backward work of operations without
weights (ReLU, pooling) lies in the dy() of the tensor that has to be passed for it to be needed.

BatchNorm is "folded" (BASELINE): a per-channel affine y = gain * z + shift without batch
statistics.  Layout NHWC; convolution weights [out, kh, kw, in]; zero padding (k-1)/2.

Storage precision.  With store=None everything is float64 (the plain definition; this is what the
pins check).  The workload fixes bf16 storage for activations and error gradients; a ReLU network
turns a rounding of a value next to zero into a dropped or passed gradient element, so on a deep
network the exact result and ANY bf16 evaluation differ by far more than a rounding.  For the
comparison with a bf16 evaluation, `store` (e.g. round_bf16) is applied to every tensor that such
an evaluation keeps in memory between two operations: each convolution output except the stem's
(kept in fp32 so that the pooling argmax is decided on unrounded values), each affine/ReLU
output, the pooled features, the bf16 copy of the logit gradient that feeds the matrix products,
and each error gradient handed from one backward operation to the next.  Arithmetic stays float64.
The column gradient of a convolution with a kernel larger than 1x1 (d @ W, before the adjoint of
im2col sums its shifted copies into the input gradient) is NOT such a tensor: the storage contract
of the bf16 workloads (stated with the model description of the C ABI) keeps it in float32, so the
input gradient is rounded once, after the sum.  For a 1x1 convolution the product is the input
gradient itself and is rounded like any other stored product.
"""
import numpy as np

from .nets import _Tiny, _run_chain, softmax_xent

_F = np.float64


def round_bf16(a):
    """Nearest bf16 (ties to even) of float64 values, returned as float64."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(f.shape).astype(_F)


def _same(a):
    return a


# ----------------------------------------------------------------------------
# elementary pieces
# ----------------------------------------------------------------------------
def im2col(x, kh, kw, stride, pad):
    """[B,H,W,C] -> [B,Ho,Wo,kh*kw*C]; column order (ky, kx, c)."""
    B, H, W, C = x.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, C), dtype=_F)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    cols = np.empty((B, Ho, Wo, kh * kw * C), dtype=_F)
    for ky in range(kh):
        for kx in range(kw):
            t = ky * kw + kx
            cols[..., t * C:(t + 1) * C] = xp[:, ky:ky + stride * Ho:stride, kx:kx + stride * Wo:stride, :]
    return cols


def col2im(dcols, shape, kh, kw, stride, pad):
    """Adjoint of im2col: scatter-add the columns back onto the (padded) image."""
    B, H, W, C = shape
    Ho, Wo = dcols.shape[1], dcols.shape[2]
    dxp = np.zeros((B, H + 2 * pad, W + 2 * pad, C), dtype=_F)
    for ky in range(kh):
        for kx in range(kw):
            t = ky * kw + kx
            dxp[:, ky:ky + stride * Ho:stride, kx:kx + stride * Wo:stride, :] += dcols[..., t * C:(t + 1) * C]
    return dxp[:, pad:pad + H, pad:pad + W, :]


class Conv:
    """One convolution with everything its backward operations need."""

    def __init__(self, x, w, stride, q=_same):
        self.x_shape = x.shape
        self.w = w
        O, self.kh, self.kw, _ = w.shape
        self.stride, self.pad = stride, (self.kh - 1) // 2
        self.cols = im2col(x, self.kh, self.kw, stride, self.pad)
        self.wm = w.reshape(O, -1)
        self.out = q(self.cols @ self.wm.T)
        self.q = q

    def dw(self, d):
        return (d.reshape(-1, d.shape[-1]).T @ self.cols.reshape(-1, self.cols.shape[-1])).reshape(self.w.shape)

    def dx(self, d):
        dcols = d @ self.wm
        if self.kh == 1 and self.kw == 1:   # the product is the input gradient itself: a stored tensor
            dcols = self.q(dcols)
        return col2im(dcols, self.x_shape, self.kh, self.kw, self.stride, self.pad)


def maxpool_3x3_s2(x):
    """3x3 window, stride 2, padding 1 (with -inf); returns the output and the argmax tap
    (first maximum in (ky, kx) order)."""
    B, H, W, C = x.shape
    Ho, Wo = (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1
    xp = np.full((B, H + 2, W + 2, C), -np.inf, dtype=_F)
    xp[:, 1:1 + H, 1:1 + W, :] = x
    taps = np.stack([xp[:, ky:ky + 2 * Ho:2, kx:kx + 2 * Wo:2, :] for ky in range(3) for kx in range(3)], axis=0)
    arg = np.argmax(taps, axis=0)
    return np.take_along_axis(taps, arg[None], axis=0)[0], arg


def maxpool_3x3_s2_backward(d, arg, shape):
    B, H, W, C = shape
    Ho, Wo = d.shape[1], d.shape[2]
    dxp = np.zeros((B, H + 2, W + 2, C), dtype=_F)
    for ky in range(3):
        for kx in range(3):
            dxp[:, ky:ky + 2 * Ho:2, kx:kx + 2 * Wo:2, :] += d * (arg == ky * 3 + kx)
    return dxp[:, 1:1 + H, 1:1 + W, :]


def _sum_channels(a):
    return a.reshape(-1, a.shape[-1]).sum(axis=0)


# ----------------------------------------------------------------------------
# forward
# ----------------------------------------------------------------------------
def block_layout(cfg):
    """[(stage, block, stride, has_projection, first tensor index)] in forward order."""
    out, t = [], 3
    for si, nb in enumerate(cfg.blocks):
        for bi in range(nb):
            proj = bi == 0
            out.append((si, bi, 2 if (bi == 0 and si > 0) else 1, proj, t))
            t += 12 if proj else 9
    return out, t


def resnet_forward(cfg, weights, x, y, store=None):
    q = store if store is not None else _same
    W = [np.asarray(w, dtype=_F) for w in weights]
    x = np.asarray(x, dtype=_F)
    c = {"W": W, "q": q}
    stem = Conv(x, W[0], 2)                                    # output not rounded (see the header)
    stem_y = np.maximum(stem.out * W[1] + W[2], 0.0)
    pooled, arg = maxpool_3x3_s2(stem_y)                       # argmax on the unrounded values
    stem_y, pooled = q(stem_y), q(pooled)
    c.update(stem=stem, stem_y=stem_y, pool_arg=arg)
    blocks = []
    h = pooled
    layout, t_head = block_layout(cfg)
    for (si, bi, stride, proj, t) in layout:
        b = {"x": h, "t": t, "proj": proj}
        b["c1"] = Conv(h, W[t], 1, q)
        b["y1"] = q(np.maximum(b["c1"].out * W[t + 1] + W[t + 2], 0.0))
        b["c2"] = Conv(b["y1"], W[t + 3], stride, q)
        b["y2"] = q(np.maximum(b["c2"].out * W[t + 4] + W[t + 5], 0.0))
        b["c3"] = Conv(b["y2"], W[t + 6], 1, q)
        m = b["c3"].out * W[t + 7] + W[t + 8]
        if proj:
            b["sc"] = Conv(h, W[t + 9], stride, q)
            sh = b["sc"].out * W[t + 10] + W[t + 11]
        else:
            sh = h
        h = q(np.maximum(m + sh, 0.0))
        b["y"] = h
        blocks.append(b)
    p = q(h.mean(axis=(1, 2)))
    logits = p @ W[t_head].T + W[t_head + 1]
    loss, dlogits = softmax_xent(logits, np.asarray(y))
    c.update(blocks=blocks, last=h, pooled_in=pooled, p=p, logits=logits, dlogits=dlogits, t_head=t_head)
    return loss, c


# ----------------------------------------------------------------------------
# masked backward on the tensor-level chain
# ----------------------------------------------------------------------------
def resnet_step(cfg, weights, x, y, mask, store=None):
    loss, c = resnet_forward(cfg, weights, x, y, store)
    q = c["q"]
    W, blocks, t_head = c["W"], c["blocks"], c["t_head"]
    N = len(W)
    # state: d    = gradient w.r.t. the output of the tiny layer being visited
    #        dsum = gradient w.r.t. the pre-ReLU sum at the end of the current block (both branches)
    #        dsc  = gradient w.r.t. the output of the current block's shortcut convolution
    #        dl   = the logit gradient as the matrix products read it
    state = {"d": c["dlogits"], "dl": q(c["dlogits"]), "dsum": None, "dsc": None}

    def identity(s):
        pass

    chain = [None] * N

    # ---- head
    def head_dy(s):
        last = c["last"]
        dp = q(s["dl"] @ W[t_head])                                # through the head matrix
        d = np.broadcast_to(dp[:, None, None, :] / (last.shape[1] * last.shape[2]), last.shape)  # average pooling
        s["d"] = q(d * (last > 0.0))                               # ReLU closing the last block
        s["dsum"] = s["d"]
    chain[t_head] = _Tiny(lambda s: s["dl"].T @ c["p"], head_dy)
    chain[t_head + 1] = _Tiny(lambda s: s["d"].sum(axis=0), identity)

    # ---- blocks
    for bi_, b in enumerate(blocks):
        t = b["t"]
        prev_y = blocks[bi_ - 1]["y"] if bi_ > 0 else None

        def gain(conv_out, gidx, key):
            def dw(s):
                return _sum_channels(s[key] * conv_out)

            def dy(s):
                s[key if key == "d" else "dsc"] = q(s[key] * W[gidx])
            return _Tiny(dw, dy)

        def shift(key):
            return _Tiny(lambda s: _sum_channels(s[key]), identity)

        if b["proj"]:
            # shortcut branch (visited first from the output side): works on the block's summed gradient
            chain[t + 11] = shift("dsum")

            def sc_gain_dy(s, b=b, t=t):
                s["dsc"] = q(s["dsum"] * W[t + 10])
            chain[t + 10] = _Tiny(lambda s, b=b: _sum_channels(s["dsum"] * b["sc"].out), sc_gain_dy)
            chain[t + 9] = _Tiny(lambda s, b=b: b["sc"].dw(s["dsc"]), identity)   # its dX is part of dy(c1.W)
        # main branch
        chain[t + 8] = shift("d")
        chain[t + 7] = gain(b["c3"].out, t + 7, "d")

        def c3_dy(s, b=b):
            s["d"] = q(b["c3"].dx(s["d"]) * (b["y2"] > 0.0))
        chain[t + 6] = _Tiny(lambda s, b=b: b["c3"].dw(s["d"]), c3_dy)
        chain[t + 5] = shift("d")
        chain[t + 4] = gain(b["c2"].out, t + 4, "d")

        def c2_dy(s, b=b):
            s["d"] = q(b["c2"].dx(s["d"]) * (b["y1"] > 0.0))
        chain[t + 3] = _Tiny(lambda s, b=b: b["c2"].dw(s["d"]), c2_dy)
        chain[t + 2] = shift("d")
        chain[t + 1] = gain(b["c1"].out, t + 1, "d")

        def c1_dy(s, b=b, prev_y=prev_y):
            dx = b["c1"].dx(s["d"])
            dx = dx + (b["sc"].dx(s["dsc"]) if b["proj"] else s["dsum"])      # the two branches meet
            if prev_y is not None:
                s["d"] = q(dx * (prev_y > 0.0))                               # ReLU closing the previous block
            else:                                                             # max pooling, then the stem's ReLU
                s["d"] = q(maxpool_3x3_s2_backward(q(dx), c["pool_arg"], c["stem_y"].shape) * (c["stem_y"] > 0.0))
            s["dsum"] = s["d"]
        chain[t + 0] = _Tiny(lambda s, b=b: b["c1"].dw(s["d"]), c1_dy)

    # ---- stem
    chain[2] = _Tiny(lambda s: _sum_channels(s["d"]), identity)

    def stem_gain_dy(s):
        s["d"] = q(s["d"] * W[1])
    chain[1] = _Tiny(lambda s: _sum_channels(s["d"] * c["stem"].out), stem_gain_dy)
    chain[0] = _Tiny(lambda s: c["stem"].dw(s["d"]), None)

    grads, work = _run_chain(chain, mask, state)
    return dict(loss=loss, grads=grads, work=work, logits=c["logits"])
