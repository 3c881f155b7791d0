"""Oracle forward pass and masked backward pass (numpy float64).  TEST INFRASTRUCTURE ONLY.

What is computed is the plain definition: the reverse-mode gradient of the
mean softmax cross-entropy loss with respect to every *selected* tensor, at
the given weights.  Selective training changes no value; it only skips work
(Section 2.2): a tensor's weight gradient is computed only if it is selected,
and the error gradient is passed backwards only as far as the input-most
selected tensor.

The backward pass is written on the tensor-level chain of Sections 2.3 and 5:
each trainable tensor j is a tiny sequential layer with two backward
operations,
    dw(j): the gradient of the loss w.r.t. tensor j,
    dy(j): passing the error gradient from the output of tensor j's tiny layer
           to the output of tensor j-1's tiny layer,
and the loop
    for j = N-1 .. j*:  if M[j]: dw(j);   if j > j*: dy(j)
with j* the smallest selected index is the whole backward pass.  Backward
work of non-trainable operations (ReLU, GELU, the attention core, residual
additions) lies inside the dy() of the tensor that has to be passed for that
work to be needed.  Every executed operation is appended to `work`, so tests
can compare the executed set with the time model's f(M).

Network internals the paper leaves to its stock models (readings, used
identically by the HIP path): pre-LN blocks, LayerNorm eps 1e-6, exact (erf)
GELU, attention scale 1/sqrt(head size), no dropout, learned position
embedding and CLS token, final LayerNorm, linear head on the CLS row, mean
cross-entropy over the batch.  Matrix weights are stored [out, in].
"""
import numpy as np
from scipy.special import erf

_F = np.float64


def _f64(a):
    return np.asarray(a, dtype=_F)


# ----------------------------------------------------------------------------
# elementary pieces
# ----------------------------------------------------------------------------
def softmax_xent(logits, y):
    """Mean cross-entropy of softmax(logits) against integer labels; also d loss / d logits."""
    B = logits.shape[0]
    z = logits - logits.max(axis=1, keepdims=True)
    lse = np.log(np.exp(z).sum(axis=1, keepdims=True))
    logp = z - lse
    loss = -logp[np.arange(B), y].mean()
    d = np.exp(logp)
    d[np.arange(B), y] -= 1.0
    return loss, d / B


def ln_forward(h, gain, shift, eps):
    mu = h.mean(axis=-1, keepdims=True)
    var = ((h - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (h - mu) * rstd
    return xhat * gain + shift, xhat, rstd


def ln_backward_input(d, xhat, rstd, gain):
    """Gradient w.r.t. the LayerNorm input, given the gradient d w.r.t. gain*xhat."""
    dxhat = d * gain
    return rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                   - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))


def gelu(u):
    return 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))


def gelu_grad(u):
    return 0.5 * (1.0 + erf(u / np.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


def _heads(a, B, T, H, dh):
    """[B, T, H*dh] -> [B, H, T, dh]"""
    return a.reshape(B, T, H, dh).transpose(0, 2, 1, 3)


def _unheads(a, B, T, H, dh):
    """[B, H, T, dh] -> [B, T, H*dh]"""
    return a.transpose(0, 2, 1, 3).reshape(B, T, H * dh)


class _Tiny:
    """One trainable tensor seen as a tiny layer: its dw() and dy() closures."""
    __slots__ = ("dw", "dy")

    def __init__(self, dw, dy):
        self.dw = dw
        self.dy = dy


def _run_chain(chain, mask, state):
    """The masked backward loop over the tensor-level chain."""
    N = len(chain)
    mask = [bool(m) for m in mask]
    assert len(mask) == N
    grads = [None] * N
    work = []
    if not any(mask):
        return grads, work                      # empty selection: no backward work at all
    jstar = mask.index(True)
    for j in range(N - 1, jstar - 1, -1):
        if mask[j]:
            grads[j] = chain[j].dw(state)
            work.append(("dw", j))
        if j > jstar:
            chain[j].dy(state)
            work.append(("dy", j))
    return grads, work


# ----------------------------------------------------------------------------
# ReLU MLP without biases (BASELINE configs[0])
# ----------------------------------------------------------------------------
def mlp_forward(cfg, weights, x, y):
    W = [_f64(w) for w in weights]
    a = _f64(x)
    acts, pre = [a], []
    for i, w in enumerate(W):
        z = a @ w.T
        pre.append(z)
        if i + 1 < len(W):
            a = np.maximum(z, 0.0)
            acts.append(a)
    loss, dlogits = softmax_xent(pre[-1], np.asarray(y))
    return loss, dict(W=W, acts=acts, pre=pre, dlogits=dlogits, logits=pre[-1])


def mlp_step(cfg, weights, x, y, mask):
    """Loss, gradients of the selected tensors (None elsewhere), executed backward work."""
    loss, c = mlp_forward(cfg, weights, x, y)
    W, acts, pre = c["W"], c["acts"], c["pre"]
    state = {"d": c["dlogits"]}
    chain = []
    for i in range(len(W)):
        def dw(s, i=i):
            return s["d"].T @ acts[i]

        def dy(s, i=i):
            # through the matrix, then through the ReLU that precedes it
            s["d"] = (s["d"] @ W[i]) * (pre[i - 1] > 0.0)
        chain.append(_Tiny(dw, dy))
    grads, work = _run_chain(chain, mask, state)
    return dict(loss=loss, grads=grads, work=work, logits=c["logits"])


# ----------------------------------------------------------------------------
# pre-LN vision transformer encoder (BASELINE configs[1..3])
# ----------------------------------------------------------------------------
def vit_forward(cfg, weights, x, y):
    W = [_f64(w) for w in weights]
    x = _f64(x)
    B, T, D, H, dh, L = x.shape[0], cfg.tokens, cfg.width, cfg.heads, cfg.head_dim, cfg.blocks
    eps, scale = cfg.ln_eps, 1.0 / np.sqrt(dh)
    pW, pb, cls, pos = W[0:4]
    e = x @ pW.T + pb                                             # [B, T-1, D]
    h = np.concatenate([np.broadcast_to(cls, (B, 1, D)), e], axis=1) + pos
    blocks = []
    for l in range(L):
        g1, b1, Wqkv, bqkv, Wo, bo, g2, b2, W1, c1, W2, c2 = W[4 + 12 * l: 16 + 12 * l]
        blk = {"h_in": h}
        a1, blk["xhat1"], blk["rstd1"] = ln_forward(h, g1, b1, eps)
        qkv = a1 @ Wqkv.T + bqkv
        q, k, v = (_heads(qkv[..., i * D:(i + 1) * D], B, T, H, dh) for i in range(3))
        s = (q @ k.transpose(0, 1, 3, 2)) * scale
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=-1, keepdims=True)
        o = _unheads(p @ v, B, T, H, dh)
        h_mid = h + (o @ Wo.T + bo)
        a2, blk["xhat2"], blk["rstd2"] = ln_forward(h_mid, g2, b2, eps)
        u = a2 @ W1.T + c1
        ga = gelu(u)
        h = h_mid + (ga @ W2.T + c2)
        blk.update(a1=a1, q=q, k=k, v=v, p=p, o=o, a2=a2, u=u, ga=ga)
        blocks.append(blk)
    gf, bf, Wh, bh = W[-4:]
    zc, xhatf, rstdf = ln_forward(h[:, 0, :], gf, bf, eps)       # the head reads the CLS row only
    logits = zc @ Wh.T + bh
    loss, dlogits = softmax_xent(logits, np.asarray(y))
    return loss, dict(W=W, x=x, blocks=blocks, zc=zc, xhatf=xhatf, rstdf=rstdf,
                      logits=logits, dlogits=dlogits, dims=(B, T, D, H, dh, L, scale))


def vit_step(cfg, weights, x, y, mask):
    """Loss, gradients of the selected tensors (None elsewhere), executed backward work."""
    loss, c = vit_forward(cfg, weights, x, y)
    W, blocks = c["W"], c["blocks"]
    B, T, D, H, dh, L, scale = c["dims"]
    N = len(W)
    # state: d = gradient w.r.t. the output of the tiny layer being visited,
    #        skip = gradient carried by the residual connection around the current sub-block
    state = {"d": c["dlogits"], "skip": None}

    def identity(s):
        pass

    def rows(a):                                   # collapse [B, T, n] to [B*T, n]
        return a.reshape(-1, a.shape[-1])

    def bias():
        return lambda s: rows(s["d"]).sum(axis=0)

    def matrix_dw(inp):
        return lambda s: rows(s["d"]).T @ rows(inp)

    chain = [None] * N

    # --- embedding -----------------------------------------------------------
    chain[0] = _Tiny(matrix_dw(c["x"]), None)                           # patch.W (never passed)
    chain[1] = _Tiny(bias(), identity)                                  # patch.b

    def cls_dy(s):
        s["d"] = s["d"][:, 1:, :]                                       # keep the patch rows
    chain[2] = _Tiny(lambda s: s["d"][:, 0, :].sum(axis=0), cls_dy)     # cls
    chain[3] = _Tiny(lambda s: s["d"].sum(axis=0), identity)            # pos

    # --- blocks --------------------------------------------------------------
    for l in range(L):
        blk = blocks[l]
        g1, b1, Wqkv, bqkv, Wo, bo, g2, b2, W1, c1, W2, c2 = W[4 + 12 * l: 16 + 12 * l]
        base = 4 + 12 * l

        def ln_gain_dw(xhat):
            return lambda s: rows(s["d"] * xhat).sum(axis=0)

        def ln_gain_dy(xhat, rstd, gain):
            def f(s):
                # LayerNorm input gradient, joined by the residual branch; the sum
                # is again split into branch + skip for the sub-block above
                s["d"] = s["skip"] + ln_backward_input(s["d"], xhat, rstd, gain)
                s["skip"] = s["d"]
            return f

        def matrix_dy(Wm):
            def f(s):
                s["d"] = s["d"] @ Wm
            return f

        def proj_dy(s, blk=blk, Wo=Wo):
            do = _heads(s["d"] @ Wo, B, T, H, dh)                       # through proj.W
            q, k, v, p = blk["q"], blk["k"], blk["v"], blk["p"]         # then the attention core
            dv = p.transpose(0, 1, 3, 2) @ do
            dp = do @ v.transpose(0, 1, 3, 2)
            ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
            dq = (ds @ k) * scale
            dk = (ds.transpose(0, 1, 3, 2) @ q) * scale
            s["d"] = np.concatenate([_unheads(t, B, T, H, dh) for t in (dq, dk, dv)], axis=-1)

        def fc2_dy(s, blk=blk, W2=W2):
            s["d"] = (s["d"] @ W2) * gelu_grad(blk["u"])               # through fc2.W, then GELU

        chain[base + 0] = _Tiny(ln_gain_dw(blk["xhat1"]), ln_gain_dy(blk["xhat1"], blk["rstd1"], g1))
        chain[base + 1] = _Tiny(bias(), identity)
        chain[base + 2] = _Tiny(matrix_dw(blk["a1"]), matrix_dy(Wqkv))
        chain[base + 3] = _Tiny(bias(), identity)
        chain[base + 4] = _Tiny(matrix_dw(blk["o"]), proj_dy)
        chain[base + 5] = _Tiny(bias(), identity)
        chain[base + 6] = _Tiny(ln_gain_dw(blk["xhat2"]), ln_gain_dy(blk["xhat2"], blk["rstd2"], g2))
        chain[base + 7] = _Tiny(bias(), identity)
        chain[base + 8] = _Tiny(matrix_dw(blk["a2"]), matrix_dy(W1))
        chain[base + 9] = _Tiny(bias(), identity)
        chain[base + 10] = _Tiny(matrix_dw(blk["ga"]), fc2_dy)
        chain[base + 11] = _Tiny(bias(), identity)

    # --- final LayerNorm (CLS rows) and head ----------------------------------
    gf, bf, Wh, bh = W[-4:]

    def lnf_dy(s):
        dcls = ln_backward_input(s["d"], c["xhatf"], c["rstdf"], gf)    # [B, D]
        d = np.zeros((B, T, D), dtype=_F)
        d[:, 0, :] = dcls                                               # only CLS rows reach the loss
        s["d"] = d
        s["skip"] = d
    chain[N - 4] = _Tiny(lambda s: (s["d"] * c["xhatf"]).sum(axis=0), lnf_dy)
    chain[N - 3] = _Tiny(lambda s: s["d"].sum(axis=0), identity)

    def head_dy(s):
        s["d"] = s["d"] @ Wh
    chain[N - 2] = _Tiny(lambda s: s["d"].T @ c["zc"], head_dy)
    chain[N - 1] = _Tiny(lambda s: s["d"].sum(axis=0), identity)

    grads, work = _run_chain(chain, mask, state)
    return dict(loss=loss, grads=grads, work=work, logits=c["logits"])


def forward(cfg, weights, x, y):
    if cfg.kind == "mobilenet":
        from . import mobilenet
        return mobilenet.mobilenet_forward(cfg, weights, x, y)
    if cfg.kind == "vgg":
        from . import vgg
        return vgg.vgg_forward(cfg, weights, x, y)
    if cfg.kind == "resnet":
        from . import resnet
        return resnet.resnet_forward(cfg, weights, x, y)
    return (mlp_forward if cfg.kind == "mlp" else vit_forward)(cfg, weights, x, y)


def step(cfg, weights, x, y, mask):
    if cfg.kind == "mobilenet":
        from . import mobilenet
        return mobilenet.mobilenet_step(cfg, weights, x, y, mask)
    if cfg.kind == "vgg":
        from . import vgg
        return vgg.vgg_step(cfg, weights, x, y, mask)
    if cfg.kind == "resnet":
        from . import resnet
        return resnet.resnet_step(cfg, weights, x, y, mask)
    return (mlp_step if cfg.kind == "mlp" else vit_step)(cfg, weights, x, y, mask)
