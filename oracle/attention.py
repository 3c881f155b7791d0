"""Oracle for the attention core of one layer, on its own (numpy float64).  TEST INFRASTRUCTURE ONLY.

The attention operations hold no weights (Section 5.4 lists them with the non-trainable layers); what they
compute is the textbook definition, written out per (batch, head):
    P = softmax(Q K^T / sqrt(d_h)) over the keys,   O = P V
and, for a gradient dO of the output,
    dV = P^T dO,   dP = dO V^T,   dS = P * (dP - rowsum(P * dP)),   dQ = dS K / sqrt(d_h),   dK = dS^T Q / sqrt(d_h).
The token matrix holds Q | K | V side by side, [B, T, 3 D] with D = heads * d_h, head h in columns h*d_h .. of each
third; outputs use the same layout.  Pinned in tests/test_oracle_attention.py (probabilities sum to one, uniform
attention for equal keys, central differences, agreement with the same operation inside the ViT oracle).
"""
import numpy as np

_F = np.float64


def _split(qkv, heads):
    qkv = np.asarray(qkv, dtype=_F)
    B, T, D3 = qkv.shape
    D = D3 // 3
    dh = D // heads
    return [qkv[..., i * D:(i + 1) * D].reshape(B, T, heads, dh).transpose(0, 2, 1, 3) for i in range(3)], (B, T, D, dh)


def _merge(a, B, T, D):
    return a.transpose(0, 2, 1, 3).reshape(B, T, D)


def attention_forward(qkv, heads):
    """(out [B, T, D], lse [B, heads, T], probabilities [B, heads, T, T])."""
    (q, k, v), (B, T, D, dh) = _split(qkv, heads)
    s = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(dh)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=-1, keepdims=True)
    p = e / z
    return _merge(p @ v, B, T, D), (m + np.log(z))[..., 0], p


def attention_backward(qkv, dout, heads):
    """Gradient w.r.t. the token matrix [B, T, 3 D] (dQ | dK | dV) for a gradient dout [B, T, D] of the output."""
    (q, k, v), (B, T, D, dh) = _split(qkv, heads)
    _, _, p = attention_forward(qkv, heads)
    do = np.asarray(dout, dtype=_F).reshape(B, T, heads, dh).transpose(0, 2, 1, 3)
    dv = p.transpose(0, 1, 3, 2) @ do
    dp = do @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = (ds @ k) / np.sqrt(dh)
    dk = (ds.transpose(0, 1, 3, 2) @ q) / np.sqrt(dh)
    return np.concatenate([_merge(t, B, T, D) for t in (dq, dk, dv)], axis=-1)
