"""Independent numpy references used to pin the oracle (dense matrices, library matmul, python sort)."""
import numpy as np

from synth import LayerConfig, make_layer, make_x, make_logits


def tiny_cfg(cfg_id=101, **kw):
    base = dict(name="t", E=4, S=0, k=2, H=8, F=16, T=5, g=4, r=2, bits=4)
    base.update(kw)
    return LayerConfig(cfg_id, **base)


def f16(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def dense_weight(layer, e, p):
    """[K, N] float64: transpose of the dequantised matrix plus A @ B, formed explicitly."""
    c = layer.cfg
    q = layer.codes_matrix(e, p).astype(np.float64)
    s = layer.scale_matrix(e, p).astype(np.float64)
    z = layer.zero_matrix(e, p).astype(np.float64)
    W = (q - np.repeat(z, c.g, axis=1)) * np.repeat(s, c.g, axis=1)     # [N, K]
    Weff = W.T.copy()
    if c.r > 0:
        Weff += layer.a_matrix(e, p).astype(np.float64) @ layer.b_matrix(e, p).astype(np.float64)
    return Weff


def dense_expert_all_tokens(layer, e, x64):
    G = x64 @ dense_weight(layer, e, 0)
    U = x64 @ dense_weight(layer, e, 1)
    h = G / (1.0 + np.exp(-G)) * U
    return h @ dense_weight(layer, e, 2)


def exhaustive_topk(logits, bias, k):
    """python sort on (-score, index); weights = softmax over ALL experts, renormalised over the chosen."""
    T, E = logits.shape
    idx = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    for t in range(T):
        l = logits[t].astype(np.float32)
        if bias is not None:
            l = (l + bias.astype(np.float32)).astype(np.float32)
        order = sorted(range(E), key=lambda e: (-float(l[e]), e))[:k]
        p = np.exp(l.astype(np.float64) - float(l.max()))
        p /= p.sum()
        sel = p[order]
        idx[t] = order
        w[t] = sel / sel.sum()
    return idx, w


def dense_moe(layer, x, idx, w):
    """Run EVERY expert densely on every token, then mask by the routing table."""
    c = layer.cfg
    x64 = x.astype(np.float64)
    y = np.zeros((x.shape[0], c.H))
    for e in range(c.E):
        Y = dense_expert_all_tokens(layer, e, x64)
        for j in range(c.k):
            m = (idx[:, j] == e)
            y[m] += w[m, j][:, None].astype(np.float64) * Y[m]
    for s in range(c.S):
        y += dense_expert_all_tokens(layer, c.E + s, x64)
    return y


def rel_err(a, b):
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))
