"""float64 brute-force statements of the layer, used only to pin the oracle.

Written from the mathematics in a different form than the oracle's loops: dense score
matrices with an explicit -inf mask, complex-number rotations for RoPE, numpy matmul for the
projections, a dense per-request gather for the paged cache.
"""
import numpy as np


def rope_complex(x, pos, base):
    """x[M,H,hd]: treat (x[i], x[i+hd/2]) as the complex number x[i] + 1j*x[i+hd/2] and
    multiply by exp(1j*pos*base**(-2i/hd))."""
    x = np.asarray(x, dtype=np.float64)
    M, H, hd = x.shape
    half = hd // 2
    z = x[..., :half] + 1j * x[..., half:]
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    rot = np.exp(1j * np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :])
    z = z * rot[:, None, :]
    return np.concatenate([z.real, z.imag], axis=-1)


def rmsnorm(x, g, eps):
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * np.asarray(g, np.float64)


def dense_causal_attention(q, k, v):
    """One request.  q[T,Hq,hd], k,v[T,Hkv,hd] -> [T,Hq,hd]; dense T x T scores, -inf above
    the diagonal, explicit softmax."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    T, Hq, hd = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    out = np.zeros_like(q)
    mask = np.triu(np.ones((T, T), dtype=bool), k=1)
    for h in range(Hq):
        s = q[:, h, :] @ k[:, h // G, :].T / np.sqrt(hd)
        s = np.where(mask, -np.inf, s)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, h // G, :]
    return out


def layer_dense(w, shape, x, cu_seqlens, prior_k=None, prior_v=None, stages=False):
    """Whole layer in float64 for a batch of independent requests, no paging at all.
    w: dict of float arrays [out,in].  Returns y[T,d], and rotated k, v [T,Hkv,hd]; with
    stages=True also a dict of the intermediates: h (first RMSNorm), qkv (rotated q, rotated k,
    v, concatenated as the projection lays them out), attn, x1 (after the attention residual),
    act (silu(gate) * up)."""
    d, Hq, Hkv, hd = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    x = np.asarray(x, np.float64)
    T = x.shape[0]
    pos = np.zeros(T, dtype=np.int64)
    for r in range(len(cu_seqlens) - 1):
        pos[cu_seqlens[r]:cu_seqlens[r + 1]] = np.arange(cu_seqlens[r + 1] - cu_seqlens[r])
    W = {k_: np.asarray(v_, np.float64) for k_, v_ in w.items()}
    h = rmsnorm(x, W["g1"], shape.rms_eps)
    qkv = h @ W["wqkv"].T
    q = qkv[:, :Hq * hd].reshape(T, Hq, hd)
    k = qkv[:, Hq * hd:(Hq + Hkv) * hd].reshape(T, Hkv, hd)
    v = qkv[:, (Hq + Hkv) * hd:].reshape(T, Hkv, hd)
    q = rope_complex(q, pos, shape.rope_base)
    k = rope_complex(k, pos, shape.rope_base)
    o = np.zeros((T, Hq, hd))
    for r in range(len(cu_seqlens) - 1):
        a, b = cu_seqlens[r], cu_seqlens[r + 1]
        o[a:b] = dense_causal_attention(q[a:b], k[a:b], v[a:b])
    x1 = x + o.reshape(T, Hq * hd) @ W["wo"].T
    h2 = rmsnorm(x1, W["g2"], shape.rms_eps)
    gate = h2 @ W["wg"].T
    up = h2 @ W["wu"].T
    act = gate / (1.0 + np.exp(-gate)) * up
    y = x1 + act @ W["wd"].T
    if stages:
        st = {"h": h, "qkv": np.concatenate([q.reshape(T, -1), k.reshape(T, -1), v.reshape(T, -1)], axis=1),
              "attn": o.reshape(T, Hq * hd), "x1": x1, "act": act}
        return y, k, v, st
    return y, k, v
