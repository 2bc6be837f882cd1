"""Mixture-of-experts feed-forward block, CPU oracle (TEST INFRASTRUCTURE ONLY).

The paper evaluates a mixture-of-experts model (Mixtral 8x7B, section 5) next to the dense one
and says nothing of the block itself, so this is the textbook sparse block of that family written
from the float32 primitives of the layer oracle:

    r        = h W_r^T                                  router logits, [tokens, E]
    (e0, e1) = the two largest logits of the token      ties: the lower expert index first
    (w0, w1) = softmax over those two logits            (softmax over all experts, then the top two
                                                         renormalised, is the same thing)
    out      = w0 * FFN_e0(h) + w1 * FFN_e1(h)          FFN_e(h) = (silu(h Wg_e^T) * (h Wu_e^T)) Wd_e^T

h is the RMS-normalised residual stream (second norm of the layer) and the layer output is
x1 + out.  Arithmetic is float32 throughout; nothing is blocked or reordered: each token's two
experts are evaluated and added in selection order.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from . import OracleLayer, linear, rmsnorm, silu_mul, widen


def router_logits(h: np.ndarray, wr_bf16: np.ndarray) -> np.ndarray:
    return linear(np.ascontiguousarray(h, dtype=np.float32), widen(wr_bf16))


def top2(logits: np.ndarray):
    """(experts [n, 2] int32, weights [n, 2] float32)."""
    lg = np.asarray(logits, dtype=np.float32)
    n, E = lg.shape
    sel = np.empty((n, 2), dtype=np.int32)
    wt = np.empty((n, 2), dtype=np.float32)
    for i in range(n):
        a = 0
        for e in range(1, E):
            if lg[i, e] > lg[i, a]:
                a = e
        b = -1
        for e in range(E):
            if e != a and (b < 0 or lg[i, e] > lg[i, b]):
                b = e
        sel[i] = (a, b)
        eb = np.exp(np.float32(lg[i, b] - lg[i, a]), dtype=np.float32)      # exp(l1 - l0) <= 1
        wt[i, 0] = np.float32(1.0) / (np.float32(1.0) + eb)
        wt[i, 1] = eb / (np.float32(1.0) + eb)
    return sel, wt


def expert_ffn(h: np.ndarray, wg_bf16, wu_bf16, wd_bf16) -> np.ndarray:
    act = silu_mul(linear(h, widen(wg_bf16)), linear(h, widen(wu_bf16)))
    return linear(act, widen(wd_bf16))


def moe_ffn(h: np.ndarray, w: Dict[str, np.ndarray], sel: Optional[np.ndarray] = None, wt: Optional[np.ndarray] = None):
    """out [n, d] for normalised rows h [n, d].  w: router [E, d], wg/wu [E, F, d], wd [E, d, F] (bf16 bits).
    sel / wt override the routing (for checking a path that routed a near-tie differently)."""
    h = np.ascontiguousarray(h, dtype=np.float32)
    if sel is None:
        sel, wt = top2(router_logits(h, w["router"]))
    n, d = h.shape
    E = w["router"].shape[0]
    per = {}
    for e in range(E):
        rows = np.nonzero((sel == e).any(axis=1))[0]
        if len(rows):
            per[e] = dict(zip(rows.tolist(), expert_ffn(h[rows], w["wg"][e], w["wu"][e], w["wd"][e])))
    out = np.zeros((n, d), dtype=np.float32)
    for i in range(n):
        out[i] = wt[i, 0] * per[int(sel[i, 0])][i] + wt[i, 1] * per[int(sel[i, 1])][i]
    return out, sel, wt


class OracleMoELayer:
    """A decoder layer whose feed-forward block is the sparse one: the attention half is the dense
    layer oracle's (its own feed-forward branch silenced by a zero down projection)."""

    def __init__(self, shape, weights_bf16: Dict[str, np.ndarray], moe_bf16: Dict[str, np.ndarray]):
        w = dict(weights_bf16)
        f_stub = 8   # the dense branch contributes nothing: a tiny stub keeps the C layer's signature
        w["wg"] = np.zeros((f_stub, shape.d_model), np.uint16)
        w["wu"] = np.zeros((f_stub, shape.d_model), np.uint16)
        w["wd"] = np.zeros((shape.d_model, f_stub), np.uint16)
        self.shape = shape
        self.attn = OracleLayer(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, f_stub, shape.rms_eps,
                                shape.rope_base, w)
        self.g2 = widen(weights_bf16["g2"])
        self.moe = moe_bf16

    def new_cache(self, n_blocks: int, fill: float = 0.0):
        return self.attn.new_cache(n_blocks, fill)

    def _ffn(self, x1, sel, wt):
        h2 = rmsnorm(x1, self.g2, self.shape.rms_eps)
        out, sel, wt = moe_ffn(h2, self.moe, sel, wt)
        return x1 + out, h2, sel, wt

    def prefill(self, x, cu_seqlens, tables, Kc, Vc, sel=None, wt=None):
        """Returns (y, x1, selected experts, routing weights) for all rows."""
        x1 = self.attn.prefill(x, cu_seqlens, tables, Kc, Vc)      # zero down projection: y of the dense layer is x1
        y, _, sel, wt = self._ffn(x1, sel, wt)
        return y, x1, sel, wt

    def decode(self, x, ctx_lens, tables, Kc, Vc, sel=None, wt=None):
        x1 = self.attn.decode(x, ctx_lens, tables, Kc, Vc)
        y, _, sel, wt = self._ffn(x1, sel, wt)
        return y, x1, sel, wt
