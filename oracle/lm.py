"""Token-level CPU oracle (TEST INFRASTRUCTURE ONLY): embedding, final norm + LM head, greedy
choice, and a whole-model driver over `OracleLayer`s with per-layer paged caches.

The paper's request life cycle (section 4.4) starts from a prompt and ends when generation
ends; it says nothing of how tokens become hidden states or logits become tokens, so these are
the textbook Llama definitions, written from the existing float32 primitives:

    x_t      = E[token_t]                              (row lookup, no scaling)
    logits   = RMSNorm(x_last; g_final) @ W_lm^T       (weights [vocab][d_model])
    next     = the smallest index among the maxima of logits   (greedy sampling)

A prompt's first generated token comes from the last prompt row after the prefill pass; every
later token from a decode step that feeds the previous token back in (section 2.1).
Nothing here is imported by the product.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

from . import OracleLayer, linear, rmsnorm, widen


def embed(tokens: Sequence[int], table_bf16: np.ndarray) -> np.ndarray:
    """Rows of the embedding table, widened to float32: out[i] = E[tokens[i]]."""
    t = np.asarray(tokens, dtype=np.int64)
    if t.size and (t.min() < 0 or t.max() >= table_bf16.shape[0]):
        raise ValueError("token id outside the vocabulary")
    return widen(np.ascontiguousarray(table_bf16[t]))


def head_logits(x: np.ndarray, g_final_bf16: np.ndarray, w_lm_bf16: np.ndarray, eps: float) -> np.ndarray:
    """float32 logits [n, vocab] of hidden rows x [n, d]."""
    h = rmsnorm(np.ascontiguousarray(x, dtype=np.float32), widen(g_final_bf16), eps)
    return linear(h, widen(w_lm_bf16))


def greedy(logits: np.ndarray) -> np.ndarray:
    """Per row, the lowest index holding the row maximum (int32)."""
    logits = np.asarray(logits)
    out = np.empty(logits.shape[0], dtype=np.int32)
    for r in range(logits.shape[0]):
        best, arg = logits[r, 0], 0
        for j in range(1, logits.shape[1]):
            if logits[r, j] > best:
                best, arg = logits[r, j], j
        out[r] = arg
    return out


class OracleModel:
    """A stack of decoder layers between an embedding and an LM head, one paged cache per layer."""

    def __init__(self, shape, layer_weights_bf16: List[Dict[str, np.ndarray]], head_bf16: Dict[str, np.ndarray],
                 n_blocks: int):
        self.shape = shape
        self.layers = [OracleLayer.from_shape(shape, w) for w in layer_weights_bf16]
        self.head = head_bf16
        self.caches = [l.new_cache(n_blocks) for l in self.layers]

    def prefill(self, tokens: Sequence[int], table_row: np.ndarray) -> np.ndarray:
        """Whole prompt of one request at positions 0..n-1; returns the logits of its last row."""
        n = len(tokens)
        x = embed(tokens, self.head["embed"])
        tab = np.asarray(table_row, dtype=np.int32).reshape(1, -1)
        for l, (Kc, Vc) in zip(self.layers, self.caches):
            x = l.prefill(x, [0, n], tab, Kc, Vc)
        return head_logits(x[n - 1:n], self.head["final_norm"], self.head["lm_head"], self.shape.rms_eps)[0]

    def decode(self, tokens: Sequence[int], ctx_lens: Sequence[int], tables: np.ndarray) -> np.ndarray:
        """One step: request i feeds tokens[i] at position ctx_lens[i]; returns logits [B, vocab]."""
        x = embed(tokens, self.head["embed"])
        for l, (Kc, Vc) in zip(self.layers, self.caches):
            x = l.decode(x, ctx_lens, tables, Kc, Vc)
        return head_logits(x, self.head["final_norm"], self.head["lm_head"], self.shape.rms_eps)

    def generate(self, prompt: Sequence[int], table_row: np.ndarray, max_new: int, eos: int = -1):
        """Free-running greedy generation of one request.  Returns (tokens, logits per token)."""
        out, lg = [], []
        logits = self.prefill(prompt, table_row)
        n = len(prompt)
        while True:
            tok = int(greedy(logits[None, :])[0])
            out.append(tok)
            lg.append(logits)
            if tok == eos or len(out) >= max_new:
                return out, lg
            logits = self.decode([tok], [n + len(out) - 1], np.asarray(table_row, np.int32).reshape(1, -1))[0]
