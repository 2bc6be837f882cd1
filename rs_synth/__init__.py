"""Seeded synthetic inputs for the prefill/decode decoder-layer path.

This module only DRAWS inputs (weights, hidden states, context lengths, block
tables, request streams) from fixed seeds and rounds them to bf16 bit patterns.
It holds none of the layer's arithmetic: both the CPU oracle and the HIP
library are handed the very same bits produced here, and neither of them is
imported from here.

Random numbers come from numpy's Philox generator (counter based, keyed by the
seed), so a given (seed, shape) always yields the same bits on every machine.

Seed plan (one stream per kind of input):
  0 weights, 1 hidden states, 2 context lengths, 3 block-table shuffles,
  4 request arrivals and lengths, 5 directly written KV-cache contents.

The shapes stand in for the workloads of the paper's evaluation section
(chat-like prompts of about 2K tokens, article-like prompts of 8K-20K tokens on
Llama-3-shaped models); no item of any dataset is reproduced.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Sequence, Tuple

import numpy as np

SEED_WEIGHTS = 0
SEED_HIDDEN = 1
SEED_CTX = 2
SEED_TABLES = 3
SEED_ARRIVALS = 4
SEED_CACHE = 5

KV_BLOCK = 16


@dataclasses.dataclass(frozen=True)
class LayerShape:
    """Dimensions of one Llama-style decoder layer."""
    name: str
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    n_layers: int = 1

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_dim(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def params_per_layer(self) -> int:
        d, f = self.d_model, self.ffn_dim
        return d * self.qkv_dim + self.q_dim * d + 3 * d * f


TINY = LayerShape("tiny", 256, 4, 4, 64, 688, 1e-5, 10000.0)
LLAMA8B = LayerShape("llama3-8b-layer", 4096, 32, 8, 128, 14336, 1e-5, 500000.0, 32)
LLAMA70B = LayerShape("llama3-70b-layer", 8192, 64, 8, 128, 28672, 1e-5, 500000.0, 80)
# A mid-size GQA shape for parity tests: several tiles, ragged tails, seconds on the CPU.
MID = LayerShape("mid-gqa", 512, 8, 2, 128, 1376, 1e-5, 500000.0)

# A wider GQA shape whose GEMMs all take the large-tile path (K multiples of 64, N >= 1024).
WIDE = LayerShape("wide-gqa", 1024, 8, 2, 128, 2816, 1e-5, 500000.0)

# Widths that are multiples of 32 but of no tile width: the large-tile GEMMs end in partly (and wholly) empty
# column tiles for every projection (1152 = 4.5 x 256, 1920 = 7.5 x 256, 3104 = 24.25 x 128).
ODD = LayerShape("odd-widths", 1152, 9, 3, 128, 3104, 1e-5, 500000.0)

SHAPES = {s.name: s for s in (TINY, LLAMA8B, LLAMA70B, MID, WIDE, ODD)}


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(shape: Sequence[int], seed: int, stream: int = 0, mean: float = 0.0,
                std: float = 1.0) -> np.ndarray:
    """N(mean, std) samples rounded once to bf16; returned as uint16 bit patterns."""
    g = _rng(seed, stream)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    chunk = 1 << 24
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        v = g.standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        out[lo:hi] = f32_to_bf16_bits(v)
    return out.reshape(tuple(shape))


def layer_weights(shape: LayerShape, layer: int = 0, seed: int = SEED_WEIGHTS,
                  std: float = 0.02, wo_std: float | None = None,
                  wd_std: float | None = None) -> Dict[str, np.ndarray]:
    """bf16 bit patterns of one layer's weights.

    Projection matrices are stored [out_features, in_features] (row = one output
    feature) and drawn N(0, std), std = 0.02 for the workloads.  wo_std / wd_std (default std)
    apply to the two matrices that project back onto the residual stream: a larger value makes
    that branch dominate the residual input, which some parity cases want.
    The two RMSNorm gains are drawn 1 + N(0, 0.02) so that a dropped or misplaced gain
    multiply is visible.
    """
    d, f = shape.d_model, shape.ffn_dim
    base = layer * 16
    wo_std = std if wo_std is None else wo_std
    wd_std = std if wd_std is None else wd_std
    return {
        "g1": normal_bf16((d,), seed, base + 0, 1.0, 0.02),
        "wqkv": normal_bf16((shape.qkv_dim, d), seed, base + 1, 0.0, std),
        "wo": normal_bf16((d, shape.q_dim), seed, base + 2, 0.0, wo_std),
        "g2": normal_bf16((d,), seed, base + 3, 1.0, 0.02),
        "wg": normal_bf16((f, d), seed, base + 4, 0.0, std),
        "wu": normal_bf16((f, d), seed, base + 5, 0.0, std),
        "wd": normal_bf16((d, f), seed, base + 6, 0.0, wd_std),
    }


def moe_weights(shape: LayerShape, n_experts: int, layer: int = 0, seed: int = SEED_WEIGHTS, std: float = 0.02,
                router_std: float = 0.1) -> Dict[str, np.ndarray]:
    """bf16 bit patterns of a sparse feed-forward block: router [E, d] ~ N(0, router_std) (wide enough that
    most tokens have a clear top two), per-expert wg / wu [E, F, d] and wd [E, d, F] ~ N(0, std)."""
    d, f = shape.d_model, shape.ffn_dim
    base = 8192 + layer * 16
    return {
        "router": normal_bf16((n_experts, d), seed, base + 0, 0.0, router_std),
        "wg": normal_bf16((n_experts, f, d), seed, base + 1, 0.0, std),
        "wu": normal_bf16((n_experts, f, d), seed, base + 2, 0.0, std),
        "wd": normal_bf16((n_experts, d, f), seed, base + 3, 0.0, std),
    }


def head_weights(d_model: int, vocab: int, seed: int = SEED_WEIGHTS, stream: int = 4096) -> Dict[str, np.ndarray]:
    """bf16 bit patterns of the token embedding [vocab, d_model] ~ N(0, 1) (the scale of the hidden
    states the layer workloads use), the final RMSNorm gain 1 + N(0, 0.02) and the LM head
    [vocab, d_model] ~ N(0, 0.02)."""
    return {
        "embed": normal_bf16((vocab, d_model), seed, stream + 0, 0.0, 1.0),
        "final_norm": normal_bf16((d_model,), seed, stream + 1, 1.0, 0.02),
        "lm_head": normal_bf16((vocab, d_model), seed, stream + 2, 0.0, 0.02),
    }


def prompt_tokens(n: int, vocab: int, stream: int = 0, seed: int = SEED_HIDDEN) -> np.ndarray:
    """n token ids uniform over the vocabulary (int32)."""
    return _rng(seed, 1 << 20 | stream).integers(0, vocab, size=n, dtype=np.int32)


def hidden_states(n_rows: int, d_model: int, stream: int = 0, seed: int = SEED_HIDDEN) -> np.ndarray:
    """N(0,1) hidden states [n_rows, d_model] as bf16 bit patterns."""
    return normal_bf16((n_rows, d_model), seed, stream, 0.0, 1.0)


def blocks_for(n_tokens: int, block: int = KV_BLOCK) -> int:
    return (int(n_tokens) + block - 1) // block


def shuffled_block_tables(token_counts: Sequence[int], n_blocks: int, seed: int = SEED_TABLES,
                          stream: int = 0, block: int = KV_BLOCK,
                          max_blk: int | None = None) -> np.ndarray:
    """Block tables [n_req, max_blk] (int32, unused entries -1).

    Physical block ids are a seeded random permutation of range(n_blocks); request
    i takes the next ceil(token_counts[i]/block) ids of that permutation, so ids are
    distinct across requests and scattered over the pool.
    """
    need = [blocks_for(t, block) for t in token_counts]
    total = sum(need)
    if total > n_blocks:
        raise ValueError(f"pool of {n_blocks} blocks too small for {total}")
    perm = _rng(seed, stream).permutation(n_blocks).astype(np.int32)
    width = max(need) if need else 0
    if max_blk is not None:
        if max_blk < width:
            raise ValueError("max_blk too small")
        width = max_blk
    tab = np.full((len(need), max(width, 1)), -1, dtype=np.int32)
    at = 0
    for i, n in enumerate(need):
        tab[i, :n] = perm[at:at + n]
        at += n
    return tab


def identity_block_tables(token_counts: Sequence[int], block: int = KV_BLOCK,
                          max_blk: int | None = None) -> np.ndarray:
    """Same as shuffled_block_tables but with consecutive physical ids 0,1,2,..."""
    need = [blocks_for(t, block) for t in token_counts]
    width = max(need) if need else 0
    if max_blk is not None:
        width = max(width, max_blk)
    tab = np.full((len(need), max(width, 1)), -1, dtype=np.int32)
    at = 0
    for i, n in enumerate(need):
        tab[i, :n] = np.arange(at, at + n, dtype=np.int32)
        at += n
    return tab


def uniform_context_lengths(batch: int, lo: int, hi: int, seed: int = SEED_CTX,
                            stream: int = 0) -> np.ndarray:
    """Decode context lengths (tokens already cached), uniform on [lo, hi] inclusive."""
    return _rng(seed, stream).integers(lo, hi + 1, size=batch, dtype=np.int64).astype(np.int32)


def kv_cache_bits(n_blocks: int, n_kv_heads: int, head_dim: int, block: int = KV_BLOCK,
                  seed: int = SEED_CACHE, stream: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Directly written cache contents: K and V pools [n_blocks, block, n_kv_heads, head_dim],
    N(0,1) bf16 bits (used where prefilling >100k tokens just to fill the cache is pointless)."""
    shp = (n_blocks, block, n_kv_heads, head_dim)
    return normal_bf16(shp, seed, 2 * stream), normal_bf16(shp, seed, 2 * stream + 1)


def _lognormal_params(mean: float, sd: float) -> Tuple[float, float]:
    sigma2 = math.log(1.0 + (sd / mean) ** 2)
    return math.log(mean) - 0.5 * sigma2, math.sqrt(sigma2)


@dataclasses.dataclass(frozen=True)
class Request:
    req_id: int
    arrival_s: float
    prompt_len: int
    output_len: int


def request_stream(n_requests: int, rate_per_s: float = 4.0, prompt_mean: float = 1024.0,
                   prompt_sd: float = 512.0, prompt_clip: Tuple[int, int] = (32, 8192),
                   output_mean: float = 256.0, output_sd: float = 128.0,
                   output_clip: Tuple[int, int] = (16, 2048),
                   seed: int = SEED_ARRIVALS) -> List[Request]:
    """Poisson arrivals with lognormal prompt and output lengths (clipped), pre-drawn."""
    g = _rng(seed, 0)
    gaps = g.exponential(1.0 / rate_per_s, size=n_requests)
    t = np.cumsum(gaps)
    mu_p, s_p = _lognormal_params(prompt_mean, prompt_sd)
    mu_o, s_o = _lognormal_params(output_mean, output_sd)
    p = np.clip(np.rint(g.lognormal(mu_p, s_p, size=n_requests)), *prompt_clip).astype(int)
    o = np.clip(np.rint(g.lognormal(mu_o, s_o, size=n_requests)), *output_clip).astype(int)
    return [Request(i, float(t[i]), int(p[i]), int(o[i])) for i in range(n_requests)]


def tiny_config() -> dict:
    """The small co-run case: 1 prefill request of 128 tokens; decode batch 4 with
    contexts {64,128,192,256}; 16-token blocks; shuffled tables; 50/50 CU split."""
    ctx = np.array([64, 128, 192, 256], dtype=np.int32)
    prefill_T = 128
    counts = [int(c) + 1 for c in ctx] + [prefill_T]
    n_blocks = sum(blocks_for(c) for c in counts) + 8
    tabs = shuffled_block_tables(counts, n_blocks, SEED_TABLES, 0)
    return {
        "shape": TINY, "prefill_T": prefill_T, "ctx": ctx, "n_blocks": n_blocks,
        "decode_tables": tabs[:4].copy(), "prefill_tables": tabs[4:5].copy(),
        "split": (128, 128),
    }
