"""Pins for the token-level oracle (embedding, final norm + LM head, greedy choice, generation loop):
special cases with closed forms, invariants and library routines, none of which call the function
under test to make the expected value."""
import math

import numpy as np
import pytest

import oracle
from oracle import lm
import rs_synth as S

RNG = np.random.default_rng(77)
SMALL = S.LayerShape("pin-small", 64, 4, 2, 16, 96, 1e-5, 10000.0)


def _bits(x):
    return S.f32_to_bf16_bits(np.asarray(x, np.float32))


def test_embed_is_a_one_hot_product():
    vocab, d = 37, 24
    E = S.normal_bf16((vocab, d), 9, 0)
    toks = RNG.integers(0, vocab, size=50)
    onehot = np.zeros((50, vocab))
    onehot[np.arange(50), toks] = 1.0
    want = onehot @ S.bf16_bits_to_f32(E).astype(np.float64)
    assert np.array_equal(lm.embed(toks, E).astype(np.float64), want)
    with pytest.raises(ValueError):
        lm.embed([vocab], E)
    with pytest.raises(ValueError):
        lm.embed([-1], E)


def test_head_constant_row_indicator_weights():
    # W row v is the indicator of feature j(v): logit v = g[j(v)] * c / sqrt(c^2 + eps).
    d, vocab, c, eps = 32, 11, 2.5, 1e-5
    g = _bits(1.0 + 0.1 * RNG.standard_normal(d))
    j = (np.arange(vocab) * 5 + 3) % d
    W = np.zeros((vocab, d), np.float32)
    W[np.arange(vocab), j] = 1.0
    got = lm.head_logits(np.full((2, d), c, np.float32), g, _bits(W), eps)
    want = S.bf16_bits_to_f32(g).astype(np.float64)[j] * c / math.sqrt(c * c + eps)
    assert got.shape == (2, vocab)
    assert np.abs(got[0] - want).max() < 1e-6 and np.array_equal(got[0], got[1])


def test_head_is_scale_invariant_and_linear_in_the_weights():
    d, vocab = 48, 19
    x = RNG.standard_normal((3, d)).astype(np.float32) * 4
    g = _bits(1.0 + 0.05 * RNG.standard_normal(d))
    W = S.normal_bf16((vocab, d), 5, 1, 0.0, 0.5)
    a = lm.head_logits(x, g, W, 1e-5)
    b = lm.head_logits(x * 8.0, g, W, 1e-5)
    assert np.abs(a - b).max() < 1e-4 * np.abs(a).max()
    # negated weights negate the logits exactly; a permutation of vocabulary rows permutes them
    Wn = (W ^ np.uint16(0x8000)).astype(np.uint16)
    assert np.array_equal(lm.head_logits(x, g, Wn, 1e-5), -a)
    perm = RNG.permutation(vocab)
    assert np.array_equal(lm.head_logits(x, g, np.ascontiguousarray(W[perm]), 1e-5), a[:, perm])


def test_round_trip_through_orthogonal_tied_tables_returns_the_token():
    # E[t] = 4 e_pi(t), W = E / 4, unit gain: the logits of embed(t) peak at t, for every t
    n = 40
    pi = RNG.permutation(n)
    E = np.zeros((n, n), np.float32)
    E[np.arange(n), pi] = 4.0
    head = {"embed": _bits(E), "final_norm": _bits(np.ones(n)), "lm_head": _bits(E / 4)}
    toks = np.arange(n)
    logits = lm.head_logits(lm.embed(toks, head["embed"]), head["final_norm"], head["lm_head"], 1e-5)
    assert np.array_equal(lm.greedy(logits), toks.astype(np.int32))
    peak = 4.0 / math.sqrt(16.0 / n + 1e-5)
    assert np.abs(logits[toks, toks] - peak).max() < 1e-5
    off = logits.copy()
    off[toks, toks] = 0
    assert np.all(off == 0)


def test_greedy_lowest_index_among_maxima():
    assert lm.greedy(np.zeros((2, 9), np.float32)).tolist() == [0, 0]
    row = np.array([[-3.0, 5.0, 1.0, 5.0, -7.0], [-3.0, -5.0, -1.0, -1.0, -7.0]], np.float32)
    assert lm.greedy(row).tolist() == [1, 2]
    x = RNG.standard_normal((20, 301)).astype(np.float32)
    x[7, 300] = 99.0
    x[8, 0] = 99.0
    got = lm.greedy(x)
    assert got.dtype == np.int32 and np.array_equal(got, np.argmax(x, axis=1)) and got[7] == 300 and got[8] == 0


def _model(n_layers=2, vocab=53, zero_branches=False, n_blocks=16):
    ws = []
    for l in range(n_layers):
        w = S.layer_weights(SMALL, l, 11, std=0.08)
        if zero_branches:
            w["wo"] = np.zeros_like(w["wo"])
            w["wd"] = np.zeros_like(w["wd"])
        ws.append(w)
    head = S.head_weights(SMALL.d_model, vocab, seed=11)
    head["lm_head"] = S.normal_bf16((vocab, SMALL.d_model), 11, 999, 0.0, 0.3)
    return lm.OracleModel(SMALL, ws, head, n_blocks), head


def test_model_with_dead_branches_is_head_of_embedding():
    m, head = _model(zero_branches=True)
    prompt = [5, 17, 3, 44, 9]
    tab = np.array([3, 7, 1, 0], np.int32)
    got = m.prefill(prompt, tab)
    want = lm.head_logits(lm.embed([9], head["embed"]), head["final_norm"], head["lm_head"], SMALL.rms_eps)[0]
    assert np.array_equal(got, want)
    step = m.decode([21], [5], tab[None, :])[0]
    want = lm.head_logits(lm.embed([21], head["embed"]), head["final_norm"], head["lm_head"], SMALL.rms_eps)[0]
    assert np.array_equal(step, want)


def test_generation_equals_prefill_of_the_extended_prompt():
    # the logits behind generated token k are those of the last row of a whole-prompt pass over
    # prompt + generated[:k]: pins the position / fed-token bookkeeping of the loop
    m, _ = _model()
    prompt = S.prompt_tokens(19, 53, 1).tolist()
    tab = np.array([9, 2, 5, 11], np.int32)
    toks, lgs = m.generate(prompt, tab, max_new=6)
    assert len(toks) == 6 and all(0 <= t < 53 for t in toks)
    for k in range(6):
        fresh, _ = _model()
        ref = fresh.prefill(prompt + toks[:k], tab)
        assert np.abs(ref - lgs[k]).max() < 2e-4 * max(1.0, np.abs(ref).max())
        assert int(np.argmax(ref)) == toks[k] or np.sort(ref)[-1] - np.sort(ref)[-2] < 1e-3


def test_generation_stops_at_the_first_eos():
    m, _ = _model()
    prompt = S.prompt_tokens(10, 53, 2).tolist()
    tab = np.array([1, 2, 3, 4], np.int32)
    free, _ = m.generate(prompt, tab, max_new=8)
    eos = free[3]
    m2, _ = _model()
    got, _ = m2.generate(prompt, tab, max_new=8, eos=eos)
    stop = free.index(eos)
    assert got == free[:stop + 1]
    m3, _ = _model()
    assert m3.generate(prompt, tab, max_new=1)[0] == free[:1]
