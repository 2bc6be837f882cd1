"""Pins for the mixture-of-experts oracle: special cases with closed forms and invariants."""
import numpy as np
import pytest

import oracle
from oracle import moe
import rs_synth as S

RNG = np.random.default_rng(2024)
SMALL = S.LayerShape("pin-small", 64, 4, 2, 16, 96, 1e-5, 10000.0)


def _bits(x):
    return S.f32_to_bf16_bits(np.asarray(x, np.float32))


def test_top2_picks_the_two_largest_with_softmax_weights():
    lg = np.array([[0.0, 3.0, 1.0, 2.0], [5.0, 5.0, 5.0, 5.0], [-1.0, -4.0, -1.0, -9.0], [2.0, 2.0, 7.0, 2.0]], np.float32)
    sel, wt = moe.top2(lg)
    assert sel.tolist() == [[1, 3], [0, 1], [0, 2], [2, 0]]          # ties: lower index first
    assert np.allclose(wt.sum(axis=1), 1.0, atol=1e-7)
    e = np.exp(np.array([3.0, 2.0], np.float64))
    assert np.allclose(wt[0], e / e.sum(), atol=1e-7)
    assert np.allclose(wt[1], [0.5, 0.5]) and np.allclose(wt[2], [0.5, 0.5])
    # against a library routine: argsort of random logits
    lg = RNG.standard_normal((200, 8)).astype(np.float32)
    sel, wt = moe.top2(lg)
    order = np.argsort(-lg, axis=1, kind="stable")[:, :2]
    assert np.array_equal(sel, order.astype(np.int32))
    full = np.exp(lg.astype(np.float64))
    full /= full.sum(axis=1, keepdims=True)                          # softmax over all, top two renormalised
    top = np.take_along_axis(full, order, axis=1)
    assert np.allclose(wt, top / top.sum(axis=1, keepdims=True), atol=1e-6)


def test_identical_experts_reduce_to_the_dense_block():
    # every expert the same matrices: whatever the routing, out = FFN(h) since the weights sum to 1
    E, d, F = 4, 32, 48
    wg, wu, wd = (S.normal_bf16(s, 3, i, 0.0, 0.2) for i, s in enumerate([(F, d), (F, d), (d, F)]))
    w = {"router": S.normal_bf16((E, d), 3, 9, 0.0, 1.0), "wg": np.stack([wg] * E), "wu": np.stack([wu] * E), "wd": np.stack([wd] * E)}
    h = RNG.standard_normal((7, d)).astype(np.float32)
    out, sel, wt = moe.moe_ffn(h, w)
    dense = moe.expert_ffn(h, wg, wu, wd)
    assert np.abs(out - dense).max() < 1e-5 * np.abs(dense).max()
    assert all(a != b for a, b in sel.tolist())


def test_routing_follows_a_planted_router_and_only_selected_experts_matter():
    # router row e is the indicator of feature e: a token whose features 5 and 2 are largest goes to experts 5 and 2
    E, d, F = 6, 16, 24
    router = np.zeros((E, d), np.float32)
    router[np.arange(E), np.arange(E)] = 1.0
    w = S.moe_weights(S.LayerShape("m", d, 2, 2, 8, F), E, seed=5, std=0.3)
    w["router"] = _bits(router)
    h = np.zeros((3, d), np.float32)
    h[0, 5], h[0, 2] = 4.0, 3.0
    h[1, 0], h[1, 1] = 1.0, 1.0                      # tie between experts 0 and 1
    h[2, 3], h[2, 4] = -1.0, 2.0                     # largest two of [0,0,0,-1,2,0]: expert 4, then the first zero
    out, sel, wt = moe.moe_ffn(h, w)
    assert sel.tolist() == [[5, 2], [0, 1], [4, 0]]
    assert np.allclose(wt[0], [1 / (1 + np.exp(-1.0)), 1 - 1 / (1 + np.exp(-1.0))], atol=1e-6)
    # changing an expert nobody selected changes nothing; zeroing a selected expert's down projection removes its term
    w2 = {k: v.copy() for k, v in w.items()}
    w2["wd"][1 if 1 not in sel[0] else 3] ^= np.uint16(0x8000)
    w2["wd"][3] = S.normal_bf16((d, F), 77, 0)
    assert np.array_equal(moe.moe_ffn(h[:1], w2)[0], out[:1])
    w3 = {k: v.copy() for k, v in w.items()}
    w3["wd"][2] = 0
    only5 = wt[0, 0] * moe.expert_ffn(h[:1], w["wg"][5], w["wu"][5], w["wd"][5])
    assert np.abs(moe.moe_ffn(h[:1], w3)[0] - only5).max() < 1e-6


def test_moe_layer_with_dead_experts_is_the_attention_half():
    shape = SMALL
    wb = S.layer_weights(shape, 0, 11, std=0.08)
    mw = S.moe_weights(shape, 4, seed=11, std=0.1)
    mw["wd"][:] = 0
    L = moe.OracleMoELayer(shape, wb, mw)
    dense = oracle.OracleLayer.from_shape(shape, {**wb, "wd": np.zeros_like(wb["wd"])})
    x = S.bf16_bits_to_f32(S.hidden_states(20, shape.d_model, 3))
    tab = np.array([[2, 0, 1]], np.int32)
    Kc, Vc = L.new_cache(4)
    Kd, Vd = dense.new_cache(4)
    y, x1, sel, wt = L.prefill(x, [0, 20], tab, Kc, Vc)
    yd = dense.prefill(x, [0, 20], tab, Kd, Vd)
    assert np.array_equal(y, yd) and np.array_equal(y, x1) and np.array_equal(Kc, Kd)
    # a decode step after it equals the dense layer's too
    xs = S.bf16_bits_to_f32(S.hidden_states(1, shape.d_model, 4))
    assert np.array_equal(L.decode(xs, [20], tab, Kc, Vc)[0], dense.decode(xs, [20], tab, Kd, Vd))


def test_moe_layer_output_is_x1_plus_weighted_experts_bruteforce():
    shape = SMALL
    wb = S.layer_weights(shape, 0, 12, std=0.08)
    mw = S.moe_weights(shape, 4, seed=12, std=0.1)
    L = moe.OracleMoELayer(shape, wb, mw)
    x = S.bf16_bits_to_f32(S.hidden_states(9, shape.d_model, 5))
    tab = np.array([[1, 0]], np.int32)
    Kc, Vc = L.new_cache(3)
    y, x1, sel, wt = L.prefill(x, [0, 9], tab, Kc, Vc)
    g2 = S.bf16_bits_to_f32(wb["g2"]).astype(np.float64)
    W = {k: S.bf16_bits_to_f32(v).astype(np.float64) for k, v in mw.items()}
    for i in range(9):
        v = x1[i].astype(np.float64)
        h = v / np.sqrt((v * v).mean() + shape.rms_eps) * g2
        r = W["router"] @ h
        a, b = np.argsort(-r, kind="stable")[:2]
        assert [a, b] == sel[i].tolist()
        p = np.exp(r[[a, b]] - r[a]); p /= p.sum()
        ref = v.copy()
        for e, pw in zip((a, b), p):
            g, u = W["wg"][e] @ h, W["wu"][e] @ h
            ref += pw * (W["wd"][e] @ (g / (1 + np.exp(-g)) * u))
        assert np.abs(y[i] - ref).max() < 2e-5 * max(1.0, np.abs(ref).max())
