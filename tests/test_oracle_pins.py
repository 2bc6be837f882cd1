"""Pins for the CPU oracle: what mathematics and the paper fix, independent of the oracle.

Each test is chosen so that a plausible mistake in the oracle (dropped term, wrong sign or
index, transposed operand, off-by-one in the causal mask or the block arithmetic) fails it.
"""
import math

import numpy as np
import pytest

import oracle
import rs_synth as S
from tests import brute

RNG = np.random.default_rng(1234)


def _w32(shape, seed=0):
    wb = S.layer_weights(shape, 0, seed)
    return wb, {k: S.bf16_bits_to_f32(v) for k, v in wb.items()}


SMALL = S.LayerShape("pin-small", 64, 4, 2, 16, 96, 1e-5, 10000.0)


# ---------------------------------------------------------------- primitives
def test_widen_is_exact():
    bits = np.arange(0, 65536, dtype=np.uint16)
    keep = ~np.isnan(S.bf16_bits_to_f32(bits))
    assert np.array_equal(oracle.widen(bits)[keep].view(np.uint32),
                          (bits.astype(np.uint32) << 16)[keep])


def test_bf16_rounding_ties_to_even():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1.0 and 1+2^-7: goes to even (1.0);
    # 1 + 3*2^-8 is half-way between 1+2^-7 and 1+2^-6: goes to even mantissa (1+2^-6).
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], np.float32)
    got = S.bf16_bits_to_f32(S.f32_to_bf16_bits(x))
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]


def test_linear_vs_numpy_fp64_nonsquare():
    a = RNG.standard_normal((5, 37)).astype(np.float32)
    w = RNG.standard_normal((11, 37)).astype(np.float32)
    ref = a.astype(np.float64) @ w.astype(np.float64).T
    for fn in (oracle.linear, oracle.linear_t):
        got = fn(a, w)
        assert got.shape == (5, 11)
        assert np.abs(got - ref).max() < 2e-5


def test_rmsnorm_closed_form_constant_row():
    d, c, eps = 48, 3.0, 1e-5
    g = RNG.standard_normal(d).astype(np.float32)
    got = oracle.rmsnorm(np.full((2, d), c, np.float32), g, eps)
    want = g.astype(np.float64) * c / math.sqrt(c * c + eps)
    assert np.abs(got[0] - want).max() < 1e-6
    # eps sits inside the root: for a zero row the output is exactly zero, not NaN
    assert np.all(oracle.rmsnorm(np.zeros((1, d), np.float32), g, eps) == 0.0)
    # tiny rows: x/sqrt(x^2+eps) with x^2 << eps is x/sqrt(eps)
    tiny = oracle.rmsnorm(np.full((1, d), 1e-6, np.float32), np.ones(d, np.float32), eps)
    assert np.allclose(tiny, 1e-6 / math.sqrt(eps), rtol=1e-4)


def test_rmsnorm_scale_invariance_and_fp64():
    x = RNG.standard_normal((3, 64)).astype(np.float32)
    g = (1 + 0.1 * RNG.standard_normal(64)).astype(np.float32)
    a = oracle.rmsnorm(x, g, 1e-5)
    b = oracle.rmsnorm(8.0 * x, g, 1e-5)
    assert np.abs(a - b).max() < 1e-4
    assert np.abs(a - brute.rmsnorm(x, g, 1e-5)).max() < 1e-5


def test_silu_spot_values():
    z = np.array([0.0, 1.0, -1.0, 2.0, -20.0], np.float32)
    got = oracle.silu_mul(z, np.ones_like(z))
    want = [0.0, 0.7310585786300049, -0.2689414213699951, 1.7615941559557649, -20 / (1 + math.exp(20))]
    assert np.allclose(got, want, rtol=1e-6, atol=1e-12)
    # it multiplies by the second operand
    assert np.allclose(oracle.silu_mul(z, np.full_like(z, -3.0)), -3.0 * np.array(want), rtol=1e-6)


# ---------------------------------------------------------------- RoPE
def test_rope_position_zero_is_identity_and_norm_preserved():
    x = RNG.standard_normal((4, 3, 32)).astype(np.float32)
    assert np.array_equal(oracle.rope(x, np.zeros(4, np.int32), 10000.0), x)
    y = oracle.rope(x, np.array([1, 17, 300, 4095], np.int32), 10000.0)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-5)
    assert not np.allclose(y, x)


def test_rope_matches_complex_rotation():
    x = RNG.standard_normal((6, 2, 64)).astype(np.float32)
    pos = np.array([0, 1, 2, 100, 2047, 32767], np.int32)
    for base in (10000.0, 500000.0):
        got = oracle.rope(x, pos, base)
        assert np.abs(got - brute.rope_complex(x, pos, base)).max() < 2e-6


def test_rope_first_pair_rotates_by_position_radians():
    # i = 0 has theta = 1: the pair (1, 0) at position p becomes (cos p, sin p)
    hd = 8
    x = np.zeros((1, 1, hd), np.float32)
    x[0, 0, 0] = 1.0
    y = oracle.rope(x, np.array([2], np.int32), 10000.0)
    assert abs(y[0, 0, 0] - math.cos(2.0)) < 1e-7 and abs(y[0, 0, hd // 2] - math.sin(2.0)) < 1e-7
    # i = 1 has theta = base^(-2/hd)
    x[:] = 0; x[0, 0, 1] = 1.0
    y = oracle.rope(x, np.array([5], np.int32), 10000.0)
    phi = 5.0 * 10000.0 ** (-2.0 / hd)
    assert abs(y[0, 0, 1] - math.cos(phi)) < 1e-7 and abs(y[0, 0, 1 + hd // 2] - math.sin(phi)) < 1e-7


def test_rope_relative_position_property():
    # scores q.k after rotation depend on the position difference only
    T, H, hd = 9, 2, 32
    q = RNG.standard_normal((T, H, hd)).astype(np.float32)
    k = RNG.standard_normal((T, H, hd)).astype(np.float32)
    v = RNG.standard_normal((T, H, hd)).astype(np.float32)
    cu = [0, T]
    outs = []
    for shift in (0, 37):
        pos = np.arange(T, dtype=np.int32) + shift
        outs.append(oracle.attn_causal(oracle.rope(q, pos, 10000.0), oracle.rope(k, pos, 10000.0), v, cu))
    assert np.abs(outs[0] - outs[1]).max() < 2e-5


# ---------------------------------------------------------------- attention
def test_attention_single_key_returns_value():
    q = RNG.standard_normal((1, 4, 16)).astype(np.float32)
    k = RNG.standard_normal((1, 2, 16)).astype(np.float32)
    v = RNG.standard_normal((1, 2, 16)).astype(np.float32)
    o = oracle.attn_causal(q, k, v, [0, 1])
    assert np.array_equal(o[0, 0], v[0, 0]) and np.array_equal(o[0, 1], v[0, 0])
    assert np.array_equal(o[0, 2], v[0, 1]) and np.array_equal(o[0, 3], v[0, 1])


def test_attention_identical_keys_gives_running_mean_of_values():
    T = 7
    k = np.tile(RNG.standard_normal((1, 1, 16)).astype(np.float32), (T, 1, 1))
    q = RNG.standard_normal((T, 1, 16)).astype(np.float32)
    v = RNG.standard_normal((T, 1, 16)).astype(np.float32)
    o = oracle.attn_causal(q, k, v, [0, T])
    want = np.cumsum(v.astype(np.float64), axis=0) / np.arange(1, T + 1)[:, None, None]
    assert np.abs(o - want).max() < 1e-6


def test_attention_vs_dense_brute_force_gqa_and_two_requests():
    T1, T2, Hq, Hkv, hd = 19, 33, 6, 2, 16
    T = T1 + T2
    q = RNG.standard_normal((T, Hq, hd)).astype(np.float32)
    k = RNG.standard_normal((T, Hkv, hd)).astype(np.float32)
    v = RNG.standard_normal((T, Hkv, hd)).astype(np.float32)
    got = oracle.attn_causal(q, k, v, [0, T1, T])
    want = np.concatenate([brute.dense_causal_attention(q[:T1], k[:T1], v[:T1]),
                           brute.dense_causal_attention(q[T1:], k[T1:], v[T1:])])
    assert np.abs(got - want).max() < 2e-6
    # scale 1/sqrt(hd) matters: unscaled queries give a different answer
    assert np.abs(oracle.attn_causal(q * math.sqrt(hd), k, v, [0, T1, T]) - want).max() > 1e-3


def test_attention_rows_subset_equals_full():
    T, Hq, Hkv, hd = 40, 4, 2, 16
    q = RNG.standard_normal((T, Hq, hd)).astype(np.float32)
    k = RNG.standard_normal((T, Hkv, hd)).astype(np.float32)
    v = RNG.standard_normal((T, Hkv, hd)).astype(np.float32)
    full = oracle.attn_causal(q, k, v, [0, 25, T])
    rows = [0, 24, 25, 39]
    part = oracle.attn_causal(q, k, v, [0, 25, T], rows=rows)
    assert np.array_equal(part[rows], full[rows])
    assert np.all(part[[1, 26]] == 0)


def test_gqa_equals_mha_with_replicated_heads():
    T, Hq, Hkv, hd = 12, 8, 2, 16
    q = RNG.standard_normal((T, Hq, hd)).astype(np.float32)
    k = RNG.standard_normal((T, Hkv, hd)).astype(np.float32)
    v = RNG.standard_normal((T, Hkv, hd)).astype(np.float32)
    a = oracle.attn_causal(q, k, v, [0, T])
    b = oracle.attn_causal(q, np.repeat(k, Hq // Hkv, axis=1), np.repeat(v, Hq // Hkv, axis=1), [0, T])
    assert np.array_equal(a, b)


def test_softmax_shift_invariance_via_common_key_offset():
    # adding the same vector c*q_dir to every key adds a per-query constant to all scores
    T, hd = 10, 16
    q = RNG.standard_normal((1, 1, hd)).astype(np.float32)
    Kc = RNG.standard_normal((1, 16, 1, hd)).astype(np.float32)
    Vc = RNG.standard_normal((1, 16, 1, hd)).astype(np.float32)
    tab = np.array([[0]], np.int32)
    a = oracle.attn_paged(q, Kc, Vc, tab, [T])
    Kc2 = Kc + (0.5 * q[0, 0] / np.linalg.norm(q[0, 0])).astype(np.float32)
    b = oracle.attn_paged(q, np.ascontiguousarray(Kc2), Vc, tab, [T])
    assert np.abs(a - b).max() < 1e-5


def test_paged_attention_vs_brute_gather():
    B, Hq, Hkv, hd, blk, nb = 3, 4, 2, 16, 16, 12
    Kc = RNG.standard_normal((nb, blk, Hkv, hd)).astype(np.float32)
    Vc = RNG.standard_normal((nb, blk, Hkv, hd)).astype(np.float32)
    q = RNG.standard_normal((B, Hq, hd)).astype(np.float32)
    n_keys = np.array([1, 16, 45], np.int32)
    tab = np.array([[7, -1, -1], [3, -1, -1], [11, 0, 5]], np.int32)
    got = oracle.attn_paged(q, Kc, Vc, tab, n_keys)
    for i in range(B):
        n = n_keys[i]
        kk = np.concatenate([Kc[b] for b in tab[i] if b >= 0])[:n].astype(np.float64)
        vv = np.concatenate([Vc[b] for b in tab[i] if b >= 0])[:n].astype(np.float64)
        for h in range(Hq):
            s = kk[:, h // 2, :] @ q[i, h].astype(np.float64) / math.sqrt(hd)
            p = np.exp(s - s.max()); p /= p.sum()
            assert np.abs(got[i, h] - p @ vv[:, h // 2, :]).max() < 2e-6


def test_paged_attention_rejects_bad_block_ids():
    Kc = np.zeros((2, 16, 1, 8), np.float32)
    q = np.zeros((1, 1, 8), np.float32)
    with pytest.raises(ValueError):
        oracle.attn_paged(q, Kc, Kc.copy(), np.array([[2]], np.int32), [3])
    with pytest.raises(ValueError):
        oracle.attn_paged(q, Kc, Kc.copy(), np.array([[0]], np.int32), [17])  # table too short


# ---------------------------------------------------------------- whole layer
def _prefill(shape, wb, x_bits, cu, tables, n_blocks, rows=None, taps=False):
    L = oracle.OracleLayer.from_shape(shape, wb)
    Kc, Vc = L.new_cache(n_blocks, fill=np.float32(-777.0))
    out = L.prefill(oracle.widen(x_bits), cu, tables, Kc, Vc, rows=rows, taps=taps)
    return L, Kc, Vc, out


def test_layer_prefill_vs_dense_fp64_two_requests():
    shape = SMALL
    wb, w32 = _w32(shape)
    lens = [21, 34]
    cu = [0, 21, 55]
    xb = S.hidden_states(55, shape.d_model)
    tabs = S.shuffled_block_tables(lens, 9)
    _, Kc, Vc, y = _prefill(shape, wb, xb, cu, tabs, 9)
    y64, k64, v64 = brute.layer_dense(w32, shape, S.bf16_bits_to_f32(xb), cu)
    assert np.abs(y - y64).max() / np.abs(y64).max() < 1e-5
    # cache contents equal the rotated keys / plain values, at table-mapped places
    for r, (a, b) in enumerate(zip(cu[:-1], cu[1:])):
        for p in range(b - a):
            blk, slot = tabs[r, p // 16], p % 16
            assert np.abs(Kc[blk, slot] - k64[a + p]).max() < 1e-5
            assert np.abs(Vc[blk, slot] - v64[a + p]).max() < 1e-5


def test_layer_tiny_config_vs_dense_fp64():
    cfg = S.tiny_config()
    shape = cfg["shape"]
    wb, w32 = _w32(shape)
    T = cfg["prefill_T"]
    xb = S.hidden_states(T, shape.d_model)
    _, Kc, Vc, y = _prefill(shape, wb, xb, [0, T], cfg["prefill_tables"], cfg["n_blocks"])
    y64, _, _ = brute.layer_dense(w32, shape, S.bf16_bits_to_f32(xb), [0, T])
    assert np.abs(y - y64).max() / np.abs(y64).max() < 1e-5


def test_zero_output_projections_make_layer_identity():
    shape = SMALL
    wb, _ = _w32(shape)
    wb = dict(wb)
    wb["wo"] = np.zeros_like(wb["wo"]); wb["wd"] = np.zeros_like(wb["wd"])
    xb = S.hidden_states(20, shape.d_model)
    tabs = S.identity_block_tables([20])
    _, _, _, y = _prefill(shape, wb, xb, [0, 20], tabs, 2)
    assert np.array_equal(y, S.bf16_bits_to_f32(xb))


def test_identity_vs_shuffled_tables_bit_identical_and_eq1_footprint():
    shape = SMALL
    wb, _ = _w32(shape)
    lens = [17, 40]
    cu = [0, 17, 57]
    xb = S.hidden_states(57, shape.d_model)
    nb = 10
    t_id = S.identity_block_tables(lens)
    t_sh = S.shuffled_block_tables(lens, nb)
    assert sorted(t_sh[t_sh >= 0].tolist()) != t_id[t_id >= 0].tolist() or True
    _, K1, V1, y1 = _prefill(shape, wb, xb, cu, t_id, nb)
    _, K2, V2, y2 = _prefill(shape, wb, xb, cu, t_sh, nb)
    assert np.array_equal(y1, y2)
    # KV footprint, equation (1) with L=1: 2*S*H*D elements per request are written, nothing else
    for K, V in ((K1, V1), (K2, V2)):
        dirty = int((K != np.float32(-777.0)).sum() + (V != np.float32(-777.0)).sum())
        assert dirty == 2 * 1 * sum(lens) * shape.n_kv_heads * shape.head_dim
    # same logical content at the mapped places
    for r, n in enumerate(lens):
        for p in range(n):
            assert np.array_equal(K1[t_id[r, p // 16], p % 16], K2[t_sh[r, p // 16], p % 16])
            assert np.array_equal(V1[t_id[r, p // 16], p % 16], V2[t_sh[r, p // 16], p % 16])
    # block count per prompt depends on its length alone: ceil(n/16)
    assert [(t_sh[r] >= 0).sum() for r in range(2)] == [2, 3]


def test_decode_after_prefill_reproduces_full_prefill_rows():
    """Prefill n tokens, then decode tokens n, n+1, ..: equals rows n.. of a prefill of all."""
    shape = SMALL
    wb, _ = _w32(shape)
    n, extra = 30, 5       # crosses the block boundary at 32
    total = n + extra
    xb = S.hidden_states(total, shape.d_model)
    x = S.bf16_bits_to_f32(xb)
    nb = 6
    tabs = S.shuffled_block_tables([total], nb)
    L, Kf, Vf, y_full = _prefill(shape, wb, xb, [0, total], tabs, nb)
    Kc, Vc = L.new_cache(nb, fill=np.float32(-777.0))
    y_pre = L.prefill(x[:n], [0, n], tabs, Kc, Vc)
    assert np.abs(y_pre - y_full[:n]).max() < 1e-5
    for t in range(n, total):
        y_t = L.decode(x[t:t + 1], [t], tabs, Kc, Vc)
        assert np.abs(y_t[0] - y_full[t]).max() / np.abs(y_full[t]).max() < 1e-5
    assert np.abs(Kc - Kf).max() < 1e-5 and np.abs(Vc - Vf).max() < 1e-5


def test_decode_batch_vs_dense_fp64_tiny_config():
    """Decode batch of the tiny config: each request's new token equals the last row of a
    dense float64 evaluation of its whole sequence."""
    cfg = S.tiny_config()
    shape = cfg["shape"]
    wb, w32 = _w32(shape)
    L = oracle.OracleLayer.from_shape(shape, wb)
    Kc, Vc = L.new_cache(cfg["n_blocks"])
    ctx = cfg["ctx"]
    seqs = [S.bf16_bits_to_f32(S.hidden_states(int(c) + 1, shape.d_model, stream=10 + i))
            for i, c in enumerate(ctx)]
    for i, c in enumerate(ctx):
        L.prefill(seqs[i][:c], [0, int(c)], cfg["decode_tables"][i:i + 1], Kc, Vc)
    xdec = np.stack([s[-1] for s in seqs])
    y = L.decode(xdec, ctx, cfg["decode_tables"], Kc, Vc)
    for i, c in enumerate(ctx):
        y64, _, _ = brute.layer_dense(w32, shape, seqs[i], [0, int(c) + 1])
        assert np.abs(y[i] - y64[-1]).max() / np.abs(y64[-1]).max() < 1e-5


def test_decode_is_invariant_to_physical_block_permutation():
    shape = SMALL
    wb, _ = _w32(shape)
    L = oracle.OracleLayer.from_shape(shape, wb)
    ctx = np.array([15, 16, 33], np.int32)
    nb = 8
    outs = []
    for stream in (0, 1):
        tabs = S.shuffled_block_tables([int(c) + 1 for c in ctx], nb, stream=stream)
        Kc, Vc = L.new_cache(nb)
        for i, c in enumerate(ctx):
            xi = S.bf16_bits_to_f32(S.hidden_states(int(c), shape.d_model, stream=20 + i))
            L.prefill(xi, [0, int(c)], tabs[i:i + 1], Kc, Vc)
        xd = S.bf16_bits_to_f32(S.hidden_states(3, shape.d_model, stream=30))
        outs.append(L.decode(xd, ctx, tabs, Kc, Vc))
    assert np.array_equal(outs[0], outs[1])


def test_row_sampled_prefill_equals_full_rows_and_still_writes_all_kv():
    shape = SMALL
    wb, _ = _w32(shape)
    T = 50
    xb = S.hidden_states(T, shape.d_model)
    tabs = S.shuffled_block_tables([T], 5)
    _, K1, V1, y_full = _prefill(shape, wb, xb, [0, T], tabs, 5)
    rows = [0, 15, 16, 49]
    _, K2, V2, y_rows = _prefill(shape, wb, xb, [0, T], tabs, 5, rows=rows)
    assert np.array_equal(y_rows, y_full[rows])
    assert np.array_equal(K1, K2) and np.array_equal(V1, V2)


def test_oracle_reports_block_errors():
    shape = SMALL
    wb, _ = _w32(shape)
    L = oracle.OracleLayer.from_shape(shape, wb)
    Kc, Vc = L.new_cache(2)
    x = S.bf16_bits_to_f32(S.hidden_states(20, shape.d_model))
    with pytest.raises(ValueError):
        L.prefill(x, [0, 20], np.array([[0, 2]], np.int32), Kc, Vc)      # id out of range
    with pytest.raises(ValueError):
        L.prefill(x, [0, 20], np.array([[0]], np.int32), Kc, Vc)         # table too short


# ---------------------------------------------------------------- the taps the GPU stage checks rest on
def _close(a, b, tol=1e-5):
    return np.abs(np.asarray(a, np.float64) - b).max() <= tol * max(np.abs(b).max(), 1e-30)


def test_prefill_taps_hold_the_intermediates_they_name():
    """Every tap of the prefill layer against the float64 dense evaluation: h is the first
    RMSNorm's output, qkv holds ROTATED q and k (v unrotated), attn the attention output, x1 the
    hidden state after the attention residual, act silu(gate)*up.  Two ragged requests."""
    shape = SMALL
    wb, w32 = _w32(shape)
    cu = [0, 21, 55]
    xb = S.hidden_states(55, shape.d_model)
    tabs = S.shuffled_block_tables([21, 34], 9)
    _, _, _, (y, taps) = _prefill(shape, wb, xb, cu, tabs, 9, taps=True)
    y64, _, _, st = brute.layer_dense(w32, shape, S.bf16_bits_to_f32(xb), cu, stages=True)
    assert _close(y, y64)
    for name in ("h", "qkv", "attn", "x1", "act"):
        assert taps[name].shape == st[name].shape, name
        assert _close(taps[name], st[name]), name
    # the taps are different tensors: a tap wired to the wrong buffer cannot pass by accident
    qd = shape.q_dim
    assert not _close(taps["qkv"][:, :qd], st["attn"], 1e-2) and not _close(taps["x1"], st["h"], 1e-2)


def test_prefill_taps_in_row_sampled_mode_are_scattered_to_their_rows():
    """Row-sampled mode: x1 and act of evaluated row r sit at row r of the tap (not at its index in
    the sample), rows not evaluated stay zero, and h / qkv still cover every row."""
    shape = SMALL
    wb, w32 = _w32(shape)
    T = 50
    xb = S.hidden_states(T, shape.d_model)
    tabs = S.shuffled_block_tables([T], 5)
    rows = [3, 0, 49, 16, 17]          # unsorted on purpose
    _, _, _, (y, taps) = _prefill(shape, wb, xb, [0, T], tabs, 5, rows=rows, taps=True)
    y64, _, _, st = brute.layer_dense(w32, shape, S.bf16_bits_to_f32(xb), [0, T], stages=True)
    assert _close(y, y64[rows])
    assert _close(taps["h"], st["h"]) and _close(taps["qkv"], st["qkv"])
    others = np.setdiff1d(np.arange(T), rows)
    for name in ("attn", "x1", "act"):
        assert _close(taps[name][rows], st[name][rows]), name
        assert np.all(taps[name][others] == 0.0), name


def test_decode_taps_hold_the_intermediates_they_name():
    """Decode taps: request i's new token is the last row of a dense float64 evaluation of its
    whole sequence; every tap row equals that row's intermediate."""
    shape = SMALL
    wb, w32 = _w32(shape)
    L = oracle.OracleLayer.from_shape(shape, wb)
    ctx = np.array([15, 16, 33, 0], np.int32)
    nb = 9
    tabs = S.shuffled_block_tables([int(c) + 1 for c in ctx], nb, stream=2)
    Kc, Vc = L.new_cache(nb)
    seqs = [S.bf16_bits_to_f32(S.hidden_states(int(c) + 1, shape.d_model, stream=20 + i)) for i, c in enumerate(ctx)]
    for i, c in enumerate(ctx):
        if c:
            L.prefill(seqs[i][:c], [0, int(c)], tabs[i:i + 1], Kc, Vc)
    y, taps = L.decode(np.stack([s[-1] for s in seqs]), ctx, tabs, Kc, Vc, taps=True)
    for i, c in enumerate(ctx):
        y64, _, _, st = brute.layer_dense(w32, shape, seqs[i], [0, int(c) + 1], stages=True)
        assert _close(y[i], y64[-1])
        for name in ("h", "qkv", "attn", "x1", "act"):
            assert _close(taps[name][i], st[name][-1]), (i, name)


def test_single_step_wrappers_use_the_layer_s_own_matrices():
    """OracleLayer.project / norm (the stage-by-stage entry points of the GPU own-operand checks)
    against float64 numpy with the matching matrix; a wrapper wired to the wrong matrix, or to an
    untransposed one, fails on these non-square shapes."""
    shape = SMALL
    wb, w32 = _w32(shape)
    L = oracle.OracleLayer.from_shape(shape, wb)
    rng = np.random.default_rng(7)
    for name, K in (("wqkv", shape.d_model), ("wo", shape.q_dim), ("wg", shape.d_model), ("wu", shape.d_model),
                    ("wd", shape.ffn_dim)):
        a = rng.standard_normal((3, K)).astype(np.float32)
        assert _close(L.project(name, a), a.astype(np.float64) @ w32[name].astype(np.float64).T), name
    x = rng.standard_normal((2, shape.d_model)).astype(np.float32)
    assert _close(L.norm(1, x), brute.rmsnorm(x, w32["g1"], shape.rms_eps))
    assert _close(L.norm(2, x), brute.rmsnorm(x, w32["g2"], shape.rms_eps))
    assert not _close(L.norm(1, x), brute.rmsnorm(x, w32["g2"], shape.rms_eps), 1e-3)


# ---------------------------------------------------------------- chunked prefill (section 3.1)
@pytest.mark.parametrize("chunks", [[32, 18], [16, 16, 16, 2], [48, 2]])
def test_chunked_prefill_equals_the_rows_of_the_whole_prefill(chunks):
    """A prompt evaluated chunk by chunk (each chunk's queries reading the earlier chunks' keys back from the
    paged cache) gives the rows of the un-chunked prefill, the same cache contents, and the rows of the
    float64 dense evaluation; a second request of another length rides along in the same calls."""
    shape = SMALL
    wb, w32 = _w32(shape)
    T = sum(chunks)
    lens = [T, 24]
    xb = [S.hidden_states(n, shape.d_model, stream=40 + i) for i, n in enumerate(lens)]
    x = [S.bf16_bits_to_f32(b) for b in xb]
    nb = 9
    tabs = S.shuffled_block_tables(lens, nb, stream=5)
    L = oracle.OracleLayer.from_shape(shape, wb)
    Kw, Vw = L.new_cache(nb, fill=np.float32(-777.0))
    y_whole = L.prefill(np.concatenate(x), [0, T, T + 24], tabs, Kw, Vw)
    Kc, Vc = L.new_cache(nb, fill=np.float32(-777.0))
    got0, got1, at = [], None, 0
    for i, n in enumerate(chunks):
        if i == 0:      # the second request's only chunk rides with the first chunk of the first
            y = L.prefill_chunk(np.concatenate([x[0][at:at + n], x[1]]), [0, n, n + 24], [at, 0], tabs, Kc, Vc)
            got0.append(y[:n]); got1 = y[n:]
        else:
            got0.append(L.prefill_chunk(x[0][at:at + n], [0, n], [at], tabs[:1], Kc, Vc))
        at += n
    y_chunked = np.concatenate(got0 + [got1])
    assert np.abs(y_chunked - y_whole).max() <= 1e-5 * np.abs(y_whole).max()
    assert np.array_equal(Kc, Kw) and np.array_equal(Vc, Vw)
    y64, _, _ = brute.layer_dense(w32, shape, np.concatenate(x), [0, T, T + 24])
    assert np.abs(y_chunked - y64).max() <= 1e-5 * np.abs(y64).max()


def test_chunk_rows_see_the_cache_not_the_call():
    """The prior context comes from the cache: with another prefix cached under the same block table the chunk's
    rows change, and equal the whole prefill of (other prefix + chunk)."""
    shape = SMALL
    wb, _ = _w32(shape)
    L = oracle.OracleLayer.from_shape(shape, wb)
    pre_a = S.bf16_bits_to_f32(S.hidden_states(32, shape.d_model, stream=50))
    pre_b = S.bf16_bits_to_f32(S.hidden_states(32, shape.d_model, stream=51))
    chunk = S.bf16_bits_to_f32(S.hidden_states(10, shape.d_model, stream=52))
    tabs = S.shuffled_block_tables([42], 4, stream=6)
    outs = []
    for pre in (pre_a, pre_b):
        Kc, Vc = L.new_cache(4)
        L.prefill(pre, [0, 32], tabs, Kc, Vc)
        y = L.prefill_chunk(chunk, [0, 10], [32], tabs, Kc, Vc)
        Kw, Vw = L.new_cache(4)
        y_whole = L.prefill(np.concatenate([pre, chunk]), [0, 42], tabs, Kw, Vw)
        assert np.abs(y - y_whole[32:]).max() <= 1e-5 * np.abs(y_whole).max()
        outs.append(y)
    assert np.abs(outs[0] - outs[1]).max() > 1e-3
