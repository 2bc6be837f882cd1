"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bit-exact on cache indexing, <= 2e-2 max relative error on activations."""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_11822_amd as rs
import rs_synth as S
from tests.gpu_util import (END_TO_END, TOL, Rig, check_cache_against_oracle, check_stages_own_operands, check_tensor,
                            rel_err, residual_err, to_bits, to_dev)

pytestmark = pytest.mark.gpu

ORC_SENT = np.float32(-777.0)
f32 = S.bf16_bits_to_f32


def _check_stages(rig, side, taps, M, x, attention_only=False, stage_elem=END_TO_END):
    """Intermediate tensors against the fp32 oracle's taps.  Upstream of the softmax (rotated q, v)
    the stated 2e-2 holds element by element; downstream of it the oracle's end-to-end value
    differs by the bf16 rounding of the stored q and k, amplified by peaked softmax rows, so the
    per-element bound there is END_TO_END times wider (max and rms bounds unchanged) -- the strict
    per-element check of those stages is check_stages_own_operands.  The first RMSNorm buffer is
    reused by the second one and the k columns of the qkv buffer stay unrotated (the rotated keys
    live in the cache, which is checked separately), so those two are not compared.
    stage_elem=None: max and rms bounds only for the attention output and the SwiGLU product."""
    sh = rig.shape
    qd, kvd = sh.q_dim, sh.kv_dim
    qkv = f32(rig.ctx.debug_read_workspace(side, 1, (M, sh.qkv_dim)))
    check_tensor("q (rotated)", qkv[:, :qd], taps["qkv"][:, :qd])
    check_tensor("v", qkv[:, qd + kvd:], taps["qkv"][:, qd + kvd:])
    check_tensor("attention out", f32(rig.ctx.debug_read_workspace(side, 2, (M, qd))), taps["attn"], elem_mult=stage_elem)
    check_tensor("x1 = x + attn Wo", f32(rig.ctx.debug_read_workspace(side, 3, (M, sh.d_model))), taps["x1"], x, 1,
                 elem_mult=END_TO_END)
    if not attention_only:
        check_tensor("silu(gate)*up", f32(rig.ctx.debug_read_workspace(side, 4, (M, sh.ffn_dim))), taps["act"],
                     elem_mult=stage_elem)


def _prefill_case(shape, lens, n_blocks_extra=3, stream=0):
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    n_blocks = sum(S.blocks_for(n) for n in lens) + n_blocks_extra
    tabs = S.shuffled_block_tables(lens, n_blocks, stream=stream)
    xb = S.hidden_states(T, shape.d_model, stream=stream)
    return cu, T, n_blocks, tabs, xb


def _run_prefill_parity(shape, lens, wo_std=None, wd_std=None, stage_elem=END_TO_END):
    cu, T, n_blocks, tabs, xb = _prefill_case(shape, lens)
    rig = Rig(shape, n_blocks, T, 1, max(lens) + 1, wo_std=wo_std, wd_std=wd_std)
    try:
        y_bits = rig.prefill(xb, cu, tabs)
        L = rig.olayers[0]
        Kc, Vc = L.new_cache(n_blocks, fill=ORC_SENT)
        x = f32(xb)
        y_ref, taps = L.prefill(x, cu, tabs, Kc, Vc, taps=True)
        print("prefill", shape.name, lens)
        # a loud attention branch perturbs everything downstream of it by the branch's own
        # relative error: only the attention half of the layer is judged in that case
        check_cache_against_oracle(rig, Kc, Vc, ORC_SENT)
        check_stages_own_operands(rig, rs.RS_SIDE_PREFILL, L, T, x, y_bits, cu=cu, tables=tabs)
        _check_stages(rig, rs.RS_SIDE_PREFILL, taps, T, x, attention_only=wo_std is not None, stage_elem=stage_elem)
        if wo_std is None:
            check_tensor("y (layer output)", f32(y_bits), y_ref, x, 2, elem_mult=END_TO_END)
        assert np.isfinite(f32(y_bits)).all()
    finally:
        rig.close()


def test_cu_masks_confine_workgroups():
    """Section 4.2: workgroups of a masked queue run only on the masked-in CUs."""
    rig = Rig(S.TINY, 4, 16, 4, 64, with_oracle=False)
    try:
        seen = {}
        for p, d in [(256, 256), (128, 128), (64, 192), (192, 64), (32, 224)]:
            rig.ctx.set_cu_split(p, d)
            hp = rig.ctx.debug_cu_histogram(0, 8192)
            hd_ = rig.ctx.debug_cu_histogram(1, 8192)
            assert hp.sum() == 8192 and hd_.sum() == 8192
            cus_p, cus_d = set(np.nonzero(hp)[0]), set(np.nonzero(hd_)[0])
            seen[(p, d)] = (cus_p, cus_d)
            print("split", (p, d), "distinct CUs used:", len(cus_p), len(cus_d),
                  "per XCC prefill", [sum(1 for c in cus_p if c >> 8 == x) for x in range(8)])
            assert len(cus_p) == p and len(cus_d) == d
            if p + d <= 256:
                assert not (cus_p & cus_d), "disjoint split shares a CU"
                for s_ in (cus_p, cus_d):
                    per_xcc = [sum(1 for c in s_ if c >> 8 == x) for x in range(8)]
                    assert len(set(per_xcc)) == 1, f"uneven XCD shares {per_xcc}"
                    # equally many units in every shader engine the side uses (id bits 7:5), in every XCD
                    for x in range(8):
                        per_se = [sum(1 for c in s_ if c >> 8 == x and (c >> 5) & 7 == e) for e in range(8)]
                        assert len({k for k in per_se if k}) == 1, f"uneven shader engines {per_se} in XCD {x}"
        assert len(seen[(256, 256)][0]) == 256
    finally:
        rig.close()


def test_prefill_tiny_config():
    _run_prefill_parity(S.TINY, [128])


def test_prefill_tiny_ragged_multi_request():
    _run_prefill_parity(S.TINY, [1, 17, 130, 64])


def test_prefill_mid_gqa_ragged():
    _run_prefill_parity(S.MID, [200, 100, 77])


def test_prefill_odd_widths_large_tile_edges():
    """Every projection's width is a multiple of 32 but of no tile width, and the row counts are ragged against the
    tile heights: the large-tile kernels' edge path (column checks per store, row-major and packed outputs,
    residual reads) is what writes the last columns of q/k/v, x1, the SwiGLU output and the layer output.
    513 rows: few tiles, so the output and down projections go through the K-split kernel and its epilogue;
    3400 rows: enough tiles that every projection ends in the large-tile kernel's own epilogue."""
    _run_prefill_parity(S.ODD, [300, 213])
    _run_prefill_parity(S.ODD, [2000, 1400])


def test_prefill_wide_large_tile_path_ragged():
    """d_model 1024: every prefill GEMM takes the large-tile LDS-DMA kernel; 600 rows is ragged
    against both tile heights."""
    _run_prefill_parity(S.WIDE, [333, 267])


@pytest.mark.parametrize("which", ["wo", "wd"])
def test_prefill_wide_loud_output_projection(which):
    _run_prefill_parity(S.WIDE, [520], **{which + "_std": 0.2})


@pytest.mark.parametrize("which", ["wo", "wd"])
def test_prefill_mid_loud_output_projection(which):
    """One output projection drawn N(0, 0.2): that branch is several times larger than the
    residual input, so its check is not cushioned by the bf16 quantum of the residual stream."""
    _run_prefill_parity(S.MID, [150, 90], **{which + "_std": 0.2})


def _fill_contexts(rig, ctx, tabs, stream0):
    """Prefill each request's context on GPU and oracle; returns oracle caches."""
    shape = rig.shape
    L = rig.olayers[0]
    Kc, Vc = L.new_cache(rig.n_blocks, fill=ORC_SENT)
    lens = [int(c) for c in ctx if c > 0]
    idx = [i for i, c in enumerate(ctx) if c > 0]
    for g in range(0, len(lens), rs.RS_MAX_PREFILL_REQS):      # a prefill call takes at most 64 prompts
        gl, gi = lens[g:g + rs.RS_MAX_PREFILL_REQS], idx[g:g + rs.RS_MAX_PREFILL_REQS]
        cu = np.concatenate([[0], np.cumsum(gl)]).astype(np.int32)
        xb = S.hidden_states(int(cu[-1]), shape.d_model, stream=stream0 + 7 * (g // rs.RS_MAX_PREFILL_REQS))
        rig.prefill(xb, cu, tabs[gi])
        L.prefill(f32(xb), cu, tabs[gi], Kc, Vc)
    return Kc, Vc


def _run_decode_parity(shape, ctx, stream=0, wo_std=None, wd_std=None):
    ctx = np.asarray(ctx, np.int32)
    B = len(ctx)
    counts = [int(c) + 1 for c in ctx]
    n_blocks = sum(S.blocks_for(c) for c in counts) + 5
    tabs = S.shuffled_block_tables(counts, n_blocks, stream=stream)
    rig = Rig(shape, n_blocks, max(int(ctx.sum()), 1), B, int(ctx.max()) + 1, wo_std=wo_std, wd_std=wd_std)
    try:
        Kc, Vc = _fill_contexts(rig, ctx, tabs, 40 + stream)
        L = rig.olayers[0]
        xb = S.hidden_states(B, shape.d_model, stream=50 + stream)
        y_bits = rig.decode(xb, ctx, tabs)
        x = f32(xb)
        y_ref, taps = L.decode(x, ctx, tabs, Kc, Vc, taps=True)
        print("decode", shape.name, ctx.tolist())
        check_cache_against_oracle(rig, Kc, Vc, ORC_SENT)
        check_stages_own_operands(rig, rs.RS_SIDE_DECODE, L, B, x, y_bits, ctx=ctx, tables=tabs)
        _check_stages(rig, rs.RS_SIDE_DECODE, taps, B, x, attention_only=wo_std is not None)
        if wo_std is None:
            check_tensor("y (layer output)", f32(y_bits), y_ref, x, 2, elem_mult=END_TO_END)
        assert np.isfinite(f32(y_bits)).all()
    finally:
        rig.close()


def test_decode_tiny_config():
    _run_decode_parity(S.TINY, [64, 128, 192, 256])


def test_decode_edge_contexts_tiny():
    # empty cache, block edges, chunk (512) edges
    _run_decode_parity(S.TINY, [0, 1, 15, 16, 17, 511, 512, 513], stream=1)


def test_decode_mid_gqa_several_chunks():
    _run_decode_parity(S.MID, [5, 127, 128, 640, 1100], stream=2)


def test_decode_batch_spanning_both_token_tiles():
    # 40 rows: the second 32-row tile of the skinny GEMMs is partly valid
    ctx = [(37 * i) % 300 for i in range(40)]
    _run_decode_parity(S.MID, ctx, stream=5)


def test_decode_batch_over_64_takes_the_tiled_gemms():
    # more than 64 rows leave the skinny path: packed activations with 3 row tiles, tiled GEMMs on the decode side
    ctx = [(53 * i) % 260 for i in range(70)]
    _run_decode_parity(S.MID, ctx, stream=6)


def test_decode_batch_130_wide_takes_the_large_tile_gemms_with_sliced_k():
    # 130 rows on the wide shape: the decode side's GEMMs are the large-tile kernel (second 128-row tile almost
    # empty), the output and down projections with their K range sliced
    ctx = [(29 * i) % 61 for i in range(130)]
    _run_decode_parity(S.WIDE, ctx, stream=8)


@pytest.mark.parametrize("which", ["wo", "wd"])
def test_decode_mid_loud_output_projection(which):
    _run_decode_parity(S.MID, [40, 513, 700], stream=4, **{which + "_std": 0.2})


def test_decode_after_prefill_matches_prefill_rows_on_gpu():
    shape = S.MID
    n, extra = 60, 6
    total = n + extra
    tabs = S.shuffled_block_tables([total], 8)
    xb = S.hidden_states(total, shape.d_model, stream=7)
    rig = Rig(shape, 8, total, 1, total + 1)
    try:
        y_full = f32(rig.prefill(xb, [0, total], tabs))
        rig.k_pool.view(torch.int16).fill_(0x7FC1); rig.v_pool.view(torch.int16).fill_(0x7FC1)
        rig.prefill(xb[:n], [0, n], tabs)
        x = f32(xb)
        for t in range(n, total):
            y_t = f32(rig.decode(xb[t:t + 1], [t], tabs))
            e = residual_err(y_t[0], y_full[t], x[t], roundings=4)   # both sides are bf16 outputs
            assert e <= 1.0, (t, e)
    finally:
        rig.close()


def _decode_setup(shape, ctx, stream):
    ctx = np.asarray(ctx, np.int32)
    counts = [int(c) + 1 for c in ctx]
    n_blocks = sum(S.blocks_for(c) for c in counts) + 40
    return ctx, counts, n_blocks


def test_decode_bit_identical_across_splits_concurrency_and_block_permutation():
    """CU masking is transparent to kernels (section 4.2): same bits under every split, with or
    without a prefill running on the other side, and under a permutation of physical blocks."""
    shape = S.MID
    ctx, counts, n_blocks = _decode_setup(shape, [33, 700, 1500, 64, 257, 900], 3)
    B = len(ctx)
    xb = S.hidden_states(B, shape.d_model, stream=60)
    kb_log, vb_log = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim)
    pre_T = 512
    pre_x = S.hidden_states(pre_T, shape.d_model, stream=61)
    results = []
    for perm_stream in (0, 1):
        tabs_all = S.shuffled_block_tables(counts + [pre_T], n_blocks + 40, stream=perm_stream)
        tabs, ptab = tabs_all[:B], tabs_all[B:B + 1]
        rig = Rig(shape, n_blocks + 40, pre_T, B, int(ctx.max()) + 1, with_oracle=False)
        try:
            # logical content: request i, position p holds row (i*4096 + p) % ... of a seeded pool
            k_log = np.zeros((n_blocks + 40, 16) + kb_log.shape[2:], np.uint16)
            v_log = np.zeros_like(k_log)
            src_k = kb_log.reshape(-1, *kb_log.shape[2:]); src_v = vb_log.reshape(-1, *vb_log.shape[2:])
            at = 0
            for i, c in enumerate(ctx):
                for p in range(int(c)):
                    k_log[tabs[i, p // 16], p % 16] = src_k[at]; v_log[tabs[i, p // 16], p % 16] = src_v[at]
                    at += 1
            for split, concurrent in [((256, 256), False), ((128, 128), False), ((192, 64), True),
                                      ((64, 192), True), ((256, 256), True), ((0, 256), False)]:
                rig.load_pools_from_logical(k_log, v_log)
                rig.ctx.set_cu_split(*split)
                if concurrent:
                    for _ in range(3):
                        rig.prefill(pre_x, [0, pre_T], ptab, sync=False)
                y = rig.decode(xb, ctx, tabs)
                rig.ctx.sync(rs.RS_SIDE_PREFILL) if split[0] else None
                results.append(y.copy())
        finally:
            rig.close()
    for y in results[1:]:
        assert np.array_equal(results[0], y)


def test_bad_block_ids_are_reported_not_dereferenced():
    shape = S.TINY
    rig = Rig(shape, 8, 64, 2, 64, with_oracle=False)
    try:
        xb = S.hidden_states(40, shape.d_model)
        before_k = rig.k_bits_logical().copy()
        with pytest.raises(rs.RapidServeError) as e:
            rig.prefill(xb, [0, 40], np.array([[0, 1 << 20, 2]], np.int32))
        assert e.value.code == rs.RS_ERR_BAD_BLOCK
        after_k = rig.k_bits_logical()
        # block 1 << 20 was skipped; blocks 0 and 2 were written
        assert (after_k[0] != before_k[0]).any() and (after_k[2, :8] != before_k[2, :8]).any()
        rig.ctx.sync(1)          # each side has its own error word: the decode side met nothing
        rig.ctx.sync(0)          # flag cleared
        with pytest.raises(rs.RapidServeError) as e:   # table too short is caught on the host
            rig.ctx.prefill_layer(0, to_dev(xb), to_dev(xb), [0, 40], torch.zeros(2, dtype=torch.int32, device="cuda"), 2)
        assert e.value.code == rs.RS_ERR_BAD_BLOCK
        with pytest.raises(rs.RapidServeError) as e:
            rig.decode(S.hidden_states(2, shape.d_model), [20, 30], np.array([[0, -1, -1, -1], [1, -5, 2, 3]], np.int32))
        assert e.value.code == rs.RS_ERR_BAD_BLOCK
        rig.ctx.sync(0)          # ... and the prefill side nothing
        # a context length beyond the launch's max_ctx (a position outside the rotary table, too): never used as an extent
        with pytest.raises(rs.RapidServeError) as e:
            rig.decode(S.hidden_states(2, shape.d_model), [70, 30], np.array([[0, 1, 2, 3], [4, 5, 6, 7]], np.int32), max_ctx=64)
        assert e.value.code == rs.RS_ERR_BAD_BLOCK
        rig.ctx.sync(1)
    finally:
        rig.close()


def test_serving_step_small_stack_matches_oracle():
    """rs_submit / rs_step: one request through a 2-layer stack; each decode step's output
    equals the oracle's stack evaluated the same way."""
    shape = S.TINY
    n_layers, prompt, out_len = 2, 40, 3
    rig = Rig(shape, 16, 64, 4, 64, n_layers=n_layers)
    try:
        pb = S.hidden_states(prompt, shape.d_model, stream=70)
        p_dev = to_dev(pb)
        rig.ctx.submit(5, prompt, out_len, p_dev)
        dec_in = [S.hidden_states(1, shape.d_model, stream=71 + i) for i in range(out_len)]
        d_out = torch.zeros((4, shape.d_model), dtype=torch.bfloat16, device="cuda")
        so = rig.ctx.step(to_dev(dec_in[0]), d_out)
        assert so.prefill_started_req == 5 and so.decode_batch == 0
        rig.ctx.sync(rs.RS_SIDE_PREFILL)
        # oracle: same block ids (fresh LIFO pool hands out 0,1,2)
        tabs = np.array([[0, 1, 2, -1]], np.int32)
        caches = [L.new_cache(16) for L in rig.olayers]
        x = f32(pb)
        for l, L in enumerate(rig.olayers):
            x = L.prefill(x, [0, prompt], tabs, *caches[l])
        outs = []
        for i in range(out_len):
            keep = to_dev(dec_in[i])
            so = rig.ctx.step(keep, d_out, wait_decode=True)
            assert so.decode_batch == 1 and so.decode_sum_ctx == prompt + i and so.decode_ms > 0
            rig.ctx.sync(rs.RS_SIDE_DECODE)
            got = f32(to_bits(d_out[:1]))
            xr = f32(dec_in[i])
            for l, L in enumerate(rig.olayers):
                xr = L.decode(xr, [prompt + i], tabs, *caches[l])
            e = residual_err(got, xr, f32(dec_in[i]), roundings=4, layers=n_layers)   # two layers: four bf16 stores
            print("step", i, "fraction of allowed error", e)
            assert e <= 1.0
        so = rig.ctx.step(to_dev(dec_in[0]), d_out)
        assert so.n_finished == 1 and rig.ctx.request_state(5) == 5 and rig.ctx.kv_num_free() == 16
    finally:
        rig.close()


@pytest.mark.parametrize("lens", [[40], [33, 31], [150, 50], [65]])
def test_8b_layer_short_prefill_passes(lens):
    """Llama-3-8B-shaped layer with a few dozen to a few hundred rows: up to 64 rows the pass takes the
    weight-streaming GEMMs, above that the large-tile kernel with its K range cut into slices for the
    projections back to d_model (few output tiles, long K).  Every stage and every row against the oracle.

    Every stage downstream of the QKV projection holds the stated 2e-2 element by element against the oracle's
    routine for that stage fed the kernel's own bf16 operands (check_stages_own_operands).  Against the fp32
    oracle's END-TO-END taps the stated bound on the maximum and the rms bound hold for every stage too, but
    no per-element bound is applied to the attention output and the SwiGLU product at this shape: with
    d_model = 4096 the vectors are long (|q| ~ 15, |k| ~ 17), so rounding q and k to bf16 for storage moves a
    score by ~1e-2 and a softmax weight by ~1 %; where two keys with weights ~0.4 carry values of opposite
    sign that is 6-7 % of the row's rms in one element -- a property of the bf16 storage format both sides of
    the comparison do not share, not of the kernel's arithmetic, which the own-operand check isolates."""
    _run_prefill_parity(S.LLAMA8B, lens, stage_elem=None)


def test_full_size_8b_layer_sampled_rows():
    """The benchmark's own configuration (Llama-3-8B-shaped layer, prefill 1x2048, decode batch 64
    with contexts U[512,4096]) in the launch configuration bench.py times: the whole K/V cache
    the prefill writes, sampled prefill rows and every decode row against the oracle."""
    shape = S.LLAMA8B
    T, B = 2048, 64
    ctx = S.uniform_context_lengths(B, 512, 4096)
    counts = [int(c) + 1 for c in ctx] + [T]
    n_blocks = sum(S.blocks_for(c) for c in counts) + 64
    tabs = S.shuffled_block_tables(counts, n_blocks, max_blk=S.blocks_for(max(counts)))
    dtab, ptab = tabs[:B], tabs[B:B + 1]
    rig = Rig(shape, n_blocks, T, B, int(ctx.max()) + 1, sentinel=0x7FC1)
    try:
        L = rig.olayers[0]
        # ---- prefill
        xb = S.hidden_states(T, shape.d_model, stream=0)
        x = f32(xb)
        rig.ctx.set_cu_split(192, 64)
        y_bits = rig.prefill(xb, [0, T], ptab)
        rng = np.random.default_rng(11)
        rows = np.unique(np.concatenate([[0, 1, 15, 16, 17, 127, 128, 255, 256, 1023, 1024, 2046, 2047],
                                         rng.integers(0, T, 19)])).astype(np.int32)
        Kc, Vc = L.new_cache(n_blocks, fill=ORC_SENT)
        y_ref = L.prefill(x, [0, T], ptab, Kc, Vc, rows=rows)
        check_cache_against_oracle(rig, Kc, Vc, ORC_SENT)
        check_tensor("8B prefill y, sampled rows", f32(y_bits)[rows], y_ref, x[rows], 2, elem_mult=END_TO_END)
        # ---- decode over a directly written cache (same bits on both sides)
        kb, vb = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim)
        rig.load_pools_from_logical(kb, vb)
        Kc, Vc = f32(kb), f32(vb)
        db = S.hidden_states(B, shape.d_model, stream=50)
        yd = rig.decode(db, ctx, dtab)
        yd_ref = L.decode(f32(db), ctx, dtab, Kc, Vc)
        check_tensor("8B decode y, batch 64", f32(yd), yd_ref, f32(db), 2, elem_mult=END_TO_END)
        # appended K/V of the new tokens: exact slots, contents to tolerance
        kg, vg = f32(rig.k_bits_logical()), f32(rig.v_bits_logical())
        changed = (rig.k_bits_logical() != kb).any(axis=(2, 3))
        want = np.zeros_like(changed)
        for i, c in enumerate(ctx):
            want[dtab[i, c // 16], c % 16] = True
            assert rel_err(kg[dtab[i, c // 16], c % 16].reshape(1, -1), Kc[dtab[i, c // 16], c % 16].reshape(1, -1)) <= TOL
            assert rel_err(vg[dtab[i, c // 16], c % 16].reshape(1, -1), Vc[dtab[i, c // 16], c % 16].reshape(1, -1)) <= TOL
        assert np.array_equal(changed, want), "decode wrote K/V slots other than each request's next position"
    finally:
        rig.close()


def test_8b_layer_bit_identical_across_splits_and_concurrency_with_oracle_rows():
    """The benchmark's layer at the partitions bench.py times.  The prefill GEMMs pick their tile
    schedule from the partition's CU count, so: the 2048-token prefill pass at 64, 128, 192 and 256
    prefill CUs, alone and beside a running decode loop, must give the same bits -- layer output and
    the K/V it writes -- and so must the batch-64 decode step at 64 ... 256 decode CUs, alone and
    beside a prefill.  Sampled prefill rows and every decode row are then compared with the oracle
    once, at the 128/128 split under co-run (stage by stage on the kernels' own operands at 2e-2
    per element, and end to end)."""
    shape = S.LLAMA8B
    T, B = 2048, 64
    ctx = S.uniform_context_lengths(B, 512, 4096)
    counts = [int(c) + 1 for c in ctx] + [T]
    n_blocks = sum(S.blocks_for(c) for c in counts) + 64
    tabs = S.shuffled_block_tables(counts, n_blocks, max_blk=S.blocks_for(max(counts)))
    dtab, ptab = tabs[:B], tabs[B:B + 1]
    rig = Rig(shape, n_blocks, T, B, int(ctx.max()) + 1, sentinel=0x7FC1)
    try:
        L = rig.olayers[0]
        xb = S.hidden_states(T, shape.d_model, stream=0)
        db = S.hidden_states(B, shape.d_model, stream=50)
        kb, vb = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim)
        mine = torch.from_numpy(ptab[0, :S.blocks_for(T)].astype(np.int64)).cuda()
        ref_bits = None
        for (pc, dc), beside in [((256, 256), False), ((64, 192), False), ((128, 128), False), ((192, 64), False),
                                 ((256, 0), False), ((0, 256), False), ((64, 192), True), ((128, 128), True)]:
            rig.load_pools_from_logical(kb, vb)
            rig.ctx.set_cu_split(pc, dc)
            print("split", (pc, dc), "co-running" if beside else "alone", flush=True)
            yp = yd = None
            if beside:
                # decode steps in front of, beside and behind the prefill pass
                for _ in range(4):
                    rig.decode(db, ctx, dtab, sync=False)
                yp_t = rig.prefill(xb, [0, T], ptab, sync=False)
                for _ in range(6):
                    yd_t = rig.decode(db, ctx, dtab, sync=False)
                rig.ctx.sync(rs.RS_SIDE_PREFILL); rig.ctx.sync(rs.RS_SIDE_DECODE)
                yp, yd = to_bits(yp_t), to_bits(yd_t)
            else:
                if pc:
                    yp = rig.prefill(xb, [0, T], ptab)
                if dc:
                    yd = rig.decode(db, ctx, dtab)
            got = {"yp": yp, "yd": yd,
                   "k": to_bits(rig.k_pool[0].index_select(0, mine)) if pc else None,
                   "v": to_bits(rig.v_pool[0].index_select(0, mine)) if pc else None}
            if ref_bits is None:
                ref_bits = got
            for name, val in got.items():
                if val is not None:
                    assert np.array_equal(val, ref_bits[name]), f"{name} differs at split {(pc, dc)}, beside={beside}"
        # ---- the state left by the last configuration (128/128 under co-run) against the oracle
        x, xd = f32(xb), f32(db)
        rng = np.random.default_rng(11)
        rows = np.unique(np.concatenate([[0, 1, 15, 16, 17, 127, 128, 255, 256, 1023, 1024, 2046, 2047],
                                         rng.integers(0, T, 19)])).astype(np.int32)
        check_stages_own_operands(rig, rs.RS_SIDE_PREFILL, L, T, x, ref_bits["yp"], cu=np.array([0, T], np.int32),
                                  tables=ptab, rows=rows)
        check_stages_own_operands(rig, rs.RS_SIDE_DECODE, L, B, xd, ref_bits["yd"], ctx=ctx, tables=dtab)
        Kc, Vc = f32(kb), f32(vb)
        y_ref = L.prefill(x, [0, T], ptab, Kc, Vc, rows=rows)
        check_tensor("8B prefill y at 128/128 beside decode, sampled rows", f32(ref_bits["yp"])[rows], y_ref, x[rows], 2,
                     elem_mult=END_TO_END)
        yd_ref = L.decode(xd, ctx, dtab, Kc, Vc)
        check_tensor("8B decode y at 128/128 beside prefill", f32(ref_bits["yd"]), yd_ref, xd, 2, elem_mult=END_TO_END)
    finally:
        rig.close()


def test_70b_shaped_layer_sampled_rows():
    """Llama-3-70B-shaped layer (d 8192, 64/8 heads, FFN 28672): the widest RMSNorm variant, GEMM
    shapes with other tile counts and schedules than the 8B layer.  Prefill of two prompts (768 rows)
    against sampled oracle rows and the whole K/V cache; one decode step of 16 requests."""
    shape = S.LLAMA70B
    lens = [500, 268]
    T, B = sum(lens), 16
    ctx = np.array([(97 * i + 40) % 1400 for i in range(B)], np.int32)
    counts = [int(c) + 1 for c in ctx] + lens
    n_blocks = sum(S.blocks_for(c) for c in counts) + 16
    tabs = S.shuffled_block_tables(counts, n_blocks, max_blk=S.blocks_for(max(counts)))
    dtab, ptab = tabs[:B], tabs[B:]
    rig = Rig(shape, n_blocks, T, B, int(ctx.max()) + 1, sentinel=0x7FC1)
    try:
        L = rig.olayers[0]
        xb = S.hidden_states(T, shape.d_model, stream=3)
        x = f32(xb)
        cu = [0, lens[0], T]
        rig.ctx.set_cu_split(160, 96)
        y_bits = rig.prefill(xb, cu, ptab)
        rows = np.array([0, 1, 31, 32, 255, 256, 499, 500, 501, 511, 512, 700, 767], np.int32)
        Kc, Vc = L.new_cache(n_blocks, fill=ORC_SENT)
        y_ref = L.prefill(x, cu, ptab, Kc, Vc, rows=rows)
        check_cache_against_oracle(rig, Kc, Vc, ORC_SENT)
        check_tensor("70B prefill y, sampled rows", f32(y_bits)[rows], y_ref, x[rows], 2, elem_mult=END_TO_END)
        kb, vb = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim)
        rig.load_pools_from_logical(kb, vb)
        db = S.hidden_states(B, shape.d_model, stream=51)
        yd = rig.decode(db, ctx, dtab)
        yd_ref = L.decode(f32(db), ctx, dtab, f32(kb), f32(vb))
        check_tensor("70B decode y, batch 16", f32(yd), yd_ref, f32(db), 2, elem_mult=END_TO_END)
    finally:
        rig.close()


def test_serving_steps_three_requests_async_matches_oracle():
    """rs_submit / rs_step with requests arriving at different steps, prefills running beside decode
    steps, steps enqueued without waiting (the host schedules step n+1 while step n runs) and a
    measured-style profile steering the split: every decode row equals the oracle's stack for the
    request rs_decode_batch_ids names, block growth included."""
    shape = S.TINY
    n_layers = 2
    prof = rs.Profile([4], [1024], [64, 128, 192], [[[900, 500, 300]]], [[2000]], slo_us=600)
    rig = Rig(shape, 40, 128, 4, 160, n_layers=n_layers, profile=prof)
    try:
        reqs = {1: (40, 4), 2: (70, 3), 3: (17, 5)}            # id -> (prompt tokens, tokens to generate)
        prompts = {i: S.hidden_states(p, shape.d_model, stream=100 + i) for i, (p, _) in reqs.items()}
        p_dev = {i: to_dev(b) for i, b in prompts.items()}
        arrive = {0: [1, 2], 3: [3]}
        d_out = torch.zeros((4, shape.d_model), dtype=torch.bfloat16, device="cuda")
        # oracle state per request: block ids as the allocator hands them out are read back from the library
        caches = {i: [L.new_cache(40) for L in rig.olayers] for i in reqs}
        prefilled, ctx_len, checked = set(), {}, 0
        splits = set()
        for step in range(40):
            for i in arrive.get(step, []):
                rig.ctx.submit(i, reqs[i][0], reqs[i][1], p_dev[i])
            x_bits = S.hidden_states(1, shape.d_model, stream=200 + step)
            x_dev = to_dev(np.repeat(x_bits, 4, axis=0))        # the same input row for every request of the step
            so = rig.ctx.step(x_dev, d_out, wait_decode=False)   # returns at once
            splits.add((so.prefill_cus, so.decode_cus))
            ids = rig.ctx.decode_batch_ids()
            assert len(ids) == so.decode_batch
            rig.ctx.sync(rs.RS_SIDE_DECODE)
            got = f32(to_bits(d_out))
            for row, i in enumerate(ids):
                if i not in prefilled:                           # first decode step of i: its prefill has completed
                    tabs = np.full((1, 10), -1, np.int32)
                    blk = rig.ctx.kv_alloc(i, reqs[i][0])        # no growth: returns the ids the request owns
                    tabs[0, :len(blk)] = blk
                    x = f32(prompts[i])
                    for l, L in enumerate(rig.olayers):
                        x = L.prefill(x, [0, reqs[i][0]], tabs, *caches[i][l])
                    prefilled.add(i); ctx_len[i] = reqs[i][0]
                tabs = np.full((1, 10), -1, np.int32)
                blk = rig.ctx.kv_alloc(i, ctx_len[i] + 1)        # the step grew the request to ctx+1 tokens already
                tabs[0, :len(blk)] = blk
                xr = f32(x_bits)
                for l, L in enumerate(rig.olayers):
                    xr = L.decode(xr, [ctx_len[i]], tabs, *caches[i][l])
                e = residual_err(got[row:row + 1], xr, f32(x_bits), roundings=4, layers=n_layers)
                assert e <= 1.0, (step, i, e)
                ctx_len[i] += 1; checked += 1
            if all(rig.ctx.request_state(i) == 5 for i in reqs) and step > 3:
                break
        assert checked == sum(o for _, o in reqs.values())
        assert all(rig.ctx.request_state(i) == 5 for i in reqs) and rig.ctx.kv_num_free() == 40
        assert len(splits) >= 2, splits                          # the manager did move the split
        print("splits used:", sorted(splits))
    finally:
        rig.close()


def test_long_context_decode_and_16k_prefill_mid_shape():
    """The long-context configuration's sizes on the mid shape: decode over contexts up to 32767 cached tokens
    (64 attention chunks, directly written cache, same bits on both sides) and a whole 16384-token prompt
    (128 query tiles), sampled rows against the oracle."""
    shape = S.MID
    ctx = np.array([8191, 8192, 20000, 32767, 3, 513], np.int32)
    B = len(ctx)
    T = 16384
    counts = [int(c) + 1 for c in ctx] + [T]
    n_blocks = sum(S.blocks_for(c) for c in counts) + 7
    tabs = S.shuffled_block_tables(counts, n_blocks, max_blk=S.blocks_for(max(counts)), stream=9)
    dtab, ptab = tabs[:B], tabs[B:B + 1]
    rig = Rig(shape, n_blocks, T, B, 32768, sentinel=0x7FC1)
    try:
        L = rig.olayers[0]
        kb, vb = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim, stream=3)
        rig.load_pools_from_logical(kb, vb)
        Kc, Vc = f32(kb), f32(vb)
        db = S.hidden_states(B, shape.d_model, stream=61)
        yd = rig.decode(db, ctx, dtab)
        yd_ref, taps = L.decode(f32(db), ctx, dtab, Kc, Vc, taps=True)
        check_tensor("long-context decode attention out", f32(rig.ctx.debug_read_workspace(rs.RS_SIDE_DECODE, 2, (B, shape.q_dim))),
                     taps["attn"], elem_mult=END_TO_END)
        check_tensor("long-context decode y", f32(yd), yd_ref, f32(db), 2, elem_mult=END_TO_END)
        # the 16384-token prompt overwrites its own blocks only (snapshot after the decode step's appends)
        kb, vb = rig.k_bits_logical(), rig.v_bits_logical()
        xb = S.hidden_states(T, shape.d_model, stream=62)
        y_bits = rig.prefill(xb, [0, T], ptab)
        rng = np.random.default_rng(5)
        rows = np.unique(np.concatenate([[0, 1, 127, 128, 8191, 8192, 16382, 16383], rng.integers(0, T, 24)])).astype(np.int32)
        Kp, Vp = L.new_cache(n_blocks, fill=ORC_SENT)
        y_ref = L.prefill(f32(xb), [0, T], ptab, Kp, Vp, rows=rows)
        check_tensor("16K prefill y, sampled rows", f32(y_bits)[rows], y_ref, f32(xb)[rows], 2, elem_mult=END_TO_END)
        # K/V written by the prompt: exactly its blocks, contents to tolerance
        kg, vg = rig.k_bits_logical(), rig.v_bits_logical()
        mine = np.zeros(n_blocks, bool)
        mine[ptab[0, :S.blocks_for(T)]] = True
        assert np.array_equal(kg[~mine], kb[~mine]) and np.array_equal(vg[~mine], vb[~mine])
        assert rel_err(f32(kg[mine]).reshape(-1, shape.head_dim), Kp[mine].reshape(-1, shape.head_dim)) <= TOL
        assert rel_err(f32(vg[mine]).reshape(-1, shape.head_dim), Vp[mine].reshape(-1, shape.head_dim)) <= TOL
    finally:
        rig.close()


def test_prefill_prompt_longer_than_the_kernel_s_lds_block_table_mid_shape():
    """A 33000-token prompt: more blocks (2063) than the 2048 ids the prefill attention kernel keeps in LDS, so the
    last key tiles take their block ids from the table in global memory, and a ragged last tile.  Sampled rows
    against the oracle, rows around the 32768-token boundary among them."""
    shape = S.MID
    T = 33000
    n_blocks = S.blocks_for(T) + 5
    ptab = S.shuffled_block_tables([T], n_blocks, max_blk=S.blocks_for(T), stream=14)
    rig = Rig(shape, n_blocks, T, 1, 33024)
    try:
        L = rig.olayers[0]
        xb = S.hidden_states(T, shape.d_model, stream=63)
        y_bits = rig.prefill(xb, [0, T], ptab)
        rng = np.random.default_rng(6)
        rows = np.unique(np.concatenate([[0, 63, 32703, 32767, 32768, 32769, 32831, 32832, 32960, 32998, 32999],
                                         rng.integers(0, T, 16)])).astype(np.int32)
        Kp, Vp = L.new_cache(n_blocks, fill=ORC_SENT)
        y_ref = L.prefill(f32(xb), [0, T], ptab, Kp, Vp, rows=rows)
        check_tensor("33000-token prefill y, sampled rows", f32(y_bits)[rows], y_ref, f32(xb)[rows], 2, elem_mult=END_TO_END)
        check_cache_against_oracle(rig, Kp, Vp, ORC_SENT)
    finally:
        rig.close()


def test_released_source_weights_are_not_read_again():
    """Wide shape (every GEMM qualifies for the packed-operand kernels): after rs_release_source_weights the
    caller's matrices are overwritten with NaN patterns; prefill (short and long pass) and decode still match."""
    shape = S.WIDE
    lens = [150, 40]
    cu, T, n_blocks, tabs, xb = _prefill_case(shape, lens, stream=11)
    rig = Rig(shape, n_blocks + 4, 256, 4, 256)
    try:
        rig.ctx.release_source_weights(0)
        for k in ("wqkv", "wo", "wg", "wu", "wd"):
            rig.wdev[0][k].view(torch.int16).fill_(0x7FC1)
        torch.cuda.synchronize()
        L = rig.olayers[0]
        Kc, Vc = L.new_cache(n_blocks + 4, fill=ORC_SENT)
        y = rig.prefill(xb, cu, tabs)
        y_ref = L.prefill(f32(xb), cu, tabs, Kc, Vc)
        check_tensor("prefill y after release (190 rows)", f32(y), y_ref, f32(xb), 2, elem_mult=END_TO_END)
        xs = S.hidden_states(40, shape.d_model, stream=12)
        one = tabs[1:2]
        ys = rig.prefill(xs, [0, 40], one)
        ys_ref = L.prefill(f32(xs), [0, 40], one, Kc, Vc)
        check_tensor("prefill y after release (40 rows)", f32(ys), ys_ref, f32(xs), 2, elem_mult=END_TO_END)
        db = S.hidden_states(2, shape.d_model, stream=13)
        ctx = np.array([150, 40], np.int32)
        yd = rig.decode(db, ctx, tabs)     # positions 150 and 40 fall inside the prompts' last blocks
        yd_ref = L.decode(f32(db), ctx, tabs, Kc, Vc)
        check_tensor("decode y after release", f32(yd), yd_ref, f32(db), 2, elem_mult=END_TO_END)
    finally:
        rig.close()
