"""GPU parity of the hybrid batch (chunked prefill co-batched with decode rows, section 3.1): chunk rows
against the oracle's chunked prefill, decode rows against the oracle's decode step, cache slots exact."""
import numpy as np
import pytest

import paper_2601_11822_amd as rs
import rs_synth as S
from tests.gpu_util import END_TO_END, TOL, Rig, check_cache_against_oracle, check_tensor, rel_err

pytestmark = pytest.mark.gpu

ORC_SENT = np.float32(-777.0)
f32 = S.bf16_bits_to_f32


def _chunk_schedule(lens, chunk):
    """Per step: (request indices, starts, lengths): every unfinished prompt advances by `chunk` tokens."""
    steps, done = [], [0] * len(lens)
    while any(d < n for d, n in zip(done, lens)):
        idx = [i for i, (d, n) in enumerate(zip(done, lens)) if d < n]
        st = [done[i] for i in idx]
        ln = [min(chunk, lens[i] - done[i]) for i in idx]
        steps.append((idx, st, ln))
        for i, l in zip(idx, ln):
            done[i] += l
    return steps


@pytest.mark.parametrize("shape_name,lens,chunk", [("TINY", [200, 77], 64), ("MID", [300, 130, 16], 128),
                                                   ("WIDE", [272], 144)])
def test_chunked_prefill_matches_oracle_chunks_and_whole_prefill(shape_name, lens, chunk):
    shape = getattr(S, shape_name)
    n_blocks = sum(S.blocks_for(n) for n in lens) + 3
    tabs = S.shuffled_block_tables(lens, n_blocks, stream=3)
    cu_all = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    xb_all = S.hidden_states(int(cu_all[-1]), shape.d_model, stream=3)
    rig = Rig(shape, n_blocks, sum(lens), 4, max(lens) + 1)
    try:
        L = rig.olayers[0]
        Kc, Vc = L.new_cache(n_blocks, fill=ORC_SENT)
        y_chunked = np.zeros((int(cu_all[-1]), shape.d_model), np.float32)
        for idx, st, ln in _chunk_schedule(lens, chunk):
            rows = np.concatenate([np.arange(cu_all[i] + s, cu_all[i] + s + l) for i, s, l in zip(idx, st, ln)])
            cu = np.concatenate([[0], np.cumsum(ln)]).astype(np.int32)
            xb = xb_all[rows]
            y_bits = rig.hybrid(xb, cu, st, tabs[idx])
            y_ref = L.prefill_chunk(f32(xb), cu, st, tabs[idx], Kc, Vc)
            print("chunk", shape.name, idx, st, ln)
            check_tensor("chunk rows y", f32(y_bits), y_ref, f32(xb), 2, elem_mult=END_TO_END)
            y_chunked[rows] = f32(y_bits)
        check_cache_against_oracle(rig, Kc, Vc, ORC_SENT)
        # the chunked sequence computes what one whole prefill computes (section 3.1: chunking changes the
        # schedule, not the result)
        Kw, Vw = L.new_cache(n_blocks, fill=ORC_SENT)
        y_whole = L.prefill(f32(xb_all), cu_all, tabs, Kw, Vw)
        check_tensor("chunked y against the whole prefill", y_chunked, y_whole, f32(xb_all), 2, elem_mult=END_TO_END)
    finally:
        rig.close()


def _hybrid_case(shape, chunk_lens, chunk_starts, ctx, rig_rows=None):
    """Prompts whose first chunk_starts[r] tokens are cached by an ordinary prefill, decode requests with
    ctx tokens cached; then one hybrid batch.  Checks both row kinds and the cache."""
    ctx = np.asarray(ctx, np.int32)
    B = len(ctx)
    plen = [s + l for s, l in zip(chunk_starts, chunk_lens)]
    counts = plen + [int(c) + 1 for c in ctx]
    n_blocks = sum(S.blocks_for(c) for c in counts) + 4
    tabs = S.shuffled_block_tables(counts, n_blocks, stream=9)
    ptab, dtab = tabs[:len(plen)], tabs[len(plen):]
    T = sum(chunk_lens)
    rig = Rig(shape, n_blocks, max(T + B, sum(chunk_starts), int(ctx.sum()), 1), max(B, 1), max(max(counts), 2))
    try:
        L = rig.olayers[0]
        Kc, Vc = L.new_cache(n_blocks, fill=ORC_SENT)
        # earlier context of the prompts and of the decode requests: ordinary prefill calls
        for tab, lens, stream in ((ptab, chunk_starts, 60), (dtab, [int(c) for c in ctx], 61)):
            keep = [i for i, n in enumerate(lens) if n > 0]
            if keep:
                cu = np.concatenate([[0], np.cumsum([lens[i] for i in keep])]).astype(np.int32)
                xb = S.hidden_states(int(cu[-1]), shape.d_model, stream=stream)
                rig.prefill(xb, cu, tab[keep])
                L.prefill(f32(xb), cu, tab[keep], Kc, Vc)
        cu = np.concatenate([[0], np.cumsum(chunk_lens)]).astype(np.int32)
        xb = S.hidden_states(T + B, shape.d_model, stream=62)
        y_bits = rig.hybrid(xb, cu, chunk_starts, ptab, ctx if B else None, dtab if B else None)
        x = f32(xb)
        y_chunk = L.prefill_chunk(x[:T], cu, chunk_starts, ptab, Kc, Vc)
        print("hybrid", shape.name, chunk_lens, chunk_starts, ctx.tolist())
        check_tensor("hybrid batch, chunk rows", f32(y_bits)[:T], y_chunk, x[:T], 2, elem_mult=END_TO_END)
        if B:
            y_dec = L.decode(x[T:], ctx, dtab, Kc, Vc)
            check_tensor("hybrid batch, decode rows", f32(y_bits)[T:], y_dec, x[T:], 2, elem_mult=END_TO_END)
        check_cache_against_oracle(rig, Kc, Vc, ORC_SENT)
        assert np.isfinite(f32(y_bits)).all()
    finally:
        rig.close()


def test_hybrid_batch_tiny_chunk_rows_and_decode_rows():
    _hybrid_case(S.TINY, [64, 40], [32, 0], [5, 0, 31, 16])


def test_hybrid_batch_mid_ragged_rows_share_a_row_tile():
    # 75 chunk rows: the decode rows start inside the chunk's last 32-row tile of the packed attention output
    _hybrid_case(S.MID, [75], [128], [200, 17, 64, 1, 300])


def test_hybrid_batch_of_at_most_64_rows_takes_the_weight_streaming_gemms():
    _hybrid_case(S.MID, [32], [64], [40, 90, 7])


def test_hybrid_batch_wide_large_tiles():
    _hybrid_case(S.WIDE, [256], [256], [100, 333, 48, 260, 15, 64, 1, 90])


def test_8b_hybrid_batch_chunk_512_after_1024_with_32_decode_rows_sampled():
    """The comparison system's own configuration (chunk 512, section 5.1) on the Llama-3-8B-shaped layer:
    a 512-token chunk at position 1024 of its prompt beside 32 decode rows, the caches written directly."""
    shape = S.LLAMA8B
    T, prior, B = 512, 1024, 32
    ctx = S.uniform_context_lengths(B, 512, 2048)
    counts = [prior + T] + [int(c) + 1 for c in ctx]
    n_blocks = sum(S.blocks_for(c) for c in counts) + 16
    tabs = S.shuffled_block_tables(counts, n_blocks, max_blk=S.blocks_for(max(counts)))
    ptab, dtab = tabs[:1], tabs[1:]
    rig = Rig(shape, n_blocks, T + B, B, int(max(counts)))
    try:
        L = rig.olayers[0]
        kb, vb = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim)
        rig.load_pools_from_logical(kb, vb)
        Kc, Vc = f32(kb), f32(vb)
        xb = S.hidden_states(T + B, shape.d_model, stream=70)
        x = f32(xb)
        y_bits = rig.hybrid(xb, [0, T], [prior], ptab, ctx, dtab)
        rng = np.random.default_rng(5)
        rows = np.unique(np.concatenate([[0, 1, 15, 16, 63, 64, 127, 128, 510, 511], rng.integers(0, T, 10)])).astype(np.int32)
        y_ref = L.prefill_chunk(x[:T], [0, T], [prior], ptab, Kc, Vc, rows=rows)
        check_tensor("8B hybrid, sampled chunk rows", f32(y_bits)[rows], y_ref, x[rows], 2, elem_mult=END_TO_END)
        y_dec = L.decode(x[T:], ctx, dtab, Kc, Vc)
        check_tensor("8B hybrid, decode rows", f32(y_bits)[T:], y_dec, x[T:], 2, elem_mult=END_TO_END)
        # slots written: the chunk's 512 positions and each decode request's next position, nothing else
        kg, vg = rig.k_bits_logical(), rig.v_bits_logical()
        changed = (kg != kb).any(axis=(2, 3)) | (vg != vb).any(axis=(2, 3))
        want = np.zeros_like(changed)
        pos = np.arange(prior, prior + T)
        want[ptab[0, pos // 16], pos % 16] = True
        for i, c in enumerate(ctx):
            want[dtab[i, c // 16], c % 16] = True
        assert np.array_equal(changed, want), "hybrid batch wrote K/V slots outside the chunk and the new tokens"
        assert rel_err(f32(kg)[want], Kc[want]) <= TOL and rel_err(f32(vg)[want], Vc[want]) <= TOL
    finally:
        rig.close()


def test_chunk_behind_32800_cached_tokens_reads_block_ids_past_the_kernels_lds_table_mid_shape():
    """A late chunk of a very long prompt: its rows attend to 32800 cached positions, more than the 2048 block ids
    the prefill attention kernel keeps in LDS, so the last key tiles (and the chunk's own blocks) take their ids
    from the table in memory; a ragged chunk length exercises the checked tile path at the end.  Cache written
    directly (same bits on both sides), every chunk row against the oracle."""
    shape = S.MID
    prior, T, B = 32800, 200, 3
    ctx = np.array([40, 700, 16], np.int32)
    counts = [prior + T] + [int(c) + 1 for c in ctx]
    n_blocks = sum(S.blocks_for(c) for c in counts) + 8
    tabs = S.shuffled_block_tables(counts, n_blocks, max_blk=S.blocks_for(max(counts)))
    ptab, dtab = tabs[:1], tabs[1:]
    rig = Rig(shape, n_blocks, T + B, B, prior + T, max_pos=prior + T)
    try:
        L = rig.olayers[0]
        kb, vb = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim)
        rig.load_pools_from_logical(kb, vb)
        Kc, Vc = f32(kb), f32(vb)
        xb = S.hidden_states(T + B, shape.d_model, stream=80)
        x = f32(xb)
        y_bits = rig.hybrid(xb, [0, T], [prior], ptab, ctx, dtab)
        y_ref = L.prefill_chunk(x[:T], [0, T], [prior], ptab, Kc, Vc)
        check_tensor("late chunk, all rows", f32(y_bits)[:T], y_ref, x[:T], 2, elem_mult=END_TO_END)
        y_dec = L.decode(x[T:], ctx, dtab, Kc, Vc)
        check_tensor("decode rows beside it", f32(y_bits)[T:], y_dec, x[T:], 2, elem_mult=END_TO_END)
        kg, vg = rig.k_bits_logical(), rig.v_bits_logical()
        changed = (kg != kb).any(axis=(2, 3)) | (vg != vb).any(axis=(2, 3))
        want = np.zeros_like(changed)
        pos = np.arange(prior, prior + T)
        want[ptab[0, pos // 16], pos % 16] = True
        for i, c in enumerate(ctx):
            want[dtab[i, c // 16], c % 16] = True
        assert np.array_equal(changed, want)
        assert rel_err(f32(kg)[want], Kc[want]) <= TOL and rel_err(f32(vg)[want], Vc[want]) <= TOL
    finally:
        rig.close()


def test_hybrid_layer_rejects_unaligned_chunk_start_and_oversized_batches():
    shape = S.TINY
    rig = Rig(shape, 8, 64, 2, 128, with_oracle=False)
    try:
        xb = S.hidden_states(48, shape.d_model, stream=1)
        tab = np.arange(4, dtype=np.int32)[None]
        with pytest.raises(rs.RapidServeError) as e:
            rig.hybrid(xb[:16], [0, 16], [8], tab)
        assert e.value.code == rs.RS_ERR_BAD_ARG
        with pytest.raises(rs.RapidServeError) as e:       # chunk runs past the block table
            rig.hybrid(xb[:32], [0, 32], [48], tab)
        assert e.value.code == rs.RS_ERR_BAD_BLOCK
        with pytest.raises(rs.RapidServeError) as e:       # more decode rows than max_decode_batch
            rig.hybrid(xb[:19], [0, 16], [0], tab, [1, 1, 1], np.zeros((3, 4), np.int32))
        assert e.value.code == rs.RS_ERR_BAD_ARG
    finally:
        rig.close()
