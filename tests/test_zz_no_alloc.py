"""rs_decode_layer_noalloc (the entry point for callers that cannot allocate: its scratch is a static
device array of the library) against rs_decode_layer on the same inputs, through the C ABI: two calls in
a row, the second with a smaller input (fewer rows, shorter contexts -- another layout of the same array,
which still holds the first call's contents), then sizes beyond the array are refused."""
import numpy as np
import pytest
import torch

import paper_2601_11822_amd as rs
import rs_synth as S
from tests.gpu_util import Rig, to_bits, to_dev

pytestmark = pytest.mark.gpu


def _step(rig, fn, xb, ctx, tabs, max_ctx):
    x = to_dev(xb)
    y = torch.zeros_like(x)
    cl = torch.from_numpy(np.ascontiguousarray(ctx, dtype=np.int32)).cuda()
    tab = torch.from_numpy(np.ascontiguousarray(tabs, dtype=np.int32)).cuda()
    torch.cuda.synchronize()
    fn(0, x, y, cl, tab, tab.shape[1], x.shape[0], max_ctx)
    rig.ctx.sync(rs.RS_SIDE_DECODE)
    return to_bits(y)


def test_noalloc_decode_matches_decode_layer_twice_second_call_smaller():
    shape = S.MID
    ctx_big = np.array([(37 * i + 5) % 900 for i in range(40)], np.int32)
    ctx_small = np.array([3, 130, 64, 0, 511, 17, 300], np.int32)
    counts = [int(c) + 1 for c in ctx_big]
    for i, c in enumerate(ctx_small):       # the same table rows serve both calls
        counts[i] = max(counts[i], int(c) + 1)
    n_blocks = sum(S.blocks_for(c) for c in counts) + 8
    tabs = S.shuffled_block_tables(counts, n_blocks, stream=4)
    rig = Rig(shape, n_blocks, 16, 40, 1024, with_oracle=False)
    try:
        kb, vb = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim, stream=2)
        for ctx, stream in ((ctx_big, 70), (ctx_small, 71)):
            B = len(ctx)
            xb = S.hidden_states(B, shape.d_model, stream=stream)
            max_ctx = int(ctx.max()) + 1
            rig.load_pools_from_logical(kb, vb)
            want = _step(rig, rig.ctx.decode_layer, xb, ctx, tabs[:B], max_ctx)
            k_want, v_want = to_bits(rig.k_pool), to_bits(rig.v_pool)
            rig.load_pools_from_logical(kb, vb)
            got = _step(rig, rig.ctx.decode_layer_noalloc, xb, ctx, tabs[:B], max_ctx)
            assert np.isfinite(S.bf16_bits_to_f32(got)).all()
            assert np.array_equal(got, want), f"batch {B}: output differs from rs_decode_layer"
            assert np.array_equal(to_bits(rig.k_pool), k_want) and np.array_equal(to_bits(rig.v_pool), v_want)
    finally:
        rig.close()


def test_noalloc_decode_refuses_what_does_not_fit_the_static_array():
    # Llama-3-8B-shaped layer: batch 64 over contexts up to 4096 fits the 32 MiB array, contexts up to 32768 do not
    shape = S.LLAMA8B
    B = 64
    n_blocks = 64
    rig = Rig(shape, n_blocks, 16, B, 32768, with_oracle=False)
    try:
        x = torch.zeros((B, shape.d_model), dtype=torch.bfloat16, device="cuda")
        cl = torch.zeros(B, dtype=torch.int32, device="cuda")
        tab = torch.zeros((B, 2048), dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        with pytest.raises(rs.RapidServeError) as e:
            rig.ctx.decode_layer_noalloc(0, x, x.clone(), cl, tab, 2048, B, 32768)
        assert e.value.code == rs.RS_ERR_BAD_ARG and "static" in str(e.value)
        rig.ctx.decode_layer_noalloc(0, x, x.clone(), cl, tab, 2048, B, 4096)    # fits
        rig.ctx.sync(rs.RS_SIDE_DECODE)
    finally:
        rig.close()
