"""GPU tests of the captured decode step (rs_decode_layer_graph)."""
import numpy as np
import pytest
import torch

import paper_2601_11822_amd as rs
import rs_synth as S
from tests.gpu_util import Rig, to_bits, to_dev

pytestmark = pytest.mark.gpu


def test_graph_launch_keeps_the_cu_mask():
    """Section 4.5.3: a graph runs under the mask it was captured with.  The probe kernel replayed
    from a graph on each side's masked stream lands on exactly that side's compute units."""
    rig = Rig(S.TINY, 4, 16, 4, 64, with_oracle=False)
    try:
        for p, d in [(128, 128), (192, 64)]:
            rig.ctx.set_cu_split(p, d)
            for side, n in ((0, p), (1, d)):
                eager = set(np.nonzero(rig.ctx.debug_cu_histogram(side, 8192))[0])
                hist = rig.ctx.debug_cu_histogram_graph(side, 8192)
                assert hist.sum() == 8192
                graphed = set(np.nonzero(hist)[0])
                assert len(graphed) == n and graphed == eager, (p, d, side, len(graphed))
    finally:
        rig.close()


def test_graphed_decode_step_is_bit_identical_to_eager_over_replays():
    """The same graph replayed over several steps, with contexts growing in place (contents of
    ctx_lens / x_in change, pointers stay), eager work and synchronisations in between, a split
    change (new capture) and a concurrent prefill: every replay equals the eager call bit for bit,
    in the output and in the K/V it appended."""
    shape = S.MID
    B = 5
    ctx0 = np.array([30, 500, 511, 64, 700], np.int32)
    steps = 4
    bucket = 1024
    counts = [bucket] * B
    pre_T = 256
    n_blocks = sum(S.blocks_for(c) for c in counts) + S.blocks_for(pre_T) + 8
    tabs_all = S.shuffled_block_tables(counts + [pre_T], n_blocks, stream=7)
    tabs, ptab = tabs_all[:B], tabs_all[B:B + 1]
    kb_log, vb_log = S.kv_cache_bits(n_blocks, shape.n_kv_heads, shape.head_dim)
    pre_x = S.hidden_states(pre_T, shape.d_model, stream=71)
    xs = [S.hidden_states(B, shape.d_model, stream=80 + s) for s in range(steps)]

    def run(graphed):
        rig = Rig(shape, n_blocks, pre_T, B, bucket, with_oracle=False)
        outs = []
        try:
            rig.load_pools_from_logical(kb_log.copy(), vb_log.copy())
            x = to_dev(xs[0]); y = torch.empty_like(x)
            cl = torch.from_numpy(ctx0.copy()).cuda()
            tab = torch.from_numpy(np.ascontiguousarray(tabs, dtype=np.int32)).cuda()
            ptab_d = torch.from_numpy(np.ascontiguousarray(ptab, dtype=np.int32)).cuda()
            px = to_dev(pre_x); py = torch.empty_like(px)
            c = rig.ctx
            for s in range(steps):
                if s == 2:
                    c.set_cu_split(192, 64)                      # new stream: a new capture under the new mask
                x.copy_(to_dev(xs[s]))
                cl.copy_(torch.from_numpy(ctx0 + s).cuda())
                torch.cuda.synchronize()
                if s % 2 == 1:
                    c.prefill_layer(0, px, py, [0, pre_T], ptab_d, tab.shape[1])     # runs beside the decode step
                if graphed:
                    c.decode_layer_graph(0, x, y, cl, tab, tab.shape[1], B, bucket)
                else:
                    c.decode_layer(0, x, y, cl, tab, tab.shape[1], B, int((ctx0 + s).max()) + 1)
                c.sync(rs.RS_SIDE_DECODE); c.sync(rs.RS_SIDE_PREFILL)
                outs.append(to_bits(y).copy())
            outs.append(rig.k_bits_logical().copy()); outs.append(rig.v_bits_logical().copy())
        finally:
            rig.close()
        return outs

    eager, graphed = run(False), run(True)
    assert len(eager) == len(graphed)
    for i, (a, b) in enumerate(zip(eager, graphed)):
        assert np.array_equal(a, b), f"item {i} differs between the eager and the graphed decode step"


def test_graph_bucket_is_validated():
    rig = Rig(S.TINY, 16, 16, 2, 1024, with_oracle=False)
    try:
        x = to_dev(S.hidden_states(2, S.TINY.d_model, stream=5)); y = torch.empty_like(x)
        cl = torch.zeros(2, dtype=torch.int32, device="cuda")
        tab = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
        with pytest.raises(rs.RapidServeError):
            rig.ctx.decode_layer_graph(0, x, y, cl, tab, 4, 2, 100)        # not a multiple of the chunk
        with pytest.raises(rs.RapidServeError):
            rig.ctx.decode_layer_graph(0, x, y, cl, tab, 4, 2, 512)        # 4 table entries cover 64 tokens only
        rig.ctx.sync(rs.RS_SIDE_DECODE)
    finally:
        rig.close()
