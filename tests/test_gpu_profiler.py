"""GPU tests of the offline profiler and of the event-completion query it paces itself with."""
import json

import numpy as np
import pytest

import paper_2601_11822_amd as rs
import rs_synth as S
from oracle.manager import Profile as OProfile, choose_split as o_choose

pytestmark = pytest.mark.gpu


def test_profiler_table_feeds_the_manager(tmp_path):
    """A small sweep on the mid-size shape: the table has the declared layout, every latency is a
    positive finite number, decode beside a prefill is never faster than decode alone on the same
    partition by more than noise, and the manager (through the C ABI) makes the choices the exact
    integer definition makes on the measured table."""
    from paper_2601_11822_amd import profiler
    shape = S.MID
    be, ce, dc = [4, 16], [1024, 8192], [64, 128, 192]
    rig = profiler.Rig(shape, be, ce, prefill_tokens=512, max_context=2049)
    d = profiler.profile(rig, be, ce, dc, n_layers=8, steps=6, warmup=2)
    lat = np.array(d["lat_distinct_us"]); over = np.array(d["lat_over_us"])
    assert lat.shape == (2, 2, 3) and over.shape == (2, 2)
    assert (lat > 0).all() and (over > 0).all() and lat.max() < 10_000_000
    for rec in d["curves"]:
        for s in rec["splits"]:
            assert s["itl_ms"] > 0.7 * s["decode_alone_ms"], rec
            assert s["prefill_ms"] > 0.7 * s["prefill_alone_ms"], rec
    # markdown and JSON round trip
    p = tmp_path / "prof.json"
    p.write_text(json.dumps(d))
    assert "decode CUs" in profiler.to_markdown(d)
    for slo in (int(lat.min()) - 1, int(np.median(lat)), int(max(lat.max(), over.max())) + 1):
        prof = profiler.load_profile(str(p), slo_us=slo)
        host = rs.Context.from_shape(shape, max_pos=16, n_blocks=4, profile=prof, device=rs.RS_HOST_ONLY)
        oprof = OProfile(be, ce, dc, lat.tolist(), over.tolist())
        for batch in (1, 4, 9, 16, 40):
            for sum_ctx in (10, 1024, 5000, 8192, 100000):
                for pending in (False, True):
                    assert host.choose_split(batch, sum_ctx, pending) == o_choose(batch, sum_ctx, pending, oprof, slo)
        host.destroy()
    rig.c.destroy()


def test_mark_done_follows_completion():
    from tests.gpu_util import Rig
    rig = Rig(S.TINY, n_blocks=8, max_prefill_tokens=16, max_decode_batch=2, max_context=32, with_oracle=False)
    try:
        c = rig.ctx
        with pytest.raises(rs.RapidServeError):
            c.mark_done(0, 77)           # never recorded
        c.mark(0, 5)
        c.sync(0)
        assert c.mark_done(0, 5) is True
    finally:
        rig.close()
