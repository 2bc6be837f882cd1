"""CPU tests through the C ABI: the library loads, exports what the header declares, and its
host logic (allocator, split validation, manager, request state machine) matches the integer
oracles.  No GPU call is made: contexts are RS_HOST_ONLY."""
import os
import re

import numpy as np
import pytest

import paper_2601_11822_amd as rs
import rs_synth as S
from oracle.kv_alloc import KVAllocator, NoBlocks
from oracle.manager import Profile as OProfile, choose_split as o_choose

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def host_ctx(n_blocks=64, profile=None, max_decode_batch=8, max_context=4096, shape=S.TINY):
    return rs.Context.from_shape(shape, max_pos=8192, n_blocks=n_blocks, max_prefill_tokens=4096,
                                 max_decode_batch=max_decode_batch, max_context=max_context,
                                 profile=profile, device=rs.RS_HOST_ONLY)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "rapid_serve.h")).read()
    declared = set(re.findall(r"\b(rs_[a-z_0-9]+)\s*\(", hdr))
    declared -= {"rs_ctx"}
    lib = rs.load()
    assert declared, "no declarations found"
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in the header but not exported"
    assert set(rs.EXPORTS) == declared


def test_header_constants_match_binding():
    hdr = open(os.path.join(ROOT, "include", "rapid_serve.h")).read()
    for name in ("RS_TOTAL_CUS", "RS_CU_GRANULE", "RS_KV_BLOCK", "RS_MAX_PREFILL_REQS", "RS_MAX_MARKS",
                 "RS_CU_HIST_BINS", "RS_N_KERNEL_SLOTS"):
        v = int(re.search(rf"#define {name}\s+\(?(-?\d+)", hdr).group(1))
        assert getattr(rs, name) == v


def test_init_rejects_bad_shapes():
    with pytest.raises(rs.RapidServeError) as e:
        rs.Context(256, 4, 4, 48, 688, 1, 1e-5, 1e4, 128, 8, device=rs.RS_HOST_ONLY)
    assert e.value.code == rs.RS_ERR_BAD_ARG
    with pytest.raises(rs.RapidServeError):
        rs.Context(256, 6, 4, 64, 688, 1, 1e-5, 1e4, 128, 8, device=rs.RS_HOST_ONLY)
    with pytest.raises(rs.RapidServeError):
        rs.Context(250, 4, 4, 64, 688, 1, 1e-5, 1e4, 128, 8, device=rs.RS_HOST_ONLY)


def test_layer_calls_fail_loudly_without_gpu():
    c = host_ctx()
    with pytest.raises(rs.RapidServeError) as e:
        c.prefill_layer(0, 1, 1, [0, 4], 1, 1)
    assert e.value.code == rs.RS_ERR_STATE


def test_allocator_matches_oracle_on_random_trace():
    rng = np.random.default_rng(7)
    c = host_ctx(n_blocks=40)
    o = KVAllocator(40)
    tokens = {}
    for step in range(400):
        r = int(rng.integers(0, 8))
        if r in tokens and rng.random() < 0.25:
            c.kv_free(r); o.release(r); del tokens[r]
            continue
        n = tokens.get(r, 0) + int(rng.integers(1, 60))
        try:
            want = o.alloc(r, n)
        except NoBlocks:
            with pytest.raises(rs.RapidServeError) as e:
                c.kv_alloc(r, n)
            assert e.value.code == rs.RS_ERR_NO_BLOCKS
            assert c.kv_num_free() == o.n_free()
            continue
        got = c.kv_alloc(r, n)
        assert got.tolist() == want and len(got) == (n + 15) // 16
        tokens[r] = n
        assert c.kv_num_free() == o.n_free()


def test_alloc_cap_too_small_changes_nothing():
    c = host_ctx(n_blocks=8)
    with pytest.raises(rs.RapidServeError) as e:
        c.kv_alloc(1, 100, cap=2)
    assert e.value.code == rs.RS_ERR_BAD_ARG and c.kv_num_free() == 8


def test_split_validation():
    c = host_ctx()
    assert c.get_cu_split() == (256, 256)
    c.set_cu_split(64, 192); assert c.get_cu_split() == (64, 192)
    c.set_cu_split(0, 256); c.set_cu_split(256, 0); c.set_cu_split(32, 32); c.set_cu_split(256, 256)
    for bad in [(64, 224), (100, 100), (-32, 64), (288, 0), (256, 32), (33, 64)]:
        with pytest.raises(rs.RapidServeError) as e:
            c.set_cu_split(*bad)
        assert e.value.code == rs.RS_ERR_BAD_SPLIT
    assert c.get_cu_split() == (256, 256)


def test_masks_are_disjoint_balanced_nested_and_right_sized():
    """Section 4.2.  Mask bit b is unit b // 8 of XCD b % 8, and unit j of an XCD sits in shader engine j % 4:
    a side must hold the same units in every XCD and equally many in each of the four engines (workgroups are
    dealt to the engines in turn), and a side's masks must be nested, so that a side that shrinks while the other
    side's previous pass is still running never lands on that pass's units."""
    c = host_ctx()
    prev_p, masks_d = 0, []
    for p in range(0, 257, 32):
        d = 256 - p
        c.set_cu_split(p, d)
        mp = int.from_bytes(c.get_cu_mask(0).tobytes(), "little")
        md = int.from_bytes(c.get_cu_mask(1).tobytes(), "little")
        assert bin(mp).count("1") == p and bin(md).count("1") == d
        assert mp & md == 0 and (mp | md) == (1 << 256) - 1
        for m, n in ((mp, p), (md, d)):
            units = [sorted(j for j in range(32) if (m >> (8 * j + x)) & 1) for x in range(8)]
            assert all(u == units[0] for u in units) and len(units[0]) == n // 8     # the same units in every XCD
            per_se = [sum(1 for j in units[0] if j % 4 == se) for se in range(4)]
            assert per_se == [n // 32] * 4, f"uneven engines {per_se} at {n} CUs"
        assert mp & prev_p == prev_p                       # prefill masks grow by adding units
        assert all(larger & md == md for larger in masks_d[-1:])    # decode masks shrink by dropping units
        prev_p = mp
        masks_d.append(md)
    c.set_cu_split(256, 256)
    assert int.from_bytes(c.get_cu_mask(0).tobytes(), "little") == (1 << 256) - 1


def _profiles():
    cus = [32, 64, 96, 128, 160, 192, 224]
    be, ce = [8, 64, 256], [10_000, 100_000, 1_000_000]
    rng = np.random.default_rng(3)
    lat = np.sort(rng.integers(200, 90_000, size=(3, 3, 7)), axis=2)[:, :, ::-1].copy()
    over = rng.integers(200, 90_000, size=(3, 3))
    return cus, be, ce, lat, over


def test_manager_matches_oracle_everywhere():
    cus, be, ce, lat, over = _profiles()
    for slo in (1_000, 20_000, 50_000, 100_000):
        c = host_ctx(profile=rs.Profile(be, ce, cus, lat, over, slo))
        op = OProfile(be, ce, cus, lat.tolist(), over.tolist())
        for b in (0, 1, 8, 9, 64, 65, 300):
            for sc in (0, 9_999, 10_000, 10_001, 500_000, 5_000_000):
                for pend in (False, True):
                    assert c.choose_split(b, sc, pend) == o_choose(b, sc, pend, op, slo), (slo, b, sc, pend)


def test_manager_without_profile_over_allocates():
    c = host_ctx()
    assert c.choose_split(4, 100, True) == (256, 256)
    assert c.choose_split(4, 100, False) == (0, 256)
    assert c.choose_split(0, 0, True) == (256, 0)


def test_request_flow_state_machine():
    """Section 4.4: blocks first, then prefill, notification, then the decode batch; FCFS."""
    WAITING, READY, PREFILLING, DONE, RUNNING, FINISHED = range(6)
    c = host_ctx(n_blocks=12, max_decode_batch=2, max_context=256)
    c.submit(10, 100, 3)      # 7 blocks
    c.submit(11, 60, 2)       # 4 blocks
    c.submit(12, 40, 2)       # 3 blocks: does not fit until something is freed
    so = c.step()
    assert (c.request_state(10), c.request_state(11), c.request_state(12)) == (PREFILLING, READY, WAITING)
    assert so.prefill_started_req == 10 and so.prefill_started_tokens == 100 and so.n_waiting == 1
    assert (so.prefill_cus, so.decode_cus) == (256, 0) and so.decode_batch == 0
    # no notification yet: nothing may join the decode batch, no second prefill may start
    so = c.step()
    assert c.request_state(10) == PREFILLING and so.decode_batch == 0 and so.prefill_started_req == -1
    with pytest.raises(rs.RapidServeError):
        c.debug_complete_prefill(11)          # not prefilling
    c.debug_complete_prefill(10)
    so = c.step()
    assert c.request_state(10) == RUNNING and so.n_promoted == 1 and so.decode_batch == 1
    assert so.decode_sum_ctx == 100 and so.prefill_started_req == 11
    assert (so.prefill_cus, so.decode_cus) == (256, 256)        # no profile: over-allocation
    c.debug_complete_prefill(11)
    so = c.step()                                                # 10 step 2, 11 step 1
    assert so.decode_batch == 2 and so.decode_sum_ctx == 101 + 60
    assert c.decode_batch_ids() == [10, 11]                      # row order = promotion order
    assert c.request_state(12) == WAITING                        # 12 blocks all in use (7 + 4 + growth)
    assert (so.prefill_cus, so.decode_cus) == (0, 256)           # no prefill pending -> decode takes all
    so = c.step()                                                # 10 step 3, 11 step 2
    so = c.step()                                                # both retire, 12 gets blocks and starts
    assert so.n_finished == 2 and c.request_state(10) == FINISHED and c.request_state(11) == FINISHED
    assert c.request_state(12) == PREFILLING and so.decode_batch == 0 and c.decode_batch_ids() == []
    c.debug_complete_prefill(12)
    c.step(); c.step()
    so = c.step()
    assert c.request_state(12) == FINISHED and c.kv_num_free() == 12


def test_decode_batch_cap_and_fcfs_promotion():
    c = host_ctx(n_blocks=64, max_decode_batch=1, max_context=256)
    for i in range(3):
        c.submit(i, 20, 2)
    c.step(); c.debug_complete_prefill(0)
    c.step(); c.debug_complete_prefill(1)      # 0 runs, 1 prefilling -> done
    so = c.step()                              # cap 1: request 1 stays PREFILL_DONE
    assert c.request_state(0) == 4 and c.request_state(1) == 3 and so.decode_batch == 1
    c.debug_complete_prefill(2)
    so = c.step()                              # 0 retires; 1 (older) is promoted before 2
    assert c.request_state(0) == 5 and c.request_state(1) == 4 and c.request_state(2) == 3


def test_operand_layouts_shared_by_host_and_kernels(tmp_path):
    """packed_offset / packed_mt / kpool_chunk_offset are bijections with the fragment structure the
    kernels assume; checked on the host by a small program compiled against the kernels' own header."""
    import shutil
    import subprocess
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "host_layout_check.hip")
    exe = str(tmp_path / "host_layout_check")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", src, "-o", exe], check=True,
                   stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr


def test_release_source_weights_only_where_the_packed_copies_suffice():
    c = host_ctx(shape=S.LLAMA8B)
    with pytest.raises(rs.RapidServeError) as e:
        c.release_source_weights(0)                      # weights not set yet
    assert e.value.code == rs.RS_ERR_STATE
    c.set_weights(0, 1, 1, 1, 1, 1, 1, 1)
    c.release_source_weights(0)
    with pytest.raises(rs.RapidServeError):
        c.release_source_weights(3)                      # layer out of range
    t = host_ctx(shape=S.TINY)                           # N < 1024: the generic kernel still reads them
    t.set_weights(0, 1, 1, 1, 1, 1, 1, 1)
    with pytest.raises(rs.RapidServeError) as e:
        t.release_source_weights(0)
    assert e.value.code == rs.RS_ERR_STATE


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py with --gpus above 1 exits with a message that says so, before touching a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "ONE GPU" in (p.stderr + p.stdout)


def test_bench_traffic_constants_are_the_profile_totals():
    """The `traffic` fields of the bench line are stored counter totals: they must be the ones the committed
    counter summary ends with, so that the two cannot drift apart when the profile is taken again."""
    import importlib.util
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "profiles", "hbm_traffic_alone_256cu_llama8b_layer.md")).read()
    m = re.search(r"`roofline\.traffic` = (\d+) and `roofline_decode\.traffic` = (\d+) bytes", text)
    assert m, "the summary no longer states the two totals"
    spec = importlib.util.spec_from_file_location("bench_for_constants", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    assert int(bench.TRAFFIC_BYTES["gateup"]) == int(m.group(1))
    assert int(bench.TRAFFIC_BYTES["decode_attn"]) == int(m.group(2))
