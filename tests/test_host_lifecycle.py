"""Closed-loop request life cycle on the CPU: pins of the integer oracle (`oracle/lifecycle.py`), then
the library's state machine (host-only context, sampled tokens injected) against it on random traces."""
import numpy as np
import pytest

import paper_2601_11822_amd as rs
import rs_synth as S
from oracle.kv_alloc import NoBlocks
from oracle.lifecycle import FINISHED, Lifecycle

EOS = 7


def _trace(seed, n_req=14, max_prompt=60, max_new=30, vocab=40):
    g = np.random.default_rng(seed)
    reqs = []
    for i in range(n_req):
        pl = int(g.integers(1, max_prompt + 1))
        mn = int(g.integers(1, max_new + 1))
        script = [int(t) for t in g.integers(0, vocab, size=mn + 4)]
        reqs.append((100 + i, pl, mn, script, int(g.integers(0, 12)), ))
    delays = [int(d) for d in g.integers(0, 3, size=400)]
    return reqs, delays


def _expected_output(script, max_new, eos):
    out = []
    for t in script:
        out.append(t)
        if t == eos or len(out) >= max_new:
            break
    return out


def _drive(sim_submit, sim_step, sim_complete, reqs, delays, max_steps=2000):
    """Submits each request at its arrival step, completes each prefill `delay` steps after it started."""
    log, due = [], {}
    todo = sorted(reqs, key=lambda r: r[4])
    n_done, step = 0, 0
    while n_done < len(reqs) and step < max_steps:
        while todo and todo[0][4] <= step:
            rid, pl, mn, script, _ = todo.pop(0)
            sim_submit(rid, pl, mn, script)
        for rid in [r for r, s in due.items() if s <= step]:
            sim_complete(rid)
            del due[rid]
        o = sim_step()
        log.append(o)
        n_done += o["n_finished"]
        if o["prefill_started_req"] >= 0:
            due[o["prefill_started_req"]] = step + 1 + delays[step % len(delays)]
        step += 1
    assert n_done == len(reqs), "trace did not drain"
    return log


# ------------------------------------------------------------------------- pins of the oracle
@pytest.mark.parametrize("n_blocks,seed", [(1000, 1), (12, 2), (8, 3), (7, 4)])
def test_oracle_outputs_are_script_prefixes_and_blocks_return(n_blocks, seed):
    reqs, delays = _trace(seed)
    lc = Lifecycle(n_blocks, max_batch=4, eos=EOS)
    held_max = 0

    def step():
        nonlocal held_max
        o = lc.step()
        held_max = max(held_max, n_blocks - lc.alloc.n_free())
        # every running request owns exactly the blocks its cached tokens need (ctx counts this step's token)
        for rid in lc.running:
            assert len(lc.alloc.owned[rid]) == -(-lc.reqs[rid].ctx // 16)
        ids = [b for v in lc.alloc.owned.values() for b in v]
        assert len(ids) == len(set(ids)) and len(ids) + lc.alloc.n_free() == n_blocks
        assert o["decode_batch"] <= 4
        return o

    log = _drive(lambda rid, pl, mn, sc: lc.submit(rid, pl, mn, sc), step, lc.complete_prefill, reqs, delays)
    for rid, pl, mn, script, _ in reqs:
        assert lc.reqs[rid].state == FINISHED
        assert lc.reqs[rid].out == _expected_output(script, mn, EOS)
    assert lc.alloc.n_free() == n_blocks and held_max <= n_blocks
    n_pre = sum(o["n_preempted"] for o in log)
    if n_blocks == 1000:
        assert n_pre == 0
        # ample pool: prompts are prefilled in arrival order, each exactly once, whole
        passes = [o for o in log if o["prefill_started_req"] >= 0]
        order = [r[0] for r in sorted(reqs, key=lambda r: r[4])]
        assert [rid for o in passes for rid in o["prefill_started_ids"]] == order
        plen = {r[0]: r[1] for r in reqs}
        assert all(o["prefill_started_tokens"] == sum(plen[rid] for rid in o["prefill_started_ids"]) for o in passes)
        assert any(o["prefill_started_count"] > 1 for o in passes)
    else:
        assert n_pre > 0


def test_oracle_preemption_worked_example():
    # Pool of 4 blocks; A and B have 16-token prompts (1 block each) and produce 40 tokens each.
    # They arrive together, so one prefill pass covers both (32 tokens) and they decode in lock
    # step from step 1: context 16 + k after step k.  Both need a 2nd block for their first decode
    # token (position 16) -> pool full.  At step 17 both sit at position 32 and need a 3rd block:
    # A (first in line) is starved, B (arrived last) is preempted.  By then B has 1 (prefill) + 16
    # (steps 1..16) = 17 tokens, so its recomputation covers 16 + 17 = 33 tokens.
    lc = Lifecycle(4, max_batch=4, eos=-1)
    lc.submit(1, 16, 40, list(range(100, 140)))
    lc.submit(2, 16, 40, list(range(200, 240)))
    log, started = [], []
    for _ in range(200):
        o = lc.step()
        log.append(o)
        if o["prefill_started_req"] >= 0:
            started.append((o["prefill_started_req"], o["prefill_started_tokens"], o["prefill_started_count"]))
            lc.complete_prefill(o["prefill_started_req"])
        if lc.reqs[1].state == FINISHED and lc.reqs[2].state == FINISHED:
            break
    assert sum(o["n_preempted"] for o in log) == 1
    assert started == [(1, 32, 2), (2, 33, 1)]
    assert [i for i, o in enumerate(log) if o["n_preempted"]] == [17]
    assert lc.reqs[1].out == list(range(100, 140)) and lc.reqs[2].out == list(range(200, 240))


def test_oracle_pool_too_small_for_one_request():
    lc = Lifecycle(2, max_batch=2)
    lc.submit(1, 30, 20)
    with pytest.raises(NoBlocks):
        for _ in range(40):
            o = lc.step()
            if o["prefill_started_req"] >= 0:
                lc.complete_prefill(1)


# ------------------------------------------------------------------ the library against the oracle
# ------------------------------------------------------------ pins of the oracle, hybrid batching
def test_oracle_hybrid_worked_example():
    # Budget 32 prompt tokens per step.  A (prompt 40, 3 tokens), B (prompt 10, 2 tokens) and C (prompt 50, 1
    # token) arrive together.
    # step 0: A[0,32).                      step 1: A[32,40) ends A, B[0,10) ends B, 14 left: C[0,0)? no -- a part
    #         that is not the end of its prompt is a multiple of 16, and 14 rounds to 0: C waits.
    # step 2: A's and B's first tokens are seen, both join the batch (decode batch 2); C[0,32).
    # step 3: A's 2nd and B's 2nd token: B ends; decode batch 1 (A); C[32,50) ends C.
    # step 4: A's 3rd token ends A; C's first token ends C (1 token).  Nothing left.
    lc = Lifecycle(100, max_batch=4, eos=-1, hybrid_chunk=32)
    lc.submit(1, 40, 3, [5, 6, 7, 8])
    lc.submit(2, 10, 2, [9, 10, 11])
    lc.submit(3, 50, 1, [12, 13])
    log = [lc.step() for _ in range(5)]
    assert [o["chunks"] for o in log] == [[(1, 0, 32)], [(1, 32, 8), (2, 0, 10)], [(3, 0, 32)], [(3, 32, 18)], []]
    assert [o["decode_batch"] for o in log] == [0, 0, 2, 1, 0]
    assert [o["n_promoted"] for o in log] == [0, 0, 2, 0, 0]
    assert [o["n_finished"] for o in log] == [0, 0, 0, 1, 2]
    assert [o["prefill_started_req"] for o in log] == [1, 2, 3, -1, -1]
    assert [o["prefill_started_tokens"] for o in log] == [40, 10, 50, 0, 0]
    assert log[2]["decode_sum_ctx"] == 40 + 10 and log[3]["decode_sum_ctx"] == 41
    assert lc.reqs[1].out == [5, 6, 7] and lc.reqs[2].out == [9, 10] and lc.reqs[3].out == [12]
    assert lc.alloc.n_free() == 100


@pytest.mark.parametrize("n_blocks,seed,chunk", [(1000, 1, 16), (1000, 2, 32), (1000, 5, 96), (12, 2, 16), (8, 3, 48), (7, 4, 16)])
def test_oracle_hybrid_tokens_equal_the_other_policy_and_parts_tile_every_prefill(n_blocks, seed, chunk):
    reqs, delays = _trace(seed)
    lc = Lifecycle(n_blocks, max_batch=4, eos=EOS, hybrid_chunk=chunk)

    def step():
        o = lc.step()
        for rid in lc.running:
            assert len(lc.alloc.owned[rid]) == -(-lc.reqs[rid].ctx // 16)
        ids = [b for v in lc.alloc.owned.values() for b in v]
        assert len(ids) == len(set(ids)) and len(ids) + lc.alloc.n_free() == n_blocks
        return o

    log = _drive(lambda rid, pl, mn, sc: lc.submit(rid, pl, mn, sc), step, lambda rid: None, reqs, delays)
    # the tokens do not depend on the batching policy: the same script prefixes as under whole-prompt prefill
    for rid, pl, mn, script, _ in reqs:
        assert lc.reqs[rid].state == FINISHED and lc.reqs[rid].out == _expected_output(script, mn, EOS)
    assert lc.alloc.n_free() == n_blocks
    # every prefill (a preempted request has several) is covered by its parts exactly once, in order; a step's parts
    # stay within the budget, only the first may continue a prompt, and every part but a prompt's last is whole blocks
    cur = None                      # [request, tokens to prefill, tokens taken]
    started = []
    for o in log:
        assert sum(n for _, _, n in o["chunks"]) <= chunk
        new = list(zip(o.get("prefill_started_ids", []), o.get("prefill_started_lens", [])))
        started += [rid for rid, _ in new]
        assert o["prefill_started_count"] == len(new) and o["prefill_started_tokens"] == sum(n for _, n in new)
        for j, (rid, start, n) in enumerate(o["chunks"]):
            if cur is None:
                assert new and new[0][0] == rid and start == 0
                cur = [rid, new.pop(0)[1], 0]
            else:
                assert j == 0, "only a step's first part continues a prompt"
            assert rid == cur[0] and start == cur[2] and n >= 1
            cur[2] += n
            assert cur[2] <= cur[1]
            if cur[2] == cur[1]:
                cur = None
            else:
                assert n % 16 == 0
        assert not new, "a prompt was taken up without a part"
    assert cur is None
    if n_blocks == 1000:
        assert sum(o["n_preempted"] for o in log) == 0
        assert started == [r[0] for r in sorted(reqs, key=lambda r: r[4])]
        if chunk >= 96:
            assert any(len(o["chunks"]) > 1 for o in log)
    else:
        assert sum(o["n_preempted"] for o in log) > 0


def _host_ctx(n_blocks, max_batch, eos, max_prefill=4096):
    c = rs.Context.from_shape(S.TINY, max_pos=8192, n_blocks=n_blocks, max_prefill_tokens=max_prefill,
                              max_decode_batch=max_batch, max_context=4096, device=rs.RS_HOST_ONLY)
    c.set_head(None, None, None, vocab=64, eos_token=eos)
    return c


KEYS = ("n_promoted", "n_finished", "n_preempted", "n_waiting", "prefill_started_req", "prefill_started_tokens",
        "prefill_started_count", "decode_batch", "decode_sum_ctx")


@pytest.mark.parametrize("n_blocks,seed,budget", [(1000, 11, 4096), (12, 12, 4096), (8, 13, 4096), (7, 14, 100), (9, 15, 120),
                                                  (1000, 16, 100)])
def test_library_life_cycle_matches_oracle(n_blocks, seed, budget):
    reqs, delays = _trace(seed)
    lc = Lifecycle(n_blocks, max_batch=4, eos=EOS, max_prefill_tokens=budget)
    ref = _drive(lambda rid, pl, mn, sc: lc.submit(rid, pl, mn, sc), lc.step, lc.complete_prefill, reqs, delays)
    if budget < 4096:   # the budget binds somewhere, and is never exceeded by a pass of several prompts
        assert all(o["prefill_started_tokens"] <= budget for o in ref if o["prefill_started_count"] > 1)
        assert any(o["prefill_started_count"] > 1 for o in ref)

    c = _host_ctx(n_blocks, 4, EOS, budget)

    def submit(rid, pl, mn, script):
        c.submit_tokens(rid, np.zeros(pl, np.int32), mn)
        for t in script:
            c.debug_push_sampled(rid, t)

    def step():
        so = c.step_tokens()
        o = {k: getattr(so, k) for k in KEYS}
        o["batch_ids"] = c.decode_batch_ids()
        return o

    got = _drive(submit, step, c.debug_complete_prefill, reqs, delays)
    assert len(got) == len(ref)
    for i, (a, b) in enumerate(zip(got, ref)):
        for k in KEYS + ("batch_ids",):
            assert a[k] == b[k], f"step {i}: {k}: library {a[k]} oracle {b[k]}"
    for rid, pl, mn, script, _ in reqs:
        toks, fin = c.request_output(rid)
        assert fin and toks.tolist() == lc.reqs[rid].out
        assert c.request_state(rid) == 5
    assert c.kv_num_free() == n_blocks


@pytest.mark.parametrize("n_blocks,seed,chunk", [(1000, 21, 16), (1000, 22, 32), (1000, 27, 96), (1000, 28, 160), (12, 23, 16), (8, 24, 48),
                                                 (7, 25, 16), (9, 26, 32), (10, 29, 96)])
def test_library_hybrid_batching_matches_oracle(n_blocks, seed, chunk):
    """The library's state machine with hybrid batching on (host-only context, tokens injected) against the
    oracle's hybrid policy, step by step: every counter, the batch, and the prompt parts each step takes."""
    reqs, delays = _trace(seed)
    lc = Lifecycle(n_blocks, max_batch=4, eos=EOS, hybrid_chunk=chunk)
    ref = _drive(lambda rid, pl, mn, sc: lc.submit(rid, pl, mn, sc), lc.step, lambda rid: None, reqs, delays)
    c = _host_ctx(n_blocks, 4, EOS)
    c.set_hybrid_batching(chunk)

    def submit(rid, pl, mn, script):
        c.submit_tokens(rid, np.zeros(pl, np.int32), mn)
        for t in script:
            c.debug_push_sampled(rid, t)

    def step():
        so = c.step_tokens()
        o = {k: getattr(so, k) for k in KEYS}
        o["batch_ids"] = c.decode_batch_ids()
        o["chunks"] = c.step_chunks()
        assert so.n_chunks == len(o["chunks"]) and so.chunk_tokens == sum(n for _, _, n in o["chunks"])
        return o

    got = _drive(submit, step, lambda rid: None, reqs, delays)
    assert len(got) == len(ref)
    for i, (a, b) in enumerate(zip(got, ref)):
        for k in KEYS + ("batch_ids", "chunks"):
            assert a[k] == b[k], f"step {i}: {k}: library {a[k]} oracle {b[k]}"
    for rid, pl, mn, script, _ in reqs:
        toks, fin = c.request_output(rid)
        assert fin and toks.tolist() == lc.reqs[rid].out == _expected_output(script, mn, EOS)
    assert c.kv_num_free() == n_blocks
    if n_blocks < 1000:
        assert sum(o["n_preempted"] for o in got) > 0
    if chunk >= 96:
        assert any(len(o["chunks"]) > 1 for o in got), "no step batched parts of several prompts"


@pytest.mark.parametrize("seed", range(300, 330))
def test_library_hybrid_batching_matches_oracle_random_pools(seed):
    """Thirty more traces with pool size, batch cap, budget and request count drawn from the seed."""
    g = np.random.default_rng(seed)
    n_blocks = int(g.integers(6, 40))
    max_batch = int(g.integers(1, 7))
    chunk = int(g.choice([16, 32, 48, 64, 96, 160]))
    reqs, delays = _trace(seed, n_req=int(g.integers(3, 25)), max_prompt=60, max_new=30)
    lc = Lifecycle(n_blocks, max_batch=max_batch, eos=EOS, hybrid_chunk=chunk)
    try:
        ref = _drive(lambda rid, pl, mn, sc: lc.submit(rid, pl, mn, sc), lc.step, lambda rid: None, reqs, delays)
    except NoBlocks:
        pytest.skip("the drawn pool cannot hold one of the drawn requests")
    c = rs.Context.from_shape(S.TINY, max_pos=8192, n_blocks=n_blocks, max_prefill_tokens=4096, max_decode_batch=max_batch,
                              max_context=4096, device=rs.RS_HOST_ONLY)
    c.set_head(None, None, None, vocab=64, eos_token=EOS)
    c.set_hybrid_batching(chunk)

    def submit(rid, pl, mn, script):
        c.submit_tokens(rid, np.zeros(pl, np.int32), mn)
        for t in script:
            c.debug_push_sampled(rid, t)

    def step():
        so = c.step_tokens()
        o = {k: getattr(so, k) for k in KEYS}
        o["batch_ids"] = c.decode_batch_ids()
        o["chunks"] = c.step_chunks()
        return o

    got = _drive(submit, step, lambda rid: None, reqs, delays)
    assert len(got) == len(ref)
    for i, (a, b) in enumerate(zip(got, ref)):
        for k in KEYS + ("batch_ids", "chunks"):
            assert a[k] == b[k], f"step {i}: {k}: library {a[k]} oracle {b[k]}"
    for rid, pl, mn, script, _ in reqs:
        toks, fin = c.request_output(rid)
        assert fin and toks.tolist() == lc.reqs[rid].out == _expected_output(script, mn, EOS)
    assert c.kv_num_free() == n_blocks


def test_library_hybrid_batching_argument_checks():
    c = _host_ctx(64, 4, EOS, max_prefill=100)
    for bad in (-16, 8, 24):
        with pytest.raises(rs.RapidServeError) as e:
            c.set_hybrid_batching(bad)
        assert e.value.code == rs.RS_ERR_BAD_ARG
    with pytest.raises(rs.RapidServeError) as e:      # 112 + 4 decode rows do not fit 100 rows of workspace
        c.set_hybrid_batching(112)
    assert e.value.code == rs.RS_ERR_BAD_ARG
    c.set_hybrid_batching(32)
    c.submit_tokens(1, np.zeros(40, np.int32), 2)
    with pytest.raises(rs.RapidServeError) as e:      # not while a request is in flight
        c.set_hybrid_batching(0)
    assert e.value.code == rs.RS_ERR_STATE
    with pytest.raises(rs.RapidServeError) as e:      # the engine threads serve with two sides
        c.engine_start()
    assert e.value.code == rs.RS_ERR_STATE


@pytest.mark.parametrize("seed", range(100, 130))
def test_library_life_cycle_matches_oracle_random_pools(seed):
    """Thirty more traces with pool size, batch cap, prefill budget and request count drawn from the seed."""
    g = np.random.default_rng(seed)
    n_blocks = int(g.integers(6, 40))
    max_batch = int(g.integers(1, 7))
    budget = int(g.choice([64, 100, 160, 4096]))
    reqs, delays = _trace(seed, n_req=int(g.integers(3, 25)), max_prompt=min(60, budget), max_new=30)
    lc = Lifecycle(n_blocks, max_batch=max_batch, eos=EOS, max_prefill_tokens=budget)
    ref = _drive(lambda rid, pl, mn, sc: lc.submit(rid, pl, mn, sc), lc.step, lc.complete_prefill, reqs, delays)
    c = rs.Context.from_shape(S.TINY, max_pos=8192, n_blocks=n_blocks, max_prefill_tokens=budget, max_decode_batch=max_batch,
                              max_context=4096, device=rs.RS_HOST_ONLY)
    c.set_head(None, None, None, vocab=64, eos_token=EOS)

    def submit(rid, pl, mn, script):
        c.submit_tokens(rid, np.zeros(pl, np.int32), mn)
        for t in script:
            c.debug_push_sampled(rid, t)

    def step():
        so = c.step_tokens()
        o = {k: getattr(so, k) for k in KEYS}
        o["batch_ids"] = c.decode_batch_ids()
        return o

    got = _drive(submit, step, c.debug_complete_prefill, reqs, delays)
    assert len(got) == len(ref)
    for i, (a, b) in enumerate(zip(got, ref)):
        for k in KEYS + ("batch_ids",):
            assert a[k] == b[k], f"step {i}: {k}: library {a[k]} oracle {b[k]}"
    for rid, pl, mn, script, _ in reqs:
        toks, fin = c.request_output(rid)
        assert fin and toks.tolist() == lc.reqs[rid].out == _expected_output(script, mn, EOS)
    assert c.kv_num_free() == n_blocks


def test_library_token_requests_argument_checks():
    c = _host_ctx(8, 2, EOS)
    with pytest.raises(rs.RapidServeError):
        c.submit_tokens(1, np.array([64], np.int32), 4)          # outside the vocabulary
    with pytest.raises(rs.RapidServeError):
        c.submit_tokens(1, np.zeros(4090, np.int32), 100)        # exceeds max_context
    with pytest.raises(rs.RapidServeError):
        c.submit_tokens(-1, np.array([1], np.int32), 4)          # ids are non-negative
    c.submit_tokens(1, np.array([1, 2, 3], np.int32), 4)
    with pytest.raises(rs.RapidServeError):
        c.submit_tokens(1, np.array([1], np.int32), 4)           # duplicate id
    with pytest.raises(rs.RapidServeError) as e:
        c.submit(2, 4, 4)                                        # hidden-state request on a token context
    assert e.value.code == rs.RS_ERR_STATE
    bare = rs.Context.from_shape(S.TINY, max_pos=128, n_blocks=8, max_prefill_tokens=64, max_decode_batch=2,
                                 max_context=128, device=rs.RS_HOST_ONLY)
    with pytest.raises(rs.RapidServeError) as e:
        bare.submit_tokens(1, np.array([1], np.int32), 4)        # no head set
    assert e.value.code == rs.RS_ERR_STATE


def test_library_reports_a_pool_too_small_for_one_request():
    c = _host_ctx(2, 2, -1)
    c.submit_tokens(1, np.zeros(30, np.int32), 20)
    with pytest.raises(rs.RapidServeError) as e:
        for _ in range(40):
            so = c.step_tokens()
            if so.prefill_started_req >= 0:
                c.debug_complete_prefill(1)
    assert e.value.code == rs.RS_ERR_NO_BLOCKS


# ------------------------------------------------------------------ the two-thread engine (host-only)
def _engine_run(n_blocks, seed, n_req=14, threads=1):
    import threading
    import time
    reqs, _ = _trace(seed, n_req=n_req)
    c = _host_ctx(n_blocks, 4, EOS)
    c.engine_start()
    try:
        def submit_some(part):
            for rid, pl, mn, script, _ in part:
                for t in script:
                    c.debug_push_sampled(rid, t)
                c.submit_tokens(rid, np.zeros(pl, np.int32), mn)
        parts = [reqs[i::threads] for i in range(threads)]
        ts = [threading.Thread(target=submit_some, args=(p,)) for p in parts]
        for t in ts:
            t.start()
        # poll while it runs: a reader must never see a count ahead of its tokens (every visible token is final)
        seen = {}
        t0 = time.time()
        while c.engine_stats()["finished"] < len(reqs) and time.time() - t0 < 30:
            for rid, *_ in reqs:
                try:
                    toks, fin = c.request_output(rid)
                except rs.RapidServeError:
                    continue   # not submitted yet
                prev = seen.get(rid, [])
                assert toks.tolist()[:len(prev)] == prev
                seen[rid] = toks.tolist()
        for t in ts:
            t.join()
    finally:
        c.engine_stop(drain=True)
    st = c.engine_stats()
    assert st["submitted"] == st["finished"] == len(reqs)
    for rid, pl, mn, script, _ in reqs:
        toks, fin = c.request_output(rid)
        assert fin and toks.tolist() == _expected_output(script, mn, EOS)
        assert c.request_state(rid) == 5
        ts_, tf, tl = c.request_times(rid)
        assert 0 < ts_ <= tf <= tl
    assert c.kv_num_free() == n_blocks
    return st


@pytest.mark.parametrize("n_blocks,seed,threads", [(1000, 21, 1), (8, 22, 1), (7, 23, 3), (12, 24, 2)])
def test_engine_threads_produce_the_scripted_outputs(n_blocks, seed, threads):
    st = _engine_run(n_blocks, seed, threads=threads)
    if n_blocks == 1000:
        assert st["preempted"] == 0


def test_engine_refuses_direct_stepping_and_restarts():
    c = _host_ctx(64, 4, EOS)
    c.engine_start()
    with pytest.raises(rs.RapidServeError) as e:
        c.step_tokens()
    assert e.value.code == rs.RS_ERR_STATE
    with pytest.raises(rs.RapidServeError):
        c.engine_start()
    c.debug_push_sampled(5, 3)
    c.debug_push_sampled(5, EOS)
    c.submit_tokens(5, np.zeros(9, np.int32), 10)
    c.engine_stop(drain=True)
    toks, fin = c.request_output(5)
    assert fin and toks.tolist() == [3, EOS]
    with pytest.raises(rs.RapidServeError):
        c.engine_stop()
    c.engine_start()                         # a drained engine can be started again
    c.submit_tokens(6, np.zeros(4, np.int32), 2)
    c.engine_stop(drain=True)
    toks, fin = c.request_output(6)
    assert fin and toks.tolist() == [0, 0]
    c.destroy()


def test_engine_reports_a_pool_too_small():
    c = _host_ctx(2, 2, -1)
    c.engine_start()
    c.submit_tokens(1, np.zeros(30, np.int32), 20)
    with pytest.raises(rs.RapidServeError) as e:
        c.engine_stop(drain=True)
    assert e.value.code == rs.RS_ERR_NO_BLOCKS


def test_request_release_forgets_finished_requests_only():
    """rs_request_release: refused while the request is live, drops the record once finished (the id can be
    used again), in the single-loop driver and with the engine."""
    c = _host_ctx(64, 4, -1)
    c.submit_tokens(1, np.zeros(5, np.int32), 2)
    with pytest.raises(rs.RapidServeError) as e:
        c.request_release(1)
    assert e.value.code == rs.RS_ERR_STATE
    for _ in range(20):
        so = c.step_tokens()
        if so.prefill_started_req >= 0:
            c.debug_complete_prefill(so.prefill_started_req)
        if c.request_state(1) == 5:
            break
    toks, fin = c.request_output(1)
    assert fin and len(toks) == 2
    c.request_release(1)
    with pytest.raises(rs.RapidServeError) as e:
        c.request_output(1)
    assert e.value.code == rs.RS_ERR_BAD_ARG
    c.submit_tokens(1, np.zeros(3, np.int32), 1)      # the id is free again
    c.destroy()

    c = _host_ctx(64, 4, -1)
    c.engine_start()
    for rid in range(40):
        c.submit_tokens(rid, np.zeros(4, np.int32), 3)
    c.engine_stop(drain=True)
    for rid in range(40):
        toks, fin = c.request_output(rid)
        assert fin and len(toks) == 3
        c.request_release(rid)
        with pytest.raises(rs.RapidServeError):
            c.request_output(rid)
    with pytest.raises(rs.RapidServeError) as e:
        c.request_release(3)
    assert e.value.code == rs.RS_ERR_BAD_ARG
    c.destroy()
