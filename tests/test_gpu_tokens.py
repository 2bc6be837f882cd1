"""GPU parity of the token boundary (embedding, final norm + LM head, greedy choice) and of closed-loop
generation through the C ABI, against the token-level oracle."""
import numpy as np
import pytest
import torch

import oracle
from oracle import lm
import paper_2601_11822_amd as rs
import rs_synth as S
from tests.gpu_util import TOL, Rig, check_tensor, to_bits, to_dev

pytestmark = pytest.mark.gpu


def _head_dev(rig, vocab, eos=-1, seed=0):
    hb = S.head_weights(rig.shape.d_model, vocab, seed=seed)
    hd = {k: to_dev(v) for k, v in hb.items()}
    rig.ctx.set_head(hd["embed"], hd["final_norm"], hd["lm_head"], vocab, eos)
    rig._keep.append(hd)
    return hb


def _check_choice(gpu_tok, gpu_logits, ref_logits):
    """The decision is exact in the kernel's own precision (lowest index among the maxima of the float32
    logits it produced); against the oracle every token must be a near-maximum, and the oracle's own
    choice wherever that choice is decisive at the parity tolerance."""
    assert np.array_equal(gpu_tok, np.argmax(gpu_logits, axis=1).astype(np.int32))
    slack = 2 * TOL * np.max(np.abs(ref_logits), axis=1)
    top = np.max(ref_logits, axis=1)
    chosen = ref_logits[np.arange(len(gpu_tok)), gpu_tok]
    assert np.all(chosen >= top - slack)
    ref_tok = lm.greedy(ref_logits)
    second = np.sort(ref_logits, axis=1)[:, -2]
    decisive = (top - second) > slack
    assert np.array_equal(gpu_tok[decisive], ref_tok[decisive])
    return float(np.mean(gpu_tok == ref_tok))


@pytest.mark.parametrize("shape,vocab,n", [(S.TINY, 1000, 5), (S.TINY, 1003, 64), (S.TINY, 64, 1), (S.MID, 4100, 70)])
def test_embed_and_lm_head_match_oracle(shape, vocab, n):
    rig = Rig(shape, n_blocks=8, max_prefill_tokens=128, max_decode_batch=max(n, 4), max_context=64, with_oracle=False)
    try:
        hb = _head_dev(rig, vocab)
        toks = S.prompt_tokens(n, vocab, 3)
        for side in (rs.RS_SIDE_DECODE, rs.RS_SIDE_PREFILL):
            t_dev = torch.from_numpy(toks).cuda()
            x = torch.zeros((n, shape.d_model), dtype=torch.bfloat16, device="cuda")
            logits = torch.zeros((n, vocab), dtype=torch.float32, device="cuda")
            out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            rig.ctx.embed(side, t_dev, n, x)
            rig.ctx.lm_head_greedy(side, x, n, logits, out)
            rig.ctx.sync(side)
            # the lookup is a copy: bit-exact
            assert np.array_equal(to_bits(x), hb["embed"][toks])
            ref = lm.head_logits(lm.embed(toks, hb["embed"]), hb["final_norm"], hb["lm_head"], shape.rms_eps)
            got = logits.cpu().numpy()
            check_tensor(f"logits side {side}", got, ref)
            frac = _check_choice(out.cpu().numpy(), got, ref)
            print(f"  side {side}: {frac:.2%} of tokens equal the oracle's choice", flush=True)
            # tokens only, no logits buffer
            out2 = torch.full((n,), -1, dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            rig.ctx.lm_head_greedy(side, x, n, None, out2)
            rig.ctx.sync(side)
            assert torch.equal(out, out2)
    finally:
        rig.close()


def test_greedy_ties_and_planted_maximum():
    # identical LM-head rows give identical logits: the lowest index must win; a planted row wins elsewhere
    shape, vocab, n = S.TINY, 520, 3
    rig = Rig(shape, n_blocks=8, max_prefill_tokens=16, max_decode_batch=4, max_context=64, with_oracle=False)
    try:
        hb = S.head_weights(shape.d_model, vocab)
        x_bits = S.hidden_states(n, shape.d_model, 5)
        h = oracle.rmsnorm(S.bf16_bits_to_f32(x_bits), oracle.widen(hb["final_norm"]), shape.rms_eps)
        W = np.zeros((vocab, shape.d_model), np.float32)
        W[:] = 0.01 * np.sign(h[0])[None, :]                # every row the same: all logits of a row are equal
        W[517] = 0.02 * np.sign(h[1])                       # row 517 beats the rest for input row 1
        hb["lm_head"] = S.f32_to_bf16_bits(W)
        hd = {k: to_dev(v) for k, v in hb.items()}
        rig.ctx.set_head(hd["embed"], hd["final_norm"], hd["lm_head"], vocab, -1)
        x = to_dev(x_bits)
        out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        logits = torch.zeros((n, vocab), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        rig.ctx.lm_head_greedy(rs.RS_SIDE_DECODE, x, n, logits, out)
        rig.ctx.sync(rs.RS_SIDE_DECODE)
        got = out.cpu().numpy()
        lg = logits.cpu().numpy()
        assert np.all(lg[0, :517] == lg[0, 0]) and got[0] == 0
        assert got[1] == 517
        assert np.array_equal(got, np.argmax(lg, axis=1))
    finally:
        rig.close()


def test_token_outside_vocabulary_is_reported_not_dereferenced():
    shape, vocab = S.TINY, 100
    rig = Rig(shape, n_blocks=8, max_prefill_tokens=16, max_decode_batch=4, max_context=64, with_oracle=False)
    try:
        hb = _head_dev(rig, vocab)
        toks = torch.tensor([3, 100, -5, 99], dtype=torch.int32, device="cuda")
        x = torch.ones((4, shape.d_model), dtype=torch.bfloat16, device="cuda")
        torch.cuda.synchronize()
        rig.ctx.embed(rs.RS_SIDE_DECODE, toks, 4, x)
        with pytest.raises(rs.RapidServeError) as e:
            rig.ctx.sync(rs.RS_SIDE_DECODE)
        assert e.value.code == rs.RS_ERR_BAD_ARG
        bits = to_bits(x)
        assert np.array_equal(bits[0], hb["embed"][3]) and np.array_equal(bits[3], hb["embed"][99])
        assert not bits[1].any() and not bits[2].any()
        rig.ctx.sync(rs.RS_SIDE_DECODE)   # the flag was cleared
    finally:
        rig.close()


def test_llama_sized_head_sampled_rows():
    # d_model 4096, vocabulary 128256, 64 rows: the choice is checked exactly on the GPU's logits for all
    # rows, the logits against the oracle on 6 rows (the product costs the oracle ~1 GFLOP per row)
    d, vocab, n = 4096, 128256, 64
    shape = S.LayerShape("head-only", d, 4, 4, 64, 64, 1e-5, 10000.0)
    rig = Rig(shape, n_blocks=4, max_prefill_tokens=16, max_decode_batch=n, max_context=64, with_oracle=False)
    try:
        hb = _head_dev(rig, vocab)
        x_bits = S.hidden_states(n, d, 9)
        x = to_dev(x_bits)
        logits = torch.zeros((n, vocab), dtype=torch.float32, device="cuda")
        out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        rig.ctx.lm_head_greedy(rs.RS_SIDE_DECODE, x, n, logits, out)
        rig.ctx.sync(rs.RS_SIDE_DECODE)
        got, tok = logits.cpu().numpy(), out.cpu().numpy()
        assert np.array_equal(tok, np.argmax(got, axis=1))
        rows = [0, 1, 31, 32, 62, 63]
        ref = lm.head_logits(S.bf16_bits_to_f32(x_bits[rows]), hb["final_norm"], hb["lm_head"], shape.rms_eps)
        check_tensor("logits (6 rows)", got[rows], ref)
        _check_choice(tok[rows], got[rows], ref)
    finally:
        rig.close()


# ------------------------------------------------------------------------------ closed loop
def _serve(rig, hb, vocab, eos, requests, wait, max_steps=4000):
    """requests: (id, prompt tokens, max_new, arrival step).  Runs rs_step_tokens until all are done."""
    todo = sorted(requests, key=lambda r: r[3])
    outs, n_pre, step, n_done = {}, 0, 0, 0
    while n_done < len(requests) and step < max_steps:
        while todo and todo[0][3] <= step:
            rid, prompt, mn, _ = todo.pop(0)
            rig.ctx.submit_tokens(rid, prompt, mn)
        so = rig.ctx.step_tokens(wait_decode=wait)
        n_pre += so.n_preempted
        n_done += so.n_finished
        step += 1
        if not wait and so.decode_batch == 0:
            rig.ctx.sync(rs.RS_SIDE_PREFILL)   # nothing to decode yet: let the prefill finish instead of spinning
    rig.ctx.sync(rs.RS_SIDE_PREFILL)
    rig.ctx.sync(rs.RS_SIDE_DECODE)
    for _ in range(3):
        rig.ctx.step_tokens(wait_decode=True)   # drains late tokens
    assert n_done == len(requests), f"{n_done} of {len(requests)} finished in {step} steps"
    for rid, *_ in requests:
        toks, fin = rig.ctx.request_output(rid)
        assert fin
        outs[rid] = toks.tolist()
    return outs, n_pre


def _check_against_oracle(shape, n_layers, hb, wbits, vocab, eos, requests, outs):
    """Teacher-forced: the oracle is fed the library's own tokens and must rate each one a near-maximum
    (and its own choice wherever that choice is decisive); lengths follow from the stop rule."""
    n_equal = n_total = 0
    for rid, prompt, mn, _ in requests:
        got = outs[rid]
        assert 1 <= len(got) <= mn
        assert all(t != eos for t in got[:-1])
        assert len(got) == mn or got[-1] == eos
        nb = S.blocks_for(len(prompt) + mn)
        m = lm.OracleModel(shape, wbits, hb, nb)
        tab = np.arange(nb, dtype=np.int32)
        logits = m.prefill(prompt, tab)
        for k, tok in enumerate(got):
            slack = 2 * TOL * np.max(np.abs(logits))
            top2 = np.sort(logits)[-2:]
            assert logits[tok] >= top2[1] - slack, f"request {rid} token {k}: {tok} is not a near-maximum"
            ref_tok = int(lm.greedy(logits[None, :])[0])
            if top2[1] - top2[0] > slack:
                assert tok == ref_tok, f"request {rid} token {k}: {tok}, oracle {ref_tok} (decisive)"
            n_equal += tok == ref_tok
            n_total += 1
            if k + 1 < len(got):
                logits = m.decode([tok], [len(prompt) + k], tab[None, :])[0]
    return n_equal / n_total


@pytest.mark.parametrize("wait", [True, False])
def test_closed_loop_generation_matches_oracle(wait):
    shape, n_layers, vocab = S.TINY, 2, 1000
    prompts = [(1, 37, 12, 0), (2, 5, 20, 0), (3, 64, 9, 2), (4, 16, 1, 3), (5, 23, 16, 6)]
    requests = [(rid, S.prompt_tokens(pl, vocab, rid), mn, arr) for rid, pl, mn, arr in prompts]
    hb = S.head_weights(shape.d_model, vocab)
    wbits = [S.layer_weights(shape, l) for l in range(n_layers)]
    # the end-of-sequence token comes from the oracle alone: what request 2 produces 6th in a free run
    free, _ = lm.OracleModel(shape, wbits, hb, 4).generate(requests[1][1], np.arange(4, dtype=np.int32), 20)
    eos = free[5]
    rig = Rig(shape, n_blocks=64, max_prefill_tokens=128, max_decode_batch=4, max_context=128, n_layers=n_layers,
              with_oracle=False)
    try:
        hd = {k: to_dev(v) for k, v in hb.items()}
        rig.ctx.set_head(hd["embed"], hd["final_norm"], hd["lm_head"], vocab, eos)
        outs, n_pre = _serve(rig, hb, vocab, eos, requests, wait)
        assert n_pre == 0
        frac = _check_against_oracle(shape, n_layers, hb, wbits, vocab, eos, requests, outs)
        print(f"  wait={wait}: {frac:.2%} of generated tokens equal the oracle's choice; lengths "
              f"{ {r: len(t) for r, t in outs.items()} }", flush=True)
        assert frac >= 0.9
        assert rig.ctx.kv_num_free() == 64
    finally:
        rig.close()


def test_closed_loop_steps_run_as_captured_graphs_and_match_oracle_and_eager():
    """Section 4.5.2: the serving loop launches each decode step (embedding, both layers, head) as one captured
    graph per (batch size, context bucket, stream).  The generated tokens are checked against the oracle like any
    closed-loop run, the counters show that every decode step went out as a graph and that graphs were reused,
    and the same requests served with graphs off give the same tokens."""
    shape, n_layers, vocab = S.TINY, 2, 1000
    prompts = [(1, 37, 30, 0), (2, 5, 40, 0), (3, 64, 25, 2), (4, 16, 3, 3), (5, 23, 33, 6)]
    requests = [(rid, S.prompt_tokens(pl, vocab, rid), mn, arr) for rid, pl, mn, arr in prompts]
    hb = S.head_weights(shape.d_model, vocab)
    wbits = [S.layer_weights(shape, l) for l in range(n_layers)]
    results, results_captured, results_launched = {}, {}, {}
    for graphs in (True, 2, False):   # 2: at most two graphs kept, so the cache is dropped and refilled over and over
        rig = Rig(shape, n_blocks=64, max_prefill_tokens=128, max_decode_batch=4, max_context=128, n_layers=n_layers,
                  with_oracle=False)
        try:
            hd = {k: to_dev(v) for k, v in hb.items()}
            rig.ctx.set_head(hd["embed"], hd["final_norm"], hd["lm_head"], vocab, -1)
            rig.ctx.set_step_graphs(graphs)
            rig.ctx.set_cu_split(128, 128)   # the manager (no profile) moves to (0,256) / (256,256): several streams, several graphs
            outs, _ = _serve(rig, hb, vocab, -1, requests, wait=False)
            captured, launched, _, _ = rig.ctx.step_graph_stats()
            print(f"  graphs={graphs}: {captured} graphs captured, {launched} steps launched as graphs", flush=True)
            if graphs == 2:
                # (how many steps a run takes depends on when its prefill passes finish, so the counts are not compared)
                assert captured > results_captured[True] and launched >= 30
            elif graphs:
                results_captured[True], results_launched[True] = captured, launched
                assert captured >= 2 and launched >= 30 and launched > 3 * captured
                frac = _check_against_oracle(shape, n_layers, hb, wbits, vocab, -1, requests, outs)
                assert frac >= 0.9
            else:
                assert captured == 0 and launched == 0
            results[graphs] = outs
        finally:
            rig.close()
    assert results[True] == results[False] == results[2]


@pytest.mark.parametrize("n_blocks,chunk", [(64, 16), (64, 48), (64, 96), (7, 16)])
def test_closed_loop_hybrid_batching_matches_oracle(n_blocks, chunk):
    """The comparison scheme (section 3.1) as a serving policy: prompts go through in chunks that share each
    step's batch with the decode rows.  The tokens are checked against the oracle exactly like the other policy's
    (a request's tokens do not depend on how its prompt was scheduled); the small pool forces a recomputation."""
    shape, n_layers, vocab = S.TINY, 2, 1000
    prompts = [(1, 37, 30, 0), (2, 5, 40, 0), (3, 64, 25, 2), (4, 16, 3, 3), (5, 23, 33, 6)] if n_blocks == 64 else \
              [(1, 20, 40, 0), (2, 20, 40, 0)]
    requests = [(rid, S.prompt_tokens(pl, vocab, rid), mn, arr) for rid, pl, mn, arr in prompts]
    hb = S.head_weights(shape.d_model, vocab)
    wbits = [S.layer_weights(shape, l) for l in range(n_layers)]
    rig = Rig(shape, n_blocks=n_blocks, max_prefill_tokens=128, max_decode_batch=4, max_context=128, n_layers=n_layers,
              with_oracle=False)
    try:
        hd = {k: to_dev(v) for k, v in hb.items()}
        rig.ctx.set_head(hd["embed"], hd["final_norm"], hd["lm_head"], vocab, -1)
        rig.ctx.set_hybrid_batching(chunk)
        chunks, mixed, several = [], 0, 0
        todo = sorted(requests, key=lambda r: r[3])
        n_pre = n_done = step = 0
        while n_done < len(requests) and step < 4000:
            while todo and todo[0][3] <= step:
                rid, prompt, mn, _ = todo.pop(0)
                rig.ctx.submit_tokens(rid, prompt, mn)
            so = rig.ctx.step_tokens(wait_decode=False)
            n_pre += so.n_preempted
            n_done += so.n_finished
            step += 1
            if so.n_chunks > 0:
                parts = rig.ctx.step_chunks()
                assert len(parts) == so.n_chunks and sum(n for _, _, n in parts) == so.chunk_tokens <= chunk
                several += len(parts) > 1
                chunks += parts
                mixed += so.decode_batch > 0
                assert (so.prefill_cus, so.decode_cus) == (256, 256)
            if so.decode_batch == 0:
                rig.ctx.sync(rs.RS_SIDE_PREFILL)
        rig.ctx.sync(rs.RS_SIDE_PREFILL)
        rig.ctx.sync(rs.RS_SIDE_DECODE)
        for _ in range(3):
            rig.ctx.step_tokens(wait_decode=True)
        assert n_done == len(requests)
        outs = {}
        for rid, *_ in requests:
            toks, fin = rig.ctx.request_output(rid)
            assert fin
            outs[rid] = toks.tolist()
        frac = _check_against_oracle(shape, n_layers, hb, wbits, vocab, -1, requests, outs)
        print(f"  budget {chunk}: {len(chunks)} parts, {mixed} steps with parts beside decode rows, {several} with several prompts, {n_pre} preemption(s); "
              f"{frac:.2%} of generated tokens equal the oracle's choice", flush=True)
        assert frac >= 0.9 and rig.ctx.kv_num_free() == n_blocks
        # every prompt went through in parts that start on block boundaries; some part shared a batch with decode
        # rows; with the larger budget some step carried parts of several prompts
        assert all(st % 16 == 0 for _, st, _ in chunks)
        assert {rid for rid, st, _ in chunks if st == 0} == {r[0] for r in requests}
        plen = {r[0]: len(r[1]) for r in requests}
        if n_pre == 0:
            for rid in plen:
                assert sum(n for r2, _, n in chunks if r2 == rid) == plen[rid]
        assert mixed >= 1 and (chunk < 96 or several >= 1)
        if n_blocks < 64:
            assert n_pre >= 1
    finally:
        rig.close()


def test_closed_loop_with_preemption_matches_oracle():
    # pool of 6 blocks: two 20-token prompts growing to 60 tokens each need 8: one is recomputed
    shape, n_layers, vocab = S.TINY, 2, 1000
    requests = [(1, S.prompt_tokens(20, vocab, 11), 40, 0), (2, S.prompt_tokens(20, vocab, 12), 40, 0)]
    hb = S.head_weights(shape.d_model, vocab)
    wbits = [S.layer_weights(shape, l) for l in range(n_layers)]
    rig = Rig(shape, n_blocks=6, max_prefill_tokens=128, max_decode_batch=4, max_context=128, n_layers=n_layers,
              with_oracle=False)
    try:
        hd = {k: to_dev(v) for k, v in hb.items()}
        rig.ctx.set_head(hd["embed"], hd["final_norm"], hd["lm_head"], vocab, -1)
        outs, n_pre = _serve(rig, hb, vocab, -1, requests, wait=False)
        assert n_pre >= 1
        frac = _check_against_oracle(shape, n_layers, hb, wbits, vocab, -1, requests, outs)
        print(f"  {n_pre} preemption(s); {frac:.2%} of generated tokens equal the oracle's choice", flush=True)
        assert frac >= 0.9 and rig.ctx.kv_num_free() == 6
    finally:
        rig.close()


# ------------------------------------------------------------------------------ two-thread engine
def _serve_engine(rig, requests, timeout_s=60.0):
    import time
    c = rig.ctx
    c.engine_start()
    try:
        for rid, prompt, mn, arr in sorted(requests, key=lambda r: r[3]):
            time.sleep(0.002 * arr)          # staggered arrivals
            c.submit_tokens(rid, prompt, mn)
        t0 = time.time()
        while c.engine_stats()["finished"] < len(requests):
            assert time.time() - t0 < timeout_s, f"engine stalled: {c.engine_stats()}"
            time.sleep(0.001)
    finally:
        c.engine_stop(drain=True)
    st = c.engine_stats()
    outs = {}
    for rid, *_ in requests:
        toks, fin = c.request_output(rid)
        assert fin
        outs[rid] = toks.tolist()
    return outs, st


@pytest.mark.parametrize("n_blocks", [64, 6])
def test_engine_generation_matches_oracle(n_blocks):
    shape, n_layers, vocab = S.TINY, 2, 1000
    if n_blocks == 64:
        prompts = [(1, 37, 12, 0), (2, 5, 20, 0), (3, 64, 9, 2), (4, 16, 1, 3), (5, 23, 16, 6)]
    else:   # two sequences growing to 60 tokens each need 8 blocks: one is recomputed
        prompts = [(1, 20, 40, 0), (2, 20, 40, 0)]
    requests = [(rid, S.prompt_tokens(pl, vocab, rid), mn, arr) for rid, pl, mn, arr in prompts]
    hb = S.head_weights(shape.d_model, vocab)
    wbits = [S.layer_weights(shape, l) for l in range(n_layers)]
    free, _ = lm.OracleModel(shape, wbits, hb, 4).generate(requests[1][1], np.arange(4, dtype=np.int32), 20)
    eos = free[5] if n_blocks == 64 else -1
    rig = Rig(shape, n_blocks=n_blocks, max_prefill_tokens=128, max_decode_batch=4, max_context=128, n_layers=n_layers,
              with_oracle=False)
    try:
        hd = {k: to_dev(v) for k, v in hb.items()}
        rig.ctx.set_head(hd["embed"], hd["final_norm"], hd["lm_head"], vocab, eos)
        outs, st = _serve_engine(rig, requests)
        frac = _check_against_oracle(shape, n_layers, hb, wbits, vocab, eos, requests, outs)
        print(f"  engine, pool {n_blocks}: {st}; {frac:.2%} of generated tokens equal the oracle's choice", flush=True)
        assert frac >= 0.9 and rig.ctx.kv_num_free() == n_blocks
        assert (st["preempted"] >= 1) == (n_blocks == 6)
    finally:
        rig.close()


def test_closed_loop_8b_shaped_layer_and_edge_prompts():
    """One Llama-3-8B-shaped layer with a 32000-token vocabulary: prompts of 1 token, of 20 tokens (the pass
    takes the weight-streaming GEMMs), of 70 tokens (large-tile GEMMs with a sliced K range) and of exactly
    max_prefill_tokens, generated through the engine and checked token by token against the oracle."""
    shape, n_layers, vocab = S.LLAMA8B, 1, 32000
    prompts = [(1, 70, 5, 0), (2, 20, 5, 0), (3, 1, 4, 1), (4, 96, 3, 2)]
    requests = [(rid, S.prompt_tokens(pl, vocab, rid), mn, arr) for rid, pl, mn, arr in prompts]
    hb = S.head_weights(shape.d_model, vocab)
    wbits = [S.layer_weights(shape, 0)]
    rig = Rig(shape, n_blocks=32, max_prefill_tokens=96, max_decode_batch=4, max_context=128, n_layers=n_layers,
              with_oracle=False)
    try:
        hd = {k: to_dev(v) for k, v in hb.items()}
        rig.ctx.set_head(hd["embed"], hd["final_norm"], hd["lm_head"], vocab, -1)
        with pytest.raises(rs.RapidServeError):
            rig.ctx.submit_tokens(9, S.prompt_tokens(97, vocab, 9), 2)     # longer than max_prefill_tokens
        outs, st = _serve_engine(rig, requests)
        frac = _check_against_oracle(shape, n_layers, hb, wbits, vocab, -1, requests, outs)
        print(f"  8B-shaped layer: {st}; {frac:.2%} of generated tokens equal the oracle's choice", flush=True)
        assert frac >= 0.8 and rig.ctx.kv_num_free() == 32
    finally:
        rig.close()
