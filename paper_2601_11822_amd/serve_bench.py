"""Closed-loop serving measurement: a whole Llama-shaped stack under an open-loop arrival process.

Requests (seeded, synthetic: Poisson arrivals, log-normal prompt and output lengths, random-weight
model, uniform random prompt tokens) are submitted on the wall clock to rs_submit_tokens while one
host loop calls rs_step_tokens; the library embeds, prefills whole prompts on the prefill
partition, decodes the running batch on the decode partition, samples greedily, grows / releases /
preempts KV blocks and re-chooses the CU split every step (sections 4.4, 4.5 of the paper).

Reported: time to first token, inter-token latency (wall-clock period of the decode steps, weighted
by the tokens each step produced), generated tokens/s, prefill tokens/s, the CU splits used and
the preemption count, for one policy:

    --policy manager   profile-driven split (needs --profile FILE, or --profile measure to run the
                       offline profiler first on a one-layer rig of the same shape)
    --policy over      no profile: both partitions see every CU whenever both have work
    --policy hybrid    the scheme the paper compares with (section 3.1): no partitions; a prompt goes through in
                       chunks of --chunk tokens, each in one batch with the decode step (rs_set_hybrid_batching)

With --engine the library's own decode and prefill threads drive the loop (rs_engine_start) and
the script only submits and polls; per-request inter-token latency is then (last - first token
time) / (tokens - 1).

    python -m paper_2601_11822_amd.serve_bench --layers 32 --requests 48 --rate 8 --policy over
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

from . import Context, RS_SIDE_DECODE, RS_SIDE_PREFILL


def _log(*a):
    print(*a, file=sys.stderr, flush=True)


def _lognormal_params(mean: float, sd: float):
    s2 = np.log(1.0 + (sd / mean) ** 2)
    return np.log(mean) - s2 / 2, np.sqrt(s2)


def make_workload(n: int, rate: float, prompt_mean: float, prompt_sd: float, out_mean: float, out_sd: float,
                  prompt_clip, out_clip, vocab: int, seed: int):
    g = np.random.Generator(np.random.Philox(key=[seed, 77]))
    t = np.cumsum(g.exponential(1.0 / rate, size=n))
    mu, sg = _lognormal_params(prompt_mean, prompt_sd)
    pl = np.clip(np.rint(g.lognormal(mu, sg, size=n)), *prompt_clip).astype(int)
    mu, sg = _lognormal_params(out_mean, out_sd)
    ol = np.clip(np.rint(g.lognormal(mu, sg, size=n)), *out_clip).astype(int)
    return [(i, float(t[i]), g.integers(0, vocab, size=pl[i], dtype=np.int32), int(ol[i])) for i in range(n)]


def build_model(shape, n_layers: int, vocab: int, n_blocks: int, max_prefill: int, max_batch: int, max_context: int,
                profile, device: int = 0, release: bool = False, experts: int = 0):
    import torch
    dev = torch.device(f"cuda:{device}")
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    Hkv, hd, d, f = shape.n_kv_heads, shape.head_dim, shape.d_model, shape.ffn_dim
    k_pool = torch.zeros((n_layers, n_blocks, Hkv, 16, hd), dtype=torch.bfloat16, device=dev)
    v_pool = torch.zeros((n_layers, n_blocks, Hkv, hd, 16), dtype=torch.bfloat16, device=dev)
    c = Context.from_shape(shape, n_layers=n_layers, max_pos=max_context, n_blocks=n_blocks, k_pool=k_pool, v_pool=v_pool,
                           max_prefill_tokens=max_prefill, max_decode_batch=max_batch, max_context=max_context,
                           profile=profile, device=device)
    rnd = lambda *s, std=0.02, mean=0.0: (torch.randn(s, generator=g, device=dev, dtype=torch.float32) * std + mean).to(torch.bfloat16)
    keep = [k_pool, v_pool]
    for l in range(n_layers):
        if experts:   # sparse feed-forward block: the experts' matrices are packed during the call and dropped here
            w = (rnd(d, mean=1.0), rnd(shape.qkv_dim, d), rnd(d, shape.q_dim), rnd(d, mean=1.0), None, None, None)
            c.set_weights(l, *w)
            router = rnd(experts, d, std=0.1)
            c.set_moe_weights(l, router, rnd(experts, f, d), rnd(experts, f, d), rnd(experts, d, f), experts)
            keep.append((w, router))
            continue
        w = (rnd(d, mean=1.0), rnd(shape.qkv_dim, d), rnd(d, shape.q_dim), rnd(d, mean=1.0), rnd(f, d), rnd(f, d), rnd(d, f))
        c.set_weights(l, *w)
        if release:   # the library keeps packed copies only: a 70B-shaped stack then fits one GPU beside its KV pool
            c.release_source_weights(l)
            w = (w[0], w[3])
        keep.append(w)
    head = (rnd(vocab, d, std=1.0), rnd(d, mean=1.0), rnd(vocab, d))
    c.set_head(*head, vocab, -1)
    keep.append(head)
    torch.cuda.synchronize()
    return c, keep


def serve(c: Context, work, wait_decode: bool, time_limit: float, max_live: int = 1 << 30):
    """Runs the arrival process; returns per-step records and per-request times.  Arrivals beyond max_live
    requests in flight wait on the host (their time to first token counts from their submission)."""
    todo = list(work)
    steps = []
    live = 0
    n_done = 0
    t0 = time.perf_counter()
    last_t = None
    t_log = 0.0
    while n_done < len(work):
        now = time.perf_counter() - t0
        if now > time_limit:
            raise RuntimeError(f"time limit: {n_done} of {len(work)} requests finished in {now:.1f}s")
        while todo and todo[0][1] <= now and live < max_live:   # the library holds 4 * max_batch + 64 live requests
            rid, _, prompt, n_out = todo.pop(0)
            c.submit_tokens(rid, prompt, n_out)
            live += 1
        if live == 0:
            time.sleep(min(0.002, max(0.0, todo[0][1] - now)))
            last_t = None
            continue
        t_call = time.perf_counter()
        so = c.step_tokens(wait_decode=wait_decode)
        t = time.perf_counter() - t0
        t_call = time.perf_counter() - t_call
        if so.decode_batch == 0 and so.prefill_started_req < 0:
            time.sleep(0.0005)   # only a prefill in flight: nothing to enqueue until it is done
        steps.append((t, so.decode_batch, so.decode_sum_ctx, so.prefill_cus, so.decode_cus, so.prefill_started_tokens,
                      so.n_preempted, so.decode_ms, (t - last_t) if (last_t is not None and so.decode_batch) else -1.0,
                      t_call if (so.decode_batch and so.prefill_started_req < 0 and not wait_decode) else -1.0))
        last_t = t if so.decode_batch else None
        n_done += so.n_finished
        live -= so.n_finished
        if t - t_log > 2.0:
            _log(f"[serve] t={t:.1f}s finished {n_done}/{len(work)} batch {so.decode_batch} split {so.prefill_cus}/{so.decode_cus}")
            t_log = t
    c.sync(RS_SIDE_PREFILL)
    c.sync(RS_SIDE_DECODE)
    wall = time.perf_counter() - t0
    for _ in range(3):
        c.step_tokens(wait_decode=True)
    return steps, wall


def serve_engine(c: Context, work, time_limit: float, max_live: int = 1 << 30):
    """The same arrival process against the library's own two threads (rs_engine_start)."""
    todo = list(work)
    c.engine_start()
    t0 = time.perf_counter()
    t_log = 0.0
    try:
        while True:
            now = time.perf_counter() - t0
            st = c.engine_stats()
            while todo and todo[0][1] <= now and len(work) - len(todo) - st["finished"] < max_live:
                rid, _, prompt, n_out = todo.pop(0)
                c.submit_tokens(rid, prompt, n_out)
            if not todo and st["finished"] >= len(work):
                break
            if now > time_limit:
                raise RuntimeError(f"time limit: {st}")
            if now - t_log > 2.0:
                _log(f"[serve] t={now:.1f}s {st}")
                t_log = now
            time.sleep(0.0005 if not todo else min(0.0005, max(0.0, todo[0][1] - now)))
        wall = time.perf_counter() - t0
    finally:
        c.engine_stop(drain=False)
    return c.engine_stats(), wall


def summarise_engine(c: Context, work, stats, wall: float):
    ttft, itl, n_gen, n_prompt = [], [], 0, 0
    for rid, t_arr, prompt, n_out in work:
        toks, fin = c.request_output(rid)
        assert fin and len(toks) == n_out, f"request {rid}: {len(toks)} of {n_out} tokens"
        ts, tf, tl = c.request_times(rid)
        ttft.append(tf - ts)
        if n_out > 1:
            itl.append((tl - tf) / (n_out - 1))
        n_gen += len(toks)
        n_prompt += len(prompt)
    return {
        "requests": len(work), "wall_s": wall, "generated_tokens": n_gen, "prompt_tokens": n_prompt,
        "generated_tok_per_s": n_gen / wall, "prompt_tok_per_s": n_prompt / wall,
        "ttft_ms_p50": float(np.percentile(ttft, 50) * 1e3), "ttft_ms_p95": float(np.percentile(ttft, 95) * 1e3),
        "request_mean_itl_ms_p50": float(np.percentile(itl, 50) * 1e3), "request_mean_itl_ms_p95": float(np.percentile(itl, 95) * 1e3),
        "decode_thread_iterations": int(stats["iterations"]), "preemptions": int(stats["preempted"]),
    }


def summarise(c: Context, work, steps, wall: float):
    ttft, n_gen, n_prompt = [], 0, 0
    for rid, t_arr, prompt, n_out in work:
        toks, fin = c.request_output(rid)
        assert fin and len(toks) == n_out, f"request {rid}: {len(toks)} of {n_out} tokens"
        ts, tf, tl = c.request_times(rid)
        ttft.append(tf - ts)
        n_gen += len(toks)
        n_prompt += len(prompt)
    per = np.array([s[8] for s in steps if s[8] > 0]) * 1e3
    wts = np.array([s[1] for s in steps if s[8] > 0], dtype=np.float64)
    order = np.argsort(per)
    cw = np.cumsum(wts[order]) / max(wts.sum(), 1)
    q = lambda p: float(per[order][np.searchsorted(cw, p)]) if len(per) else float("nan")
    gpu = np.array([s[7] for s in steps if s[7] >= 0])
    splits, by_split = {}, {}
    for s in steps:
        if s[1] > 0:
            splits[f"{s[3]}/{s[4]}"] = splits.get(f"{s[3]}/{s[4]}", 0) + 1
            if s[8] > 0:
                by_split.setdefault(f"{s[3]}/{s[4]}", []).append(s[8] * 1e3)
    return {
        "requests": len(work), "wall_s": wall, "generated_tokens": n_gen, "prompt_tokens": n_prompt,
        "generated_tok_per_s": n_gen / wall, "prompt_tok_per_s": n_prompt / wall,
        "ttft_ms_p50": float(np.percentile(ttft, 50) * 1e3), "ttft_ms_p95": float(np.percentile(ttft, 95) * 1e3),
        "itl_ms_p50": q(0.5), "itl_ms_p95": q(0.95), "itl_ms_mean": float((per * wts).sum() / max(wts.sum(), 1)),
        "decode_step_gpu_ms_p50": float(np.percentile(gpu, 50)) if len(gpu) else None,
        "decode_steps": int(sum(1 for s in steps if s[1] > 0)), "mean_batch": float(wts.mean()) if len(wts) else 0.0,
        "max_batch": int(max((s[1] for s in steps), default=0)), "preemptions": int(sum(s[6] for s in steps)),
        "splits_used": splits,
        # host time inside rs_step_tokens for a step that enqueued a decode step and no prefill (scheduling + launches)
        "host_us_per_decode_step_p50": (lambda v: float(np.percentile(v, 50) * 1e6) if len(v) else None)(
            [s[9] for s in steps if len(s) > 9 and s[9] > 0]),
        "step_graphs": dict(zip(("captured", "launched", "steps_enqueued", "enqueue_ns_total"), c.step_graph_stats())),
        "host_launch_us_per_decode_step": (lambda g: g[3] / max(g[2], 1) / 1e3)(c.step_graph_stats()),
        "step_ms_p50_by_split": {k: float(np.percentile(v, 50)) for k, v in sorted(by_split.items())},
    }


def main(argv=None):
    import rs_synth as S
    from . import profiler
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shape", default="llama3-8b-layer", choices=sorted(S.SHAPES))
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--vocab", type=int, default=128256)
    ap.add_argument("--requests", type=int, default=48)
    ap.add_argument("--rate", type=float, default=8.0, help="arrivals per second (Poisson)")
    ap.add_argument("--prompt-mean", type=float, default=1024.0)
    ap.add_argument("--prompt-sd", type=float, default=512.0)
    ap.add_argument("--out-mean", type=float, default=128.0)
    ap.add_argument("--out-sd", type=float, default=64.0)
    ap.add_argument("--max-prompt", type=int, default=8192)
    ap.add_argument("--min-prompt", type=int, default=32)
    ap.add_argument("--max-out", type=int, default=1024)
    ap.add_argument("--max-batch", type=int, default=64)
    ap.add_argument("--kv-tokens", type=int, default=262144, help="KV pool size in tokens")
    ap.add_argument("--policy", choices=("manager", "over", "hybrid"), default="over")
    ap.add_argument("--chunk", type=int, default=512, help="--policy hybrid: prompt tokens per step (a multiple of 16)")
    ap.add_argument("--profile", default=None, help="JSON written by the profiler, or 'measure'")
    ap.add_argument("--slo-ms", type=float, default=50.0)
    ap.add_argument("--profile-ctx-edges", default="32768,131072",
                    help="with --profile measure: bucket edges of the batch's total cached tokens")
    ap.add_argument("--profile-prefill-tokens", type=int, default=2048,
                    help="with --profile measure: size of the prefill pass that runs beside the measured decode steps")
    ap.add_argument("--wait-decode", action="store_true", help="wait for each decode step (exact per-step GPU times)")
    ap.add_argument("--experts", type=int, default=0, help="sparse feed-forward block with this many experts (two per token)")
    ap.add_argument("--release-weights", action="store_true", help="free each layer's row-major matrices after packing")
    ap.add_argument("--no-step-graphs", action="store_true", help="launch each decode step's kernels one by one (rs_set_step_graphs(0))")
    ap.add_argument("--engine", action="store_true", help="let the library's two threads drive (rs_engine_start)")
    ap.add_argument("--time-limit", type=float, default=120.0)
    ap.add_argument("--seed", type=int, default=4)
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)

    shape = S.SHAPES[a.shape]
    prof = None
    if a.policy == "manager":
        if not a.profile:
            ap.error("--policy manager needs --profile")
        if a.profile == "measure":
            be = sorted({b for b in (16, 32, 64, 128, 256) if b < a.max_batch} | {a.max_batch})
            ce, dc = sorted(int(x) for x in a.profile_ctx_edges.split(",")), [32, 64, 96, 128, 160, 192]
            rig = profiler.Rig(shape, be, ce, prefill_tokens=a.profile_prefill_tokens, max_context=a.max_prompt + a.max_out,
                               experts=a.experts)
            d = profiler.profile(rig, be, ce, dc, a.layers, steps=6, warmup=2)
            rig.c.destroy()
            del rig
        else:
            d = json.load(open(a.profile))
        prof = profiler.load_profile(d, int(a.slo_ms * 1000))
    work = make_workload(a.requests, a.rate, a.prompt_mean, a.prompt_sd, a.out_mean, a.out_sd, (a.min_prompt, a.max_prompt),
                         (16, a.max_out), a.vocab, a.seed)
    t0 = time.time()
    c, keep = build_model(shape, a.layers, a.vocab, a.kv_tokens // 16, a.max_prompt, a.max_batch, a.max_prompt + a.max_out, prof,
                          release=a.release_weights, experts=a.experts)
    _log(f"[serve] model of {a.layers} layers built in {time.time() - t0:.1f}s; {a.requests} requests over "
         f"{work[-1][1]:.1f}s, {sum(len(w[2]) for w in work)} prompt tokens, {sum(w[3] for w in work)} to generate")
    if a.no_step_graphs:
        c.set_step_graphs(False)
    if a.policy == "hybrid":
        if a.engine:
            ap.error("--policy hybrid runs in the host step loop")
        c.set_hybrid_batching(a.chunk)
    # one throw-away request settles lazy runtime work (first launches, masked streams)
    settle_id = 1 << 40
    c.submit_tokens(settle_id, work[0][2][:64], 4)
    t_settle = time.time()
    while not c.step_tokens(wait_decode=True).n_finished:
        if time.time() - t_settle > 30:
            raise RuntimeError("the settling request did not finish")
    if a.engine:
        stats, wall = serve_engine(c, work, a.time_limit, max_live=4 * a.max_batch + 60)
        rec = summarise_engine(c, work, stats, wall)
    else:
        steps, wall = serve(c, work, a.wait_decode, a.time_limit, max_live=4 * a.max_batch + 60)
        rec = summarise(c, work, steps, wall)
    rec.update({"policy": a.policy, "shape": shape.name, "layers": a.layers, "rate_per_s": a.rate, "slo_ms": a.slo_ms,
                "wait_decode": bool(a.wait_decode), "driver": "engine threads" if a.engine else "host step loop", "max_batch_cap": a.max_batch, "experts": a.experts, "data": "synthetic",
                "chunk": a.chunk if a.policy == "hybrid" else None,
                "step_graphs": rec.get("step_graphs") if not a.no_step_graphs else "off"})
    line = json.dumps(rec)
    print(line, flush=True)
    if a.out:
        with open(a.out, "w") as f:
            f.write(line + "\n")
    c.destroy()
    return rec


if __name__ == "__main__":
    main()
