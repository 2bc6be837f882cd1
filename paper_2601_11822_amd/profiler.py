"""Offline profiler: measures, on this GPU, the table the adaptive resource manager reads.

Section 4.5.3 of the paper: the manager knows, from offline profiling, how the decode step
latency of a given decode load depends on the number of compute units decode is given, with a
prefill running on the others, and how it behaves when both phases are given every compute unit
(over-allocation).  Section 3.3 and the figures on decode interference show the same quantities
as curves: decode latency against compute units, prefill time against compute units, and the
slowdown of each phase when the other runs beside it.

This module runs those sweeps through the C ABI (rs_set_cu_split, rs_prefill_layer,
rs_decode_layer, timed with rs_mark / rs_mark_done) on synthetic, seeded inputs and writes

  * a JSON profile in the layout of rs_profile (batch_edges, ctx_edges, decode_cus,
    lat_distinct_us[batch][ctx][split], lat_over_us[batch][ctx]), which `load_profile` turns
    into the `Profile` that `Context(profile=...)` / rs_init take, and
  * a markdown summary with the curves.

Latencies in the table are for one decode step of the whole model: the measured step of one
layer times `n_layers` (every layer of a Llama-style stack has the same shape).

Decode loads are keyed like the manager keys them: decode batch size and total cached tokens.
A load (B, S) is profiled with B requests of S / B cached tokens each, shuffled block tables.

    python -m paper_2601_11822_amd.profiler --out profile.json --md profile.md
    python -m paper_2601_11822_amd.profiler --rows-curve [--shape ..] [--cus 256,128] [--rows ..] [--md out.md]
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from typing import Dict, List, Sequence

import numpy as np

from . import KERNEL_SLOT_NAMES, Context, Profile, timing

TOTAL_CUS = 256


def _log(*a):
    print(*a, file=sys.stderr, flush=True)


class Rig:
    """Weights, KV pools and activations of one layer, sized for the largest profiled load."""

    def __init__(self, shape, batch_edges: Sequence[int], ctx_edges: Sequence[int], prefill_tokens: int,
                 max_context: int, device: int = 0, experts: int = 0):
        import torch
        import rs_synth as S
        self.S, self.torch, self.shape = S, torch, shape
        self.T = prefill_tokens
        self.loads = []
        for b in batch_edges:
            for s in ctx_edges:
                per = max(1, min(max_context - 1, s // b))
                self.loads.append((b, s, per))
        max_tokens = max(b * (per + 1) for b, _, per in self.loads) + prefill_tokens
        self.n_blocks = max_tokens // 16 + max(batch_edges) + 64
        dev = torch.device(f"cuda:{device}")
        self.dev = dev
        wb = S.layer_weights(shape, 0)
        to_dev = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev)
        self.to_dev = to_dev
        w = {k: to_dev(v) for k, v in wb.items()}
        g = torch.Generator(device=dev)
        g.manual_seed(S.SEED_CACHE)
        Hkv, hd = shape.n_kv_heads, shape.head_dim
        self.k_pool = torch.randn((self.n_blocks, Hkv, 16, hd), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        self.v_pool = torch.randn((self.n_blocks, Hkv, hd, 16), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        self.max_batch = max(batch_edges)
        self.c = Context.from_shape(shape, max_pos=max(max_context, prefill_tokens), n_blocks=self.n_blocks,
                                    k_pool=self.k_pool, v_pool=self.v_pool, max_prefill_tokens=prefill_tokens,
                                    max_decode_batch=self.max_batch, max_context=max_context, device=device)
        self.c.set_weights(0, w["g1"], w["wqkv"], w["wo"], w["g2"], w["wg"], w["wu"], w["wd"])
        self._w = w
        if experts:   # sparse feed-forward block (random weights: only the timing matters here)
            d, f = shape.d_model, shape.ffn_dim
            rnd = lambda *sh, std=0.02: (torch.randn(sh, generator=g, device=dev, dtype=torch.float32) * std).to(torch.bfloat16)
            self._router = rnd(experts, d, std=0.1)
            self.c.set_moe_weights(0, self._router, rnd(experts, f, d), rnd(experts, f, d), rnd(experts, d, f), experts)
        self.xp = to_dev(S.hidden_states(prefill_tokens, shape.d_model, stream=0))
        self.yp = torch.empty_like(self.xp)
        self.xd = to_dev(S.hidden_states(self.max_batch, shape.d_model, stream=50))
        self.yd = torch.empty_like(self.xd)
        timing.precreate_marks(self.c)
        self.set_load(*self.loads[0])

    def set_load(self, batch: int, sum_ctx: int, per_req: int):
        S, torch = self.S, self.torch
        counts = [per_req + 1] * batch + [self.T]
        tabs = S.shuffled_block_tables(counts, self.n_blocks, max_blk=S.blocks_for(max(counts)))
        self.B, self.max_ctx, self.max_blk = batch, per_req + 1, tabs.shape[1]
        self.dtab = torch.from_numpy(tabs[:batch].copy()).to(self.dev)
        self.ptab = torch.from_numpy(tabs[batch:batch + 1].copy()).to(self.dev)
        self.cl = torch.full((batch,), per_req, dtype=torch.int32, device=self.dev)
        torch.cuda.synchronize()

    def enqueue_prefill(self):
        self.c.prefill_layer(0, self.xp, self.yp, [0, self.T], self.ptab, self.max_blk)

    def enqueue_decode(self):
        self.c.decode_layer(0, self.xd, self.yd, self.cl, self.dtab, self.max_blk, self.B, self.max_ctx)


def _itl_corun(rig: Rig, steps: int, warmup: int):
    """(decode step p50 ms, prefill pass ms) with both sides running; measured again (at most twice) if a host call stalled inside the timed window."""
    out = None
    for _ in range(3):
        out = timing.run_corun(rig.c, rig.enqueue_prefill, rig.enqueue_decode, steps, warmup)
        if not out[4]:
            break
    wall_ms, _, d_in, n_dec, _ = out
    itl = float(np.percentile(d_in, 50)) if len(d_in) else wall_ms / max(n_dec, 1)
    return itl, wall_ms / steps


def profile(rig: Rig, batch_edges: Sequence[int], ctx_edges: Sequence[int], decode_cus: Sequence[int], n_layers: int,
            steps: int = 10, warmup: int = 2) -> Dict:
    c = rig.c
    nb, nc, ns = len(batch_edges), len(ctx_edges), len(decode_cus)
    lat_distinct = np.zeros((nb, nc, ns), dtype=np.int64)
    lat_over = np.zeros((nb, nc), dtype=np.int64)
    curves: List[Dict] = []
    t0 = time.time()
    # the run that settles the runtime (see timing.run_corun) once, outside the table
    c.set_cu_split(TOTAL_CUS // 2, TOTAL_CUS // 2)
    timing.run_corun(c, rig.enqueue_prefill, rig.enqueue_decode, 30, 5)
    for bi, b in enumerate(batch_edges):
        for ci, s in enumerate(ctx_edges):
            per = max(1, min(c.max_context - 1, s // b))
            rig.set_load(b, s, per)
            c.set_cu_split(TOTAL_CUS, TOTAL_CUS)
            d_alone_full = float(np.median(timing.run_alone(c, 1, rig.enqueue_decode, 20, 3)[0]))
            itl, p_ms = _itl_corun(rig, steps, warmup)
            lat_over[bi, ci] = int(round(itl * 1e3 * n_layers))
            rec = {"batch": b, "sum_ctx": b * per, "ctx_per_request": per, "decode_alone_256_ms": d_alone_full,
                   "over": {"itl_ms": itl, "prefill_ms": p_ms}, "splits": []}
            for si, dc in enumerate(decode_cus):
                c.set_cu_split(TOTAL_CUS - dc, dc)
                d_alone = float(np.median(timing.run_alone(c, 1, rig.enqueue_decode, 20, 3)[0]))
                p_alone = float(np.median(timing.run_alone(c, 0, rig.enqueue_prefill, 5, 2)[0]))
                itl, p_ms = _itl_corun(rig, steps, warmup)
                lat_distinct[bi, ci, si] = int(round(itl * 1e3 * n_layers))
                rec["splits"].append({"decode_cus": dc, "prefill_cus": TOTAL_CUS - dc, "decode_alone_ms": d_alone,
                                      "prefill_alone_ms": p_alone, "itl_ms": itl, "prefill_ms": p_ms})
            curves.append(rec)
            _log(f"[profiler] batch {b} sum_ctx {b * per}: over {lat_over[bi, ci]} us; "
                 f"distinct {lat_distinct[bi, ci].tolist()} us  ({time.time() - t0:.0f}s)")
    return {
        "batch_edges": list(map(int, batch_edges)), "ctx_edges": list(map(int, ctx_edges)),
        "decode_cus": list(map(int, decode_cus)), "lat_distinct_us": lat_distinct.tolist(),
        "lat_over_us": lat_over.tolist(),
        "meta": {"shape": rig.shape.name, "n_layers": n_layers, "prefill_tokens": rig.T, "steps": steps,
                 "unit": "microseconds per decode step of the whole model (one layer x n_layers), p50 under co-run"},
        "curves": curves,
    }


def load_profile(path_or_dict, slo_us: int) -> Profile:
    d = path_or_dict if isinstance(path_or_dict, dict) else json.load(open(path_or_dict))
    return Profile(d["batch_edges"], d["ctx_edges"], d["decode_cus"], d["lat_distinct_us"], d["lat_over_us"], slo_us)


def to_markdown(d: Dict) -> str:
    m = d["meta"]
    out = [f"# Offline profile of the decode step against the CU split ({m['shape']}, prefill of {m['prefill_tokens']} tokens beside it)\n",
           "Written by `python -m paper_2601_11822_amd.profiler` (command at the end).  Milliseconds for ONE layer; the",
           f"manager's table holds the same co-run latencies x {m['n_layers']} layers in microseconds.\n"]
    for rec in d["curves"]:
        out.append(f"## decode batch {rec['batch']}, {rec['sum_ctx']} cached tokens ({rec['ctx_per_request']} per request); "
                   f"decode alone on 256 CUs {rec['decode_alone_256_ms']:.3f} ms\n")
        out.append("| decode CUs | prefill CUs | decode alone | decode beside prefill (ITL p50) | slowdown | prefill alone | prefill beside decode | slowdown |")
        out.append("|---:|---:|---:|---:|---:|---:|---:|---:|")
        for s in rec["splits"]:
            out.append(f"| {s['decode_cus']} | {s['prefill_cus']} | {s['decode_alone_ms']:.3f} | {s['itl_ms']:.3f} | "
                       f"{s['itl_ms'] / s['decode_alone_ms']:.2f} | {s['prefill_alone_ms']:.3f} | {s['prefill_ms']:.3f} | "
                       f"{s['prefill_ms'] / s['prefill_alone_ms']:.2f} |")
        o = rec["over"]
        out.append(f"| 256 (shared) | 256 (shared) | {rec['decode_alone_256_ms']:.3f} | {o['itl_ms']:.3f} | "
                   f"{o['itl_ms'] / rec['decode_alone_256_ms']:.2f} | | {o['prefill_ms']:.3f} | |\n")
    return "\n".join(out)


def main(argv=None):
    import rs_synth as S
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--shape", default="llama3-8b-layer", choices=sorted(S.SHAPES))
    ap.add_argument("--n-layers", type=int, default=32, help="layers of the model the one-layer latency is scaled to")
    ap.add_argument("--batch-edges", default="16,64")
    ap.add_argument("--ctx-edges", default="32768,131072,262144", help="totals of cached tokens")
    ap.add_argument("--decode-cus", default="32,64,96,128,160,192,224")
    ap.add_argument("--prefill-tokens", type=int, default=2048)
    ap.add_argument("--max-context", type=int, default=16385)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--out", default="profile.json")
    ap.add_argument("--md", default=None)
    a = ap.parse_args(argv)
    ints = lambda s: [int(v) for v in s.split(",")]
    be, ce, dc = ints(a.batch_edges), ints(a.ctx_edges), ints(a.decode_cus)
    rig = Rig(S.SHAPES[a.shape], be, ce, a.prefill_tokens, a.max_context)
    d = profile(rig, be, ce, dc, a.n_layers, steps=a.steps)
    d["meta"]["command"] = "python -m paper_2601_11822_amd.profiler " + " ".join(sys.argv[1:] if argv is None else argv)
    with open(a.out, "w") as f:
        json.dump(d, f)
    if a.md:
        with open(a.md, "w") as f:
            f.write(to_markdown(d) + "\nCommand: `" + d["meta"]["command"] + "`\n")
    print(json.dumps({k: d[k] for k in ("batch_edges", "ctx_edges", "decode_cus", "lat_distinct_us", "lat_over_us")}))


def rows_curve(argv=None):
    """Layer time against the number of rows in the pass, per CU partition (`--rows-curve` as the first
    argument): one layer, one prompt of T tokens, per-kernel events, for T from a few dozen rows to the
    largest pass, on the whole chip and on a partition; shows where each GEMM path takes over.  With
    --experts E the feed-forward block is the sparse one (the Mixtral-8x7B shape is `--shape
    llama3-8b-layer --experts 8`); with --decode B1,B2,.. decode steps of those batch sizes (1024 cached
    tokens per request) are timed too."""
    import torch
    import rs_synth as S
    ap = argparse.ArgumentParser(description=rows_curve.__doc__)
    ap.add_argument("--shape", default="llama3-8b-layer", choices=sorted(S.SHAPES))
    ap.add_argument("--cus", default="256,128")
    ap.add_argument("--rows", default="32,64,65,128,256,384,512,768,1024,1536,2048,3000,4096,8192")
    ap.add_argument("--md", default=None)
    ap.add_argument("--experts", type=int, default=0)
    ap.add_argument("--decode", default="")
    a = ap.parse_args(argv)
    shape = S.SHAPES[a.shape]
    rows = [int(v) for v in a.rows.split(",")]
    t_max = max(rows)
    dec = [int(v) for v in a.decode.split(",")] if a.decode else []
    dec_ctx = 1024
    nb = t_max // 16 + 8 + sum(dec_ctx // 16 + 1 for _ in range(max(dec, default=0)))
    dev = torch.device("cuda:0")
    kp = torch.zeros((1, nb, shape.n_kv_heads, 16, shape.head_dim), dtype=torch.bfloat16, device=dev)
    vp = torch.zeros((1, nb, shape.n_kv_heads, shape.head_dim, 16), dtype=torch.bfloat16, device=dev)
    c = Context.from_shape(shape, n_layers=1, max_pos=max(t_max, dec_ctx + 16), n_blocks=nb, k_pool=kp, v_pool=vp,
                           max_prefill_tokens=t_max, max_decode_batch=max(dec + [4]), max_context=max(t_max, dec_ctx + 16), device=0)
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    rnd = lambda *s, std=0.02, mean=0.0: (torch.randn(s, generator=g, device=dev) * std + mean).to(torch.bfloat16)
    d, f = shape.d_model, shape.ffn_dim
    if a.experts:
        w = (rnd(d, mean=1.0), rnd(shape.qkv_dim, d), rnd(d, shape.q_dim), rnd(d, mean=1.0), None, None, None)
        c.set_weights(0, *w)
        E = a.experts
        router = rnd(E, d, std=0.1)
        c.set_moe_weights(0, router, rnd(E, f, d), rnd(E, f, d), rnd(E, d, f), E)
    else:
        w = (rnd(d, mean=1.0), rnd(shape.qkv_dim, d), rnd(d, shape.q_dim), rnd(d, mean=1.0), rnd(f, d), rnd(f, d), rnd(d, f))
        c.set_weights(0, *w)
    tab = torch.arange(nb, dtype=torch.int32, device=dev).reshape(1, -1)
    c.set_kernel_timing(True)
    p_layer = d * shape.qkv_dim + d * shape.q_dim + 3 * d * f * (2 if a.experts else 1)   # active parameters per row
    lines = ["| CUs | rows | ms | M tok/s | TFLOP/s | " + " | ".join(n for n in KERNEL_SLOT_NAMES) + " |",
             "|---|---|---|---|---|" + "---|" * len(KERNEL_SLOT_NAMES)]
    for cus in [int(v) for v in a.cus.split(",")]:
        c.set_cu_split(cus, 256 if cus == 256 else 256 - cus)
        for T in rows:
            x = rnd(T, d, std=1.0)
            y = torch.empty_like(x)
            torch.cuda.synchronize()
            for _ in range(2):
                c.prefill_layer(0, x, y, [0, T], tab, nb)
            c.mark(0, 0)
            n = 5
            for _ in range(n):
                c.prefill_layer(0, x, y, [0, T], tab, nb)
            c.mark(0, 1)
            ms = c.elapsed_ms(0, 0, 1) / n
            kt = c.kernel_times(0)
            flops = 2 * T * p_layer + 2 * shape.n_q_heads * shape.head_dim * T * (T + 1)
            line = (f"| {cus} | {T} | {ms:.3f} | {T / ms / 1e3:.2f} | {flops / ms / 1e9:.0f} | "
                    + " | ".join(f"{v * 1e3:.0f}" for v in kt) + " |")
            lines.append(line)
            print(line, file=sys.stderr, flush=True)
    if dec:
        lines += ["", "| CUs | decode batch | ms | " + " | ".join(n for n in KERNEL_SLOT_NAMES) + " |",
                  "|---|---|---|" + "---|" * len(KERNEL_SLOT_NAMES)]
        per_req = dec_ctx // 16 + 1
        for cus in [int(v) for v in a.cus.split(",")]:
            c.set_cu_split(256 if cus == 256 else 256 - cus, cus)
            for B in dec:
                tabs = (t_max // 16 + 8 + torch.arange(B * per_req, dtype=torch.int32, device=dev)).reshape(B, per_req)
                cl = torch.full((B,), dec_ctx, dtype=torch.int32, device=dev)
                x = rnd(B, d, std=1.0)
                y = torch.empty_like(x)
                torch.cuda.synchronize()
                for _ in range(3):
                    c.decode_layer(0, x, y, cl, tabs, per_req, B, dec_ctx + 1)
                c.mark(1, 0)
                n = 20
                for _ in range(n):
                    c.decode_layer(0, x, y, cl, tabs, per_req, B, dec_ctx + 1)
                c.mark(1, 1)
                ms = c.elapsed_ms(1, 0, 1) / n
                kt = c.kernel_times(1)
                line = f"| {cus} | {B} | {ms:.3f} | " + " | ".join(f"{v * 1e3:.0f}" for v in kt) + " |"
                lines.append(line)
                print(line, file=sys.stderr, flush=True)
    out = "\n".join(lines)
    print(out)
    if a.md:
        with open(a.md, "w") as fh:
            fh.write(out + "\n")
    c.destroy()



if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "--rows-curve":
        rows_curve(sys.argv[2:])
        sys.exit(0)
    main()
