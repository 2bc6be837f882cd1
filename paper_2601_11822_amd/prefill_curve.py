"""Prefill layer time against the number of rows in the pass, per CU partition.

One Llama-shaped layer (random weights, one prompt of T tokens, synthetic hidden states), timed
through the C ABI with per-kernel events, for T from a few dozen rows (a single short prompt) to
the largest pass, on the whole chip and on a partition.  Shows where each GEMM path takes over:
up to 64 rows the weight-streaming kernels, above that the large-tile kernel with a sliced K range
while the output has few tiles.

    python -m paper_2601_11822_amd.prefill_curve [--shape llama3-8b-layer] [--cus 256,128] [--md out.md]

With --experts E the layer's feed-forward block is the sparse one (E experts of the shape's FFN
width, two per row): the Mixtral-8x7B shape is `--shape llama3-8b-layer --experts 8`.  With
--decode B1,B2,.. decode steps of those batch sizes (1024 cached tokens per request) are timed too.
"""
from __future__ import annotations

import argparse
import sys

import numpy as np

from . import Context, KERNEL_SLOT_NAMES


def main(argv=None):
    import torch
    import rs_synth as S
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
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
    main()
