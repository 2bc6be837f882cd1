"""Helpers for the GPU parity tests: device buffers via torch, calls through the C-ABI binding,
and the error metric of the parity bar."""
import math

import numpy as np
import torch

import oracle
import paper_2601_11822_amd as rs
import rs_synth as S

TOL = 2e-2  # max relative error for bf16 activations with fp32 accumulation


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 device tensor holding exactly those bits."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).copy())
    return t.view(torch.bfloat16).cuda()


def to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def rel_err(got_f32: np.ndarray, ref_f32: np.ndarray) -> float:
    """Element-wise relative error max_i |got_i - ref_i| / max(|ref_i|, rms(ref row of i)): the
    denominator is floored at the rms of the element's own row (one token's vector), so that
    near-zero elements do not blow it up and rows of different scale are judged on their own."""
    ref = np.atleast_2d(ref_f32.astype(np.float64))
    got = np.atleast_2d(got_f32.astype(np.float64))
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    den = np.maximum(np.abs(ref), np.maximum(rms, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


Q = 2.0 ** -8   # half an ulp of bf16 (8 significant bits) relative to the value, at most


def tensor_fracs(got, ref, x=None, roundings=0, elem_mult=1.0, layers=1):
    """The parity bar for one activation tensor, as fractions of what is allowed (<= 1 passes).

    `got` was computed with bf16 operands and fp32 accumulation, `ref` by the fp32 oracle.  With
    e = got - ref (for a residual-stream tensor, x given: e is the error of the branch delta
    got - x against ref - x):
      max   : max|e| <= TOL * max|ref|            the stated bound: max relative error 2e-2
      rms   : rms(e) <= TOL/2 * rms(ref)          the bulk of the tensor, twice as tight
      elem  : |e_i|  <= elem_mult * TOL * max(|ref_i|, rms(ref row))   no element far off on its own
              row's scale.  elem_mult is 1 (the stated 2e-2, element by element) wherever the
              reference was computed from the SAME operands the kernel read (the own-operand stage
              checks, and every tensor upstream of the softmax); it is 3 only where the fp32 oracle's
              end-to-end value is compared downstream of the softmax, because the oracle keeps q and k
              in fp32 while the kernels store them in bf16, which sharply peaked softmax rows amplify.
    For residual-stream tensors each bound is widened by `roundings` half-ulps of bf16 at the
    stored value (Q*|y|; Q*rms(y)/sqrt(3) in the rms bound): the hidden state is STORED in bf16,
    so the delta cannot resolve finer than that whatever the branch computes.
    elem_mult=None leaves the per-element bound out (max and rms only).  layers=n is for the output
    of a stack of n layers compared end to end: each layer's branch adds its own error and passes
    the error of its input on with unit gain along the residual path, so to first order the errors
    add and the three bounds are n times those of one layer."""
    ref = np.atleast_2d(np.asarray(ref, np.float64))
    got = np.atleast_2d(np.asarray(got, np.float64))
    if x is not None:
        x = np.atleast_2d(np.asarray(x, np.float64))
        y_ref = ref
        ref, got = ref - x, got - x
    e = np.abs(got - ref)
    rms_all = max(float(np.sqrt(np.mean(ref * ref))), 1e-30)
    row_rms = np.maximum(np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True)), 1e-30)
    q_max = q_rms = 0.0
    q_el = 0.0
    if x is not None and roundings:
        q_max = roundings * Q * float(np.max(np.abs(y_ref)))
        q_rms = math.sqrt(roundings) * Q / math.sqrt(3.0) * float(np.sqrt(np.mean(y_ref * y_ref)))
        q_el = roundings * Q * np.abs(y_ref)
    tol = TOL * layers
    out = {
        "max": float(e.max() / (tol * float(np.max(np.abs(ref))) + q_max)),
        "rms": float(np.sqrt(np.mean(e * e)) / (tol / 2 * rms_all + q_rms)),
    }
    if elem_mult is not None:
        out["elem"] = float(np.max(e / (elem_mult * tol * np.maximum(np.abs(ref), row_rms) + q_el)))
    return out


END_TO_END = 3.0   # elem_mult of the fp32-oracle comparisons downstream of the softmax (see tensor_fracs)


def check_tensor(name, got, ref, x=None, roundings=0, elem_mult=1.0, layers=1):
    f = tensor_fracs(got, ref, x, roundings, elem_mult, layers)
    print(f"  {name}: fractions of allowed error " + ", ".join(f"{k} {v:.3f}" for k, v in f.items()), flush=True)
    for k, v in f.items():
        assert v <= 1.0, f"{name}: {k} error is {v:.3f} of the allowed"
    return f


def residual_err(y_got, y_ref, x, roundings: int = 2, elem_mult: float = END_TO_END, layers: int = 1) -> float:
    """Worst of the three fractions for a residual-stream output against the fp32 oracle's
    end-to-end value (see tensor_fracs)."""
    return max(tensor_fracs(y_got, y_ref, x, roundings, elem_mult, layers).values())


class Rig:
    """One layer stack on the GPU with its pools, plus the matching oracle layers."""

    def __init__(self, shape, n_blocks, max_prefill_tokens, max_decode_batch, max_context, n_layers=1,
                 sentinel=0x7FC1, profile=None, with_oracle=True, max_pos=None, wo_std=None, wd_std=None):
        self.shape, self.n_blocks, self.n_layers = shape, n_blocks, n_layers
        self.sentinel = sentinel
        Hkv, hd = shape.n_kv_heads, shape.head_dim
        self.k_pool = torch.empty((n_layers, n_blocks, Hkv, 16, hd), dtype=torch.bfloat16, device="cuda")
        self.v_pool = torch.empty((n_layers, n_blocks, Hkv, hd, 16), dtype=torch.bfloat16, device="cuda")
        self.k_pool.view(torch.int16).fill_(int(np.array(sentinel, np.uint16).view(np.int16)))
        self.v_pool.view(torch.int16).fill_(int(np.array(sentinel, np.uint16).view(np.int16)))
        self.ctx = rs.Context.from_shape(shape, n_layers=n_layers, max_pos=max_pos or max(max_context, max_prefill_tokens, 1),
                                         n_blocks=n_blocks, k_pool=self.k_pool, v_pool=self.v_pool,
                                         max_prefill_tokens=max_prefill_tokens, max_decode_batch=max_decode_batch,
                                         max_context=max_context, profile=profile, device=0)
        self.wbits, self.wdev, self.olayers = [], [], []
        self._keep = []   # device tensors of enqueued calls stay alive until the rig is closed
        for l in range(n_layers):
            wb = S.layer_weights(shape, l, wo_std=wo_std, wd_std=wd_std)
            wd = {k: to_dev(v) for k, v in wb.items()}
            self.ctx.set_weights(l, wd["g1"], wd["wqkv"], wd["wo"], wd["g2"], wd["wg"], wd["wu"], wd["wd"])
            self.wbits.append(wb); self.wdev.append(wd)
            if with_oracle:
                self.olayers.append(oracle.OracleLayer.from_shape(shape, wb))

    def close(self):
        self.ctx.destroy()
        self._keep.clear()

    # ---- GPU calls
    def prefill(self, x_bits, cu, tables, layer=0, sync=True):
        x = to_dev(x_bits)
        y = torch.empty_like(x)
        tab = torch.from_numpy(np.ascontiguousarray(tables, dtype=np.int32)).cuda()
        torch.cuda.synchronize()
        self.ctx.prefill_layer(layer, x, y, cu, tab, tab.shape[1])
        self._keep.append((x, y, tab))
        if sync:
            self.ctx.sync(rs.RS_SIDE_PREFILL)
            return to_bits(y)
        return y

    def decode(self, x_bits, ctx_lens, tables, layer=0, max_ctx=None, sync=True):
        x = to_dev(x_bits)
        y = torch.empty_like(x)
        cl = torch.from_numpy(np.ascontiguousarray(ctx_lens, dtype=np.int32)).cuda()
        tab = torch.from_numpy(np.ascontiguousarray(tables, dtype=np.int32)).cuda()
        if max_ctx is None:
            max_ctx = int(np.max(ctx_lens)) + 1
        torch.cuda.synchronize()
        self.ctx.decode_layer(layer, x, y, cl, tab, tab.shape[1], x.shape[0], max_ctx)
        self._keep.append((x, y, cl, tab))
        if sync:
            self.ctx.sync(rs.RS_SIDE_DECODE)
            return to_bits(y)
        return y

    def hybrid(self, x_bits, cu, start_pos, ptables, ctx_lens=None, dtables=None, layer=0, max_ctx=None):
        """One hybrid batch: chunk rows of the prompts first, then the decode rows."""
        x = to_dev(x_bits)
        y = torch.empty_like(x)
        ptab = torch.from_numpy(np.ascontiguousarray(ptables, dtype=np.int32)).cuda()
        B = 0 if ctx_lens is None else len(ctx_lens)
        cl = dtab = None
        if B:
            cl = torch.from_numpy(np.ascontiguousarray(ctx_lens, dtype=np.int32)).cuda()
            dtab = torch.from_numpy(np.ascontiguousarray(dtables, dtype=np.int32)).cuda()
            if max_ctx is None:
                max_ctx = int(np.max(ctx_lens)) + 1
        torch.cuda.synchronize()
        self.ctx.hybrid_layer(layer, x, y, cu, start_pos, ptab, ptab.shape[1], cl, dtab, dtab.shape[1] if B else 0, B,
                              max_ctx or 1)
        self._keep.append((x, y, ptab, cl, dtab))
        self.ctx.sync(rs.RS_SIDE_PREFILL)
        return to_bits(y)

    # ---- pools in the oracle's logical order [n_blocks, 16, Hkv, hd]
    # K pool: [n_blocks][Hkv][hd/32][4][16 permuted slots][8]; slot t sits in row t with bits 2, 3 swapped
    _PROW = [(t & 3) | ((t & 8) >> 1) | ((t & 4) << 1) for t in range(16)]

    def k_bits_logical(self, layer=0):
        nb, Hkv, _, hd = self.k_pool[layer].shape
        k = self.k_pool[layer].reshape(nb, Hkv, hd // 32, 4, 16, 8)[:, :, :, :, self._PROW, :]   # -> slot order
        return to_bits(k.permute(0, 4, 1, 2, 3, 5).reshape(nb, 16, Hkv, hd).contiguous())

    def v_bits_logical(self, layer=0):
        return to_bits(self.v_pool[layer].permute(0, 3, 1, 2).contiguous())

    def load_pools_from_logical(self, k_bits, v_bits, layer=0):
        """k_bits, v_bits: uint16 [n_blocks,16,Hkv,hd] -> device pools in the library's layouts."""
        nb, Hkv, _, hd = self.k_pool[layer].shape
        k = to_dev(k_bits).reshape(nb, 16, Hkv, hd // 32, 4, 8).permute(0, 2, 3, 4, 1, 5)   # [nb,Hkv,s,kh,slot,8]
        inv = [self._PROW.index(r) for r in range(16)]                                        # row r holds slot inv[r]
        self.k_pool[layer].copy_(k[:, :, :, :, inv, :].reshape(nb, Hkv, 16, hd))
        self.v_pool[layer].copy_(to_dev(v_bits).permute(0, 2, 3, 1))


def check_cache_against_oracle(rig, Kc, Vc, oracle_sentinel, layer=0):
    """Bit-exact indexing: the set of slots the GPU dirtied equals the oracle's set; dirtied
    contents match to tolerance."""
    kb, vb = rig.k_bits_logical(layer), rig.v_bits_logical(layer)
    for bits, ref in ((kb, Kc), (vb, Vc)):
        dirty_gpu = bits != np.uint16(rig.sentinel)
        dirty_ref = ref != np.float32(oracle_sentinel)
        assert np.array_equal(dirty_gpu, dirty_ref), "set of written cache slots differs from the oracle"
        if dirty_ref.any():
            got = S.bf16_bits_to_f32(bits)[dirty_ref]
            e = rel_err(got, ref[dirty_ref])
            assert e <= TOL, f"cache contents rel err {e}"


def gather_prompt_kv(rig, cu, tables, layer=0):
    """K and V of every prompt token as the GPU cache holds them (bf16 widened), [T, Hkv, hd] each,
    gathered through the block tables: the operands the prefill attention kernel really read."""
    kb, vb = rig.k_bits_logical(layer), rig.v_bits_logical(layer)
    T = int(cu[-1])
    k = np.zeros((T,) + kb.shape[2:], np.float32)
    v = np.zeros_like(k)
    for r in range(len(cu) - 1):
        a, b = int(cu[r]), int(cu[r + 1])
        pos = np.arange(b - a)
        blk = np.asarray(tables)[r, pos // 16]
        k[a:b] = S.bf16_bits_to_f32(kb[blk, pos % 16])
        v[a:b] = S.bf16_bits_to_f32(vb[blk, pos % 16])
    return k, v


def check_stages_own_operands(rig, side, L, M, x, y_bits, *, cu=None, tables=None, ctx=None, rows=None, layer=0):
    """Every stage downstream of the QKV projection against the oracle's routine for that stage fed
    the operands the kernel itself read (its own bf16 intermediates, read back through
    rs_debug_read_workspace, and the cache bits): element by element at the stated 2e-2, so that the
    rounding of stored intermediates is outside the budget and a kernel error of a few per cent of
    an element cannot hide.  Prefill: cu and tables given; decode: ctx and tables.  `rows` limits
    the evaluation to those rows (large shapes)."""
    f32 = S.bf16_bits_to_f32
    sh = rig.shape
    qd = sh.q_dim
    rd = lambda which, width: f32(rig.ctx.debug_read_workspace(side, which, (M, width)))
    q = rd(1, sh.qkv_dim)[:, :qd]
    attn, x1, act = rd(2, qd), rd(3, sh.d_model), rd(4, sh.ffn_dim)
    try:
        h2 = rd(0, sh.d_model)
    except rs.RapidServeError as e:
        # a decode step that folded the second RMSNorm into the gate/up projection wrote no normalised rows: the
        # stage that reads x1 is then RMSNorm + gate/up + SwiGLU as one, checked as one
        assert e.code == rs.RS_ERR_STATE
        h2 = None
    y = f32(y_bits)
    sel = np.arange(M) if rows is None else np.asarray(rows)
    if ctx is None:
        k, v = gather_prompt_kv(rig, cu, tables, layer)
        a_ref = oracle.attn_causal(q.reshape(M, sh.n_q_heads, sh.head_dim), k, v, cu, rows=rows).reshape(M, qd)
    else:
        a_ref = oracle.attn_paged(q.reshape(M, sh.n_q_heads, sh.head_dim), f32(rig.k_bits_logical(layer)),
                                  f32(rig.v_bits_logical(layer)), tables, np.asarray(ctx, np.int32) + 1).reshape(M, qd)
    out = {}
    out["attn"] = check_tensor("own operands: attention(q, cached K/V as stored)", attn[sel], a_ref[sel])
    out["x1"] = check_tensor("own operands: x + attn Wo", x1[sel], x[sel] + L.project("wo", attn[sel]), x[sel], 1)
    if h2 is not None:
        out["h2"] = check_tensor("own operands: RMSNorm(x1)", h2[sel], L.norm(2, x1[sel]))
        h2s = h2[sel]
    else:
        # The folded stage stages x1 . g2 ROUNDED TO BF16 as its GEMM operand and applies the row's scale
        # 1/sqrt(mean(x1^2) + eps) to the float32 products: the operand the kernel read is that rounded product.
        # The projection is linear, so the oracle's routines are fed it times the scale; the scale itself is tied
        # to the oracle's RMSNorm (equal to it up to the operand's bf16 rounding).
        g2 = f32(rig.wbits[layer]["g2"]).astype(np.float32)
        hg = f32(S.f32_to_bf16_bits((x1[sel] * g2[None, :]).astype(np.float32)))
        inv = 1.0 / np.sqrt(np.mean(x1[sel].astype(np.float64) ** 2, axis=1, keepdims=True) + sh.rms_eps)
        h2s = (hg * inv).astype(np.float32)
        h2_orc = L.norm(2, x1[sel])
        assert np.abs(h2s - h2_orc).max() <= 2.0 ** -8 * np.abs(h2_orc).max() + 1e-6
    out["act"] = check_tensor("own operands: silu(h2 Wg) * (h2 Wu)" + ("" if h2 is not None else ", h2 = RMSNorm(x1) folded in"),
                              act[sel], oracle.silu_mul(L.project("wg", h2s), L.project("wu", h2s)))
    out["y"] = check_tensor("own operands: x1 + act Wd", y[sel], x1[sel] + L.project("wd", act[sel]), x1[sel], 1)
    return out
