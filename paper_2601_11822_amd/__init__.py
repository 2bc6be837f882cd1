"""Thin Python binding of librapid_serve.so (the C ABI in include/rapid_serve.h).

Only argument marshalling happens here: every step of the prefill/decode path runs in the
library's HIP kernels.  PyTorch is used by callers for device memory; this module takes raw
device pointers (`tensor.data_ptr()`).  There is no CPU fallback: a missing library is an
ImportError-like failure at first use.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librapid_serve.so")

RS_OK = 0
RS_ERR_BAD_ARG, RS_ERR_NO_BLOCKS, RS_ERR_BAD_SPLIT, RS_ERR_BAD_BLOCK, RS_ERR_HIP, RS_ERR_STATE = -1, -2, -3, -4, -5, -6
RS_SIDE_PREFILL, RS_SIDE_DECODE = 0, 1
RS_TOTAL_CUS, RS_CU_GRANULE, RS_KV_BLOCK, RS_MAX_PREFILL_REQS, RS_HOST_ONLY = 256, 32, 16, 64, -1
RS_MAX_MARKS = 4096
RS_N_KERNEL_SLOTS = 8
KERNEL_SLOT_NAMES = ("rmsnorm1", "qkv_gemm", "rope_kvwrite", "attention", "o_gemm", "rmsnorm2",
                     "gateup_swiglu_gemm", "down_gemm")
RS_CU_HIST_BINS = 4096

EXPORTS = [
    "rs_init", "rs_destroy", "rs_set_weights", "rs_last_error", "rs_kv_alloc", "rs_kv_free",
    "rs_kv_num_free", "rs_prefill_layer", "rs_decode_layer", "rs_decode_layer_noalloc", "rs_hybrid_layer", "rs_set_hybrid_batching", "rs_step_chunks", "rs_set_cu_split", "rs_get_cu_split",
    "rs_get_cu_mask", "rs_choose_split", "rs_get_stream", "rs_sync", "rs_mark", "rs_mark_done", "rs_elapsed_ms", "rs_decode_layer_graph", "rs_debug_cu_histogram_graph", "rs_decode_batch_ids", "rs_set_kernel_timing", "rs_kernel_times",
    "rs_debug_cu_histogram", "rs_debug_read_workspace", "rs_debug_stream_read", "rs_debug_mfma_probe", "rs_submit", "rs_step", "rs_request_state", "rs_debug_complete_prefill",
    "rs_set_head", "rs_embed", "rs_lm_head_greedy", "rs_submit_tokens", "rs_step_tokens", "rs_request_output",
    "rs_debug_push_sampled", "rs_request_times", "rs_request_release", "rs_set_step_graphs", "rs_step_graph_stats", "rs_engine_start", "rs_engine_stop", "rs_engine_stats", "rs_release_source_weights", "rs_set_moe_weights", "rs_debug_read_moe_routing",
]


class RapidServeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"rapid_serve error {code}: {msg}")
        self.code = code


class ModelDesc(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("ffn_dim", ctypes.c_int32), ("n_layers", ctypes.c_int32),
                ("rms_eps", ctypes.c_float), ("rope_base", ctypes.c_float), ("max_pos", ctypes.c_int32)]


class PoolDesc(ctypes.Structure):
    _fields_ = [("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p), ("layer_stride", ctypes.c_int64),
                ("n_blocks", ctypes.c_int32)]


class Limits(ctypes.Structure):
    _fields_ = [("max_prefill_tokens", ctypes.c_int32), ("max_decode_batch", ctypes.c_int32),
                ("max_context", ctypes.c_int32)]


_i32p = ctypes.POINTER(ctypes.c_int32)


class ProfileDesc(ctypes.Structure):
    _fields_ = [("n_batch", ctypes.c_int32), ("n_ctx", ctypes.c_int32), ("n_split", ctypes.c_int32),
                ("batch_edges", _i32p), ("ctx_edges", _i32p), ("decode_cus", _i32p),
                ("lat_distinct_us", _i32p), ("lat_over_us", _i32p), ("slo_us", ctypes.c_int32)]


class LayerWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("g1", "wqkv", "wo", "g2", "wg", "wu", "wd")]


class StepIn(ctypes.Structure):
    _fields_ = [("decode_hidden", ctypes.c_void_p), ("decode_out", ctypes.c_void_p),
                ("wait_decode", ctypes.c_int32)]


class StepOut(ctypes.Structure):
    _fields_ = [("prefill_cus", ctypes.c_int32), ("decode_cus", ctypes.c_int32), ("decode_batch", ctypes.c_int32),
                ("decode_sum_ctx", ctypes.c_int64), ("prefill_started_tokens", ctypes.c_int32),
                ("prefill_started_req", ctypes.c_int64), ("n_promoted", ctypes.c_int32),
                ("n_finished", ctypes.c_int32), ("n_waiting", ctypes.c_int32), ("decode_ms", ctypes.c_float),
                ("n_preempted", ctypes.c_int32), ("prefill_started_count", ctypes.c_int32),
                ("n_chunks", ctypes.c_int32), ("chunk_tokens", ctypes.c_int32)]


class MoeWeights(ctypes.Structure):
    _fields_ = [("router", ctypes.c_void_p), ("wg", ctypes.c_void_p), ("wu", ctypes.c_void_p), ("wd", ctypes.c_void_p),
                ("n_experts", ctypes.c_int32), ("top_k", ctypes.c_int32)]


class HeadWeights(ctypes.Structure):
    _fields_ = [("embed", ctypes.c_void_p), ("final_norm", ctypes.c_void_p), ("lm_head", ctypes.c_void_p),
                ("vocab", ctypes.c_int32), ("eos_token", ctypes.c_int32)]


_lib: Optional[ctypes.CDLL] = None


def load() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(LIB_PATH)
        lib.rs_last_error.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name != "rs_last_error":
                getattr(lib, name).restype = ctypes.c_int32
        _lib = lib
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise RapidServeError(rc, load().rs_last_error().decode())
    return rc


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(x) -> ctypes.c_void_p:
    """Device pointer of a torch tensor (or an int address)."""
    if x is None:
        return ctypes.c_void_p(0)
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    return ctypes.c_void_p(x.data_ptr())


class Profile:
    """Host-side offline profile for the manager (see rs_profile)."""

    def __init__(self, batch_edges, ctx_edges, decode_cus, lat_distinct_us, lat_over_us, slo_us: int):
        self.batch_edges, self.ctx_edges, self.decode_cus = _i32(batch_edges), _i32(ctx_edges), _i32(decode_cus)
        self.lat_distinct_us, self.lat_over_us = _i32(lat_distinct_us), _i32(lat_over_us)
        nb, nc, ns = len(self.batch_edges), len(self.ctx_edges), len(self.decode_cus)
        assert self.lat_distinct_us.shape == (nb, nc, ns) and self.lat_over_us.shape == (nb, nc)
        self.slo_us = int(slo_us)

    def desc(self) -> ProfileDesc:
        p = lambda a: a.ctypes.data_as(_i32p)
        return ProfileDesc(len(self.batch_edges), len(self.ctx_edges), len(self.decode_cus), p(self.batch_edges),
                           p(self.ctx_edges), p(self.decode_cus), p(self.lat_distinct_us), p(self.lat_over_us),
                           self.slo_us)


class Context:
    """Owns one rs_ctx.  Method names mirror the C entry points without the rs_ prefix."""

    def __init__(self, d_model: int, n_q_heads: int, n_kv_heads: int, head_dim: int, ffn_dim: int,
                 n_layers: int, rms_eps: float, rope_base: float, max_pos: int, n_blocks: int,
                 k_pool=None, v_pool=None, layer_stride: int = 0, max_prefill_tokens: int = 0,
                 max_decode_batch: int = 0, max_context: int = 1, profile: Optional[Profile] = None,
                 device: int = 0):
        self._lib = load()
        self._h = ctypes.c_void_p(0)
        m = ModelDesc(d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, n_layers, rms_eps, rope_base, max_pos)
        if layer_stride == 0:
            layer_stride = n_blocks * RS_KV_BLOCK * n_kv_heads * head_dim
        p = PoolDesc(_ptr(k_pool), _ptr(v_pool), layer_stride, n_blocks)
        lim = Limits(max_prefill_tokens, max_decode_batch, max_context)
        self._prof = profile
        pd = profile.desc() if profile is not None else None
        self._keep = [k_pool, v_pool]
        self._keep_layers = []
        self.n_layers = n_layers
        self.max_context = max_context
        _check(self._lib.rs_init(ctypes.byref(m), ctypes.byref(p), ctypes.byref(lim),
                                 ctypes.byref(pd) if pd is not None else None, ctypes.c_int32(device),
                                 ctypes.byref(self._h)))

    @classmethod
    def from_shape(cls, shape, **kw):
        return cls(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn_dim,
                   kw.pop("n_layers", 1), shape.rms_eps, shape.rope_base, **kw)

    def destroy(self):
        if self._h:
            self._lib.rs_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- weights
    def set_weights(self, layer: int, g1, wqkv, wo, g2, wg, wu, wd):
        while len(self._keep_layers) <= layer:
            self._keep_layers.append(None)
        self._keep_layers[layer] = (g1, wqkv, wo, g2, wg, wu, wd)   # the library borrows them
        w = LayerWeights(*[_ptr(t) for t in (g1, wqkv, wo, g2, wg, wu, wd)])
        _check(self._lib.rs_set_weights(self._h, ctypes.c_int32(layer), ctypes.byref(w)))

    def set_moe_weights(self, layer: int, router, wg, wu, wd, n_experts: int, top_k: int = 2):
        self._keep.append(router)   # the experts' matrices are packed during the call and not referenced afterwards
        w = MoeWeights(_ptr(router), _ptr(wg), _ptr(wu), _ptr(wd), n_experts, top_k)
        _check(self._lib.rs_set_moe_weights(self._h, ctypes.c_int32(layer), ctypes.byref(w)))

    def debug_read_moe_routing(self, side: int, n_rows: int):
        sel = np.empty((n_rows, 2), dtype=np.int32)
        wt = np.empty((n_rows, 2), dtype=np.float32)
        _check(self._lib.rs_debug_read_moe_routing(self._h, ctypes.c_int32(side), ctypes.c_int32(n_rows),
                                                   sel.ctypes.data_as(_i32p), wt.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))
        return sel, wt

    def release_source_weights(self, layer: int):
        """The five matrices given to set_weights(layer) may be freed afterwards (packed copies remain)."""
        _check(self._lib.rs_release_source_weights(self._h, ctypes.c_int32(layer)))
        if layer < len(self._keep_layers):
            g1, _, _, g2, _, _, _ = self._keep_layers[layer]
            self._keep_layers[layer] = (g1, None, None, g2, None, None, None)

    # -- allocator
    def kv_alloc(self, req_id: int, n_tokens_total: int, cap: int = 1 << 16) -> np.ndarray:
        out = np.empty(cap, dtype=np.int32)
        n = ctypes.c_int32(0)
        _check(self._lib.rs_kv_alloc(self._h, ctypes.c_int64(req_id), ctypes.c_int32(n_tokens_total),
                                     out.ctypes.data_as(_i32p), ctypes.c_int32(cap), ctypes.byref(n)))
        return out[:n.value].copy()

    def kv_free(self, req_id: int):
        _check(self._lib.rs_kv_free(self._h, ctypes.c_int64(req_id)))

    def kv_num_free(self) -> int:
        n = ctypes.c_int32(0)
        _check(self._lib.rs_kv_num_free(self._h, ctypes.byref(n)))
        return n.value

    # -- layers
    def prefill_layer(self, layer: int, x_in, x_out, cu_seqlens: Sequence[int], block_tables, max_blk: int):
        cu = _i32(cu_seqlens)
        _check(self._lib.rs_prefill_layer(self._h, ctypes.c_int32(layer), _ptr(x_in), _ptr(x_out),
                                          cu.ctypes.data_as(_i32p), ctypes.c_int32(len(cu) - 1),
                                          _ptr(block_tables), ctypes.c_int32(max_blk)))

    def decode_layer(self, layer: int, x_in, x_out, ctx_lens, block_tables, max_blk: int, B: int, max_ctx: int):
        _check(self._lib.rs_decode_layer(self._h, ctypes.c_int32(layer), _ptr(x_in), _ptr(x_out), _ptr(ctx_lens),
                                         _ptr(block_tables), ctypes.c_int32(max_blk), ctypes.c_int32(B),
                                         ctypes.c_int32(max_ctx)))

    def hybrid_layer(self, layer: int, x_in, x_out, cu_seqlens: Sequence[int], start_pos: Sequence[int], prefill_tables,
                     max_blk_prefill: int, ctx_lens=None, decode_tables=None, max_blk_decode: int = 0, B: int = 0, max_ctx: int = 1):
        cu = (ctypes.c_int32 * len(cu_seqlens))(*[int(v) for v in cu_seqlens])
        sp = (ctypes.c_int32 * max(len(start_pos), 1))(*[int(v) for v in start_pos])
        _check(self._lib.rs_hybrid_layer(self._h, ctypes.c_int32(layer), _ptr(x_in), _ptr(x_out), cu, sp,
                                         ctypes.c_int32(len(cu_seqlens) - 1), _ptr(prefill_tables), ctypes.c_int32(max_blk_prefill),
                                         _ptr(ctx_lens) if ctx_lens is not None else None,
                                         _ptr(decode_tables) if decode_tables is not None else None,
                                         ctypes.c_int32(max_blk_decode), ctypes.c_int32(B), ctypes.c_int32(max_ctx)))

    def set_hybrid_batching(self, chunk_tokens: int):
        _check(self._lib.rs_set_hybrid_batching(self._h, ctypes.c_int32(chunk_tokens)))

    def step_chunks(self):
        """[(request, first position, length)] of the prompt parts in the latest step's batch (hybrid batching)."""
        cap = RS_MAX_PREFILL_REQS
        ids, st, ln = (ctypes.c_int64 * cap)(), (ctypes.c_int32 * cap)(), (ctypes.c_int32 * cap)()
        n = ctypes.c_int32(0)
        _check(self._lib.rs_step_chunks(self._h, ids, st, ln, ctypes.c_int32(cap), ctypes.byref(n)))
        return [(int(ids[i]), int(st[i]), int(ln[i])) for i in range(n.value)]

    def decode_layer_noalloc(self, layer: int, x_in, x_out, ctx_lens, block_tables, max_blk: int, B: int, max_ctx: int):
        _check(self._lib.rs_decode_layer_noalloc(self._h, ctypes.c_int32(layer), _ptr(x_in), _ptr(x_out), _ptr(ctx_lens),
                                                 _ptr(block_tables), ctypes.c_int32(max_blk), ctypes.c_int32(B),
                                                 ctypes.c_int32(max_ctx)))

    def decode_layer_graph(self, layer: int, x_in, x_out, ctx_lens, block_tables, max_blk: int, B: int, max_ctx_bucket: int):
        _check(self._lib.rs_decode_layer_graph(self._h, ctypes.c_int32(layer), _ptr(x_in), _ptr(x_out), _ptr(ctx_lens),
                                               _ptr(block_tables), ctypes.c_int32(max_blk), ctypes.c_int32(B),
                                               ctypes.c_int32(max_ctx_bucket)))

    # -- CU split / manager
    def set_cu_split(self, prefill_cus: int, decode_cus: int):
        _check(self._lib.rs_set_cu_split(self._h, ctypes.c_int32(prefill_cus), ctypes.c_int32(decode_cus)))

    def get_cu_split(self):
        p, d = ctypes.c_int32(0), ctypes.c_int32(0)
        _check(self._lib.rs_get_cu_split(self._h, ctypes.byref(p), ctypes.byref(d)))
        return p.value, d.value

    def get_cu_mask(self, side: int) -> np.ndarray:
        m = (ctypes.c_uint32 * 8)()
        _check(self._lib.rs_get_cu_mask(self._h, ctypes.c_int32(side), m))
        return np.array(list(m), dtype=np.uint32)

    def choose_split(self, decode_batch: int, sum_ctx: int, prefill_pending: bool):
        p, d = ctypes.c_int32(0), ctypes.c_int32(0)
        _check(self._lib.rs_choose_split(self._h, ctypes.c_int32(decode_batch), ctypes.c_int64(sum_ctx),
                                         ctypes.c_int32(1 if prefill_pending else 0), ctypes.byref(p), ctypes.byref(d)))
        return p.value, d.value

    def debug_cu_histogram(self, side: int, n_workgroups: int) -> np.ndarray:
        h = np.zeros(RS_CU_HIST_BINS, dtype=np.int32)
        _check(self._lib.rs_debug_cu_histogram(self._h, ctypes.c_int32(side), ctypes.c_int32(n_workgroups),
                                               h.ctypes.data_as(_i32p)))
        return h

    def debug_cu_histogram_graph(self, side: int, n_workgroups: int) -> np.ndarray:
        h = np.zeros(RS_CU_HIST_BINS, dtype=np.int32)
        _check(self._lib.rs_debug_cu_histogram_graph(self._h, ctypes.c_int32(side), ctypes.c_int32(n_workgroups),
                                                     h.ctypes.data_as(_i32p)))
        return h

    def debug_mfma_probe(self, side: int) -> float:
        """TFLOP/s of register-only bf16 MFMAs on the side's partition."""
        t = ctypes.c_float(0)
        _check(self._lib.rs_debug_mfma_probe(self._h, ctypes.c_int32(side), ctypes.byref(t)))
        return t.value

    def debug_stream_read(self, side: int, buf, n_bytes: int) -> float:
        """GPU milliseconds to read n_bytes of `buf` once on the side's CU partition."""
        ms = ctypes.c_float(0)
        _check(self._lib.rs_debug_stream_read(self._h, ctypes.c_int32(side), _ptr(buf), ctypes.c_int64(n_bytes),
                                              ctypes.byref(ms)))
        return ms.value

    def debug_read_workspace(self, side: int, which: int, shape) -> np.ndarray:
        """bf16 bit patterns (uint16) of an intermediate buffer, shaped `shape`."""
        out = np.empty(shape, dtype=np.uint16)
        _check(self._lib.rs_debug_read_workspace(self._h, ctypes.c_int32(side), ctypes.c_int32(which),
                                                 out.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(out.nbytes)))
        return out

    # -- streams / timing
    def get_stream(self, side: int) -> int:
        s = ctypes.c_void_p(0)
        _check(self._lib.rs_get_stream(self._h, ctypes.c_int32(side), ctypes.byref(s)))
        return s.value or 0

    def sync(self, side: int):
        _check(self._lib.rs_sync(self._h, ctypes.c_int32(side)))

    def mark(self, side: int, slot: int):
        _check(self._lib.rs_mark(self._h, ctypes.c_int32(side), ctypes.c_int32(slot)))

    def mark_done(self, side: int, slot: int) -> bool:
        """True once the work enqueued in front of the mark has completed (non-blocking)."""
        done = ctypes.c_int32(0)
        _check(self._lib.rs_mark_done(self._h, ctypes.c_int32(side), ctypes.c_int32(slot), ctypes.byref(done)))
        return bool(done.value)

    def elapsed_ms(self, side_begin: int, slot_begin: int, slot_end: int, side_end: Optional[int] = None) -> float:
        ms = ctypes.c_float(0)
        if side_end is None:
            side_end = side_begin
        _check(self._lib.rs_elapsed_ms(self._h, ctypes.c_int32(side_begin), ctypes.c_int32(slot_begin),
                                       ctypes.c_int32(side_end), ctypes.c_int32(slot_end), ctypes.byref(ms)))
        return ms.value

    def set_kernel_timing(self, on: bool):
        _check(self._lib.rs_set_kernel_timing(self._h, ctypes.c_int32(1 if on else 0)))

    def kernel_times(self, side: int) -> np.ndarray:
        out = (ctypes.c_float * RS_N_KERNEL_SLOTS)()
        _check(self._lib.rs_kernel_times(self._h, ctypes.c_int32(side), out))
        return np.array(list(out), dtype=np.float64)

    # -- serving step
    def submit(self, req_id: int, prompt_len: int, output_len: int, prompt_hidden=None):
        self._keep.append(prompt_hidden)
        _check(self._lib.rs_submit(self._h, ctypes.c_int64(req_id), ctypes.c_int32(prompt_len),
                                   ctypes.c_int32(output_len), _ptr(prompt_hidden)))

    def decode_batch_ids(self) -> list:
        """Request ids of the rows of the most recent step's decode batch."""
        ids = (ctypes.c_int64 * 4096)()
        n = ctypes.c_int32(0)
        _check(self._lib.rs_decode_batch_ids(self._h, ids, ctypes.c_int32(4096), ctypes.byref(n)))
        return [int(ids[i]) for i in range(n.value)]

    def step(self, decode_hidden=None, decode_out=None, wait_decode: bool = False) -> StepOut:
        si = StepIn(_ptr(decode_hidden), _ptr(decode_out), 1 if wait_decode else 0)
        so = StepOut()
        _check(self._lib.rs_step(self._h, ctypes.byref(si), ctypes.byref(so)))
        return so

    # -- token boundary and closed-loop serving
    def set_head(self, embed, final_norm, lm_head, vocab: int, eos_token: int = -1):
        self._keep.append((embed, final_norm, lm_head))
        w = HeadWeights(_ptr(embed), _ptr(final_norm), _ptr(lm_head), vocab, eos_token)
        _check(self._lib.rs_set_head(self._h, ctypes.byref(w)))

    def embed(self, side: int, tokens, n: int, x_out):
        _check(self._lib.rs_embed(self._h, ctypes.c_int32(side), _ptr(tokens), ctypes.c_int32(n), _ptr(x_out)))

    def lm_head_greedy(self, side: int, x, n: int, logits_out=None, tokens_out=None):
        _check(self._lib.rs_lm_head_greedy(self._h, ctypes.c_int32(side), _ptr(x), ctypes.c_int32(n), _ptr(logits_out),
                                           _ptr(tokens_out)))

    def submit_tokens(self, req_id: int, prompt_tokens, max_new_tokens: int):
        t = _i32(prompt_tokens)
        _check(self._lib.rs_submit_tokens(self._h, ctypes.c_int64(req_id), t.ctypes.data_as(_i32p), ctypes.c_int32(len(t)),
                                          ctypes.c_int32(max_new_tokens)))

    def step_tokens(self, wait_decode: bool = False) -> StepOut:
        so = StepOut()
        _check(self._lib.rs_step_tokens(self._h, ctypes.c_int32(1 if wait_decode else 0), ctypes.byref(so)))
        return so

    def request_output(self, req_id: int, cap: int = 1 << 16):
        """(tokens generated so far, finished flag)."""
        out = np.empty(cap, dtype=np.int32)
        n = ctypes.c_int32(0)
        fin = ctypes.c_int32(0)
        _check(self._lib.rs_request_output(self._h, ctypes.c_int64(req_id), out.ctypes.data_as(_i32p), ctypes.c_int32(cap),
                                           ctypes.byref(n), ctypes.byref(fin)))
        return out[:n.value].copy(), bool(fin.value)

    def request_times(self, req_id: int):
        """(submitted, first token seen, latest token seen), host seconds since the context was created."""
        t = (ctypes.c_double * 3)()
        _check(self._lib.rs_request_times(self._h, ctypes.c_int64(req_id), t))
        return t[0], t[1], t[2]

    def request_release(self, req_id: int):
        _check(self._lib.rs_request_release(self._h, ctypes.c_int64(req_id)))

    def set_step_graphs(self, on):
        """False / True, or an int n > 1: on, keeping at most n captured steps."""
        _check(self._lib.rs_set_step_graphs(self._h, ctypes.c_int32(int(on))))

    def step_graph_stats(self):
        """(graphs captured, decode steps launched as a graph, decode steps enqueued outside a capture, host ns of their launches)."""
        st = (ctypes.c_int64 * 4)()
        _check(self._lib.rs_step_graph_stats(self._h, st))
        return st[0], st[1], st[2], st[3]

    def engine_start(self):
        _check(self._lib.rs_engine_start(self._h))

    def engine_stop(self, drain: bool = True):
        _check(self._lib.rs_engine_stop(self._h, ctypes.c_int32(1 if drain else 0)))

    def engine_stats(self) -> dict:
        st = (ctypes.c_int64 * 4)()
        _check(self._lib.rs_engine_stats(self._h, st))
        return {"submitted": st[0], "finished": st[1], "iterations": st[2], "preempted": st[3]}

    def debug_push_sampled(self, req_id: int, token: int):
        _check(self._lib.rs_debug_push_sampled(self._h, ctypes.c_int64(req_id), ctypes.c_int32(token)))

    def request_state(self, req_id: int) -> int:
        return _check(self._lib.rs_request_state(self._h, ctypes.c_int64(req_id)))

    def debug_complete_prefill(self, req_id: int):
        _check(self._lib.rs_debug_complete_prefill(self._h, ctypes.c_int64(req_id)))
