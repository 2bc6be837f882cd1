"""CPU oracle (TEST INFRASTRUCTURE ONLY) for the prefill/decode decoder-layer path.

`rs_oracle.c` is the plain float32 definition of the layer; this package builds
it with gcc and exposes it through numpy arrays.  `manager.py` and `kv_alloc.py`
are the exact integer definitions of the CU-split choice and of the block
allocator.  Nothing here is used by the product: only tests, the smoke check and
the benchmark's cpu_baseline leg import it, and it imports nothing from the GPU
package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rs_oracle.c")
_LIB = os.path.join(_HERE, "librs_oracle.so")

_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)


def build(force: bool = False) -> str:
    """Compile rs_oracle.c into librs_oracle.so (gcc, -O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-fPIC", "-shared",
                               "-std=c11", "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Layer(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32),
                ("hd", ctypes.c_int32), ("f", ctypes.c_int32), ("block", ctypes.c_int32),
                ("eps", ctypes.c_float), ("rope_base", ctypes.c_double),
                ("g1", _f32p), ("g2", _f32p), ("wqkv_t", _f32p), ("wo_t", _f32p),
                ("wg_t", _f32p), ("wu_t", _f32p), ("wd_t", _f32p)]


class _Taps(ctypes.Structure):
    _fields_ = [("h", _f32p), ("qkv", _f32p), ("attn", _f32p), ("x1", _f32p), ("act", _f32p)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        # RS_ORACLE_LIB: a test that plants a mistake in a copy of rs_oracle.c points the pins at that copy
        _lib = ctypes.CDLL(os.environ.get("RS_ORACLE_LIB") or build())
        _lib.orc_prefill_layer.restype = ctypes.c_int
        _lib.orc_decode_layer.restype = ctypes.c_int
        _lib.orc_prefill_chunk_layer.restype = ctypes.c_int
        _lib.orc_attn_causal.restype = ctypes.c_int
        _lib.orc_attn_paged.restype = ctypes.c_int
        _lib.orc_kv_write.restype = ctypes.c_int
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def _fp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_f32p)


def _ip(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_i32p)


def _f32c(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32c(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def widen(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exactly (done by the C code)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    lib().orc_bf16_to_f32(bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), _fp(out),
                          ctypes.c_int64(bits.size))
    return out


def rmsnorm(x, g, eps: float) -> np.ndarray:
    x = _f32c(x); g = _f32c(g)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_fp(x), _fp(g), ctypes.c_int64(x.shape[0]), ctypes.c_int64(x.shape[1]),
                      ctypes.c_float(eps), _fp(out))
    return out


def linear(a, w) -> np.ndarray:
    """a[M,K] @ w[N,K]^T via the dot-product form."""
    a = _f32c(a); w = _f32c(w)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K
    out = np.empty((M, N), dtype=np.float32)
    lib().orc_linear(_fp(a), _fp(w), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), _fp(out))
    return out


def linear_t(a, w) -> np.ndarray:
    """Same product through the transposed-copy form used inside the layer."""
    a = _f32c(a); w = _f32c(w)
    M, K = a.shape
    N = w.shape[0]
    wt = np.empty((K, N), dtype=np.float32)
    lib().orc_transpose(_fp(w), ctypes.c_int64(N), ctypes.c_int64(K), _fp(wt))
    out = np.empty((M, N), dtype=np.float32)
    lib().orc_linear_t(_fp(a), _fp(wt), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), _fp(out))
    return out


def rope(x, pos, base: float) -> np.ndarray:
    """x[M,H,hd] rotated at positions pos[M]; returns a new array."""
    x = _f32c(x).copy(); pos = _i32c(pos)
    M, H, hd = x.shape
    lib().orc_rope(_fp(x), _ip(pos), ctypes.c_int64(M), ctypes.c_int64(H), ctypes.c_int64(hd),
                   ctypes.c_double(base), ctypes.c_int64(H * hd))
    return x


def silu_mul(g, u) -> np.ndarray:
    g = _f32c(g); u = _f32c(u)
    out = np.empty_like(g)
    lib().orc_silu_mul(_fp(g), _fp(u), ctypes.c_int64(g.size), _fp(out))
    return out


def attn_causal(q, k, v, cu_seqlens, rows=None) -> np.ndarray:
    """q[T,Hq,hd], k,v[T,Hkv,hd] -> o[T,Hq,hd] (rows not listed in `rows` stay 0)."""
    q = _f32c(q); k = _f32c(k); v = _f32c(v); cu = _i32c(cu_seqlens)
    T, Hq, hd = q.shape
    Hkv = k.shape[1]
    o = np.zeros((T, Hq, hd), dtype=np.float32)
    r = None if rows is None else _i32c(rows)
    rc = lib().orc_attn_causal(_fp(q), ctypes.c_int64(Hq * hd), _fp(k), _fp(v),
                               ctypes.c_int64(Hkv * hd), _ip(cu), ctypes.c_int32(len(cu) - 1),
                               ctypes.c_int64(Hq), ctypes.c_int64(Hkv), ctypes.c_int64(hd),
                               _ip(r), ctypes.c_int64(0 if r is None else len(r)), _fp(o))
    if rc:
        raise ValueError(f"orc_attn_causal failed: {rc}")
    return o


def attn_paged(q, Kc, Vc, tables, n_keys) -> np.ndarray:
    """q[B,Hq,hd]; pools [n_blocks,block,Hkv,hd]; request i sees n_keys[i] cached tokens."""
    q = _f32c(q); tables = _i32c(tables); n_keys = _i32c(n_keys)
    assert Kc.dtype == np.float32 and Kc.flags.c_contiguous
    assert Vc.dtype == np.float32 and Vc.flags.c_contiguous
    B, Hq, hd = q.shape
    n_blocks, block, Hkv, _ = Kc.shape
    o = np.zeros_like(q)
    rc = lib().orc_attn_paged(_fp(q), _fp(Kc), _fp(Vc), ctypes.c_int64(n_blocks),
                              ctypes.c_int64(block), ctypes.c_int64(Hq), ctypes.c_int64(Hkv),
                              ctypes.c_int64(hd), _ip(tables), ctypes.c_int64(tables.shape[1]),
                              _ip(n_keys), ctypes.c_int64(B), _fp(o))
    if rc:
        raise ValueError(f"orc_attn_paged failed: {rc}")
    return o


class OracleLayer:
    """One decoder layer's weights (bf16 bit patterns widened to float32)."""

    def __init__(self, d_model: int, n_q_heads: int, n_kv_heads: int, head_dim: int, ffn_dim: int,
                 rms_eps: float, rope_base: float, weights_bf16: Dict[str, np.ndarray],
                 block: int = 16):
        self.d, self.hq, self.hkv, self.hd, self.f = d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim
        self.eps, self.rope_base, self.block = float(rms_eps), float(rope_base), int(block)
        self.qd, self.kvd = n_q_heads * head_dim, n_kv_heads * head_dim
        self.nqkv = self.qd + 2 * self.kvd
        L = lib()
        self._keep = {}
        for name in ("g1", "g2"):
            self._keep[name] = widen(weights_bf16[name])
        for name in ("wqkv", "wo", "wg", "wu", "wd"):
            w = widen(weights_bf16[name])
            N, K = w.shape
            wt = np.empty((K, N), dtype=np.float32)
            L.orc_transpose(_fp(w), ctypes.c_int64(N), ctypes.c_int64(K), _fp(wt))
            self._keep[name + "_t"] = wt
        k = self._keep
        assert k["wqkv_t"].shape == (self.d, self.nqkv)
        assert k["wo_t"].shape == (self.qd, self.d)
        assert k["wg_t"].shape == (self.d, self.f) and k["wu_t"].shape == (self.d, self.f)
        assert k["wd_t"].shape == (self.f, self.d)
        self._c = _Layer(self.d, self.hq, self.hkv, self.hd, self.f, self.block, self.eps,
                         self.rope_base, _fp(k["g1"]), _fp(k["g2"]), _fp(k["wqkv_t"]),
                         _fp(k["wo_t"]), _fp(k["wg_t"]), _fp(k["wu_t"]), _fp(k["wd_t"]))

    @classmethod
    def from_shape(cls, shape, weights_bf16):
        return cls(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                   shape.ffn_dim, shape.rms_eps, shape.rope_base, weights_bf16)

    # ---- single steps of the layer on caller-supplied operands: the same C routines the layer
    # calls (orc_linear_t, orc_rmsnorm), with this layer's weights, for stage-by-stage checks
    def project(self, name: str, a) -> np.ndarray:
        """a[M,K] @ W^T for W = one of "wqkv", "wo", "wg", "wu", "wd" ([N,K])."""
        a = _f32c(a)
        wt = self._keep[name + "_t"]
        K, N = wt.shape
        assert a.ndim == 2 and a.shape[1] == K
        out = np.empty((a.shape[0], N), dtype=np.float32)
        lib().orc_linear_t(_fp(a), _fp(wt), ctypes.c_int64(a.shape[0]), ctypes.c_int64(N), ctypes.c_int64(K), _fp(out))
        return out

    def norm(self, which: int, x) -> np.ndarray:
        """RMSNorm with the layer's first (which = 1) or second (which = 2) gain vector."""
        return rmsnorm(x, self._keep["g1" if which == 1 else "g2"], self.eps)

    def new_cache(self, n_blocks: int, fill: float = 0.0):
        shp = (n_blocks, self.block, self.hkv, self.hd)
        return np.full(shp, fill, dtype=np.float32), np.full(shp, fill, dtype=np.float32)

    def _taps(self, M: int, want: bool):
        if not want:
            return None, None
        arrs = {"h": np.zeros((M, self.d), np.float32), "qkv": np.zeros((M, self.nqkv), np.float32),
                "attn": np.zeros((M, self.qd), np.float32), "x1": np.zeros((M, self.d), np.float32),
                "act": np.zeros((M, self.f), np.float32)}
        t = _Taps(_fp(arrs["h"]), _fp(arrs["qkv"]), _fp(arrs["attn"]), _fp(arrs["x1"]), _fp(arrs["act"]))
        return t, arrs

    def prefill(self, x, cu_seqlens: Sequence[int], tables, Kc, Vc, rows=None, taps: bool = False):
        """x: float32 [T,d] (already widened).  Returns y [n_eval,d] (and taps dict)."""
        x = _f32c(x); cu = _i32c(cu_seqlens); tables = _i32c(tables)
        T = int(cu[-1])
        assert x.shape == (T, self.d)
        assert Kc.dtype == np.float32 and Kc.flags.c_contiguous and Vc.flags.c_contiguous
        r = None if rows is None else _i32c(rows)
        n_eval = T if r is None else len(r)
        y = np.empty((n_eval, self.d), dtype=np.float32)
        t, arrs = self._taps(T, taps)
        rc = lib().orc_prefill_layer(ctypes.byref(self._c), _fp(x), _ip(cu),
                                     ctypes.c_int32(len(cu) - 1), _ip(tables),
                                     ctypes.c_int64(tables.shape[1]), _fp(Kc), _fp(Vc),
                                     ctypes.c_int64(Kc.shape[0]), _ip(r),
                                     ctypes.c_int64(0 if r is None else len(r)), _fp(y),
                                     ctypes.byref(t) if t is not None else None)
        if rc:
            raise ValueError(f"orc_prefill_layer failed: {rc}")
        return (y, arrs) if taps else y

    def prefill_chunk(self, x, cu_seqlens: Sequence[int], start_pos: Sequence[int], tables, Kc, Vc, rows=None,
                      taps: bool = False):
        """One chunk of each prompt: request r's rows sit at positions start_pos[r].. and attend to everything
        cached before them plus themselves.  Returns y [n_eval,d] (and taps dict)."""
        x = _f32c(x); cu = _i32c(cu_seqlens); tables = _i32c(tables); sp = _i32c(start_pos)
        T = int(cu[-1])
        assert x.shape == (T, self.d) and len(sp) == len(cu) - 1
        assert Kc.dtype == np.float32 and Kc.flags.c_contiguous and Vc.flags.c_contiguous
        r = None if rows is None else _i32c(rows)
        n_eval = T if r is None else len(r)
        y = np.empty((n_eval, self.d), dtype=np.float32)
        t, arrs = self._taps(T, taps)
        rc = lib().orc_prefill_chunk_layer(ctypes.byref(self._c), _fp(x), _ip(cu), ctypes.c_int32(len(cu) - 1), _ip(sp),
                                           _ip(tables), ctypes.c_int64(tables.shape[1]), _fp(Kc), _fp(Vc),
                                           ctypes.c_int64(Kc.shape[0]), _ip(r),
                                           ctypes.c_int64(0 if r is None else len(r)), _fp(y),
                                           ctypes.byref(t) if t is not None else None)
        if rc:
            raise ValueError(f"orc_prefill_chunk_layer failed: {rc}")
        return (y, arrs) if taps else y

    def decode(self, x, ctx_lens, tables, Kc, Vc, taps: bool = False):
        """x: float32 [B,d]; ctx_lens[i] tokens already cached.  Returns y [B,d]."""
        x = _f32c(x); ctx = _i32c(ctx_lens); tables = _i32c(tables)
        B = x.shape[0]
        assert Kc.dtype == np.float32 and Kc.flags.c_contiguous and Vc.flags.c_contiguous
        y = np.empty((B, self.d), dtype=np.float32)
        t, arrs = self._taps(B, taps)
        rc = lib().orc_decode_layer(ctypes.byref(self._c), _fp(x), _ip(ctx), _ip(tables),
                                    ctypes.c_int64(tables.shape[1]), _fp(Kc), _fp(Vc),
                                    ctypes.c_int64(Kc.shape[0]), ctypes.c_int64(B), _fp(y),
                                    ctypes.byref(t) if t is not None else None)
        if rc:
            raise ValueError(f"orc_decode_layer failed: {rc}")
        return (y, arrs) if taps else y
