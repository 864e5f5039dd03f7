"""ctypes wrapper around oracle/libpod_oracle.so (the CPU oracle, test infrastructure only).

Marshalling only: every number comes out of pod_oracle.c.  bf16 tensors travel as
numpy uint16 arrays holding the raw bit patterns; outputs are float64.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

OK, ERR_ARG, ERR_CAPACITY, ERR_STATE = 0, -1, -2, -3

_lib = None


def lib():
    global _lib
    if _lib is None:
        # POD_ORACLE_LIB: another build of pod_oracle.c (the mutation tests load deliberately broken ones)
        path = os.environ.get("POD_ORACLE_LIB") or _build.build(force=False)
        L = C.CDLL(path)
        u16p, i32p, f64p, lp = (C.POINTER(C.c_uint16), C.POINTER(C.c_int32),
                                C.POINTER(C.c_double), C.POINTER(C.c_long))
        L.oracle_pod_attention.restype = C.c_int
        L.oracle_pod_attention.argtypes = [C.c_long, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                           C.c_double, u16p, u16p, u16p, u16p, u16p, lp, C.c_long, f64p]
        L.oracle_pod_attention_gate.restype = C.c_int
        L.oracle_pod_attention_gate.argtypes = L.oracle_pod_attention.argtypes + [f64p]
        L.oracle_cache_create.restype = C.c_void_p
        L.oracle_cache_create.argtypes = [C.c_int] * 7 + [C.c_long]
        L.oracle_cache_create_map.restype = C.c_void_p
        L.oracle_cache_create_map.argtypes = [C.c_int] * 7 + [C.c_long, i32p]
        L.oracle_cache_bytes_formula_map.restype = None
        L.oracle_cache_bytes_formula_map.argtypes = [C.c_int] * 5 + [C.c_long, C.c_int, i32p, f64p, f64p]
        L.oracle_cache_destroy.restype = None
        L.oracle_cache_destroy.argtypes = [C.c_void_p]
        L.oracle_cache_reset.restype = C.c_int
        L.oracle_cache_reset.argtypes = [C.c_void_p, C.c_int]
        L.oracle_cache_len.restype = C.c_long
        L.oracle_cache_len.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.oracle_cache_append.restype = C.c_int
        L.oracle_cache_append.argtypes = [C.c_void_p, C.c_int, u16p, u16p, i32p, C.c_int]
        L.oracle_cache_append_many.restype = C.c_int
        L.oracle_cache_append_many.argtypes = [C.c_void_p, C.c_int, u16p, u16p, i32p, i32p, C.c_int, C.c_int]
        L.oracle_chunk_attention.restype = C.c_int
        L.oracle_chunk_attention.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_double, C.c_int,
                                             u16p, u16p, u16p, u16p, u16p, f64p]
        L.oracle_cache_fill.restype = C.c_int
        L.oracle_cache_fill.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_long, u16p, u16p]
        L.oracle_cache_export.restype = C.c_int
        L.oracle_cache_export.argtypes = [C.c_void_p, C.c_int, C.c_int, lp] + [u16p] * 6
        L.oracle_cache_stored_elems.restype = C.c_long
        L.oracle_cache_stored_elems.argtypes = [C.c_void_p]
        L.oracle_cache_bytes_formula.restype = None
        L.oracle_cache_bytes_formula.argtypes = [C.c_int] * 6 + [C.c_long, C.c_int, f64p, f64p]
        L.oracle_decode_attention.restype = C.c_int
        L.oracle_decode_attention.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_double, u16p, u16p,
                                              i32p, C.c_int, f64p]
        L.oracle_decode_attention_gated.restype = C.c_int
        L.oracle_decode_attention_gated.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_double, u16p, u16p,
                                                    i32p, C.c_int, C.c_double, f64p, f64p, i32p]
        L.oracle_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _u16(a):
    if a is None:
        return None
    assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_uint16))


def _chk(rc, what):
    if rc != OK:
        raise OracleError(rc, what)


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: oracle error {code}")
        self.code = code


def num_threads() -> int:
    return lib().oracle_num_threads()


def pod_attention(q, k, v, q_shared, k_shared, rows, S, W, scale, gate=False):
    """Attention by definition.  q/q_shared: uint16 [nrows][Hq][d]; k/v/k_shared: uint16 [n][Hkv][d];
    rows: positions of the query rows.  Returns float64 [nrows][Hq][d] (and the gate if asked)."""
    n, Hkv, d = k.shape
    nrows, Hq, _ = q.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.shape == (nrows,)
    out = np.empty((nrows, Hq, d), dtype=np.float64)
    rp = rows.ctypes.data_as(C.POINTER(C.c_long))
    op = out.ctypes.data_as(C.POINTER(C.c_double))
    if gate:
        g = np.empty((nrows, Hq), dtype=np.float64)
        rc = lib().oracle_pod_attention_gate(n, Hq, Hkv, d, S, W, float(scale), _u16(q), _u16(k), _u16(v),
                                             _u16(q_shared), _u16(k_shared), rp, nrows, op,
                                             g.ctypes.data_as(C.POINTER(C.c_double)))
        _chk(rc, "oracle_pod_attention_gate")
        return out, g
    rc = lib().oracle_pod_attention(n, Hq, Hkv, d, S, W, float(scale), _u16(q), _u16(k), _u16(v),
                                    _u16(q_shared), _u16(k_shared), rp, nrows, op)
    _chk(rc, "oracle_pod_attention")
    return out


def cache_bytes_formula(L, G, Hkv, d, S, W, n, elem_bytes=2):
    p, dn = C.c_double(), C.c_double()
    lib().oracle_cache_bytes_formula(L, G, Hkv, d, S, W, n, elem_bytes, C.byref(p), C.byref(dn))
    return p.value, dn.value


def cache_bytes_formula_map(lowest, d, S, W, n, elem_bytes=2):
    """Closed-form bytes for head-wise blocks; lowest: int [L][Hkv] (lowest layer of each layer's block per kv head)."""
    lowest = np.ascontiguousarray(lowest, dtype=np.int32)
    L, Hkv = lowest.shape
    p, dn = C.c_double(), C.c_double()
    lib().oracle_cache_bytes_formula_map(L, Hkv, d, S, W, n, elem_bytes, lowest.ctypes.data_as(C.POINTER(C.c_int32)),
                                         C.byref(p), C.byref(dn))
    return p.value, dn.value


class Cache:
    """Logical model of the split cache (lists per layer and sequence).  block_lowest: optional int [L][Hkv]
    table of head-wise blocks (lowest layer of the block each layer belongs to, per kv head); default: uniform
    blocks of G layers."""

    def __init__(self, L, G, Hkv, d, S, W, B, max_ctx, block_lowest=None):
        self.L, self.G, self.Hkv, self.d, self.S, self.W, self.B, self.max_ctx = L, G, Hkv, d, S, W, B, max_ctx
        if block_lowest is None:
            self.lowest = np.array([[l - l % G] * Hkv for l in range(L)], dtype=np.int32)
            self._h = lib().oracle_cache_create(L, G, Hkv, d, S, W, B, max_ctx)
        else:
            self.lowest = np.ascontiguousarray(block_lowest, dtype=np.int32)
            assert self.lowest.shape == (L, Hkv)
            self._h = lib().oracle_cache_create_map(L, G, Hkv, d, S, W, B, max_ctx,
                                                    self.lowest.ctypes.data_as(C.POINTER(C.c_int32)))
        if not self._h:
            raise OracleError(ERR_ARG, "oracle_cache_create")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().oracle_cache_destroy(self._h)
            self._h = None

    def reset(self, seq=-1):
        _chk(lib().oracle_cache_reset(self._h, seq), "oracle_cache_reset")

    def length(self, layer, seq):
        return lib().oracle_cache_len(self._h, layer, seq)

    def append(self, layer, k_new, v_new, positions):
        positions = np.ascontiguousarray(positions, dtype=np.int32)
        B = positions.shape[0]
        assert k_new.shape == (B, self.Hkv, self.d) and v_new.shape == k_new.shape
        rc = lib().oracle_cache_append(self._h, layer, _u16(k_new), _u16(v_new),
                                       positions.ctypes.data_as(C.POINTER(C.c_int32)), B)
        _chk(rc, "oracle_cache_append")

    def append_many(self, layer, k_new, v_new, positions, counts=None):
        """T tokens per sequence at once: k_new, v_new uint16 [B][T][Hkv][d]; counts: rows taken per sequence."""
        positions = np.ascontiguousarray(positions, dtype=np.int32)
        B, T = k_new.shape[0], k_new.shape[1]
        assert positions.shape == (B,) and k_new.shape == (B, T, self.Hkv, self.d) and v_new.shape == k_new.shape
        cp = None
        if counts is not None:
            counts = np.ascontiguousarray(counts, dtype=np.int32)
            assert counts.shape == (B,)
            cp = counts.ctypes.data_as(C.POINTER(C.c_int32))
        rc = lib().oracle_cache_append_many(self._h, layer, _u16(k_new), _u16(v_new),
                                            positions.ctypes.data_as(C.POINTER(C.c_int32)), cp, T, B)
        _chk(rc, "oracle_cache_append_many")

    def chunk_attention(self, layer, seq, q, k, v, q_shared, k_shared, scale):
        """Attention of a chunk of new tokens (not stored yet at this layer) over the cache and the chunk.
        q, q_shared: uint16 [T][Hq][d]; k, v, k_shared: uint16 [T][Hkv][d].  Returns float64 [T][Hq][d]."""
        T, Hq, d = q.shape
        assert k.shape == (T, self.Hkv, d) and v.shape == k.shape
        out = np.empty((T, Hq, d), dtype=np.float64)
        rc = lib().oracle_chunk_attention(self._h, layer, seq, Hq, float(scale), T, _u16(q), _u16(k), _u16(v),
                                          _u16(q_shared), _u16(k_shared), out.ctypes.data_as(C.POINTER(C.c_double)))
        _chk(rc, "oracle_chunk_attention")
        return out

    def fill(self, layer, seq, k, v):
        n = k.shape[0]
        assert k.shape == (n, self.Hkv, self.d) and v.shape == k.shape
        _chk(lib().oracle_cache_fill(self._h, layer, seq, n, _u16(k), _u16(v)), "oracle_cache_fill")

    def export(self, layer, seq):
        """dict of uint16 arrays [tokens][Hkv][d]: sinkK, sinkV, recentK, recentV, distV and,
        at a layer that is the lowest of a block for some kv head, distK (zeros in the other heads' slices)."""
        counts = (C.c_long * 3)()
        _chk(lib().oracle_cache_export(self._h, layer, seq, counts, *([None] * 6)), "oracle_cache_export")
        ns, nr, nd = counts[0], counts[1], counts[2]
        mk = lambda t: np.zeros((t, self.Hkv, self.d), dtype=np.uint16)
        out = dict(sinkK=mk(ns), sinkV=mk(ns), recentK=mk(nr), recentV=mk(nr), distV=mk(nd))
        lowest = bool((self.lowest[layer] == layer).any())   # a lowest layer for at least one kv head
        if lowest:
            out["distK"] = mk(nd)
        rc = lib().oracle_cache_export(self._h, layer, seq, counts, _u16(out["sinkK"]), _u16(out["sinkV"]),
                                       _u16(out["recentK"]), _u16(out["recentV"]),
                                       _u16(out["distK"]) if lowest else None, _u16(out["distV"]))
        _chk(rc, "oracle_cache_export")
        return out

    def stored_elems(self):
        return lib().oracle_cache_stored_elems(self._h)

    def decode_attention(self, layer, q, q_shared, ctx_lens, scale):
        B, Hq, d = q.shape
        ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        out = np.empty((B, Hq, d), dtype=np.float64)
        rc = lib().oracle_decode_attention(self._h, layer, Hq, float(scale), _u16(q), _u16(q_shared),
                                           ctx_lens.ctypes.data_as(C.POINTER(C.c_int32)), B,
                                           out.ctypes.data_as(C.POINTER(C.c_double)))
        _chk(rc, "oracle_decode_attention")
        return out

    def decode_attention_gated(self, layer, q, q_shared, ctx_lens, scale, tau):
        """Decode attention with the gated skip of distant tokens; returns (out, g, skipped)."""
        B, Hq, d = q.shape
        ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        out = np.empty((B, Hq, d), dtype=np.float64)
        g = np.empty((B, Hq), dtype=np.float64)
        skipped = np.empty((B, Hq), dtype=np.int32)
        rc = lib().oracle_decode_attention_gated(self._h, layer, Hq, float(scale), _u16(q), _u16(q_shared),
                                                 ctx_lens.ctypes.data_as(C.POINTER(C.c_int32)), B, float(tau),
                                                 out.ctypes.data_as(C.POINTER(C.c_double)),
                                                 g.ctypes.data_as(C.POINTER(C.c_double)),
                                                 skipped.ctypes.data_as(C.POINTER(C.c_int32)))
        _chk(rc, "oracle_decode_attention_gated")
        return out, g, skipped
