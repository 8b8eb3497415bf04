"""Builds oracle/glm_oracle.c with gcc and exposes it through ctypes (numpy in, numpy out)."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "glm_oracle.c")
_LIB = os.path.join(_HERE, "libglm_oracle.so")
_lib = None


class _Geom(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("num_blocks", "block_size", "num_kv_heads", "num_q_heads", "head_dim")]


def lib_path() -> str:
    return _LIB


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.glm_oracle_attention_weights.restype = ctypes.c_int64
    return _lib


def _geom(g) -> _Geom:
    return _Geom(g.num_blocks, g.block_size, g.num_kv_heads, g.num_q_heads, g.head_dim)


def _p(a: Optional[np.ndarray], dtype):
    if a is None:
        return None
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _threads(n: Optional[int]) -> int:
    return int(n) if n else (os.cpu_count() or 1)


def attention(geom, pool, q, block_tables, seq_lens, scale, cu_q_lens=None, nthreads: Optional[int] = None):
    """All output rows, float64 [sum_q, Hq, d] (decode: [B, Hq, d])."""
    bt, sl, cu = _i32(block_tables), _i32(seq_lens), _i32(cu_q_lens)
    B = sl.shape[0]
    rows = int(cu[B]) if cu is not None else B
    out = np.zeros((rows, geom.num_q_heads, geom.head_dim), np.float64)
    pool = np.ascontiguousarray(pool); q = np.ascontiguousarray(q)
    st = _load().glm_oracle_attention(_geom(geom), _p(pool, np.uint16), _p(q, np.uint16), _p(out, np.float64),
                                      _p(bt, np.int32), ctypes.c_int32(bt.shape[1]), _p(sl, np.int32), _p(cu, np.int32),
                                      ctypes.c_int32(B), ctypes.c_float(scale), ctypes.c_int32(_threads(nthreads)))
    if st:
        raise RuntimeError("oracle attention failed: %d" % st)
    return out


def attention_rows(geom, pool, q, block_tables, seq_lens, scale, sel_req, sel_h, sel_i=None, cu_q_lens=None,
                   nthreads: Optional[int] = None):
    """Selected rows only: float64 [n_sel, d] for (request, new-token index, q head) triples."""
    bt, sl, cu = _i32(block_tables), _i32(seq_lens), _i32(cu_q_lens)
    sr, sh, si = _i32(sel_req), _i32(sel_h), _i32(sel_i)
    out = np.zeros((sr.shape[0], geom.head_dim), np.float64)
    pool = np.ascontiguousarray(pool); q = np.ascontiguousarray(q)
    st = _load().glm_oracle_attention_rows(_geom(geom), _p(pool, np.uint16), _p(q, np.uint16), _p(out, np.float64),
                                           _p(bt, np.int32), ctypes.c_int32(bt.shape[1]), _p(sl, np.int32),
                                           _p(cu, np.int32), ctypes.c_int32(sl.shape[0]), ctypes.c_float(scale),
                                           _p(sr, np.int32), _p(si, np.int32), _p(sh, np.int32),
                                           ctypes.c_int32(sr.shape[0]), ctypes.c_int32(_threads(nthreads)))
    if st:
        raise RuntimeError("oracle attention_rows failed: %d" % st)
    return out


def attention_weights(geom, pool, q, block_tables, seq_lens, scale, r, h, i=0, cu_q_lens=None):
    """(weights float64 [n_visible], out float64 [d]) of one row."""
    bt, sl, cu = _i32(block_tables), _i32(seq_lens), _i32(cu_q_lens)
    w = np.zeros(max(1, int(sl[r])), np.float64)
    out = np.zeros(geom.head_dim, np.float64)
    pool = np.ascontiguousarray(pool); q = np.ascontiguousarray(q)
    n = _load().glm_oracle_attention_weights(_geom(geom), _p(pool, np.uint16), _p(q, np.uint16), _p(bt, np.int32),
                                             ctypes.c_int32(bt.shape[1]), _p(sl, np.int32), _p(cu, np.int32),
                                             ctypes.c_int32(sl.shape[0]), ctypes.c_float(scale), ctypes.c_int32(r),
                                             ctypes.c_int32(i), ctypes.c_int32(h), _p(w, np.float64), _p(out, np.float64))
    if n < 0:
        raise RuntimeError("oracle attention_weights failed: %d" % n)
    return w[:n], out


def fork_copy(geom, pool, src_ids, dst_ids, n_tokens) -> None:
    """In place on `pool` (uint16 [num_blocks, 2, Hkv, bs, d])."""
    s, t, n = _i32(src_ids), _i32(dst_ids), _i32(n_tokens)
    assert pool.dtype == np.uint16 and pool.flags["C_CONTIGUOUS"]
    st = _load().glm_oracle_fork_copy(_geom(geom), _p(pool, np.uint16), _p(s, np.int32), _p(t, np.int32),
                                      _p(n, np.int32), ctypes.c_int32(s.shape[0]))
    if st:
        raise RuntimeError("oracle fork_copy failed: %d" % st)


def gather(geom, src, src_ids, dst, dst_ids, n: Optional[int] = None) -> None:
    """dst[dst_ids[k]] = src[src_ids[k]] for whole blocks; either list may be None (identity)."""
    s, t = _i32(src_ids), _i32(dst_ids)
    if n is None:
        n = s.shape[0] if s is not None else t.shape[0]
    assert src.dtype == np.uint16 and dst.dtype == np.uint16 and dst.flags["C_CONTIGUOUS"]
    src = np.ascontiguousarray(src)
    st = _load().glm_oracle_gather(_geom(geom), _p(src, np.uint16), _p(s, np.int32), _p(dst, np.uint16),
                                   _p(t, np.int32), ctypes.c_int32(n))
    if st:
        raise RuntimeError("oracle gather failed: %d" % st)


def kv_append(geom, pool, k_new, v_new, slots) -> None:
    """In place on `pool`: token i's rows k_new[i], v_new[i] ([Hkv, d] uint16) go to token slot slots[i]."""
    sl = np.ascontiguousarray(slots, dtype=np.int64)
    k_new = np.ascontiguousarray(k_new); v_new = np.ascontiguousarray(v_new)
    assert pool.dtype == np.uint16 and pool.flags["C_CONTIGUOUS"]
    st = _load().glm_oracle_kv_append(_geom(geom), _p(pool, np.uint16), _p(k_new, np.uint16), _p(v_new, np.uint16),
                                      sl.ctypes.data_as(ctypes.c_void_p), ctypes.c_int32(sl.shape[0]))
    if st:
        raise RuntimeError("oracle kv_append failed: %d" % st)


def gather_tokens(geom, pool, block_tables, seq_lens, dst_offsets, dst) -> None:
    """In place on `dst` (uint16, flat): request r's tokens as [2, Hkv, seq_lens[r], d] at element dst_offsets[r]."""
    tb = np.ascontiguousarray(block_tables, dtype=np.int32)
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    off = np.ascontiguousarray(dst_offsets, dtype=np.int64)
    pool = np.ascontiguousarray(pool)
    assert dst.dtype == np.uint16 and dst.flags["C_CONTIGUOUS"]
    st = _load().glm_oracle_gather_tokens(_geom(geom), _p(pool, np.uint16), _p(tb, np.int32), ctypes.c_int32(tb.shape[1]),
                                          _p(sl, np.int32), off.ctypes.data_as(ctypes.c_void_p), ctypes.c_int32(sl.shape[0]),
                                          _p(dst, np.uint16))
    if st:
        raise RuntimeError("oracle gather_tokens failed: %d" % st)
