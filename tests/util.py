"""Helpers for tests, written independently of the oracle and of the GPU library."""
from __future__ import annotations

import math

import numpy as np


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


def f32_to_bf16(x) -> np.ndarray:
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def dense_kv(w, r: int, kvh: int, n: int):
    """K, V of request r, kv head kvh, first n tokens, as float64 [n, d] (walks the block table)."""
    bs = w.geom.block_size
    d = w.geom.head_dim
    K = np.zeros((n, d)); V = np.zeros((n, d))
    for j in range(n):
        blk = int(w.block_tables[r, j // bs])
        K[j] = bf16_to_f64(w.pool[blk, 0, kvh, j % bs])
        V[j] = bf16_to_f64(w.pool[blk, 1, kvh, j % bs])
    return K, V


def q_row_index(w, r: int, i: int) -> int:
    return r if w.q_lens is None else int(w.cu_q_lens[r]) + i


def visible(w, r: int, i: int) -> int:
    L = int(w.seq_lens[r])
    ql = 1 if w.q_lens is None else int(w.q_lens[r])
    return L - ql + i + 1


def brute_force_row(w, r: int, i: int, h: int):
    """Pure-Python attention of one row with math.fsum; returns (weights list, out list)."""
    g = w.geom
    d, bs = g.head_dim, g.block_size
    kvh = h // (g.num_q_heads // g.num_kv_heads)
    n = visible(w, r, i)
    qrow = q_row_index(w, r, i)
    qv = [float(x) for x in bf16_to_f64(w.q[qrow, h])]
    scale = float(np.float32(w.scale))
    s = []
    vs = []
    for j in range(n):
        blk = int(w.block_tables[r][j // bs]); t = j % bs
        kv = [float(x) for x in bf16_to_f64(w.pool[blk][0][kvh][t])]
        vs.append([float(x) for x in bf16_to_f64(w.pool[blk][1][kvh][t])])
        s.append(scale * math.fsum(a * b for a, b in zip(qv, kv)))
    if n == 0:
        return [], [0.0] * d
    m = max(s)
    e = [math.exp(x - m) for x in s]
    z = math.fsum(e)
    wts = [x / z for x in e]
    out = [math.fsum(wts[j] * vs[j][c] for j in range(n)) for c in range(d)]
    return wts, out
