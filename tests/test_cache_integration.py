"""The block manager drives the attention path: block tables come from glm_cache_acquire under memory pressure,
block contents are a function of the block's key, and attention through those tables must equal attention on the
K/V assembled densely from the keys.  A hit whose block was handed to somebody else in between, or a table that
aliases two different contents, shows up as a wrong result."""
import zlib

import numpy as np
import pytest

import oracle
import paper_2511_01633_amd as glm
import workloads as W

BS = 16


def _keys(names):
    out, acc = [], b""
    for n in names:
        acc += b"/" + n.encode()
        out.append((zlib.crc32(acc) | (zlib.adler32(acc) << 32)) or 1)
    return out


def _content(key, hkv, d, salt=0):
    """bf16 bits of the K and V planes of the block with this key: [2, Hkv, 16, d]."""
    rng = np.random.default_rng([int(key) & 0xFFFFFFFF, int(key) >> 32, salt])
    return W.f32_to_bf16_bits(rng.standard_normal((2, hkv, BS, d), dtype=np.float32))


def _scenario(seed, hq, hkv, d, num_blocks=40, rounds=6, batch=5):
    """Yields, per round, (geom, pool, q, tables, seq_lens, dense) for `batch` concurrent calls."""
    rng = np.random.default_rng(seed)
    geom = W.Geometry(num_blocks, BS, hkv, hq, d)
    pool = np.full((num_blocks, 2, hkv, BS, d), 0x7FC0, np.uint16)          # bf16 NaN: a block nobody wrote must not be read
    cache = glm.Cache(num_blocks)
    written = {}                                                             # id -> key whose content the pool holds
    for p in ("PC", "PR", "PA"):
        ids, _ = cache.acquire(_keys([p]), [1], 0)
        pool[ids[0]] = _content(_keys([p])[0], hkv, d); written[int(ids[0])] = _keys([p])[0]
        cache.release(ids)
    for rnd in range(rounds):
        calls = []
        for b in range(batch):
            sess = int(rng.integers(1, 4))
            p = ("PC", "PR", "PA")[int(rng.integers(3))]
            names, tiers = [p], [1]
            if p == "PR":
                for f in range(int(rng.integers(0, 3))):
                    names.append("s%d.f%d" % (sess, f)); tiers.append(2)
            for qn in range(int(rng.integers(1, 4))):
                names.append("q%d.%d" % (int(rng.integers(0, 6)), qn)); tiers.append(4)
            keys = _keys(names) + [0]                                        # plus a partly filled private tail
            tiers = tiers + [4]
            r = cache.acquire(keys, tiers, sess, check=False)
            if isinstance(r, int):
                continue
            ids, n_hit = r
            tail_tokens = int(rng.integers(1, BS + 1))
            tail = _content(int(rng.integers(1, 1 << 62)), hkv, d, salt=1)
            dense = []
            for j, (k, i) in enumerate(zip(keys, ids)):
                i = int(i)
                if k == 0:
                    pool[i] = tail; written[i] = None
                    dense.append(tail)
                    continue
                if j < n_hit:
                    assert written.get(i) == k, "a hit points at a block that holds something else"
                else:
                    pool[i] = _content(k, hkv, d); written[i] = k                # the 'prefill' of a missed block
                dense.append(_content(k, hkv, d))
            calls.append((ids, (len(keys) - 1) * BS + tail_tokens, np.stack(dense)))
        if not calls:
            continue
        B = len(calls)
        max_blocks = max(len(c[0]) for c in calls) + 1
        tables = np.full((B, max_blocks), -1, np.int32)
        seq_lens = np.zeros(B, np.int32)
        for r, (ids, L, _) in enumerate(calls):
            tables[r, :len(ids)] = ids
            seq_lens[r] = L
        q = W.f32_to_bf16_bits(rng.standard_normal((B, hq, d), dtype=np.float32))
        yield geom, pool.copy(), q, tables, seq_lens, [c[2] for c in calls]
        for ids, _, _ in calls:
            cache.release(ids)
        if rnd % 2 == 1:
            cache.end_session(int(rng.integers(1, 4)))
    assert cache.stats()["evicted_IV"] > 0, "the scenario must run under memory pressure"


def _dense_reference(geom, q, dense_blocks, L, scale):
    """Attention of one request on its own contiguous copy of K/V: a one-request pool with the identity table."""
    nb = dense_blocks.shape[0]
    g1 = W.Geometry(nb, BS, geom.num_kv_heads, geom.num_q_heads, geom.head_dim)
    return oracle.attention(g1, np.ascontiguousarray(dense_blocks), q[None], np.arange(nb, dtype=np.int32)[None],
                            np.array([L], np.int32), scale)[0]


def test_tables_from_the_manager_address_the_right_contents():
    hq, hkv, d = 4, 2, 64
    scale = np.float32(1.0 / np.sqrt(d))
    n = 0
    for geom, pool, q, tables, seq_lens, dense in _scenario(5, hq, hkv, d):
        got = oracle.attention(geom, pool, q, tables, seq_lens, scale)
        for r in range(len(dense)):
            ref = _dense_reference(geom, q[r], dense[r], int(seq_lens[r]), scale)
            assert np.abs(got[r] - ref).max() < 1e-12
            n += 1
    assert n >= 15


@pytest.mark.gpu
@pytest.mark.parametrize("hq,hkv,d", [(8, 2, 128), (4, 4, 64)])
def test_decode_through_manager_tables(hq, hkv, d):
    import torch
    import gpu_util as gu
    scale = np.float32(1.0 / np.sqrt(d))
    for geom, pool, q, tables, seq_lens, dense in _scenario(9, hq, hkv, d):
        B = q.shape[0]
        out = torch.full((B, hq, d), float("nan"), dtype=torch.float32, device="cuda")
        plan = glm.glm_plan_create(geom, tables, tables.shape[1], seq_lens, None, B)
        ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
        glm.glm_attn_decode(geom, gu.dev(pool), gu.dev(q), out, gu.dev(tables), tables.shape[1], gu.dev(seq_lens), B,
                            float(scale), plan, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        for r in range(B):
            ref = _dense_reference(geom, q[r], dense[r], int(seq_lens[r]), scale)
            assert np.abs(got[r] - ref).max() <= gu.TOL
