"""The seeded generators: determinism, sharing structure, and the sizes the roofline figures use."""
import json
import os

import numpy as np

import oracle
import workloads as W


def test_tiny_config_is_deterministic_and_shares_its_prefix():
    a, b = W.tiny_decode(), W.tiny_decode()
    np.testing.assert_array_equal(a.pool, b.pool)
    np.testing.assert_array_equal(a.block_tables, b.block_tables)
    assert a.B == 8 and a.geom.head_dim == 64 and a.geom.num_q_heads == 4
    assert (a.block_tables[:, :8] == a.block_tables[0, :8]).all()          # 128-token prefix = 8 shared blocks
    tails = a.block_tables[:, 8:]
    live_tail = tails[tails >= 0]
    assert len(set(live_tail.tolist())) == live_tail.size                  # suffix blocks are private
    assert ((a.seq_lens >= 129) & (a.seq_lens <= 193)).all()


def test_golden_tiny_decode_oracle_values():
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_decode_oracle.json")
    rec = json.load(open(path))
    w = W.tiny_decode()
    assert rec["seq_lens"] == [int(x) for x in w.seq_lens]
    out = oracle.attention(w.geom, w.pool, w.q, w.block_tables, w.seq_lens, w.scale)
    for key, vals in rec["rows"].items():
        r, h = (int(x) for x in key.split(","))
        np.testing.assert_allclose(out[r, h, :8], [float.fromhex(v) for v in vals], rtol=0, atol=1e-15)


def test_llama8b_decode_shape_and_bytes():
    w = W.llama8b_decode()
    assert w.B == 64 and w.geom.num_q_heads == 32 and w.geom.num_kv_heads == 8 and w.geom.head_dim == 128
    groups = w.meta["prefix_groups"]
    assert len(groups) == 4 and all(len(g) == 16 for g in groups)
    for g in groups:
        assert (w.block_tables[g, :128] == w.block_tables[g[0], :128]).all()
    assert len({int(w.block_tables[g[0], 0]) for g in groups}) == 4
    assert ((w.seq_lens >= 2048 + 128 + 1) & (w.seq_lens <= 2048 + 1024 + 1)).all()
    # 4 KiB per distinct cached token
    assert w.unique_kv_bytes() == (4 * 2048 + int((w.seq_lens - 2048).sum())) * 4096
    assert w.logical_kv_bytes() == int(w.seq_lens.sum()) * 4096
    live = w.live_block_ids()
    assert (w.pool[live[0]] != W.gen.SENTINEL_BITS).any()
    dead = np.setdiff1d(np.arange(w.geom.num_blocks), live)
    assert (w.pool[dead] == W.gen.SENTINEL_BITS).all()


def test_prefill_flop_count_is_the_exact_causal_count():
    w = W.custom_prefill(1, prefix_groups=[list(range(16))], prefix_tokens=[4096], q_lens=[512] * 16, num_q_heads=32,
                         num_kv_heads=8, head_dim=8, block_size=16)
    assert w.visible_pairs() == 35655680
    assert w.visible_pairs() * 32 * 4 * 128 == 584182661120


def test_churn_step_lists_are_consistent():
    w = W.eviction_churn(branches=16, median=300, lo=64, hi=1200, head_dim=8, num_q_heads=4, num_kv_heads=2)
    live = set(w.live_block_ids().tolist())
    assert abs(len(live) / w.geom.num_blocks - 0.8) < 0.02
    for fam, fp in zip(w.meta["families"], w.meta["fork_points"]):
        nsh = fp // 16
        assert fp % 16 != 0
        assert (w.block_tables[fam, :nsh] == w.block_tables[fam[0], :nsh]).all()
        assert len(set(w.block_tables[fam, nsh].tolist())) == len(fam)
    st = W.churn_step(w, 0, n_fork=4)
    assert not (set(st.fork_dst.tolist()) & live) and not (set(st.readmit_ids.tolist()) & live)
    assert not (set(st.fork_dst.tolist()) & set(st.readmit_ids.tolist()))
    assert len(set(st.readmit_ids.tolist())) == st.readmit_ids.size == st.evict_ids.size
    assert ((st.fork_ntok >= 1) & (st.fork_ntok <= 16)).all()
    assert not (set(st.evict_ids.tolist()) & set(st.block_tables[st.block_tables >= 0].tolist()))


def test_agent_trace_is_seeded_and_well_formed():
    a = list(W.agent_trace(n_sessions=6, concurrency=3))
    b = list(W.agent_trace(n_sessions=6, concurrency=3))
    assert a == b
    ended = [op[1] for op in a if op[0] == "end"]
    assert sorted(ended) == list(range(6))
    for op in a:
        if op[0] == "call":
            _, names, tiers, sess = op
            assert len(names) == len(tiers) and set(tiers) <= {1, 2, 4}
            assert tiers == sorted(tiers)[:len(tiers)] or tiers[-1] == 4      # prefix (I), notebook (II), question (IV)
            assert names[0].startswith("P") and sess not in ended[:0]
