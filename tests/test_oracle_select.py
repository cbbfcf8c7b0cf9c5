"""Pins for the oracle's smoothing, chunk selection and position restoration."""
import os

import numpy as np
import pytest

from oracle import specprefill_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _cu(lens):
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    return cu


# ------------------------------ a4: pooling ---------------------------------
def test_pool_window_one_is_identity():
    x = np.random.default_rng(0).random(37)
    assert (orc.avg_pool(x, _cu([37]), 1) == x).all()


def test_pool_uniform_stays_uniform_including_edges():
    x = np.full(20, 0.125)
    np.testing.assert_allclose(orc.avg_pool(x, _cu([20]), 7), 0.125, rtol=1e-15)
    np.testing.assert_allclose(orc.avg_pool(x, _cu([3, 17]), 13), 0.125, rtol=1e-15)


def test_pool_hand_computed_seven_elements():
    x = np.array([1.0, 2.0, 4.0, 8.0, 16.0, 32.0, 64.0])
    got = orc.avg_pool(x, _cu([7]), 3)
    want = [(1 + 2) / 2, (1 + 2 + 4) / 3, (2 + 4 + 8) / 3, (4 + 8 + 16) / 3, (8 + 16 + 32) / 3,
            (16 + 32 + 64) / 3, (32 + 64) / 2]
    np.testing.assert_allclose(got, want, rtol=1e-15)
    got5 = orc.avg_pool(x, _cu([7]), 5)
    want5 = [7 / 3, 15 / 4, 31 / 5, 62 / 5, 124 / 5, 120 / 4, 112 / 3]
    np.testing.assert_allclose(got5, want5, rtol=1e-15)


def test_pool_preserves_mass_of_interior_bump_and_never_crosses_sequences():
    x = np.zeros(40)
    x[18:22] = [1.0, 3.0, 2.0, 5.0]
    assert abs(orc.avg_pool(x, _cu([40]), 9).sum() - x.sum()) < 1e-12
    # a spike at the end of sequence 0 must not leak into sequence 1
    y = np.zeros(30)
    y[9] = 1.0
    p = orc.avg_pool(y, _cu([10, 20]), 5)
    assert (p[10:] == 0).all() and p[9] == 1.0 / 3 and p[7] == 1.0 / 5


# ------------------------------ a5: chunk means -----------------------------
def test_chunk_means_with_short_tail():
    x = np.arange(10, dtype=np.float64)
    cs, cu_c = orc.chunk_means(x, _cu([10]), 4)
    assert cu_c.tolist() == [0, 3]
    np.testing.assert_allclose(cs, [1.5, 5.5, 8.5])
    cs2, cu_c2 = orc.chunk_means(x, _cu([3, 7]), 4)
    assert cu_c2.tolist() == [0, 1, 3]
    np.testing.assert_allclose(cs2, [1.0, 4.5, 8.0])


# ------------------------------ a6: k and top-k -----------------------------
def test_keep_count_formula():
    assert orc.keep_count(10, 0.3) == 3          # 0.3 * 10 = 3.0000000000000004 must not become 4
    assert orc.keep_count(32, 0.25) == 8
    assert orc.keep_count(256, 0.1) == 26
    assert orc.keep_count(1024, 0.1) == 103
    assert orc.keep_count(2048, 0.05) == 103
    assert orc.keep_count(5, 0.01) == 1
    assert orc.keep_count(7, 1.0) == 7
    assert orc.keep_count(1, 0.5) == 1
    assert orc.keep_count(0, 0.5) == 0


def test_token_topk_equals_full_sort_brute_force():
    g = np.random.default_rng(1)
    for trial in range(20):
        M = int(g.integers(1, 60))
        x = g.random(M)
        if trial % 2:
            x = np.round(x * 4) / 4                 # many ties
        rate = float(g.choice([0.1, 0.3, 0.5, 1.0]))
        kept, cu_keep, cs, _ = orc.pool_select(x, _cu([M]), 1, 1, rate)
        k = orc.keep_count(M, rate)
        ranked = sorted(range(M), key=lambda j: (-x[j], j))
        assert kept.tolist() == sorted(ranked[:k])
        assert cu_keep.tolist() == [0, k]
        assert (cs == x).all()


def test_keep_rate_one_keeps_everything_in_order():
    x = np.random.default_rng(2).random(77)
    kept, cu_keep, _, _ = orc.pool_select(x, _cu([30, 47]), 8, 5, 1.0)
    assert kept.tolist() == list(range(77))
    assert cu_keep.tolist() == [0, 30, 77]


def test_all_equal_scores_keep_the_first_chunks():
    x = np.full(64, 0.5)
    kept, cu_keep, _, _ = orc.pool_select(x, _cu([64]), 8, 3, 0.25)
    assert kept.tolist() == list(range(16))


def test_kept_token_count_with_partial_last_chunk():
    # 10 tokens, chunk 4 -> chunks {0..3},{4..7},{8,9}; make the short tail the best chunk
    x = np.array([0, 0, 0, 0, 1, 1, 1, 1, 9, 9], dtype=np.float64)
    kept, cu_keep, cs, _ = orc.pool_select(x, _cu([10]), 4, 1, 0.5)
    assert kept.tolist() == [4, 5, 6, 7, 8, 9] and cu_keep.tolist() == [0, 6]


def test_batch_result_is_concatenation_of_single_runs():
    g = np.random.default_rng(3)
    lens = [50, 7, 33, 1]
    x = g.random(sum(lens))
    cu = _cu(lens)
    kept, cu_keep, cs, cu_c = orc.pool_select(x, cu, 8, 5, 0.3)
    off = 0
    for b, M in enumerate(lens):
        kb, ckb, csb, _ = orc.pool_select(x[cu[b]:cu[b + 1]], _cu([M]), 8, 5, 0.3)
        assert (kept[cu_keep[b]:cu_keep[b + 1]] == kb + cu[b]).all()
        assert cu_keep[b + 1] - cu_keep[b] == ckb[1]
        np.testing.assert_array_equal(cs[cu_c[b]:cu_c[b + 1]], csb)


def test_order_is_pool_then_chunk_then_topk():
    # one isolated spike at a chunk border: pooling spreads it into the neighbour chunk.
    x = np.zeros(16)
    x[7] = 1.0                                       # last token of chunk 1 (chunk = 4)
    x[12] = 0.3                                      # chunk 3
    # pooled by hand (window 3): p[6]=p[7]=p[8]=1/3, p[11]=p[12]=p[13]=0.1, rest 0.
    # Without pooling chunk 2 would score 0 and chunk 3 would be second; with it chunk 2 wins.
    kept, _, cs, _ = orc.pool_select(x, _cu([16]), 4, 3, 0.5)
    np.testing.assert_allclose(cs, [0.0, (1 / 3 + 1 / 3) / 4, (1 / 3 + 0.1) / 4, (0.1 + 0.1) / 4], rtol=1e-14)
    kept_raw, _, _, _ = orc.pool_select(x, _cu([16]), 4, 1, 0.5)
    assert kept_raw.tolist() == [4, 5, 6, 7, 12, 13, 14, 15]
    assert kept.tolist() == [4, 5, 6, 7, 8, 9, 10, 11]


# ------------------------------ a8: positions -------------------------------
def _read_golden():
    vals = {}
    with open(os.path.join(GOLDEN, "position_ids_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = [int(v) for v in rest]
    return vals


def test_paper_position_id_example():
    gold = _read_golden()
    M = gold["prompt_len"][0]
    keep = gold["speculated_pos_ids"]
    scores = np.full(M, 0.01)
    scores[keep] = [0.9, 0.8, 0.7, 0.6, 0.5]
    kept, cu_keep, _, _ = orc.pool_select(scores, _cu([M]), 1, 1, 0.5)
    ids = np.arange(100, 100 + M, dtype=np.int32)
    kept_ids, kept_pos, decode_pos, _ = orc.gather(kept, cu_keep, _cu([M]), ids)
    assert kept_pos.tolist() == keep
    assert kept_ids.tolist() == [100 + p for p in keep]
    assert [int(decode_pos[0]) + i for i in range(3)] == gold["decoding_pos_ids"]
    assert list(range(M)) == gold["original_pos_ids"]


def test_positions_restart_in_every_sequence_and_rows_are_table_rows():
    g = np.random.default_rng(4)
    lens = [12, 20]
    cu = _cu(lens)
    x = g.random(32)
    kept, cu_keep, _, _ = orc.pool_select(x, cu, 4, 1, 0.5)
    ids = g.integers(0, 50, size=32).astype(np.int32)
    table = g.integers(0, 65535, size=(50, 6)).astype(np.uint16)
    kept_ids, kept_pos, decode_pos, rows = orc.gather(kept, cu_keep, cu, ids, table)
    assert decode_pos.tolist() == lens
    for b in range(2):
        seg = slice(cu_keep[b], cu_keep[b + 1])
        assert (kept_pos[seg] == kept[seg] - cu[b]).all()
        assert (np.diff(kept_pos[seg]) > 0).all()
        assert kept_pos[seg].min() >= 0 and kept_pos[seg].max() < lens[b]
    assert (rows == table[ids[kept]]).all()
    with pytest.raises(AssertionError):
        orc.gather(kept, cu_keep, cu, ids + 100, table)
