"""Pins for the oracle's paged decode attention (CPU only).

None of the expected values below comes from the function under test: they come from numpy's
textbook softmax attention on the logical tensors, from closed forms (one token, zero query,
equal keys), from invariances the mathematics fixes, and from the paper's printed logical
table example.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP, Geometry, View
from paper_2602_22593_amd import workloads as wl

from helpers import Case, bf16_bits_to_f64, make_case, make_mixed_case, q_slice, textbook_attention

TINY = wl.WORKLOADS["tiny"]
TINY_VIEWS = [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 0), (LAYOUT_TP, 2, 1), (LAYOUT_DP, 2, 1)]


def rank_rows(full: np.ndarray, info: dict, rank: int) -> np.ndarray:
    hql = info["n_q_local"]
    return full[:, rank * hql:(rank + 1) * hql, :]


@pytest.mark.parametrize("view", TINY_VIEWS)
def test_paged_equals_textbook_on_logical_tensors(view):
    """Tiny config: scatter -> paged decode through the view must equal numpy's
    softmax(q K^T / sqrt(d)) V computed on the un-paged logical K, V (GQA map h -> h // G),
    restricted to the rank's query heads.  Covers the address map, the table indirection,
    the head partition and the attention arithmetic at once; the pool is NaN-poisoned, so
    any read outside the valid tokens shows up as NaN."""
    c = make_case(TINY, view)
    want = textbook_attention(c.q_full, c.K, c.V, c.seq_off, TINY.n_q_heads, TINY.n_kv_heads,
                              1.0 / np.sqrt(TINY.head_dim))
    got = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, rank_rows(want, c.info, c.view.rank), rtol=0, atol=1e-12)


@pytest.mark.parametrize("rank", [0, 1])
def test_mixed_layouts_in_one_batch_equal_textbook(rank):
    """Sequences stored under two layouts in one pool (the TP layout of rank r, and rank r's head
    slice inside DP-layout blocks), one block table whose rows are indexed with each sequence's own
    block capacity: the per-sequence-view oracle must equal numpy's textbook attention on the
    logical tensors, whatever the layout.  A wrong capacity, stride or head offset for either
    layout reads NaN poison or another head."""
    ctx = np.array([17, 64, 150, 300, 1, 33, 0, 95], dtype=np.int32)
    ids = np.array([0, 1, 1, 0, 1, 0, 1, 0], dtype=np.int32)
    c = make_mixed_case(TINY, [(LAYOUT_TP, 2, rank), (LAYOUT_DP, 2, rank)], ids, ctx)
    want = textbook_attention(c.q_full, c.K, c.V, c.seq_off, TINY.n_q_heads, TINY.n_kv_heads,
                              1.0 / np.sqrt(TINY.head_dim))
    got = oracle.paged_decode_mixed(c.views, c.view_ids, c.q, c.pool, c.table, c.ctx)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, rank_rows(want, c.views[0].query(), rank), rtol=0, atol=1e-12)
    # reading every sequence under one layout must NOT work (the pin can tell the layouts apart)
    wrong = oracle.paged_decode(c.views[0], c.q, c.pool, c.table, c.ctx)
    assert not np.isfinite(wrong[ids == 1][ctx[ids == 1] > 0]).all()


def test_dense_oracle_equals_textbook_and_paged():
    c = make_case(TINY, (LAYOUT_DP, 1, 0))
    scale = 0.37
    want = textbook_attention(c.q_full, c.K, c.V, c.seq_off, TINY.n_q_heads, TINY.n_kv_heads, scale)
    dense = oracle.dense_decode(c.geom, c.q_full, c.K, c.V, c.seq_off, scale)
    paged = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx, scale)
    np.testing.assert_allclose(dense, want, rtol=0, atol=1e-12)
    np.testing.assert_allclose(paged, dense, rtol=0, atol=1e-12)
    # the scale really enters: default (1/sqrt(d) = 0.125) differs from 0.37
    assert np.abs(oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx) - paged).max() > 1e-3


@pytest.mark.parametrize("p", [1, 2, 4, 8])
def test_tp_view_is_the_head_slice_of_dp(p):
    """Heads are disjoint per rank and attention needs no cross-rank exchange (Sec. 4.1.1):
    the TP(p, r) output equals rows [r*Hq/p, (r+1)*Hq/p) of the DP output, exactly (same fp64
    operations in the same order)."""
    w = wl.Workload("g8", 7, 32, 8, 32, 4, 3, "x", ())
    ctx = np.array([5, 33, 70], dtype=np.int32)
    dp = make_case(w, (LAYOUT_DP, 1, 0), ctx)
    full = oracle.paged_decode(dp.view, dp.q, dp.pool, dp.table, dp.ctx)
    for r in range(p):
        for layout in (LAYOUT_TP, LAYOUT_DP):
            if layout == LAYOUT_DP and p == 1 and r == 0:
                continue
            c = make_case(w, (layout, p, r), ctx, K=dp.K, V=dp.V, q_full=dp.q_full)
            got = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
            assert np.array_equal(got, rank_rows(full, c.info, r)), (layout, p, r)


def test_single_token_returns_v_row():
    """softmax over one token is 1, so out = V exactly (bf16-exact values in fp64)."""
    ctx = np.array([1, 1, 1, 1], dtype=np.int32)
    for view in TINY_VIEWS:
        c = make_case(TINY, view, ctx)
        got = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
        G = c.info["group"]
        for s in range(4):
            for i in range(c.info["n_q_local"]):
                g = c.info["kv_head0"] + i // G
                assert np.array_equal(got[s, i], bf16_bits_to_f64(c.V[c.seq_off[s], g]))


def test_zero_query_and_equal_keys_give_the_mean_of_v():
    """q = 0 makes all scores 0; equal K rows make all scores equal: out = mean_t V_t."""
    ctx = np.array([7, 40], dtype=np.int32)
    w = wl.Workload("t2", 8, 8, 2, 64, 16, 2, "x", ())
    base = make_case(w, (LAYOUT_TP, 2, 1), ctx)
    Vf = bf16_bits_to_f64(base.V)
    # (a) zero query
    q0 = np.zeros_like(base.q)
    got = oracle.paged_decode(base.view, q0, base.pool, base.table, base.ctx)
    for s in range(2):
        mean = Vf[base.seq_off[s]:base.seq_off[s + 1], 1, :].mean(axis=0)
        for i in range(base.info["n_q_local"]):
            np.testing.assert_allclose(got[s, i], mean, rtol=0, atol=1e-13)
    # (b) all K rows of a sequence equal
    K2 = base.K.copy()
    for s in range(2):
        K2[base.seq_off[s]:base.seq_off[s + 1]] = K2[base.seq_off[s]]
    c = make_case(w, (LAYOUT_TP, 2, 1), ctx, K=K2, V=base.V, q_full=base.q_full)
    got = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    for s in range(2):
        mean = Vf[c.seq_off[s]:c.seq_off[s + 1], 1, :].mean(axis=0)
        for i in range(c.info["n_q_local"]):
            np.testing.assert_allclose(got[s, i], mean, rtol=0, atol=1e-12)


def test_output_is_a_convex_combination_of_v_rows():
    c = make_case(TINY, (LAYOUT_DP, 1, 0))
    got = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    Vf = bf16_bits_to_f64(c.V)
    G = c.info["group"]
    for s in range(len(c.ctx)):
        rows = Vf[c.seq_off[s]:c.seq_off[s + 1]]
        for i in range(TINY.n_q_heads):
            lo, hi = rows[:, i // G, :].min(axis=0), rows[:, i // G, :].max(axis=0)
            assert (got[s, i] >= lo - 1e-12).all() and (got[s, i] <= hi + 1e-12).all()


def test_token_order_does_not_matter():
    """Permuting a sequence's tokens (K and V rows together) leaves the result unchanged up
    to fp64 rounding."""
    c = make_case(TINY, (LAYOUT_TP, 2, 0))
    rng = np.random.default_rng(5)
    K2, V2 = c.K.copy(), c.V.copy()
    for s in range(len(c.ctx)):
        a, b = int(c.seq_off[s]), int(c.seq_off[s + 1])
        perm = rng.permutation(b - a) + a
        K2[a:b], V2[a:b] = c.K[perm], c.V[perm]
    c2 = make_case(TINY, (LAYOUT_TP, 2, 0), K=K2, V=V2, q_full=c.q_full)
    a = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    b = oracle.paged_decode(c2.view, c2.q, c2.pool, c2.table, c2.ctx)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


def test_physical_block_permutation_is_invisible():
    """Moving the blocks around in the pool together with the table changes nothing, bit for
    bit: only the table decides where a token lives."""
    c = make_case(TINY, (LAYOUT_DP, 1, 0))
    rng = np.random.default_rng(11)
    perm = rng.permutation(c.pool.shape[0]).astype(np.int32)   # old id -> new id
    pool2 = np.empty_like(c.pool)
    pool2[perm] = c.pool
    table2 = np.where(c.table >= 0, perm[np.clip(c.table, 0, None)], -1).astype(np.int32)
    a = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    b = oracle.paged_decode(c.view, c.q, pool2, table2, c.ctx)
    assert np.array_equal(a, b)


def test_split_and_merge_equals_whole():
    """Partial results over two token ranges, combined with
    m = max(m1, m2), l = l1 e^{m1-m} + l2 e^{m2-m}, acc = acc1 e^{m1-m} + acc2 e^{m2-m},
    give the whole-context result (the identity the split-KV merge relies on)."""
    c = make_case(TINY, (LAYOUT_TP, 2, 1))
    whole = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    for s, n in enumerate(c.ctx):
        for head in range(c.info["n_q_local"]):
            for cut in (1, int(n) // 2, int(n) - 1):
                a1, m1, l1 = oracle.paged_decode_partial(c.view, c.q, c.pool, c.table, s, head, 0, cut)
                a2, m2, l2 = oracle.paged_decode_partial(c.view, c.q, c.pool, c.table, s, head, cut, int(n))
                m = max(m1, m2)
                l = l1 * np.exp(m1 - m) + l2 * np.exp(m2 - m)
                acc = a1 * np.exp(m1 - m) + a2 * np.exp(m2 - m)
                np.testing.assert_allclose(acc / l, whole[s, head], rtol=0, atol=1e-12)


def test_tail_slots_and_spare_blocks_never_matter():
    """Only tokens t < ctx_len take part: overwriting every unused slot, every unused block
    and every table entry past the last block leaves the result bit-identical."""
    c = make_case(TINY, (LAYOUT_TP, 2, 0))
    ref = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    pool2 = c.pool.copy()
    poisoned = pool2 == wl.BF16_NAN
    assert poisoned.any()
    rng = np.random.default_rng(3)
    pool2[poisoned] = rng.integers(0, 0x7F00, size=int(poisoned.sum()), dtype=np.uint16)
    table2 = c.table.copy()
    table2[table2 < 0] = 0
    assert np.array_equal(ref, oracle.paged_decode(c.view, c.q, pool2, table2, c.ctx))


def test_zero_length_context_gives_zeros():
    ctx = np.array([0, 9, 0, 16], dtype=np.int32)
    c = make_case(TINY, (LAYOUT_DP, 1, 0), ctx)
    got = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    assert np.array_equal(got[0], np.zeros_like(got[0])) and np.array_equal(got[2], np.zeros_like(got[2]))
    want = textbook_attention(c.q_full, c.K, c.V, c.seq_off, 8, 2, 0.125)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_pairs_entry_point_matches_rows():
    c = make_case(TINY, (LAYOUT_TP, 2, 1))
    full = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    ps = np.array([3, 0, 2, 2], dtype=np.int32)
    ph = np.array([1, 3, 0, 2], dtype=np.int32)
    got = oracle.paged_decode_pairs(c.view, c.q, c.pool, c.table, c.ctx, ps, ph)
    for k in range(4):
        assert np.array_equal(got[k], full[ps[k], ph[k]])


def read_table_example(golden_dir):
    rows = {}
    with open(os.path.join(golden_dir, "logical_table_example.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                parts = [int(x) for x in line.split()]
                rows[parts[0]] = parts[1:]
    return rows


def test_paper_logical_table_example(golden_dir):
    """The paper's example table (Sec. 4.2.2): request 0 -> blocks {1,3}, 1 -> {0}, 2 -> {2}.
    The pool is filled here with numpy indexing of the [n_blocks][2][B][H][d] array (not with
    the oracle's scatter); gather must return those rows in request order and attention must
    equal the textbook result on them."""
    mapping = read_table_example(golden_dir)
    assert mapping == {0: [1, 3], 1: [0], 2: [2]}
    geom = Geometry(4, 2, 8, 4)
    view = View(geom, LAYOUT_DP, 1, 0)
    ctx = np.array([7, 3, 4], dtype=np.int32)          # request 0 spills into its 2nd block
    table = np.full((3, 2), -1, dtype=np.int32)
    for req, blocks in mapping.items():
        table[req, :len(blocks)] = blocks
    g = wl.generator(9, wl.SUB_DATA)
    pool5 = wl.randn_bf16((4, 2, 4, 2, 8), g)          # every slot holds distinct random data
    seq_off = wl.seq_offsets(ctx)
    K = np.zeros((int(ctx.sum()), 2, 8), dtype=np.uint16)
    V = np.zeros_like(K)
    for req in range(3):
        for t in range(ctx[req]):
            blk = mapping[req][t // 4]
            K[seq_off[req] + t] = pool5[blk, 0, t % 4]
            V[seq_off[req] + t] = pool5[blk, 1, t % 4]
    Kg, Vg = np.zeros_like(K), np.zeros_like(V)
    pool = pool5.reshape(4, -1)
    oracle.gather(view, pool, table, ctx, seq_off, Kg, Vg)
    assert np.array_equal(Kg, K) and np.array_equal(Vg, V)
    q = wl.randn_bf16((3, 4, 8), g)
    want = textbook_attention(q, K, V, seq_off, 4, 2, 1.0 / np.sqrt(8))
    got = oracle.paged_decode(view, q, pool, table, ctx)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_capacity_reinterpretation_fig4(golden_dir):
    """Fig. 4's picture on one physical block: a block written as 2TP (8 tokens x H/2 heads,
    B_base = 4) read back with numpy as [2][8][H/2][d] holds the rank's rows; the same bytes
    read as DP would be 4 tokens x H heads -- same byte count."""
    geom = Geometry(4, 2, 8, 4)
    tp = View(geom, LAYOUT_TP, 2, 1)
    ctx = np.array([8], dtype=np.int32)
    K = wl.randn_bf16((8, 2, 8), wl.generator(9, wl.SUB_MISC))
    V = wl.randn_bf16((8, 2, 8), wl.generator(9, wl.SUB_QUERY))
    pool = wl.poisoned_pool(2, tp.query()["block_bytes"] // 2)
    table = np.array([[1]], dtype=np.int32)
    oracle.scatter(tp, pool, table, ctx, wl.seq_offsets(ctx), K, V)
    blk = pool[1].reshape(2, 8, 1, 8)
    assert np.array_equal(blk[0, :, 0, :], K[:, 1, :]) and np.array_equal(blk[1, :, 0, :], V[:, 1, :])
    assert (pool[0] == wl.BF16_NAN).all()
    assert pool[1].size == 2 * 4 * 2 * 8  # = DP's [2][4 tokens][2 heads][8]
