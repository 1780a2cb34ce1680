"""Pins for the oracle's repack, scatter and gather (CPU only): round-trip identities,
equivalence with gather-then-scatter, conservation of untouched bytes, and coexistence of
layouts in one pool (paper Sec. 5.2.3)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP, Geometry, View
from paper_2602_22593_amd import workloads as wl

from helpers import geometry, make_case, q_slice, textbook_attention

TINY = wl.WORKLOADS["tiny"]


def fresh_tables(ctx, views_and_counts, n_pool_blocks, seed_sub=wl.SUB_PERM, index=0):
    """Disjoint block tables for several (view, label) users out of one shuffled pool."""
    perm = torch.randperm(n_pool_blocks, generator=wl.generator(index, seed_sub)).numpy().astype(np.int32)
    tables, used = [], 0
    for view in views_and_counts:
        t, k = wl.assign_blocks(ctx, view.query()["block_tokens"], perm[used:])
        tables.append(t)
        used += k
    return tables, used


def test_scatter_then_gather_is_identity_per_view():
    geom = geometry(TINY)
    ctx = wl.draw_ctx_lens(TINY)
    K, V = wl.logical_kv(TINY, ctx)
    off = wl.seq_offsets(ctx)
    for triple in [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 0), (LAYOUT_TP, 2, 1), (LAYOUT_DP, 2, 0)]:
        view = View(geom, *triple)
        info = view.query()
        (table,), _ = fresh_tables(ctx, [view], 128)
        pool = wl.poisoned_pool(128, info["block_bytes"] // 2)
        oracle.scatter(view, pool, table, ctx, off, K, V)
        Kg = np.full_like(K, 0xAAAA)
        Vg = np.full_like(V, 0xAAAA)
        oracle.gather(view, pool, table, ctx, off, Kg, Vg)
        h0, hl = info["kv_head0"], info["n_kv_local"]
        assert np.array_equal(Kg[:, h0:h0 + hl], K[:, h0:h0 + hl])
        assert np.array_equal(Vg[:, h0:h0 + hl], V[:, h0:h0 + hl])
        other = np.ones(TINY.n_kv_heads, dtype=bool)
        other[h0:h0 + hl] = False
        assert (Kg[:, other] == 0xAAAA).all() and (Vg[:, other] == 0xAAAA).all()
        # bytes written = tokens * local heads * d * 2 planes; the rest is still poison
        written = int((pool != wl.BF16_NAN).sum())
        assert written <= int(ctx.sum()) * hl * TINY.head_dim * 2
        assert written >= int(0.99 * ctx.sum() * hl * TINY.head_dim * 2)


def test_tiny_dp_to_tp2_to_dp_restores_every_valid_byte():
    """The Tiny flow: DP blocks -> TP2 rank 0 and rank 1 blocks -> fresh DP blocks.  The TP
    blocks equal a direct scatter under the TP views; the returned DP blocks equal the
    original DP blocks on every valid byte; nothing else in the pool changed."""
    geom = geometry(TINY)
    dp = View(geom, LAYOUT_DP, 1, 0)
    tp0, tp1 = View(geom, LAYOUT_TP, 2, 0), View(geom, LAYOUT_TP, 2, 1)
    ctx = wl.draw_ctx_lens(TINY)
    K, V = wl.logical_kv(TINY, ctx)
    off = wl.seq_offsets(ctx)
    (t_dp, t_tp0, t_tp1, t_back), used = fresh_tables(ctx, [dp, tp0, tp1, dp], 128)
    assert used == 35 + 18 + 18 + 35
    block_elems = dp.query()["block_bytes"] // 2
    pool = wl.poisoned_pool(128, block_elems)
    oracle.scatter(dp, pool, t_dp, ctx, off, K, V)
    before = pool.copy()

    oracle.repack(dp, tp0, pool, t_dp, t_tp0, ctx)
    oracle.repack(dp, tp1, pool, t_dp, t_tp1, ctx)
    expect = before.copy()
    oracle.scatter(tp0, expect, t_tp0, ctx, off, K, V)
    oracle.scatter(tp1, expect, t_tp1, ctx, off, K, V)
    assert np.array_equal(pool, expect)

    # attention through the TP views of the repacked blocks == textbook on the logical data
    q_full = wl.queries(TINY)
    want = textbook_attention(q_full, K, V, off, 8, 2, 0.125)
    for r, (view, table) in enumerate([(tp0, t_tp0), (tp1, t_tp1)]):
        got = oracle.paged_decode(view, q_slice(q_full, view.query(), r), pool, table, ctx)
        np.testing.assert_allclose(got, want[:, 4 * r:4 * r + 4], rtol=0, atol=1e-12)

    mid = pool.copy()
    oracle.repack(tp0, dp, pool, t_tp0, t_back, ctx)
    # after rank 0 only: head 0 rows valid, head 1 rows of the fresh DP blocks still poison
    Kg, Vg = np.zeros_like(K), np.zeros_like(V)
    oracle.gather(View(geom, LAYOUT_DP, 2, 0), pool, t_back, ctx, off, Kg, Vg)
    assert np.array_equal(Kg[:, 0], K[:, 0]) and np.array_equal(Vg[:, 0], V[:, 0])
    Kp, Vp = np.zeros_like(K), np.zeros_like(V)
    oracle.gather(View(geom, LAYOUT_DP, 2, 1), pool, t_back, ctx, off, Kp, Vp)
    assert (Kp[:, 1] == wl.BF16_NAN).all() and (Vp[:, 1] == wl.BF16_NAN).all()
    oracle.repack(tp1, dp, pool, t_tp1, t_back, ctx)
    expect2 = mid.copy()
    oracle.scatter(dp, expect2, t_back, ctx, off, K, V)
    assert np.array_equal(pool, expect2)
    # the round trip reproduces the original DP blocks byte for byte (tail slots are poison
    # in both, since neither the scatter nor the repack touches them)
    for s in range(len(ctx)):
        nb = int(wl.blocks_needed(ctx[s:s + 1], 16)[0])
        assert np.array_equal(pool[t_back[s, :nb]], before[t_dp[s, :nb]])


@pytest.mark.parametrize("src,dst", [
    ((LAYOUT_DP, 1, 0), (LAYOUT_TP, 4, 2)),
    ((LAYOUT_TP, 4, 2), (LAYOUT_DP, 1, 0)),
    ((LAYOUT_TP, 2, 1), (LAYOUT_TP, 4, 3)),    # TP2 r1 holds heads 4..7, TP4 r3 heads 6..7
    ((LAYOUT_TP, 4, 0), (LAYOUT_TP, 2, 0)),
    ((LAYOUT_TP, 2, 0), (LAYOUT_TP, 4, 3)),    # no common head: nothing moves
    ((LAYOUT_DP, 4, 1), (LAYOUT_TP, 4, 1)),    # in-place slice view -> compact TP blocks
])
def test_repack_equals_gather_then_scatter_on_common_heads(src, dst):
    w = wl.Workload("r8", 6, 32, 8, 16, 4, 5, "x", ())
    geom = geometry(w)
    sv, dv = View(geom, *src), View(geom, *dst)
    ctx = np.array([1, 4, 5, 37, 64], dtype=np.int32)
    K, V = wl.logical_kv(w, ctx)
    off = wl.seq_offsets(ctx)
    (t_src, t_dst), used = fresh_tables(ctx, [sv, dv], 96, index=6)
    block_elems = sv.query()["block_bytes"] // 2
    pool = wl.poisoned_pool(96, block_elems)
    oracle.scatter(sv, pool, t_src, ctx, off, K, V)
    before = pool.copy()
    oracle.repack(sv, dv, pool, t_src, t_dst, ctx)

    si, di = sv.query(), dv.query()
    lo = max(si["kv_head0"], di["kv_head0"])
    hi = min(si["kv_head0"] + si["n_kv_local"], di["kv_head0"] + di["n_kv_local"])
    # expected: gather under src, keep only the common heads, scatter under dst into `before`
    Kg, Vg = np.full_like(K, wl.BF16_NAN), np.full_like(V, wl.BF16_NAN)
    oracle.gather(sv, before, t_src, ctx, off, Kg, Vg)
    expect = before.copy()
    if hi > lo:
        # scatter under dst writes all of dst's heads; restrict to common ones by writing the
        # others with what is already there (read them back first)
        Kd, Vd = np.zeros_like(K), np.zeros_like(V)
        oracle.gather(dv, before, t_dst, ctx, off, Kd, Vd)
        Kd[:, lo:hi], Vd[:, lo:hi] = Kg[:, lo:hi], Vg[:, lo:hi]
        oracle.scatter(dv, expect, t_dst, ctx, off, Kd, Vd)
        assert not np.array_equal(expect, before)
    assert np.array_equal(pool, expect)
    # source blocks untouched
    src_ids = t_src[t_src >= 0]
    assert np.array_equal(pool[src_ids], before[src_ids])
    # gather under dst returns the logical rows of the common heads
    K2, V2 = np.zeros_like(K), np.zeros_like(V)
    oracle.gather(dv, pool, t_dst, ctx, off, K2, V2)
    assert np.array_equal(K2[:, lo:hi], K[:, lo:hi]) and np.array_equal(V2[:, lo:hi], V[:, lo:hi])


def test_tp_to_dp_to_tp_round_trip():
    w = wl.Workload("r8", 6, 32, 8, 16, 4, 3, "x", ())
    geom = geometry(w)
    tp, dp = View(geom, LAYOUT_TP, 4, 1), View(geom, LAYOUT_DP, 1, 0)
    ctx = np.array([3, 16, 41], dtype=np.int32)
    K, V = wl.logical_kv(w, ctx)
    off = wl.seq_offsets(ctx)
    (t_a, t_dp, t_b), _ = fresh_tables(ctx, [tp, dp, tp], 64, index=6)
    pool = wl.poisoned_pool(64, tp.query()["block_bytes"] // 2)
    oracle.scatter(tp, pool, t_a, ctx, off, K, V)
    oracle.repack(tp, dp, pool, t_a, t_dp, ctx)
    oracle.repack(dp, tp, pool, t_dp, t_b, ctx)
    for s in range(3):
        nb = int(wl.blocks_needed(ctx[s:s + 1], 16)[0])
        assert np.array_equal(pool[t_b[s, :nb]], pool[t_a[s, :nb]])


def test_layouts_coexist_in_one_pool():
    """Blocks written under DP and blocks written under TP live side by side in one pool and
    both read back correctly (paper Sec. 5.2.3, Hard Preempt keeps paused DP state valid)."""
    geom = geometry(TINY)
    dp, tp = View(geom, LAYOUT_DP, 1, 0), View(geom, LAYOUT_TP, 2, 1)
    ctx_a = np.array([30, 70], dtype=np.int32)
    ctx_b = np.array([65, 5, 130], dtype=np.int32)
    wa = wl.Workload("a", 11, 8, 2, 64, 16, 2, "x", ())
    wb = wl.Workload("b", 12, 8, 2, 64, 16, 3, "x", ())
    Ka, Va = wl.logical_kv(wa, ctx_a)
    Kb, Vb = wl.logical_kv(wb, ctx_b)
    qa, qb = wl.queries(wa), wl.queries(wb)
    perm = torch.randperm(40, generator=wl.generator(11, wl.SUB_PERM)).numpy().astype(np.int32)
    t_a, used = wl.assign_blocks(ctx_a, 16, perm)
    t_b, _ = wl.assign_blocks(ctx_b, 32, perm[used:])
    pool = wl.poisoned_pool(40, dp.query()["block_bytes"] // 2)
    oracle.scatter(dp, pool, t_a, ctx_a, wl.seq_offsets(ctx_a), Ka, Va)
    oracle.scatter(tp, pool, t_b, ctx_b, wl.seq_offsets(ctx_b), Kb, Vb)
    got_a = oracle.paged_decode(dp, qa, pool, t_a, ctx_a)
    got_b = oracle.paged_decode(tp, q_slice(qb, tp.query(), 1), pool, t_b, ctx_b)
    np.testing.assert_allclose(got_a, textbook_attention(qa, Ka, Va, wl.seq_offsets(ctx_a), 8, 2, 0.125),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(got_b, textbook_attention(qb, Kb, Vb, wl.seq_offsets(ctx_b), 8, 2, 0.125)[:, 4:],
                               rtol=0, atol=1e-12)


def test_repack_rejects_mismatched_views():
    geom = geometry(TINY)
    pool = wl.poisoned_pool(4, 4096)
    t = np.zeros((1, 1), dtype=np.int32)
    n = np.array([1], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.repack(View(geom, LAYOUT_TP, 4, 0), View(geom, LAYOUT_DP, 1, 0), pool, t, t, n)
