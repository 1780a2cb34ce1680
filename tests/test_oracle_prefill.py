"""Pins for the oracle's multi-token causal paged attention (CPU only).

Expected values come from numpy's textbook masked-softmax attention on the logical tensors, from
the already pinned single-query oracle, from a closed form (the first token of a sequence can only
see itself) and from causality itself (later tokens cannot influence earlier rows).
"""
import numpy as np
import pytest

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, make_prefill_case, textbook_causal_attention

TINY = wl.WORKLOADS["tiny"]
VIEWS = [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 0), (LAYOUT_TP, 2, 1), (LAYOUT_DP, 2, 1)]
CTX = np.array([17, 64, 150, 300, 5, 33], dtype=np.int32)
QLEN = np.array([17, 1, 40, 300, 0, 32], dtype=np.int32)   # full prefill, decode, chunks, none


def rank_rows(full, info, rank):
    hql = info["n_q_local"]
    return full[:, rank * hql:(rank + 1) * hql, :]


@pytest.mark.parametrize("view", VIEWS)
def test_prefill_equals_textbook_causal_attention(view):
    c = make_prefill_case(TINY, view, CTX, QLEN)
    want = textbook_causal_attention(c, 1.0 / np.sqrt(TINY.head_dim))
    got = oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, rank_rows(want, c.info, c.view.rank), rtol=0, atol=1e-12)


def test_one_query_token_is_decode():
    """q_len = 1 everywhere: the decode oracle on the same pool."""
    ctx = np.array([17, 64, 150, 1], dtype=np.int32)
    c = make_prefill_case(TINY, (LAYOUT_TP, 2, 1), ctx, np.ones(4, dtype=np.int32))
    got = oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    np.testing.assert_array_equal(got, want)


def test_first_token_sees_only_itself():
    ctx = np.array([40, 9], dtype=np.int32)
    c = make_prefill_case(TINY, (LAYOUT_DP, 1, 0), ctx, ctx)
    got = oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off)
    G = TINY.n_q_heads // TINY.n_kv_heads
    for s in range(2):
        row = int(c.q_off[s])
        for i in range(c.info["n_q_local"]):
            np.testing.assert_array_equal(got[row, i], bf16_bits_to_f64(c.V[c.seq_off[s], i // G]))


def test_later_tokens_cannot_change_earlier_rows():
    """Overwrite the K and V of the last 10 tokens of each sequence: every row whose position lies
    before them is bit-identical, the rows at or after them change."""
    ctx = np.array([64, 150], dtype=np.int32)
    c = make_prefill_case(TINY, (LAYOUT_TP, 2, 0), ctx, np.array([30, 150], dtype=np.int32))
    before = oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off)
    K2, V2 = c.K.copy(), c.V.copy()
    for s in range(2):
        a = int(c.seq_off[s + 1])
        K2[a - 10:a] = K2[a - 10:a][::-1] ^ 0x8000
        V2[a - 10:a] = V2[a - 10:a][::-1] ^ 0x8000
    pool2 = c.pool.copy()
    oracle.scatter(c.view, pool2, c.table, c.ctx, c.seq_off, K2, V2)
    after = oracle.paged_prefill(c.view, c.q, pool2, c.table, c.ctx, c.q_off)
    for s in range(2):
        qa, m = int(c.q_off[s]), int(c.q_lens[s])
        np.testing.assert_array_equal(before[qa:qa + m - 10], after[qa:qa + m - 10])
        assert not np.array_equal(before[qa + m - 10:qa + m], after[qa + m - 10:qa + m])


def test_rows_entry_point_matches_full():
    c = make_prefill_case(TINY, (LAYOUT_DP, 2, 1), CTX, QLEN)
    full = oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off)
    rq = np.array([0, 16, 17, 57, 300, int(c.q_off[-1]) - 1], dtype=np.int64)
    rh = np.array([0, 3, 1, 2, 0, 3], dtype=np.int32)
    got = oracle.paged_prefill_rows(c.view, c.q, c.pool, c.table, c.ctx, c.q_off, rq, rh)
    for k in range(len(rq)):
        np.testing.assert_array_equal(got[k], full[rq[k], rh[k]])
    with pytest.raises(ValueError):
        oracle.paged_prefill_rows(c.view, c.q, c.pool, c.table, c.ctx, c.q_off,
                                  np.array([int(c.q_off[-1])], dtype=np.int64), np.array([0], dtype=np.int32))
