"""Pins for the oracle's view arithmetic and address function (CPU only).

Expected values come from the paper's printed example (Fig. 4 caption), from Eq. 2-4 evaluated
by hand in this file, from numpy's own stride arithmetic, and from brute-force enumeration.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP, Geometry, View


def read_fig4(golden_dir):
    base, rows = None, []
    with open(os.path.join(golden_dir, "fig4_block_capacity.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            a, b = line.split()
            if a == "base_block_size":
                base = int(b)
            else:
                rows.append((int(a), int(b)))
    return base, rows


def test_fig4_capacities_and_constant_block_bytes(golden_dir):
    """Fig. 4 caption: B_base = 4 gives 4 / 8 / 16 tokens per block for DP / 2TP / 4TP; the
    physical bytes of a block do not change (Eq. 2 held constant, Eq. 3)."""
    base, rows = read_fig4(golden_dir)
    assert base == 4 and rows == [(1, 4), (2, 8), (4, 16)]
    geom = Geometry(8, 4, 32, base)
    bytes_seen = set()
    for p, tokens in rows:
        v = View(geom, LAYOUT_DP if p == 1 else LAYOUT_TP, p, 0).query()
        assert v["block_tokens"] == tokens
        bytes_seen.add(v["block_bytes"])
    assert len(bytes_seen) == 1


@pytest.mark.parametrize("hq,hkv,d,b0", [(32, 8, 128, 16), (64, 8, 128, 16), (8, 2, 64, 16)])
def test_eq3_eq4_closed_forms(hq, hkv, d, b0):
    """B(p) = p * B_base (Eq. 3); H_req = H_base / N_eng (Eq. 4); rank r owns the r-th
    contiguous slice of heads (Sec. 4.1.1); block bytes = 2 planes * B0 * Hkv * d * 2 B."""
    geom = Geometry(hq, hkv, d, b0)
    for p in (1, 2, 4, 8):
        if hkv % p:
            continue
        for r in range(p):
            v = View(geom, LAYOUT_TP, p, r).query()
            assert v["block_tokens"] == p * b0
            assert v["n_kv_local"] == hkv // p and v["row_heads"] == hkv // p
            assert v["n_q_local"] == hq // p
            assert v["kv_head0"] == r * (hkv // p) and v["row_head0"] == 0
            assert v["block_bytes"] == 2 * b0 * hkv * d * 2
            assert v["token_stride_elems"] == (hkv // p) * d
            assert v["group"] == hq // hkv
            # Eq. 2: tokens * local width * element size is the same number for every p
            assert v["block_tokens"] * v["n_kv_local"] * d * 2 == b0 * hkv * d * 2
    dp = View(geom, LAYOUT_DP, 1, 0).query()
    assert dp["block_tokens"] == b0 and dp["n_kv_local"] == hkv and dp["kv_head0"] == 0
    if (hq, hkv, d, b0) != (8, 2, 64, 16):
        assert dp["block_bytes"] == 65536
    else:
        assert dp["block_bytes"] == 8192


def test_alias_view_keeps_dp_rows():
    """DP-arranged blocks read as rank r's head slice: capacity and row width stay DP's."""
    geom = Geometry(32, 8, 128, 16)
    v = View(geom, LAYOUT_DP, 4, 3).query()
    assert v["block_tokens"] == 16 and v["row_heads"] == 8
    assert v["n_kv_local"] == 2 and v["kv_head0"] == 6 and v["row_head0"] == 6
    assert v["n_q_local"] == 8


@pytest.mark.parametrize("args", [
    (32, 8, 128, 16, LAYOUT_TP, 16, 0),   # p does not divide Hkv
    (32, 8, 128, 16, LAYOUT_TP, 3, 0),
    (32, 8, 128, 16, LAYOUT_TP, 2, 2),    # rank out of range
    (32, 8, 128, 16, LAYOUT_TP, 2, -1),
    (32, 8, 128, 16, LAYOUT_TP, 0, 0),
    (30, 8, 128, 16, LAYOUT_DP, 1, 0),    # Hkv does not divide Hq
    (32, 8, 128, 16, 7, 1, 0),            # unknown layout
    (32, 8, 0, 16, LAYOUT_DP, 1, 0),
])
def test_invalid_views_rejected(args):
    with pytest.raises(ValueError):
        View(Geometry(*args[:4]), *args[4:]).query()


@pytest.mark.parametrize("layout,p", [(LAYOUT_DP, 1), (LAYOUT_TP, 1), (LAYOUT_TP, 2)])
def test_address_map_is_a_bijection_onto_the_pool(layout, p):
    """Brute force on the Tiny geometry: over all (blk, plane, slot, hl, e) the element index
    covers [0, pool_elems) exactly once, and it equals numpy's own index arithmetic for the
    array [n_blocks][2][Bv][Hrow][d]."""
    geom = Geometry(8, 2, 64, 16)
    n_blocks = 3
    for r in range(p):
        view = View(geom, layout, p, r)
        v = view.query()
        shape = (n_blocks, 2, v["block_tokens"], v["row_heads"], geom.head_dim)
        total = int(np.prod(shape))
        assert total == n_blocks * v["block_bytes"] // 2
        seen = np.zeros(total, dtype=np.int32)
        for blk, plane, slot, hl in itertools.product(range(n_blocks), range(2),
                                                      range(v["block_tokens"]),
                                                      range(v["n_kv_local"])):
            for e in (0, 1, geom.head_dim // 2, geom.head_dim - 1):
                idx = oracle.elem_index(view, blk, plane, slot, hl, e)
                assert idx == np.ravel_multi_index(
                    (blk, plane, slot, v["row_head0"] + hl, e), shape)
            base = oracle.elem_index(view, blk, plane, slot, hl, 0)
            seen[base:base + geom.head_dim] += 1
        assert seen.min() == 1 and seen.max() == 1


def test_alias_views_tile_a_dp_block():
    """The p alias views of DP-arranged blocks are disjoint and together cover the block."""
    geom = Geometry(8, 2, 64, 16)
    n_blocks, p = 2, 2
    total = n_blocks * 2 * 16 * 2 * 64
    seen = np.zeros(total, dtype=np.int32)
    for r in range(p):
        view = View(geom, LAYOUT_DP, p, r)
        v = view.query()
        for blk, plane, slot, hl in itertools.product(range(n_blocks), range(2), range(16),
                                                      range(v["n_kv_local"])):
            base = oracle.elem_index(view, blk, plane, slot, hl, 0)
            seen[base:base + 64] += 1
    assert seen.min() == 1 and seen.max() == 1


def test_views_of_one_block_span_the_same_bytes():
    """Block ids and the pool stay put across modes (Sec. 4.2.2): block b read under DP and
    under every TP view occupies exactly elements [b * block_elems, (b+1) * block_elems)."""
    geom = Geometry(32, 8, 128, 16)
    b = 5
    for layout, p in [(LAYOUT_DP, 1), (LAYOUT_TP, 2), (LAYOUT_TP, 4), (LAYOUT_TP, 8)]:
        view = View(geom, layout, p, 0)
        v = view.query()
        block_elems = v["block_bytes"] // 2
        first = oracle.elem_index(view, b, 0, 0, 0, 0)
        last = oracle.elem_index(view, b, 1, v["block_tokens"] - 1, v["n_kv_local"] - 1,
                                 geom.head_dim - 1)
        assert first == b * block_elems and last == (b + 1) * block_elems - 1
        # V plane starts half a block in, whatever the view
        assert oracle.elem_index(view, b, 1, 0, 0, 0) == b * block_elems + block_elems // 2


def test_elem_index_rejects_out_of_range():
    view = View(Geometry(8, 2, 64, 16), LAYOUT_TP, 2, 1)
    assert oracle.elem_index(view, 0, 0, 32, 0, 0) == -1     # slot beyond B(2) = 32
    assert oracle.elem_index(view, 0, 0, 0, 1, 0) == -1      # only one local head
    assert oracle.elem_index(view, 0, 2, 0, 0, 0) == -1
    assert oracle.elem_index(view, 0, 0, 0, 0, 64) == -1
