"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side logic (view resolution, argument validation, error strings) behaves as the
header says.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

import oracle
from paper_2602_22593_amd import binding as kv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built_library():
    if not os.path.exists(kv.LIB_PATH):
        from paper_2602_22593_amd.build import build
        build()
    return kv.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flying_kv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:int|void|size_t|int64_t|const char\*)\s+\*?\s*(\w+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert {"kv_view_create", "paged_decode_attn", "kv_repack", "kv_append", "kv_view_query",
            "paged_decode_attn_workspace_bytes", "kv_validate_tables", "kv_strerror"} <= set(names)
    L = kv.lib()
    for n in names:
        assert hasattr(L, n), n


@pytest.mark.parametrize("geom", [(32, 8, 128, 16), (64, 8, 128, 16), (8, 2, 64, 16), (8, 4, 32, 4)])
def test_view_resolution_matches_paper_formulas_and_oracle(geom):
    """B(p) = p * B_base, H_req = H_base / p, constant block bytes (Eq. 2-4); the oracle, written
    separately from the same formulas, must agree on every integer."""
    hq, hkv, d, b0 = geom
    og = oracle.Geometry(*geom)
    for layout in (kv.KV_LAYOUT_DP, kv.KV_LAYOUT_TP):
        for p in (1, 2, 4, 8):
            if hkv % p:
                continue
            for r in range(p):
                v = kv.kv_view_create(hq, hkv, d, b0, layout, p, r)
                o = oracle.View(og, layout, p, r).query()
                assert v.block_tokens == o["block_tokens"] == (p * b0 if layout == kv.KV_LAYOUT_TP else b0)
                assert v.n_kv_local == o["n_kv_local"] == hkv // p
                assert v.n_q_local == o["n_q_local"] == hq // p
                assert v.kv_head0 == o["kv_head0"] == r * (hkv // p)
                assert v.block_bytes == o["block_bytes"] == 2 * b0 * hkv * d * 2
                assert v.token_stride_elems == o["token_stride_elems"]
                assert v.row_heads == o["row_heads"] and v.row_head0 == o["row_head0"]


def test_fig4_example_through_the_abi():
    """Fig. 4: B_base = 4 -> 4 / 8 / 16 tokens per block for DP / 2TP / 4TP, same block bytes."""
    caps = [kv.kv_view_create(8, 4, 32, 4, kv.KV_LAYOUT_TP if p > 1 else kv.KV_LAYOUT_DP, p, 0)
            for p in (1, 2, 4)]
    assert [v.block_tokens for v in caps] == [4, 8, 16]
    assert len({v.block_bytes for v in caps}) == 1


@pytest.mark.parametrize("args,status", [
    ((32, 8, 128, 16, kv.KV_LAYOUT_TP, 16, 0), kv.KV_ERR_INVALID_ARG),   # p does not divide Hkv
    ((32, 8, 128, 16, kv.KV_LAYOUT_TP, 2, 2), kv.KV_ERR_INVALID_ARG),    # rank >= p
    ((32, 8, 128, 16, kv.KV_LAYOUT_TP, 2, -1), kv.KV_ERR_INVALID_ARG),
    ((32, 8, 128, 16, kv.KV_LAYOUT_TP, 0, 0), kv.KV_ERR_INVALID_ARG),
    ((30, 8, 128, 16, kv.KV_LAYOUT_DP, 1, 0), kv.KV_ERR_INVALID_ARG),    # Hkv does not divide Hq
    ((32, 8, 100, 16, kv.KV_LAYOUT_DP, 1, 0), kv.KV_ERR_INVALID_ARG),    # rows not 16-byte multiples
    ((32, 8, 128, 0, kv.KV_LAYOUT_DP, 1, 0), kv.KV_ERR_INVALID_ARG),
    ((32, 8, 128, 16, 5, 1, 0), kv.KV_ERR_INVALID_ARG),                  # unknown layout
])
def test_view_create_rejects(args, status):
    with pytest.raises(kv.KVError) as e:
        kv.kv_view_create(*args)
    assert e.value.status == status


def test_unsupported_dtype():
    with pytest.raises(kv.KVError) as e:
        kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_DP, 1, 0, dtype=1)
    assert e.value.status == kv.KV_ERR_UNSUPPORTED


def test_null_and_size_checks_without_a_gpu():
    """Argument validation happens on the host before anything touches the device."""
    L = kv.lib()
    v = kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_TP, 4, 0)
    g = kv.kv_geometry(32, 8, 128, 16, 0)
    out = C.c_void_p()
    assert L.kv_view_create(None, 0, 1, 0, C.byref(out)) == kv.KV_ERR_INVALID_ARG
    assert L.kv_view_create(C.byref(g), 0, 1, 0, None) == kv.KV_ERR_INVALID_ARG
    assert L.kv_view_query(None, None, None, None, None, None) == kv.KV_ERR_INVALID_ARG
    # null view / null buffers / negative sizes
    assert L.paged_decode_attn(None, None, None, 0, None, 0, None, 4, 16, None, 0.0, None, 0, None) \
        == kv.KV_ERR_INVALID_ARG
    assert L.paged_decode_attn(None, None, None, 0, None, 0, None, 4, 16, v.handle, 0.0, None, 0, None) \
        == kv.KV_ERR_INVALID_ARG
    assert L.paged_decode_attn(None, None, None, 0, None, 0, None, -1, 16, v.handle, 0.0, None, 0, None) \
        == kv.KV_ERR_INVALID_ARG
    # batch 0 is a no-op
    assert L.paged_decode_attn(None, None, None, 0, None, 0, None, 0, 16, v.handle, 0.0, None, 0, None) \
        == kv.KV_OK
    # block table too narrow for max_ctx_len: 131072 tokens need 2048 columns at 64 tokens/block
    fake = C.c_void_p(256)
    assert L.paged_decode_attn(fake, fake, fake, 10, fake, 2047, fake, 1, 131072, v.handle, 0.0, fake,
                               1 << 30, None) == kv.KV_ERR_INVALID_ARG
    # workspace too small / misaligned
    need = L.paged_decode_attn_workspace_bytes(v.handle, 1, 131072)
    assert need > 256
    assert L.paged_decode_attn(fake, fake, fake, 10, fake, 2048, fake, 1, 131072, v.handle, 0.0, fake,
                               need - 1, None) == kv.KV_ERR_WORKSPACE
    assert L.paged_decode_attn(fake, fake, fake, 10, fake, 2048, fake, 1, 131072, v.handle, 0.0,
                               C.c_void_p(264), need, None) == kv.KV_ERR_INVALID_ARG
    # repack: views over different geometries, null tables, narrow tables
    other = kv.kv_view_create(64, 8, 128, 16, kv.KV_LAYOUT_DP, 1, 0)
    dp = kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_DP, 1, 0)
    assert L.kv_repack(fake, 10, other.handle, v.handle, fake, 8, fake, 8, fake, 1, 16, None) \
        == kv.KV_ERR_INVALID_ARG
    assert L.kv_repack(fake, 10, dp.handle, v.handle, None, 8, fake, 8, fake, 1, 16, None) \
        == kv.KV_ERR_INVALID_ARG
    assert L.kv_repack(fake, 10, dp.handle, v.handle, fake, 1, fake, 8, fake, 1, 64, None) \
        == kv.KV_ERR_INVALID_ARG
    assert L.kv_repack(fake, 10, dp.handle, v.handle, fake, 8, fake, 8, fake, 0, 64, None) == kv.KV_OK
    # disjoint head sets: nothing to do, returns before any launch
    v3 = kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_TP, 4, 3)
    assert L.kv_repack(fake, 10, v3.handle, v.handle, fake, 8, fake, 8, fake, 1, 64, None) == kv.KV_OK
    assert L.kv_append(None, 10, v.handle, fake, fake, fake, 8, fake, 1, None) == kv.KV_ERR_INVALID_ARG


def test_mixed_entry_point_checks_without_a_gpu():
    """paged_decode_attn_mixed validates its view list on the host."""
    L = kv.lib()
    fake = C.c_void_p(256)
    tp = kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_TP, 4, 1)
    alias = kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_DP, 4, 1)
    other_rank = kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_DP, 4, 2)
    other_p = kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_TP, 2, 1)
    other_geom = kv.kv_view_create(64, 8, 128, 16, kv.KV_LAYOUT_TP, 4, 1)

    def call(views, n=None, stride=2048, ws=1 << 30, ids=fake, batch=2, max_ctx=16384):
        arr = (C.c_void_p * len(views))(*[v.handle if v is not None else None for v in views])
        return L.paged_decode_attn_mixed(fake, fake, fake, 10, fake, stride, fake, ids, batch, max_ctx,
                                         C.cast(arr, C.c_void_p), len(views) if n is None else n, 0.0,
                                         fake, ws, None)

    assert L.paged_decode_attn_mixed(fake, fake, fake, 10, fake, 8, fake, fake, 2, 16, None, 1, 0.0, fake,
                                     1 << 20, None) == kv.KV_ERR_INVALID_ARG
    assert call([tp, alias], n=0) == kv.KV_ERR_INVALID_ARG
    assert call([tp, alias, tp, alias, tp]) == kv.KV_ERR_INVALID_ARG        # more than 4 views
    assert call([tp, None]) == kv.KV_ERR_INVALID_ARG
    assert call([tp, other_rank]) == kv.KV_ERR_INVALID_ARG
    assert call([tp, other_p]) == kv.KV_ERR_INVALID_ARG
    assert call([tp, other_geom]) == kv.KV_ERR_INVALID_ARG
    assert call([tp, alias], ids=None) == kv.KV_ERR_INVALID_ARG
    # 16384 tokens need 1024 columns under the 16-token alias layout (256 would do for TP alone)
    assert call([tp, alias], stride=1023) == kv.KV_ERR_INVALID_ARG
    assert call([tp, alias], ws=1024) == kv.KV_ERR_WORKSPACE
    assert call([tp, alias], batch=0) == kv.KV_OK
    # head_dim 64 is served by the plain call only
    a64 = kv.kv_view_create(8, 2, 64, 16, kv.KV_LAYOUT_TP, 2, 0)
    b64 = kv.kv_view_create(8, 2, 64, 16, kv.KV_LAYOUT_DP, 2, 0)
    assert call([a64, b64]) == kv.KV_ERR_UNSUPPORTED


def test_weight_view_and_linear_view_checks_without_a_gpu():
    L = kv.lib()
    fake = C.c_void_p(256)
    v = kv.kv_weight_view_make(0, 1, 2, 256, 512)
    assert (v.row_start[0], v.row_count[0], v.col_start, v.col_count) == (128, 128, 0, 512)
    out = kv.kv_weight_view()
    assert L.kv_weight_view_make(0, 2, 2, 256, 512, C.byref(out)) == kv.KV_ERR_INVALID_ARG
    assert L.kv_weight_view_make(1, 0, 3, 256, 512, C.byref(out)) == kv.KV_ERR_INVALID_ARG
    assert L.kv_weight_view_make(2, 0, 1, 256, 512, C.byref(out)) == kv.KV_ERR_INVALID_ARG
    assert L.kv_linear_view(fake, 512, fake, 256, 512, None, fake, 128, 4, fake, 1 << 30, None) == kv.KV_ERR_INVALID_ARG
    assert L.kv_linear_view(fake, 512, fake, 200, 512, C.byref(v), fake, 128, 4, fake, 1 << 30, None) == kv.KV_ERR_INVALID_ARG  # view outside the weight
    assert L.kv_linear_view(fake, 256, fake, 256, 512, C.byref(v), fake, 128, 4, fake, 1 << 30, None) == kv.KV_ERR_INVALID_ARG  # ldx < cols
    assert L.kv_linear_view(fake, 512, fake, 256, 512, C.byref(v), fake, 64, 4, fake, 1 << 30, None) == kv.KV_ERR_INVALID_ARG   # ldy < rows
    assert L.kv_linear_view(None, 512, fake, 256, 512, C.byref(v), fake, 128, 4, fake, 1 << 30, None) == kv.KV_ERR_INVALID_ARG
    assert L.kv_linear_view(None, 512, None, 256, 512, C.byref(v), None, 128, 0, None, 0, None) == kv.KV_OK
    odd = kv.kv_weight_view_make(1, 0, 8, 256, 512)      # 64 columns: not a whole 128-wide slab
    assert L.kv_linear_view(fake, 64, fake, 256, 512, C.byref(odd), fake, 256, 4, fake, 1 << 30, None) == kv.KV_ERR_UNSUPPORTED
    big = kv.kv_weight_view_make(0, 0, 1, 256, 4096)     # few tiles, many slabs: the input dimension is split
    need = L.kv_linear_view_workspace_bytes(C.byref(big), 8)
    assert need > 0 and need % (8 * 256 * 4) == 0
    assert L.kv_linear_view(fake, 4096, fake, 256, 4096, C.byref(big), fake, 256, 8, fake, need - 1, None) == kv.KV_ERR_WORKSPACE
    assert L.kv_linear_view(fake, 4096, fake, 256, 4096, C.byref(big), fake, 256, 8, None, need, None) == kv.KV_ERR_INVALID_ARG
    thin = kv.kv_weight_view_make(0, 0, 8, 256, 512)     # 32 rows: not a whole 64-row tile
    assert L.kv_linear_view(fake, 512, fake, 256, 512, C.byref(thin), fake, 32, 4, fake, 1 << 30, None) == kv.KV_ERR_UNSUPPORTED


def test_prefill_entry_point_checks_without_a_gpu():
    L = kv.lib()
    fake = C.c_void_p(256)
    v = kv.kv_view_create(8, 2, 64, 16, kv.KV_LAYOUT_DP, 1, 0)          # head_dim 64
    assert L.paged_prefill_attn(fake, fake, fake, 10, fake, 64, fake, fake, 1, 8, 64, 8, v.handle, 0.0, fake, 1 << 30, None) \
        == kv.KV_ERR_UNSUPPORTED
    v = kv.kv_view_create(8 * 24, 8, 128, 16, kv.KV_LAYOUT_DP, 1, 0)    # group of 24
    assert L.paged_prefill_attn(fake, fake, fake, 10, fake, 64, fake, fake, 1, 8, 64, 8, v.handle, 0.0, fake, 1 << 30, None) \
        == kv.KV_ERR_UNSUPPORTED
    v = kv.kv_view_create(32, 8, 128, 16, kv.KV_LAYOUT_DP, 1, 0)
    assert L.paged_prefill_attn(fake, fake, fake, 10, fake, 64, fake, fake, 1, 8, 64, 65, v.handle, 0.0, fake, 1 << 30, None) \
        == kv.KV_ERR_INVALID_ARG                                         # max_q_len > max_ctx_len
    assert L.paged_prefill_attn(fake, fake, fake, 10, fake, 3, fake, fake, 1, 8, 64, 8, v.handle, 0.0, fake, 1 << 30, None) \
        == kv.KV_ERR_INVALID_ARG                                         # table too narrow
    assert L.paged_prefill_attn(fake, fake, fake, 10, fake, 64, fake, None, 1, 8, 64, 8, v.handle, 0.0, fake, 1 << 30, None) \
        == kv.KV_ERR_INVALID_ARG
    assert L.paged_prefill_attn(None, None, None, 0, None, 0, None, None, 0, 0, 0, 0, v.handle, 0.0, None, 0, None) == kv.KV_OK


def test_unsupported_shapes_are_reported():
    L = kv.lib()
    fake = C.c_void_p(256)
    v = kv.kv_view_create(32, 8, 256, 16, kv.KV_LAYOUT_DP, 1, 0)       # head_dim 256: no kernel
    assert L.paged_decode_attn(fake, fake, fake, 10, fake, 8, fake, 1, 16, v.handle, 0.0, fake, 1 << 20,
                               None) == kv.KV_ERR_UNSUPPORTED
    v = kv.kv_view_create(8 * 24, 8, 128, 16, kv.KV_LAYOUT_DP, 1, 0)   # group of 24: above the MFMA tile, not a VALU size
    assert L.paged_decode_attn(fake, fake, fake, 10, fake, 8, fake, 1, 16, v.handle, 0.0, fake, 1 << 20,
                               None) == kv.KV_ERR_UNSUPPORTED


def test_strerror_and_options():
    assert kv.strerror(0) == "ok"
    for code in range(-6, 0):
        assert kv.strerror(code) not in ("ok", "unknown status")
    assert kv.strerror(-99) == "unknown status"
    kv.kv_set_option("chunk_tokens", 256)
    assert kv.kv_get_option("chunk_tokens") == 256
    with pytest.raises(kv.KVError):
        kv.kv_set_option("chunk_tokens", 100)       # not a multiple of 64
    with pytest.raises(kv.KVError):
        kv.kv_set_option("no_such_option", 1)
    kv.kv_set_option("chunk_tokens", 0)
    # the share moved between XCDs: -1 (library default) .. 256; the input splits of kv_linear_view: 0 .. 16
    assert kv.kv_get_option("xcd_skew") == -1
    kv.kv_set_option("xcd_skew", 256)
    assert kv.kv_get_option("xcd_skew") == 256
    for bad in (-2, 257):
        with pytest.raises(kv.KVError):
            kv.kv_set_option("xcd_skew", bad)
    kv.kv_set_option("xcd_skew", -1)
    assert kv.kv_get_option("piece_cost") == -1
    kv.kv_set_option("piece_cost", 64)
    with pytest.raises(kv.KVError):
        kv.kv_set_option("piece_cost", 65)
    kv.kv_set_option("piece_cost", -1)
    kv.kv_set_option("linear_splits", 16)
    with pytest.raises(kv.KVError):
        kv.kv_set_option("linear_splits", 17)
    kv.kv_set_option("linear_splits", 0)


def test_product_package_does_not_import_the_oracle():
    """The HIP package must not depend on the oracle (and the oracle not on the package)."""
    pkg = os.path.join(ROOT, "paper_2602_22593_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "flying_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2602_22593_amd" not in text and "flying_kv.h" not in text, f
