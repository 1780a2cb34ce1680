"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle on the same
seeded inputs.  Attention: max-abs <= 2e-2 and mean-abs <= 2e-3 (bf16 K/V/out, fp32
accumulation); repack, append and table indexing: bit-exact on the whole pool."""
import numpy as np
import pytest
import torch

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import workloads as wl

from helpers import make_mixed_case, bf16_bits_to_f64, geometry, make_case, q_slice

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3
TINY = wl.WORKLOADS["tiny"]
DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def require_gpu_and_library():
    assert torch.cuda.is_available(), "these tests need a GPU"
    kv.lib()  # raises if the HIP library is not built: there is no fallback
    yield
    for key in ("chunk_tokens", "force_kernel", "heads_per_wave", "merge_mode", "waves_per_cu"):
        kv.kv_set_option(key, 0)


def dev_u16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int16)).to(DEV)


def gpu_view(w, triple) -> kv.KVView:
    return kv.kv_view_create(w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size, *triple)


def run_gpu_decode(c, view, scale=0.0):
    out = kv.paged_decode_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                               torch.from_numpy(c.ctx).to(DEV), view,
                               max_ctx_len=int(c.ctx.max()) if len(c.ctx) else 0, scale=scale)
    torch.cuda.synchronize()
    return bf16_bits_to_f64(out.cpu().numpy().view(np.uint16))


def check_close(got, want, what=""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.3e}"


@pytest.mark.parametrize("chunk", [0, 64, 128])
@pytest.mark.parametrize("triple", [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 0), (LAYOUT_TP, 2, 1),
                                    (LAYOUT_DP, 2, 1)])
def test_tiny_config_all_views(triple, chunk):
    """Tiny: 8 q heads, 2 KV heads, d 64, B_base 16, ctx {17, 64, 150, 300}; pool NaN-poisoned
    outside the valid tokens.  chunk 64 / 128 force the split-KV + merge path."""
    kv.kv_set_option("chunk_tokens", chunk)
    c = make_case(TINY, triple, n_pool_blocks=128)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    got = run_gpu_decode(c, gpu_view(TINY, triple))
    check_close(got, want, f"tiny {triple} chunk {chunk}")


RAGGED = np.array([1, 15, 16, 17, 0, 511, 513, 1300, 2049, 64], dtype=np.int32)


@pytest.mark.parametrize("kernel", [0, 2, 3])   # 0 = automatic (even-split matrix-core kernel at d = 128), 2 = vector-ALU, 3 = chunked matrix-core
@pytest.mark.parametrize("chunk", [0, 256])
@pytest.mark.parametrize("hq,hkv,triple", [
    (32, 8, (LAYOUT_DP, 1, 0)), (32, 8, (LAYOUT_TP, 2, 1)), (32, 8, (LAYOUT_TP, 4, 3)),
    (32, 8, (LAYOUT_TP, 8, 5)), (32, 8, (LAYOUT_DP, 4, 2)), (64, 8, (LAYOUT_TP, 8, 7)),
    (64, 8, (LAYOUT_DP, 1, 0)), (16, 8, (LAYOUT_TP, 2, 0)), (8, 8, (LAYOUT_TP, 4, 1)),
])
def test_multi_tile_ragged_lengths(hq, hkv, triple, chunk, kernel):
    """Head dim 128 at the Llama shapes (G = 4, 8) and smaller groups (G = 2, 1): lengths that
    span several tiles, end mid-block, are empty, or are exactly one block."""
    kv.kv_set_option("chunk_tokens", chunk)
    kv.kv_set_option("force_kernel", kernel)
    w = wl.Workload("ragged", 20 + hq // 8, hq, hkv, 128, 16, len(RAGGED), "x", ())
    c = make_case(w, triple, RAGGED)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    got = run_gpu_decode(c, gpu_view(w, triple))
    kv.kv_set_option("force_kernel", 0)
    check_close(got, want, f"{hq}/{hkv} {triple} chunk {chunk} kernel {kernel}")
    assert (got[4] == 0).all()                       # ctx_len 0 -> zeros
    # ctx_len 1 -> the V row itself, exactly (bf16 in, bf16 out)
    G = hq // hkv
    for i in range(c.info["n_q_local"]):
        g = c.info["kv_head0"] + i // G
        assert np.array_equal(got[0, i], bf16_bits_to_f64(c.V[c.seq_off[0], g]))


def poisoned_workspace(nbytes: int, fill: int) -> torch.Tensor:
    """A workspace full of garbage except for what the ABI asks to be zero at first use: the arrival
    words in its first KV_DECODE_SYNC_BYTES."""
    ws = torch.full((nbytes,), fill, dtype=torch.uint8, device=DEV)
    ws[:kv.KV_DECODE_SYNC_BYTES] = 0
    return ws


def sync_words_are_zero(ws: torch.Tensor) -> bool:
    torch.cuda.synchronize()
    return not bool(ws[:kv.KV_DECODE_SYNC_BYTES].any())


@pytest.mark.parametrize("merge_mode", [0, 1, 2])
@pytest.mark.parametrize("one_head", [0, 1])
@pytest.mark.parametrize("wpc", [4, 12])
def test_even_split_kernel_variants(one_head, merge_mode, wpc):
    """The even-split matrix-core kernels in their modes (several adjacent KV heads per wavefront
    where the shape allows, or always one; cut sequences finished inside the main kernel or by the
    merge kernel) and launch widths; lengths chosen so that wavefront ranges cross sequence and head
    boundaries and single-piece pairs occur."""
    kv.kv_set_option("heads_per_wave", one_head)
    kv.kv_set_option("merge_mode", merge_mode)
    kv.kv_set_option("waves_per_cu", wpc)
    try:
        lens = np.array([1, 31, 32, 33, 0, 511, 513, 4100, 2049, 64, 7000, 96], dtype=np.int32)
        for hq, hkv, triple in [(32, 8, (LAYOUT_DP, 1, 0)), (32, 8, (LAYOUT_TP, 4, 1)),
                                (64, 8, (LAYOUT_TP, 8, 2)), (32, 8, (LAYOUT_DP, 2, 1))]:
            w = wl.Workload("variants", 60 + hq // 8, hq, hkv, 128, 16, len(lens), "x", ())
            c = make_case(w, triple, lens)
            want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
            got = run_gpu_decode(c, gpu_view(w, triple))
            check_close(got, want, f"one_head {one_head} merge {merge_mode} wpc {wpc} {hq}/{hkv} {triple}")
            assert (got[4] == 0).all()
    finally:
        kv.kv_set_option("heads_per_wave", 0)
        kv.kv_set_option("merge_mode", 0)
        kv.kv_set_option("waves_per_cu", 0)


@pytest.mark.parametrize("hq,hkv,triple", [
    (32, 8, (LAYOUT_DP, 1, 0)),    # G 4: four heads per wavefront, two head groups per sequence
    (32, 8, (LAYOUT_TP, 2, 1)),    # G 4: the rank's four heads are one group (contiguous 1 KiB rows)
    (32, 8, (LAYOUT_DP, 2, 1)),    # the same heads read in place from DP-layout blocks
    (64, 8, (LAYOUT_DP, 1, 0)),    # G 8: two heads per wavefront
    (64, 8, (LAYOUT_TP, 2, 0)),
    (24, 8, (LAYOUT_DP, 1, 0)),    # G 3: 12 of the 16 columns in use
    (16, 8, (LAYOUT_TP, 2, 1)),    # G 2
    (8, 8, (LAYOUT_DP, 1, 0)),     # G 1
])
def test_several_heads_per_wavefront_every_tail_length(hq, hkv, triple):
    """The kernel that gives a wavefront 2 or 4 adjacent KV heads: every context length from 0 to
    40 (every fill of the last 8- or 16-token tile, with and without full tiles before it), plus
    lengths around block and window boundaries; the pool is NaN-poisoned outside the valid tokens.
    Same shapes with one head per wavefront as the cross-check of the option."""
    lens = np.array(list(range(41)) + [127, 128, 129, 1023, 1025, 2050], dtype=np.int32)
    w = wl.Workload("wide", 80 + hq // 8, hq, hkv, 128, 16, len(lens), "x", ())
    c = make_case(w, triple, lens)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    try:
        for one_head in (0, 1):
            kv.kv_set_option("heads_per_wave", one_head)
            got = run_gpu_decode(c, gpu_view(w, triple))
            check_close(got, want, f"{hq}/{hkv} {triple} one_head {one_head}")
            assert (got[0] == 0).all()
            G = hq // hkv
            for i in range(c.info["n_q_local"]):     # ctx_len 1 -> the V row itself
                g = c.info["kv_head0"] + i // G
                assert np.array_equal(got[1, i], bf16_bits_to_f64(c.V[c.seq_off[1], g]))
    finally:
        kv.kv_set_option("heads_per_wave", 0)


@pytest.mark.parametrize("merge_mode", [0, 1, 2])
def test_long_sequences_cut_over_every_wavefront_head_groups(merge_mode):
    """DP view, four heads per wavefront: two head groups of one long sequence cut over all
    wavefronts (hundreds of pieces per pair: the merge kernel's long-list grid by default, one
    wavefront walking the whole list when the main kernel is made to finish it), next to a short
    sequence whose pairs are single pieces."""
    w = wl.Workload("long4", 73, 32, 8, 128, 16, 3, "x", ())
    ctx = np.array([9, 30011, 200], dtype=np.int32)
    c = make_case(w, (LAYOUT_DP, 1, 0), ctx)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    kv.kv_set_option("merge_mode", merge_mode)
    try:
        got = run_gpu_decode(c, gpu_view(w, (LAYOUT_DP, 1, 0)))
    finally:
        kv.kv_set_option("merge_mode", 0)
    check_close(got, want, f"long sequence, head groups, merge mode {merge_mode}")


@pytest.mark.parametrize("cost", [0, 8, 64])
def test_cost_of_a_pair_start_in_the_cut(cost):
    """The cut over the wavefronts counts the start of every (sequence, head group) pair as `cost`
    eighths of a tile; 64 (eight tiles) is the largest the option allows.  Many short sequences
    (the cost dominates the weighted axis, many wavefronts get ranges that start exactly at a pair),
    a mix, and a few long ones; four heads and one head per wavefront."""
    kv.kv_set_option("piece_cost", cost)
    try:
        for lens in (list(range(1, 120)), [1, 31, 32, 33, 0, 511, 513, 4100, 2049, 64, 7000, 96], [20000, 0, 12345]):
            lens = np.array(lens, dtype=np.int32)
            for triple in [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 8, 5)]:
                w = wl.Workload("cost", 74, 32, 8, 128, 16, len(lens), "x", ())
                c = make_case(w, triple, lens)
                want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
                got = run_gpu_decode(c, gpu_view(w, triple))
                check_close(got, want, f"cost {cost} {triple} {len(lens)} sequences")
    finally:
        kv.kv_set_option("piece_cost", -1)


@pytest.mark.parametrize("skew", [0, 100, 256])
def test_uneven_shares_between_xcds(skew):
    """The split gives wavefronts on even- and odd-numbered XCDs ranges of different length; 256 is
    the largest the option allows (5 : 3).  Few tiles (most wavefronts have none, and pairs are cut
    between wavefronts that have neighbours without tiles) and many (every wavefront busy), with
    four heads and one head per wavefront."""
    kv.kv_set_option("xcd_skew", skew)
    try:
        for lens in ([1, 31, 32, 33, 0, 511, 513, 4100, 2049, 64, 7000, 96], [20000, 17, 9000, 12345, 0, 700],
                     [3, 0, 9]):
            lens = np.array(lens, dtype=np.int32)
            for triple in [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 8, 5)]:
                w = wl.Workload("shares", 72, 32, 8, 128, 16, len(lens), "x", ())
                c = make_case(w, triple, lens)
                want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
                got = run_gpu_decode(c, gpu_view(w, triple))
                check_close(got, want, f"skew {skew} {triple} {len(lens)} sequences")
    finally:
        kv.kv_set_option("xcd_skew", -1)


@pytest.mark.parametrize("merge_mode", [0, 1])
def test_one_long_sequence_cut_over_every_wavefront(merge_mode):
    """A single (sequence, head) pair cut over every wavefront of the launch (about a thousand
    pieces to combine), twice in a row on one workspace that is garbage apart from the zeroed
    arrival words, which then serves a call of another kernel and another shape."""
    w = wl.Workload("long1", 70, 32, 8, 128, 16, 2, "x", ())
    ctx = np.array([40000, 3], dtype=np.int32)
    triple = (LAYOUT_TP, 8, 3)
    c = make_case(w, triple, ctx)
    view = gpu_view(w, triple)
    ws = poisoned_workspace(kv.paged_decode_attn_workspace_bytes(view, 2, 40000), 0xAB)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    q, pool = dev_u16(c.q), dev_u16(c.pool)
    table, n = torch.from_numpy(c.table).to(DEV), torch.from_numpy(c.ctx).to(DEV)
    kv.kv_set_option("merge_mode", merge_mode)
    try:
        for _ in range(2):
            out = kv.paged_decode_attn(q, pool, table, n, view, 40000, workspace=ws)
            torch.cuda.synchronize()
            check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)), want, "long sequence")
            assert sync_words_are_zero(ws)
        # same workspace, chunked vector-ALU kernel on a different shape, then the even-split kernel again
        c2 = make_case(TINY, (LAYOUT_TP, 2, 1))
        ws2 = poisoned_workspace(max(ws.numel(), kv.paged_decode_attn_workspace_bytes(gpu_view(TINY, (LAYOUT_TP, 2, 1)), 4, 300)),
                                 0xCD)
        kv.kv_set_option("chunk_tokens", 64)
        out2 = kv.paged_decode_attn(dev_u16(c2.q), dev_u16(c2.pool), torch.from_numpy(c2.table).to(DEV),
                                    torch.from_numpy(c2.ctx).to(DEV), gpu_view(TINY, (LAYOUT_TP, 2, 1)), 300,
                                    workspace=ws2)
        kv.kv_set_option("chunk_tokens", 0)
        out = kv.paged_decode_attn(q, pool, table, n, view, 40000, workspace=ws2)
        torch.cuda.synchronize()
    finally:
        kv.kv_set_option("merge_mode", 0)
        kv.kv_set_option("chunk_tokens", 0)
    check_close(bf16_bits_to_f64(out2.cpu().numpy().view(np.uint16)),
                oracle.paged_decode(c2.view, c2.q, c2.pool, c2.table, c2.ctx), "tiny on shared workspace")
    check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)), want, "long sequence after reuse")
    assert sync_words_are_zero(ws2)


def test_repeated_calls_on_one_workspace():
    """Calls of changing shapes in a row on one workspace (garbage apart from the zeroed arrival
    words), each compared with the oracle: nothing a call leaves in the workspace may leak into the
    next one, and every call leaves the arrival words zero."""
    w = wl.Workload("tuned", 71, 32, 8, 128, 16, 9, "x", ())
    ctx = np.array([7000, 4100, 9000, 33, 6000, 8000, 3000, 5111, 1], dtype=np.int32)
    short = np.array([300, 5000, 0, 1200, 64, 2500, 17, 800, 4000], dtype=np.int32)
    views = {t: gpu_view(w, t) for t in [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 1), (LAYOUT_TP, 8, 6)]}
    ws = poisoned_workspace(max(kv.paged_decode_attn_workspace_bytes(v, len(ctx), 9000) for v in views.values()), 0x5A)
    for call, (triple, lens) in enumerate([((LAYOUT_DP, 1, 0), ctx), ((LAYOUT_DP, 1, 0), ctx), ((LAYOUT_TP, 8, 6), short),
                                           ((LAYOUT_TP, 2, 1), ctx), ((LAYOUT_TP, 8, 6), ctx), ((LAYOUT_DP, 1, 0), short),
                                           ((LAYOUT_TP, 2, 1), short)]):
        c = make_case(w, triple, lens)
        want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
        out = kv.paged_decode_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                                   torch.from_numpy(c.ctx).to(DEV), views[triple], int(lens.max()), workspace=ws)
        torch.cuda.synchronize()
        check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)), want, f"{triple} call {call}")
        assert sync_words_are_zero(ws), f"call {call} left arrival words behind"


@pytest.mark.parametrize("p,r", [(2, 1), (4, 2), (8, 0)])
def test_mixed_layouts_in_one_launch(p, r):
    """One launch over a batch whose sequences are stored under two layouts of one pool: the TP
    layout of rank r and rank r's head slice inside DP-layout blocks (requests taken over from a
    DP engine without repacking).  Lengths make wavefront ranges cross sequences of different
    layouts; pool NaN-poisoned outside valid tokens."""
    w = wl.Workload("mixed", 73, 32, 8, 128, 16, 12, "x", ())
    ctx = np.array([1, 31, 4100, 33, 0, 511, 513, 2049, 64, 7000, 96, 1500], dtype=np.int32)
    ids = np.array([0, 1, 1, 0, 1, 0, 0, 1, 1, 0, 1, 1], dtype=np.int32)
    triples = [(LAYOUT_TP, p, r), (LAYOUT_DP, p, r)]
    c = make_mixed_case(w, triples, ids, ctx)
    want = oracle.paged_decode_mixed(c.views, c.view_ids, c.q, c.pool, c.table, c.ctx)
    views = [gpu_view(w, t) for t in triples]
    for order in (0, 1):   # the same batch with the view list (and ids) swapped
        vs = views[::-1] if order else views
        vid = (1 - ids) if order else ids
        out = kv.paged_decode_attn_mixed(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                                         torch.from_numpy(c.ctx).to(DEV),
                                         torch.from_numpy(vid.astype(np.int32)).to(DEV), vs, int(ctx.max()))
        torch.cuda.synchronize()
        got = bf16_bits_to_f64(out.cpu().numpy().view(np.uint16))
        check_close(got, want, f"mixed p={p} r={r} order {order}")
        assert (got[4] == 0).all()
    # a one-view list is the plain call
    c1 = make_case(w, triples[0], ctx)
    one = kv.paged_decode_attn_mixed(dev_u16(c1.q), dev_u16(c1.pool), torch.from_numpy(c1.table).to(DEV),
                                     torch.from_numpy(c1.ctx).to(DEV),
                                     torch.zeros(len(ctx), dtype=torch.int32, device=DEV), views[:1],
                                     int(ctx.max()))
    torch.cuda.synchronize()
    check_close(bf16_bits_to_f64(one.cpu().numpy().view(np.uint16)),
                oracle.paged_decode(c1.view, c1.q, c1.pool, c1.table, c1.ctx), "one view")


@pytest.mark.parametrize("batch", [2048, 2049])
def test_batch_at_and_past_the_even_split_limit(batch):
    """2048 sequences is the most the even-split kernel keeps in its LDS prefix table; one more and
    the call is served by the chunked matrix-core kernel.  Short contexts (1..80 tokens, some empty),
    every row compared."""
    rng = np.random.default_rng(batch)
    ctx = rng.integers(0, 81, size=batch).astype(np.int32)
    ctx[:4] = [0, 1, 16, 80]
    w = wl.Workload("bigbatch", 74, 32, 8, 128, 16, batch, "x", ())
    triple = (LAYOUT_TP, 4, 2)
    c = make_case(w, triple, ctx)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    got = run_gpu_decode(c, gpu_view(w, triple))
    check_close(got, want, f"batch {batch}")
    assert (got[ctx == 0] == 0).all()


def test_explicit_scale_and_large_logits():
    """A scale of 1.0 (8x the default at d = 64) makes the softmax nearly one-hot: checks the
    running-max handling."""
    c = make_case(TINY, (LAYOUT_TP, 2, 0))
    for scale in (1.0, 0.01):
        want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx, scale)
        got = run_gpu_decode(c, gpu_view(TINY, (LAYOUT_TP, 2, 0)), scale)
        check_close(got, want, f"scale {scale}")


def test_non_power_of_two_block_size():
    """B_base = 12 (capacity 24 at TP2): token -> (block, slot) needs a real division."""
    w = wl.Workload("b12", 31, 8, 2, 64, 12, 3, "x", ())
    ctx = np.array([11, 100, 313], dtype=np.int32)
    for triple in [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 1)]:
        c = make_case(w, triple, ctx)
        want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
        check_close(run_gpu_decode(c, gpu_view(w, triple)), want, f"b12 {triple}")


@pytest.mark.parametrize("hq,triple", [(32, (LAYOUT_DP, 1, 0)), (32, (LAYOUT_TP, 2, 1)), (64, (LAYOUT_DP, 1, 0)),
                                        (32, (LAYOUT_TP, 8, 3)), (32, (LAYOUT_DP, 4, 1))])
def test_block_capacity_48_on_the_matrix_core_kernels(hq, triple):
    """B_base = 48 (a multiple of 16 that is no power of two; 96 / 384 tokens per block at TP2 / TP8):
    the even-split kernels find a tile's block by division.  Shapes for four, two and one head per
    wavefront; lengths inside one block, at block boundaries and over many blocks."""
    ctx = np.array([5, 47, 48, 49, 95, 97, 383, 385, 1000, 3000], dtype=np.int32)
    w = wl.Workload("b48", 33 + hq // 32, hq, 8, 128, 48, len(ctx), "x", ())
    c = make_case(w, triple, ctx)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    check_close(run_gpu_decode(c, gpu_view(w, triple)), want, f"b48 {hq} {triple}")


@pytest.mark.parametrize("hq,triple", [(32, (LAYOUT_DP, 1, 0)), (64, (LAYOUT_TP, 2, 1)), (32, (LAYOUT_TP, 8, 0))])
@pytest.mark.parametrize("scale", [1.0, 0.3, 0.002])
def test_sharp_and_flat_softmax_at_head_dim_128(hq, triple, scale):
    """scale 1.0 at d = 128 gives logits of +-30 and more: the softmax is nearly one-hot and the
    reference maximum of the lazily rescaled kernels moves many times per sequence; 0.002 is
    nearly uniform.  Four, two and one head per wavefront."""
    ctx = np.array([1, 40, 700, 2500, 33], dtype=np.int32)
    w = wl.Workload("sharp", 35 + hq // 32, hq, 8, 128, 16, len(ctx), "x", ())
    c = make_case(w, triple, ctx)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx, scale)
    check_close(run_gpu_decode(c, gpu_view(w, triple), scale), want, f"scale {scale} {hq} {triple}")


def test_layouts_coexist_in_one_pool_on_gpu():
    """DP-written and TP-written blocks side by side in one pool, two calls (Sec. 5.2.3)."""
    dp_t, tp_t = (LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 1)
    geom = geometry(TINY)
    dp, tp = oracle.View(geom, *dp_t), oracle.View(geom, *tp_t)
    ctx_a, ctx_b = np.array([30, 70], dtype=np.int32), np.array([65, 5, 130], dtype=np.int32)
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
    dpool = dev_u16(pool)
    qb_r = q_slice(qb, tp.query(), 1)
    out_a = kv.paged_decode_attn(dev_u16(qa), dpool, torch.from_numpy(t_a).to(DEV),
                                 torch.from_numpy(ctx_a).to(DEV), gpu_view(TINY, dp_t), 70)
    out_b = kv.paged_decode_attn(dev_u16(qb_r), dpool, torch.from_numpy(t_b).to(DEV),
                                 torch.from_numpy(ctx_b).to(DEV), gpu_view(TINY, tp_t), 130)
    torch.cuda.synchronize()
    check_close(bf16_bits_to_f64(out_a.cpu().numpy().view(np.uint16)),
                oracle.paged_decode(dp, qa, pool, t_a, ctx_a), "dp part")
    check_close(bf16_bits_to_f64(out_b.cpu().numpy().view(np.uint16)),
                oracle.paged_decode(tp, qb_r, pool, t_b, ctx_b), "tp part")


# ------------------------------------------------------------------------------------ repack

def disjoint_tables(ctx, views, n_pool_blocks, index):
    perm = torch.randperm(n_pool_blocks, generator=wl.generator(index, wl.SUB_PERM)).numpy().astype(np.int32)
    tables, used = [], 0
    for v in views:
        t, k = wl.assign_blocks(ctx, v.query()["block_tokens"], perm[used:])
        tables.append(t)
        used += k
    return tables


def gpu_repack(dpool, w, src_t, dst_t, t_src, t_dst, ctx):
    sv, dv = gpu_view(w, src_t), gpu_view(w, dst_t)
    ts, td = torch.from_numpy(t_src).to(DEV), torch.from_numpy(t_dst).to(DEV)
    n = torch.from_numpy(ctx).to(DEV)
    n_blocks = dpool.numel() * 2 // sv.block_bytes
    assert kv.kv_validate_tables(sv, n_blocks, ts, n, dv, td) == kv.KV_OK
    kv.kv_repack(dpool, sv, dv, ts, td, n, int(ctx.max()))


def test_tiny_repack_dp_tp2_dp_bit_exact():
    """Tiny flow: DP -> TP2 r0 and r1 -> fresh DP blocks; after every step the whole pool must
    equal the oracle's pool byte for byte; the round trip restores the DP blocks."""
    geom = geometry(TINY)
    dp_t, tp0_t, tp1_t = (LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 0), (LAYOUT_TP, 2, 1)
    dp, tp0, tp1 = (oracle.View(geom, *t) for t in (dp_t, tp0_t, tp1_t))
    ctx = wl.draw_ctx_lens(TINY)
    K, V = wl.logical_kv(TINY, ctx)
    off = wl.seq_offsets(ctx)
    t_dp, t_tp0, t_tp1, t_back = disjoint_tables(ctx, [dp, tp0, tp1, dp], 128, 0)
    pool = wl.poisoned_pool(128, dp.query()["block_bytes"] // 2)
    oracle.scatter(dp, pool, t_dp, ctx, off, K, V)
    dpool = dev_u16(pool)
    steps = [(dp_t, tp0_t, t_dp, t_tp0, dp, tp0), (dp_t, tp1_t, t_dp, t_tp1, dp, tp1),
             (tp0_t, dp_t, t_tp0, t_back, tp0, dp), (tp1_t, dp_t, t_tp1, t_back, tp1, dp)]
    for src_t, dst_t, ts, td, sv, dv in steps:
        gpu_repack(dpool, TINY, src_t, dst_t, ts, td, ctx)
        oracle.repack(sv, dv, pool, ts, td, ctx)
        torch.cuda.synchronize()
        assert np.array_equal(dpool.cpu().numpy().view(np.uint16), pool), (src_t, dst_t)
    got = dpool.cpu().numpy().view(np.uint16)
    for s in range(len(ctx)):
        nb = int(wl.blocks_needed(ctx[s:s + 1], 16)[0])
        assert np.array_equal(got[t_back[s, :nb]], got[t_dp[s, :nb]])
    # and attention through the TP views of the repacked blocks matches the oracle
    q_full = wl.queries(TINY)
    for r, (triple, view, table) in enumerate([(tp0_t, tp0, t_tp0), (tp1_t, tp1, t_tp1)]):
        qr = q_slice(q_full, view.query(), r)
        out = kv.paged_decode_attn(dev_u16(qr), dpool, torch.from_numpy(table).to(DEV),
                                   torch.from_numpy(ctx).to(DEV), gpu_view(TINY, triple), 300)
        torch.cuda.synchronize()
        check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)),
                    oracle.paged_decode(view, qr, pool, table, ctx), f"after repack r{r}")


@pytest.mark.parametrize("hkv,d,b0,src_t,dst_t", [
    (8, 128, 16, (LAYOUT_DP, 1, 0), (LAYOUT_TP, 4, 0)),
    (8, 128, 16, (LAYOUT_TP, 4, 2), (LAYOUT_DP, 1, 0)),
    (8, 128, 16, (LAYOUT_TP, 2, 1), (LAYOUT_TP, 8, 6)),
    (8, 128, 16, (LAYOUT_DP, 8, 3), (LAYOUT_TP, 8, 3)),       # strided in-place slice -> compact
    (6, 64, 12, (LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 1)),        # 3 common heads: run not a power of two
    (8, 128, 16, (LAYOUT_TP, 2, 0), (LAYOUT_TP, 4, 3)),       # nothing in common: pool unchanged
])
def test_repack_bit_exact_various_views(hkv, d, b0, src_t, dst_t):
    w = wl.Workload("rp", 40 + hkv, 4 * hkv, hkv, d, b0, 7, "x", ())
    geom = geometry(w)
    sv, dv = oracle.View(geom, *src_t), oracle.View(geom, *dst_t)
    ctx = np.array([0, 1, b0, b0 + 1, 700, 1025, 64], dtype=np.int32)
    K, V = wl.logical_kv(w, ctx)
    t_src, t_dst = disjoint_tables(ctx, [sv, dv], 400, w.index)
    pool = wl.poisoned_pool(400, sv.query()["block_bytes"] // 2)
    oracle.scatter(sv, pool, t_src, ctx, wl.seq_offsets(ctx), K, V)
    dpool = dev_u16(pool)
    gpu_repack(dpool, w, src_t, dst_t, t_src, t_dst, ctx)
    oracle.repack(sv, dv, pool, t_src, t_dst, ctx)
    torch.cuda.synchronize()
    assert np.array_equal(dpool.cpu().numpy().view(np.uint16), pool)


def test_append_then_decode_matches_oracle():
    """kv_append writes token n of every sequence through the view; the pool must equal the
    oracle's scatter of n+1 tokens, and a decode over n+1 tokens must match."""
    w = wl.Workload("ap", 50, 32, 8, 128, 16, 5, "x", ())
    ctx1 = np.array([1, 16, 17, 129, 640], dtype=np.int32)       # lengths after the append
    for triple in [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 4, 1), (LAYOUT_DP, 2, 1)]:
        c = make_case(w, triple, ctx1)                            # pool holds all ctx1 tokens
        ov, info = c.view, c.info
        # start from a pool holding only the first ctx1 - 1 tokens
        pool0 = wl.poisoned_pool(c.pool.shape[0], c.pool.shape[1])
        oracle.scatter(ov, pool0, c.table, ctx1 - 1, c.seq_off, c.K, c.V)
        h0, hl = info["kv_head0"], info["n_kv_local"]
        last = c.seq_off[1:] - 1
        k_new = np.ascontiguousarray(c.K[last][:, h0:h0 + hl])
        v_new = np.ascontiguousarray(c.V[last][:, h0:h0 + hl])
        dpool = dev_u16(pool0)
        view = gpu_view(w, triple)
        table = torch.from_numpy(c.table).to(DEV)
        kv.kv_append(dpool, view, dev_u16(k_new), dev_u16(v_new), table,
                     torch.from_numpy((ctx1 - 1).astype(np.int32)).to(DEV))
        torch.cuda.synchronize()
        assert np.array_equal(dpool.cpu().numpy().view(np.uint16), c.pool), triple
        out = kv.paged_decode_attn(dev_u16(c.q), dpool, table, torch.from_numpy(ctx1).to(DEV), view, 640)
        torch.cuda.synchronize()
        check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)),
                    oracle.paged_decode(ov, c.q, c.pool, c.table, ctx1), f"append {triple}")


def test_validate_tables_reports_bad_contents():
    view = gpu_view(TINY, (LAYOUT_DP, 1, 0))
    n = torch.tensor([40, 20], dtype=torch.int32, device=DEV)
    good = torch.tensor([[3, 1, 2], [0, 5, -1]], dtype=torch.int32, device=DEV)
    assert kv.kv_validate_tables(view, 8, good, n) == kv.KV_OK
    assert kv.kv_validate_tables(view, 4, good, n) == kv.KV_ERR_RANGE          # id 5 >= 4 blocks
    dup = torch.tensor([[3, 1, 2], [0, 1, -1]], dtype=torch.int32, device=DEV)
    assert kv.kv_validate_tables(view, 8, dup, n) == kv.KV_ERR_ALIAS
    neg = torch.tensor([[3, -1, 2], [0, 5, -1]], dtype=torch.int32, device=DEV)
    assert kv.kv_validate_tables(view, 8, neg, n) == kv.KV_ERR_RANGE
    other = torch.tensor([[6, 7, 4], [2, 8, -1]], dtype=torch.int32, device=DEV)   # shares block 2
    assert kv.kv_validate_tables(view, 16, good, n, view, other) == kv.KV_ERR_ALIAS
    apart = torch.tensor([[6, 7, 4], [9, 8, -1]], dtype=torch.int32, device=DEV)
    assert kv.kv_validate_tables(view, 16, good, n, view, apart) == kv.KV_OK
