"""GPU parity of paged_prefill_attn (multi-token causal attention through a view) with the oracle."""
import numpy as np
import pytest
import torch

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, make_prefill_case

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MAX_ABS, MEAN_ABS = 2e-2, 2e-3   # bf16 output of O(1) values; same bar as decode


def dev_u16(a):
    return torch.from_numpy(a.view(np.int16)).to(DEV)


def gpu_view(w, triple):
    return kv.kv_view_create(w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size, *triple)


def run_gpu(c, view):
    out = kv.paged_prefill_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                                torch.from_numpy(c.ctx).to(DEV),
                                torch.from_numpy(c.q_off.astype(np.int32)).to(DEV), view,
                                max_ctx_len=int(c.ctx.max()), max_q_len=int(c.q_lens.max()))
    torch.cuda.synchronize()
    return bf16_bits_to_f64(out.cpu().numpy().view(np.uint16))


def check_close(got, want, what):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.3e}"


CTX = np.array([17, 64, 150, 300, 5, 33, 613, 96], dtype=np.int32)
QLEN = np.array([17, 1, 40, 300, 0, 32, 77, 96], dtype=np.int32)   # whole prompt, decode, chunks, none


@pytest.mark.parametrize("hq,hkv,triple", [
    (32, 8, (LAYOUT_DP, 1, 0)), (32, 8, (LAYOUT_TP, 2, 1)), (32, 8, (LAYOUT_TP, 8, 5)),
    (32, 8, (LAYOUT_DP, 4, 3)), (64, 8, (LAYOUT_TP, 8, 2)), (8, 8, (LAYOUT_TP, 2, 0)),
    (16, 8, (LAYOUT_DP, 1, 0)), (128, 8, (LAYOUT_TP, 4, 1)), (48, 8, (LAYOUT_TP, 2, 1)), (24, 2, (LAYOUT_DP, 1, 0))])
def test_prefill_matches_oracle(hq, hkv, triple):
    """Group sizes 1, 2, 4, 6, 8, 12 and 16; every layout; query lengths that are the whole context, one
    token, none, and chunks whose ends fall inside key tiles and query tiles; pool NaN-poisoned
    outside the valid tokens.  Every output row is compared."""
    w = wl.Workload("prefill", 80 + hq // 8, hq, hkv, 128, 16, len(CTX), "x", ())
    c = make_prefill_case(w, triple, CTX, QLEN)
    want = oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off)
    got = run_gpu(c, gpu_view(w, triple))
    check_close(got, want, f"{hq}/{hkv} {triple}")


def test_one_query_token_per_sequence_is_decode():
    w = wl.Workload("prefill1", 85, 32, 8, 128, 16, 5, "x", ())
    ctx = np.array([1, 31, 32, 700, 65], dtype=np.int32)
    c = make_prefill_case(w, (LAYOUT_TP, 2, 0), ctx, np.ones(5, dtype=np.int32))
    view = gpu_view(w, (LAYOUT_TP, 2, 0))
    got = run_gpu(c, view)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    check_close(got, want, "q_len 1")


@pytest.mark.parametrize("triple", [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 4, 1)])
def test_short_chunks_on_long_contexts_split_the_key_range(triple):
    """Two sequences, a few dozen new tokens each on thousands of cached ones: too few query tiles
    to fill the chip, so the library cuts each tile's key range over several workgroups and merges
    their partial results (the workspace path).  Includes splits that see no key at all for the
    early rows of a tile.  Every row compared; the workspace starts as garbage."""
    w = wl.Workload("prefill_split", 87, 32, 8, 128, 16, 2, "x", ())
    ctx, qlen = np.array([9000, 3000], dtype=np.int32), np.array([70, 33], dtype=np.int32)
    c = make_prefill_case(w, triple, ctx, qlen)
    view = gpu_view(w, triple)
    need = kv.lib().paged_prefill_attn_workspace_bytes(view.handle, 2, int(qlen.sum()), 9000, 70)
    assert need > 0
    ws = torch.full((need,), 0x7F, dtype=torch.uint8, device=DEV)
    out = kv.paged_prefill_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                                torch.from_numpy(c.ctx).to(DEV), torch.from_numpy(c.q_off.astype(np.int32)).to(DEV),
                                view, 9000, 70, workspace=ws)
    torch.cuda.synchronize()
    got = bf16_bits_to_f64(out.cpu().numpy().view(np.uint16))
    want = oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off)
    check_close(got, want, f"split {triple}")
    # too small a workspace is reported, not overrun
    import ctypes as C
    rc = kv.lib().paged_prefill_attn(C.c_void_p(256), C.c_void_p(256), C.c_void_p(256), 10, C.c_void_p(256), 1024,
                                     C.c_void_p(256), C.c_void_p(256), 2, int(qlen.sum()), 9000, 70, view.handle,
                                     0.0, C.c_void_p(256), need - 1, None)
    assert rc == kv.KV_ERR_WORKSPACE


def test_long_prompt_sampled_rows():
    """A 4096-token prompt prefilled whole next to a 1000-token chunk on a 5000-token context:
    many query tiles per sequence, the oracle on sampled rows (first, last, tile borders)."""
    w = wl.Workload("prefill_long", 86, 32, 8, 128, 16, 2, "x", ())
    ctx = np.array([4096, 5000], dtype=np.int32)
    qlen = np.array([4096, 1000], dtype=np.int32)
    for triple in [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 4, 3)]:
        c = make_prefill_case(w, triple, ctx, qlen)
        got = run_gpu(c, gpu_view(w, triple))
        rows = np.array([0, 1, 15, 16, 31, 32, 33, 1000, 2047, 2048, 4095, 4096, 4097, 4596, 5094, 5095],
                        dtype=np.int64)
        hql = c.info["n_q_local"]
        rq = np.repeat(rows, hql)
        rh = np.tile(np.arange(hql, dtype=np.int32), len(rows))
        want = oracle.paged_prefill_rows(c.view, c.q, c.pool, c.table, c.ctx, c.q_off, rq, rh)
        check_close(got[rq, rh], want, f"long {triple}")


@pytest.mark.parametrize("scale", [1.0, 0.3, 0.002])
@pytest.mark.parametrize("triple", [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 4, 2)])
def test_sharp_and_flat_softmax(triple, scale):
    """scale 1.0 at d = 128 gives logits of +-30 and more: nearly one-hot weights, and the reference
    maximum of the lazily rescaled accumulators moves many times along a row of tiles (also across
    the split key ranges of the second sequence); 0.002 is nearly uniform.  Every row compared."""
    w = wl.Workload("prefill_sharp", 88, 32, 8, 128, 16, 3, "x", ())
    ctx, qlen = np.array([700, 5000, 65], dtype=np.int32), np.array([700, 40, 1], dtype=np.int32)
    c = make_prefill_case(w, triple, ctx, qlen)
    out = kv.paged_prefill_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                                torch.from_numpy(c.ctx).to(DEV), torch.from_numpy(c.q_off.astype(np.int32)).to(DEV),
                                gpu_view(w, triple), max_ctx_len=int(ctx.max()), max_q_len=int(qlen.max()), scale=scale)
    torch.cuda.synchronize()
    got = bf16_bits_to_f64(out.cpu().numpy().view(np.uint16))
    want = oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off, scale)
    check_close(got, want, f"scale {scale} {triple}")
