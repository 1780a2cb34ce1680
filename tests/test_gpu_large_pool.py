"""Block ids whose byte offsets lie past 4 GiB: a 5 GiB pool of 64 KiB blocks, the tables spread over
all of it.  Decode through two views, a repack into other blocks of the same pool, multi-token
attention and an append, each against the oracle on the same (host) pool; only the blocks a step
touches are copied back."""
import numpy as np
import pytest
import torch

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, geometry, q_slice

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MAX_ABS, MEAN_ABS = 2e-2, 2e-3
BLOCK_BYTES = 65536
N_BLOCKS = 5 * 2**30 // BLOCK_BYTES + 7


def dev_u16(a):
    return torch.from_numpy(a.view(np.int16)).to(DEV)


def check_close(got, want, what):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.3e}"


def test_every_entry_point_on_a_pool_past_4gib():
    w = wl.Workload("large_pool", 61, 32, 8, 128, 16, 5, "x", ())
    geom = geometry(w)
    dp_t, tp_t = (LAYOUT_DP, 1, 0), (LAYOUT_TP, 2, 1)
    dp, tp = oracle.View(geom, *dp_t), oracle.View(geom, *tp_t)
    assert dp.query()["block_bytes"] == BLOCK_BYTES
    ctx = np.array([700, 33, 1500, 64, 257], dtype=np.int32)
    K, V = wl.logical_kv(w, ctx)
    off = wl.seq_offsets(ctx)
    perm = torch.randperm(N_BLOCKS, generator=wl.generator(w.index, wl.SUB_PERM)).numpy().astype(np.int32)
    # the drawn ids are spread over the whole pool; make sure both tables reach past 4 GiB
    t_dp, used = wl.assign_blocks(ctx + 1, 16, perm)              # room for one appended token
    t_tp, _ = wl.assign_blocks(ctx, 32, perm[used:])
    assert int(t_dp.max()) * BLOCK_BYTES > 2**32 and int(t_tp.max()) * BLOCK_BYTES > 2**32
    pool = wl.poisoned_pool(N_BLOCKS, BLOCK_BYTES // 2)
    oracle.scatter(dp, pool, t_dp, ctx, off, K, V)
    dpool = dev_u16(pool)
    assert dpool.numel() * 2 > 2**32
    gv_dp = kv.kv_view_create(32, 8, 128, 16, *dp_t)
    gv_tp = kv.kv_view_create(32, 8, 128, 16, *tp_t)
    d_ctx = torch.from_numpy(ctx).to(DEV)
    d_tdp, d_ttp = torch.from_numpy(t_dp).to(DEV), torch.from_numpy(t_tp).to(DEV)
    q_full = wl.queries(w)

    def touched(table):
        ids = np.unique(table[table >= 0]).astype(np.int64)
        return ids, dpool.view(N_BLOCKS, BLOCK_BYTES // 2)[torch.from_numpy(ids).to(DEV)].cpu().numpy().view(np.uint16)

    # decode through the DP view
    out = kv.paged_decode_attn(dev_u16(q_full), dpool, d_tdp, d_ctx, gv_dp, int(ctx.max()))
    torch.cuda.synchronize()
    check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)),
                oracle.paged_decode(dp, q_full, pool, t_dp, ctx), "decode, DP view")

    # repack into TP2 rank-1 blocks elsewhere in the pool: bit-exact on the destination blocks
    assert kv.kv_validate_tables(gv_dp, N_BLOCKS, d_tdp, d_ctx, gv_tp, d_ttp) == kv.KV_OK
    kv.kv_repack(dpool, gv_dp, gv_tp, d_tdp, d_ttp, d_ctx, int(ctx.max()))
    oracle.repack(dp, tp, pool, t_dp, t_tp, ctx)
    torch.cuda.synchronize()
    ids, got = touched(t_tp)
    assert np.array_equal(got, pool[ids]), "repack destination blocks"
    q_tp = q_slice(q_full, tp.query(), 1)
    out = kv.paged_decode_attn(dev_u16(q_tp), dpool, d_ttp, d_ctx, gv_tp, int(ctx.max()))
    torch.cuda.synchronize()
    check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)),
                oracle.paged_decode(tp, q_tp, pool, t_tp, ctx), "decode, TP2 view after repack")

    # multi-token attention: the last 70 / 33 / 1 / 64 / 200 tokens of each sequence as queries
    qlen = np.array([70, 33, 1, 64, 200], dtype=np.int32)
    q_off = wl.seq_offsets(qlen)
    qp = wl.randn_bf16((int(q_off[-1]), 32, 128), wl.generator(w.index, wl.SUB_MISC))
    out = kv.paged_prefill_attn(dev_u16(qp), dpool, d_tdp, d_ctx, torch.from_numpy(q_off.astype(np.int32)).to(DEV),
                                gv_dp, max_ctx_len=int(ctx.max()), max_q_len=int(qlen.max()))
    torch.cuda.synchronize()
    check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)),
                oracle.paged_prefill(dp, qp, pool, t_dp, ctx, q_off), "multi-token attention, DP view")

    # append one token to every sequence through the DP view: bit-exact on the DP blocks
    k_new = wl.randn_bf16((len(ctx), 8, 128), wl.generator(w.index, wl.SUB_DATA + 5))
    v_new = wl.randn_bf16((len(ctx), 8, 128), wl.generator(w.index, wl.SUB_DATA + 6))
    kv.kv_append(dpool, gv_dp, dev_u16(k_new), dev_u16(v_new), d_tdp, d_ctx)
    K2 = np.concatenate([np.concatenate([K[off[s]:off[s + 1]], k_new[s:s + 1]]) for s in range(len(ctx))])
    V2 = np.concatenate([np.concatenate([V[off[s]:off[s + 1]], v_new[s:s + 1]]) for s in range(len(ctx))])
    oracle.scatter(dp, pool, t_dp, ctx + 1, wl.seq_offsets(ctx + 1), K2, V2)
    torch.cuda.synchronize()
    ids, got = touched(t_dp)
    assert np.array_equal(got, pool[ids]), "DP blocks after the append"


@pytest.mark.parametrize("hq,hkv", [(4, 1), (16, 4)])
def test_one_million_token_sequence(hq, hkv):
    """One sequence of 2^20 tokens next to a short one: tile counts, prefix sums and piece lists
    eight times longer than the longest benchmark sequence (one head per wavefront, and four)."""
    from helpers import make_case
    w = wl.Workload("million", 62 + hkv, hq, hkv, 128, 16, 2, "x", ())
    ctx = np.array([1 << 20, 100], dtype=np.int32)
    c = make_case(w, (LAYOUT_DP, 1, 0), ctx, slack=1.01)
    view = kv.kv_view_create(hq, hkv, 128, 16, LAYOUT_DP, 1, 0)
    out = kv.paged_decode_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                               torch.from_numpy(c.ctx).to(DEV), view, max_ctx_len=int(ctx.max()))
    torch.cuda.synchronize()
    check_close(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)),
                oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx), f"2^20 tokens, {hq}/{hkv} heads")
