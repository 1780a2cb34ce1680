"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: the pool is
N(0,1) everywhere (drawn on the device from a seeded generator and copied back for the
oracle), outputs are checked on sampled (sequence, query head) rows that the CPU oracle
computes one by one.  Repack at full size is checked bit-exactly on whole sampled blocks."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import harness
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, geometry

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 2e-2, 2e-3

CASES = [(name, tr) for name in ("llama8b_dp_b64", "llama8b_tp_b128", "llama70b_tp8_b256",
                                 "llama8b_tp4_longmix") for tr in wl.WORKLOADS[name].views]
CASES += [("llama8b_tp_b128", (1, 4, 3)), ("llama70b_tp8_b256", (1, 8, 5))]     # non-zero ranks


def host_u16(t: torch.Tensor) -> np.ndarray:
    return t.view(dtype=torch.int16).cpu().numpy().view(np.uint16)


def sample_pairs(ctx, n_q_local, how_many, seed):
    rng = np.random.default_rng(seed)
    seqs = list(rng.integers(0, len(ctx), size=how_many))
    seqs[0], seqs[1] = int(np.argmax(ctx)), int(np.argmin(ctx))
    heads = list(rng.integers(0, n_q_local, size=how_many))
    heads[0] = n_q_local - 1
    return np.array(seqs, dtype=np.int32), np.array(heads, dtype=np.int32)


@pytest.mark.parametrize("name,triple", CASES)
def test_decode_full_size_sampled_rows(name, triple):
    w = wl.WORKLOADS[name]
    case = harness.build_decode_case(w, triple, n_copies=1)
    run = case.prepared()
    run(0)
    torch.cuda.synchronize()
    got_all = bf16_bits_to_f64(host_u16(case.out))
    assert np.isfinite(got_all).all()
    ps, ph = sample_pairs(case.ctx, case.view.n_q_local, 48, 1234 + w.index)
    view = oracle.View(geometry(w), *triple)
    want = oracle.paged_decode_pairs(view, host_u16(case.q), host_u16(case.pools[0]), case.tables[0],
                                     case.ctx, ps, ph)
    err = np.abs(got_all[ps, ph] - want)
    assert err.max() <= MAX_ABS, f"{name} {triple}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS, f"{name} {triple}: mean-abs {err.mean():.3e}"
    # every row is a convex combination of V rows drawn from N(0,1): |out| stays small, and rows of
    # long contexts average many values, so their magnitude shrinks
    assert np.abs(got_all).max() < 6.0


@pytest.mark.parametrize("name,src,dst,lens", [
    ("llama8b_tp_b128", (0, 1, 0), (1, 4, 0), None),                      # whole batch DP <-> TP4 r0
    ("llama8b_tp4_longmix", (0, 1, 0), (1, 4, 0), [131072, 131072]),      # the two long sequences
])
def test_repack_full_size_bit_exact(name, src, dst, lens):
    w = wl.WORKLOADS[name]
    n_tokens = None if lens is None else np.array(lens, dtype=np.int32)
    rc = harness.build_repack_case(w, src, dst, n_tokens)
    assert kv.kv_validate_tables(rc.src_view, rc.pool.shape[0], rc.src_dev, rc.n_dev,
                                 rc.dst_view, rc.dst_dev) == kv.KV_OK
    before = host_u16(rc.pool)
    rc.forward()
    rc.backward()
    torch.cuda.synchronize()
    after = host_u16(rc.pool)
    sv, dv = oracle.View(geometry(w), *src), oracle.View(geometry(w), *dst)
    # the oracle redoes both repacks for a sample of sequences on a copy of the original pool
    rng = np.random.default_rng(7)
    pick = np.unique(np.concatenate([[int(np.argmax(rc.n_tokens))],
                                     rng.integers(0, len(rc.n_tokens), size=3)])).astype(np.int64)
    expect = before.copy()
    sub_n = np.ascontiguousarray(rc.n_tokens[pick])
    oracle.repack(sv, dv, expect, rc.src_table[pick], rc.dst_table[pick], sub_n)
    oracle.repack(dv, sv, expect, rc.dst_table[pick], rc.back_table[pick], sub_n)
    for table in (rc.dst_table, rc.back_table, rc.src_table):
        ids = table[pick]
        ids = ids[ids >= 0]
        assert np.array_equal(after[ids], expect[ids])
    # property over the whole pool: source blocks untouched; blocks in no table untouched
    src_ids = rc.src_table[rc.src_table >= 0]
    assert np.array_equal(after[src_ids], before[src_ids])
    used = np.zeros(before.shape[0], dtype=bool)
    for table in (rc.src_table, rc.dst_table, rc.back_table):
        used[table[table >= 0]] = True
    assert np.array_equal(after[~used], before[~used])
    # round trip: slice r of every valid token came back (compare src blocks with returned blocks
    # on the heads of rank 0: columns [0, 2 heads * 128) of each token row of the DP blocks)
    dinfo = dv.query()
    row = geometry(w).n_kv_heads * w.head_dim
    run = dinfo["n_kv_local"] * w.head_dim
    for s in pick:
        nb = int(wl.blocks_needed(rc.n_tokens[s:s + 1], 16)[0])
        full = int(rc.n_tokens[s]) // 16                  # blocks whose 16 slots are all valid
        a = after[rc.back_table[s, :full]].reshape(full, 2, 16, row)[..., :run]
        b = before[rc.src_table[s, :full]].reshape(full, 2, 16, row)[..., :run]
        assert np.array_equal(a, b)
        assert nb >= full


def test_mixed_layout_full_size_sampled_rows():
    """The mixed-layout case bench.py times (llama8b_tp_b128 under TP2 rank 0, every other sequence in
    DP-layout blocks), sampled rows against the single-view oracle under each row's own view."""
    w = wl.WORKLOADS["llama8b_tp_b128"]
    mc = harness.build_mixed_case(w, 2, 0)
    mc.run()
    torch.cuda.synchronize()
    got_all = bf16_bits_to_f64(host_u16(mc.out))
    assert np.isfinite(got_all).all()
    ps, ph = sample_pairs(mc.ctx, mc.views[0].n_q_local, 48, 4321)
    pool, q, table = host_u16(mc.pool), host_u16(mc.q), mc.table_dev.cpu().numpy()
    ids = mc.ids_dev.cpu().numpy()
    for k, triple in enumerate([(1, 2, 0), (0, 2, 0)]):
        sel = ids[ps] == k
        assert sel.any()
        view = oracle.View(geometry(w), *triple)
        want = oracle.paged_decode_pairs(view, q, pool, table, mc.ctx, ps[sel], ph[sel])
        err = np.abs(got_all[ps[sel], ph[sel]] - want)
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (triple, err.max(), err.mean())


def test_prefill_bench_cases_sampled_rows():
    """The first and the last prefill case of bench.py at full size: sampled query rows (first and last
    tokens of sequences, query-tile and key-tile borders) against the oracle."""
    w8 = wl.Workload("llama8b_recompute", 90, 32, 8, 128, 16, 8, "fixed", ())
    for triple, ctx, ql in (((0, 1, 0), [4096] * 8, [4096] * 8), ((0, 1, 0), [8192] * 16, [512] * 16)):
        pc = harness.build_prefill_case(w8, triple, ctx, ql)
        pc.run()
        torch.cuda.synchronize()
        got_all = bf16_bits_to_f64(host_u16(pc.out))
        assert np.isfinite(got_all).all()
        q_off = wl.seq_offsets(pc.q_lens)
        rng = np.random.default_rng(99)
        rows = np.unique(np.concatenate([q_off[:-1], q_off[1:] - 1, q_off[:2] + 31, q_off[:2] + 32,
                                         rng.integers(0, q_off[-1], size=12)]))[:24].astype(np.int64)
        hql = pc.view.n_q_local
        rq = np.repeat(rows, 2)
        rh = np.tile(np.array([0, hql - 1], dtype=np.int32), len(rows))
        view = oracle.View(geometry(w8), *triple)
        want = oracle.paged_prefill_rows(view, host_u16(pc.q), host_u16(pc.pool), pc.table_dev.cpu().numpy(),
                                         pc.ctx, q_off, rq, rh)
        err = np.abs(got_all[rq, rh] - want)
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (triple, err.max(), err.mean())


def test_linear_view_full_size_sampled_outputs():
    """Llama-8B projections at full size (hidden 4096) on rank views, M = 64 and 256: every output of
    a sample of batch rows against the fp64 product."""
    from oracle import weights as ow
    hq, hkv, d, hidden = 32, 8, 128, 4096
    g = wl.generator(42, 1)
    wq = wl.randn_bf16(((hq + 2 * hkv) * d, hidden), g)
    wo = wl.randn_bf16((hidden, hq * d), g)
    dev = lambda a: torch.from_numpy(a.view(np.int16)).to("cuda:0").view(torch.bfloat16)
    dwq, dwo = dev(wq), dev(wo)
    for M, m, r in ((64, 1, 0), (256, 2, 1), (100, 8, 7)):
        x = wl.randn_bf16((M, hidden), g)
        a = wl.randn_bf16((M, hq * d), g)
        rows = np.unique(np.array([0, 1, 15, 16, 63, M // 2, M - 1]))
        ov = ow.weight_view_fused_qkv(hq, hkv, d, hidden, r, m)
        y = kv.kv_linear_view(dev(x), dwq, kv.kv_weight_view_fused_qkv(hq, hkv, d, hidden, r, m))
        ov2 = ow.weight_view(1, r, m, hidden, hq * d)
        xs = np.ascontiguousarray(a[:, ov2.col_start:ov2.col_start + ov2.col_count])
        y2 = kv.kv_linear_view(dev(a)[:, ov2.col_start:ov2.col_start + ov2.col_count], dwo,
                               kv.kv_weight_view_make(1, r, m, hidden, hq * d))
        torch.cuda.synchronize()
        for got, want, K in ((bf16_bits_to_f64(host_u16(y))[rows], ow.linear_view(x[rows], wq, ov), hidden),
                             (bf16_bits_to_f64(host_u16(y2))[rows], ow.linear_view(xs[rows], wo, ov2), ov2.col_count)):
            tol = np.abs(want) * 2.0 ** -8 + 2.0 * K * K * 2.0 ** -24 + 1e-6
            assert np.isfinite(got).all() and (np.abs(got - want) <= tol).all(), (M, m, r, np.abs(got - want).max())
