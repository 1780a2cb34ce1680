"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: the pool is
N(0,1) everywhere (drawn on the device from a seeded generator and copied back for the
oracle).  Decode: every output row of every named workload and view against the CPU oracle.
Repack: the whole pool, byte for byte, against the oracle's repack of a copy of the original pool.
The multi-token and linear-view rows, whose oracle costs minutes at these sizes, are checked on
sampled rows."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import harness
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, geometry, linear_tolerance

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 2e-2, 2e-3

CASES = [(name, tr) for name in ("llama8b_dp_b64", "llama8b_tp_b128", "llama70b_tp8_b256",
                                 "llama8b_tp4_longmix") for tr in wl.WORKLOADS[name].views]
CASES += [("llama8b_tp_b128", (1, 4, 3)), ("llama70b_tp8_b256", (1, 8, 5))]     # non-zero ranks


def host_u16(t: torch.Tensor) -> np.ndarray:
    return t.view(dtype=torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("name,triple", CASES)
def test_decode_full_size_all_rows(name, triple):
    w = wl.WORKLOADS[name]
    case = harness.build_decode_case(w, triple, n_copies=1)
    run = case.prepared()
    run(0)
    torch.cuda.synchronize()
    got_all = bf16_bits_to_f64(host_u16(case.out))
    assert np.isfinite(got_all).all()
    view = oracle.View(geometry(w), *triple)
    want = oracle.paged_decode(view, host_u16(case.q), host_u16(case.pools[0]), case.tables[0], case.ctx)
    assert want.shape == got_all.shape
    err = np.abs(got_all - want)
    worst = np.unravel_index(int(np.argmax(err)), err.shape)
    assert err.max() <= MAX_ABS, f"{name} {triple}: max-abs {err.max():.3e} at (sequence, head, element) {worst}"
    assert err.mean() <= MEAN_ABS, f"{name} {triple}: mean-abs {err.mean():.3e}"
    # per sequence as well: a wrong row in a short sequence must not hide in the batch mean
    per_seq = err.reshape(err.shape[0], -1).mean(axis=1)
    assert per_seq.max() <= MEAN_ABS, f"{name} {triple}: sequence {int(per_seq.argmax())} mean-abs {per_seq.max():.3e}"


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
    # the oracle redoes both repacks, all sequences, on a copy of the original pool; then every byte
    # of the pool must agree: moved rows, untouched tails and head slices, unused blocks
    expect = before.copy()
    oracle.repack(sv, dv, expect, rc.src_table, rc.dst_table, rc.n_tokens)
    oracle.repack(dv, sv, expect, rc.dst_table, rc.back_table, rc.n_tokens)
    assert not np.array_equal(expect, before)
    if not np.array_equal(after, expect):
        bad = np.flatnonzero((after != expect).any(axis=1))
        raise AssertionError(f"{name}: {len(bad)} pool blocks differ from the oracle's, first {bad[:8]}")
    pick = np.unique(np.concatenate([[int(np.argmax(rc.n_tokens))],
                                     np.random.default_rng(7).integers(0, len(rc.n_tokens), size=3)])).astype(np.int64)
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


def test_mixed_layout_full_size_all_rows():
    """The mixed-layout case bench.py times (llama8b_tp_b128 under TP2 rank 0, every other sequence in
    DP-layout blocks): every output row against the oracle, each sequence under its own view."""
    w = wl.WORKLOADS["llama8b_tp_b128"]
    mc = harness.build_mixed_case(w, 2, 0)
    mc.run()
    torch.cuda.synchronize()
    got_all = bf16_bits_to_f64(host_u16(mc.out))
    assert np.isfinite(got_all).all()
    pool, q, table = host_u16(mc.pool), host_u16(mc.q), mc.table_dev.cpu().numpy()
    ids = mc.ids_dev.cpu().numpy()
    assert (ids == 0).any() and (ids == 1).any()
    views = [oracle.View(geometry(w), *triple) for triple in ((1, 2, 0), (0, 2, 0))]
    want = oracle.paged_decode_mixed(views, ids, q, pool, table, mc.ctx)
    err = np.abs(got_all - want)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (err.max(), err.mean())
    per_seq = err.reshape(err.shape[0], -1).mean(axis=1)
    assert per_seq.max() <= MEAN_ABS, (int(per_seq.argmax()), per_seq.max())


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
        for got, xr, wt, view in ((bf16_bits_to_f64(host_u16(y))[rows], x[rows], wq, ov),
                                  (bf16_bits_to_f64(host_u16(y2))[rows], xs[rows], wo, ov2)):
            want = ow.linear_view(xr, wt, view)
            tol = linear_tolerance(xr, wt, view, want)
            assert np.isfinite(got).all() and (np.abs(got - want) <= tol).all(), (M, m, r, np.abs(got - want).max())
