"""Seeded random sweep of paged_decode_attn, paged_prefill_attn, kv_repack + kv_append and
kv_linear_view against the oracle.

Shapes the hand-picked cases do not enumerate: every combination of KV-head count, group size,
base block size (16, 32, 48 tokens), layout, rank, batch size and context-length mix the draw
produces, under random kernel options (variants, forced split-KV chunks, XCD skew, the cost of a
piece in the cut).  All inputs are valid; every output row is compared."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, linear_tolerance, make_case, make_prefill_case

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MAX_ABS, MEAN_ABS = 2e-2, 2e-3


def dev_u16(a):
    return torch.from_numpy(a.view(np.int16)).to(DEV)


def draw_lens(rng, batch, hi):
    out = []
    for _ in range(batch):
        k = rng.integers(0, 6)
        if k == 0:
            out.append(int(rng.integers(1, 40)))
        elif k == 1:   # at or next to a tile / block border
            m = int(rng.choice([16, 32, 64, 128, 256, 512])) * int(rng.integers(1, 6))
            out.append(max(1, m + int(rng.integers(-1, 2))))
        elif k == 2:
            out.append(int(rng.integers(1, hi)))
        elif k == 3:
            out.append(int(rng.integers(hi // 2, hi)))
        else:
            out.append(int(rng.integers(1, 700)))
    return np.array(out, dtype=np.int32)


def draw_geometry(rng):
    hkv = int(rng.choice([1, 2, 4, 8]))
    group = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16]))
    base_block = int(rng.choice([16, 16, 16, 32, 48]))
    layout = int(rng.integers(0, 2))
    p = int(rng.choice([d for d in (1, 2, 4, 8) if hkv % d == 0]))
    return hkv * group, hkv, base_block, (layout, p, int(rng.integers(0, p)))


def check(got, want, what):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.3e}"


@pytest.fixture
def default_options():
    yield
    for k, v in {"heads_per_wave": 0, "merge_mode": 0, "chunk_tokens": 0, "xcd_skew": -1, "piece_cost": -1}.items():
        kv.kv_set_option(k, v)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_decode_cases(seed, default_options):
    rng = np.random.default_rng(seed)
    for it in range(25):
        hq, hkv, bb, triple = draw_geometry(rng)
        batch = int(rng.integers(1, 25))
        ctx = draw_lens(rng, batch, int(rng.choice([300, 1500, 5000])))
        if rng.integers(0, 5) == 0:
            ctx[int(rng.integers(0, batch))] = 0          # an empty context among the others
        opts = {"heads_per_wave": int(rng.integers(0, 2)), "merge_mode": int(rng.integers(0, 3)),
                "chunk_tokens": int(rng.choice([0, 0, 0, 64, 128, 512])),
                "xcd_skew": int(rng.choice([-1, 0, 64, 200])), "piece_cost": int(rng.choice([-1, 0, 8, 40]))}
        what = f"seed {seed} case {it}: hq {hq} hkv {hkv} block {bb} view {triple} ctx {ctx.tolist()} {opts}"
        w = wl.Workload("sweep", 40 + it, hq, hkv, 128, bb, batch, "x", ())
        c = make_case(w, triple, ctx)
        for k, v in opts.items():
            kv.kv_set_option(k, v)
        view = kv.kv_view_create(hq, hkv, 128, bb, *triple)
        out = kv.paged_decode_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                                   torch.from_numpy(c.ctx).to(DEV), view, max_ctx_len=int(ctx.max()))
        torch.cuda.synchronize()
        check(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)),
              oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx), what)


@pytest.mark.parametrize("seed", [21, 22])
def test_random_prefill_cases(seed):
    rng = np.random.default_rng(seed)
    for it in range(12):
        hq, hkv, bb, triple = draw_geometry(rng)
        batch = int(rng.integers(1, 9))
        ctx = draw_lens(rng, batch, int(rng.choice([300, 1500, 4000])))
        # whole prompt, one token, half, chunks that end inside tiles, none
        qlen = np.array([int(rng.choice([n, 1, max(1, n // 2), min(n, 33), min(n, 70), 0])) for n in ctx],
                        dtype=np.int32)
        if qlen.sum() == 0:
            qlen[0] = min(int(ctx[0]), 5)
        what = f"seed {seed} case {it}: hq {hq} hkv {hkv} block {bb} view {triple} ctx {ctx.tolist()} q {qlen.tolist()}"
        w = wl.Workload("sweep_prefill", 40 + it, hq, hkv, 128, bb, batch, "x", ())
        c = make_prefill_case(w, triple, ctx, qlen)
        view = kv.kv_view_create(hq, hkv, 128, bb, *triple)
        out = kv.paged_prefill_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                                    torch.from_numpy(c.ctx).to(DEV),
                                    torch.from_numpy(c.q_off.astype(np.int32)).to(DEV), view,
                                    max_ctx_len=int(ctx.max()), max_q_len=int(qlen.max()))
        torch.cuda.synchronize()
        check(bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)),
              oracle.paged_prefill(c.view, c.q, c.pool, c.table, c.ctx, c.q_off), what)


@pytest.mark.parametrize("seed", [31, 32])
def test_random_repack_then_append(seed):
    """Random pairs of views (layouts, degrees, ranks; 2 to 8 KV heads, head dims 64 and 128, base
    blocks of 12, 16 and 32 tokens): kv_repack must leave the pool byte for byte as the oracle's
    repack does, and kv_append through the destination view must then change exactly the rows of
    the new tokens, to exactly the oracle's bytes."""
    from helpers import geometry
    rng = np.random.default_rng(seed)
    for it in range(20):
        hkv, d = int(rng.choice([2, 4, 8])), int(rng.choice([64, 128]))
        bb = int(rng.choice([16, 16, 32, 12]))

        def draw_view():
            p = int(rng.choice([x for x in (1, 2, 4, 8) if hkv % x == 0]))
            return (int(rng.integers(0, 2)), p, int(rng.integers(0, p)))

        src_t, dst_t = draw_view(), draw_view()
        batch = int(rng.integers(1, 9))
        ctx = np.array([int(rng.choice([0, 1, bb, bb + 1, int(rng.integers(1, 900))])) for _ in range(batch)],
                       dtype=np.int32)
        what = f"seed {seed} case {it}: hkv {hkv} d {d} block {bb} {src_t} -> {dst_t} ctx {ctx.tolist()}"
        w = wl.Workload("sweep_repack", 80 + it % 10, 2 * hkv, hkv, d, bb, batch, "x", ())
        geom = geometry(w)
        sv, dv = oracle.View(geom, *src_t), oracle.View(geom, *dst_t)
        K, V = wl.logical_kv(w, ctx)
        n_pool = 700
        perm = torch.randperm(n_pool, generator=wl.generator(w.index, wl.SUB_PERM)).numpy().astype(np.int32)
        t_src, used = wl.assign_blocks(ctx, sv.query()["block_tokens"], perm)
        t_dst, _ = wl.assign_blocks(ctx + 1, dv.query()["block_tokens"], perm[used:])
        pool = wl.poisoned_pool(n_pool, sv.query()["block_bytes"] // 2)
        off = wl.seq_offsets(ctx)
        oracle.scatter(sv, pool, t_src, ctx, off, K, V)
        dpool = dev_u16(pool)
        gs = kv.kv_view_create(2 * hkv, hkv, d, bb, *src_t)
        gd = kv.kv_view_create(2 * hkv, hkv, d, bb, *dst_t)
        ts, td = torch.from_numpy(t_src).to(DEV), torch.from_numpy(t_dst).to(DEV)
        n = torch.from_numpy(ctx).to(DEV)
        assert kv.kv_validate_tables(gs, n_pool, ts, n, gd, td) == kv.KV_OK, what
        kv.kv_repack(dpool, gs, gd, ts, td, n, int(ctx.max()))
        oracle.repack(sv, dv, pool, t_src, t_dst, ctx)
        torch.cuda.synchronize()
        assert np.array_equal(dpool.cpu().numpy().view(np.uint16), pool), "repack, " + what

        info = dv.query()
        h0, hl = info["kv_head0"], info["n_kv_local"]
        k_new = wl.randn_bf16((batch, hl, d), wl.generator(71, it))
        v_new = wl.randn_bf16((batch, hl, d), wl.generator(72, it))
        kv.kv_append(dpool, gd, dev_u16(k_new), dev_u16(v_new), td, n)
        # the rows an append may touch: where the oracle's scatter of ctx + 1 tokens differs from
        # its scatter of the first ctx of them
        off2 = wl.seq_offsets(ctx + 1)
        K2 = np.zeros((int(off2[-1]), hkv, d), dtype=np.uint16)
        V2 = np.zeros_like(K2)
        for s in range(batch):
            K2[off2[s]:off2[s] + ctx[s]] = K[off[s]:off[s + 1]]
            V2[off2[s]:off2[s] + ctx[s]] = V[off[s]:off[s + 1]]
            K2[off2[s + 1] - 1, h0:h0 + hl] = k_new[s]
            V2[off2[s + 1] - 1, h0:h0 + hl] = v_new[s]
        with_new = pool.copy()
        oracle.scatter(dv, with_new, t_dst, ctx + 1, off2, K2, V2)
        without = pool.copy()
        oracle.scatter(dv, without, t_dst, ctx, off, K, V)
        new_rows = with_new != without
        expected = pool.copy()
        expected[new_rows] = with_new[new_rows]
        torch.cuda.synchronize()
        assert np.array_equal(dpool.cpu().numpy().view(np.uint16), expected), "append, " + what


@pytest.mark.parametrize("seed", [41])
def test_random_linear_views(seed):
    """Random weight views (fused QKV slices of random head geometries, row and column shards of plain
    weights), batch sizes around the 64-row tile, 1 to 17 slabs of the input dimension, forced and
    automatic cuts of it, padded leading dimensions of x and of the stored weight."""
    from oracle import weights as ow
    rng = np.random.default_rng(seed)
    try:
        for it in range(40):
            M = int(rng.choice([1, 3, 16, 17, 63, 64, 65, 100, 128, 200, 256, 300]))
            slabs = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17]))
            kind = int(rng.integers(0, 3))
            splits = int(rng.choice([0, 0, 0, 1, 2, 3, 7, 16]))
            if kind == 0:
                hkv, group, d = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 4, 8])), int(rng.choice([64, 128]))
                hq, hidden = hkv * group, 128 * slabs
                m = int(rng.choice([x for x in (1, 2, 4, 8) if hkv % x == 0]))
                r = int(rng.integers(0, m))
                if (hq // m) * d % 64 or (hkv // m) * d % 64:
                    continue                      # segments must be whole 64-row tiles
                ov = ow.weight_view_fused_qkv(hq, hkv, d, hidden, r, m)
                gv = kv.kv_weight_view_fused_qkv(hq, hkv, d, hidden, r, m)
                n_rows, n_cols = (hq + 2 * hkv) * d, hidden
            else:
                n_out, dim = 64 * int(rng.integers(1, 9)), kind - 1
                m = int(rng.choice([1, 2, 4]))
                r = int(rng.integers(0, m))
                n_rows, n_cols = (n_out * m, 128 * slabs) if dim == 0 else (n_out, 128 * slabs * m)
                ov = ow.weight_view(dim, r, m, n_rows, n_cols)
                gv = kv.kv_weight_view_make(dim, r, m, n_rows, n_cols)
            pad = int(rng.choice([0, 8, 64]))
            what = f"seed {seed} case {it}: M {M} kind {kind} rows {n_rows} cols {n_cols} {r}/{m} splits {splits} pad {pad}"
            kv.kv_set_option("linear_splits", splits)
            w = wl.randn_bf16((n_rows, n_cols + pad), wl.generator(70, 100 + it))
            xw = wl.randn_bf16((M, ov.col_count + pad), wl.generator(70, 500 + it))
            dw = torch.from_numpy(w.view(np.int16)).to(DEV).view(torch.bfloat16)[:, :n_cols]
            dx = torch.from_numpy(xw.view(np.int16)).to(DEV).view(torch.bfloat16)[:, :ov.col_count]
            y = kv.kv_linear_view(dx, dw, gv)
            torch.cuda.synchronize()
            got = bf16_bits_to_f64(y.cpu().view(torch.int16).numpy().view(np.uint16))
            xs, wsl = np.ascontiguousarray(xw[:, :ov.col_count]), np.ascontiguousarray(w[:, :n_cols])
            want = ow.linear_view(xs, wsl, ov)
            tol = linear_tolerance(xs, wsl, ov, want)
            assert np.isfinite(got).all() and not (np.abs(got - want) > tol).any(), what
    finally:
        kv.kv_set_option("linear_splits", 0)
