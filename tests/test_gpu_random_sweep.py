"""Seeded random sweep of paged_decode_attn and paged_prefill_attn against the oracle.

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

from helpers import bf16_bits_to_f64, make_case, make_prefill_case

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
    for k, v in {"variant": 0, "chunk_tokens": 0, "xcd_skew": -1, "piece_cost": -1}.items():
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
        opts = {"variant": int(rng.integers(0, 8)), "chunk_tokens": int(rng.choice([0, 0, 0, 64, 128, 512])),
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
