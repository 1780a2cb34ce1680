"""Shared test scaffolding: builds seeded cases on the CPU with the oracle.

Everything here is host-side numpy.  Pools are filled with ``oracle.scatter`` (or, where a
test wants independence from it, with numpy reshapes), so the GPU path never produces an
input or an expected value.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

import oracle
from paper_2602_22593_amd import workloads as wl


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64, exact."""
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def geometry(w: wl.Workload) -> oracle.Geometry:
    return oracle.Geometry(w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size)


@dataclass
class Case:
    w: wl.Workload
    geom: oracle.Geometry
    view: oracle.View
    info: dict
    ctx: np.ndarray          # int32[batch]
    seq_off: np.ndarray      # int64[batch+1]
    K: np.ndarray            # uint16[total][Hkv][d]
    V: np.ndarray
    q_full: np.ndarray       # uint16[batch][Hq][d]
    q: np.ndarray            # uint16[batch][Hql][d]  (rank's slice)
    table: np.ndarray        # int32[batch][cols]
    pool: np.ndarray         # uint16[n_blocks][block_elems]


def q_slice(q_full: np.ndarray, info: dict, rank: int) -> np.ndarray:
    """Query heads of rank r: the contiguous range [r*Hql, (r+1)*Hql) (paper Sec. 4.1.1)."""
    hql = info["n_q_local"]
    return np.ascontiguousarray(q_full[:, rank * hql:(rank + 1) * hql, :])


def make_case(w: wl.Workload, view_triple, ctx: Optional[np.ndarray] = None, slack: float = 1.2,
              n_pool_blocks: Optional[int] = None, K=None, V=None, q_full=None) -> Case:
    geom = geometry(w)
    view = oracle.View(geom, *view_triple)
    info = view.query()
    ctx = wl.draw_ctx_lens(w) if ctx is None else np.asarray(ctx, dtype=np.int32)
    w_eff = w if len(ctx) == w.batch else wl.Workload(w.name, w.index, w.n_q_heads, w.n_kv_heads,
                                                       w.head_dim, w.base_block_size, len(ctx),
                                                       w.lengths, w.views)
    if K is None:
        K, V = wl.logical_kv(w_eff, ctx)
    if q_full is None:
        q_full = wl.queries(w_eff)
    need = int(wl.blocks_needed(ctx, info["block_tokens"]).sum())
    g = wl.generator(w.index, wl.SUB_PERM)
    if n_pool_blocks is None:
        perm = wl.shuffled_pool(max(need, 1), slack, g)
    else:
        import torch
        perm = torch.randperm(n_pool_blocks, generator=g).numpy().astype(np.int32)
    table, _ = wl.assign_blocks(ctx, info["block_tokens"], perm)
    pool = wl.poisoned_pool(len(perm), info["block_bytes"] // 2)
    seq_off = wl.seq_offsets(ctx)
    oracle.scatter(view, pool, table, ctx, seq_off, K, V)
    return Case(w_eff, geom, view, info, ctx, seq_off, K, V, q_full,
                q_slice(q_full, info, view.rank), table, pool)


@dataclass
class MixedCase:
    w: wl.Workload
    views: list              # oracle.View per layout
    view_ids: np.ndarray     # int32[batch]
    ctx: np.ndarray
    seq_off: np.ndarray
    K: np.ndarray
    V: np.ndarray
    q_full: np.ndarray
    q: np.ndarray            # the rank's query heads (same for every view)
    table: np.ndarray        # row s indexed with the block capacity of sequence s's view
    pool: np.ndarray


def make_mixed_case(w: wl.Workload, triples, view_ids, ctx, slack: float = 1.3) -> MixedCase:
    """One pool in which sequence s is stored under ``triples[view_ids[s]]`` (all with the same TP
    degree and rank); NaN-poisoned wherever no valid token lies."""
    geom = geometry(w)
    views = [oracle.View(geom, *t) for t in triples]
    infos = [v.query() for v in views]
    ctx = np.asarray(ctx, dtype=np.int32)
    view_ids = np.asarray(view_ids, dtype=np.int32)
    w_eff = wl.Workload(w.name, w.index, w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size,
                        len(ctx), w.lengths, w.views)
    K, V = wl.logical_kv(w_eff, ctx)
    q_full = wl.queries(w_eff)
    caps = np.array([infos[k]["block_tokens"] for k in view_ids], dtype=np.int64)
    need = (ctx.astype(np.int64) + caps - 1) // caps
    perm = wl.shuffled_pool(max(int(need.sum()), 1), slack, wl.generator(w.index, wl.SUB_PERM))
    # wide enough for the longest sequence under the smallest capacity (what the ABI asks for)
    min_cap = min(i["block_tokens"] for i in infos)
    cols = max(int(need.max()), (int(ctx.max()) + min_cap - 1) // min_cap, 1)
    table = np.full((len(ctx), cols), -1, dtype=np.int32)
    used = 0
    for s, k in enumerate(need):
        table[s, :k] = perm[used:used + int(k)]
        used += int(k)
    pool = wl.poisoned_pool(len(perm), infos[0]["block_bytes"] // 2)
    seq_off = wl.seq_offsets(ctx)
    for k, v in enumerate(views):
        oracle.scatter(v, pool, table, np.where(view_ids == k, ctx, 0).astype(np.int32), seq_off, K, V)
    return MixedCase(w_eff, views, view_ids, ctx, seq_off, K, V, q_full,
                     q_slice(q_full, infos[0], views[0].rank), table, pool)


@dataclass
class PrefillCase:
    w: wl.Workload
    view: oracle.View
    info: dict
    ctx: np.ndarray          # int32[batch] tokens in the cache (the new ones included)
    q_lens: np.ndarray       # int32[batch] new tokens = last q_lens[s] of the ctx[s]
    q_off: np.ndarray        # int64[batch+1]
    seq_off: np.ndarray
    K: np.ndarray
    V: np.ndarray
    q_full: np.ndarray       # uint16[total_q][Hq][d]
    q: np.ndarray            # uint16[total_q][Hql][d]
    table: np.ndarray
    pool: np.ndarray


def make_prefill_case(w: wl.Workload, view_triple, ctx, q_lens, slack: float = 1.2) -> PrefillCase:
    """Cached K/V for ctx[s] tokens per sequence (scattered through the view into a NaN-poisoned
    pool) and q_lens[s] <= ctx[s] query tokens per sequence, all bf16 N(0,1), seeded."""
    geom = geometry(w)
    view = oracle.View(geom, *view_triple)
    info = view.query()
    ctx = np.asarray(ctx, dtype=np.int32)
    q_lens = np.asarray(q_lens, dtype=np.int32)
    assert (q_lens <= ctx).all() and (q_lens >= 0).all()
    w_eff = wl.Workload(w.name, w.index, w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size,
                        len(ctx), w.lengths, w.views)
    K, V = wl.logical_kv(w_eff, ctx)
    q_off = wl.seq_offsets(q_lens)
    q_full = wl.randn_bf16((int(q_off[-1]), w.n_q_heads, w.head_dim), wl.generator(w.index, wl.SUB_QUERY))
    need = int(wl.blocks_needed(ctx, info["block_tokens"]).sum())
    perm = wl.shuffled_pool(max(need, 1), slack, wl.generator(w.index, wl.SUB_PERM))
    table, _ = wl.assign_blocks(ctx, info["block_tokens"], perm)
    pool = wl.poisoned_pool(len(perm), info["block_bytes"] // 2)
    seq_off = wl.seq_offsets(ctx)
    oracle.scatter(view, pool, table, ctx, seq_off, K, V)
    return PrefillCase(w_eff, view, info, ctx, q_lens, q_off, seq_off, K, V, q_full,
                       q_slice(q_full, info, view.rank), table, pool)


def textbook_causal_attention(c: PrefillCase, scale: float) -> np.ndarray:
    """softmax(mask(scale * Q K^T)) V per sequence and head with numpy matrix products, fp64, on
    the logical tensors: Q rows are the sequence's last q_len tokens, the mask keeps key t for the
    query at position pos iff t <= pos.  out[total_q][Hq][d]."""
    hq, hkv, d = c.w.n_q_heads, c.w.n_kv_heads, c.w.head_dim
    G = hq // hkv
    qf, Kf, Vf = bf16_bits_to_f64(c.q_full), bf16_bits_to_f64(c.K), bf16_bits_to_f64(c.V)
    out = np.zeros((int(c.q_off[-1]), hq, d))
    for s in range(len(c.ctx)):
        n, m = int(c.ctx[s]), int(c.q_lens[s])
        if m == 0:
            continue
        a, qa = int(c.seq_off[s]), int(c.q_off[s])
        pos = np.arange(n - m, n)[:, None]
        keep = np.arange(n)[None, :] <= pos
        for h in range(hq):
            S = (qf[qa:qa + m, h, :] @ Kf[a:a + n, h // G, :].T) * scale
            S = np.where(keep, S, -np.inf)
            P = np.exp(S - S.max(axis=1, keepdims=True))
            P /= P.sum(axis=1, keepdims=True)
            out[qa:qa + m, h, :] = P @ Vf[a:a + n, h // G, :]
    return out


def textbook_attention(q_full: np.ndarray, K: np.ndarray, V: np.ndarray, seq_off: np.ndarray,
                       n_q_heads: int, n_kv_heads: int, scale: float) -> np.ndarray:
    """softmax(scale * q K^T) V per sequence and head with numpy matmuls, fp64.

    The textbook single-query attention on the logical (un-paged) tensors; query head h
    reads KV head h // (Hq // Hkv).
    """
    batch, hq, d = q_full.shape
    G = n_q_heads // n_kv_heads
    qf = bf16_bits_to_f64(q_full)
    Kf = bf16_bits_to_f64(K)
    Vf = bf16_bits_to_f64(V)
    out = np.zeros((batch, hq, d))
    for s in range(batch):
        a, b = int(seq_off[s]), int(seq_off[s + 1])
        if b == a:
            continue
        for h in range(hq):
            g = h // G
            logits = (Kf[a:b, g, :] @ qf[s, h, :]) * scale
            p = np.exp(logits - logits.max())
            p = p / p.sum()
            out[s, h, :] = p @ Vf[a:b, g, :]
    return out


def linear_tolerance(x_bits: np.ndarray, w_bits: np.ndarray, view, want: np.ndarray) -> np.ndarray:
    """Per-output bound on |bf16(fp32-accumulated x W^T) - exact| for ``oracle.weights.linear_view``
    results ``want`` (fp64) on the weight view ``view``.

    Error model.  The inputs are exact in fp32 and every product of two bf16 values is exact in
    fp32, so the only errors are the K - 1 roundings of the running sums (unit roundoff
    u = 2^-24, whatever the order of summation) and the final rounding to bf16.  The a-priori
    worst case for the first is K u S with S = sum_k |x_k w_k|; rounding errors of a sum behave
    like independent zero-mean perturbations, for which the bound lambda sqrt(K) u S holds with
    overwhelming probability (Higham & Mary, "A new approach to probabilistic rounding error
    analysis", 2019); lambda = 4 here.  S is computed exactly for each output (the same product on
    the absolute values).  The final rounding adds half a bf16 ulp of the computed value, at most
    2^-8 of its magnitude.  At K = 4096 with N(0,1) data the accumulation term is about 0.04 on
    outputs of standard deviation 64, against 0.25 for the output rounding: one dropped product
    (typical magnitude 0.6, often above 2) moves an output well outside the bound.
    """
    from oracle import weights as ow
    K = view.col_count
    mask = np.uint16(0x7FFF)
    S = ow.linear_view(x_bits & mask, w_bits & mask, view)
    acc = 4.0 * np.sqrt(K) * 2.0 ** -24 * S
    return (np.abs(want) + acc) * 2.0 ** -8 + acc + 1e-30
