"""Device-side set-up of the named workloads, shared by bench.py and the full-size GPU tests so
that both run the same launch configuration.  Plumbing only: draws the seeded inputs, puts
them in HBM and calls the library through the binding."""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from . import binding as kv
from . import workloads as wl


@dataclass
class DecodeCase:
    workload: wl.Workload
    triple: tuple
    view: kv.KVView
    ctx: np.ndarray                 # int32[batch] (host copy)
    max_ctx: int
    tables: List[np.ndarray]        # one per pool copy (host)
    q: torch.Tensor                 # bf16 [batch][n_q_local][d]
    pools: List[torch.Tensor]       # bf16 [n_blocks][block_elems], independent copies
    tables_dev: List[torch.Tensor]
    ctx_dev: torch.Tensor
    out: torch.Tensor
    workspace: torch.Tensor
    kv_bytes: int                   # algorithmic K+V bytes of one call

    def run(self, i: int = 0) -> torch.Tensor:
        k = i % len(self.pools)
        return kv.paged_decode_attn(self.q, self.pools[k], self.tables_dev[k], self.ctx_dev, self.view,
                                    self.max_ctx, out=self.out, workspace=self.workspace)

    def prepared(self):
        """run(i) with the argument marshalling done once (keeps the Python cost of a step to
        one foreign call, so that short kernels are not timed behind the interpreter)."""
        import ctypes as C
        fn = kv.lib().paged_decode_attn
        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        n_blocks = [p.numel() * 2 // self.view.block_bytes for p in self.pools]
        packs = [(C.c_void_p(self.q.data_ptr()), C.c_void_p(self.out.data_ptr()),
                  C.c_void_p(self.pools[k].data_ptr()), n_blocks[k],
                  C.c_void_p(self.tables_dev[k].data_ptr()), self.tables_dev[k].stride(0),
                  C.c_void_p(self.ctx_dev.data_ptr()), len(self.ctx), self.max_ctx, self.view.handle,
                  C.c_float(0.0), C.c_void_p(self.workspace.data_ptr()), self.workspace.numel(), stream)
                 for k in range(len(self.pools))]

        def run(i: int = 0):
            rc = fn(*packs[i % len(packs)])
            if rc != 0:
                raise kv.KVError(rc, "paged_decode_attn")
        return run


def random_pool(n_blocks: int, block_elems: int, seed: int, device) -> torch.Tensor:
    """A pool filled with bf16 N(0,1), drawn on the device from a seeded generator."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    pool = torch.empty((n_blocks, block_elems), dtype=torch.bfloat16, device=device)
    step = max(1, (1 << 27) // block_elems)
    for a in range(0, n_blocks, step):
        b = min(n_blocks, a + step)
        pool[a:b] = torch.randn((b - a, block_elems), generator=g, device=device,
                                dtype=torch.float32).to(torch.bfloat16)
    return pool


def make_view(w: wl.Workload, triple) -> kv.KVView:
    return kv.kv_view_create(w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size, *triple)


def build_decode_case(w: wl.Workload, triple, device="cuda:0", n_copies: int = 1,
                      slack: float = 1.2) -> DecodeCase:
    """Context lengths by the workload's recipe; block table = the next ids of a shuffled pool
    sized ``slack`` x the blocks needed; pool contents N(0,1) everywhere (timing recipe)."""
    view = make_view(w, triple)
    ctx = wl.draw_ctx_lens(w)
    need = int(wl.blocks_needed(ctx, view.block_tokens).sum())
    q_full = wl.queries(w)
    lo = view.rank * view.n_q_local
    q = torch.from_numpy(np.ascontiguousarray(q_full[:, lo:lo + view.n_q_local]).view(np.int16)) \
        .to(device).view(torch.bfloat16)
    pools, tables, tables_dev = [], [], []
    block_elems = view.block_bytes // 2
    for k in range(n_copies):
        g = wl.generator(w.index, wl.SUB_PERM + 100 * (k + 1))
        perm = wl.shuffled_pool(need, slack, g)
        table, _ = wl.assign_blocks(ctx, view.block_tokens, perm)
        tables.append(table)
        tables_dev.append(torch.from_numpy(table).to(device))
        pools.append(random_pool(len(perm), block_elems,
                                 wl.SEED_BASE + 10 * w.index + wl.SUB_DATA + 1000 * (k + 1), device))
    max_ctx = int(ctx.max())
    ws_bytes = kv.paged_decode_attn_workspace_bytes(view, len(ctx), max_ctx)
    workspace = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device=device)
    kv_bytes = int(ctx.astype(np.int64).sum()) * view.n_kv_local * view.head_dim * 2 * 2
    return DecodeCase(w, tuple(triple), view, ctx, max_ctx, tables, q, pools, tables_dev,
                      torch.from_numpy(ctx).to(device),
                      torch.empty_like(q), workspace, kv_bytes)


@dataclass
class MixedCase:
    views: list
    ctx: np.ndarray
    q: torch.Tensor
    out: torch.Tensor
    pool: torch.Tensor
    table_dev: torch.Tensor
    ctx_dev: torch.Tensor
    ids_dev: torch.Tensor
    workspace: torch.Tensor
    kv_bytes: int

    def run(self, i: int = 0) -> None:
        kv.paged_decode_attn_mixed(self.q, self.pool, self.table_dev, self.ctx_dev, self.ids_dev, self.views,
                                   int(self.ctx.max()), out=self.out, workspace=self.workspace)


def build_mixed_case(w: wl.Workload, p: int, r: int, device="cuda:0", slack: float = 1.2) -> MixedCase:
    """The workload's batch with every other sequence stored in DP-layout blocks (read through rank
    r's alias view) and the rest in the TP layout of degree p: one pool, one table."""
    views = [make_view(w, (kv.KV_LAYOUT_TP, p, r)), make_view(w, (kv.KV_LAYOUT_DP, p, r))]
    ctx = wl.draw_ctx_lens(w)
    ids = (np.arange(len(ctx)) % 2).astype(np.int32)
    caps = np.where(ids == 0, views[0].block_tokens, views[1].block_tokens).astype(np.int64)
    need = (ctx.astype(np.int64) + caps - 1) // caps
    perm = wl.shuffled_pool(int(need.sum()), slack, wl.generator(w.index, wl.SUB_PERM + 500))
    cols = max(int(need.max()), (int(ctx.max()) + int(caps.min()) - 1) // int(caps.min()))
    table = np.full((len(ctx), cols), -1, dtype=np.int32)
    used = 0
    for s, k in enumerate(need):
        table[s, :k] = perm[used:used + int(k)]
        used += int(k)
    pool = random_pool(len(perm), views[0].block_bytes // 2, wl.SEED_BASE + 10 * w.index + wl.SUB_DATA + 5000, device)
    q_full = wl.queries(w)
    lo = r * views[0].n_q_local
    q = torch.from_numpy(np.ascontiguousarray(q_full[:, lo:lo + views[0].n_q_local]).view(np.int16)) \
        .to(device).view(torch.bfloat16)
    ws = torch.zeros(max(kv.paged_decode_attn_workspace_bytes(views[0], len(ctx), int(ctx.max())), 256),
                     dtype=torch.uint8, device=device)
    kv_bytes = int(ctx.astype(np.int64).sum()) * views[0].n_kv_local * views[0].head_dim * 2 * 2
    return MixedCase(views, ctx, q, torch.empty_like(q), pool, torch.from_numpy(table).to(device),
                     torch.from_numpy(ctx).to(device), torch.from_numpy(ids).to(device), ws, kv_bytes)


@dataclass
class PrefillCase:
    view: kv.KVView
    ctx: np.ndarray
    q_lens: np.ndarray
    q: torch.Tensor
    out: torch.Tensor
    pool: torch.Tensor
    table_dev: torch.Tensor
    ctx_dev: torch.Tensor
    q_off_dev: torch.Tensor
    flops: float                    # 4 * head_dim * n_q_local * (unmasked query-key pairs)
    kv_bytes: int                   # K and V of the cached tokens, read once

    def run(self, i: int = 0) -> None:
        kv.paged_prefill_attn(self.q, self.pool, self.table_dev, self.ctx_dev, self.q_off_dev, self.view,
                              int(self.ctx.max()), int(self.q_lens.max()), out=self.out)


def build_prefill_case(w: wl.Workload, triple, ctx, q_lens, device="cuda:0", slack: float = 1.2) -> PrefillCase:
    """Sequences with ctx[s] cached tokens of which the last q_lens[s] are queried; random pool,
    shuffled block table, bf16 N(0,1) queries (timing recipe)."""
    view = make_view(w, triple)
    ctx = np.asarray(ctx, dtype=np.int32)
    q_lens = np.asarray(q_lens, dtype=np.int32)
    need = int(wl.blocks_needed(ctx, view.block_tokens).sum())
    perm = wl.shuffled_pool(need, slack, wl.generator(w.index, wl.SUB_PERM + 300))
    table, _ = wl.assign_blocks(ctx, view.block_tokens, perm)
    pool = random_pool(len(perm), view.block_bytes // 2, wl.SEED_BASE + 10 * w.index + wl.SUB_DATA + 3000, device)
    q_off = wl.seq_offsets(q_lens)
    g = torch.Generator(device=device)
    g.manual_seed(wl.SEED_BASE + 10 * w.index + wl.SUB_QUERY + 3000)
    q = torch.randn((int(q_off[-1]), view.n_q_local, view.head_dim), generator=g, device=device,
                    dtype=torch.float32).to(torch.bfloat16)
    n, m = ctx.astype(np.float64), q_lens.astype(np.float64)
    pairs = float((m * (n - m) + m * (m + 1) / 2).sum())
    return PrefillCase(view, ctx, q_lens, q, torch.empty_like(q), pool, torch.from_numpy(table).to(device),
                       torch.from_numpy(ctx).to(device), torch.from_numpy(q_off.astype(np.int32)).to(device),
                       4.0 * view.head_dim * view.n_q_local * pairs,
                       int(ctx.astype(np.int64).sum()) * view.n_kv_local * view.head_dim * 2 * 2)


@dataclass
class RepackCase:
    workload: wl.Workload
    src_view: kv.KVView
    dst_view: kv.KVView
    n_tokens: np.ndarray
    max_tokens: int
    pool: torch.Tensor
    src_table: np.ndarray
    dst_table: np.ndarray
    back_table: np.ndarray
    src_dev: torch.Tensor
    dst_dev: torch.Tensor
    back_dev: torch.Tensor
    n_dev: torch.Tensor
    moved_bytes: int                # payload bytes one direction moves (read == written)

    def forward(self):
        kv.kv_repack(self.pool, self.src_view, self.dst_view, self.src_dev, self.dst_dev, self.n_dev,
                     self.max_tokens)

    def backward(self):
        kv.kv_repack(self.pool, self.dst_view, self.src_view, self.dst_dev, self.back_dev, self.n_dev,
                     self.max_tokens)


def build_repack_case(w: wl.Workload, src_triple, dst_triple, n_tokens: Optional[np.ndarray] = None,
                      device="cuda:0", slack: float = 1.2) -> RepackCase:
    """src blocks -> dst blocks -> fresh src-layout blocks, all out of one shuffled pool sized
    ``slack`` x the three block sets."""
    sv, dv = make_view(w, src_triple), make_view(w, dst_triple)
    n_tokens = wl.draw_ctx_lens(w) if n_tokens is None else np.asarray(n_tokens, dtype=np.int32)
    need_s = int(wl.blocks_needed(n_tokens, sv.block_tokens).sum())
    need_d = int(wl.blocks_needed(n_tokens, dv.block_tokens).sum())
    perm = wl.shuffled_pool(2 * need_s + need_d, slack, wl.generator(w.index, wl.SUB_PERM + 7))
    t_src, u1 = wl.assign_blocks(n_tokens, sv.block_tokens, perm)
    t_dst, u2 = wl.assign_blocks(n_tokens, dv.block_tokens, perm[u1:])
    t_back, _ = wl.assign_blocks(n_tokens, sv.block_tokens, perm[u1 + u2:])
    pool = random_pool(len(perm), sv.block_bytes // 2, wl.SEED_BASE + 10 * w.index + 77, device)
    lo = max(sv.kv_head0, dv.kv_head0)
    hi = min(sv.kv_head0 + sv.n_kv_local, dv.kv_head0 + dv.n_kv_local)
    moved = int(n_tokens.astype(np.int64).sum()) * max(hi - lo, 0) * w.head_dim * 2 * 2
    return RepackCase(w, sv, dv, n_tokens, int(n_tokens.max()), pool, t_src, t_dst, t_back,
                      torch.from_numpy(t_src).to(device), torch.from_numpy(t_dst).to(device),
                      torch.from_numpy(t_back).to(device), torch.from_numpy(n_tokens).to(device), moved)


def time_calls(fn, steps: int, warmup: int) -> float:
    """Milliseconds per call: ``warmup`` untimed calls, then ``steps`` calls between two events
    recorded on torch's current stream (the stream the binding launches on)."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps
