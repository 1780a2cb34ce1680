"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle.

This module draws random numbers and lays out bookkeeping arrays; it contains
none of the method's arithmetic (no address function, no attention, no head
partition).  Whoever calls it passes in the view-dependent integers it needs
(tokens per block under a view), obtained from the library under test or from
the oracle, each through its own code.

Shapes follow the decode workloads the paper's setting implies (Sec. 6.1.3:
prompts uniform in [128, 4000] tokens plus up to 512 generated tokens; Sec. 6.5:
contexts of 128K tokens and beyond) at Llama-3-8B / 70B attention geometry.
The datasets the paper samples request text from are not needed: this path
consumes only shapes and lengths.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np
import torch

BF16_NAN = 0x7FC0  # quiet NaN bit pattern, used to poison bytes that must never be read
SEED_BASE = 2259300

SUB_LENGTHS, SUB_PERM, SUB_DATA, SUB_QUERY, SUB_MISC = 1, 2, 3, 4, 5


@dataclass(frozen=True)
class Workload:
    """One named configuration: attention geometry, batch and the context-length recipe."""
    name: str
    index: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    base_block_size: int
    batch: int
    lengths: str                       # recipe id, see draw_ctx_lens
    # (layout, tp_degree, rank) triples this workload is evaluated under; layout 0 = DP, 1 = TP
    views: Tuple[Tuple[int, int, int], ...] = field(default_factory=tuple)


WORKLOADS = {
    w.name: w for w in (
        Workload("tiny", 0, 8, 2, 64, 16, 4, "tiny", ((0, 1, 0), (1, 2, 0), (1, 2, 1))),
        Workload("llama8b_dp_b64", 1, 32, 8, 128, 16, 64, "u512_4096", ((0, 1, 0),)),
        Workload("llama8b_tp_b128", 2, 32, 8, 128, 16, 128, "u256_8192",
                 ((1, 2, 0), (1, 4, 0), (1, 8, 0))),
        Workload("llama70b_tp8_b256", 3, 64, 8, 128, 16, 256, "lognormal2048", ((1, 8, 0),)),
        Workload("llama8b_tp4_longmix", 4, 32, 8, 128, 16, 8, "longmix", ((1, 4, 0),)),
    )
}


def generator(workload_index: int, substream: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(SEED_BASE + 10 * workload_index + substream)
    return g


def _uniform_int(lo: int, hi: int, n: int, g: torch.Generator) -> np.ndarray:
    """Integers uniform in [lo, hi], both ends included."""
    return torch.randint(lo, hi + 1, (n,), generator=g, dtype=torch.int64).numpy().astype(np.int32)


def draw_ctx_lens(w: Workload) -> np.ndarray:
    """Context lengths (tokens already in the cache) of the batch, int32[batch]."""
    g = generator(w.index, SUB_LENGTHS)
    if w.lengths == "tiny":
        return np.array([17, 64, 150, 300], dtype=np.int32)
    if w.lengths == "u512_4096":
        return _uniform_int(512, 4096, w.batch, g)
    if w.lengths == "u256_8192":
        return _uniform_int(256, 8192, w.batch, g)
    if w.lengths == "lognormal2048":
        z = torch.randn(w.batch, generator=g, dtype=torch.float64).numpy()
        n = np.rint(np.exp(math.log(2048.0) + 1.0 * z))
        return np.clip(n, 1, 16384).astype(np.int32)
    if w.lengths == "longmix":
        short = _uniform_int(1024, 8192, w.batch - 2, g)
        lens = np.concatenate([np.array([131072, 131072], dtype=np.int32), short])
        order = torch.randperm(w.batch, generator=g).numpy()
        return lens[order].astype(np.int32)
    raise ValueError(w.lengths)


def randn_bf16(shape, g: torch.Generator) -> np.ndarray:
    """N(0,1) drawn in fp32, rounded to bf16 (nearest even); returned as uint16 bit patterns."""
    x = torch.randn(*shape, generator=g, dtype=torch.float32).to(torch.bfloat16)
    return x.view(torch.int16).numpy().view(np.uint16).copy()


def blocks_needed(n_tokens: np.ndarray, block_tokens: int) -> np.ndarray:
    """Blocks a sequence occupies when one block holds ``block_tokens`` tokens."""
    n = np.asarray(n_tokens, dtype=np.int64)
    return ((n + block_tokens - 1) // block_tokens).astype(np.int64)


def assign_blocks(n_tokens: np.ndarray, block_tokens: int, free_ids: np.ndarray,
                  min_cols: int = 1) -> Tuple[np.ndarray, int]:
    """Hand the next ids of ``free_ids`` to each sequence in turn.

    Returns (table int32[n_seqs][cols] padded with -1, number of ids consumed).
    """
    need = blocks_needed(n_tokens, block_tokens)
    cols = max(int(need.max()) if need.size else 0, min_cols)
    table = np.full((len(need), cols), -1, dtype=np.int32)
    used = 0
    for s, k in enumerate(need):
        k = int(k)
        table[s, :k] = free_ids[used:used + k]
        used += k
    assert used <= len(free_ids), "pool too small for the requested tables"
    return table, used


def shuffled_pool(n_blocks_needed: int, slack: float, g: torch.Generator) -> np.ndarray:
    """A random permutation of the ids of a pool sized ``slack`` x the blocks needed."""
    n_pool = int(math.ceil(slack * n_blocks_needed))
    return torch.randperm(n_pool, generator=g).numpy().astype(np.int32)


def seq_offsets(n_tokens: np.ndarray) -> np.ndarray:
    """Exclusive prefix sum, int64[n_seqs + 1]: where each sequence starts in a flat token list."""
    off = np.zeros(len(n_tokens) + 1, dtype=np.int64)
    np.cumsum(np.asarray(n_tokens, dtype=np.int64), out=off[1:])
    return off


def logical_kv(w: Workload, n_tokens: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Logical K and V, uint16[total_tokens][n_kv_heads][head_dim], bf16 N(0,1)."""
    g = generator(w.index, SUB_DATA)
    total = int(np.sum(n_tokens))
    K = randn_bf16((total, w.n_kv_heads, w.head_dim), g)
    V = randn_bf16((total, w.n_kv_heads, w.head_dim), g)
    return K, V


def queries(w: Workload) -> np.ndarray:
    """q for all query heads, uint16[batch][n_q_heads][head_dim], bf16 N(0,1)."""
    return randn_bf16((w.batch, w.n_q_heads, w.head_dim), generator(w.index, SUB_QUERY))


def poisoned_pool(n_blocks: int, block_elems: int) -> np.ndarray:
    """A pool whose every element is a bf16 NaN: anything read but never written shows up."""
    return np.full((n_blocks, block_elems), BF16_NAN, dtype=np.uint16)
