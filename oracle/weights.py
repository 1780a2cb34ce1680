"""TEST INFRASTRUCTURE, NOT PRODUCT CODE: weight shard views and the linear layer on a view.

Plain numpy, fp64.  Follows the Model Weights Manager of the paper: Megatron-style sharding
(Sec. 4.1.1: the fused QKV projection is column-parallel, the output projection row-parallel)
realised as a zero-copy view of the full weight, W_active^(r) = View(W_full, dim, r, m) (Eq. 1).

Storage convention (this build's reading; the paper defers to the serving engine's linear layer): a
weight is stored [out_features][in_features], row-major, so a linear layer is y = x W^T.  Sharding
the *output* dimension (column-parallel in the paper's y = x W picture) selects stored ROWS; sharding
the *input* dimension (row-parallel) selects stored COLUMNS.  The fused QKV weight stacks
[Q heads | K heads | V heads] along the output dimension, head-major, head_dim rows per head; rank r
owns the same contiguous head range in each of the three parts (Sec. 4.1.1), i.e. three row
segments.
"""
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class WeightView:
    row_segments: Tuple[Tuple[int, int], ...]   # (first stored row, count), concatenated in order
    col_start: int
    col_count: int

    @property
    def n_rows(self) -> int:
        return sum(c for _, c in self.row_segments)

    def row_index(self) -> np.ndarray:
        return np.concatenate([np.arange(a, a + c) for a, c in self.row_segments]) if self.row_segments \
            else np.zeros(0, dtype=np.int64)


def weight_view(dim: int, r: int, m: int, n_rows: int, n_cols: int) -> WeightView:
    """Eq. 1: the r-th of m equal parts of a stored [n_rows][n_cols] weight along `dim`
    (0: stored rows = output features, 1: stored columns = input features)."""
    if m < 1 or not 0 <= r < m or dim not in (0, 1):
        raise ValueError("bad (dim, r, m)")
    if dim == 0:
        if n_rows % m:
            raise ValueError("rows not divisible")
        return WeightView(((r * (n_rows // m), n_rows // m),), 0, n_cols)
    if n_cols % m:
        raise ValueError("columns not divisible")
    return WeightView(((0, n_rows),), r * (n_cols // m), n_cols // m)


def weight_view_fused_qkv(n_q_heads: int, n_kv_heads: int, head_dim: int, hidden: int, r: int,
                          m: int) -> WeightView:
    """Rank r's slice of a fused [(Hq + 2 Hkv) d][hidden] QKV weight: its Hq/m query heads, its
    Hkv/m key heads and its Hkv/m value heads (contiguous head ranges, Sec. 4.1.1)."""
    if m < 1 or not 0 <= r < m or n_q_heads % m or n_kv_heads % m:
        raise ValueError("bad (r, m)")
    d, hq, hkv = head_dim, n_q_heads // m, n_kv_heads // m
    q0, k0, v0 = 0, n_q_heads * d, (n_q_heads + n_kv_heads) * d
    return WeightView(((q0 + r * hq * d, hq * d), (k0 + r * hkv * d, hkv * d), (v0 + r * hkv * d, hkv * d)),
                      0, hidden)


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def linear_view(x_bits: np.ndarray, w_full_bits: np.ndarray, view: WeightView) -> np.ndarray:
    """y[M][view.n_rows] fp64 = x W_active^T, W_active = the view's rows and columns of the full
    stored weight; x is [M][view.col_count] (bf16 bit patterns, as the weight)."""
    assert x_bits.shape[1] == view.col_count
    w = bf16_bits_to_f64(w_full_bits[view.row_index()][:, view.col_start:view.col_start + view.col_count])
    return bf16_bits_to_f64(x_bits) @ w.T
