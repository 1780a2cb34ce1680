"""CPU fp64 oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

ctypes front end of ``flying_oracle.c``: the plain definition of paged decode
attention through the KV Cache Adaptor's layout views (paper Sec. 4.2.2,
Eq. 2-3; Alg. 1 step 4 / Eq. 4), of logical<->pool scatter / gather and of the
byte-exact repack between two views.  Only ``tests/``, the smoke check and the
CPU-baseline leg of the benchmark may import this package; it imports nothing
from the HIP package and the HIP package imports nothing from here.

Arrays are numpy: bf16 tensors travel as ``uint16`` bit patterns, tables and
lengths as ``int32``, results as ``float64``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flying_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

LAYOUT_DP = 0
LAYOUT_TP = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (host only). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_elem_index.restype = C.c_int64
    return _lib


@dataclass(frozen=True)
class Geometry:
    """Model-side constants: query heads, KV heads, head dim, B_base (Alg. 1 'Require')."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    base_block_size: int


@dataclass(frozen=True)
class View:
    """(layout, TP degree p, rank r) over a geometry."""
    geom: Geometry
    layout: int
    tp_degree: int = 1
    rank: int = 0

    def _args(self):
        g = self.geom
        return [C.c_int32(x) for x in (g.n_q_heads, g.n_kv_heads, g.head_dim, g.base_block_size,
                                       self.layout, self.tp_degree, self.rank)]

    def query(self) -> dict:
        out = (C.c_int64 * 10)()
        rc = lib().oracle_view_query(*self._args(), out)
        if rc:
            raise ValueError(f"invalid view {self}")
        keys = ("block_tokens", "row_heads", "n_kv_local", "n_q_local", "kv_head0", "row_head0",
                "plane_elems", "block_bytes", "token_stride_elems", "group")
        return dict(zip(keys, [int(x) for x in out]))


def _p(a: np.ndarray, dtype):
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype, a.flags["C_CONTIGUOUS"])
    return a.ctypes.data_as(C.c_void_p)


def elem_index(view: View, blk: int, plane: int, slot: int, hl: int, e: int) -> int:
    return int(lib().oracle_elem_index(*view._args(), C.c_int64(blk), C.c_int32(plane),
                                       C.c_int32(slot), C.c_int32(hl), C.c_int32(e)))


def paged_decode(view: View, q, pool, table, ctx_lens, scale: float = 0.0) -> np.ndarray:
    """out[batch][Hql][d] fp64 = softmax(scale * q K^T) V through the view."""
    info = view.query()
    batch = int(ctx_lens.shape[0])
    d = view.geom.head_dim
    assert q.shape == (batch, info["n_q_local"], d), q.shape
    table = np.ascontiguousarray(table, dtype=np.int32).reshape(batch, -1)
    out = np.empty((batch, info["n_q_local"], d), dtype=np.float64)
    rc = lib().oracle_paged_decode(*view._args(), _p(q, np.uint16), _p(pool.reshape(-1), np.uint16),
                                   _p(table, np.int32), C.c_int64(table.shape[1]),
                                   _p(ctx_lens, np.int32), C.c_int32(batch), C.c_double(scale),
                                   _p(out, np.float64))
    if rc:
        raise ValueError(f"oracle_paged_decode rc={rc}")
    return out


def paged_decode_mixed(views, view_ids, q, pool, table, ctx_lens, scale: float = 0.0) -> np.ndarray:
    """Decode attention for a batch in which sequence s keeps its KV as ``views[view_ids[s]]``
    says (blocks written under different parallelism modes coexist in one pool, paper
    Sec. 5.2.3; each request carries its own stride and block capacity, Sec. 4.2.3).

    By definition the result is, sequence by sequence, what ``paged_decode`` gives under that
    sequence's view: computed exactly so, one pass per view with the other sequences' lengths
    set to zero.  All views must expose the same heads (same TP degree and rank).
    """
    ctx_lens = np.asarray(ctx_lens, dtype=np.int32)
    view_ids = np.asarray(view_ids)
    infos = [v.query() for v in views]
    assert all((i["n_q_local"], i["kv_head0"]) == (infos[0]["n_q_local"], infos[0]["kv_head0"]) for i in infos)
    out = np.zeros((len(ctx_lens), infos[0]["n_q_local"], views[0].geom.head_dim), dtype=np.float64)
    for k, v in enumerate(views):
        mine = view_ids == k
        if not mine.any():
            continue
        part = paged_decode(v, q, pool, table, np.where(mine, ctx_lens, 0).astype(np.int32), scale)
        out[mine] = part[mine]
    return out


def paged_prefill_rows(view: View, q, pool, table, ctx_lens, q_off, row_q, row_head,
                       scale: float = 0.0) -> np.ndarray:
    """Causal multi-token attention for selected (row of q, local head) pairs: out[n][d] fp64.

    q is [total_q][Hql][d]; sequence s owns rows [q_off[s], q_off[s+1]), which are the LAST
    q_len tokens of its ctx_lens[s] cached ones; each attends to every token up to itself.
    """
    info = view.query()
    d = view.geom.head_dim
    batch = int(len(ctx_lens))
    q_off = np.ascontiguousarray(q_off, dtype=np.int64)
    assert q.shape == (int(q_off[-1]), info["n_q_local"], d), q.shape
    table = np.ascontiguousarray(table, dtype=np.int32).reshape(batch, -1)
    rq = np.ascontiguousarray(row_q, dtype=np.int64)
    rh = np.ascontiguousarray(row_head, dtype=np.int32)
    out = np.empty((rq.shape[0], d), dtype=np.float64)
    rc = lib().oracle_paged_prefill_rows(*view._args(), _p(q, np.uint16), _p(pool.reshape(-1), np.uint16),
                                         _p(table, np.int32), C.c_int64(table.shape[1]),
                                         _p(np.ascontiguousarray(ctx_lens, dtype=np.int32), np.int32),
                                         _p(q_off, np.int64), C.c_int32(batch), _p(rq, np.int64),
                                         _p(rh, np.int32), C.c_int64(rq.shape[0]), C.c_double(scale),
                                         _p(out, np.float64))
    if rc:
        raise ValueError(f"oracle_paged_prefill_rows rc={rc}")
    return out


def paged_prefill(view: View, q, pool, table, ctx_lens, q_off, scale: float = 0.0) -> np.ndarray:
    """All rows: out[total_q][Hql][d] fp64 (see paged_prefill_rows)."""
    info = view.query()
    total, hql = int(q_off[-1]), info["n_q_local"]
    rq = np.repeat(np.arange(total, dtype=np.int64), hql)
    rh = np.tile(np.arange(hql, dtype=np.int32), total)
    return paged_prefill_rows(view, q, pool, table, ctx_lens, q_off, rq, rh, scale).reshape(
        total, hql, view.geom.head_dim)


def paged_decode_pairs(view: View, q, pool, table, ctx_lens, pair_seq, pair_head,
                       scale: float = 0.0) -> np.ndarray:
    """Rows for selected (sequence, local query head) pairs: out[n_pairs][d] fp64."""
    info = view.query()
    batch = int(ctx_lens.shape[0])
    d = view.geom.head_dim
    assert q.shape == (batch, info["n_q_local"], d), q.shape
    table = np.ascontiguousarray(table, dtype=np.int32).reshape(batch, -1)
    ps = np.ascontiguousarray(pair_seq, dtype=np.int32)
    ph = np.ascontiguousarray(pair_head, dtype=np.int32)
    out = np.empty((ps.shape[0], d), dtype=np.float64)
    rc = lib().oracle_paged_decode_pairs(*view._args(), _p(q, np.uint16),
                                         _p(pool.reshape(-1), np.uint16), _p(table, np.int32),
                                         C.c_int64(table.shape[1]), _p(ctx_lens, np.int32),
                                         _p(ps, np.int32), _p(ph, np.int32),
                                         C.c_int64(ps.shape[0]), C.c_double(scale),
                                         _p(out, np.float64))
    if rc:
        raise ValueError(f"oracle_paged_decode_pairs rc={rc}")
    return out


def paged_decode_partial(view: View, q, pool, table, seq: int, head: int, t_begin: int,
                         t_end: int, scale: float = 0.0):
    """Un-normalised (acc[d], m, l) over tokens [t_begin, t_end) of one (sequence, head)."""
    d = view.geom.head_dim
    table = np.ascontiguousarray(table, dtype=np.int32)
    table = table.reshape(q.shape[0], -1)
    acc = np.empty(d, dtype=np.float64)
    st = np.empty(2, dtype=np.float64)
    rc = lib().oracle_paged_decode_partial(*view._args(), _p(q, np.uint16),
                                           _p(pool.reshape(-1), np.uint16), _p(table, np.int32),
                                           C.c_int64(table.shape[1]), C.c_int32(seq),
                                           C.c_int32(head), C.c_int64(t_begin), C.c_int64(t_end),
                                           C.c_double(scale), _p(acc, np.float64),
                                           _p(st, np.float64))
    if rc:
        raise ValueError(f"oracle_paged_decode_partial rc={rc}")
    return acc, float(st[0]), float(st[1])


def dense_decode(geom: Geometry, q_full, K, V, seq_off, scale: float = 0.0) -> np.ndarray:
    """No pool/table/view: q_full[batch][Hq][d], K,V[total_tokens][Hkv][d] -> out[batch][Hq][d]."""
    batch = q_full.shape[0]
    seq_off = np.ascontiguousarray(seq_off, dtype=np.int64)
    assert seq_off.shape == (batch + 1,)
    out = np.empty((batch, geom.n_q_heads, geom.head_dim), dtype=np.float64)
    rc = lib().oracle_dense_decode(C.c_int32(geom.n_q_heads), C.c_int32(geom.n_kv_heads),
                                   C.c_int32(geom.head_dim), _p(q_full, np.uint16),
                                   _p(K, np.uint16), _p(V, np.uint16), _p(seq_off, np.int64),
                                   C.c_int32(batch), C.c_double(scale), _p(out, np.float64))
    if rc:
        raise ValueError(f"oracle_dense_decode rc={rc}")
    return out


def scatter(view: View, pool, table, n_tokens, seq_off, K, V) -> None:
    """Write logical K,V rows (heads the view exposes) into the pool through the table."""
    n = int(n_tokens.shape[0])
    table = np.ascontiguousarray(table, dtype=np.int32).reshape(n, -1)
    seq_off = np.ascontiguousarray(seq_off, dtype=np.int64)
    rc = lib().oracle_scatter(*view._args(), _p(pool.reshape(-1), np.uint16), _p(table, np.int32),
                              C.c_int64(table.shape[1]), _p(n_tokens, np.int32), C.c_int32(n),
                              _p(seq_off, np.int64), _p(K, np.uint16), _p(V, np.uint16))
    if rc:
        raise ValueError(f"oracle_scatter rc={rc}")


def gather(view: View, pool, table, n_tokens, seq_off, K, V) -> None:
    """Read the heads the view exposes from the pool into logical K,V (other heads untouched)."""
    n = int(n_tokens.shape[0])
    table = np.ascontiguousarray(table, dtype=np.int32).reshape(n, -1)
    seq_off = np.ascontiguousarray(seq_off, dtype=np.int64)
    rc = lib().oracle_gather(*view._args(), _p(pool.reshape(-1), np.uint16), _p(table, np.int32),
                             C.c_int64(table.shape[1]), _p(n_tokens, np.int32), C.c_int32(n),
                             _p(seq_off, np.int64), _p(K, np.uint16), _p(V, np.uint16))
    if rc:
        raise ValueError(f"oracle_gather rc={rc}")


def repack(src: View, dst: View, pool, src_table, dst_table, n_tokens) -> None:
    """In-pool byte-exact copy of the common heads from src-view blocks to dst-view blocks."""
    assert src.geom == dst.geom
    n = int(n_tokens.shape[0])
    st = np.ascontiguousarray(src_table, dtype=np.int32).reshape(n, -1)
    dt = np.ascontiguousarray(dst_table, dtype=np.int32).reshape(n, -1)
    g = src.geom
    rc = lib().oracle_repack(C.c_int32(g.n_q_heads), C.c_int32(g.n_kv_heads), C.c_int32(g.head_dim),
                             C.c_int32(g.base_block_size), C.c_int32(src.layout),
                             C.c_int32(src.tp_degree), C.c_int32(src.rank), C.c_int32(dst.layout),
                             C.c_int32(dst.tp_degree), C.c_int32(dst.rank),
                             _p(pool.reshape(-1), np.uint16), _p(st, np.int32),
                             C.c_int64(st.shape[1]), _p(dt, np.int32), C.c_int64(dt.shape[1]),
                             _p(n_tokens, np.int32), C.c_int32(n))
    if rc:
        raise ValueError(f"oracle_repack rc={rc}")


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(C.c_int(n))
