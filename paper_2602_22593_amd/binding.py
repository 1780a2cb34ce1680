"""Thin ctypes binding of libflyingkv.so: same names as the C ABI (include/flying_kv.h),
argument marshalling only.  torch supplies device memory and the stream; every step of the
path runs in the library's HIP kernels.  There is no fallback: if the library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libflyingkv.so")

KV_LAYOUT_DP = 0
KV_LAYOUT_TP = 1

KV_DECODE_SYNC_BYTES = 16384 * 8    # leading bytes of a decode workspace that must start out zero

KV_OK, KV_ERR_INVALID_ARG, KV_ERR_UNSUPPORTED, KV_ERR_WORKSPACE, KV_ERR_HIP, KV_ERR_RANGE, KV_ERR_ALIAS = \
    0, -1, -2, -3, -4, -5, -6


class KVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = f"{where}: {strerror(status)} ({status})"
        if status == KV_ERR_HIP:
            msg += f" -- {lib().kv_last_hip_error().decode()}"
        super().__init__(msg)


class kv_geometry(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("base_block_size", C.c_int32), ("dtype", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with "
                           "`python -m paper_2602_22593_amd.build` (needs hipcc)")
    L = C.CDLL(LIB_PATH)
    vp, i32p, i64 = C.c_void_p, C.POINTER(C.c_int32), C.c_int64
    L.kv_view_create.argtypes = [C.POINTER(kv_geometry), C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
    L.kv_view_destroy.argtypes = [vp]
    L.kv_view_destroy.restype = None
    L.kv_view_query.argtypes = [vp, i32p, i32p, i32p, i32p, C.POINTER(i64)]
    L.kv_view_strides.argtypes = [vp, i32p, i32p, i32p]
    L.paged_decode_attn_workspace_bytes.argtypes = [vp, C.c_int, C.c_int]
    L.paged_decode_attn_workspace_bytes.restype = C.c_size_t
    L.paged_decode_attn.argtypes = [vp, vp, vp, i64, vp, i64, vp, C.c_int, C.c_int, vp, C.c_float,
                                    vp, C.c_size_t, vp]
    L.paged_decode_attn_static.argtypes = [vp, vp, vp, i64, vp, i64, vp, C.c_int, C.c_int, vp, C.c_float, vp]
    L.paged_decode_attn_mixed.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, C.c_int, C.c_int, vp, C.c_int,
                                          C.c_float, vp, C.c_size_t, vp]
    L.paged_prefill_attn.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, C.c_int, i64, C.c_int, C.c_int, vp,
                                     C.c_float, vp, C.c_size_t, vp]
    L.paged_prefill_attn_workspace_bytes.argtypes = [vp, C.c_int, i64, C.c_int, C.c_int]
    L.paged_prefill_attn_workspace_bytes.restype = C.c_size_t
    L.kv_weight_view_make.argtypes = [C.c_int, C.c_int, C.c_int, i64, i64, vp]
    L.kv_weight_view_fused_qkv.argtypes = [vp, i64, C.c_int, C.c_int, vp]
    L.kv_linear_view.argtypes = [vp, i64, vp, i64, i64, vp, vp, i64, C.c_int, vp, C.c_size_t, vp]
    L.kv_linear_view_workspace_bytes.argtypes = [vp, C.c_int]
    L.kv_linear_view_workspace_bytes.restype = C.c_size_t
    L.kv_repack.argtypes = [vp, i64, vp, vp, vp, i64, vp, i64, vp, C.c_int, C.c_int, vp]
    L.kv_append.argtypes = [vp, i64, vp, vp, vp, vp, i64, vp, C.c_int, vp]
    L.kv_validate_tables.argtypes = [vp, i64, vp, i64, vp, C.c_int, vp, vp, i64, vp]
    L.kv_set_option.argtypes = [C.c_char_p, i64]
    L.kv_get_option.argtypes = [C.c_char_p]
    L.kv_get_option.restype = i64
    L.kv_probe_read.argtypes = [vp, C.c_size_t, vp, C.c_int, vp]
    L.kv_probe_copy.argtypes = [vp, vp, C.c_size_t, C.c_int, vp]
    L.kv_profile_enable.argtypes = [C.c_int]
    L.kv_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(i64)]
    for name in ("kv_strerror", "kv_last_hip_error", "kv_version"):
        getattr(L, name).restype = C.c_char_p
    L.kv_strerror.argtypes = [C.c_int]
    _lib = L
    return L


def strerror(status: int) -> str:
    return lib().kv_strerror(status).decode()


def _check(rc: int, where: str) -> None:
    if rc != KV_OK:
        raise KVError(rc, where)


class KVView:
    """Owner of a kv_view handle plus its resolved integers (read back through the ABI)."""

    def __init__(self, handle: int, geometry: kv_geometry, layout: int, tp_degree: int, rank: int):
        self.handle = C.c_void_p(handle)
        self.geometry, self.layout, self.tp_degree, self.rank = geometry, layout, tp_degree, rank
        bt, hl, hq, h0 = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
        bb = C.c_int64()
        _check(lib().kv_view_query(self.handle, bt, hl, hq, h0, bb), "kv_view_query")
        self.block_tokens, self.n_kv_local, self.n_q_local = bt.value, hl.value, hq.value
        self.kv_head0, self.block_bytes = h0.value, bb.value
        ts, rh, r0 = C.c_int32(), C.c_int32(), C.c_int32()
        _check(lib().kv_view_strides(self.handle, ts, rh, r0), "kv_view_strides")
        self.token_stride_elems, self.row_heads, self.row_head0 = ts.value, rh.value, r0.value
        self.head_dim = geometry.head_dim
        self.group = geometry.n_q_heads // geometry.n_kv_heads

    def __del__(self):
        try:
            if self.handle:
                lib().kv_view_destroy(self.handle)
                self.handle = None
        except Exception:
            pass


def kv_view_create(n_q_heads: int, n_kv_heads: int, head_dim: int, base_block_size: int,
                   layout: int, tp_degree: int = 1, rank: int = 0, dtype: int = 0) -> KVView:
    g = kv_geometry(n_q_heads, n_kv_heads, head_dim, base_block_size, dtype)
    out = C.c_void_p()
    _check(lib().kv_view_create(C.byref(g), layout, tp_degree, rank, C.byref(out)), "kv_view_create")
    return KVView(out.value, g, layout, tp_degree, rank)


def _stream_ptr(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dev(t: torch.Tensor, dtypes, name: str) -> C.c_void_p:
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if t.dtype not in dtypes:
        raise ValueError(f"{name} has dtype {t.dtype}, expected one of {dtypes}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return C.c_void_p(t.data_ptr())


def _dev_rows(t: torch.Tensor, dtypes, name: str) -> C.c_void_p:
    """A 2-d device tensor whose rows are contiguous (the row stride itself is free)."""
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if t.dtype not in dtypes:
        raise ValueError(f"{name} has dtype {t.dtype}, expected one of {dtypes}")
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-d with contiguous rows")
    return C.c_void_p(t.data_ptr())


_BF16 = (torch.bfloat16, torch.int16, torch.uint16)
_workspaces = {}


def paged_decode_attn_workspace_bytes(view: KVView, batch: int, max_ctx_len: int) -> int:
    return int(lib().paged_decode_attn_workspace_bytes(view.handle, batch, max_ctx_len))


def _workspace(device, nbytes: int, stream=None, kind: str = "scratch") -> torch.Tensor:
    """Scratch for a call that was given none: one buffer per (device, stream, kind), grown on demand.
    Calls on one stream are ordered and may share it; calls on different streams get their own.
    Decode calls (kind "decode") keep a buffer to themselves: its leading arrival words must stay
    zero between calls, and the other entry points write their scratch from the first byte on."""
    if stream is None:
        stream = torch.cuda.current_stream(device)
    key = (device.index, stream.cuda_stream, kind)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        # zero-filled: the kernels expect their arrival words (the first bytes) to start at zero
        with torch.cuda.stream(stream):
            ws = torch.zeros(max(nbytes, 1 << 20), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def paged_decode_attn(q: torch.Tensor, kv_pool: torch.Tensor, block_table: torch.Tensor,
                      ctx_lens: torch.Tensor, view: KVView, max_ctx_len: int,
                      out: Optional[torch.Tensor] = None, scale: float = 0.0,
                      workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """out[batch][n_q_local][head_dim] (bf16) = decode attention through ``view``.

    ``max_ctx_len`` is the caller's host-side bound of ``ctx_lens`` (no device sync here).
    """
    batch = int(ctx_lens.shape[0])
    if tuple(q.shape) != (batch, view.n_q_local, view.head_dim):
        raise ValueError(f"q has shape {tuple(q.shape)}, expected {(batch, view.n_q_local, view.head_dim)}")
    if out is None:
        out = torch.empty_like(q)
    if block_table.dim() != 2 or block_table.shape[0] != batch:
        raise ValueError("block_table must be [batch][max_blocks]")
    if kv_pool.numel() * kv_pool.element_size() % view.block_bytes:
        raise ValueError("kv_pool size is not a whole number of blocks")
    n_pool_blocks = kv_pool.numel() * kv_pool.element_size() // view.block_bytes
    need = paged_decode_attn_workspace_bytes(view, batch, max_ctx_len)
    if workspace is None:
        workspace = _workspace(q.device, need, stream, "decode")
    rc = lib().paged_decode_attn(
        _dev(q, _BF16, "q"), _dev(out, _BF16, "out"), _dev(kv_pool, _BF16, "kv_pool"),
        n_pool_blocks, _dev(block_table, (torch.int32,), "block_table"), block_table.stride(0),
        _dev(ctx_lens, (torch.int32,), "ctx_lens"), batch, int(max_ctx_len), view.handle,
        float(scale), _dev(workspace, (torch.uint8,), "workspace"),
        workspace.numel(), _stream_ptr(stream))
    _check(rc, "paged_decode_attn")
    return out


def paged_decode_attn_static(q: torch.Tensor, kv_pool: torch.Tensor, block_table: torch.Tensor,
                             ctx_lens: torch.Tensor, view: KVView, max_ctx_len: int,
                             out: torch.Tensor, scale: float = 0.0, stream=None) -> torch.Tensor:
    """paged_decode_attn on the library's own fixed scratch array: no workspace argument and no
    allocation anywhere in the call (``out`` must be given)."""
    batch = int(ctx_lens.shape[0])
    if tuple(q.shape) != (batch, view.n_q_local, view.head_dim) or tuple(out.shape) != tuple(q.shape):
        raise ValueError(f"q and out must have shape {(batch, view.n_q_local, view.head_dim)}")
    if block_table.dim() != 2 or block_table.shape[0] != batch:
        raise ValueError("block_table must be [batch][max_blocks]")
    n_pool_blocks = kv_pool.numel() * kv_pool.element_size() // view.block_bytes
    rc = lib().paged_decode_attn_static(
        _dev(q, _BF16, "q"), _dev(out, _BF16, "out"), _dev(kv_pool, _BF16, "kv_pool"),
        n_pool_blocks, _dev(block_table, (torch.int32,), "block_table"), block_table.stride(0),
        _dev(ctx_lens, (torch.int32,), "ctx_lens"), batch, int(max_ctx_len), view.handle,
        float(scale), _stream_ptr(stream))
    _check(rc, "paged_decode_attn_static")
    return out


def paged_decode_attn_mixed(q: torch.Tensor, kv_pool: torch.Tensor, block_table: torch.Tensor,
                            ctx_lens: torch.Tensor, view_ids: torch.Tensor, views, max_ctx_len: int,
                            out: Optional[torch.Tensor] = None, scale: float = 0.0,
                            workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Decode attention for a batch whose sequence s keeps its KV as ``views[view_ids[s]]`` says.

    All views share geometry, TP degree and rank (same local heads); they differ in block layout.
    """
    batch = int(ctx_lens.shape[0])
    v0 = views[0]
    if tuple(q.shape) != (batch, v0.n_q_local, v0.head_dim):
        raise ValueError(f"q has shape {tuple(q.shape)}, expected {(batch, v0.n_q_local, v0.head_dim)}")
    if out is None:
        out = torch.empty_like(q)
    if block_table.dim() != 2 or block_table.shape[0] != batch:
        raise ValueError("block_table must be [batch][max_blocks]")
    n_pool_blocks = kv_pool.numel() * kv_pool.element_size() // v0.block_bytes
    need = paged_decode_attn_workspace_bytes(v0, batch, max_ctx_len)
    if workspace is None:
        workspace = _workspace(q.device, need, stream, "decode")
    handles = (C.c_void_p * len(views))(*[v.handle for v in views])
    rc = lib().paged_decode_attn_mixed(
        _dev(q, _BF16, "q"), _dev(out, _BF16, "out"), _dev(kv_pool, _BF16, "kv_pool"),
        n_pool_blocks, _dev(block_table, (torch.int32,), "block_table"), block_table.stride(0),
        _dev(ctx_lens, (torch.int32,), "ctx_lens"), _dev(view_ids, (torch.int32,), "view_ids"), batch,
        int(max_ctx_len), C.cast(handles, C.c_void_p), len(views), float(scale),
        _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(), _stream_ptr(stream))
    _check(rc, "paged_decode_attn_mixed")
    return out


def paged_prefill_attn(q: torch.Tensor, kv_pool: torch.Tensor, block_table: torch.Tensor,
                       ctx_lens: torch.Tensor, q_offsets: torch.Tensor, view: KVView, max_ctx_len: int,
                       max_q_len: int, out: Optional[torch.Tensor] = None, scale: float = 0.0,
                       workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Causal attention of each sequence's last q_len tokens over its cached tokens, through ``view``.

    q: bf16 [total_q][n_q_local][head_dim]; q_offsets: int32 [batch + 1] (device); the K/V of the
    new tokens are already in the pool.  ``max_ctx_len`` / ``max_q_len`` are host-side bounds.
    """
    batch = int(ctx_lens.shape[0])
    if q.dim() != 3 or tuple(q.shape[1:]) != (view.n_q_local, view.head_dim):
        raise ValueError(f"q has shape {tuple(q.shape)}, expected [total_q, {view.n_q_local}, {view.head_dim}]")
    if q_offsets.shape[0] != batch + 1:
        raise ValueError("q_offsets must be [batch + 1]")
    if out is None:
        out = torch.empty_like(q)
    if block_table.dim() != 2 or block_table.shape[0] != batch:
        raise ValueError("block_table must be [batch][max_blocks]")
    n_pool_blocks = kv_pool.numel() * kv_pool.element_size() // view.block_bytes
    total_q = int(q.shape[0])
    need = int(lib().paged_prefill_attn_workspace_bytes(view.handle, batch, total_q, int(max_ctx_len),
                                                        int(max_q_len)))
    if workspace is None:
        workspace = _workspace(q.device, need, stream)
    rc = lib().paged_prefill_attn(
        _dev(q, _BF16, "q"), _dev(out, _BF16, "out"), _dev(kv_pool, _BF16, "kv_pool"), n_pool_blocks,
        _dev(block_table, (torch.int32,), "block_table"), block_table.stride(0),
        _dev(ctx_lens, (torch.int32,), "ctx_lens"), _dev(q_offsets, (torch.int32,), "q_offsets"), batch,
        total_q, int(max_ctx_len), int(max_q_len), view.handle, float(scale),
        _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(), _stream_ptr(stream))
    _check(rc, "paged_prefill_attn")
    return out


class kv_weight_view(C.Structure):
    """Mirror of the C struct: stored rows (up to three segments) and columns that are active."""
    _fields_ = [("n_segments", C.c_int32), ("row_start", C.c_int64 * 3), ("row_count", C.c_int64 * 3),
                ("col_start", C.c_int64), ("col_count", C.c_int64)]

    @property
    def n_rows(self) -> int:
        return sum(self.row_count[i] for i in range(self.n_segments))


def kv_weight_view_make(dim: int, r: int, m: int, n_rows: int, n_cols: int) -> kv_weight_view:
    v = kv_weight_view()
    _check(lib().kv_weight_view_make(dim, r, m, n_rows, n_cols, C.byref(v)), "kv_weight_view_make")
    return v


def kv_weight_view_fused_qkv(n_q_heads: int, n_kv_heads: int, head_dim: int, hidden: int, r: int,
                             m: int) -> kv_weight_view:
    g = kv_geometry(n_q_heads, n_kv_heads, head_dim, 16, 0)
    v = kv_weight_view()
    _check(lib().kv_weight_view_fused_qkv(C.byref(g), hidden, r, m, C.byref(v)), "kv_weight_view_fused_qkv")
    return v


def kv_linear_view(x: torch.Tensor, w_full: torch.Tensor, view: kv_weight_view,
                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                   stream=None) -> torch.Tensor:
    """y[M][view rows] (bf16) = x @ W_active^T, W_active = ``view`` of the stored ``w_full`` [out][in]."""
    if x.dim() != 2 or w_full.dim() != 2 or x.shape[1] != view.col_count:
        raise ValueError("x must be [M][view.col_count], w_full [out][in]")
    M = int(x.shape[0])
    if out is None:
        out = torch.empty((M, view.n_rows), dtype=torch.bfloat16, device=x.device)
    need = int(lib().kv_linear_view_workspace_bytes(C.byref(view), M))
    if workspace is None:
        workspace = _workspace(x.device, need, stream)
    rc = lib().kv_linear_view(_dev_rows(x, _BF16, "x"), x.stride(0), _dev_rows(w_full, _BF16, "w_full"),
                              int(w_full.shape[0]), w_full.stride(0), C.byref(view),
                              _dev_rows(out, _BF16, "out"), out.stride(0), M,
                              _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(),
                              _stream_ptr(stream))
    _check(rc, "kv_linear_view")
    return out


def kv_repack(kv_pool: torch.Tensor, src_view: KVView, dst_view: KVView,
              src_block_table: torch.Tensor, dst_block_table: torch.Tensor,
              n_tokens: torch.Tensor, max_tokens: int, stream=None) -> None:
    """Copy the heads common to both views from src-view blocks to dst-view blocks, in the pool."""
    n_seqs = int(n_tokens.shape[0])
    n_pool_blocks = kv_pool.numel() * kv_pool.element_size() // src_view.block_bytes
    rc = lib().kv_repack(
        _dev(kv_pool, _BF16, "kv_pool"), n_pool_blocks, src_view.handle, dst_view.handle,
        _dev(src_block_table, (torch.int32,), "src_block_table"), src_block_table.stride(0),
        _dev(dst_block_table, (torch.int32,), "dst_block_table"), dst_block_table.stride(0),
        _dev(n_tokens, (torch.int32,), "n_tokens"), n_seqs, int(max_tokens), _stream_ptr(stream))
    _check(rc, "kv_repack")


def kv_append(kv_pool: torch.Tensor, view: KVView, k_new: torch.Tensor, v_new: torch.Tensor,
              block_table: torch.Tensor, positions: torch.Tensor, stream=None) -> None:
    """Write each sequence's new K and V rows at token index positions[s] through ``view``."""
    n_seqs = int(positions.shape[0])
    want = (n_seqs, view.n_kv_local, view.head_dim)
    if tuple(k_new.shape) != want or tuple(v_new.shape) != want:
        raise ValueError(f"k_new / v_new must be {want}")
    n_pool_blocks = kv_pool.numel() * kv_pool.element_size() // view.block_bytes
    rc = lib().kv_append(
        _dev(kv_pool, _BF16, "kv_pool"), n_pool_blocks, view.handle, _dev(k_new, _BF16, "k_new"),
        _dev(v_new, _BF16, "v_new"), _dev(block_table, (torch.int32,), "block_table"),
        block_table.stride(0), _dev(positions, (torch.int32,), "positions"), n_seqs,
        _stream_ptr(stream))
    _check(rc, "kv_append")


def kv_validate_tables(view: KVView, n_pool_blocks: int, block_table: torch.Tensor,
                       n_tokens: torch.Tensor, other_view: Optional[KVView] = None,
                       other_table: Optional[torch.Tensor] = None, stream=None) -> int:
    """Debug check of table contents (synchronises). Returns the kv_status instead of raising."""
    return int(lib().kv_validate_tables(
        view.handle, n_pool_blocks, _dev(block_table, (torch.int32,), "block_table"),
        block_table.stride(0), _dev(n_tokens, (torch.int32,), "n_tokens"), int(n_tokens.shape[0]),
        other_view.handle if other_view is not None else None,
        _dev(other_table, (torch.int32,), "other_table") if other_table is not None else None,
        other_table.stride(0) if other_table is not None else 0, _stream_ptr(stream)))


def kv_set_option(key: str, value: int) -> None:
    _check(lib().kv_set_option(key.encode(), int(value)), f"kv_set_option({key})")


def kv_get_option(key: str) -> int:
    return int(lib().kv_get_option(key.encode()))


KV_PROF_DECODE_MAIN, KV_PROF_DECODE_MERGE, KV_PROF_REPACK, KV_PROF_PREFILL, KV_PROF_LINEAR = 0, 1, 2, 3, 4


def kv_profile_enable(on: bool) -> None:
    _check(lib().kv_profile_enable(1 if on else 0), "kv_profile_enable")


def kv_profile_read(which: int):
    """(total milliseconds, launches) of kernel ``which`` since profiling was enabled."""
    ms, n = C.c_double(), C.c_int64()
    _check(lib().kv_profile_read(which, C.byref(ms), C.byref(n)), "kv_profile_read")
    return ms.value, n.value


def kv_probe_read(src: torch.Tensor, n_workgroups: int, stream=None) -> None:
    """Stream ``src`` from HBM once (known-traffic reference kernel)."""
    _check(lib().kv_probe_read(C.c_void_p(src.data_ptr()), src.numel() * src.element_size(), None,
                               n_workgroups, _stream_ptr(stream)), "kv_probe_read")


def kv_probe_copy(dst: torch.Tensor, src: torch.Tensor, n_workgroups: int, stream=None) -> None:
    """Copy ``src`` to ``dst`` once (known-traffic reference kernel)."""
    assert dst.numel() * dst.element_size() == src.numel() * src.element_size()
    _check(lib().kv_probe_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()),
                               src.numel() * src.element_size(), n_workgroups, _stream_ptr(stream)),
           "kv_probe_copy")


def kv_probe_read_placed(src: torch.Tensor, n_workgroups: int, stream=None) -> torch.Tensor:
    """Stream ``src`` once in contiguous per-workgroup shares; returns int64 [n_workgroups][3] on the
    device: XCD of the workgroup, start tick, end tick (100 MHz)."""
    L = lib()
    L.kv_probe_read_placed.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
    rec = torch.zeros((n_workgroups, 3), dtype=torch.int64, device=src.device)
    _check(L.kv_probe_read_placed(C.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                                  C.c_void_p(rec.data_ptr()), None, n_workgroups, _stream_ptr(stream)),
           "kv_probe_read_placed")
    return rec


def kv_probe_read_blocks(pool: torch.Tensor, block_ids: torch.Tensor, block_bytes: int,
                         n_workgroups: int, stream=None) -> None:
    """Stream the pool blocks listed in ``block_ids`` (int32, device) once, block by block."""
    L = lib()
    L.kv_probe_read_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_void_p, C.c_int,
                                       C.c_void_p]
    _check(L.kv_probe_read_blocks(C.c_void_p(pool.data_ptr()), C.c_void_p(block_ids.data_ptr()),
                                  int(block_ids.numel()), int(block_bytes), None, n_workgroups,
                                  _stream_ptr(stream)), "kv_probe_read_blocks")
