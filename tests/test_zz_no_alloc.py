"""GPU test of paged_decode_attn_static, the entry point for callers that cannot allocate: its
output against paged_decode_attn's (the same kernels on a caller's workspace) and against the CPU
oracle, on two calls in a row that share the library's fixed scratch array, the second with a
smaller input.  Collected last: it runs after every other GPU test and also passes alone."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, make_case

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3
DEV = "cuda:0"


def dev_u16(a):
    return torch.from_numpy(a.view(np.int16)).to(DEV)


def static_call(c, view):
    """paged_decode_attn_static through the raw C ABI on the case's host arrays."""
    q, pool = dev_u16(c.q), dev_u16(c.pool)
    table, ctx = torch.from_numpy(c.table).to(DEV), torch.from_numpy(c.ctx).to(DEV)
    out = torch.full_like(q, 0x7FC0)       # bf16 NaN: every row must be written
    torch.cuda.synchronize()
    vp = C.c_void_p
    rc = kv.lib().paged_decode_attn_static(
        vp(q.data_ptr()), vp(out.data_ptr()), vp(pool.data_ptr()), pool.shape[0], vp(table.data_ptr()),
        table.stride(0), vp(ctx.data_ptr()), len(c.ctx), int(c.ctx.max()), view.handle, C.c_float(0.0),
        vp(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, kv.strerror(rc)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


def workspace_call(c, view):
    out = kv.paged_decode_attn(dev_u16(c.q), dev_u16(c.pool), torch.from_numpy(c.table).to(DEV),
                               torch.from_numpy(c.ctx).to(DEV), view, int(c.ctx.max()))
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint16)


def check(c, view, what):
    got = static_call(c, view)
    same = workspace_call(c, view)
    want = oracle.paged_decode(c.view, c.q, c.pool, c.table, c.ctx)
    err = np.abs(bf16_bits_to_f64(got) - bf16_bits_to_f64(same))
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (what, "vs paged_decode_attn", err.max())
    # the same kernels in the same launch shape: the two entry points agree bit for bit
    assert np.array_equal(got, same), what
    err = np.abs(bf16_bits_to_f64(got) - want)
    assert np.isfinite(bf16_bits_to_f64(got)).all(), what
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (what, "vs oracle", err.max(), err.mean())
    assert (got[c.ctx == 0] == 0).all(), what


@pytest.mark.parametrize("triple", [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 4, 1), (LAYOUT_TP, 8, 3)])
def test_static_scratch_two_calls_second_smaller(triple):
    """First a batch whose longest sequence is cut over many wavefronts (long piece lists in the
    scratch array), then, with no clearing in between, a smaller batch whose pieces land in slots
    the first call used."""
    assert torch.cuda.is_available(), "needs a GPU"
    w = wl.Workload("static_scratch", 97, 32, 8, 128, 16, 12, "fixed", ())
    view = kv.kv_view_create(w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size, *triple)
    big = make_case(w, triple, ctx=np.array([9000, 17, 0, 2049, 511, 1, 4096, 33, 1300, 64, 700, 3000],
                                            dtype=np.int32))
    check(big, view, f"{triple} first call")
    small = make_case(w, triple, ctx=np.array([300, 0, 1500, 16, 47], dtype=np.int32))
    check(small, view, f"{triple} second, smaller call")
    check(big, view, f"{triple} third call, large again")


def test_static_scratch_rejects_sizes_beyond_the_array():
    """A batch whose scratch need exceeds the fixed array is refused on the host, before any launch."""
    view = kv.kv_view_create(64, 64, 128, 16, LAYOUT_DP, 1, 0)
    batch, max_ctx = 2048, 64
    need = kv.paged_decode_attn_workspace_bytes(view, batch, max_ctx)
    assert need > (32 << 20)
    fake = C.c_void_p(256)
    rc = kv.lib().paged_decode_attn_static(fake, fake, fake, 10, fake, 8, fake, batch, max_ctx, view.handle,
                                           C.c_float(0.0), None)
    assert rc == kv.KV_ERR_WORKSPACE
