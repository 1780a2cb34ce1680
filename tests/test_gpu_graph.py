"""The entry points under HIP graph capture: the library allocates nothing and synchronises nothing in
its hot path, so a serving loop can record append + attention once and replay it per token."""
import numpy as np
import pytest
import torch

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, linear_tolerance, make_case

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev_u16(a):
    return torch.from_numpy(a.view(np.int16)).to(DEV)


@pytest.mark.parametrize("triple", [(LAYOUT_DP, 1, 0), (LAYOUT_TP, 8, 3)])
def test_decode_call_replayed_from_a_graph(triple):
    """Capture one paged_decode_attn call (main + merge kernels) with fixed buffers, then replay it
    three times with fresh query rows copied into the captured buffer, eager work and
    synchronisations in between; every replay is compared with the oracle."""
    lens = np.array([700, 33, 2049, 1, 5000, 64, 0, 1300], dtype=np.int32)
    w = wl.Workload("graph", 76, 32, 8, 128, 16, len(lens), "x", ())
    c = make_case(w, triple, lens)
    view = kv.kv_view_create(w.n_q_heads, w.n_kv_heads, w.head_dim, w.base_block_size, *triple)
    q = dev_u16(c.q)
    pool, table, n = dev_u16(c.pool), torch.from_numpy(c.table).to(DEV), torch.from_numpy(c.ctx).to(DEV)
    out = torch.zeros_like(q)
    ws = torch.zeros(kv.paged_decode_attn_workspace_bytes(view, len(lens), int(lens.max())), dtype=torch.uint8, device=DEV)
    kv.paged_decode_attn(q, pool, table, n, view, int(lens.max()), out=out, workspace=ws)   # eager warm-up
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        kv.paged_decode_attn(q, pool, table, n, view, int(lens.max()), out=out, workspace=ws)
    gen = wl.generator(76, wl.SUB_MISC)
    for rep in range(3):
        q_new = wl.randn_bf16(c.q.shape, gen)
        q.copy_(dev_u16(q_new))
        out.zero_()                                   # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want = oracle.paged_decode(c.view, q_new, c.pool, c.table, c.ctx)
        got = bf16_bits_to_f64(out.cpu().numpy().view(np.uint16))
        err = np.abs(got - want)
        assert np.isfinite(got).all() and err.max() <= 2e-2 and err.mean() <= 2e-3, (rep, err.max(), err.mean())


def test_prefill_and_projection_replayed_from_a_graph():
    """One graph holding the QKV projection on a weight view and a multi-token attention call (with its
    split-key-range merge kernel): replayed three times with fresh inputs copied into the captured
    buffers, eager work in between; every replay against the oracle."""
    from oracle import weights as ow
    from helpers import make_prefill_case
    w = wl.Workload("graph_prefill", 77, 32, 8, 128, 16, 2, "x", ())
    ctx, qlen = np.array([6000, 900], dtype=np.int32), np.array([40, 33], dtype=np.int32)
    c = make_prefill_case(w, (LAYOUT_TP, 2, 1), ctx, qlen)
    view = kv.kv_view_create(32, 8, 128, 16, LAYOUT_TP, 2, 1)
    q = dev_u16(c.q)
    pool, table, n = dev_u16(c.pool), torch.from_numpy(c.table).to(DEV), torch.from_numpy(c.ctx).to(DEV)
    q_off = torch.from_numpy(c.q_off.astype(np.int32)).to(DEV)
    out = torch.zeros_like(q)
    need = kv.lib().paged_prefill_attn_workspace_bytes(view.handle, 2, int(qlen.sum()), int(ctx.max()), int(qlen.max()))
    assert need > 0                                   # the split path is the one captured
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    # the projection: 64 rows on rank 1's slice of a fused [6144][512] weight
    hidden, M = 512, 64
    gen = wl.generator(77, wl.SUB_MISC)
    w_bits = wl.randn_bf16((6144, hidden), gen)
    x_bits = wl.randn_bf16((M, hidden), gen)
    wv = kv.kv_weight_view_fused_qkv(32, 8, 128, hidden, 1, 2)
    ov = ow.weight_view_fused_qkv(32, 8, 128, hidden, 1, 2)
    dw = torch.from_numpy(w_bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    dx = torch.from_numpy(x_bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    y = torch.zeros((M, wv.n_rows), dtype=torch.bfloat16, device=DEV)
    lws = torch.empty(max(int(kv.lib().kv_linear_view_workspace_bytes(__import__("ctypes").byref(wv), M)), 256),
                      dtype=torch.uint8, device=DEV)

    def step():
        kv.kv_linear_view(dx, dw, wv, out=y, workspace=lws)
        kv.paged_prefill_attn(q, pool, table, n, q_off, view, int(ctx.max()), int(qlen.max()), out=out, workspace=ws)

    step()                                            # eager warm-up
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        q_new = wl.randn_bf16(c.q.shape, gen)
        x_new = wl.randn_bf16((M, hidden), gen)
        q.copy_(dev_u16(q_new))
        dx.copy_(torch.from_numpy(x_new.view(np.int16)).to(DEV).view(torch.bfloat16))
        out.zero_()
        y.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want = oracle.paged_prefill(c.view, q_new, c.pool, c.table, c.ctx, c.q_off)
        got = bf16_bits_to_f64(out.cpu().numpy().view(np.uint16))
        err = np.abs(got - want)
        assert np.isfinite(got).all() and err.max() <= 2e-2 and err.mean() <= 2e-3, (rep, err.max(), err.mean())
        want_y = ow.linear_view(x_new, w_bits, ov)
        got_y = bf16_bits_to_f64(y.cpu().view(torch.int16).numpy().view(np.uint16))
        tol = linear_tolerance(x_new, w_bits, ov, want_y)
        assert np.isfinite(got_y).all() and not (np.abs(got_y - want_y) > tol).any(), rep
