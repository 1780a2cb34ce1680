"""The decode step under HIP graph capture: the library allocates nothing and synchronises nothing in
its hot path, so a serving loop can record append + attention once and replay it per token."""
import numpy as np
import pytest
import torch

import oracle
from oracle import LAYOUT_DP, LAYOUT_TP
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, make_case

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
    ws = torch.empty(kv.paged_decode_attn_workspace_bytes(view, len(lens), int(lens.max())), dtype=torch.uint8, device=DEV)
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
