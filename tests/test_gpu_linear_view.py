"""GPU parity of kv_linear_view (linear layer on a zero-copy weight shard view) with the oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import weights as ow
from paper_2602_22593_amd import binding as kv
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64, linear_tolerance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits(shape, seed):
    return wl.randn_bf16(shape, wl.generator(41, seed))


def dev(a):
    return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)


def check(got_bits, x, w, ov, what):
    """Every output against the fp64 product, within the bound of helpers.linear_tolerance (half a
    bf16 ulp of the result plus a sqrt(K)-scaled fp32 accumulation term on the exact sum of
    |x w|)."""
    want = ow.linear_view(x, w, ov)
    got = bf16_bits_to_f64(got_bits)
    assert np.isfinite(got).all(), what
    bad = np.abs(got - want) > linear_tolerance(x, w, ov, want)
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, worst {np.abs(got - want).max():.4g}"


def gpu_view(o: ow.WeightView) -> kv.kv_weight_view:
    v = kv.kv_weight_view()
    v.n_segments = len(o.row_segments)
    for i, (a, c) in enumerate(o.row_segments):
        v.row_start[i], v.row_count[i] = a, c
    v.col_start, v.col_count = o.col_start, o.col_count
    return v


@pytest.mark.parametrize("M", [1, 17, 64, 100, 256])
@pytest.mark.parametrize("m,r", [(1, 0), (2, 1), (8, 5)])
def test_fused_qkv_column_slice(M, m, r):
    """Llama-8B-shaped heads on a narrow hidden size (oracle cost): rank r's Q, K and V rows of the
    fused weight, batch sizes inside, at and past the 64-row tile."""
    hq, hkv, d, hidden = 32, 8, 128, 512
    x, w = bits((M, hidden), 10 + M), bits(((hq + 2 * hkv) * d, hidden), 20)
    ov = ow.weight_view_fused_qkv(hq, hkv, d, hidden, r, m)
    gv = kv.kv_weight_view_fused_qkv(hq, hkv, d, hidden, r, m)
    assert [(gv.row_start[i], gv.row_count[i]) for i in range(3)] == list(ov.row_segments)
    y = kv.kv_linear_view(dev(x), dev(w), gv)
    torch.cuda.synchronize()
    check(y.cpu().view(torch.int16).numpy().view(np.uint16), x, w, ov, f"qkv M={M} {r}/{m}")


@pytest.mark.parametrize("M", [3, 64, 130])
@pytest.mark.parametrize("m,r", [(1, 0), (2, 0), (4, 3), (8, 2)])
def test_output_projection_row_slice(M, m, r):
    """W^O [hidden][Hq d]: rank r multiplies its slice of the attention output by the matching
    column range of the stored weight (partial sum).  x is itself a column slice of a wider
    tensor (row stride larger than its width).  K per rank from 4096 (pipelined loop, several
    slabs per wavefront) down to 512 (one slab each)."""
    hidden, kin = 256, 4096
    a_full, w = bits((M, kin), 30 + M), bits((hidden, kin), 31)
    ov = ow.weight_view(1, r, m, hidden, kin)
    gv = kv.kv_weight_view_make(1, r, m, hidden, kin)
    assert (gv.col_start, gv.col_count) == (ov.col_start, ov.col_count)
    x_slice = dev(a_full)[:, ov.col_start:ov.col_start + ov.col_count]
    y = kv.kv_linear_view(x_slice, dev(w), gv)
    torch.cuda.synchronize()
    check(y.cpu().view(torch.int16).numpy().view(np.uint16),
          np.ascontiguousarray(a_full[:, ov.col_start:ov.col_start + ov.col_count]), w, ov, f"wo M={M} {r}/{m}")


def test_output_rows_outside_the_batch_are_untouched():
    hidden, kin, M = 64, 256, 5
    x, w = bits((M, kin), 40), bits((hidden, kin), 41)
    out = torch.full((8, hidden + 4), 7.0, dtype=torch.bfloat16, device=DEV)
    kv.kv_linear_view(dev(x), dev(w), kv.kv_weight_view_make(0, 0, 1, hidden, kin), out=out[:M, :hidden])
    torch.cuda.synchronize()
    assert (out[M:] == 7.0).all() and (out[:, hidden:] == 7.0).all()
    check(out[:M, :hidden].contiguous().cpu().view(torch.int16).numpy().view(np.uint16),
          x, w, ow.weight_view(0, 0, 1, hidden, kin), "padded out")


@pytest.mark.parametrize("splits", [0, 1, 2, 3, 5, 16])
@pytest.mark.parametrize("slabs", [1, 4, 7, 9])
def test_every_cut_of_the_input_dimension(slabs, splits):
    """The input dimension in 128-wide slabs, four to a chunk: one slab, exactly one chunk, a chunk
    and a part (7), two chunks and one slab (9); cut over 1, 2, 3, 5 and (capped at the slab count)
    16 workgroups, and by the library's own choice (0).  A row-parallel view (column range) of a
    wider stored weight, batch past one tile."""
    K, M, N = 128 * slabs, 70, 192
    x, w = bits((M, K), 60 + slabs), bits((N, 2 * K + 64), 70 + slabs)
    ov = ow.WeightView(((0, N),), K + 64, K)
    gv = gpu_view(ov)
    kv.kv_set_option("linear_splits", splits)
    try:
        y = kv.kv_linear_view(dev(x), dev(w), gv)
        torch.cuda.synchronize()
    finally:
        kv.kv_set_option("linear_splits", 0)
    check(y.cpu().view(torch.int16).numpy().view(np.uint16), x, w, ov, f"slabs {slabs} splits {splits}")


@pytest.mark.parametrize("M,N,K,what", [
    (64, 8256, 4096, "8 row blocks per workgroup, four slices; the last workgroup of a column has 4 of its 8 blocks"),
    (64, 6208, 4096, "6 row blocks, four slices; the last workgroup has 4 of its 6"),
    (64, 4160, 4096, "4 row blocks, four slices"),
    (128, 1600, 4096, "3 row blocks, two batch tiles; the last workgroup has 1 of its 3"),
    (256, 1344, 2048, "2 row blocks, four batch tiles, two slices"),
    (40, 832, 640, "1 row block, one slice of 5 slabs: wavefront 0 has two slabs, the others one"),
    (200, 320, 1152, "1 row block, four batch tiles, slices of 8 slabs and of 1"),
])
def test_every_rows_per_workgroup_shape(M, N, K, what):
    """Shapes that make the library pick each of its row-blocks-per-workgroup instantiations (8, 6, 4,
    3, 2, 1), with block counts that do not divide evenly (trailing blocks are requested from idle
    addresses and multiplied by zero) and slices whose slab count is not a multiple of the four
    wavefronts.  Rows and columns are a sub-range of a larger stored weight."""
    x, w = bits((M, K), 60 + M), bits((N + 128, K + 256), 61 + (N % 97))
    ov = ow.WeightView(((64, N),), 128, K)
    y = kv.kv_linear_view(dev(x), dev(w), gpu_view(ov))
    torch.cuda.synchronize()
    check(y.cpu().view(torch.int16).numpy().view(np.uint16), x, w, ov, what)
