"""Pins for the weight-view oracle (CPU only): brute force on tiny inputs, the partition property
of the views, and the two Megatron identities (concatenation for the column-parallel layer, sum of
partials for the row-parallel one) that make a TP group's result equal the unsharded layer's."""
import numpy as np
import pytest

from oracle import weights as ow
from paper_2602_22593_amd import workloads as wl

from helpers import bf16_bits_to_f64


def rand_bits(shape, seed):
    return wl.randn_bf16(shape, wl.generator(40, seed))


def test_linear_view_equals_brute_force():
    M, rows, cols = 3, 8, 12
    x, w = rand_bits((M, 6), 1), rand_bits((rows, cols), 2)
    view = ow.WeightView(((1, 2), (5, 3)), 4, 6)
    got = ow.linear_view(x, w, view)
    xf, wf = bf16_bits_to_f64(x), bf16_bits_to_f64(w)
    phys = [1, 2, 5, 6, 7]
    for i in range(M):
        for j, pr in enumerate(phys):
            acc = 0.0
            for k in range(6):
                acc += xf[i, k] * wf[pr, 4 + k]
            assert abs(got[i, j] - acc) < 1e-12
    assert got.shape == (M, 5)


@pytest.mark.parametrize("m", [1, 2, 4, 8])
def test_views_partition_the_weight(m):
    rows, cols = 64, 32
    seen_r, seen_c = [], []
    for r in range(m):
        v0, v1 = ow.weight_view(0, r, m, rows, cols), ow.weight_view(1, r, m, rows, cols)
        assert (v0.col_start, v0.col_count) == (0, cols) and v1.row_segments == ((0, rows),)
        seen_r += v0.row_index().tolist()
        seen_c += list(range(v1.col_start, v1.col_start + v1.col_count))
    assert seen_r == list(range(rows)) and seen_c == list(range(cols))
    # fused QKV: every stored row owned once; rank r's K/V heads are the KV view's head range
    hq, hkv, d, hidden = 32, 8, 128, 64
    owned = np.concatenate([ow.weight_view_fused_qkv(hq, hkv, d, hidden, r, m).row_index() for r in range(m)])
    assert sorted(owned.tolist()) == list(range((hq + 2 * hkv) * d))
    import oracle
    for r in range(m):
        v = ow.weight_view_fused_qkv(hq, hkv, d, hidden, r, m)
        info = oracle.View(oracle.Geometry(hq, hkv, d, 16), oracle.LAYOUT_TP, m, r).query()
        (qa, qn), (ka, kn), (va, vn) = v.row_segments
        assert qa == r * info["n_q_local"] * d and qn == info["n_q_local"] * d
        assert ka == hq * d + info["kv_head0"] * d and kn == info["n_kv_local"] * d
        assert va == (hq + hkv) * d + info["kv_head0"] * d and vn == kn
    with pytest.raises(ValueError):
        ow.weight_view(0, m, m, rows, cols)
    with pytest.raises(ValueError):
        ow.weight_view_fused_qkv(hq, 6, d, hidden, 0, 4)


@pytest.mark.parametrize("m", [2, 4])
def test_megatron_identities(m):
    """Column-parallel: the ranks' outputs, put back in head order, are the full layer's output.
    Row-parallel: the ranks' partial outputs add up to the full layer's output."""
    hq, hkv, d, hidden, M = 8, 4, 16, 48, 5
    x = rand_bits((M, hidden), 3)
    wqkv = rand_bits(((hq + 2 * hkv) * d, hidden), 4)
    full = ow.linear_view(x, wqkv, ow.weight_view(0, 0, 1, wqkv.shape[0], hidden))
    rebuilt = np.zeros_like(full)
    for r in range(m):
        v = ow.weight_view_fused_qkv(hq, hkv, d, hidden, r, m)
        rebuilt[:, v.row_index()] = ow.linear_view(x, wqkv, v)
    np.testing.assert_array_equal(rebuilt, full)

    wo = rand_bits((hidden, hq * d), 5)
    a = rand_bits((M, hq * d), 6)
    whole = ow.linear_view(a, wo, ow.weight_view(1, 0, 1, hidden, hq * d))
    parts = np.zeros_like(whole)
    for r in range(m):
        v = ow.weight_view(1, r, m, hidden, hq * d)
        parts += ow.linear_view(np.ascontiguousarray(a[:, v.col_start:v.col_start + v.col_count]), wo, v)
    np.testing.assert_allclose(parts, whole, rtol=0, atol=1e-10)
