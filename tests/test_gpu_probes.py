"""The measurement aids of the library do what their declarations say (they are not part of the method,
but bench.py and the profiles rely on them)."""
import numpy as np
import pytest
import torch

from paper_2602_22593_amd import binding as kv

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_placement_probe_records_every_workgroup():
    n_wg = torch.cuda.get_device_properties(0).multi_processor_count
    src = torch.empty(64 << 20, dtype=torch.uint8, device=DEV).random_(0, 255)
    rec = kv.kv_probe_read_placed(src, n_wg)
    torch.cuda.synchronize()
    rec = rec.cpu().numpy()
    assert rec.shape == (n_wg, 3)
    assert ((rec[:, 0] >= 0) & (rec[:, 0] < 8)).all()            # an XCD number
    assert (rec[:, 2] > rec[:, 1]).all()                          # ended after it started
    assert (rec[:, 2] - rec[:, 1]).max() < 100 * 1000 * 100       # well under a second of 100 MHz ticks
    assert len(np.unique(rec[:, 0])) == 8                         # a full launch reaches every XCD


def test_copy_probe_copies():
    src = torch.empty(1 << 20, dtype=torch.uint8, device=DEV).random_(0, 255)
    dst = torch.zeros_like(src)
    kv.kv_probe_copy(dst, src, 64)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
