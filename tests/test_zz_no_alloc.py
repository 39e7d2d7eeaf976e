"""The entry point that allocates nothing (mqg_sum_squares_batch_static: partial sums in the library's own
device array) against the one that takes a caller workspace, through the C ABI: bit-identical results on
two calls in a row, the second with smaller inputs, and the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_1804_08066_amd import mqgrad, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(grads):
    count = len(grads)
    L = mqgrad.lib()
    items = (mqgrad.SumsqItem * count)()
    for k, g in enumerate(grads):
        items[k].grad, items[k].n = g.data_ptr(), g.numel()
    ws = torch.empty(L.mqg_sum_squares_workspace_bytes(count) // 8, dtype=torch.float64, device=DEV)
    want = torch.full((count,), -1.0, dtype=torch.float64, device=DEV)
    got = torch.full((count,), -2.0, dtype=torch.float64, device=DEV)
    assert L.mqg_sum_squares_batch(items, count, ws.data_ptr(), want.data_ptr(), None) == mqgrad.MQG_OK
    assert L.mqg_sum_squares_batch_static(items, count, got.data_ptr(), None) == mqgrad.MQG_OK
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    torch.cuda.set_device(0)
    big = [workloads.normal(n, 10.0 ** -(k % 3 + 1), 900 + k, DEV) for k, n in
           enumerate([3_000_011, 1 << 21, 2048 * 512 * 2 + 5, 77, 1])]
    got, want = both(big)
    assert got.tobytes() == want.tobytes()
    assert np.all(got > 0)
    exact = float(np.sum(big[0].cpu().numpy().astype(np.float64) ** 2))
    assert abs(got[0] - exact) <= 1e-12 * exact
    # second call, fewer and smaller tensors: what the first call left in the array must not matter
    small = [workloads.normal(n, 1e-3, 950 + k, DEV) for k, n in enumerate([5, 4099])]
    got2, want2 = both(small)
    assert got2.tobytes() == want2.tobytes()
    exact2 = float(np.sum(small[1].cpu().numpy().astype(np.float64) ** 2))
    assert abs(got2[1] - exact2) <= 1e-12 * exact2
    # and the first inputs again give the first result to the bit
    got3, _ = both(big)
    assert got3.tobytes() == got.tobytes()


def test_static_scratch_entry_point_rejects_more_tensors_than_its_array_holds():
    L = mqgrad.lib()
    g = workloads.normal(64, 1.0, 1, DEV)
    out = torch.zeros(80, dtype=torch.float64, device=DEV)
    items = (mqgrad.SumsqItem * 65)()
    for it in items:
        it.grad, it.n = g.data_ptr(), 64
    assert L.mqg_sum_squares_batch_static(items, 65, out.data_ptr(), None) == mqgrad.MQG_EINVAL
    assert L.mqg_sum_squares_batch_static(items, 64, out.data_ptr(), None) == mqgrad.MQG_OK
    assert L.mqg_sum_squares_batch_static(items, 0, None, None) == mqgrad.MQG_OK
    assert L.mqg_sum_squares_batch_static(None, 2, out.data_ptr(), None) == mqgrad.MQG_EINVAL
    assert L.mqg_sum_squares_batch_static(items, 2, None, None) == mqgrad.MQG_EINVAL
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = float(np.sum(g.cpu().numpy().astype(np.float64) ** 2))
    assert np.all(np.abs(got[:64] - want) <= 1e-12 * want) and np.all(got[64:] == 0)
