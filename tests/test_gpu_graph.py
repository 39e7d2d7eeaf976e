"""The entry points allocate nothing, keep no state and clear memory with kernels only, so a whole
step can be captured into a HIP graph and replayed: every replay must give what eager launches give."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_1804_08066_amd import mqgrad, workloads
from helpers import to_u32, ulp_distance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_captured_step_replays_like_eager_launches():
    n, W, bits, bucket, lr = 300000 + 17, 4, 5, 512, 0.1
    grads = [workloads.normal(n, 0.01, 50 + w, DEV) for w in range(W)]
    outs = [mqgrad.alloc_outputs(n, bits, bucket, DEV) for _ in range(W)]
    mm = [(torch.empty(mqgrad.mqg_packed_words(n, bits), dtype=torch.int32, device=DEV),
           torch.empty(2 * mqgrad.mqg_num_buckets(n, bucket), dtype=torch.float32, device=DEV)) for _ in range(W)]
    params = workloads.uniform(n, -0.05, 0.05, 3, DEV)
    params_mm = params.clone()
    sumsq = torch.zeros(1, dtype=torch.float64, device=DEV)
    p_host = params.cpu().numpy().copy()
    pm_host = p_host.copy()

    def step():
        for w in range(W):
            mqgrad.mqg_quantize(grads[w], bits, bucket, seed=9, iteration=3, worker=w, packed_out=outs[w][0],
                                scales_out=outs[w][1])
            mqgrad.mqg_quantize_minmax(grads[w], bits, bucket, mm[w][0], mm[w][1])
        mqgrad.mqg_aggregate_update([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket, lr, params)
        mqgrad.mqg_aggregate_update_minmax([m[0] for m in mm], [m[1] for m in mm], n, bits, bucket, lr, params_mm)
        mqgrad.mqg_sum_squares(grads[0], sumsq)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    params.copy_(torch.from_numpy(p_host))
    params_mm.copy_(torch.from_numpy(pm_host))

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    # capture launches nothing: the parameters are still the initial ones
    assert np.array_equal(params.cpu().numpy(), p_host)

    want = [ref.quantize(g.cpu().numpy(), bits, bucket, 9, 3, w) for w, g in enumerate(grads)]
    want_mm = [ref.quantize_minmax(g.cpu().numpy(), bits, bucket) for g in grads]
    exact_ss = float(np.sum(grads[0].cpu().numpy().astype(np.float64) ** 2))
    for replay in range(4):
        graph.replay()
        torch.cuda.synchronize()
        p_host = ref.aggregate_update([x[0] for x in want], [x[1] for x in want], n, bits, bucket, lr, p_host)
        pm_host = ref.aggregate_update_minmax([x[0] for x in want_mm], [x[1] for x in want_mm], n, bits, bucket, lr,
                                              pm_host)
        for w in range(W):
            assert np.array_equal(to_u32(outs[w][0]), want[w][0]), "replay %d worker %d" % (replay, w)
            assert np.array_equal(to_u32(mm[w][0]), want_mm[w][0])
        assert ulp_distance(params.cpu().numpy(), p_host).max() == 0, "replay %d" % replay
        assert ulp_distance(params_mm.cpu().numpy(), pm_host).max() == 0, "replay %d" % replay
        assert abs(sumsq.item() - exact_ss) <= 1e-12 * exact_ss
        # eager work and a synchronisation between the replays
        outs[0][0].zero_()
        sumsq.fill_(123.0)
        torch.cuda.synchronize()


def test_workers_on_concurrent_streams_give_the_sequential_result():
    # the library keeps no state between or across calls: W quantize calls in flight on W streams at
    # once (default priority) write exactly what they write one after the other
    n, W, bits, bucket = 3_000_000 + 5, 6, 3, 2048
    grads = [workloads.laplace(n, 1e-3, 20 + w, DEV) for w in range(W)]
    seq = [mqgrad.mqg_quantize(g, bits, bucket, seed=8, iteration=4, worker=w) for w, g in enumerate(grads)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(W)]
    outs = [mqgrad.alloc_outputs(n, bits, bucket, DEV) for _ in range(W)]
    for rep in range(3):
        for w in range(W):
            outs[w][0].zero_()
        torch.cuda.synchronize()
        for w in range(W):
            mqgrad.mqg_quantize(grads[w], bits, bucket, seed=8, iteration=4, worker=w, packed_out=outs[w][0],
                                scales_out=outs[w][1], stream=streams[w])
        torch.cuda.synchronize()
        for w in range(W):
            assert torch.equal(outs[w][0], seq[w][0]) and torch.equal(outs[w][1], seq[w][1]), "stream %d rep %d" % (w, rep)
    params_a = workloads.uniform(n, -0.05, 0.05, 1, DEV)
    params_b = params_a.clone()
    mqgrad.mqg_aggregate_update([o[0] for o in seq], [o[1] for o in seq], n, bits, bucket, 0.1, params_a)
    with torch.cuda.stream(streams[0]):
        mqgrad.mqg_aggregate_update([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket, 0.1, params_b)
    torch.cuda.synchronize()
    assert torch.equal(params_a, params_b)
