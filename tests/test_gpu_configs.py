"""GPU parity at the benchmark configurations' real shapes and sizes.

Small configurations are compared with the oracle element by element; at the large ones the
oracle evaluates sampled bucket ranges (the random stream is counter based, so any range can be
evaluated in isolation with elem_base = its first element) and the rest is covered by properties
that hold at any size.  Oracle inputs are always the generated gradients, never library output.
"""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_1804_08066_amd import mqgrad, workloads
from helpers import to_u32, ulp_distance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sample_starts(n, span, k, seed):
    """k range starts (multiples of span), always including the first and the last (ragged) range."""
    nr = (n + span - 1) // span
    rng = np.random.default_rng(seed)
    picks = set(rng.integers(0, nr, size=k).tolist()) | {0, nr - 1, max(0, nr - 2)}
    return sorted(p * span for p in picks)


def check_quantize_ranges(g, pk, sc, bits, bucket, seed, it, wk, starts, span, elem_base=0):
    n = g.numel()
    for lo in starts:
        hi = min(n, lo + span)
        gh = g[lo:hi].cpu().numpy()
        pk_o, sc_o = ref.quantize(gh, bits, bucket, seed, it, wk, elem_base + lo)
        w0 = lo * bits // 32
        got_pk = to_u32(pk[w0:w0 + pk_o.size])
        got_sc = sc[lo // bucket: lo // bucket + sc_o.size].cpu().numpy()
        assert np.array_equal(got_sc, sc_o), "scales differ in range starting at %d" % lo
        assert np.array_equal(got_pk, pk_o), "packed words differ in range starting at %d" % lo


# ---- configuration 2: small-CNN layer tensors, W = 4, 100 iterations -----------------------------

def test_config2_training_loop_stays_on_the_oracle():
    W, bucket, lr, iters, seed = 4, 512, 0.1, 100, 0
    shapes = workloads.SMALL_CNN_SHAPES
    bases = workloads.config2_elem_bases(bucket)
    bits_seq = workloads.config2_bits_sequence(iters, seed)
    assert set(bits_seq) <= {1, 2, 4, 8} and len(set(bits_seq)) == 4
    params = workloads.config2_params(seed, DEV)
    p_ref = [p.cpu().numpy().copy() for p in params]
    assert sum(n for _, n in shapes) == 1068298
    for it in range(iters):
        bits = bits_seq[it]
        grads = [workloads.config2_grads(it, w, seed, DEV) for w in range(W)]
        for li, (_, n) in enumerate(shapes):
            outs = [mqgrad.mqg_quantize(grads[w][li], bits, bucket, seed=seed + w, iteration=it, worker=w,
                                        elem_base=bases[li]) for w in range(W)]
            mqgrad.mqg_aggregate_update([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket, lr, params[li])
            want = [ref.quantize(grads[w][li].cpu().numpy(), bits, bucket, seed + w, it, w, bases[li]) for w in range(W)]
            for w in range(W):
                assert np.array_equal(to_u32(outs[w][0]), want[w][0]), "it %d layer %d worker %d codes" % (it, li, w)
                assert np.array_equal(outs[w][1].cpu().numpy(), want[w][1]), "it %d layer %d worker %d scales" % (it, li, w)
            p_ref[li] = ref.aggregate_update([x[0] for x in want], [x[1] for x in want], n, bits, bucket, lr, p_ref[li])
        # after EVERY iteration the parameters equal the oracle's: nothing accumulates
        for li in range(len(shapes)):
            got = params[li].cpu().numpy()
            assert np.all(np.abs(got.astype(np.float64) - p_ref[li]) <= 1e-6 * np.maximum(np.abs(p_ref[li]), 1e-6)), \
                "iteration %d layer %d" % (it, li)
            assert ulp_distance(got, p_ref[li]).max() == 0, "iteration %d layer %d: not bit-equal" % (it, li)


# ---- configuration 3: 25.6M elements, W = 8, straddling widths ----------------------------------

@pytest.fixture(scope="module")
def config3_grads():
    return [workloads.config3_grad(w, 25_600_000, DEV) for w in range(8)]


def test_config3_full_oracle_one_point(config3_grads):
    # one (b, bucket) point against the oracle in full: every word of every worker, every parameter
    n, bits, bucket, lr, W = 25_600_000, 5, 512, 0.05, 8
    params = workloads.uniform(n, -0.05, 0.05, 33, DEV)
    p0 = params.cpu().numpy().copy()
    outs = [mqgrad.mqg_quantize(config3_grads[w], bits, bucket, seed=3, iteration=1, worker=w) for w in range(W)]
    mqgrad.mqg_aggregate_update([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket, lr, params)
    torch.cuda.synchronize()
    want = []
    for w in range(W):
        pk_o, sc_o = ref.quantize(config3_grads[w].cpu().numpy(), bits, bucket, 3, 1, w)
        assert np.array_equal(outs[w][1].cpu().numpy(), sc_o)
        assert np.array_equal(to_u32(outs[w][0]), pk_o)
        want.append((pk_o, sc_o))
    p_ref = ref.aggregate_update([x[0] for x in want], [x[1] for x in want], n, bits, bucket, lr, p0)
    got = params.cpu().numpy()
    assert ulp_distance(got, p_ref).max() == 0
    # outliers (0.1% at 100x) put most of an outlier bucket's elements on the two middle codes
    codes = ref.unpack(want[0][0][: 512 * bits // 32 * 64], 512 * 64, bits)
    assert np.isin(codes, [15, 16]).mean() > 0.2


@pytest.mark.parametrize("bucket", [128, 512, 2048])
def test_config3_sampled_ranges(config3_grads, bucket):
    n, W, lr = 25_600_000, 8, 0.05
    span = 4 * 2048
    for bits in (3, 5, 6, 7):
        params = workloads.uniform(n, -0.05, 0.05, 33, DEV)
        p0 = params.clone()
        outs = [mqgrad.mqg_quantize(config3_grads[w], bits, bucket, seed=3, iteration=bits, worker=w) for w in range(W)]
        mqgrad.mqg_aggregate_update([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket, lr, params)
        torch.cuda.synchronize()
        starts = sample_starts(n, span, 6, seed=bits * 7 + bucket)
        for w in (0, 5):
            check_quantize_ranges(config3_grads[w], outs[w][0], outs[w][1], bits, bucket, 3, bits, w, starts, span)
        for lo in starts[:4] + starts[-1:]:
            hi = min(n, lo + span)
            want = [ref.quantize(config3_grads[w][lo:hi].cpu().numpy(), bits, bucket, 3, bits, w, lo) for w in range(W)]
            p_ref = ref.aggregate_update([x[0] for x in want], [x[1] for x in want], hi - lo, bits, bucket, lr,
                                         p0[lo:hi].cpu().numpy())
            assert ulp_distance(params[lo:hi].cpu().numpy(), p_ref).max() == 0, "b=%d B=%d range %d" % (bits, bucket, lo)


# ---- configuration 4: 100M elements, W = 8, the benchmark's launch configuration ----------------

def test_config4_sampled_ranges_and_global_properties():
    n, W, lr = 100_000_000, 8, 0.1
    grads = [workloads.config4_grad(w, n, DEV) for w in range(W)]
    span = 16384
    for bucket in (128, 1024, 8192):
        for bits in (1, 2, 4, 8):
            params = workloads.uniform(n, -0.05, 0.05, 1, DEV)
            p0 = params.clone()
            outs = [mqgrad.mqg_quantize(grads[w], bits, bucket, seed=1234, iteration=bits, worker=w) for w in range(W)]
            mqgrad.mqg_aggregate_update([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket, lr, params)
            torch.cuda.synchronize()
            starts = sample_starts(n, span, 3, seed=bits + bucket)
            check_quantize_ranges(grads[2], outs[2][0], outs[2][1], bits, bucket, 1234, bits, 2, starts, span)
            for lo in starts[:2] + starts[-1:]:
                hi = min(n, lo + span)
                want = [ref.quantize(grads[w][lo:hi].cpu().numpy(), bits, bucket, 1234, bits, w, lo) for w in range(W)]
                p_ref = ref.aggregate_update([x[0] for x in want], [x[1] for x in want], hi - lo, bits, bucket, lr,
                                             p0[lo:hi].cpu().numpy())
                assert ulp_distance(params[lo:hi].cpu().numpy(), p_ref).max() == 0, "b=%d B=%d range %d" % (bits, bucket, lo)
            # properties at full size: scales are the bucket maxima; the step is bounded by lr * mean scale
            nb = mqgrad.mqg_num_buckets(n, bucket)
            full = (n // bucket) * bucket
            smax = grads[0][:full].abs().view(-1, bucket).amax(dim=1)
            assert torch.equal(outs[0][1][: n // bucket], smax)
            if full < n:
                assert outs[0][1][nb - 1] == grads[0][full:].abs().max()
            mean_scale = torch.stack([o[1] for o in outs]).mean(dim=0)
            bound = lr * mean_scale.repeat_interleave(bucket)[:n] * (1 + 1e-5) + 1e-9
            assert bool(((params - p0).abs() <= bound).all())


def test_config4_size_with_buckets_that_are_not_powers_of_two():
    # the cell-granular quantizer at the benchmark's size: sampled ranges against the oracle (ranges start on
    # bucket boundaries), every scale against the bucket maxima, and the server step on the same ranges
    n, W, lr = 100_000_000, 2, 0.1
    grads = [workloads.config4_grad(w, n, DEV) for w in range(W)]
    for bucket in (96, 1504, 2752):
        span = bucket * (16384 // bucket)
        for bits in (1, 4, 7):
            params = workloads.uniform(n, -0.05, 0.05, 1, DEV)
            p0 = params.clone()
            outs = [mqgrad.mqg_quantize(grads[w], bits, bucket, seed=99, iteration=bits, worker=w) for w in range(W)]
            mqgrad.mqg_aggregate_update([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket, lr, params)
            torch.cuda.synchronize()
            starts = sample_starts(n, span, 3, seed=bits + bucket)
            check_quantize_ranges(grads[1], outs[1][0], outs[1][1], bits, bucket, 99, bits, 1, starts, span)
            for lo in starts[:1] + starts[-1:]:
                hi = min(n, lo + span)
                want = [ref.quantize(grads[w][lo:hi].cpu().numpy(), bits, bucket, 99, bits, w, lo) for w in range(W)]
                p_ref = ref.aggregate_update([x[0] for x in want], [x[1] for x in want], hi - lo, bits, bucket, lr,
                                             p0[lo:hi].cpu().numpy())
                assert ulp_distance(params[lo:hi].cpu().numpy(), p_ref).max() == 0, "b=%d B=%d range %d" % (bits, bucket, lo)
            nb = mqgrad.mqg_num_buckets(n, bucket)
            full = (n // bucket) * bucket
            smax = grads[0][:full].abs().view(-1, bucket).amax(dim=1)
            assert torch.equal(outs[0][1][: n // bucket], smax), "B=%d b=%d" % (bucket, bits)
            if full < n:
                assert outs[0][1][nb - 1] == grads[0][full:].abs().max()
            del outs


def test_config4_exchange_and_minmax_on_sampled_ranges():
    # the widened rows at the benchmark's full size and launch configuration: the re-quantized mean, the
    # worker's update from it, and the deterministic [min, max] encoding with its server step
    n, W, lr, span = 100_000_000, 8, 0.1, 16384
    grads = [workloads.config4_grad(w, n, DEV) for w in range(W)]
    for bucket, bits in ((1024, 4), (128, 1), (8192, 8), (1024, 5)):
        params = workloads.uniform(n, -0.05, 0.05, 1, DEV)
        p0 = params.clone()
        outs = [mqgrad.mqg_quantize(grads[w], bits, bucket, seed=77, iteration=1, worker=w) for w in range(W)]
        mean_pk, mean_sc = mqgrad.mqg_aggregate_requantize([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket,
                                                           seed=77, iteration=1, worker=W)
        mqgrad.mqg_dequantize_update(mean_pk, mean_sc, n, bits, bucket, lr, params)
        torch.cuda.synchronize()
        starts = sample_starts(n, span, 2, seed=bits * 3 + bucket)
        for lo in starts:
            hi = min(n, lo + span)
            want = [ref.quantize(grads[w][lo:hi].cpu().numpy(), bits, bucket, 77, 1, w, lo) for w in range(W)]
            m_pk, m_sc = ref.aggregate_requantize([x[0] for x in want], [x[1] for x in want], hi - lo, bits, bucket,
                                                  77, 1, W, lo)
            w0 = lo * bits // 32
            assert np.array_equal(mean_sc[lo // bucket: lo // bucket + m_sc.size].cpu().numpy(), m_sc)
            assert np.array_equal(to_u32(mean_pk[w0:w0 + m_pk.size]), m_pk), "b=%d B=%d range %d" % (bits, bucket, lo)
            p_ref = ref.dequantize_update(m_pk, m_sc, hi - lo, bits, bucket, lr, p0[lo:hi].cpu().numpy())
            assert ulp_distance(params[lo:hi].cpu().numpy(), p_ref).max() == 0
        del outs, mean_pk, mean_sc

        params = p0.clone()
        mm = [mqgrad.mqg_quantize_minmax(grads[w], bits, bucket) for w in range(W)]
        mqgrad.mqg_aggregate_update_minmax([m[0] for m in mm], [m[1] for m in mm], n, bits, bucket, lr, params)
        torch.cuda.synchronize()
        for lo in starts:
            hi = min(n, lo + span)
            want = [ref.quantize_minmax(grads[w][lo:hi].cpu().numpy(), bits, bucket) for w in range(W)]
            w0 = lo * bits // 32
            for w in (0, W - 1):
                assert np.array_equal(mm[w][1][2 * (lo // bucket): 2 * (lo // bucket) + want[w][1].size].cpu().numpy(), want[w][1])
                assert np.array_equal(to_u32(mm[w][0][w0:w0 + want[w][0].size]), want[w][0])
            p_ref = ref.aggregate_update_minmax([x[0] for x in want], [x[1] for x in want], hi - lo, bits, bucket, lr,
                                                p0[lo:hi].cpu().numpy())
            assert ulp_distance(params[lo:hi].cpu().numpy(), p_ref).max() == 0
        # at full size: the stored ranges are the bucket minima and maxima
        full = (n // bucket) * bucket
        v = grads[0][:full].view(-1, bucket)
        assert torch.equal(mm[0][1][0:2 * (n // bucket):2], v.amin(dim=1))
        assert torch.equal(mm[0][1][1:2 * (n // bucket):2], v.amax(dim=1))
        ss = mqgrad.mqg_sum_squares(grads[0])
        torch.cuda.synchronize()
        want_ss = float((grads[0].double() ** 2).sum().item())
        assert abs(ss.item() - want_ss) <= 1e-11 * want_ss
        del mm


# ---- configuration 5: 1B parameters, W = 16, bit width chosen by the host MDP --------------------

def test_config5_large_model_with_mdp_policy():
    n, W, bucket, lr, iters = 1_000_000_000, 16, 1024, 0.05, 20
    losses = workloads.synthetic_loss_sequence(iters, seed=2)
    agent = mqgrad.Mdp(seed=2, bits_min=1, bits_max=8, decide_every=1, epsilon=0.3)
    params = torch.zeros(n, dtype=torch.float32, device=DEV)
    packed = [torch.empty(mqgrad.mqg_packed_words(n, 8), dtype=torch.int32, device=DEV) for _ in range(W)]
    scales = [torch.empty(mqgrad.mqg_num_buckets(n, bucket), dtype=torch.float32, device=DEV) for _ in range(W)]
    span = 4096
    starts = sample_starts(n, span, 2, seed=11)       # includes the ragged tail: 1e9 % 1024 = 512
    p_ref = {lo: np.zeros(min(n, lo + span) - lo, dtype=np.float32) for lo in starts}
    seen_bits = []
    cost = 0.0
    for it in range(iters):
        bits = agent.step(losses[it], cost)
        seen_bits.append(bits)
        cost = 40.0 + 5.0 * bits                        # deterministic cost model: the b sequence is reproducible
        want = {lo: [] for lo in starts}
        for w in range(W):
            g = workloads.config5_grad(w, it, n, DEV)
            mqgrad.mqg_quantize(g, bits, bucket, seed=55, iteration=it, worker=w, packed_out=packed[w], scales_out=scales[w])
            for lo in starts:
                hi = min(n, lo + span)
                want[lo].append(ref.quantize(g[lo:hi].cpu().numpy(), bits, bucket, 55, it, w, lo))
                w0 = lo * bits // 32
                assert np.array_equal(to_u32(packed[w][w0:w0 + want[lo][-1][0].size]), want[lo][-1][0]), \
                    "it %d worker %d range %d" % (it, w, lo)
            del g
        mqgrad.mqg_aggregate_update(packed, scales, n, bits, bucket, lr, params)
        torch.cuda.synchronize()
        for lo in starts:
            hi = min(n, lo + span)
            p_ref[lo] = ref.aggregate_update([x[0] for x in want[lo]], [x[1] for x in want[lo]], hi - lo, bits, bucket, lr, p_ref[lo])
            assert ulp_distance(params[lo:hi].cpu().numpy(), p_ref[lo]).max() == 0, "it %d range %d" % (it, lo)
    assert all(1 <= b <= 8 for b in seen_bits) and len(set(seen_bits)) >= 3     # the policy did switch widths (1, 3, 4)
    assert bool(torch.isfinite(params[-4096:]).all()) and float(params.abs().max()) > 0
