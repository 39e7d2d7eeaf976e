#!/usr/bin/env python3
"""Benchmark of the MQGrad hot path on one MI355X.

A step is one training iteration's worth of gradient traffic through the whole path: W workers'
fp32 gradients are each quantized and packed (mqg_quantize), then the server unpacks, de-quantizes
and averages the W streams and updates the parameters (mqg_aggregate_update).  Inputs are resident
in HBM before the timed region.  `value` is GB/s of fp32 gradient processed (4*N*W bytes per step).

The headline workload is the bandwidth-sweep configuration: a flat 100M-element gradient
~ N(0, 0.01^2), W = 8 worker buffers, at b = 4 bits and bucket 1024; `--sweep` adds the whole
(b, bucket) grid to the JSON line.  Synthetic data stands in for the paper's CIFAR-10 CNN
gradients (Section 4.1); the paper reports no throughput for this path.

One JSON line on stdout; progress on stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

PROFILES = os.path.join(ROOT, "profiles")
TRAFFIC_PROFILE = os.path.join(PROFILES, "quantize_aggregate_100M_W8_b4_B1024_hbm_traffic.md")
MACHINE_STATE_PROFILE = os.path.join(PROFILES, "machine_state_100M_W8_b4_B1024.md")


def measured_traffic(n, W, bits, bucket):
    """HBM bytes per launch of the two hot kernels as rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE read them
    (scaled by a copy of known size), taken from the tracked summary of that measurement: its line
    `traffic_json: {...}` names the workload and the commit it was measured at.  A workload that was
    not profiled reports null."""
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("traffic_json:"):
                d = json.loads(line[len("traffic_json:"):])
                wl = d["workload"]
                if (wl["n"], wl["workers"], wl["bits"], wl["bucket"]) == (n, W, bits, bucket):
                    return d
    except (OSError, ValueError, KeyError):
        pass
    return None


def load_clock_mhz():
    """Engine clock under sustained load as the tracked machine-state summary recorded it (rocm-smi)."""
    try:
        for line in open(MACHINE_STATE_PROFILE):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 3 and cells[1] == "under load" and cells[2].isdigit():
                return int(cells[2])
    except OSError:
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def quantize_bytes(n, bits, bucket):
    """Algorithmic bytes of one quantize launch: read the gradient once, write codes and scales once."""
    return 4.0 * n + n * bits / 8.0 + 4.0 * ((n + bucket - 1) // bucket)


def aggregate_bytes(n, bits, bucket, W):
    """Algorithmic bytes of one aggregate_update launch: W code streams + scales in, parameters in and out."""
    return W * (n * bits / 8.0 + 4.0 * ((n + bucket - 1) // bucket)) + 8.0 * n


class Workload:
    dest = None   # mqg_quantize's cache policy for the code words (None: the library's default, keep cached)

    def __init__(self, n, W, device, buffers=0):
        """W workers over `buffers` distinct gradient buffers (0: one per worker); worker w reads buffer
        w % buffers -- for shapes whose W full-size gradients would not fit beside the code streams."""
        import torch
        from paper_1804_08066_amd import workloads
        self.n, self.W, self.device = n, W, device
        G = W if buffers <= 0 else min(buffers, W)
        log("generating %d gradient buffers of %d fp32 (%.2f GB) for %d workers" % (G, n, 4e-9 * n * G, W))
        distinct = [workloads.config4_grad(w, n, device) for w in range(G)]
        self.grads = [distinct[w % G] for w in range(W)]
        self.params = workloads.uniform(n, -0.05, 0.05, 1, device)
        self.bufs = {}
        torch.cuda.synchronize()

    def outputs(self, bits, bucket):
        from paper_1804_08066_amd import mqgrad
        key = (bits, bucket)
        if key not in self.bufs:
            self.bufs.clear()
            self.bufs[key] = [mqgrad.alloc_outputs(self.n, bits, bucket, self.device) for _ in range(self.W)]
        return self.bufs[key]


def run_steps(wl, bits, bucket, lr, steps, iteration0, events=None):
    """Enqueue `steps` iterations.  events: optional list that receives (e0, e1, e2) per step."""
    import torch
    from paper_1804_08066_amd import mqgrad
    outs = wl.outputs(bits, bucket)
    pk = [o[0] for o in outs]
    sc = [o[1] for o in outs]
    for k in range(steps):
        if events is not None:
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            ev[0].record()
        for w in range(wl.W):
            mqgrad.mqg_quantize(wl.grads[w], bits, bucket, seed=1234, iteration=iteration0 + k, worker=w,
                                packed_out=pk[w], scales_out=sc[w], dest=wl.dest)
        if events is not None:
            ev[1].record()
        mqgrad.mqg_aggregate_update(pk, sc, wl.n, bits, bucket, lr, wl.params)
        if events is not None:
            ev[2].record()
            events.append(ev)


def time_config(wl, bits, bucket, lr, steps, warmup):
    """`warmup` untimed steps, then exactly `steps` steps between two synchronizations.  Returns
    (ms per step by the host clock, ms per quantize launch, ms per aggregate launch) with the launch
    times from HIP events on the launch stream; time_config.last holds the spread of the per-step series."""
    import torch
    run_steps(wl, bits, bucket, lr, warmup, 0)
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    run_steps(wl, bits, bucket, lr, steps, warmup, events)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    q_series = [e[0].elapsed_time(e[1]) / wl.W for e in events]             # per quantize launch, one value per step
    a_series = [e[1].elapsed_time(e[2]) for e in events]                    # per aggregate launch
    q_all, a_all = sorted(q_series), sorted(a_series)
    q_ms, a_ms = sum(q_all) / steps, sum(a_all) / steps
    head = min(5, steps)
    time_config.last = {"quantize_us_median": q_all[steps // 2] * 1e3, "quantize_us_min": q_all[0] * 1e3,
                        "quantize_us_first5": sum(q_series[:head]) / head * 1e3,
                        "aggregate_us_median": a_all[steps // 2] * 1e3, "aggregate_us_min": a_all[0] * 1e3,
                        "aggregate_us_first5": sum(a_series[:head]) / head * 1e3}
    return (t1 - t0) / steps * 1e3, q_ms, a_ms


def choose_code_stores(wl, bits, bucket, lr, policy):
    """The quantizer's cache policy for the code words (mqg_quantize_to): kept in the last-level cache for the
    update that follows, or streamed to memory.  Which is faster depends on how the W streams together sit
    in that cache; a caller knows W, the library does not, so the caller chooses: here, under "auto", by
    timing a few untimed steps each way (streaming stores must win by more than 1 % to be taken).  Sets
    wl.dest and returns what was decided."""
    from paper_1804_08066_amd import mqgrad
    stores = {"policy": policy}
    if policy == "auto":
        probe = {}
        for name, dest in (("cached", None), ("stream", mqgrad.MQG_CODES_TO_MEMORY)):
            wl.dest = dest
            probe[name] = time_config(wl, bits, bucket, lr, 10, 5)[0]
        stores["probe_ms_per_step"] = probe
        stores["chosen"] = "stream" if probe["stream"] < 0.99 * probe["cached"] else "cached"
    else:
        stores["chosen"] = policy
    wl.dest = mqgrad.MQG_CODES_TO_MEMORY if stores["chosen"] == "stream" else None
    return stores


def condition(wl, bits, bucket, lr, ms):
    """Untimed steps of the benchmark's own loop until `ms` milliseconds have passed.  After any idle gap
    (even the half second a synchronize and a child process take) the chip runs about three steps at
    boost clocks, drops into a throttled state and recovers over some 20 ms (profiles/transient_*.md): a
    region timed right after input generation measures that state, not the one a training loop runs in."""
    import torch
    t0 = time.perf_counter()
    done = 0
    while (time.perf_counter() - t0) * 1e3 < ms:
        run_steps(wl, bits, bucket, lr, 8, done)
        done += 8
        torch.cuda.synchronize()   # keeps the queue short so that the loop ends on time
    return done, (time.perf_counter() - t0) * 1e3


def time_cold_codes(wl, bits, bucket, lr, steps=20, warmup=5, origin=0):
    """The server step when the code words are NOT in this GPU's caches -- the state on a real parameter
    server, where the W streams arrive over the network: each step quantizes as usual, then copies two
    gradient buffers (torch copy_, ordinary loads and stores: 1.6 GB through the caches, untimed) and only
    then times mqg_aggregate_update."""
    import torch
    from paper_1804_08066_amd import mqgrad
    outs = wl.outputs(bits, bucket)
    pk, sc = [o[0] for o in outs], [o[1] for o in outs]
    dst = torch.empty_like(wl.grads[0])
    ev = []
    for k in range(warmup + steps):
        for w in range(wl.W):
            mqgrad.mqg_quantize(wl.grads[w], bits, bucket, seed=1234, iteration=k, worker=w, packed_out=pk[w], scales_out=sc[w])
        for f in range(2):
            dst.copy_(wl.grads[f % wl.W])
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record()
        mqgrad.mqg_aggregate_update(pk, sc, wl.n, bits, bucket, lr, wl.params, origin=origin)
        e[1].record()
        if k >= warmup:
            ev.append(e)
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in ev) / len(ev)


_bench_lib = None


def bench_lib():
    """libmqgrad_bench.so: streaming kernels with the hot kernels' read/write mix (csrc/bench_stream.hip)."""
    global _bench_lib
    if _bench_lib is None:
        import ctypes as C
        from paper_1804_08066_amd import build
        L = C.CDLL(build.BENCH_LIB)
        L.mqg_bench_stream_quantize.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        L.mqg_bench_stream_quantize.restype = C.c_int
        L.mqg_bench_stream_update.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        L.mqg_bench_stream_update.restype = C.c_int
        L.mqg_bench_stream_read.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
        L.mqg_bench_stream_read.restype = C.c_int
        L.mqg_bench_stream_write.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        L.mqg_bench_stream_write.restype = C.c_int
        _bench_lib = L
    return _bench_lib


def stream_ceilings(wl, bits, bucket, steps=40, warmup=20):
    """What this machine's HBM gives to the two kernels' read/write mixes: the benchmark's step with each
    kernel replaced by a streaming kernel that moves the same bytes in the same launch shape with the same
    cache hints and does no arithmetic (W reads of a gradient buffer + writes of n*bits/8 bytes, then one
    pass that reads the W code streams and reads and writes the parameters).  Also a plain device copy of
    one gradient buffer (torch's copy_), for reference."""
    import ctypes as C
    import torch
    L = bench_lib()
    n8 = wl.n // 8192 * 8192
    outs = wl.outputs(bits, bucket)
    pk = [o[0] for o in outs]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    codes = (C.c_void_p * wl.W)(*[t.data_ptr() for t in pk])
    best, best_u = None, None
    for shape, label in ((0, "2048 floats per wave, 4 waves per workgroup"), (1, "1024 per wave, 4 waves"), (2, "2048 per wave, 2 waves")):
        ev = []
        for k in range(warmup + steps):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record()
            for w in range(wl.W):
                rc = L.mqg_bench_stream_quantize(wl.grads[w].data_ptr(), n8, bits, shape, pk[w].data_ptr(), stream)
                assert rc == 0, rc
            e[1].record()
            rc = L.mqg_bench_stream_update(codes, wl.W, n8, bits, shape & 1, wl.params.data_ptr(), stream)
            assert rc == 0, rc
            e[2].record()
            if k >= warmup:
                ev.append(e)
        torch.cuda.synchronize()
        q = sum(e[0].elapsed_time(e[1]) for e in ev) / len(ev) / wl.W
        u = sum(e[1].elapsed_time(e[2]) for e in ev) / len(ev)
        if best is None or q < best[0]:
            best = (q, label)
        if best_u is None or u < best_u[0]:
            best_u = (u, "at most four waves per SIMD" if shape & 1 else "up to eight waves per SIMD")
    (q_ms, q_shape), (u_ms, u_shape) = best, best_u
    q_gbs = n8 * (4.0 + bits / 8.0) / (q_ms * 1e-3) / 1e9
    u_gbs = n8 * (8.0 + wl.W * bits / 8.0) / (u_ms * 1e-3) / 1e9
    # pure read and pure write of one gradient buffer: the additive bound of a mix is its read bytes at the
    # read rate plus its written bytes at the write rate
    dst = torch.empty_like(wl.grads[0])
    sink = torch.zeros(256, dtype=torch.float32, device=wl.device)
    def pure(fn, reps=30):
        for k in range(10):
            fn(k)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for k in range(reps):
            fn(k)
            ev[k + 1].record()
        torch.cuda.synchronize()
        ts = sorted(ev[k].elapsed_time(ev[k + 1]) for k in range(reps))
        return 4.0 * n8 / (ts[reps // 2] * 1e-3) / 1e9
    def rd(k):
        assert L.mqg_bench_stream_read(wl.grads[k % wl.W].data_ptr(), n8, sink.data_ptr(), stream) == 0
    def wr(k):
        assert L.mqg_bench_stream_write(dst.data_ptr(), n8, stream) == 0
    read_gbs, write_gbs = pure(rd), pure(wr)
    q_add_us = (4.0 * n8 / read_gbs + n8 * bits / 8.0 / write_gbs) * 1e-3
    u_add_us = ((4.0 + wl.W * bits / 8.0) * n8 / read_gbs + 4.0 * n8 / write_gbs) * 1e-3
    reps = 30
    for k in range(10):
        dst.copy_(wl.grads[k % wl.W])
    cev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    cev[0].record()
    for k in range(reps):
        dst.copy_(wl.grads[k % wl.W])
        cev[k + 1].record()
    torch.cuda.synchronize()
    ts = sorted(cev[k].elapsed_time(cev[k + 1]) for k in range(reps))
    del dst
    copy_gbs = 8.0 * wl.n / (ts[reps // 2] * 1e-3) / 1e9
    return {"quantize_mix": {"kernel": "stream_quantize_kernel (bench only), best of three launch shapes: " + q_shape,
                             "us": q_ms * 1e3, "gbs": q_gbs,
                             "frac_of_peak": q_gbs / HBM_PEAK_GBS},
            "update_mix": {"kernel": "stream_update_kernel (bench only), best of two occupancy caps: " + u_shape,
                           "us": u_ms * 1e3, "gbs": u_gbs,
                           "frac_of_peak": u_gbs / HBM_PEAK_GBS},
            "pure_read": {"kernel": "stream_read_kernel (bench only)", "gbs": read_gbs, "frac_of_peak": read_gbs / HBM_PEAK_GBS},
            "pure_write": {"kernel": "stream_write_kernel (bench only)", "gbs": write_gbs, "frac_of_peak": write_gbs / HBM_PEAK_GBS},
            "additive_bound": {"what": "read bytes / pure read rate + written bytes / pure write rate",
                               "quantize_us": q_add_us, "update_us": u_add_us},
            "torch_copy": {"kernel": "torch copy_ of one gradient buffer", "gbs": copy_gbs, "frac_of_peak": copy_gbs / HBM_PEAK_GBS}}


def machine_state(wl, bits, bucket, seconds=2.0):
    """Clock levels and performance level as rocm-smi reports them, idle and while the quantize kernel
    runs back to back (a reader of the numbers wants to know what state the chip was in).  rocm-smi is
    started as a child process from a thread; the launches go on from the main thread meanwhile."""
    import re
    import subprocess
    import threading
    import torch
    from paper_1804_08066_amd import mqgrad

    def sample():
        try:
            txt = subprocess.run(["rocm-smi", "--showclocks", "--showperflevel", "--showpower"], capture_output=True,
                                 text=True, timeout=20).stdout
        except (OSError, subprocess.SubprocessError) as e:
            return {"error": str(e)}
        res = {}
        for name in ("sclk", "mclk", "fclk", "socclk"):
            m = re.search(r"GPU\[0\]\s*:\s*%s clock level: \d+: \((\d+)Mhz\)" % name, txt)
            if m:
                res[name + "_mhz"] = int(m.group(1))
        m = re.search(r"GPU\[0\]\s*:\s*Performance Level: (\w+)", txt)
        if m:
            res["performance_level"] = m.group(1)
        m = re.search(r"GPU\[0\]\s*:.*?Power.*?:\s*([\d.]+)", txt)
        if m:
            res["power_w"] = float(m.group(1))
        return res

    torch.cuda.synchronize()
    state = {"idle": sample()}
    outs = wl.outputs(bits, bucket)
    got = {}
    th = threading.Thread(target=lambda: got.update(sample()))
    t0 = time.time()
    started = False
    k = 0
    while time.time() - t0 < seconds or th.is_alive():
        for w in range(wl.W):
            mqgrad.mqg_quantize(wl.grads[w], bits, bucket, seed=1234, iteration=k, worker=w,
                                packed_out=outs[w][0], scales_out=outs[w][1])
        k += 1
        if k % 8 == 0:
            torch.cuda.synchronize()   # keep the queue short so that the loop follows the clock
        if not started and time.time() - t0 > 0.3 * seconds:
            th.start()
            started = True
    torch.cuda.synchronize()
    th.join()
    state["under_load"] = got
    state["load"] = "mqg_quantize back to back for %.1f s (b=%d, bucket=%d)" % (time.time() - t0, bits, bucket)
    return state


def smi_clocks():
    """Clock and performance levels as rocm-smi reports them (started as a child process)."""
    import re
    import subprocess
    try:
        txt = subprocess.run(["rocm-smi", "--showclocks", "--showperflevel"], capture_output=True, text=True, timeout=20).stdout
    except (OSError, subprocess.SubprocessError) as e:
        return {"error": str(e)}
    res = {}
    for name in ("sclk", "mclk", "fclk", "socclk"):
        m = re.search(r"GPU\[0\]\s*:\s*%s clock level: \d+: \((\d+)Mhz\)" % name, txt)
        if m:
            res[name + "_mhz"] = int(m.group(1))
    m = re.search(r"GPU\[0\]\s*:\s*Performance Level: (\w+)", txt)
    if m:
        res["performance_level"] = m.group(1)
    return res


def transient(wl, bits, bucket, lr, steps):
    """Per-step launch times of the first `steps` steps: right after the inputs were generated (the
    state the timed region of a short run starts in), after two seconds of idling, and right after
    that series (the settled state); rocm-smi's clock levels after each series."""
    import torch
    series = []
    for name, idle_s in (("right after input generation", 0.0), ("after 2 s idle", 2.0), ("back to back with the previous series", 0.0)):
        if idle_s:
            time.sleep(idle_s)
        ev = []
        run_steps(wl, bits, bucket, lr, steps, 0, ev)
        torch.cuda.synchronize()
        q = [e[0].elapsed_time(e[1]) / wl.W * 1e3 for e in ev]
        a = [e[1].elapsed_time(e[2]) * 1e3 for e in ev]
        t_ms, acc = [], 0.0
        for e in ev:
            t_ms.append(acc)
            acc += e[0].elapsed_time(e[2])
        series.append({"start": name, "quantize_us": [round(v, 1) for v in q], "aggregate_us": [round(v, 1) for v in a],
                       "step_start_ms": [round(v, 2) for v in t_ms], "clocks_after": smi_clocks()})
        log("transient, %s: quantize first 5 %.1f us, steps 5..24 %.1f us, last 20 %.1f us | aggregate %.1f / %.1f / %.1f us" %
            (name, sum(q[:5]) / 5, sum(q[5:25]) / 20, sum(q[-20:]) / 20, sum(a[:5]) / 5, sum(a[5:25]) / 20, sum(a[-20:]) / 20))
    return series


VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12   # 256 compute units x 64 lanes per clock x 2.4 GHz, one-lane-op units


def alu_row(kernel, ms, ops, extra=None):
    """Roofline entry of a kernel bound by vector-ALU issue: against the nominal peak (2.4 GHz) and against
    the peak at the engine clock that rocm-smi read under sustained load (tracked machine-state summary)."""
    tops = ops / (ms * 1e-3) / 1e12
    row = {"kernel": kernel, "avg_launch_us": ms * 1e3, "bound": "alu", "achieved": tops, "peak": VALU_PEAK_TOPS,
           "unit": "T lane-ops/s", "frac": tops / VALU_PEAK_TOPS, "algorithmic_ops_per_launch": ops}
    mhz = load_clock_mhz()
    if mhz:
        row["load_clock_mhz"] = mhz
        row["peak_at_load_clock"] = 256 * 64 * mhz * 1e6 / 1e12
        row["frac_at_load_clock"] = tops / row["peak_at_load_clock"]
    if extra:
        row.update(extra)
    return row


def time_exchange(wl, bits, bucket, lr, steps, warmup):
    """The second leg of Algorithm 1: mqg_aggregate_requantize (server) + mqg_dequantize_update (worker).

    The re-quantize kernel is bound by vector-ALU issue, not by HBM: per element it executes
    W * 4 (bit-field extract, 2c - L, convert, fma) + about 17 (range, rounding, Philox / 8, packing)
    vector operations while moving only (W + 1) * bits / 8 bytes."""
    import torch
    from paper_1804_08066_amd import mqgrad
    n, W = wl.n, wl.W
    outs = wl.outputs(bits, bucket)
    pk, sc = [o[0] for o in outs], [o[1] for o in outs]
    for w in range(W):
        mqgrad.mqg_quantize(wl.grads[w], bits, bucket, seed=1234, iteration=0, worker=w, packed_out=pk[w], scales_out=sc[w])
    mean_pk, mean_sc = mqgrad.alloc_outputs(n, bits, bucket, wl.device)
    mean_out = torch.empty(n, dtype=torch.float32, device=wl.device)
    ev = []
    for k in range(warmup + steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record()
        mqgrad.mqg_aggregate_requantize(pk, sc, n, bits, bucket, seed=1234, iteration=k, worker=W,
                                        packed_out=mean_pk, scales_out=mean_sc)
        e[1].record()
        mqgrad.mqg_dequantize_update(mean_pk, mean_sc, n, bits, bucket, lr, wl.params)
        e[2].record()
        mqgrad.mqg_aggregate_mean(pk, sc, n, bits, bucket, mean_out)
        e[3].record()
        if k >= warmup:
            ev.append(e)
    torch.cuda.synchronize()
    r_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / len(ev)
    d_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / len(ev)
    m_ms = sum(e[2].elapsed_time(e[3]) for e in ev) / len(ev)
    nb = (n + bucket - 1) // bucket
    m_bytes = W * (n * bits / 8.0 + 4.0 * nb) + 4.0 * n
    r_bytes = (W + 1) * (n * bits / 8.0 + 4.0 * nb)
    d_bytes = n * bits / 8.0 + 4.0 * nb + 8.0 * n
    # vector operations the kernel's algorithm issues per element: per worker's code 1.5 (1 bit: quad table)
    # or 1.75 (2-4 bits: pair table) for table offsets + the chain's fma, 3 at 8 bits, 3.5 at 5-7 bits
    # (arithmetic decode); about 14 to encode (range, Philox / 8, fixed-point rounding, packing)
    per_code = 1.5 if bits == 1 else (1.75 if bits <= 4 else (3.0 if bits == 8 else 3.5))
    r_ops = n * (per_code * W + 14.0)
    log("exchange: requantize %.1f us (%.1f T lane-ops/s, %.0f GB/s), dequantize_update %.1f us (%.0f GB/s), "
        "aggregate_mean %.1f us (%.0f GB/s)" %
        (r_ms * 1e3, r_ops / (r_ms * 1e-3) / 1e12, r_bytes / (r_ms * 1e-3) / 1e9, d_ms * 1e3, d_bytes / (d_ms * 1e-3) / 1e9,
         m_ms * 1e3, m_bytes / (m_ms * 1e-3) / 1e9))
    return {
        "requantize": alu_row("requantize_wave_kernel", r_ms, r_ops,
                              {"algorithmic_bytes_per_launch": r_bytes, "hbm_gbs": r_bytes / (r_ms * 1e-3) / 1e9}),
        "dequantize_update": {"kernel": "aggregate_update_rows_kernel (W=1)", "avg_launch_us": d_ms * 1e3, "bound": "hbm",
                              "achieved": d_bytes / (d_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": d_bytes / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "algorithmic_bytes_per_launch": d_bytes},
        "aggregate_mean": {"kernel": "aggregate_mean_kernel", "avg_launch_us": m_ms * 1e3, "bound": "hbm",
                           "achieved": m_bytes / (m_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": m_bytes / (m_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": m_bytes},
        "grad_gbs_server_leg": 4.0 * n * W / (r_ms * 1e-3) / 1e9,
    }


def time_tensors(W, bits, bucket, lr, steps, warmup, device):
    """Configuration 2 (the small CNN's ten layer tensors, about 1.07 M values per worker): one iteration
    with one launch per layer and worker versus the multi-tensor entry points (one quantize launch per
    worker, one update launch). The large layers are quantized, the small ones travel uncompressed."""
    import torch
    from paper_1804_08066_amd import mqgrad, workloads
    shapes = workloads.SMALL_CNN_SHAPES
    q_idx = [i for i, (_, n) in enumerate(shapes) if n >= 4096]
    bases = workloads.config2_elem_bases(bucket)
    grads = [workloads.config2_grads(0, w, 0, device) for w in range(W)]
    params = workloads.config2_params(0, device)
    outs = [[mqgrad.alloc_outputs(shapes[i][1], bits, bucket, device) for i in q_idx] for _ in range(W)]
    layers = []
    for i in range(len(shapes)):
        if i in q_idx:
            k = q_idx.index(i)
            layers.append({"params": params[i], "packed": [outs[w][k][0] for w in range(W)],
                           "scales": [outs[w][k][1] for w in range(W)]})
        else:
            layers.append({"params": params[i], "raw": [grads[w][i] for w in range(W)]})

    def per_layer(it):
        for w in range(W):
            for k, i in enumerate(q_idx):
                mqgrad.mqg_quantize(grads[w][i], bits, bucket, seed=w, iteration=it, worker=w, elem_base=bases[i],
                                    packed_out=outs[w][k][0], scales_out=outs[w][k][1])
        for k, i in enumerate(q_idx):
            mqgrad.mqg_aggregate_update([outs[w][k][0] for w in range(W)], [outs[w][k][1] for w in range(W)],
                                        shapes[i][1], bits, bucket, lr, params[i])

    def batched(it):
        for w in range(W):
            mqgrad.mqg_quantize_tensors([grads[w][i] for i in q_idx], bits, bucket, seed=w, iteration=it, worker=w,
                                        elem_bases=[bases[i] for i in q_idx], outputs=outs[w])
        mqgrad.mqg_aggregate_update_tensors(layers, W, bits, bucket, lr)

    res = {}
    for name, fn in (("per_layer", per_layer), ("batched", batched)):
        for it in range(warmup):
            fn(it)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for it in range(steps):
            fn(it)
        torch.cuda.synchronize()
        res[name + "_us_per_iteration"] = (time.perf_counter() - t0) / steps * 1e6
    # the same batched iteration captured once into a HIP graph and replayed (the entry points allocate
    # nothing and clear memory with kernels only, so they can be captured; the iteration counter of the
    # random stream is frozen at capture, which does not matter for timing)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        batched(0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        batched(0)
    for it in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    res["graph_replay_us_per_iteration"] = (time.perf_counter() - t0) / steps * 1e6
    n_total = sum(n for _, n in shapes)
    res["launches_per_iteration"] = {"per_layer": (W + 1) * len(q_idx), "batched": W + 1}
    res["grad_gbs_batched"] = 4.0 * n_total * W / (res["batched_us_per_iteration"] * 1e-6) / 1e9
    res["note"] = "host-inclusive wall clock; the per-layer variant skips the uncompressed layers' update"
    log("tensors: per-layer %.1f us/iteration, batched %.1f us/iteration, batched in a replayed graph %.1f us/iteration" %
        (res["per_layer_us_per_iteration"], res["batched_us_per_iteration"], res["graph_replay_us_per_iteration"]))
    return res


def time_minmax(wl, bits, bucket, lr, steps, warmup):
    """The footnote's deterministic [min, max] encoding and the sum of squares of the Adaptive rule."""
    import torch
    from paper_1804_08066_amd import mqgrad
    n, W = wl.n, wl.W
    pk = [torch.empty(mqgrad.mqg_packed_words(n, bits), dtype=torch.int32, device=wl.device) for _ in range(W)]
    rg = [torch.empty(2 * mqgrad.mqg_num_buckets(n, bucket), dtype=torch.float32, device=wl.device) for _ in range(W)]
    ss = torch.empty(1, dtype=torch.float64, device=wl.device)
    mpk = torch.empty_like(pk[0])
    mrg = torch.empty_like(rg[0])
    trg = torch.zeros(2, dtype=torch.float32, device=wl.device)
    trs = [torch.tensor([-0.06, 0.06], dtype=torch.float32, device=wl.device) for _ in range(W)]   # one range per worker
    ev = []
    for k in range(warmup + steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(7)]
        e[0].record()
        for w in range(W):
            mqgrad.mqg_quantize_minmax(wl.grads[w], bits, bucket, pk[w], rg[w])
        e[1].record()
        mqgrad.mqg_aggregate_update_minmax(pk, rg, n, bits, bucket, lr, wl.params)
        e[2].record()
        for w in range(W):
            mqgrad.mqg_sum_squares(wl.grads[w], ss)
        e[3].record()
        mqgrad.mqg_aggregate_requantize_minmax(pk, rg, n, bits, bucket, mpk, mrg)
        e[4].record()
        mqgrad.mqg_quantize_minmax_tensor(wl.grads[k % W], bits, mpk, trg)
        e[5].record()
        mqgrad.mqg_aggregate_requantize_minmax_tensor(pk, trs, n, bits, mpk, trg)
        e[6].record()
        if k >= warmup:
            ev.append(e)
    torch.cuda.synchronize()
    q_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / len(ev) / W
    a_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / len(ev)
    s_ms = sum(e[2].elapsed_time(e[3]) for e in ev) / len(ev) / W
    r_ms = sum(e[3].elapsed_time(e[4]) for e in ev) / len(ev)
    t_ms = sum(e[4].elapsed_time(e[5]) for e in ev) / len(ev)
    rt_ms = sum(e[5].elapsed_time(e[6]) for e in ev) / len(ev)
    rt_bytes = (2 * W + 1) * n * bits / 8.0   # the W streams are read twice (range of the sum, then the encode)
    nb = (n + bucket - 1) // bucket
    q_bytes = n * (4.0 + bits / 8.0) + 8.0 * nb
    a_bytes = W * (n * bits / 8.0 + 8.0 * nb) + 8.0 * n
    s_bytes = 4.0 * n
    t_bytes = n * (8.0 + bits / 8.0)   # two passes over the gradient (range, then encode)
    frac = lambda by, ms: by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    r_ops = n * (4.0 * W + 12.0)   # decode: extract, convert, fma, add per worker; encode about 12
    log("minmax b=%d B=%d: quantize %.1f us (%.1f%%), aggregate %.1f us (%.1f%%), sum_squares %.1f us (%.1f%%), "
        "requantize %.1f us (%.1f T lane-ops/s), whole-tensor range + encode %.1f us (%.1f%%)" %
        (bits, bucket, q_ms * 1e3, 100 * frac(q_bytes, q_ms), a_ms * 1e3, 100 * frac(a_bytes, a_ms), s_ms * 1e3,
         100 * frac(s_bytes, s_ms), r_ms * 1e3, r_ops / (r_ms * 1e-3) / 1e12, t_ms * 1e3, 100 * frac(t_bytes, t_ms)))
    row = lambda name, by, ms: {"kernel": name, "avg_launch_us": ms * 1e3, "bound": "hbm", "unit": "GB/s",
                                "achieved": by / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "frac": frac(by, ms),
                                "algorithmic_bytes_per_launch": by}
    return {"bits": bits, "bucket": bucket,
            "quantize_minmax": row("quantize_minmax_wave_kernel", q_bytes, q_ms),
            "aggregate_update_minmax": row("aggregate_update_minmax_kernel", a_bytes, a_ms),
            "sum_squares": row("sum_squares_kernel", s_bytes, s_ms),
            "quantize_minmax_tensor": row("tensor_range_kernel + quantize_minmax_wave_kernel", t_bytes, t_ms),
            "requantize_minmax": alu_row("requantize_minmax_kernel", r_ms, r_ops),
            "requantize_minmax_tensor": alu_row("range_init + sum_range_minmax_tensor + range_finish + "
                                                "requantize_minmax_tensor + range_divide kernels", rt_ms,
                                                n * (8.0 * W + 14.0),   # two decodes of W workers, min/max, encode
                                                {"algorithmic_bytes_per_launch": rt_bytes, "hbm_gbs": rt_bytes / (rt_ms * 1e-3) / 1e9})}


def cpu_baseline(bits, bucket, W, lr, sample_n, steps):
    """The oracle as it stands, single thread, on a slice of the same workload (host tensors)."""
    import numpy as np
    from oracle import ref
    from paper_1804_08066_amd import workloads
    log("cpu baseline: oracle on a %d-element slice, W=%d, %d step(s)" % (sample_n, W, steps))
    grads = [workloads.config4_grad(w, sample_n, "cpu").numpy() for w in range(W)]
    params = workloads.uniform(sample_n, -0.05, 0.05, 1, "cpu").numpy()
    t0 = time.perf_counter()
    for k in range(steps):
        outs = [ref.quantize(grads[w], bits, bucket, 1234, k, w) for w in range(W)]
        params = ref.aggregate_update([o[0] for o in outs], [o[1] for o in outs], sample_n, bits, bucket, lr, params)
    dt = time.perf_counter() - t0
    gbs = 4.0 * sample_n * W * steps / dt / 1e9
    res = {"value": gbs, "unit": "GB/s fp32 gradient", "cores": 1, "kind": "oracle",
           "sample": "%d-element slice of the same workload, W=%d, b=%d, bucket=%d, %d step(s), %.1f s"
                     % (sample_n, W, bits, bucket, steps, dt)}

    # the same single-threaded functions called over disjoint bucket ranges from one thread per core
    # (the random stream is counter based: a range is evaluated in isolation with elem_base = its start)
    from concurrent.futures import ThreadPoolExecutor
    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    span = ((sample_n + cores - 1) // cores + bucket * 32 - 1) // (bucket * 32) * (bucket * 32)
    ranges = [(lo, min(sample_n, lo + span)) for lo in range(0, sample_n, span)]
    params = workloads.uniform(sample_n, -0.05, 0.05, 1, "cpu").numpy()

    def one_range(args):
        k, lo, hi = args
        outs = [ref.quantize(grads[w][lo:hi], bits, bucket, 1234, k, w, lo) for w in range(W)]
        params[lo:hi] = ref.aggregate_update([o[0] for o in outs], [o[1] for o in outs], hi - lo, bits, bucket, lr,
                                             params[lo:hi])

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        for k in range(steps):
            list(pool.map(one_range, [(k, lo, hi) for lo, hi in ranges]))
    dt = time.perf_counter() - t0
    res["all_cores"] = {"value": 4.0 * sample_n * W * steps / dt / 1e9, "unit": "GB/s fp32 gradient",
                        "cores": min(cores, len(ranges)), "kind": "oracle over disjoint bucket ranges, one thread per range",
                        "sample": "same slice, %d step(s), %.1f s" % (steps, dt)}
    log("cpu baseline: 1 core %.3f GB/s, %d cores %.3f GB/s" % (gbs, res["all_cores"]["cores"], res["all_cores"]["value"]))
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100, help="untimed steps right before the timed region")
    ap.add_argument("--condition-ms", type=float, default=100.0,
                    help="milliseconds of untimed steps of the same loop before the counted warm-up (0: none); the "
                         "same --steps / --warmup are also timed BEFORE them and reported as `cold`")
    ap.add_argument("--n", type=int, default=100_000_000)
    ap.add_argument("--workers", type=int, default=8)
    ap.add_argument("--grad-buffers", type=int, default=0,
                    help="distinct gradient buffers shared by the workers (0 = one per worker); for sizes like "
                         "--n 1000000000 --workers 16, where 16 full gradients do not need to be resident")
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--bucket", type=int, default=1024)
    ap.add_argument("--lr", type=float, default=0.1)
    ap.add_argument("--code-stores", choices=("auto", "cached", "stream"), default="auto",
                    help="cache policy of the quantizer's code words: kept for the update that follows, streamed to "
                         "memory, or whichever a short untimed probe finds faster (the cold region always runs 'cached')")
    ap.add_argument("--sweep", action="store_true", help="also time every (b, bucket) of the sweep")
    ap.add_argument("--exchange", action="store_true",
                    help="also time the paper's full exchange: server re-quantizes the mean, worker de-quantizes and updates")
    ap.add_argument("--tensors", action="store_true",
                    help="also time the small CNN's layer list: one launch per layer versus the multi-tensor calls")
    ap.add_argument("--minmax", action="store_true",
                    help="also time the deterministic [min, max] encoding, its server step and the sum of squares")
    ap.add_argument("--machine-state", action="store_true",
                    help="also record rocm-smi's clock and performance levels, idle and while the quantize kernel runs")
    ap.add_argument("--transient", type=int, default=0, metavar="STEPS",
                    help="before anything else, record the per-step launch times of the first STEPS steps "
                         "(cold, after idling, settled) into the JSON line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 3 plain device copies of one gradient buffer (4n bytes read, 4n written): "
                         "the known-size kernel that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--cpu-sample", type=int, default=16_000_000)
    ap.add_argument("--cpu-steps", type=int, default=6)
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; W workers are W gradient buffers on it. "
              "--gpus %d is not supported (no inter-GPU path exists)." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1804_08066_amd import mqgrad
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    mqgrad.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    n, W, bits, bucket = args.n, args.workers, args.bits, args.bucket
    wl = Workload(n, W, dev, args.grad_buffers)

    transient_series = transient(wl, bits, bucket, args.lr, args.transient) if args.transient > 0 else None
    qb, ab = quantize_bytes(n, bits, bucket), aggregate_bytes(n, bits, bucket, W)

    # Cold region: what the same flags measure with no conditioning, i.e. right after the inputs were
    # generated; then untimed conditioning steps; then the counted warm-up and the timed region.
    cold = None
    conditioning = {"ms": 0.0, "steps": 0}
    if args.condition_ms > 0:
        c_ms, c_q, c_a = time_config(wl, bits, bucket, args.lr, args.steps, args.warmup)
        c_spread = dict(time_config.last)
        cold = {"what": "the same --steps / --warmup timed right after input generation, before the conditioning steps",
                "ms_per_step": c_ms, "value": 4.0 * n * W / (c_ms * 1e-3) / 1e9,
                "quantize_us": c_q * 1e3, "quantize_hbm_frac": qb / (c_q * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "aggregate_us": c_a * 1e3, "aggregate_hbm_frac": ab / (c_a * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "quantize_us_first5": c_spread["quantize_us_first5"], "quantize_us_median": c_spread["quantize_us_median"],
                "quantize_us_min": c_spread["quantize_us_min"]}
        log("cold (no conditioning): step %.3f ms | quantize %.1f us (%.1f%%) | aggregate %.1f us (%.1f%%)" %
            (c_ms, c_q * 1e3, 100 * cold["quantize_hbm_frac"], c_a * 1e3, 100 * cold["aggregate_hbm_frac"]))
        done, took = condition(wl, bits, bucket, args.lr, args.condition_ms)
        conditioning = {"ms": took, "steps": done,
                        "what": "untimed steps of the same loop between the cold region and the counted warm-up: after an "
                                "idle gap the chip passes through a throttled state for about 20 ms (profiles/transient_*.md)"}
    stores = choose_code_stores(wl, bits, bucket, args.lr, args.code_stores)
    log("code stores: %s" % json.dumps(stores))
    ms_step, q_ms, a_ms = time_config(wl, bits, bucket, args.lr, args.steps, args.warmup)
    value = 4.0 * n * W / (ms_step * 1e-3) / 1e9
    q_gbs, a_gbs = qb / (q_ms * 1e-3) / 1e9, ab / (a_ms * 1e-3) / 1e9
    log("step %.3f ms | quantize %.1f us/launch %.0f GB/s (%.1f%%) | aggregate %.1f us %.0f GB/s (%.1f%%)" %
        (ms_step, q_ms * 1e3, q_gbs, 100 * q_gbs / HBM_PEAK_GBS, a_ms * 1e3, a_gbs, 100 * a_gbs / HBM_PEAK_GBS))

    spread = dict(time_config.last)
    ceil = stream_ceilings(wl, bits, bucket)
    log("streaming ceilings: quantize mix %.1f us = %.0f GB/s (%.1f%% of peak), update mix %.1f us = %.0f GB/s (%.1f%%), "
        "torch copy_ %.0f GB/s (%.1f%%); pure read %.0f GB/s, pure write %.0f GB/s -> additive bounds %.1f us / %.1f us" %
        (ceil["quantize_mix"]["us"], ceil["quantize_mix"]["gbs"], 100 * ceil["quantize_mix"]["frac_of_peak"],
         ceil["update_mix"]["us"], ceil["update_mix"]["gbs"], 100 * ceil["update_mix"]["frac_of_peak"],
         ceil["torch_copy"]["gbs"], 100 * ceil["torch_copy"]["frac_of_peak"], ceil["pure_read"]["gbs"], ceil["pure_write"]["gbs"],
         ceil["additive_bound"]["quantize_us"], ceil["additive_bound"]["update_us"]))

    a_cold_ms = time_cold_codes(wl, bits, bucket, args.lr)
    a_cold_hint_ms = time_cold_codes(wl, bits, bucket, args.lr, origin=mqgrad.MQG_CODES_FROM_MEMORY)
    log("aggregate_update with the code words out of cache (two 400 MB copies in between): %.1f us (%.1f%%); called with "
        "MQG_CODES_FROM_MEMORY: %.1f us" %
        (a_cold_ms * 1e3, 100 * ab / (a_cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, a_cold_hint_ms * 1e3))
    traffic = measured_traffic(n, W, bits, bucket)
    q_traffic = traffic["quantize_wave_kernel"] if traffic else None
    a_traffic = traffic["aggregate_update_rows_kernel"] if traffic else None
    out = {
        "metric": "GB/s fp32 gradient quantize+pack and unpack+aggregate+update; % HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "bandwidth sweep point: flat fp32 gradient of %d elements ~ N(0, 0.01^2), "
                               "W=%d worker buffers, b=%d, bucket=%d; one step = %d x quantize + 1 x aggregate_update"
                               % (n, W, bits, bucket, W),
                   "n": n, "workers": W, "bits": bits, "bucket": bucket, "code_stores": stores},
        # the quantize kernel runs W times per step and is the dominant kernel by time
        "roofline": {"bound": "hbm", "kernel": "quantize_wave_kernel", "achieved": q_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": q_gbs / HBM_PEAK_GBS, "traffic": q_traffic,
                     "traffic_source": ("profiles/%s at commit %s" % (os.path.basename(TRAFFIC_PROFILE), traffic.get("commit"))) if traffic else None,
                     "algorithmic_bytes_per_launch": qb, "avg_launch_us": q_ms * 1e3,
                     "median_launch_us": spread["quantize_us_median"], "min_launch_us": spread["quantize_us_min"],
                     "first5_launch_us": spread["quantize_us_first5"],
                     "frac_of_stream_ceiling": q_gbs / ceil["quantize_mix"]["gbs"]},
        "roofline_aggregate": {"bound": "hbm", "kernel": "aggregate_update_rows_kernel", "achieved": a_gbs,
                               "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a_gbs / HBM_PEAK_GBS, "traffic": a_traffic,
                               "algorithmic_bytes_per_launch": ab, "avg_launch_us": a_ms * 1e3,
                               "median_launch_us": spread["aggregate_us_median"], "min_launch_us": spread["aggregate_us_min"],
                               "first5_launch_us": spread["aggregate_us_first5"],
                               "frac_of_stream_ceiling": a_gbs / ceil["update_mix"]["gbs"],
                               "codes_out_of_cache": {"what": "the same launch after two 400 MB device copies, so that no "
                                                              "code word is left in this GPU's caches (the state on a parameter "
                                                              "server whose streams arrive over the network)",
                                                      "avg_launch_us": a_cold_ms * 1e3,
                                                      "frac": ab / (a_cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                                      "avg_launch_us_told_so": a_cold_hint_ms * 1e3,
                                                      "frac_told_so": ab / (a_cold_hint_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                                      "told_so": "mqg_aggregate_update_from(..., MQG_CODES_FROM_MEMORY): "
                                                                 "streaming loads of the code words at every width"}},
        "hbm_frac_end_to_end": (W * qb + ab) / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "conditioning": conditioning,
        "cold": cold,
        "stream_ceiling": ceil,
    }

    if transient_series is not None:
        out["transient"] = transient_series

    if args.sweep:
        rows = []
        for bk in (128, 1024, 8192):
            for b in (1, 2, 4, 8):
                point_stores = choose_code_stores(wl, b, bk, args.lr, args.code_stores)
                ms, q, a = time_config(wl, b, bk, args.lr, max(5, args.steps // 4), max(2, args.warmup // 4))
                rows.append({"bits": b, "bucket": bk, "ms_per_step": ms, "code_stores": point_stores["chosen"],
                             "grad_gbs": 4.0 * n * W / (ms * 1e-3) / 1e9,
                             "quantize_us": q * 1e3, "quantize_hbm_frac": quantize_bytes(n, b, bk) / (q * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "aggregate_us": a * 1e3, "aggregate_hbm_frac": aggregate_bytes(n, b, bk, W) / (a * 1e-3) / 1e9 / HBM_PEAK_GBS})
                log("sweep b=%d B=%d: quantize %.1f us (%.1f%%), aggregate %.1f us (%.1f%%)" %
                    (b, bk, q * 1e3, 100 * rows[-1]["quantize_hbm_frac"], a * 1e3, 100 * rows[-1]["aggregate_hbm_frac"]))
        out["sweep"] = rows
        choose_code_stores(wl, bits, bucket, args.lr, stores["chosen"])   # back to the headline's policy

    if args.exchange:
        out["exchange"] = time_exchange(wl, bits, bucket, args.lr, max(10, args.steps // 4), max(5, args.warmup // 4))

    if args.minmax:
        out["minmax"] = [time_minmax(wl, b, bucket, args.lr, max(10, args.steps // 4), max(5, args.warmup // 4))
                         for b in ((1, 2, 4, 8) if args.sweep else (bits,))]

    if args.tensors:
        out["tensors"] = time_tensors(W, bits, 512, args.lr, 200, 20, wl.device)

    if args.machine_state:
        out["machine_state"] = machine_state(wl, bits, bucket)
        log("machine state: %s" % json.dumps(out["machine_state"]))

    if args.calibrate_copy:
        dst = torch.empty_like(wl.grads[0])
        for w in range(3):
            dst.copy_(wl.grads[w % W])
        torch.cuda.synchronize()
        del dst

    del wl
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(bits, bucket, W, args.lr, min(args.cpu_sample, n), args.cpu_steps)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
