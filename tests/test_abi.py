"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol that
include/mqgrad.h declares, does its size arithmetic, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_1804_08066_amd import mqgrad

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mqgrad.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mqg_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = mqgrad.lib()
    names = declared_symbols()
    assert set(names) == set(mqgrad.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None


def test_size_helpers():
    assert mqgrad.mqg_num_buckets(0, 512) == 0
    assert mqgrad.mqg_num_buckets(1, 512) == 1
    assert mqgrad.mqg_num_buckets(512, 512) == 1
    assert mqgrad.mqg_num_buckets(513, 512) == 2
    assert mqgrad.mqg_num_buckets(100_000_000, 1024) == 97657
    for bits in range(1, 9):
        for n in (0, 1, 31, 32, 33, 65536, 100_000_000, 1_000_000_000, (1 << 40) + 5):
            assert mqgrad.mqg_packed_words(n, bits) == (n * bits + 31) // 32


def test_status_strings():
    for st in (0, -1, -2, -3, 5):
        assert mqgrad.status_string(st)
    assert "EINVAL" in mqgrad.status_string(mqgrad.MQG_EINVAL)


def test_invalid_arguments_are_rejected_before_any_launch():
    L = mqgrad.lib()
    fake = C.c_void_p(0x1000)            # never dereferenced: validation fails first
    q = lambda **kw: L.mqg_quantize(kw.get("grad", fake), kw.get("n", 64), kw.get("bits", 4),
                                    kw.get("bucket", 512), 0, 0, 0, kw.get("elem_base", 0),
                                    kw.get("packed", fake), kw.get("scales", fake), None)
    assert q(bits=0) == mqgrad.MQG_EINVAL
    assert q(bits=9) == mqgrad.MQG_EINVAL
    assert q(bucket=0) == mqgrad.MQG_EINVAL
    assert q(bucket=16) == mqgrad.MQG_EINVAL
    assert q(bucket=48) == mqgrad.MQG_EINVAL
    assert q(bucket=16416) == mqgrad.MQG_EINVAL
    assert q(elem_base=4) == mqgrad.MQG_EINVAL
    assert q(grad=None) == mqgrad.MQG_EINVAL
    assert q(packed=None) == mqgrad.MQG_EINVAL
    assert q(scales=None) == mqgrad.MQG_EINVAL
    assert q(grad=C.c_void_p(0x1002)) == mqgrad.MQG_EALIGN
    assert q(packed=C.c_void_p(0x1001)) == mqgrad.MQG_EALIGN
    assert q(n=0, grad=None, packed=None, scales=None) == mqgrad.MQG_OK      # empty input is a no-op
    assert L.mqg_quantize_mode(fake, 64, 4, 512, 7, 0, 0, 0, 0, fake, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_quantize_with_scales(fake, 64, 4, 512, 0, 0, 0, 0, None, fake, fake, None) == mqgrad.MQG_EINVAL

    vp = C.c_void_p
    one = (vp * 1)(0x1000)
    null1 = (vp * 1)(None)
    a = lambda packed=one, scales=one, W=1, n=64, bits=4, bucket=512, params=fake: \
        L.mqg_aggregate_update(packed, scales, W, n, bits, bucket, 0.1, params, None)
    assert a(W=0) == mqgrad.MQG_EINVAL
    assert a(W=65) == mqgrad.MQG_EINVAL
    assert a(bits=0) == mqgrad.MQG_EINVAL
    assert a(bucket=100) == mqgrad.MQG_EINVAL
    assert a(params=None) == mqgrad.MQG_EINVAL
    assert a(packed=None) == mqgrad.MQG_EINVAL
    assert a(packed=null1) == mqgrad.MQG_EINVAL
    assert a(scales=null1) == mqgrad.MQG_EINVAL
    assert a(params=C.c_void_p(0x1003)) == mqgrad.MQG_EALIGN
    assert a(n=0, params=None) == mqgrad.MQG_OK
    m = lambda packed=one, scales=one, W=1, n=64, bits=4, bucket=512, out=fake: \
        L.mqg_aggregate_mean(packed, scales, W, n, bits, bucket, out, None)
    assert m(W=0) == mqgrad.MQG_EINVAL
    assert m(bits=9) == mqgrad.MQG_EINVAL
    assert m(out=None) == mqgrad.MQG_EINVAL
    assert m(scales=null1) == mqgrad.MQG_EINVAL
    assert m(out=C.c_void_p(0x1002)) == mqgrad.MQG_EALIGN
    assert m(n=0, out=None) == mqgrad.MQG_OK


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        mqgrad.mqg_quantize(torch.zeros(64), 4, 32, 0)


def test_multi_tensor_and_minmax_arguments_are_rejected_before_any_launch():
    L = mqgrad.lib()
    vp = C.c_void_p
    fake = vp(0x1000)
    one = (vp * 1)(0x1000)
    # several tensors per launch
    items = (mqgrad.QuantizeItem * 2)()
    items[0] = mqgrad.QuantizeItem(0x1000, 64, 0, 0x2000, 0x3000)
    items[1] = mqgrad.QuantizeItem(0x1000, 64, 4, 0x2000, 0x3000)          # elem_base not a multiple of 8
    assert L.mqg_quantize_tensors(items, 2, 4, 512, 0, 0, 0, None) == mqgrad.MQG_EINVAL
    assert L.mqg_quantize_tensors(items, 1, 0, 512, 0, 0, 0, None) == mqgrad.MQG_EINVAL
    assert L.mqg_quantize_tensors(items, 33, 4, 512, 0, 0, 0, None) == mqgrad.MQG_EINVAL
    assert L.mqg_quantize_tensors(None, 1, 4, 512, 0, 0, 0, None) == mqgrad.MQG_EINVAL
    assert L.mqg_quantize_tensors(items, 0, 4, 512, 0, 0, 0, None) == mqgrad.MQG_OK
    items[0] = mqgrad.QuantizeItem(0x1002, 64, 0, 0x2000, 0x3000)
    assert L.mqg_quantize_tensors(items, 1, 4, 512, 0, 0, 0, None) == mqgrad.MQG_EALIGN
    up = (mqgrad.UpdateItem * 1)()
    up[0] = mqgrad.UpdateItem(64, 0x1000, None, None, None)                 # neither quantized nor raw
    assert L.mqg_aggregate_update_tensors(up, 1, 1, 4, 512, 0.1, None) == mqgrad.MQG_EINVAL
    assert L.mqg_aggregate_update_tensors(up, 1, 0, 4, 512, 0.1, None) == mqgrad.MQG_EINVAL
    assert L.mqg_aggregate_update_tensors(up, 0, 1, 4, 512, 0.1, None) == mqgrad.MQG_OK
    # deterministic [min, max] encoding
    q = lambda grad=fake, n=64, bits=4, bucket=512, packed=fake, ranges=fake: \
        L.mqg_quantize_minmax(grad, n, bits, bucket, packed, ranges, None)
    assert q(bits=9) == mqgrad.MQG_EINVAL
    assert q(bucket=40) == mqgrad.MQG_EINVAL
    assert q(grad=None) == mqgrad.MQG_EINVAL
    assert q(ranges=None) == mqgrad.MQG_EINVAL
    assert q(ranges=vp(0x1004)) == mqgrad.MQG_EALIGN                        # pairs are read 8 bytes at a time
    assert q(n=0, grad=None, packed=None, ranges=None) == mqgrad.MQG_OK
    a = lambda packed=one, ranges=one, W=1, n=64, bits=4, bucket=512, params=fake: \
        L.mqg_aggregate_update_minmax(packed, ranges, W, n, bits, bucket, 0.1, params, None)
    assert a(W=0) == mqgrad.MQG_EINVAL
    assert a(W=65) == mqgrad.MQG_EINVAL
    assert a(params=None) == mqgrad.MQG_EINVAL
    assert a(ranges=(vp * 1)(0x1004)) == mqgrad.MQG_EALIGN
    assert a(ranges=(vp * 1)(None)) == mqgrad.MQG_EINVAL
    assert a(n=0, params=None) == mqgrad.MQG_OK
    r = lambda packed=one, ranges=one, W=1, n=64, bits=4, bucket=512, po=fake, ro=fake: \
        L.mqg_aggregate_requantize_minmax(packed, ranges, W, n, bits, bucket, po, ro, None)
    assert r(W=0) == mqgrad.MQG_EINVAL
    assert r(bits=0) == mqgrad.MQG_EINVAL
    assert r(po=None) == mqgrad.MQG_EINVAL
    assert r(ro=vp(0x1004)) == mqgrad.MQG_EALIGN
    assert r(ranges=(vp * 1)(0x1004)) == mqgrad.MQG_EALIGN
    assert r(n=0, po=None, ro=None) == mqgrad.MQG_OK
    assert L.mqg_tensor_range(fake, 10, None, None) == mqgrad.MQG_EINVAL
    assert L.mqg_tensor_range(fake, 10, vp(0x1004), None) == mqgrad.MQG_EALIGN
    assert L.mqg_tensor_range(None, 0, None, None) == mqgrad.MQG_OK
    assert L.mqg_quantize_minmax_tensor(fake, 10, 9, fake, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_quantize_minmax_tensor(fake, 10, 4, None, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_quantize_minmax_tensor(fake, 10, 4, fake, vp(0x1004), None) == mqgrad.MQG_EALIGN
    assert L.mqg_aggregate_update_minmax_tensor(one, one, 0, 10, 4, 0.1, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_aggregate_update_minmax_tensor(one, (vp * 1)(0x1004), 1, 10, 4, 0.1, fake, None) == mqgrad.MQG_EALIGN
    assert L.mqg_aggregate_update_minmax_tensor(one, one, 1, 0, 4, 0.1, None, None) == mqgrad.MQG_OK
    assert L.mqg_aggregate_requantize_minmax_tensor(one, one, 0, 10, 4, fake, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_aggregate_requantize_minmax_tensor(one, one, 1, 10, 9, fake, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_aggregate_requantize_minmax_tensor(one, one, 1, 10, 4, None, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_aggregate_requantize_minmax_tensor(one, one, 1, 10, 4, fake, vp(0x1004), None) == mqgrad.MQG_EALIGN
    assert L.mqg_aggregate_requantize_minmax_tensor(one, (vp * 1)(0x1004), 1, 10, 4, fake, fake, None) == mqgrad.MQG_EALIGN
    assert L.mqg_aggregate_requantize_minmax_tensor(one, one, 1, 0, 4, None, None, None) == mqgrad.MQG_OK
    assert L.mqg_sum_squares(fake, 10, None, None) == mqgrad.MQG_EINVAL
    assert L.mqg_sum_squares(None, 10, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_sum_squares(fake, 10, vp(0x1004), None) == mqgrad.MQG_EALIGN
    items = (mqgrad.SumsqItem * 65)()
    for it in items:
        it.grad, it.n = 0x1000, 10
    assert L.mqg_sum_squares_workspace_bytes(3) == 3 * 512 * 8
    assert L.mqg_sum_squares_batch(items, 0, None, None, None) == mqgrad.MQG_OK
    assert L.mqg_sum_squares_batch(items, 65, fake, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_sum_squares_batch(None, 2, fake, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_sum_squares_batch(items, 2, None, fake, None) == mqgrad.MQG_EINVAL
    assert L.mqg_sum_squares_batch(items, 2, fake, None, None) == mqgrad.MQG_EINVAL
    assert L.mqg_sum_squares_batch(items, 2, vp(0x1004), fake, None) == mqgrad.MQG_EALIGN
    assert L.mqg_sum_squares_batch(items, 2, fake, vp(0x1004), None) == mqgrad.MQG_EALIGN
    items[1].grad = 0x1002
    assert L.mqg_sum_squares_batch(items, 2, fake, fake, None) == mqgrad.MQG_EALIGN
    items[1].grad = None
    assert L.mqg_sum_squares_batch(items, 2, fake, fake, None) == mqgrad.MQG_EINVAL


def test_adaptive_rule_matches_the_oracle_rule():
    # host-only policy: the library's rule against the oracle's statement of it, over a dense sweep
    from oracle import policy_ref
    import random
    rnd = random.Random(5)
    for i in range(3000):
        W = rnd.randint(1, 12)
        norms = [rnd.random() * 10 ** rnd.uniform(-5, -2) for _ in range(W)]
        assert mqgrad.mqg_adaptive_bits(norms) == policy_ref.adaptive_bits(norms)
    for z in [0.0, 0.0005, 0.001, 0.0015, 0.002, 0.0025, 0.003, 0.0035, 1.0, float("inf")]:
        assert mqgrad.mqg_adaptive_bits([z]) == policy_ref.adaptive_bits([z])
        assert mqgrad.mqg_adaptive_bits([z], bits_min=1, bits_max=6, base_bits=1) == \
            policy_ref.adaptive_bits([z], base_bits=1, bits_min=1, bits_max=6)
    for bad in ([], [-1.0], [float("nan")]):
        with pytest.raises(mqgrad.MqgError):
            mqgrad.mqg_adaptive_bits(bad)
    with pytest.raises(mqgrad.MqgError):
        mqgrad.mqg_adaptive_bits([0.1], norm_per_bit=0.0)
    with pytest.raises(mqgrad.MqgError):
        mqgrad.mqg_adaptive_bits([0.1], bits_min=5, bits_max=4)


def test_header_compiles_as_plain_c(tmp_path):
    # the boundary is a C ABI: the header must stand alone under a C compiler, warnings as errors
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "mqgrad.h"\nint main(void) { return (int)mqg_packed_words(0, 1) + (int)MQG_CODES_FROM_MEMORY * 0; }\n')
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                        "-c", str(src), "-o", str(tmp_path / "use_header.o")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
