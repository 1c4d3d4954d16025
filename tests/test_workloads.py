"""The seeded input generator: reproducible, index-addressable, N(0,1), bf16 round-to-nearest-even."""
import math
import struct

import numpy as np

import workloads as wl


def test_subrange_equals_full_stream():
    full = wl.normal_bf16(7, 3, 10_000)
    for off, n in ((0, 1), (1, 1), (4097, 333), (9_999, 1)):
        np.testing.assert_array_equal(wl.normal_bf16(7, 3, n, offset=off), full[off:off + n])


def test_streams_and_seeds_differ():
    a, b, c = wl.normal_bf16(0, 1, 4096), wl.normal_bf16(0, 2, 4096), wl.normal_bf16(1, 1, 4096)
    assert np.mean(a == b) < 0.05 and np.mean(a == c) < 0.05


def test_moments_and_tails():
    x = wl.bf16_to_f32(wl.normal_bf16(123, 0, 2_000_000)).astype(np.float64)
    assert abs(x.mean()) < 4e-3 and abs(x.std() - 1.0) < 4e-3
    assert abs(np.mean(x ** 3)) < 2e-2 and abs(np.mean(x ** 4) - 3.0) < 5e-2
    assert abs(np.mean(np.abs(x) < 1.0) - math.erf(1 / math.sqrt(2))) < 3e-3
    # neighbouring elements (the cos / sin pair of one counter) are uncorrelated
    assert abs(np.mean(x[0::2] * x[1::2])) < 4e-3


def test_bf16_round_to_nearest_even():
    def bits(f):
        return struct.unpack("<I", struct.pack("<f", f))[0]
    cases = {1.0: 0x3F80, 1.00390625: 0x3F80,            # exactly halfway between 0x3F80 and 0x3F81: to even
             1.01171875: 0x3F82,                          # halfway between 0x3F81 and 0x3F82: to even (up)
             struct.unpack('<f', struct.pack('<I', 0x3F808001))[0]: 0x3F81,     # one fp32 ulp above halfway: up
              -2.5: 0xC020, 0.0: 0x0000, 3.3895314e38: 0x7F7F, 3.4e38: 0x7F80}
    for f, want in cases.items():
        got = int(wl.f32_to_bf16(np.array([f], dtype=np.float32))[0])
        assert got == want, (f, hex(got), hex(want), hex(bits(np.float32(f))))
    x = wl.normal_bf16(5, 0, 1000)
    np.testing.assert_array_equal(wl.f32_to_bf16(wl.bf16_to_f32(x)), x)     # round trip is the identity


def test_generator_value_is_rne_of_its_fp64_draw():
    for i in (0, 1, 2, 77, 1234567):
        z = wl.normal_f64(9, 4, i)
        assert wl.normal_bf16(9, 4, 1, offset=i)[0] == wl.f32_to_bf16(np.array([z], dtype=np.float32))[0]


def test_config_lengths_follow_their_recipes():
    c = wl.CONFIGS
    assert list(c["tiny"].kv_lens()) == [17, 64, 100, 256]
    L = c["qwen3_8b_decode"].kv_lens()
    assert L.shape == (64,) and L.min() >= 512 and L.max() <= 4096
    L = c["long_context"].kv_lens()
    assert L.shape == (16,) and L.min() >= 16384 and L.max() <= 32768
    L = c["spec_verify"].kv_lens()                      # cached prefix in [1024, 8192] plus the 4 new tokens
    assert L.shape == (128,) and L.min() >= 1024 + 4 and L.max() <= 8192 + 4
    L = c["skewed_xtensor"].kv_lens().astype(np.float64)
    assert L.shape == (256,) and L.min() >= 16 and L.max() <= 65536
    assert 700 < np.median(L) < 1500 and 0.9 < np.std(np.log(L)) < 1.5       # log-normal(ln 1024, 1.2)
    for w in c.values():
        np.testing.assert_array_equal(w.kv_lens(), w.kv_lens())
        assert w.n_q_heads % w.n_kv_heads == 0 and w.head_dim == 128
    assert c["tiny"].kv_bytes() == 437 * 2 * 128 * 2 * 2


def test_make_kv_matches_streams():
    w = wl.CONFIGS["tiny"]
    ks, vs = w.make_kv()
    assert [k.shape for k in ks] == [(17, 2, 128), (64, 2, 128), (100, 2, 128), (256, 2, 128)]
    np.testing.assert_array_equal(ks[2].ravel(), wl.normal_bf16(0, 5, 100 * 256))
    np.testing.assert_array_equal(vs[2].ravel(), wl.normal_bf16(0, 6, 100 * 256))
    assert w.make_q().shape == (4, 1, 8, 128)
