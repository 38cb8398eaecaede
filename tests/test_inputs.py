"""The seeded generator: determinism, order independence, distributions, bf16 rounding."""
import numpy as np

from paper_2512_23424_amd import inputs as I


def test_mix_is_splitmix64_finaliser():
    # splitmix64 seeded with 0: first output is mix(0 + golden gamma); published test vector
    assert I._mix_int(0x9E3779B97F4A7C15) == 0xE220A8397B1DCDAF
    v = I._mix_vec(np.array([0x9E3779B97F4A7C15], dtype=np.uint64))
    assert int(v[0]) == 0xE220A8397B1DCDAF


def test_counter_based_and_stream_separated():
    k = I.stream_key(0, 0)
    a = I.unit_uniform(k, 0, 1000)
    b = I.unit_uniform(k, 500, 100)
    assert np.array_equal(a[500:600], b)
    assert (a >= 0).all() and (a < 1).all()
    assert I.stream_key(0, 0) != I.stream_key(0, 1) != I.stream_key(1, 0)
    x1 = I.draw(0, "X", (64, 32), ("normal", 0.0, 1.0))
    x2 = I.draw(0, "X", (64, 32), ("normal", 0.0, 1.0))
    assert np.array_equal(x1, x2)
    # the draw does not depend on the chunking or on the trailing shape
    assert np.array_equal(I.draw(0, "X", (2048,), ("normal", 0.0, 1.0)), x1.reshape(-1))
    assert not np.array_equal(x1, I.draw(1, "X", (64, 32), ("normal", 0.0, 1.0)))
    assert not np.array_equal(x1, I.draw(0, "W", (64, 32), ("normal", 0.0, 1.0)))


def test_distributions():
    n = I.draw(0, "X", (1 << 18,), ("normal", 1.0, 0.1)).astype(np.float64)
    assert abs(n.mean() - 1.0) < 1e-3 and abs(n.std() - 0.1) < 1e-3
    u = I.draw(0, "b", (1 << 18,), ("uniform", -0.1, 0.1)).astype(np.float64)
    assert u.min() >= -0.1 and u.max() <= 0.1 and abs(u.mean()) < 1e-3
    assert abs(u.std() - 0.2 / np.sqrt(12)) < 1e-3
    z = I.draw(0, "X", (4096,), ("int", -2, 2))
    assert set(np.unique(z)) == {-2.0, -1.0, 0.0, 1.0, 2.0}


def test_bf16_round_to_nearest_even_patterns():
    def f32(bits):
        return np.array([bits], dtype=np.uint32).view(np.float32)
    # exact ties go to the even mantissa
    assert I.f32_to_bf16_bits(f32(0x3F808000))[0] == 0x3F80
    assert I.f32_to_bf16_bits(f32(0x3F818000))[0] == 0x3F82
    assert I.f32_to_bf16_bits(f32(0x3F808001))[0] == 0x3F81
    assert I.f32_to_bf16_bits(f32(0x3F807FFF))[0] == 0x3F80
    assert I.f32_to_bf16_bits(f32(0xBF818000))[0] == 0xBF82
    for bits in (0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0xBF818000, 0x00000000, 0x40490FDB):
        assert I.f64_to_bf16_bits(f32(bits).astype(np.float64))[0] == I.f32_to_bf16_bits(f32(bits))[0]
    # a float64 just above a tie must round up even though fp32 rounding would land on the tie
    x = np.array([1.00390625 + 2.0 ** -40])                   # 1 + 2^-8 (tie) + tiny
    assert I.f64_to_bf16_bits(x)[0] == 0x3F81
    assert I.f32_to_bf16_bits(x.astype(np.float32))[0] == 0x3F80   # the double-rounding trap
    # idempotent
    v = np.random.default_rng(0).standard_normal(10000)
    b = I.f64_to_bf16_bits(v)
    assert np.array_equal(I.f64_to_bf16_bits(I.bf16_bits_to_f32(b).astype(np.float64)), b)
    err = np.abs(I.bf16_bits_to_f32(b).astype(np.float64) - v) / np.abs(v)
    assert err.max() <= 2.0 ** -8


def test_workloads_match_their_description():
    w = I.WORKLOADS
    assert (w["cfg2"].M, w["cfg2"].K, w["cfg2"].N) == (4096, 1024, 1024)
    assert w["cfg4"].rows == 32768 and w["cfg3"].in_dtype == I.BF16
    assert w["cfg3"].dist.get("b") is None
    assert abs(w["cfg5"].algorithmic_bytes / 1e6 - 605.2) < 0.1
    assert abs(w["cfg3"].algorithmic_bytes / 1e6 - 167.8) < 0.1
    assert abs(w["cfg3"].flops / 1e9 - 274.9) < 0.1
    g = I.generate(I.scaled(w["cfg3"], M=16, K=64, N=32))
    assert g["X"].dtype == np.uint16 and g["gamma"].dtype == np.float32 and g["b"] is None
    g2 = I.generate(I.scaled(w["cfg3"], M=16, K=64, N=32), rows=np.array([3, 7]))
    assert np.array_equal(g2["X"], g["X"][[3, 7]])


def test_fp16_storage_rounds_once_to_nearest_even():
    """fp16 tensors: one rounding from float64, ties to even (hand-built cases), and the drawn
    values are exactly what the float16 array holds."""
    v = np.array([1.0 + 2.0 ** -11, 1.0 + 3.0 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -40, -(1.0 + 2.0 ** -11),
                  65504.0, 2.0 ** -24, 2.0 ** -25], dtype=np.float64)
    got = I._store(v, I.F16)
    assert got.dtype == np.float16
    want = np.array([1.0, 1.0 + 2.0 ** -9, 1.0 + 2.0 ** -10, -1.0, 65504.0, 2.0 ** -24, 0.0])
    assert np.array_equal(got.astype(np.float64), want)
    w = I.Workload(name="h", M=5, K=8, N=8, in_dtype=I.F16, out_dtype=I.F16,
                   dist={"X": ("normal", 0.0, 1.0), "W": ("uniform", -1.0, 1.0)})
    t = I.generate(w)
    assert t["X"].dtype == np.float16 and t["W"].dtype == np.float16
    assert np.array_equal(I.as_f64(t["X"]), t["X"].astype(np.float64))


def test_e4m3_storage_patterns_and_rounding():
    """8-bit E4M3 (bias 7, 3 mantissa bits, no infinities): hand-made patterns, ties to even,
    subnormals, saturation at 448, and the whole code table against torch's CPU conversion of
    the same format (float8_e4m3fn), a routine independent of this module."""
    import torch
    enc, dec = I.f64_to_e4m3_bits, I.e4m3_bits_to_f64
    val = dec(np.arange(256, dtype=np.uint8))
    assert val[0x38] == 1.0 and val[0x7E] == 448.0 and val[0x01] == 2.0 ** -9 and val[0x08] == 2.0 ** -6
    assert val[0xB8] == -1.0 and np.isnan(val[0x7F]) and np.isnan(val[0xFF]) and val[0x80] == 0.0
    tb = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.nan_to_num(val, nan=7e9), np.nan_to_num(tb, nan=7e9))
    # grid spacing is 1/8 in [1, 2): 1.0625 is a tie between 1.0 (even) and 1.125; 1.1875 between 1.125 and 1.25 (even)
    assert list(enc(np.array([1.0625, 1.1875, 1.07, -1.0625]))) == [0x38, 0x3A, 0x39, 0xB8]
    # below the smallest normal the grid is 2^-9; half of it is a tie with zero (even)
    assert list(enc(np.array([2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 0.9 * 2.0 ** -6, 0.0]))) == [0x01, 0x00, 0x02, 0x07, 0x00]
    # rounding up across a binade and saturation
    assert list(enc(np.array([1.97, 15.9, 448.0, 1e6, -1e6]))) == [0x40, 0x58, 0x7E, 0x7E, 0xFE]
    # every finite pattern survives a round trip; random values agree with torch below the saturation range
    finite = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    assert np.array_equal(enc(dec(finite)) & 0x7F, finite & 0x7F)
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.normal(0, 1, 5000), rng.normal(0, 0.01, 5000), rng.uniform(-440, 440, 2000)]).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(enc(v.astype(np.float64)), ref)
    x = I.draw(0, "X", (64, 64), ("normal", 0.0, 1.0), I.F8E4M3)
    assert x.dtype == np.uint8 and np.array_equal(enc(I.as_f64(x)), x)
