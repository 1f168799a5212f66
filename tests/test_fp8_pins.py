"""Pins of oracle/fp8.py (the E4M3 format and attention over an 8-bit suffix cache) against what the format's
definition and the mathematics fix, and against torch's float8_e4m3fn conversions (an independent implementation).
CPU only."""
import numpy as np
import torch

from oracle import fp8
from paper_2402_05099_amd import workloads as wl


def test_decode_values_fixed_by_the_format():
    # (code, value): zero, smallest subnormal, largest subnormal, smallest normal, one, largest finite, negatives
    fixed = [(0x00, 0.0), (0x01, 2.0 ** -9), (0x07, 7 * 2.0 ** -9), (0x08, 2.0 ** -6), (0x38, 1.0), (0x3C, 1.5),
             (0x40, 2.0), (0x7E, 448.0), (0x77, 240.0), (0xB8, -1.0), (0xFE, -448.0), (0x81, -(2.0 ** -9))]
    for code, value in fixed:
        assert fp8.e4m3_decode(np.array([code], dtype=np.uint8))[0] == value, hex(code)
    both = fp8.e4m3_decode(np.array([0x7F, 0xFF, 0x80], dtype=np.uint8))
    assert np.isnan(both[0]) and np.isnan(both[1])
    assert both[2] == 0.0 and np.signbit(both[2])


def test_decode_is_increasing_in_the_code_and_has_254_finite_values():
    v = fp8.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert np.isfinite(v).sum() == 254
    assert (np.diff(v[:127]) > 0).all()
    assert np.array_equal(v[128:255], -v[:127])


def test_decode_agrees_with_torch():
    codes = torch.arange(256, dtype=torch.uint8)
    t = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    v = fp8.e4m3_decode(codes.numpy())
    assert np.array_equal(np.isnan(t), np.isnan(v))
    ok = ~np.isnan(v)
    assert np.array_equal(t[ok], v[ok])
    assert np.array_equal(np.signbit(t[ok]), np.signbit(v[ok]))


def test_encode_round_trip_over_all_codes():
    codes = np.arange(256, dtype=np.uint8)
    back = fp8.e4m3_encode(fp8.e4m3_decode(codes))
    nan = (codes & 0x7F) == 0x7F
    assert np.array_equal(back[~nan], codes[~nan])      # -0 stays -0
    assert ((back[nan] & 0x7F) == 0x7F).all()


def test_encode_is_the_nearest_value_by_brute_force():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 1, 400), rng.normal(0, 100, 400), rng.uniform(-0.03, 0.03, 400)])
    grid = fp8.e4m3_decode(np.arange(256, dtype=np.uint8))
    finite = np.where(np.isfinite(grid))[0]
    got = fp8.e4m3_decode(fp8.e4m3_encode(x))
    for xi, gi in zip(x, got):
        best = np.min(np.abs(grid[finite] - np.clip(xi, -448, 448)))
        assert abs(gi - np.clip(xi, -448, 448)) == best, (xi, gi)


def test_encode_ties_go_to_the_even_mantissa():
    grid = fp8.e4m3_decode(np.arange(127, dtype=np.uint8))
    mids = (grid[:-1] + grid[1:]) / 2            # exactly representable in fp64
    codes = fp8.e4m3_encode(mids)
    lower = np.arange(126)
    expect = np.where(lower % 2 == 0, lower, lower + 1)
    assert np.array_equal(codes, expect.astype(np.uint8))
    assert np.array_equal(fp8.e4m3_encode(-mids), (expect | 0x80).astype(np.uint8))
    # just off a tie the nearer neighbour wins
    assert np.array_equal(fp8.e4m3_encode(np.nextafter(mids, np.inf)), (lower + 1).astype(np.uint8))
    assert np.array_equal(fp8.e4m3_encode(np.nextafter(mids, -np.inf)), lower.astype(np.uint8))


def test_encode_saturates_and_keeps_nan():
    c = fp8.e4m3_encode(np.array([449.0, 464.0, 1e30, np.inf, -500.0, -np.inf, np.nan, 2.0 ** -11, 2.0 ** -10, 0.0, -0.0]))
    # 2^-10 is the tie between 0 and the smallest subnormal: even code 0; below it rounds to 0
    assert list(c[:6]) == [0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE]
    assert c[6] & 0x7F == 0x7F
    assert list(c[7:]) == [0x00, 0x00, 0x00, 0x80]


def test_encode_agrees_with_torch_inside_the_finite_range():
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.normal(0, 1, 3000), rng.normal(0, 120, 3000), rng.uniform(-0.02, 0.02, 3000)]).astype(np.float32)
    x = np.clip(x, -448, 448)
    grid = fp8.e4m3_decode(np.arange(127, dtype=np.uint8))
    x = np.concatenate([x, ((grid[:-1] + grid[1:]) / 2).astype(np.float32)])     # ties are exact in fp32 too
    t = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(fp8.e4m3_encode(x.astype(np.float64)), t)


def test_quantize_divides_in_fp32():
    # 1/3 in fp32 differs from 1/3 in fp64; pick x so that the fp32 quotient lands exactly on a tie and the fp64 one does not
    scale = np.float32(3.0)
    x = np.float32(3.0) * np.float32(1.0625)          # 1.0625 is the tie between 1.0 and 1.125
    assert fp8.quantize(np.array([x], dtype=np.float32), scale)[0] == 0x38      # tie -> even (1.0)
    assert fp8.quantize(np.array([2.0, -7.0, 0.0], dtype=np.float32), 0.5).tolist() == [0x48, 0xD6, 0x00]  # 4, -14, 0


def test_every_e4m3_value_is_a_bf16_value():
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    bits = fp8.e4m3_as_bf16_bits(codes)
    back = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(back, fp8.e4m3_decode(codes))


def test_attention_over_an_8bit_cache_is_attention_over_the_decoded_values():
    # numpy softmax attention in fp64 on decode(code) * scale, written out here, against the composed routine
    rng = np.random.default_rng(3)
    B, Hq, Hkv, D = 3, 4, 2, 64
    lengths = np.array([5, 0, 9], dtype=np.int32)
    offsets = np.array([0, 5, 7], dtype=np.int32)          # two unowned rows (5, 6) that hold NaN codes
    T = 16
    Ks8 = rng.integers(0, 256, (T, Hkv, D)).astype(np.uint8)
    Vs8 = rng.integers(0, 256, (T, Hkv, D)).astype(np.uint8)
    for a in (Ks8, Vs8):
        nan = (a & 0x7F) == 0x7F
        a[nan] = 0x3A
        a[5:7] = 0x7F
    Ks8 = (Ks8 & 0xBF) | 0x20      # keep magnitudes moderate so that the softmax is not one-hot
    Q = wl.f32_to_bf16_bits(rng.normal(0, 1, (B, Hq, D)).astype(np.float32))
    ks, vs, scale = 0.043, 1.7, 0.125
    O, LSE = fp8.suffix_attention_fp8(Q, Hkv, Ks8, Vs8, ks, vs, offsets, lengths, scale)
    q = wl.bf16_bits_to_f32(Q).astype(np.float64)
    for b in range(B):
        for h in range(Hq):
            kv = h // (Hq // Hkv)
            rows = slice(int(offsets[b]), int(offsets[b]) + int(lengths[b]))
            K = fp8.e4m3_decode(Ks8[rows, kv]) * float(np.float32(ks))
            V = fp8.e4m3_decode(Vs8[rows, kv]) * float(np.float32(vs))
            if lengths[b] == 0:
                assert np.all(O[b, h] == 0) and LSE[b, h] == -np.inf
                continue
            s = K @ q[b, h] * scale
            m = s.max()
            p = np.exp(s - m)
            assert np.allclose(O[b, h], p @ V / p.sum(), rtol=1e-12, atol=1e-12)
            assert np.isclose(LSE[b, h], m + np.log(p.sum()), rtol=1e-12)


def test_append_on_an_8bit_cache_by_hand():
    Hkv, D = 1, 64
    Ks8 = np.zeros((6, Hkv, D), dtype=np.uint8)
    Vs8 = np.zeros((6, Hkv, D), dtype=np.uint8)
    offsets = np.array([0, 3], dtype=np.int32)
    lengths = np.array([1, 3], dtype=np.int32)      # the second sequence is full (capacity 3)
    Knew = np.full((2, Hkv, D), 3.0, dtype=np.float32)
    Vnew = np.full((2, Hkv, D), -0.75, dtype=np.float32)
    K2, V2, L2 = fp8.kv_append_fp8(Ks8, Vs8, offsets, lengths, 3, Knew, Vnew, 2.0, 0.5)
    assert L2.tolist() == [2, 3]
    assert (K2[1] == 0x3C).all() and (V2[1] == 0xBC).all()     # 3/2 = 1.5 -> 0x3c; -0.75/0.5 = -1.5 -> 0xbc
    assert (K2[[0, 2, 3, 4, 5]] == 0).all() and (V2[[0, 2, 3, 4, 5]] == 0).all()
    assert (Ks8 == 0).all()
