"""8-bit suffix cache: the E4M3 number format and what attention over such a cache means.  TEST INFRASTRUCTURE ONLY.

Not part of the paper: a bandwidth variant of the suffix part of Sec. 3.2 in which suffix keys and values are stored
as 8-bit floating-point codes with one fp32 scale per tensor, value = decode(code) * scale.  The format is the OCP
8-bit floating point E4M3 ("FN": finite, no infinities): 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits;
exponent field 0 holds subnormals m/8 * 2^-6; exponent field 15 with mantissa 7 is NaN and every other code is a
finite number, the largest 1.75 * 2^8 = 448.

  decode   : the definition above, code by code.
  encode   : the nearest representable value, ties to the code with an even mantissa bit, magnitudes above 448
             saturate to 448, NaN stays NaN; the sign is kept (also of zero).
  quantize : encode(x / scale) with the division taken in fp32 (the precision the device takes it in: the quotient
             decides an integer code, so both sides must form it the same way).
  attention: linear algebra only.  Scores are q . (decode(k) * k_scale) * scale = q . decode(k) * (k_scale * scale)
             and the output is (sum_j p_j decode(v_j)) * v_scale, so the exact attention routine of this package is
             called on the decoded codes (every E4M3 value is exactly a bf16 value) with the scale k_scale * scale,
             and its output is multiplied by v_scale.

Pinned in tests/test_fp8_pins.py: code values the format's definition fixes, the round trip over all codes, brute
force nearest-value search, ties, saturation, and torch's float8_e4m3fn conversions (an independent implementation).
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode(codes) -> np.ndarray:
    """uint8 codes -> float64 values (NaN for the two NaN codes)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where((c >> 7) & 1, -1.0, 1.0)
    e = (c >> 3) & 15
    m = c & 7
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    sub = (m / 8.0) * 2.0 ** -6
    v = np.where(e == 0, sub, normal)
    v = np.where((e == 15) & (m == 7), np.nan, v)
    return sign * v


def _positive_grid() -> np.ndarray:
    """The 127 finite non-negative values in code order (codes 0 .. 126), which is also increasing order."""
    return e4m3_decode(np.arange(127, dtype=np.uint8))


def e4m3_encode(x) -> np.ndarray:
    """float values -> uint8 codes: nearest value, ties to even mantissa, saturating; NaN -> a NaN code (0x7f or 0xff)."""
    x = np.asarray(x, dtype=np.float64)
    grid = _positive_grid()
    out = np.empty(x.shape, dtype=np.uint8)
    flat_x = x.reshape(-1)
    flat_o = out.reshape(-1)
    for i in range(flat_x.shape[0]):
        v = flat_x[i]
        s = 0x80 if np.signbit(v) else 0
        if np.isnan(v):
            flat_o[i] = s | 0x7F
            continue
        a = min(abs(v), E4M3_MAX)
        hi = int(np.searchsorted(grid, a, side="left"))      # first code whose value is >= a
        if grid[hi] == a:
            code = hi
        else:
            lo = hi - 1
            dl, dh = a - grid[lo], grid[hi] - a
            if dl < dh:
                code = lo
            elif dh < dl:
                code = hi
            else:
                code = lo if lo % 2 == 0 else hi              # the mantissa's last bit is the code's last bit
        flat_o[i] = s | code
    return out


def quantize(x_f32, scale: float) -> np.ndarray:
    """Codes of x / scale; x and scale are taken as fp32 and the quotient is the fp32 quotient."""
    q = np.asarray(x_f32, dtype=np.float32) / np.float32(scale)
    return e4m3_encode(q.astype(np.float64))


def e4m3_as_bf16_bits(codes) -> np.ndarray:
    """The bf16 bit patterns of the decoded values (exact: 4 significant bits, exponents -9 .. 8)."""
    v = e4m3_decode(codes).astype(np.float32)
    assert not np.isnan(v).any(), "NaN codes have no place in a cache row that is read"
    bits = v.view(np.uint32)
    assert not (bits & 0xFFFF).any()
    return (bits >> 16).astype(np.uint16)


def suffix_attention_fp8(Q, Hkv: int, Ks8, Vs8, k_scale: float, v_scale: float, offsets, lengths, scale=None):
    """Exact suffix attention over an 8-bit cache.  Q: bf16 bits [B,Hq,D] or [B,nq,Hq,D]; Ks8, Vs8: uint8 [T,Hkv,D].

    Rows outside every sequence's range may hold any code (NaN codes included): they are replaced by zero before the
    exact routine sees them, as they carry no weight.  Returns (O, LSE) in float64.
    """
    from . import attention_arrays

    Ks8 = np.asarray(Ks8, dtype=np.uint8).copy()
    Vs8 = np.asarray(Vs8, dtype=np.uint8).copy()
    offsets = np.asarray(offsets)
    lengths = np.asarray(lengths)
    owned = np.zeros(Ks8.shape[0], dtype=bool)
    for b in range(lengths.shape[0]):
        owned[int(offsets[b]): int(offsets[b]) + int(lengths[b])] = True
    Ks8[~owned] = 0
    Vs8[~owned] = 0
    D = Q.shape[-1]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O, LSE = attention_arrays(Q, Hkv, [], e4m3_as_bf16_bits(Ks8), e4m3_as_bf16_bits(Vs8), offsets, lengths,
                              float(scale) * float(np.float32(k_scale)))
    return O * float(np.float32(v_scale)), LSE


def kv_append_fp8(Ks8, Vs8, offsets, lengths, capacity: int, Knew_f32, Vnew_f32, k_scale: float, v_scale: float):
    """Cache update of a decode step on an 8-bit cache: the new rows are quantized, then placed as in kv_append.

    Knew_f32, Vnew_f32: the new rows' values (fp32 arrays holding bf16 values), [B,Hkv,D] or [B,nq,Hkv,D].
    Returns new (Ks8, Vs8, lengths).
    """
    from .kvcache import kv_append

    return kv_append(np.asarray(Ks8, dtype=np.uint8), np.asarray(Vs8, dtype=np.uint8), offsets, lengths, capacity,
                     quantize(Knew_f32, k_scale), quantize(Vnew_f32, v_scale))
