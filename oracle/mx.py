"""Block-scaled (MX) outputs in the oracle.  TEST INFRASTRUCTURE ONLY.

Some of the benchmark kernels of GEAK section 4.1 (Table 1: the MXFP matmul, the fp8 kernels) belong to a
family whose outputs may be quantised: a payload of narrow elements plus one shared scale per block of 32
elements (OCP Microscaling Formats (MX) specification v1.0).  Two such tensors are equivalent when the VALUES
they stand for are close under the rule of section 3.1 -- a candidate may pick another scale for a block and
still encode the same numbers -- so the oracle first writes every element out as the value it encodes and then
applies the unchanged binary32 rule (check_segment with dtype "f32").

Value of element i of a block with scale byte X and payload code P_i (the specification's section 5 and 6):
    X == 0xFF                       -> NaN for all 32 elements
    otherwise                       -> 2^(X - 127) * value(P_i)
with value(P) by the element format's own definition (sign, exponent, mantissa; subnormals; the format's NaN and
infinity codes, which the scale does not change).  The product is formed exactly (binary64 holds it) and then
rounded to binary32, the precision the rule runs in: it is exact there too unless it overflows binary32, where
it becomes +-Inf (E4M3's 448 * 2^127, say) -- the specification leaves that case to the implementation; this is
the reading used here and by the kernels.

Formats: "mxfp8e4m3", "mxfp8e5m2" (one byte per element), "mxfp4e2m1" (two elements per byte, element 2j in the
low nibble of byte j), "mxfp6e2m3", "mxfp6e3m2" (six bits per element, no infinities and no NaN; the specification
does not fix how they lie in memory: here the codes are packed without gaps, element i in bits 6 i .. 6 i + 5 of the
payload read as one little-endian number, so a block of 32 elements is 24 bytes), "mxint8" (two's complement,
value P / 64).  Plain Python loops and numpy; nothing here is shared with the HIP path.
"""
from __future__ import annotations

import math

import numpy as np

from .oracle import check_segment, report_segment

MX_BLOCK = 32
MX_FORMATS = ("mxfp8e4m3", "mxfp8e5m2", "mxfp4e2m1", "mxint8", "mxfp6e2m3", "mxfp6e3m2")
MX_BITS = {"mxfp8e4m3": 8, "mxfp8e5m2": 8, "mxfp4e2m1": 4, "mxint8": 8, "mxfp6e2m3": 6, "mxfp6e3m2": 6}


def minifloat_value(code: int, ebits: int, mbits: int, bias: int, ieee_specials: bool, nan_is_all_ones: bool) -> float:
    """Value of a sign / exponent / mantissa code of 1 + ebits + mbits bits.  ieee_specials: the largest
    exponent encodes infinity (mantissa 0) and NaN (else), as in E5M2; nan_is_all_ones: only exponent and mantissa
    all ones is NaN and there is no infinity, as in E4M3; neither: every code is a number, as in E2M1."""
    sign = -1.0 if (code >> (ebits + mbits)) & 1 else 1.0
    e = (code >> mbits) & ((1 << ebits) - 1)
    m = code & ((1 << mbits) - 1)
    if ieee_specials and e == (1 << ebits) - 1:
        return sign * math.inf if m == 0 else math.nan
    if nan_is_all_ones and e == (1 << ebits) - 1 and m == (1 << mbits) - 1:
        return math.nan
    if e == 0:
        return sign * m * 2.0 ** (1 - bias - mbits)                     # subnormal (and zero)
    return sign * (1.0 + m * 2.0 ** -mbits) * 2.0 ** (e - bias)


def element_table(fmt: str) -> np.ndarray:
    """value(P) for every code P of the element format, binary64."""
    if fmt == "mxfp8e4m3":
        return np.array([minifloat_value(c, 4, 3, 7, False, True) for c in range(256)])
    if fmt == "mxfp8e5m2":
        return np.array([minifloat_value(c, 5, 2, 15, True, False) for c in range(256)])
    if fmt == "mxfp4e2m1":
        return np.array([minifloat_value(c, 2, 1, 1, False, False) for c in range(16)])
    if fmt == "mxfp6e2m3":
        return np.array([minifloat_value(c, 2, 3, 1, False, False) for c in range(64)])
    if fmt == "mxfp6e3m2":
        return np.array([minifloat_value(c, 3, 2, 3, False, False) for c in range(64)])
    if fmt == "mxint8":
        return np.array([(c - 256 if c >= 128 else c) / 64.0 for c in range(256)])
    raise ValueError(fmt)


def scale_value(x: int) -> float:
    """The shared scale an E8M0 byte stands for: a power of two, or NaN."""
    return math.nan if x == 0xFF else 2.0 ** (x - 127)


def payload_codes(payload, numel: int, fmt: str) -> np.ndarray:
    """The numel element codes of a payload, one per entry."""
    raw = np.ascontiguousarray(payload).view(np.uint8).reshape(-1)
    if MX_BITS[fmt] == 8:
        return raw[:numel].astype(np.int64)
    codes = np.zeros(numel, dtype=np.int64)
    if MX_BITS[fmt] == 6:
        for i in range(numel):
            bit = 6 * i                                                  # the code may straddle two bytes
            pair = int(raw[bit // 8]) | (int(raw[bit // 8 + 1]) << 8 if bit % 8 > 2 else 0)
            codes[i] = (pair >> (bit % 8)) & 0x3F
        return codes
    for i in range(numel):
        byte = int(raw[i // 2])
        codes[i] = (byte >> 4) & 0xF if i % 2 else byte & 0xF
    return codes


def dequantize(payload, scales, numel: int, fmt: str) -> np.ndarray:
    """The numel values as binary32, element by element."""
    table = element_table(fmt)
    codes = payload_codes(payload, numel, fmt)
    sc = np.ascontiguousarray(scales).view(np.uint8).reshape(-1)
    out = np.zeros(numel, dtype=np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        for i in range(numel):
            x = scale_value(int(sc[i // MX_BLOCK]))
            v = math.nan if math.isnan(x) else float(table[codes[i]]) * x          # exact in binary64
            out[i] = np.float32(v)                                                # rounds only by overflowing
    return out


def check_segment_mx(ref_payload, ref_scales, cand_payload, cand_scales, numel: int, fmt: str, atol: float, rtol: float,
                     equal_nan: bool):
    """One (segment, candidate) pair of block-scaled tensors: the record of the binary32 rule on the values."""
    b = dequantize(ref_payload, ref_scales, numel, fmt)
    a = dequantize(cand_payload, cand_scales, numel, fmt)
    return check_segment(b, a, numel, "f32", atol, rtol, equal_nan)


def report_segment_mx(ref_payload, ref_scales, cand_payload, cand_scales, numel: int, fmt: str, atol: float, rtol: float,
                      equal_nan: bool, max_records: int):
    b = dequantize(ref_payload, ref_scales, numel, fmt)
    a = dequantize(cand_payload, cand_scales, numel, fmt)
    return report_segment(b, a, numel, "f32", atol, rtol, equal_nan, max_records)
