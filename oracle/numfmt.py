"""Number formats for the oracle: decode stored bit patterns to fp64, and round
an fp64 result once, to nearest even, to the dtype it is compared in.

The paper states no precision; the formats are those of the benchmark
configurations (bf16, fp8 e4m3 in the OCP "fn" encoding with a per-tensor
scale, fp32).  Written from the formats' definitions, independently of the
input generators' encoders and of the GPU code.
"""
import numpy as np


def decode_bf16(bits):
    """uint16 bf16 patterns -> fp64 (bf16 is the top half of an IEEE fp32)."""
    bits = np.asarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):       # signalling-NaN patterns stay NaN
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def _e4m3_table():
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            v = float("nan")            # the only non-finite pattern
        elif e == 0:
            v = (m / 8.0) * 2.0 ** -6   # subnormal
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[code] = sign * v
    return t


_E4M3 = _e4m3_table()


def decode_e4m3(codes, scale=1.0):
    """uint8 fp8-e4m3 codes times the per-tensor scale -> fp64."""
    codes = np.asarray(codes, dtype=np.uint8)
    return _E4M3[codes] * float(scale)


def decode(raw, dtype, scale=1.0):
    if dtype == "f32":
        return np.asarray(raw, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return decode_bf16(raw)
    if dtype == "fp8_e4m3":
        return decode_e4m3(raw, scale)
    raise ValueError(dtype)


def round_to_bf16(x):
    """fp64 -> nearest bf16 value (ties to even), returned as fp64.

    bf16 keeps 8 significant bits with the fp32 exponent range, so the spacing
    at ``x = m * 2**e`` (0.5 <= |m| < 1) is ``2**(e-8)``, never below the
    subnormal spacing ``2**-133``.
    """
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    e = np.maximum(e, -125)
    quantum = np.ldexp(1.0, e - 8)
    r = np.rint(x / quantum) * quantum      # rint rounds ties to even
    big = np.ldexp(1.0, 128)                # first magnitude that does not fit
    r = np.where(np.abs(r) >= big, np.copysign(np.inf, r), r)
    return np.where(np.isfinite(x), r, x)


def bf16_bits(x):
    """bit pattern (uint16) of a value that is exactly representable in bf16."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def round_to_f32(x):
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_to(x, dtype):
    if dtype == "f32":
        return round_to_f32(x)
    if dtype == "bf16":
        return round_to_bf16(x)
    raise ValueError(dtype)
