"""bf16 <-> fp64 conversion for the oracle (test infrastructure).

bf16 is the upper half of an IEEE-754 binary32 word: 1 sign, 8 exponent and 7
fraction bits.  Decoding is exact; encoding rounds to nearest, ties to even,
directly from fp64 (no intermediate fp32 rounding).
"""
import numpy as np


def decode(bits) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    with np.errstate(invalid="ignore"):          # signalling-NaN patterns widen quietly
        return b.view(np.float32).astype(np.float64)


def decode_fields(bits) -> np.ndarray:
    """Same as :func:`decode`, spelled out from the sign/exponent/fraction
    fields (used to pin :func:`decode`)."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.int64)
    sign = np.where((b >> 15) & 1, -1.0, 1.0)
    e = (b >> 7) & 0xFF
    f = (b & 0x7F).astype(np.float64)
    normal = sign * (1.0 + f / 128.0) * np.exp2((e - 127).astype(np.float64))
    sub = sign * (f / 128.0) * 2.0 ** -126
    out = np.where(e == 0, sub, normal)
    out = np.where((e == 255) & (f == 0), sign * np.inf, out)
    out = np.where((e == 255) & (f != 0), np.nan, out)
    return out


def encode_rne(x) -> np.ndarray:
    """float64 -> bf16 bit patterns, round to nearest even."""
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(x.shape, dtype=np.uint16)
    flat_x = x.reshape(-1)
    flat_o = out.reshape(-1)
    for i, v in enumerate(flat_x):
        flat_o[i] = _encode_one(float(v))
    return out


def _encode_one(v: float) -> int:
    if v != v:
        return 0x7FC0
    sign = 0x8000 if (v < 0 or (v == 0 and np.signbit(v))) else 0
    a = abs(v)
    if a == 0.0:
        return sign
    if a == np.inf:
        return sign | 0x7F80
    m, e = np.frexp(a)                 # a = m * 2**e, m in [0.5, 1)
    # normal bf16: 8 significant bits, unbiased exponent of the leading bit e-1
    lead = e - 1
    if lead < -126:                    # subnormal range: fixed quantum 2**-133
        q = int(np.rint(np.ldexp(a, 133)))
        return sign | q                # q == 128 rolls into the smallest normal
    q = int(np.rint(np.ldexp(m, 8)))   # in [128, 256]
    if q == 256:
        q = 128
        lead += 1
    if lead > 127:
        return sign | 0x7F80
    return sign | ((lead + 127) << 7) | (q - 128)
