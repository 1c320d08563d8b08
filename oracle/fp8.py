"""FP8 E4M3 codes for the KV cache (test infrastructure only; plain numpy, written from the OCP 8-bit
floating point format: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, the single NaN
pattern S.1111.111, largest finite value 448, subnormals m/8 * 2^-6).

The paper stores the KV cache in the model's 16-bit type; an 8-bit cache on the decode instance is this
build's extension of Sec. 3.3.4 / 3.4 (half the bytes on the link between the instances and half the bytes a
decode iteration reads).  The reading taken: a value x of the cache is stored as the code of
    clamp(fl32(x * inv_scale), -448, 448)   rounded to nearest E4M3, ties to even,
with inv_scale = fl32(1 / scale) and one scale per tensor (K, V); a code c stands for value(c) * scale.
"""
import numpy as np

MAX = 448.0


def decode_table():
    """The value of each of the 256 codes (float64; NaN for 0x7F and 0xFF), from the format definition."""
    t = np.zeros(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e, m = (code >> 3) & 0xF, code & 0x7
        if e == 0xF and m == 0x7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sign * (m / 8.0) * 2.0 ** -6
        else:
            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


def encode(y):
    """Codes (uint8) of float32 values y: clamp to [-448, 448], round to nearest representable value,
    ties to the code with even mantissa.  Searches the table of values: slow and plain."""
    y = np.asarray(y, dtype=np.float32).astype(np.float64)
    flat = np.clip(y.reshape(-1), -MAX, MAX)
    table = decode_table()
    pos_codes = np.arange(0, 0x7F)                     # 0x00 .. 0x7E: non-negative finite values, ascending
    pos_vals = table[pos_codes]
    out = np.zeros(flat.shape, dtype=np.uint8)
    for i, v in enumerate(flat):
        a = abs(v)
        hi = int(np.searchsorted(pos_vals, a, side="left"))      # first value >= a
        if hi == 0:
            code = 0
        elif hi >= len(pos_vals):
            code = 0x7E
        else:
            lo = hi - 1
            d_lo, d_hi = a - pos_vals[lo], pos_vals[hi] - a
            if d_lo < d_hi:
                code = lo
            elif d_hi < d_lo:
                code = hi
            else:
                code = lo if lo % 2 == 0 else hi      # consecutive codes: the even one has mantissa bit 0 clear
        out[i] = code | (0x80 if (v < 0 or (v == 0 and np.signbit(v))) else 0)
    return out.reshape(y.shape)


def quantize(x, scale):
    """Codes of cache values x (float32 holding bf16 values) under one per-tensor scale."""
    inv = np.float32(1.0) / np.float32(scale)
    with np.errstate(over="ignore"):                   # a product that overflows to infinity saturates below
        return encode(np.asarray(x, dtype=np.float32) * inv)


def dequantize(codes, scale):
    return decode_table()[np.asarray(codes, dtype=np.uint8)] * np.float64(np.float32(scale))
