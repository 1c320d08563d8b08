"""Pins of the FP8 E4M3 oracle (format definition: OCP 8-bit floating point) against things other than itself:
hand-written values of the format, torch's CPU float8_e4m3fn conversion as a black box (inside the finite
range; torch turns overflow into NaN, the cache format here saturates), and invariants."""
import numpy as np
import torch

from oracle import fp8


def test_hand_written_codes():
    t = fp8.decode_table()
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and np.signbit(t[0x80])
    assert t[0x38] == 1.0 and t[0x3C] == 1.5 and t[0x40] == 2.0 and t[0xB8] == -1.0
    assert t[0x7E] == 448.0 and t[0x78] == 256.0 and t[0x77] == 240.0
    assert t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9 and t[0x08] == 2.0 ** -6
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])


def test_table_equals_library_view():
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    t = fp8.decode_table()
    assert np.array_equal(np.isnan(lib), np.isnan(t))
    ok = ~np.isnan(t)
    assert np.array_equal(lib[ok], t[ok]) and np.array_equal(np.signbit(lib[ok]), np.signbit(t[ok]))


def test_hand_written_roundings():
    enc = lambda v: int(fp8.encode(np.float32(v)))
    assert enc(1.0) == 0x38 and enc(-1.0) == 0xB8 and enc(0.0) == 0x00 and enc(-0.0) == 0x80
    assert enc(1.0625) == 0x38            # tie between 1.0 (mantissa 000) and 1.125 (001): even
    assert enc(1.1875) == 0x3A            # tie between 1.125 (001) and 1.25 (010): even
    assert enc(1.07) == 0x39 and enc(1.05) == 0x38
    assert enc(448.0) == 0x7E and enc(460.0) == 0x7E and enc(1e9) == 0x7E and enc(-1e9) == 0xFE   # saturates
    assert enc(2.0 ** -10) == 0x00        # tie between 0 and the smallest subnormal: even
    assert enc(2.0 ** -10 * 1.01) == 0x01 and enc(3 * 2.0 ** -10) == 0x02      # tie 1|2 -> even
    assert enc(2.0 ** -6) == 0x08 and enc(0.3) == 0x2A  # 0.3 -> 0.3125 = 1.25 * 2^-2


def test_encode_matches_library_on_every_bf16_value_in_range():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).float()
    keep = torch.isfinite(vals) & (vals.abs() <= 448.0)
    x = vals[keep]
    lib = x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(fp8.encode(x.numpy()), lib)


def test_encode_matches_library_on_scaled_random_floats():
    rng = np.random.default_rng(71)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-12, 6, size=20000))).astype(np.float32)
    x = x[np.abs(x) <= 448.0]
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(fp8.encode(x), lib)


def test_round_trip_and_monotone():
    t = fp8.decode_table()
    codes = np.array([c for c in range(256) if not np.isnan(t[c])], dtype=np.uint8)
    assert np.array_equal(fp8.encode(t[codes].astype(np.float32)), codes)
    xs = np.linspace(-460, 460, 20001).astype(np.float32)
    vals = t[fp8.encode(xs)]
    assert (np.diff(vals) >= 0).all()
    assert np.abs(vals - np.clip(xs, -448, 448)).max() <= 16.0       # half of the largest spacing (32)


def test_quantize_uses_the_float32_reciprocal():
    x = np.float32(3.0)
    for scale in (0.37, 2.0, 1.0 / 3.0):
        inv = np.float32(1.0) / np.float32(scale)
        assert fp8.quantize(x, scale) == fp8.encode(np.float32(x * inv))
    assert np.allclose(fp8.dequantize(fp8.quantize(np.float32(0.5), 0.01), 0.01), 0.5, rtol=0.07)


def test_export_fp8_hand_example_and_scales():
    """Pages of 2 slots, one head, one element: K values 3, -1.5 under scale 0.5 -> codes of 6 and -3;
    V values 0.75, 100 under scale 0.25 -> codes of 3 and 400."""
    from oracle import kv_transfer
    pool = np.zeros((3, 2, 1, 2, 1), dtype=np.float32)
    pool[2, 0, 0, 1, 0], pool[0, 0, 0, 0, 0] = 3.0, -1.5       # request tokens 1, 2 -> page 2 slot 1, page 0 slot 0
    pool[2, 1, 0, 1, 0], pool[0, 1, 0, 0, 0] = 0.75, 100.0
    bt = np.array([[2, 0]], dtype=np.int32)
    codes = kv_transfer.kv_export_fp8(pool, bt, [0, 2], [1], 0.5, 0.25)
    t = fp8.decode_table()
    assert t[codes].tolist() == [6.0, -3.0, 3.0, 384.0]        # 400 lies between 384 and 416: nearer to 384


def test_decode_fp8_closed_forms():
    """All cached keys are the zero code: equal scores, so the output is the mean of the dequantised cached
    values and the new token's own value, written out from the table by hand."""
    from oracle import decode
    rng = np.random.default_rng(72)
    hq, hkv, d, P, L = 4, 2, 8, 16, 21
    codes = np.zeros((4, 2, hkv, P, d), dtype=np.uint8)
    bt = np.array([[2, 0, 3]], dtype=np.int32)
    vcodes = rng.integers(0, 0x7F, size=(L, hkv, d)).astype(np.uint8)
    for j in range(L):
        codes[bt[0][j // P], 1, :, j % P, :] = vcodes[j]
    t = fp8.decode_table()
    q = rng.standard_normal((1, hq, d)).astype(np.float32)
    v_new = rng.standard_normal((1, hkv, d)).astype(np.float32)
    out = decode.decode_attn_fp8(q, np.zeros((1, hkv, d), np.float32), v_new, codes, bt, [L], 0.7, 3.0, 0.125)
    for h in range(hq):
        want = (t[vcodes[:, h // 2, :]].sum(axis=0) * 0.125 + v_new[0, h // 2]) / (L + 1)
        assert np.abs(out[0, h] - want).max() <= 1e-12
    # the K scale multiplies the cached scores only: one cached key with code of 2.0 and scale 5 scores 10 * q0
    codes[:] = 0
    codes[bt[0][0], 0, :, 0, 0] = 0x40                     # 2.0
    codes[bt[0][0], 1, :, 0, :] = 0x38                     # value 1.0 (times v_scale)
    q1 = np.zeros((1, hq, d), np.float32)
    q1[0, :, 0] = 1.0
    out = decode.decode_attn_fp8(q1, np.zeros((1, hkv, d), np.float32), np.zeros((1, hkv, d), np.float32), codes, bt,
                                 [1], 1.0, 5.0, 0.5)
    w = np.exp(10.0) / (np.exp(10.0) + 1.0)
    assert np.abs(out[0] - w * 0.5).max() <= 1e-12


def test_decode_append_fp8_places_the_codes():
    from oracle import decode
    codes = np.full((3, 2, 1, 16, 2), 0x7F, dtype=np.uint8)
    bt = np.array([[1, 2], [0, 0]], dtype=np.int32)
    k = np.array([[[1.0, -2.0]], [[0.5, 448.0]]], dtype=np.float32)
    v = np.array([[[3.0, 0.25]], [[-1.0, 8.0]]], dtype=np.float32)
    decode.decode_append_fp8(k, v, codes, bt, [17, 0], 1.0, 2.0)
    t = fp8.decode_table()
    assert t[codes[2, 0, 0, 1]].tolist() == [1.0, -2.0] and t[codes[2, 1, 0, 1]].tolist() == [1.5, 0.125]
    assert t[codes[0, 0, 0, 0]].tolist() == [0.5, 448.0] and t[codes[0, 1, 0, 0]].tolist() == [-0.5, 4.0]
    assert (codes == 0x7F).sum() == codes.size - 8


def test_the_product_is_rounded_to_float32_before_the_code_is_chosen():
    """Two inputs where the definition's single-precision product and an exact division fall on different
    sides of a code boundary.  x = 4.5 * 2^-10 with scale 0.3f: fl32(1 / 0.3f) = 3.33333325..., the product
    0.01464843712... rounds in float32 to 7.5 * 2^-9 exactly, a tie between the codes 7 and 8 -> 8 (even);
    the exact quotient 0.014648436918 lies below the tie and would give 7.  With scale 1.7f and
    x = 0.02490234375 the float32 product lies below the same tie (-> 7), the exact quotient above it."""
    assert int(fp8.quantize(np.float32(4.5 * 2.0 ** -10), 0.3)) == 0x08
    assert int(fp8.quantize(np.float32(0.02490234375), 1.7)) == 0x07
