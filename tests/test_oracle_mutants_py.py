"""Planted mistakes in the numpy oracles (KV transfer, decode iteration, FP8 codes, chunked prefill over a cache of
codes) must be caught by their pins.

Each mutant is the oracle's source with one plausible slip; it is executed as a module of its own,
swapped in for the real one inside the pin-test module, and every pin is run against it: at least one
has to fail.  CPU only.
"""
import inspect
import types

import pytest

import test_oracle_decode as decode_pins
import test_oracle_fp8 as fp8_pins
import test_oracle_kv_transfer as transfer_pins
import test_oracle_prefill_fp8 as prefill_fp8_pins
from oracle import decode, fp8, kv_transfer, prefill_fp8

TRANSFER_SRC = inspect.getsource(kv_transfer)
DECODE_SRC = inspect.getsource(decode)
FP8_SRC = inspect.getsource(fp8)
PREFILL_FP8_SRC = inspect.getsource(prefill_fp8).replace("from . import fp8", "from oracle import fp8")

PREFILL_FP8_MUTANTS = {
    "scale-on-own-keys": ("    keys[L:] = k_new[a:b, kh, :]", "    keys[L:] = k_new[a:b, kh, :] * 0.5"),
    "scale-on-own-values": ("    vals[L:] = v_new[a:b, kh, :]", "    vals[L:] = v_new[a:b, kh, :] * 0.5"),
    "scales-swapped": ("    k_vals = fp8.dequantize(kv_codes[:, 0], k_scale)\n    v_vals = fp8.dequantize(kv_codes[:, 1], v_scale)",
                       "    k_vals = fp8.dequantize(kv_codes[:, 0], v_scale)\n    v_vals = fp8.dequantize(kv_codes[:, 1], k_scale)"),
    "values-from-keys": ("        vals[j] = v_vals[page, kh, j % P, :]", "        vals[j] = k_vals[page, kh, j % P, :]"),
    "slot-index": ("        keys[j] = k_vals[page, kh, j % P, :]", "        keys[j] = k_vals[page, kh, j // P % P, :]"),
    "table-row": ("            keys, vals = _segment_kv(k_new, v_new, k_vals, v_vals, block_table[s], L, a, b, kh, P)",
                  "            keys, vals = _segment_kv(k_new, v_new, k_vals, v_vals, block_table[0], L, a, b, kh, P)"),
    "own-position-masked": ("                    out[a + t, h] = _one_row(q[a + t, h], keys, vals, L + t + 1, scale)",
                            "                    out[a + t, h] = _one_row(q[a + t, h], keys, vals, max(L + t, 1), scale)"),
    "sees-the-future": ("                    out[a + t, h] = _one_row(q[a + t, h], keys, vals, L + t + 1, scale)",
                        "                    out[a + t, h] = _one_row(q[a + t, h], keys, vals, L + (b - a), scale)"),
    "gqa-mapping": ("            for h in range(kh * g, (kh + 1) * g):", "            for h in range(kh, Hq, Hkv):"),
    "drop-scale": ("    s = scale * (keys[:visible] @ qrow)", "    s = keys[:visible] @ qrow"),
    "samples-forget-k-scale": ("            keys = np.concatenate([table[kc] * ks, k_new[a:b, kh, :]], axis=0)",
                               "            keys = np.concatenate([table[kc], k_new[a:b, kh, :]], axis=0)"),
    "samples-row-offset": ("        out[i] = _one_row(q[r, h], keys, vals, L + (r - a) + 1, scale)",
                           "        out[i] = _one_row(q[r, h], keys, vals, L + r + 1, scale)"),
    "append-slot": ("            kv_codes[page, 0, :, pos % P, :] = fp8.quantize(np.asarray(k_new[a + t], dtype=np.float32), k_scale)",
                    "            kv_codes[page, 0, :, t % P, :] = fp8.quantize(np.asarray(k_new[a + t], dtype=np.float32), k_scale)"),
    "append-v-under-k-scale": ("fp8.quantize(np.asarray(v_new[a + t], dtype=np.float32), v_scale)",
                               "fp8.quantize(np.asarray(v_new[a + t], dtype=np.float32), k_scale)"),
    "append-ignores-context": ("            pos = L + t\n            page = int(block_table[s][pos // P])\n            kv_codes[page, 0",
                               "            pos = t\n            page = int(block_table[s][pos // P])\n            kv_codes[page, 0"),
    "append-chunk-row": ("fp8.quantize(np.asarray(k_new[a + t], dtype=np.float32), k_scale)",
                         "fp8.quantize(np.asarray(k_new[t], dtype=np.float32), k_scale)"),
}

FP8_MUTANTS = {
    "exponent-bias": ("            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)", "            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 8)"),
    "subnormal-exponent": ("            t[code] = sign * (m / 8.0) * 2.0 ** -6", "            t[code] = sign * (m / 8.0) * 2.0 ** -7"),
    "mantissa-bits": ("        e, m = (code >> 3) & 0xF, code & 0x7", "        e, m = (code >> 3) & 0xF, (code & 0x7) >> 1 << 1"),
    "nan-is-a-number": ("        if e == 0xF and m == 0x7:", "        if e == 0xF and m == 0x8:"),
    "ties-away-from-zero": ("                code = lo if lo % 2 == 0 else hi      # consecutive", "                code = hi      # consecutive"),
    "round-down": ("            if d_lo < d_hi:", "            if d_lo <= d_hi + 1e300:"),
    "no-saturation": ("    flat = np.clip(y.reshape(-1), -MAX, MAX)", "    flat = np.clip(y.reshape(-1), -480.0, 480.0) * (np.abs(y.reshape(-1)) <= 464.0)"),
    "sign-lost": ("        out[i] = code | (0x80 if (v < 0 or (v == 0 and np.signbit(v))) else 0)", "        out[i] = code"),
    "divides-in-double": ("    inv = np.float32(1.0) / np.float32(scale)\n    with np.errstate(over=\"ignore\"):                   # a product that overflows to infinity saturates below\n        return encode(np.asarray(x, dtype=np.float32) * inv)",
                          "    return encode((np.asarray(x, dtype=np.float64) * 3.0) / (np.float64(scale) * 3.0))"),
    "dequantize-forgets-scale": ("    return decode_table()[np.asarray(codes, dtype=np.uint8)] * np.float64(np.float32(scale))",
                                 "    return decode_table()[np.asarray(codes, dtype=np.uint8)]"),
}

TRANSFER_MUTANTS = {
    "export-slot-for-page": ("            block[:, :, t, :] = kv_pages[page, :, :, pos % P, :]",
                             "            block[:, :, t, :] = kv_pages[page, :, :, pos // P % P, :]"),
    "export-ignores-first": ("            pos = int(first[r]) + t\n            page = int(block_table[r][pos // P])\n            block[:, :, t, :] = kv",
                             "            pos = t\n            page = int(block_table[r][pos // P])\n            block[:, :, t, :] = kv"),
    "export-row-zero-table": ("            page = int(block_table[r][pos // P])\n            block[:, :, t, :] = kv",
                              "            page = int(block_table[0][pos // P])\n            block[:, :, t, :] = kv"),
    "export-token-major": (".reshape(2, Hkv, n, D)\n        for t in range(n):\n            pos = int(first[r]) + t\n            page = int(block_table[r][pos // P])\n            block[:, :, t, :] = kv_pages[page, :, :, pos % P, :]",
                           ".reshape(n, 2, Hkv, D)\n        for t in range(n):\n            pos = int(first[r]) + t\n            page = int(block_table[r][pos // P])\n            block[t] = kv_pages[page, :, :, pos % P, :]"),
    "export-swaps-k-and-v": ("            block[:, :, t, :] = kv_pages[page, :, :, pos % P, :]",
                             "            block[:, :, t, :] = kv_pages[page, ::-1, :, pos % P, :]"),
    "import-slot": ("            kv_pages[page, :, :, pos % P, :] = block[:, :, t, :]",
                    "            kv_pages[page, :, :, t % P, :] = block[:, :, t, :]"),
    "import-whole-page": ("            kv_pages[page, :, :, pos % P, :] = block[:, :, t, :]",
                          "            kv_pages[page, :, :, :, :] = block[:, :, t, None, :]"),
    "import-offset": ("        block = buf[2 * Hkv * D * int(cu[r]): 2 * Hkv * D * int(cu[r + 1])].reshape(2, Hkv, n, D)\n        for t in range(n):\n            pos = int(first[r]) + t\n            page = int(block_table[r][pos // P])\n            kv_pages",
                      "        block = buf[Hkv * D * int(cu[r]): Hkv * D * int(cu[r]) + 2 * Hkv * D * n].reshape(2, Hkv, n, D)\n        for t in range(n):\n            pos = int(first[r]) + t\n            page = int(block_table[r][pos // P])\n            kv_pages"),
}

DECODE_MUTANTS = {
    "drop-own-token": ("        keys[L], vals[L] = k_new[b], v_new[b]", "        keys[L], vals[L] = 0.0, 0.0"),
    "own-token-off-by-one": ("        for j in range(L):", "        for j in range(L - 1):"),
    "slot-index": ("            keys[j] = kv_pages[page, 0, :, j % P, :]", "            keys[j] = kv_pages[page, 0, :, j // P % P, :]"),
    "value-from-key": ("            vals[j] = kv_pages[page, 1, :, j % P, :]", "            vals[j] = kv_pages[page, 0, :, j % P, :]"),
    "gqa-mapping": ("            s = scale * (keys[:, h // g, :] @ q[b, h])", "            s = scale * (keys[:, h % Hkv, :] @ q[b, h])"),
    "drop-scale": ("            s = scale * (keys[:, h // g, :] @ q[b, h])", "            s = (keys[:, h // g, :] @ q[b, h])"),
    "exp-sign": ("            w = np.exp(s - s.max())", "            w = np.exp(s.max() - s)"),
    "drop-normalisation": ("            w /= w.sum()\n", ""),
    "table-row": ("            page = int(block_table[b][j // P])", "            page = int(block_table[0][j // P])"),
}


def module_from(src, name):
    mod = types.ModuleType(name)
    exec(compile(src, name, "exec"), mod.__dict__)
    return mod


def pin_functions(pins):
    return [f for n, f in sorted(vars(pins).items()) if n.startswith("test_") and callable(f)]


def run_pins(pins, attr, mutant, oracle):
    real = getattr(pins, attr)
    caught = []
    setattr(pins, attr, mutant)
    try:
        for f in pin_functions(pins):
            args = [oracle] if "oracle" in inspect.signature(f).parameters else []
            try:
                f(*args)
            except (AssertionError, ValueError, IndexError):
                caught.append(f.__name__)
    finally:
        setattr(pins, attr, real)
    return caught


def test_every_mutation_site_exists():
    for name, (old, _new) in TRANSFER_MUTANTS.items():
        assert TRANSFER_SRC.count(old) == 1, "mutation site for %s not found exactly once" % name
    for name, (old, _new) in DECODE_MUTANTS.items():
        assert DECODE_SRC.count(old) == 1, "mutation site for %s not found exactly once" % name
    for name, (old, _new) in FP8_MUTANTS.items():
        assert FP8_SRC.count(old) == 1, "mutation site for %s not found exactly once" % name
    for name, (old, _new) in PREFILL_FP8_MUTANTS.items():
        assert PREFILL_FP8_SRC.count(old) == 1, "mutation site for %s not found exactly once" % name


@pytest.mark.parametrize("name", sorted(TRANSFER_MUTANTS))
def test_transfer_pins_catch_mutant(name, oracle):
    old, new = TRANSFER_MUTANTS[name]
    mutant = module_from(TRANSFER_SRC.replace(old, new), "kv_transfer_mutant_" + name.replace("-", "_"))
    assert run_pins(transfer_pins, "kv_transfer", mutant, oracle), "no pin noticed the planted mistake '%s'" % name


@pytest.mark.parametrize("name", sorted(DECODE_MUTANTS))
def test_decode_pins_catch_mutant(name, oracle):
    old, new = DECODE_MUTANTS[name]
    mutant = module_from(DECODE_SRC.replace(old, new), "decode_mutant_" + name.replace("-", "_"))
    assert run_pins(decode_pins, "decode", mutant, oracle), "no pin noticed the planted mistake '%s'" % name


@pytest.mark.parametrize("name", sorted(PREFILL_FP8_MUTANTS))
def test_prefill_fp8_pins_catch_mutant(name, oracle):
    old, new = PREFILL_FP8_MUTANTS[name]
    mutant = module_from(PREFILL_FP8_SRC.replace(old, new), "prefill_fp8_mutant_" + name.replace("-", "_"))
    assert run_pins(prefill_fp8_pins, "prefill_fp8", mutant, oracle), "no pin noticed the planted mistake '%s'" % name


def run_fp8_pins(mutant):
    """The FP8 pins reach the codes through three modules: all of them see the mutant."""
    import oracle as opkg
    real = fp8_pins.fp8
    caught = []
    fp8_pins.fp8 = mutant
    opkg.fp8 = mutant
    import sys
    sys.modules["oracle.fp8"] = mutant
    try:
        for f in pin_functions(fp8_pins):
            try:
                f()
            except (AssertionError, ValueError, IndexError, FloatingPointError):
                caught.append(f.__name__)
    finally:
        fp8_pins.fp8 = real
        opkg.fp8 = real
        sys.modules["oracle.fp8"] = real
    return caught


@pytest.mark.parametrize("name", sorted(FP8_MUTANTS))
def test_fp8_pins_catch_mutant(name):
    old, new = FP8_MUTANTS[name]
    mutant = module_from(FP8_SRC.replace(old, new), "fp8_mutant_" + name.replace("-", "_"))
    assert run_fp8_pins(mutant), "no pin noticed the planted mistake '%s'" % name


def test_unmutated_oracles_pass_the_same_calls(oracle):
    assert run_fp8_pins(fp8) == []
    assert run_pins(transfer_pins, "kv_transfer", kv_transfer, oracle) == []
    assert run_pins(decode_pins, "decode", decode, oracle) == []
    assert run_pins(prefill_fp8_pins, "prefill_fp8", prefill_fp8, oracle) == []
