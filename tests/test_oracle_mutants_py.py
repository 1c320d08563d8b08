"""Planted mistakes in the numpy oracles (KV transfer, decode iteration) must be caught by their pins.

Each mutant is the oracle's source with one plausible slip; it is executed as a module of its own,
swapped in for the real one inside the pin-test module, and every pin is run against it: at least one
has to fail.  CPU only.
"""
import inspect
import types

import pytest

import test_oracle_decode as decode_pins
import test_oracle_kv_transfer as transfer_pins
from oracle import decode, kv_transfer

TRANSFER_SRC = inspect.getsource(kv_transfer)
DECODE_SRC = inspect.getsource(decode)

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


def test_unmutated_oracles_pass_the_same_calls(oracle):
    assert run_pins(transfer_pins, "kv_transfer", kv_transfer, oracle) == []
    assert run_pins(decode_pins, "decode", decode, oracle) == []
