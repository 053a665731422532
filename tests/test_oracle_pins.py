"""CPU-only: the oracle against its pins, and the pins against planted mistakes."""
import importlib.util
import os

import numpy as np
import pytest

import oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_PATH = os.path.join(ROOT, "oracle", "rotq_oracle.py")


def load_oracle(patch=None):
    """A fresh copy of the oracle module, optionally with source text replaced (to plant a bug)."""
    with open(ORACLE_PATH) as f:
        src = f.read()
    if patch is not None:
        old, new = patch
        assert src.count(old) >= 1, f"mutation anchor not found: {old!r}"
        src = src.replace(old, new)
    spec = importlib.util.spec_from_loader("rotq_oracle_copy", loader=None)
    mod = importlib.util.module_from_spec(spec)
    exec(compile(src, ORACLE_PATH, "exec"), mod.__dict__)
    return mod


@pytest.fixture(scope="module")
def oracle():
    return load_oracle()


@pytest.mark.parametrize("check", pins.ALL_CHECKS, ids=lambda c: c.__name__)
def test_pin(oracle, check):
    check(oracle)


# Each entry: a plausible mistake planted in the oracle's source; some pin must fail.
MUTATIONS = {
    "sylvester_sign": ("np.block([[h, h], [h, -h]])", "np.block([[h, h], [-h, h]])"),
    "legendre_flipped": ("return 1 if a in _nonzero_squares(p) else -1", "return -1 if a in _nonzero_squares(p) else 1"),
    "paley1_diag_plus": ("jacobsthal(p) - np.eye(p, dtype=np.int64)", "jacobsthal(p) + np.eye(p, dtype=np.int64)"),
    "paley1_transposed": ("return chi[(idx[:, None] - idx[None, :]) % q]", "return chi[(idx[None, :] - idx[:, None]) % q]"),
    "paley1_border": ("    h[0, 0] = 1\n    h[1:, 1:] = jacobsthal(p)", "    h[0, :] = 1\n    h[1:, 1:] = jacobsthal(p)"),
    "paley1_no_guard": ("if prime_power(p) is None or p % 4 != 3:", "if prime_power(p) is None:"),
    "paley2_b_sign": ("b = np.array([[1, -1], [-1, -1]]", "b = np.array([[1, -1], [-1, 1]]"),
    "paley2_border": ("    c[0, 0] = 0\n    c[1:, 1:] = jacobsthal(q)", "    c[1:, 0] = -1\n    c[0, 0] = 0\n    c[1:, 1:] = jacobsthal(q)"),
    "paley2_kron_order": ("return np.kron(c, a) + np.kron(np.eye(m, dtype=np.int64), b)",
                          "return np.kron(a, c) + np.kron(b, np.eye(m, dtype=np.int64))"),
    "paley_kind_priority": ("if p >= 4 and is_prime(p - 1) and (p - 1) % 4 == 3:\n        return 1, p - 1",
                            "if False:\n        return 1, p - 1"),
    "factor_smallest_pow2": ("    while n % (1 << (k + 1)) == 0:\n        k += 1\n", "    k = 5\n"),
    "kron_swapped": ("return np.kron(hp, hs)", "return np.kron(hs, hp)"),
    "rotate_transposed_block": ('np.einsum("ab,rbc->rac"', 'np.einsum("ba,rbc->rac"'),
    "rotate_axes_swapped": ("xm = xp.reshape(rows, p, m)", "xm = xp.reshape(rows, m, p).transpose(0, 2, 1)"),
    "rotate_no_norm": ("return y.reshape(rows, n) / math.sqrt(n)", "return y.reshape(rows, n) / n"),
    "bf16_shift": ("<< np.uint32(16)", "<< np.uint32(15)"),
    "levels_pow2": ("return (1 << b) - 1, -(1 << (b - 1)), (1 << (b - 1)) - 1",
                    "return (1 << b), -(1 << (b - 1)), (1 << (b - 1)) - 1"),
    "range_symmetric": ("return (1 << b) - 1, -(1 << (b - 1)), (1 << (b - 1)) - 1",
                        "return (1 << b) - 1, -(1 << (b - 1)) + 1, (1 << (b - 1)) - 1"),
    "clip_dropped": ("delta = clip64 * amax / lvl", "delta = amax / lvl"),
    "clip_not_f32": ("clip64 = float(np.float32(clip))", "clip64 = float(clip)"),
    "round_floor": ("codes = np.clip(np.rint(t), qmin, qmax)", "codes = np.clip(np.floor(t + 0.5), qmin, qmax)"),
    "amax_signed": ("amax = np.max(np.abs(y), axis=1)", "amax = np.max(y, axis=1)"),
    "mse_sum": ("out[k] = np.mean((dequantize(codes, delta) - y) ** 2)",
                "out[k] = np.sum((dequantize(codes, delta) - y) ** 2)"),
    "mse_abs": ("out[k] = np.mean((dequantize(codes, delta) - y) ** 2)",
                "out[k] = np.mean(np.abs(dequantize(codes, delta) - y))"),
    "pack_big_endian": ('np.packbits(bits, axis=1, bitorder="little")', 'np.packbits(bits, axis=1, bitorder="big")'),
    "pack_field_msb_first": ("(field[:, :, None] >> np.arange(b)) & 1", "(field[:, :, None] >> np.arange(b)[::-1]) & 1"),
    "unpack_no_sign": ("field = np.where(field >= (1 << (b - 1)), field - (1 << b), field)", "field = field"),
    "boundary_tol": ("return (frac < tol)", "return (frac < 10 * tol)"),
    "large_block_smallest_k": ("    # (section 5.2.2: 1536 + 8 = 1544 = 1543 + 1 \"managed by the Paley algorithm\"), again with\n    # the largest 2^k\n    k = 0\n    while n % (1 << (k + 1)) == 0:\n        k += 1\n    while k >= 0:", "    kmax = 0\n    while n % (1 << (kmax + 1)) == 0:\n        kmax += 1\n    for k in range(0, kmax + 1):"),
    "gf_modulus_order": ("low = [(idx // p ** (k - 1 - j)) % p for j in range(k)]", "low = [(idx // p ** j) % p for j in range(k)]"),
    "gf_reduce_sign": ("a[i - k + j] = (a[i - k + j] - c * f[j]) % p", "a[i - k + j] = (a[i - k + j] + c * f[j]) % p"),
    "gf_difference": ("d = tuple(((i // p ** t) % p - (j // p ** t) % p) % p for t in range(k))", "d = tuple(((i - j) // p ** t) % p for t in range(k))"),
    "gf_character_flipped": ("return 1 if d in _field_squares(q) else -1", "return -1 if d in _field_squares(q) else 1"),
    "back_not_transposed": ('x = np.einsum("ba,rbc->rac", hp.astype(np.float64), x)', 'x = np.einsum("ab,rbc->rac", hp.astype(np.float64), x)'),
    "back_unnormalised": ("    x = x.reshape(rows, n) / math.sqrt(n)\n", "    x = x.reshape(rows, n) / n\n"),
    "fuse_wrong_side": ("    return rotate(w.T, n).T\n", "    return rotate_back(np.pad(w.T, ((0, 0), (0, n - w.shape[0]))), n).T\n"),
    "limit_rounds_up": ("    return (n * (b - b_prime)) // b_prime", "    return -((-n * (b - b_prime)) // b_prime)"),
    "limit_wrong_divisor": ("    return (n * (b - b_prime)) // b_prime", "    return (n * (b - b_prime)) // b"),
    "qe_asym_symmetric_codes": ("        codes, delta, lo, _ = quantize_asym(y, b, c, group)\n        out[k] = np.mean((dequantize_asym(codes, delta, lo, group) - y) ** 2)", "        codes, delta, _ = quantize(y, b, c)\n        out[k] = np.mean((dequantize(codes, delta) - y) ** 2)"),
    "asym_clip_one_side": ("    hi = clip64 * yg.max(axis=2)", "    hi = yg.max(axis=2)"),
    "asym_levels": ("    delta = (hi - lo) / lvl\n", "    delta = (hi - lo) / (lvl + 1)\n"),
    "asym_offset_dropped": ("return (cg * delta[:, :, None] + lo[:, :, None]).reshape(rows, n)", "return (cg * delta[:, :, None]).reshape(rows, n)"),
    "asym_signed_range": ("codes = np.clip(np.rint(t), 0, lvl).astype(np.uint8)", "codes = np.clip(np.rint(t), 0, lvl - 1).astype(np.uint8)"),
    "asym_group_axis": ("yg = y.reshape(rows, n // group, group)\n    lo = clip64", "yg = y.reshape(rows, group, n // group).transpose(0, 2, 1)\n    lo = clip64"),
    "gbs_probe_parity": ("    side = 0 ", "    side = 1 "),
    "gbs_keep_worse": ("        if fx < f_best:", "        if fx > f_best:"),
    "gbs_bracket_swap": ("            near[side] = x", "            near[1 - side] = x"),
    "gbs_stop": ("while near[1] - near[0] > eps and", "while near[1] - near[0] > 4 * eps and"),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name):
    broken = load_oracle(MUTATIONS[name])
    failed = []
    # cheap pins first; one failing pin is enough
    for check in sorted(pins.ALL_CHECKS, key=lambda c: c.__name__ == "check_large_paley_blocks"):
        try:
            check(broken)
        except Exception:
            failed.append(check.__name__)
            break
    assert failed, f"no pin notices the planted mistake {name!r}"


def test_clip_is_taken_as_float32(oracle):
    # the library receives clip as a C float; 0.9 is not representable, so the widened value differs
    y = np.array([[1.0, -0.3, 0.7, 0.2]])
    _, d32, _ = oracle.quantize(y, 4, 0.9)
    assert d32[0] == float(np.float32(0.9)) / 15
    assert d32[0] != 0.9 / 15
