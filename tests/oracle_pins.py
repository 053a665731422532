"""Pins for the CPU oracle: checks against what the paper and the mathematics fix.

Every check takes the oracle module as its argument, so the same checks can be run on a
deliberately broken copy (tests/test_oracle_pins.py plants mistakes and expects a pin to
fail).  Nothing here calls the HIP path.
"""
from __future__ import annotations

import math
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ----------------------------------------------------------------------------- fixtures

def _read_matrices(name):
    mats, cur, key = {}, None, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line[0].isalpha():
                key = line
                mats[key] = []
            else:
                mats[key].append([int(v) for v in line.split()])
    return {k: np.array(v, dtype=np.int64) for k, v in mats.items()}


def _read_residues():
    out = {}
    with open(os.path.join(GOLDEN, "quadratic_residues.txt")) as f:
        for line in f:
            if line.startswith("#") or ":" not in line:
                continue
            p, r = line.split(":")
            out[int(p)] = {int(v) for v in r.split()}
    return out


def _read_pack_examples():
    out = []
    with open(os.path.join(GOLDEN, "pack_examples.txt")) as f:
        for line in f:
            if line.startswith("#") or "|" not in line:
                continue
            b, codes, by = line.split("|")
            out.append((int(b), [int(v) for v in codes.split()], [int(v, 16) for v in by.split()]))
    return out


def fwht_reference(v):
    """Textbook in-place fast Walsh-Hadamard transform (natural order), test helper only."""
    v = np.array(v, dtype=np.float64)
    n = v.shape[-1]
    h = 1
    while h < n:
        for i in range(0, n, 2 * h):
            a = v[..., i:i + h].copy()
            b = v[..., i + h:i + 2 * h].copy()
            v[..., i:i + h] = a + b
            v[..., i + h:i + 2 * h] = a - b
        h *= 2
    return v


# ----------------------------------------------------------------------------- P1 Sylvester

def check_sylvester_literal(o):
    g = _read_matrices("eq1_sylvester.txt")
    assert np.array_equal(o.sylvester(1), g["H2"])
    assert np.array_equal(o.sylvester(2), g["H4"])


def check_sylvester_popcount(o):
    for k in range(0, 8):
        h = o.sylvester(k)
        n = 1 << k
        i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
        pc = np.array([[bin(a & b).count("1") for b in range(n)] for a in range(n)])
        assert np.array_equal(h, 1 - 2 * (pc % 2))
        assert np.array_equal(h @ h.T, n * np.eye(n, dtype=np.int64))


# ----------------------------------------------------------------------------- P2 Legendre

def check_legendre_tables(o):
    for p, res in _read_residues().items():
        for a in range(-p, 2 * p):
            want = 0 if a % p == 0 else (1 if (a % p) in res else -1)
            assert o.legendre_symbol(a, p) == want, (a, p)


def check_legendre_euler(o):
    for p in (3, 7, 11, 13, 29, 73, 103):
        tot = 0
        for a in range(p):
            e = pow(a, (p - 1) // 2, p)
            e = -1 if e == p - 1 else e
            assert o.legendre_symbol(a, p) == e
            tot += e
        assert tot == 0
        for a in range(1, p):
            for b in (2, 3, p - 1):
                assert o.legendre_symbol(a * b, p) == o.legendre_symbol(a, p) * o.legendre_symbol(b, p)


# ----------------------------------------------------------------------------- P3 Paley

def check_paley1_literal(o):
    g = _read_matrices("alg2_paley_p3.txt")
    assert np.array_equal(o.paley1(3), g["H4"])


def check_paley1_structure(o):
    # Algorithm 2's fixed entries, and its orientation: entry [i,j] is the symbol of i-j, so for
    # p = 11 (residues 1,3,4,5,9) H[2,1] = (1/11) = +1 and H[1,2] = (-1/11) = (10/11) = -1.
    h = o.paley1(11)
    assert h[0, 0] == 1 and np.all(h[0, 1:] == -1) and np.all(h[1:, 0] == -1)
    assert np.all(np.diag(h)[1:] == -1)
    assert h[2, 1] == 1 and h[1, 2] == -1
    assert h[4, 1] == 1 and h[1, 4] == -1     # 3 is a residue, -3 = 8 is not


def check_paley2_structure(o):
    # layout of the stated Paley II definition: 2x2 blocks indexed [2i+u, 2j+v]; diagonal blocks
    # are B = [[1,-1],[-1,-1]] (C has a zero diagonal), block (0, j>0) is +A = [[1,1],[1,-1]],
    # block (i, j) off the border is legendre(i-j, q) * A.  q = 5: residues 1, 4.
    h = o.paley2(5)
    for i in range(6):
        assert h[2 * i:2 * i + 2, 2 * i:2 * i + 2].tolist() == [[1, -1], [-1, -1]]
    for j in range(1, 6):
        assert h[0:2, 2 * j:2 * j + 2].tolist() == [[1, 1], [1, -1]]
        assert h[2 * j:2 * j + 2, 0:2].tolist() == [[1, 1], [1, -1]]
    assert h[2:4, 4:6].tolist() == [[1, 1], [1, -1]]          # i=1, j=2: (-1/5) = (4/5) = +1
    assert h[2:4, 6:8].tolist() == [[-1, -1], [-1, 1]]        # i=1, j=3: (-2/5) = (3/5) = -1


def check_paley_orthogonal(o):
    for q in (3, 7, 11, 19, 23, 43, 103):
        h = o.paley1(q)
        n = q + 1
        assert h.shape == (n, n) and set(np.unique(h)) == {-1, 1}
        assert np.array_equal(h @ h.T, n * np.eye(n, dtype=np.int64))
    for q in (5, 13, 17, 29, 73):
        h = o.paley2(q)
        n = 2 * (q + 1)
        assert h.shape == (n, n) and set(np.unique(h)) == {-1, 1}
        assert np.array_equal(h @ h.T, n * np.eye(n, dtype=np.int64))
        assert np.array_equal(h, h.T)          # Paley II matrices are symmetric


def check_paley_guards(o):
    for bad in (5, 13, 9, 15):                  # = 1 (mod 4), or not a prime power
        try:
            o.paley1(bad)
        except ValueError:
            pass
        else:
            raise AssertionError(f"paley1({bad}) must be refused")
    for bad in (3, 7, 27, 15, 21):            # = 3 (mod 4), or not a prime power
        try:
            o.paley2(bad)
        except ValueError:
            pass
        else:
            raise AssertionError(f"paley2({bad}) must be refused")


def check_order_rules(o):
    # the orders the benchmark configurations use
    assert o.factor_order(4096) == (1, 0, 0, 12)
    assert o.factor_order(256) == (1, 0, 0, 8)
    assert o.factor_order(128) == (1, 0, 0, 7)
    assert o.factor_order(3584) == (28, 2, 13, 7)
    assert o.factor_order(18944) == (148, 2, 73, 7)
    assert o.factor_order(3072) == (12, 1, 11, 8)
    assert o.factor_order(1536) == (12, 1, 11, 7)
    # 3000 and 3008 have no block of at most 256 (only large ones: 1500 = 1499 + 1, 752 = 751 + 1),
    # so the expansion helper, which keeps to small blocks, moves on to 3072
    assert o.factor_order(3000) == (1500, 1, 1499, 1) and o.factor_order(3008) == (752, 1, 751, 2)
    assert o.factor_order(3002) is None
    assert o.next_order(3000) == 3072
    assert o.next_order(4096) == 4096
    # q+1 for q = 3 (mod 4), 2(q+1) for q = 1 (mod 4); Paley I wins where both exist (12)
    assert o.paley_kind(12) == (1, 11) and o.paley_kind(28) == (2, 13)
    assert o.paley_kind(148) == (2, 73) and o.paley_kind(20) == (1, 19)
    assert o.paley_kind(16) is None and o.paley_kind(40) is None and o.paley_kind(56) is None


def check_composite_orthogonal(o):
    for n in (12, 24, 48, 56, 96, 296, 384):
        h = o.hadamard_dense(n)
        assert h.shape == (n, n)
        assert np.array_equal(h @ h.T, n * np.eye(n, dtype=np.int64))
    # Kronecker index convention: flat index = a * 2^k + c
    hp, hs = o.hadamard_factors(48)
    h = o.hadamard_dense(48)
    m = hs.shape[0]
    for (i, j) in ((0, 0), (5, 17), (47, 3), (13, 46), (31, 31)):
        assert h[i, j] == hp[i // m, j // m] * hs[i % m, j % m]


# ----------------------------------------------------------------------------- P4 rotation

def check_rotate_bruteforce(o):
    # y_i = sum_j H[i,j] x_j / sqrt(n), by explicit loops over the dense matrix (catches a
    # transposed operand: Paley I matrices are not symmetric)
    rng = np.random.default_rng(1)
    for n, d in ((12, 12), (24, 20), (48, 48), (56, 50), (32, 32)):
        h = o.hadamard_dense(n)
        x = rng.standard_normal((3, d))
        y = o.rotate(x, n)
        for r in range(3):
            for i in range(n):
                s = 0.0
                for j in range(d):
                    s += h[i, j] * x[r, j]
                assert abs(y[r, i] - s / math.sqrt(n)) < 1e-12


def check_rotate_fwht(o):
    rng = np.random.default_rng(2)
    for k in (1, 3, 6, 10):
        n = 1 << k
        x = rng.standard_normal((4, n))
        assert np.allclose(o.rotate(x, n), fwht_reference(x) / math.sqrt(n), rtol=0, atol=1e-11)


def check_rotate_norm_and_involution(o):
    rng = np.random.default_rng(3)
    for n in (64, 96, 224, 1184, 3072):
        x = rng.standard_normal((2, n)) * 3
        y = o.rotate(x, n)
        assert np.allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)
    for n in (64, 224, 1184):                     # symmetric H (Sylvester, Paley II): H(Hx)/n = x
        x = rng.standard_normal((2, n))
        assert np.allclose(o.rotate(o.rotate(x, n), n), x, atol=1e-12)


def check_rotate_onehot(o):
    # Lemma "Hadamard incoherence" / Theorem "Hadamard optimality": |y_i| = c / sqrt(n) for all i
    for n in (16, 48, 224, 4096):
        for j in (0, n // 3, n - 1):
            x = np.zeros((1, n))
            x[0, j] = 7.5
            y = o.rotate(x, n)
            assert np.allclose(np.abs(y), 7.5 / math.sqrt(n), rtol=1e-14)


def check_rotate_zero_pad(o):
    # Eq. 2: order 4, rows [x0, x1] padded with two zeros -> (x0+x1, x0-x1, x0+x1, x0-x1)/2
    g = _read_matrices("eq2_expand.txt")["M"]
    assert np.array_equal(o.hadamard_dense(4), g)
    x = np.array([[3.0, 5.0], [-2.0, 0.25]])
    y = o.rotate(x, 4)
    for r in range(2):
        a, c = x[r]
        assert np.allclose(y[r], np.array([a + c, a - c, a + c, a - c]) / 2.0)
    # padding explicitly with zeros gives the same result, at a Paley order too
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 40))
    xp = np.concatenate([x, np.zeros((2, 8))], axis=1)
    assert np.array_equal(o.rotate(x, 48), o.rotate(xp, 48))


def check_rotate_peak_experiment(o):
    # Appendix A.1.2: N(0, 0.1^2) vector plus a peak of 200 -> max|Hx| tracks 200/sqrt(n)
    rng = np.random.default_rng(5)
    for n in (64, 256, 1024, 4096):
        x = rng.normal(0.0, 0.1, size=(1, n))
        x[0, 17] += 200.0
        m = np.max(np.abs(o.rotate(x, n)))
        assert abs(m - 200.0 / math.sqrt(n)) < 0.5


def check_bf16_widening(o):
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000, 0x7F7F, 0x0001], dtype=np.uint16)
    want = [1.0, -1.0, 3.140625, 0.0, -0.0, 3.3895313892515355e38, 2.0 ** -133]
    assert np.array_equal(o.bf16_bits_to_f64(bits), np.array(want))


# ----------------------------------------------------------------------------- P5 quantizer

def check_quant_params(o):
    assert o.quant_params(3) == (7, -4, 3)
    assert o.quant_params(4) == (15, -8, 7)


def check_quantize_properties(o):
    rng = np.random.default_rng(6)
    y = rng.standard_t(3.0, size=(16, 96))
    for b in (3, 4):
        lvl, qmin, qmax = o.quant_params(b)
        for clip in (1.0, 0.9, 0.5):
            q, delta, t = o.quantize(y, b, clip)
            c64 = float(np.float32(clip))
            assert q.min() >= qmin and q.max() <= qmax
            assert np.allclose(delta, c64 * np.abs(y).max(axis=1) / lvl, rtol=1e-15)
            yh = o.dequantize(q, delta)
            inside = (t >= qmin - 0.5) & (t <= qmax + 0.5)
            assert np.all(np.abs(yh - y)[inside] <= delta[:, None].repeat(96, 1)[inside] * 0.5 * (1 + 1e-12))
            # clamped elements sit on the range ends
            assert np.all(q[t > qmax + 0.5] == qmax) and np.all(q[t < qmin - 0.5] == qmin)
            # idempotence with the scale held fixed
            q2 = np.clip(np.rint(yh / delta[:, None]), qmin, qmax).astype(np.int8)
            assert np.array_equal(q2, q)
            # scale equivariance (power of two: bit exact)
            q3, d3, _ = o.quantize(4.0 * y, b, clip)
            assert np.array_equal(q3, q) and np.array_equal(d3, 4.0 * delta)


def check_quantize_ties_and_zero(o):
    # ties go to even; zero row -> zero scale and codes
    y = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5], [0.0] * 8])
    q, delta, _ = o.quantize(y, 3, 1.0)            # delta = 1 for the first row
    assert delta[0] == 1.0 and delta[1] == 0.0
    assert q[0].tolist() == [3, 0, 2, 2, 0, -2, -2, 3]
    assert q[1].tolist() == [0] * 8


def check_quantize_onehot(o):
    # one-hot through Sylvester: all |y| equal, t = +-L/clip, codes = qmax / qmin by sign,
    # delta = clip * c / (sqrt(n) L)
    n, c = 256, 12.0
    x = np.zeros((1, n))
    x[0, 5] = c
    for b in (3, 4):
        lvl, qmin, qmax = o.quant_params(b)
        q, delta, t, y = o.rotate_quantize(x, n, b, 0.9)
        c64 = float(np.float32(0.9))
        assert np.allclose(delta, c64 * c / (math.sqrt(n) * lvl), rtol=1e-14)
        assert np.all(q[y > 0] == qmax) and np.all(q[y < 0] == qmin)
        assert np.allclose(np.abs(t), lvl / c64, rtol=1e-14)


# ----------------------------------------------------------------------------- P6 quant_error

def check_quant_error_bruteforce(o):
    rng = np.random.default_rng(7)
    n, d, b = 24, 22, 3
    x = rng.standard_normal((3, d))
    clips = np.array([0.5, 0.75, 1.0], dtype=np.float32)
    got = o.quant_error(x, n, b, clips)
    h = o.hadamard_dense(n)
    lvl, qmin, qmax = (1 << b) - 1, -(1 << (b - 1)), (1 << (b - 1)) - 1
    for k, c in enumerate(clips):
        tot = 0.0
        for r in range(3):
            y = [sum(h[i, j] * x[r, j] for j in range(d)) / math.sqrt(n) for i in range(n)]
            amax = max(abs(v) for v in y)
            dl = float(c) * amax / lvl
            for v in y:
                code = min(max(round(v / dl), qmin), qmax)      # Python round = half to even
                tot += (code * dl - v) ** 2
        assert abs(got[k] - tot / (3 * n)) < 1e-13


def check_quant_error_closed_form(o):
    # one-hot: every |y| = c/sqrt(n) =: a; positive entries saturate at qmax, negative at qmin:
    # err+ = a (1 - qmax clip / L), err- = a (1 - |qmin| clip / L) (negative side may not clamp)
    n, c, b = 64, 3.0, 3
    x = np.zeros((2, n))
    x[:, 9] = c
    clips = np.array([0.5, 0.9, 0.9, 1.0], dtype=np.float32)
    mse = o.quant_error(x, n, b, clips)
    assert mse[1] == mse[2]
    a = c / math.sqrt(n)
    y = o.rotate(x, n)
    npos = np.sum(y > 0) / y.size
    for k, cl in enumerate(clips):
        cl = float(cl)
        tpos = 7.0 / cl                      # > 3.5 always -> code 3
        tneg = -7.0 / cl                     # code max(-4, rint(tneg))
        qneg = max(-4, round(tneg))
        want = npos * (a - 3 * cl * a / 7) ** 2 + (1 - npos) * (-a - qneg * cl * a / 7) ** 2
        assert tpos > 3.5
        assert abs(mse[k] - want) < 1e-14


def check_quant_error_rotation_invariance(o):
    # orthonormal rotation: error measured after rotating back equals error in the rotated domain
    rng = np.random.default_rng(8)
    n = 64
    x = rng.standard_normal((4, n))
    y = o.rotate(x, n)
    q, delta, _ = o.quantize(y, 4, 0.8)
    back = o.rotate(o.dequantize(q, delta), n)          # Sylvester is symmetric: inverse = itself
    e1 = np.mean((back - x) ** 2)
    assert abs(e1 - o.quant_error(x, n, 4, np.array([0.8], dtype=np.float32))[0]) < 1e-13


# ----------------------------------------------------------------------------- P7 packing

def check_pack_examples(o):
    for b, codes, by in _read_pack_examples():
        got = o.pack_codes(np.array([codes], dtype=np.int8), b)
        assert got.tolist() == [by], (b, got.tolist(), by)
        assert o.unpack_codes(np.array([by], dtype=np.uint8), b, len(codes)).tolist() == [codes]


def check_pack_roundtrip(o):
    rng = np.random.default_rng(9)
    for b in (3, 4):
        _, qmin, qmax = o.quant_params(b)
        q = rng.integers(qmin, qmax + 1, size=(5, 96)).astype(np.int8)
        pk = o.pack_codes(q, b)
        assert pk.shape == (5, 96 * b // 8) and pk.dtype == np.uint8
        assert np.array_equal(o.unpack_codes(pk, b, 96), q)
        # bit-level definition, element by element
        for r in (0, 4):
            for j in (0, 1, 37, 95):
                f = 0
                for i in range(b):
                    s = j * b + i
                    f |= ((int(pk[r, s // 8]) >> (s % 8)) & 1) << i
                assert f == (int(q[r, j]) & ((1 << b) - 1))


def check_boundary_mask(o):
    t = np.array([[0.5, 0.5 + 5e-7, 0.5 + 2e-6, 2.5 - 9e-7, 3.5, -3.5, -4.5, 7.5, 1.0]])
    m3 = o.boundary_exempt(t, 3)
    assert m3.tolist() == [[True, True, False, True, False, True, False, False, False]]
    m4 = o.boundary_exempt(t, 4)
    assert m4.tolist() == [[True, True, False, True, True, True, True, False, False]]


# ----------------------------------------------------------------------------- prime powers

def check_prime_power_fields(o):
    assert o.prime_power(27) == (3, 3) and o.prime_power(49) == (7, 2) and o.prime_power(13) == (13, 1)
    assert o.prime_power(12) is None and o.prime_power(1) is None and o.prime_power(45) is None
    # moduli worked by hand (smallest monic irreducible polynomial, coefficients low first):
    # GF(9): x^2 + 1 (x^2 + 0 has a root); GF(27): x^3 + 2x + 1 (x^3+1, x^3+2, x^3+x+1, x^3+x+2 have roots 2, 1,
    # 1, 2); GF(25): x^2 + 2 (x^2 + 1 has the root 2); GF(49): x^2 + 1 (-1 is no square mod 7)
    assert o.field_modulus(3, 2) == (1, 0, 1) and o.field_modulus(3, 3) == (1, 2, 0, 1)
    assert o.field_modulus(5, 2) == (2, 0, 1) and o.field_modulus(7, 2) == (1, 0, 1)
    for q in (9, 25, 27, 49):
        p, k = o.prime_power(q)
        f = o.field_modulus(p, k)
        els = o.field_elements(q)
        assert len(set(els)) == q and els[0] == (0,) * k and els[1] == (1,) + (0,) * (k - 1)
        # a field: every non-zero element has an inverse; exactly (q - 1) / 2 non-zero squares
        one = els[1]
        for a in els[1:]:
            assert any(o.field_mul(a, b, p, f) == one for b in els[1:])
        sq = {o.field_mul(a, a, p, f) for a in els[1:]}
        assert len(sq) == (q - 1) // 2
        # the character: antisymmetric for q = 3 (mod 4), symmetric for q = 1 (mod 4), rows sum to 0
        for i in (0, 1, q // 2, q - 1):
            row = [o.quadratic_character(i, j, q) for j in range(q)]
            assert row[i] == 0 and sum(row) == 0
            for j in (0, 2, q - 2):
                if i != j:
                    assert o.quadratic_character(j, i, q) == (row[j] if q % 4 == 1 else -row[j])
    # GF(9) = GF(3)[x] / (x^2 + 1) by hand: the non-zero squares are 1, 2 = x^2, x = (x + 2)^2 and
    # 2x = (x + 1)^2, i.e. the elements number 1, 2, 3, 6
    assert [o.quadratic_character(i, 0, 9) for i in range(9)] == [0, 1, 1, 1, -1, -1, 1, -1, -1]
    # for a prime the character is the Legendre symbol
    for i in range(11):
        for j in range(11):
            assert o.quadratic_character(i, j, 11) == o.legendre_symbol(i - j, 11)
    # the matrices, and the orders they add: 52, 100, 244 (20, 28, 164, 252 stay with their primes)
    for fn, q, n in ((o.paley2, 9, 20), (o.paley2, 25, 52), (o.paley1, 27, 28), (o.paley2, 49, 100),
                     (o.paley1, 243, 244)):
        h = fn(q)
        assert h.shape == (n, n) and set(np.unique(h)) == {-1, 1}
        assert np.array_equal(h @ h.T, n * np.eye(n, dtype=np.int64))
    assert o.paley_kind(52) == (2, 25) and o.paley_kind(100) == (2, 49) and o.paley_kind(244) == (1, 243)
    assert o.paley_kind(20) == (1, 19) and o.paley_kind(28) == (2, 13) and o.paley_kind(164) == (1, 163)
    assert o.factor_order(52 * 128) == (52, 2, 25, 7) and o.factor_order(100 * 32) == (100, 2, 49, 5)
    assert o.paley_kind(116) is None and o.paley_kind(92) is None     # 115, 57 / 91, 45: nothing applies


# ----------------------------------------------------------------------------- large blocks

def check_large_paley_blocks(o):
    # section 5.2.2: 1536 + 8 = 1544 = 1543 + 1, the whole dimension as one Paley block
    assert o.is_prime(1543) and 1543 % 4 == 3
    assert o.factor_order(1544) == (1544, 1, 1543, 0)
    assert o.factor_order(3088) == (1544, 1, 1543, 1)          # largest 2^k first
    assert o.factor_order(1540) == (1540, 2, 769, 0)           # 2 (769 + 1), 769 = 1 (mod 4)
    assert o.factor_order(1536) == (12, 1, 11, 7)              # a small block wins where one exists
    assert o.factor_order(1542) is None and o.factor_order(1546) is None
    h = o.hadamard_dense(1544).astype(np.float64)               # exact: integers far below 2^53
    assert np.array_equal(h @ h.T, 1544 * np.eye(1544))
    # the expansion helper keeps its cost rule (blocks of at most 256)
    assert o.next_order(1537) == 1664 and o.next_order(1544) == 1664      # 52 * 32, 52 = 2 (25 + 1)
    # rotation through the large block against explicit loops on a few outputs
    rng = np.random.default_rng(41)
    x = rng.standard_normal((2, 1544))
    y = o.rotate(x, 1544)
    for r, i in ((0, 0), (0, 1), (1, 777), (1, 1543)):
        assert abs(y[r, i] - sum(int(h[i, j]) * x[r, j] for j in range(1544)) / np.sqrt(1544)) < 1e-10
    assert np.allclose(o.rotate_back(y, 1544), x, atol=1e-11)


# ----------------------------------------------------------------------------- inverse, fusion, limit

def check_rotate_back_inverts(o):
    rng = np.random.default_rng(21)
    for n, d in ((64, 64), (96, 96), (96, 70), (224, 200), (3584, 3584)):       # 96 = 12*8, 224 = 28*8
        x = rng.standard_normal((3, d))
        y = o.rotate(x, n)
        xb = o.rotate_back(y, n, d)
        assert np.allclose(xb, x, atol=1e-12), n
        full = o.rotate_back(y, n)
        assert np.allclose(full[:, d:], 0.0, atol=1e-12)
        # against the dense definition: x = H^T y / sqrt(n)
        if n <= 224:
            h = o.hadamard_dense(n).astype(np.float64)
            assert np.allclose(full, (h.T @ y.T).T / np.sqrt(n), atol=1e-12)
    # a Paley I block is not symmetric: using H instead of H^T must not invert
    h12 = o.hadamard_dense(96).astype(np.float64)
    assert not np.array_equal(h12, h12.T)
    e = np.zeros((1, 96)); e[0, 5] = 1.0
    assert np.allclose(o.rotate_back(e, 96), h12[5:6, :] / np.sqrt(96))        # row 5 of H = column 5 of H^T


def check_fuse_weight(o):
    # Eq. 2: order 4, W = [[a, b], [c, d]] padded with two zero rows
    g = _read_matrices("eq2_expand.txt")["M"]
    a, b, c, d = 3.0, -1.0, 0.5, 2.0
    w = np.array([[a, b], [c, d]])
    want = g @ np.array([[a, b], [c, d], [0, 0], [0, 0]]) / 2.0
    assert np.allclose(o.fuse_weight(w, 4), want)
    # the product is preserved: rotate(x) @ W' = x @ W, also with padding and a Paley block
    rng = np.random.default_rng(22)
    for n, din in ((64, 64), (96, 80), (224, 224)):
        w = rng.standard_normal((din, 7))
        x = rng.standard_normal((5, din))
        assert np.allclose(o.rotate(x, n) @ o.fuse_weight(w, n), x @ w, atol=1e-11)
        assert o.fuse_weight(w, n).shape == (n, 7)


def check_expand_limit(o):
    # section 4.2's example: n = 4096, 4 -> 3 bits; n (b - b') / b' = 1365.33 (printed rounded up, 1366)
    assert o.expand_limit(4096, 4, 3) == 1365
    for n, b, bp in ((4096, 4, 3), (1536, 8, 4), (100, 4, 4), (7, 5, 2)):
        d = o.expand_limit(n, b, bp)
        assert (n + d) * bp <= n * b < (n + d + 1) * bp
        # the lemma's own inequality on the squared cost (m, p cancel)
        assert (n + d) ** 2 * bp ** 2 <= n ** 2 * b ** 2 < (n + d + 1) ** 2 * bp ** 2
    assert o.expand_limit(100, 4, 4) == 0 and o.expand_limit(1536, 8, 4) == 1536


# ----------------------------------------------------------------------------- asymmetric groups

def check_asym_properties(o):
    rng = np.random.default_rng(11)
    y = rng.standard_t(3.0, size=(6, 256)) + 0.7
    for b in (3, 4):
        lvl = (1 << b) - 1
        for clip in (1.0, 0.9):
            q, delta, lo, t = o.quantize_asym(y, b, clip)
            c64 = float(np.float32(clip))
            assert q.dtype == np.uint8 and q.min() >= 0 and q.max() <= lvl
            yg = y.reshape(6, 2, 128)
            assert np.allclose(lo, c64 * yg.min(axis=2), rtol=1e-15)
            assert np.allclose(delta, c64 * (yg.max(axis=2) - yg.min(axis=2)) / lvl, rtol=1e-14)
            yh = o.dequantize_asym(q, delta, lo)
            dfull = np.repeat(delta, 128, axis=1)
            inside = (t >= -0.5) & (t <= lvl + 0.5)
            assert np.all(np.abs(yh - y)[inside] <= 0.5 * dfull[inside] * (1 + 1e-12))
            assert np.all(q[t > lvl + 0.5] == lvl) and np.all(q[t < -0.5] == 0)
            if clip == 1.0:
                # the extremes of every group land on the end codes and are reproduced exactly
                for r in range(6):
                    for g in range(2):
                        seg = slice(128 * g, 128 * g + 128)
                        assert q[r, seg][np.argmin(y[r, seg])] == 0 and q[r, seg][np.argmax(y[r, seg])] == lvl
                        assert abs(yh[r, seg].min() - y[r, seg].min()) < 1e-12
                        assert abs(yh[r, seg].max() - y[r, seg].max()) < 1e-12
            # idempotence with the group parameters held fixed
            q2 = np.clip(np.rint((yh.reshape(6, 2, 128) - lo[:, :, None]) / delta[:, :, None]), 0, lvl)
            assert np.array_equal(q2.reshape(6, 256).astype(np.uint8), q)
            # scaling by a power of two: same codes, scaled parameters
            q3, d3, l3, _ = o.quantize_asym(8.0 * y, b, clip)
            assert np.array_equal(q3, q) and np.array_equal(d3, 8 * delta) and np.array_equal(l3, 8 * lo)


def check_asym_closed_forms(o):
    # a group that is an exact arithmetic progression over the levels is reproduced exactly
    for b in (3, 4):
        lvl = (1 << b) - 1
        base = np.arange(128) % (lvl + 1)
        y = (base * 0.25 - 1.0)[None, :]
        q, delta, lo, _ = o.quantize_asym(y, b, 1.0)
        assert np.array_equal(q[0], base.astype(np.uint8))
        assert delta[0, 0] == 0.25 and lo[0, 0] == -1.0
        assert np.array_equal(o.dequantize_asym(q, delta, lo), y)
    # a shift moves only the offset; a constant group has delta 0, codes 0, y^ = clip * value
    y = np.linspace(-1, 2, 128)[None, :]
    q, delta, lo, _ = o.quantize_asym(y, 4, 1.0)
    q2, d2, l2, _ = o.quantize_asym(y + 4.0, 4, 1.0)
    assert np.array_equal(q, q2) and np.allclose(d2, delta, rtol=1e-15) and np.allclose(l2, lo + 4.0)
    qc, dc, lc, _ = o.quantize_asym(np.full((1, 128), 3.0), 3, 0.5)
    assert not qc.any() and dc[0, 0] == 0 and lc[0, 0] == 1.5
    # unsigned fields round-trip through the packer
    rng = np.random.default_rng(12)
    qq = rng.integers(0, 8, size=(3, 128)).astype(np.uint8)
    assert np.array_equal(o.unpack_codes(o.pack_codes(qq, 3), 3, 128, signed=False), qq)
    tt = np.array([[0.5, 6.5, 7.5, -0.5, 14.5, 3.2]])
    assert o.boundary_exempt_asym(tt, 3).tolist() == [[True, True, False, False, False, False]]
    assert o.boundary_exempt_asym(tt, 4).tolist() == [[True, True, True, False, True, False]]


def check_quant_error_asym(o):
    # explicit loops on the rotated rows, formula written out per element
    rng = np.random.default_rng(13)
    x = rng.standard_normal((3, 128)) + 0.4
    y = o.rotate(x, 128)
    clips = [np.float32(0.6), np.float32(1.0)]
    got = o.quant_error_asym(x, 128, 3, clips)
    for k, c in enumerate(clips):
        c = float(c)
        tot = 0.0
        for r in range(3):
            lo, hi = c * min(y[r]), c * max(y[r])
            delta = (hi - lo) / 7
            for v in y[r]:
                q = min(max(round((v - lo) / delta), 0), 7)      # Python rounds halves to even as well
                tot += (q * delta + lo - v) ** 2
        assert abs(got[k] - tot / (3 * 128)) <= 1e-12 * max(tot, 1e-30)
    # values on the grid with clip 1 are reproduced: zero error; a constant group costs (1 - clip)^2 v^2
    grid = (np.arange(128) % 8) * 0.5 - 1.0
    h = o.hadamard_dense(128).astype(np.float64)
    xg = (h.T @ grid / np.sqrt(128))[None, :]                  # rotates onto the grid
    assert o.quant_error_asym(xg, 128, 3, [1.0])[0] < 1e-24
    xc = np.zeros((1, 128)); xc[0, 0] = 4.0                    # rotated row is constant 4 / sqrt(128)
    e = o.quant_error_asym(xc, 128, 4, [np.float32(0.75)])[0]
    assert abs(e - (0.25 * 4.0 / np.sqrt(128)) ** 2) < 1e-15


def check_quantize_plain(o):
    # no rotation: the section 2.1 quantizer on the row itself
    x = np.array([[0.0, 1.0, -2.0, 7.0, -7.0, 3.5, 0.4, -0.6]])
    q, delta, t = o.quantize_plain(x, 3, 1.0)
    assert delta[0] == 1.0 and q[0].tolist() == [0, 1, -2, 3, -4, 3, 0, -1]
    bits = np.array([[0x3F80, 0xC000, 0x40E0, 0x0000]], dtype=np.uint16)      # 1, -2, 7, 0
    q, delta, _ = o.quantize_plain(bits, 4, 1.0)
    assert delta[0] == 7.0 / 15 and q[0].tolist() == [2, -4, 7, 0]


# ----------------------------------------------------------------------------- Algorithm 1

def check_gbs_trace(o):
    # hand-worked run of Algorithm 1 on f(x) = (x - 0.3)^2 with eps = 0.1 (tests/golden/alg1_trace.txt)
    rows = []
    with open(os.path.join(GOLDEN, "alg1_trace.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([float(v) for v in line.split()])
    m, fm, trace = o.gbs_search(lambda x: (x - 0.3) ** 2, 0.1)
    assert [t[0] for t in trace] == [r[0] for r in rows]
    assert m == rows[-1][3] and fm == (m - 0.3) ** 2


def check_gbs_converges(o):
    # unimodal objectives: the result is within the final bracket width of the minimiser, the
    # objective never increases along the accepted middles, probes stay inside (0, 1)
    for cstar in (0.07, 0.3, 0.5, 0.61, 0.93, 1.0):
        for eps in (1 / 16, 1 / 64, 1 / 1024):
            f = lambda x, c=cstar: abs(x - c) ** 1.5
            m, fm, trace = o.gbs_search(f, eps)
            assert abs(m - cstar) <= 2 * eps + 1e-12, (cstar, eps, m)
            assert all(0.0 < x < 1.0 for x, _ in trace)
            assert fm == min(v for _, v in trace)
    # a flat objective never moves the middle; the bracket still closes
    m, fm, trace = o.gbs_search(lambda x: 1.0, 1 / 32)
    assert m == 0.5 and len(trace) > 4
    assert o.gbs([lambda x: (x - 0.25) ** 2, lambda x: (x - 0.75) ** 2], 1 / 256) == [0.25, 0.75]


ALL_CHECKS = [v for k, v in sorted(globals().items()) if k.startswith("check_")]
