"""CPU oracle for the online rotate-and-quantize path (TEST INFRASTRUCTURE ONLY).

A plain, slow, fp64 NumPy implementation of what the GPU library computes, written
from the paper (arXiv 2504.13989) so the HIP kernels can be checked element by
element.  It shares no code with the HIP path and must never be imported by it:
only the tests, the smoke check and the benchmark's CPU-baseline leg may use it.

What it follows
  * Sylvester matrices H_{2^k}: section 2.3.2, Eq. 1 (the block recursion).
  * Legendre symbol: section 2.3.3 (the three-case definition).
  * Paley construction, order p+1, p prime = 3 (mod 4): Appendix B, Algorithm 2.
  * Paley II construction, order 2(q+1), q prime = 1 (mod 4): NOT in the paper; the
    benchmark configurations need H_28 (q=13) and H_148 (q=73).  Standard textbook
    form: H = C (x) [[1,1],[1,-1]] + I (x) [[1,-1],[-1,-1]] with C the symmetric
    conference matrix bordered from the Legendre symbols.
  * Composite order n = p * 2^k ("known small matrices and power of 2", section
    2.3.3): H_n = H_p (x) H_{2^k}, flat index j = a * 2^k + c.
  * Dimension expansion: a row of width d < n is zero-padded to n (section 4.2, Eq. 2).
  * Rotation is H_n / sqrt(n) (Appendix A.1.1: H H^T = n I before normalisation).
  * Quantizer: section 2.1, X^ = round(X / Delta) * Delta, Delta = max|X| / (2^b - 1),
    per token (one Delta per row), with the clip ratio of section 3.1 scaling the
    maximum: Delta = clip * max|y| / (2^b - 1).

Readings taken where the paper is silent (each also listed in the design notes)
  * codes are clamped to the signed b-bit range [-2^(b-1), 2^(b-1)-1] while Delta
    keeps the paper's 2^b - 1 denominator;
  * "round" is round-half-to-even;
  * an all-zero row gets Delta = 0 and all-zero codes;
  * the mean in the quantization error runs over all rows * n rotated elements.
  * the asymmetric group quantizer of section 5.1 (named there, no formula): lo = clip * min,
    hi = clip * max per group of 128, Delta = (hi - lo) / (2^b - 1), unsigned codes, real offset;
  * Algorithm 1 (section 4.1) searches one projection at a time; its objective is a callable;
  * the expanding limit (lemma of section 4.2) is the floor of n (b - b') / b' (the text prints
    1366 for 1365.33);
  * the fused weight of section 4.2, Eq. 2 carries the same 1 / sqrt(n) as the activation side.
  PARITY UNPINNED for the first two readings and for the asymmetric quantizer's formula: the
  paper prints no worked numeric quantization example, so only the properties of the stated
  definitions pin them.

Everything is float64 unless stated.  Rotation is always a dense product of the
constructed +-1 matrices - never a butterfly.
"""
from __future__ import annotations

import functools
import math

import numpy as np

MAX_PALEY_ORDER = 256
MAX_LARGE_ORDER = 4096


# --------------------------------------------------------------------------- matrices

def sylvester(k: int) -> np.ndarray:
    """H_{2^k} by the block recursion of Eq. 1: H_{2m} = [[H_m, H_m], [H_m, -H_m]], H_1 = [1]."""
    h = np.ones((1, 1), dtype=np.int64)
    for _ in range(k):
        h = np.block([[h, h], [h, -h]])
    return h


def is_prime(p: int) -> bool:
    if p < 2:
        return False
    for f in range(2, int(math.isqrt(p)) + 1):
        if p % f == 0:
            return False
    return True


def legendre_symbol(a: int, p: int) -> int:
    """(a/p) for a prime p, by the definition of section 2.3.3: 0 if a = 0 (mod p), +1 if some
    x has x^2 = a (mod p), else -1."""
    a %= p
    if a == 0:
        return 0
    return 1 if a in _nonzero_squares(p) else -1


@functools.lru_cache(maxsize=None)
def _nonzero_squares(p: int) -> frozenset:
    return frozenset((x * x) % p for x in range(1, p))


# --- finite fields GF(p^k) for Paley orders from prime powers (the textbook generalisation: the
# Legendre symbol becomes the quadratic character of GF(q); not used by the paper's examples).
# An element is the tuple of its k coefficients, lowest degree first; element number i has the
# base-p digits of i as coefficients; the modulus is the lexicographically smallest monic
# irreducible polynomial of degree k (comparing coefficients from the highest degree down).

def prime_power(q: int):
    """(p, k) with q = p^k, p prime, k >= 1; None if q is not a prime power."""
    if q < 2:
        return None
    for p in range(2, q + 1):
        if q % p == 0:
            if not is_prime(p):
                return None
            k, v = 0, q
            while v % p == 0:
                v //= p
                k += 1
            return (p, k) if v == 1 else None
    return None


def _poly_mod(a: list, f: list, p: int) -> list:
    """Remainder of polynomial a modulo the monic polynomial f over GF(p) (coefficients low first)."""
    a = [c % p for c in a]
    k = len(f) - 1
    for i in range(len(a) - 1, k - 1, -1):
        c = a[i]
        if c:
            for j in range(k + 1):
                a[i - k + j] = (a[i - k + j] - c * f[j]) % p
    return (a + [0] * k)[:k]


def _poly_irreducible(f: list, p: int) -> bool:
    """Monic f of degree k is irreducible iff no monic polynomial of degree 1 .. k // 2 divides it."""
    k = len(f) - 1
    for deg in range(1, k // 2 + 1):
        for idx in range(p ** deg):
            g = [(idx // p ** j) % p for j in range(deg)] + [1]
            r = list(f)
            for i in range(k, deg - 1, -1):          # long division by the monic g
                c = r[i] % p
                if c:
                    for j in range(deg + 1):
                        r[i - deg + j] = (r[i - deg + j] - c * g[j]) % p
            if not any(r[:deg]):
                return False
    return True


@functools.lru_cache(maxsize=None)
def field_modulus(p: int, k: int) -> tuple:
    """Coefficients (low first, monic) of the modulus of GF(p^k): the lexicographically smallest
    monic irreducible polynomial of degree k, coefficients compared from x^(k-1) down to x^0."""
    for idx in range(p ** k):
        low = [(idx // p ** (k - 1 - j)) % p for j in range(k)]     # c_{k-1}, ..., c_0
        f = list(reversed(low)) + [1]
        if _poly_irreducible(f, p):
            return tuple(f)
    raise AssertionError("an irreducible polynomial of every degree exists")


def field_elements(q: int) -> list:
    p, k = prime_power(q)
    return [tuple((i // p ** j) % p for j in range(k)) for i in range(q)]


def field_mul(a: tuple, b: tuple, p: int, f: tuple) -> tuple:
    prod = [0] * (2 * len(a) - 1)
    for i, x in enumerate(a):
        for j, y in enumerate(b):
            prod[i + j] += x * y
    return tuple(_poly_mod(prod, list(f), p))


@functools.lru_cache(maxsize=None)
def _field_squares(q: int) -> frozenset:
    p, k = prime_power(q)
    f = field_modulus(p, k)
    return frozenset(field_mul(x, x, p, f) for x in field_elements(q) if any(x))


def quadratic_character(i: int, j: int, q: int) -> int:
    """chi(a_i - a_j) in GF(q): 0 if the elements are equal, +1 if their difference is a non-zero
    square, else -1.  For a prime q this is the Legendre symbol of i - j."""
    p, k = prime_power(q)
    if k == 1:
        return legendre_symbol(i - j, q)
    d = tuple(((i // p ** t) % p - (j // p ** t) % p) % p for t in range(k))
    if not any(d):
        return 0
    return 1 if d in _field_squares(q) else -1


def jacobsthal(q: int) -> np.ndarray:
    """Q[i, j] = chi(a_i - a_j) over GF(q) (section 2.3.3): zero diagonal, +1 where the difference of
    the two field elements is a non-zero square, -1 elsewhere.  For a prime q the elements are the
    residues and Q is the circulant of the Legendre symbols; for a prime power the differences are
    taken digit by digit (elements numbered by their base-p coefficient vectors)."""
    p, k = prime_power(q)
    idx = np.arange(q)
    if k == 1:
        chi = np.array([legendre_symbol(r, q) for r in range(q)], dtype=np.int64)
        return chi[(idx[:, None] - idx[None, :]) % q]
    digits = np.stack([(idx // p ** t) % p for t in range(k)], axis=1)           # [q, k]
    diff = (digits[:, None, :] - digits[None, :, :]) % p                        # [q, q, k]
    diff_idx = (diff * (p ** np.arange(k))).sum(axis=2)
    squares = _field_squares(q)
    chi = np.array([0 if i == 0 else (1 if x in squares else -1) for i, x in enumerate(field_elements(q))],
                   dtype=np.int64)
    return chi[diff_idx]


def paley1(p: int) -> np.ndarray:
    """Order p+1 Hadamard matrix, p a prime (power) with p = 3 (mod 4); Appendix B, Algorithm 2.

    The matrix is the Jacobsthal matrix with -1 on its diagonal, Q - I, bordered by a first row and a
    first column of -1 around a +1 corner - the same entries as the listing's element-wise rule
    (the pins hold the order-4 matrix written out)."""
    if prime_power(p) is None or p % 4 != 3:
        raise ValueError("Paley construction needs a prime (power) p = 3 (mod 4)")
    n = p + 1
    h = np.full((n, n), -1, dtype=np.int64)
    h[0, 0] = 1
    h[1:, 1:] = jacobsthal(p) - np.eye(p, dtype=np.int64)
    return h


def paley2(q: int) -> np.ndarray:
    """Order 2(q+1) Hadamard matrix, q a prime (power) with q = 1 (mod 4) (textbook Paley II).

    C = the symmetric conference matrix of order q+1: the Jacobsthal matrix bordered by a row and a
    column of +1 around a 0 corner.  H = C (x) [[1,1],[1,-1]] + I (x) [[1,-1],[-1,-1]]."""
    if prime_power(q) is None or q % 4 != 1:
        raise ValueError("Paley II construction needs a prime (power) q = 1 (mod 4)")
    m = q + 1
    c = np.ones((m, m), dtype=np.int64)
    c[0, 0] = 0
    c[1:, 1:] = jacobsthal(q)
    a = np.array([[1, 1], [1, -1]], dtype=np.int64)
    b = np.array([[1, -1], [-1, -1]], dtype=np.int64)
    return np.kron(c, a) + np.kron(np.eye(m, dtype=np.int64), b)


def paley_kind(p: int):
    """(kind, q) for a block order p: (1, p-1) if Paley I applies, else (2, p/2-1) if Paley II
    applies, else None.  Order rules: q+1 for q = 3 (mod 4), 2(q+1) for q = 1 (mod 4); q a prime,
    or failing that a prime power."""
    if p >= 4 and is_prime(p - 1) and (p - 1) % 4 == 3:
        return 1, p - 1
    if p >= 4 and p % 2 == 0 and is_prime(p // 2 - 1) and (p // 2 - 1) % 4 == 1:
        return 2, p // 2 - 1
    # prime powers only where no prime serves the order (52 = 2 (25 + 1), 100 = 2 (49 + 1), 244 = 243 + 1)
    if p >= 4 and prime_power(p - 1) is not None and (p - 1) % 4 == 3:
        return 1, p - 1
    if p >= 4 and p % 2 == 0 and prime_power(p // 2 - 1) is not None and (p // 2 - 1) % 4 == 1:
        return 2, p // 2 - 1
    return None


def factor_order(n: int):
    """n = p * 2^k with the largest 2^k such that p is 1 or a constructible Paley order
    (p <= MAX_PALEY_ORDER); failing that, with a large Paley block (p <= MAX_LARGE_ORDER).
    Returns (p, kind, q, k); kind 0 = pure Sylvester.  None if no such factorisation exists."""
    if n < 1:
        return None
    k = 0
    while n % (1 << (k + 1)) == 0:
        k += 1
    while k >= 0:
        p = n >> k
        if p == 1:
            return 1, 0, 0, k
        if p <= MAX_PALEY_ORDER:
            kq = paley_kind(p)
            if kq is not None:
                return p, kq[0], kq[1], k
        k -= 1
    # no block of at most MAX_PALEY_ORDER: a large Paley block, up to the whole dimension
    # (section 5.2.2: 1536 + 8 = 1544 = 1543 + 1 "managed by the Paley algorithm"), again with
    # the largest 2^k
    k = 0
    while n % (1 << (k + 1)) == 0:
        k += 1
    while k >= 0:
        p = n >> k
        if MAX_PALEY_ORDER < p <= MAX_LARGE_ORDER:
            kq = paley_kind(p)
            if kq is not None:
                return p, kq[0], kq[1], k
        k -= 1
    return None


def next_order(d: int, min_pow2: int = 32) -> int:
    """Dimension expansion target (section 4.2): the smallest n >= d with a factorisation
    p * 2^k as above and 2^k >= min_pow2."""
    n = d
    while True:
        f = factor_order(n)
        if f is not None and (1 << f[3]) >= min_pow2 and f[0] <= MAX_PALEY_ORDER:
            return n
        n += 1


def hadamard_factors(n: int):
    """(H_p, H_{2^k}) with H_n = H_p (x) H_{2^k}."""
    f = factor_order(n)
    if f is None:
        raise ValueError(f"no Hadamard order {n}")
    p, kind, q, k = f
    hp = np.ones((1, 1), dtype=np.int64) if kind == 0 else (paley1(q) if kind == 1 else paley2(q))
    return hp, sylvester(k)


def hadamard_dense(n: int) -> np.ndarray:
    hp, hs = hadamard_factors(n)
    return np.kron(hp, hs)


# --------------------------------------------------------------------------- rotation

def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float64."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def as_f64(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x)
    return bf16_bits_to_f64(x) if x.dtype == np.uint16 else x.astype(np.float64)


def rotate(x: np.ndarray, n: int) -> np.ndarray:
    """y = H_n pad(x) / sqrt(n) for every row of x [rows, d], d <= n.

    The dense product with H_p (x) H_{2^k} is taken as the two dense Kronecker factors on the
    row viewed as [p, 2^k]: y[a', c'] = sum_a sum_c H_p[a', a] H_{2^k}[c', c] x[a, c]."""
    x = as_f64(x)
    rows, d = x.shape
    if d > n:
        raise ValueError("d > n")
    hp, hs = hadamard_factors(n)
    p, m = hp.shape[0], hs.shape[0]
    xp = np.zeros((rows, n), dtype=np.float64)
    xp[:, :d] = x
    xm = xp.reshape(rows, p, m)
    y = np.matmul(xm, hs.astype(np.float64).T)               # along c
    y = np.einsum("ab,rbc->rac", hp.astype(np.float64), y)   # along a
    return y.reshape(rows, n) / math.sqrt(n)


def rotate_back(y: np.ndarray, n: int, d: int = None) -> np.ndarray:
    """x = H_n^T y / sqrt(n), first d columns: the inverse of rotate (H_n^T H_n = n I,
    section 2.3), which also drops the coordinates that section 4.2 padded with zeros.
    (H_p (x) H_{2^k})^T = H_p^T (x) H_{2^k}: the Sylvester factor is symmetric, a Paley block
    in general is not."""
    y = np.asarray(y, dtype=np.float64)
    rows, width = y.shape
    if width != n:
        raise ValueError("rotated rows have width n")
    hp, hs = hadamard_factors(n)
    p, m = hp.shape[0], hs.shape[0]
    ym = y.reshape(rows, p, m)
    x = np.matmul(ym, hs.astype(np.float64))                   # along c: H^T[c, c'] = H[c', c]
    x = np.einsum("ba,rbc->rac", hp.astype(np.float64), x)     # along a: H_p^T
    x = x.reshape(rows, n) / math.sqrt(n)
    return x if d is None else x[:, :d]


def fuse_weight(w: np.ndarray, n: int) -> np.ndarray:
    """Offline weight fusion of section 4.2, Eq. 2: W [d, out] is padded with zero rows to
    [n, out] and multiplied by the Hadamard matrix, W' = H_n pad(W) / sqrt(n), so that
    rotate(x) @ W' = x @ W for every row x (the 1 / sqrt(n) of both sides included)."""
    w = as_f64(w)
    return rotate(w.T, n).T


def expand_limit(n: int, b: int, b_prime: int) -> int:
    """Lemma "Expanding limit" (section 4.2): the largest number d of added dimensions for which
    the product at b' bits costs no more bit operations than the original at b bits,
    (n + d) b' <= n b, i.e. floor(n (b - b') / b')."""
    if not (1 <= b_prime <= b) or n < 1:
        raise ValueError("need 1 <= b' <= b and n >= 1")
    return (n * (b - b_prime)) // b_prime


# --------------------------------------------------------------------------- quantizer

def quant_params(b: int):
    """(L, qmin, qmax): L = 2^b - 1 is the paper's denominator; codes live in the signed b-bit
    range."""
    return (1 << b) - 1, -(1 << (b - 1)), (1 << (b - 1)) - 1


def quantize(y: np.ndarray, b: int, clip) -> tuple:
    """Per-row symmetric quantization of rotated rows y [rows, n].

    Returns (codes int8 [rows, n], delta f64 [rows], t f64 [rows, n]) with
    delta = clip * max|y| / (2^b - 1), t = y / delta, codes = clamp(round_half_even(t)).
    ``clip`` is a float32 value widened to float64 (the library takes it as a C float)."""
    lvl, qmin, qmax = quant_params(b)
    clip64 = float(np.float32(clip))
    amax = np.max(np.abs(y), axis=1)
    delta = clip64 * amax / lvl
    safe = np.where(delta > 0, delta, 1.0)
    t = y / safe[:, None]
    t[delta == 0] = 0.0
    codes = np.clip(np.rint(t), qmin, qmax).astype(np.int8)
    return codes, delta, t


def dequantize(codes: np.ndarray, delta: np.ndarray) -> np.ndarray:
    return codes.astype(np.float64) * np.asarray(delta, dtype=np.float64)[:, None]


def rotate_quantize(x: np.ndarray, n: int, b: int, clip) -> tuple:
    """The whole path for rows of x: returns (codes, delta, t, y)."""
    y = rotate(x, n)
    codes, delta, t = quantize(y, b, clip)
    return codes, delta, t, y


def quant_error(x: np.ndarray, n: int, b: int, clips) -> np.ndarray:
    """mse[k] = mean over all rows * n rotated elements of (dequant(quant(y; clips[k])) - y)^2."""
    y = rotate(x, n)
    out = np.empty(len(clips), dtype=np.float64)
    for k, c in enumerate(clips):
        codes, delta, _ = quantize(y, b, c)
        out[k] = np.mean((dequantize(codes, delta) - y) ** 2)
    return out


# --------------------------------------------------------------------------- asymmetric groups

GROUP = 128


def quantize_asym(y: np.ndarray, b: int, clip, group: int = GROUP) -> tuple:
    """Asymmetric uniform quantization of rotated rows in groups of `group` consecutive values
    (the KV-cache setting of section 5.1: "asymmetric quantization with a group size of 128").

    The paper names the scheme without a formula; the reading taken: per group, lo = clip * min,
    hi = clip * max (the clip ratio of section 3.1 shrinks the range towards zero),
    delta = (hi - lo) / (2^b - 1), code = clamp(round_half_even((y - lo) / delta), 0, 2^b - 1),
    y^ = code * delta + lo.  The offset is kept as the real number lo, not as a rounded integer
    zero point.  A constant group has delta = 0 and all-zero codes (y^ = lo).
    Returns (codes uint8 [rows, n], delta f64 [rows, n/group], lo f64 [rows, n/group], t f64)."""
    rows, n = y.shape
    if n % group:
        raise ValueError("row length must be a multiple of the group size")
    lvl = (1 << b) - 1
    clip64 = float(np.float32(clip))
    yg = y.reshape(rows, n // group, group)
    lo = clip64 * yg.min(axis=2)
    hi = clip64 * yg.max(axis=2)
    delta = (hi - lo) / lvl
    safe = np.where(delta > 0, delta, 1.0)
    t = (yg - lo[:, :, None]) / safe[:, :, None]
    t[delta == 0] = 0.0
    codes = np.clip(np.rint(t), 0, lvl).astype(np.uint8)
    return codes.reshape(rows, n), delta, lo, t.reshape(rows, n)


def dequantize_asym(codes: np.ndarray, delta: np.ndarray, lo: np.ndarray, group: int = GROUP) -> np.ndarray:
    rows, n = codes.shape
    cg = codes.reshape(rows, n // group, group).astype(np.float64)
    return (cg * delta[:, :, None] + lo[:, :, None]).reshape(rows, n)


def quant_error_asym(x: np.ndarray, n: int, b: int, clips, group: int = GROUP) -> np.ndarray:
    """quant_error with the asymmetric group quantizer: mse[k] = mean over all rows * n rotated
    elements of (dequantize_asym(quantize_asym(y; clips[k])) - y)^2 (the objective a clip search
    sees for the KV cache, sections 4.1 and 5.1)."""
    y = rotate(x, n)
    out = np.empty(len(clips), dtype=np.float64)
    for k, c in enumerate(clips):
        codes, delta, lo, _ = quantize_asym(y, b, c, group)
        out[k] = np.mean((dequantize_asym(codes, delta, lo, group) - y) ** 2)
    return out


def quantize_plain(x: np.ndarray, b: int, clip) -> tuple:
    """Per-token symmetric quantization of rows as they are (no rotation): the quantizer of
    section 2.1 applied to activations whose rotation was fused into the weights offline."""
    return quantize(as_f64(x), b, clip)


# --------------------------------------------------------------------------- packing

def pack_codes(codes: np.ndarray, b: int) -> np.ndarray:
    """Dense little-endian bitstream per row: element j occupies stream bits [j*b, (j+1)*b),
    stream bit i is bit i % 8 of byte i // 8; the field is the code's low b bits (two's
    complement).  Returns uint8 [rows, n*b/8]."""
    rows, n = codes.shape
    if (n * b) % 8:
        raise ValueError("row bit length must be a whole number of bytes")
    field = codes.astype(np.int64) & ((1 << b) - 1)
    bits = ((field[:, :, None] >> np.arange(b)) & 1).astype(np.uint8).reshape(rows, n * b)
    return np.packbits(bits, axis=1, bitorder="little")


def unpack_codes(packed: np.ndarray, b: int, n: int, signed: bool = True) -> np.ndarray:
    """Inverse of pack_codes: int8 codes [rows, n] (sign-extended), or uint8 fields as stored
    when signed is False."""
    rows = packed.shape[0]
    bits = np.unpackbits(np.asarray(packed, dtype=np.uint8), axis=1, bitorder="little")[:, : n * b]
    field = (bits.reshape(rows, n, b).astype(np.int64) << np.arange(b)).sum(axis=2)
    if not signed:
        return field.astype(np.uint8)
    field = np.where(field >= (1 << (b - 1)), field - (1 << b), field)
    return field.astype(np.int8)


# --------------------------------------------------------------------------- checker helpers

def boundary_exempt_asym(t: np.ndarray, b: int, tol: float = 1e-6) -> np.ndarray:
    """As boundary_exempt, for unsigned codes 0 .. 2^b - 1 (boundaries 1/2 .. 2^b - 3/2)."""
    lvl = (1 << b) - 1
    frac = np.abs(t - np.floor(t) - 0.5)
    return (frac < tol) & (t >= 0.5 - tol) & (t <= lvl - 0.5 + tol)


def boundary_exempt(t: np.ndarray, b: int, tol: float = 1e-6) -> np.ndarray:
    """Mask of elements whose pre-round value t lies within ``tol`` of a rounding boundary
    k + 1/2, k in [qmin, qmax - 1] (beyond those the clamp makes the code insensitive)."""
    _, qmin, qmax = quant_params(b)
    frac = np.abs(t - np.floor(t) - 0.5)
    return (frac < tol) & (t >= qmin + 0.5 - tol) & (t <= qmax - 0.5 + tol)


# --------------------------------------------------------------------------- gradual binary search

def gbs_search(f, eps: float, max_evals: int = 64):
    """Clip-ratio search for ONE projection: the inner loop of Algorithm 1 (section 4.1).

    State: the best point so far and, on either side of it, the nearest point already evaluated (0 and
    1 to begin with, the best point 1/2).  Each step probes the midpoint between the best point and
    one of those two neighbours - left, right, left, ... - and either the probe becomes the best point
    (the old best point is then its neighbour on that side) or it becomes the nearer neighbour on its
    own side.  Stops when the two neighbours are within eps of each other.
    Returns (best, f(best), trace) with trace = [(x, f(x)), ...] in evaluation order (first entry is
    the initial middle).  The paper leaves eps open; max_evals only guards against eps <= 0."""
    near = [0.0, 1.0]                                   # nearest evaluated points: [left of best, right of best]
    best = 0.5
    f_best = f(best)
    trace = [(best, f_best)]
    side = 0                                            # 0: probe towards the left neighbour, 1: the right one
    while near[1] - near[0] > eps and len(trace) < max_evals:
        x = (near[side] + best) / 2
        fx = f(x)
        trace.append((x, fx))
        if fx < f_best:
            near[1 - side] = best                       # the old best point now bounds the far side
            best, f_best = x, fx
        else:
            near[side] = x
        side = 1 - side
    return best, f_best, trace


def gbs(objectives, eps: float):
    """Algorithm 1 over a list of projections: one search per projection, in order, each appended to
    the list L.  Reading: the loop runs over all projections (the listing's upper bound n - 1 is
    taken as an off-by-one), and with a quantization-error objective the projections do not
    interact, so objectives[i] is a function of its own clip ratio only."""
    out = []
    for f in objectives:
        m, _, _ = gbs_search(f, eps)
        out.append(m)
    return out
