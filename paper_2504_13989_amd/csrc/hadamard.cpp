// Hadamard block construction on the host: Legendre symbols, the Paley construction of
// Appendix B (Algorithm 2) for q = 3 (mod 4), Paley II for q = 1 (mod 4), both also for prime
// powers q through the quadratic character of GF(q), and the order factorisation n = p * 2^k
// (section 2.3.3).
#include "hadamard.h"

#include <algorithm>

namespace rq {

bool is_prime(int v) {
    if (v < 2) return false;
    for (int f = 2; (int64_t)f * f <= v; ++f)
        if (v % f == 0) return false;
    return true;
}

static int64_t pow_mod(int64_t base, int64_t e, int64_t m) {
    int64_t r = 1 % m;
    base %= m;
    while (e > 0) {
        if (e & 1) r = r * base % m;
        base = base * base % m;
        e >>= 1;
    }
    return r;
}

int legendre(int64_t a, int q) {
    int64_t r = a % q;
    if (r < 0) r += q;
    if (r == 0) return 0;
    return pow_mod(r, (q - 1) / 2, q) == 1 ? 1 : -1;
}

bool prime_power(int q, int* p, int* k) {
    if (q < 2) return false;
    int f = 2;
    while (q % f != 0) ++f;                 // smallest divisor: a prime
    int v = q, e = 0;
    while (v % f == 0) {
        v /= f;
        ++e;
    }
    if (v != 1) return false;
    *p = f;
    *k = e;
    return true;
}

// GF(p^k) as polynomials over GF(p) modulo a monic irreducible polynomial of degree k; an element
// is its coefficient vector (lowest degree first), element number i has the base-p digits of i.
namespace {

using Poly = std::vector<int>;

// remainder of `a` modulo the monic polynomial `f` (degree k), coefficients low first
Poly poly_rem(Poly a, const Poly& f, int p) {
    const int k = (int)f.size() - 1;
    for (int i = (int)a.size() - 1; i >= k; --i) {
        const int c = a[i] % p;
        if (c)
            for (int j = 0; j <= k; ++j) a[i - k + j] = ((a[i - k + j] - c * f[j]) % p + p) % p;
    }
    a.resize(k, 0);
    return a;
}

bool poly_irreducible(const Poly& f, int p) {
    const int k = (int)f.size() - 1;
    for (int deg = 1; deg <= k / 2; ++deg) {
        int count = 1;
        for (int j = 0; j < deg; ++j) count *= p;
        for (int idx = 0; idx < count; ++idx) {
            Poly g(deg + 1, 1);
            for (int j = 0, v = idx; j < deg; ++j, v /= p) g[j] = v % p;
            bool zero = true;
            for (int c : poly_rem(f, g, p)) zero = zero && c == 0;
            if (zero) return false;
        }
    }
    return true;
}

// the smallest monic irreducible polynomial of degree k, coefficients compared from x^(k-1) down
Poly field_modulus(int p, int k) {
    int count = 1;
    for (int j = 0; j < k; ++j) count *= p;
    for (int idx = 0; idx < count; ++idx) {
        Poly f(k + 1, 1);
        for (int j = 0, v = idx; j < k; ++j, v /= p) f[j] = v % p;    // digit j of idx is c_j: idx orders by c_{k-1} first
        if (poly_irreducible(f, p)) return f;
    }
    return Poly();
}

Poly field_mul(const Poly& a, const Poly& b, const Poly& f, int p) {
    Poly prod(a.size() + b.size() - 1, 0);
    for (size_t i = 0; i < a.size(); ++i)
        for (size_t j = 0; j < b.size(); ++j) prod[i + j] = (prod[i + j] + a[i] * b[j]) % p;
    return poly_rem(prod, f, p);
}

// table of the quadratic character by element number: a^((q-1)/2) is 1 for non-zero squares
std::vector<int8_t> character_table(int q) {
    int p = 0, k = 0;
    prime_power(q, &p, &k);
    const Poly f = field_modulus(p, k);
    std::vector<int8_t> chi(q, 0);
    for (int i = 1; i < q; ++i) {
        Poly base(k), r(k, 0);
        for (int j = 0, v = i; j < k; ++j, v /= p) base[j] = v % p;
        r[0] = 1;
        for (int e = (q - 1) / 2; e > 0; e >>= 1) {
            if (e & 1) r = field_mul(r, base, f, p);
            base = field_mul(base, base, f, p);
        }
        bool one = r[0] == 1;
        for (int j = 1; j < k; ++j) one = one && r[j] == 0;
        chi[i] = one ? 1 : -1;
    }
    return chi;
}

// number of the element a_i - a_j (digit-wise difference mod p)
int element_diff(int i, int j, int p, int k) {
    int out = 0, w = 1;
    for (int t = 0; t < k; ++t, i /= p, j /= p, w *= p) out += (((i % p) - (j % p) + p) % p) * w;
    return out;
}

}  // namespace

void paley_kind(int p, int* kind, int* q) {
    *kind = 0;
    *q = 0;
    if (p < 4) return;
    int pp, kk;
    if (is_prime(p - 1) && (p - 1) % 4 == 3) {
        *kind = 1;
        *q = p - 1;
    } else if (p % 2 == 0 && is_prime(p / 2 - 1) && (p / 2 - 1) % 4 == 1) {
        *kind = 2;
        *q = p / 2 - 1;
    } else if (prime_power(p - 1, &pp, &kk) && (p - 1) % 4 == 3) {
        // prime powers only where no prime serves the order (52, 100, 244 ...)
        *kind = 1;
        *q = p - 1;
    } else if (p % 2 == 0 && prime_power(p / 2 - 1, &pp, &kk) && (p / 2 - 1) % 4 == 1) {
        *kind = 2;
        *q = p / 2 - 1;
    }
}

bool factor_order(int n, Factorisation* f) {
    if (n < 1) return false;
    // p only grows as k shrinks: the first constructible p met is the smallest one, so blocks of at
    // most kMaxPaleyOrder are preferred and a large block (up to the whole dimension, e.g.
    // 1544 = 1543 + 1, section 5.2.2) is used only where no small one exists
    for (int k = __builtin_ctz((unsigned)n); k >= 0; --k) {
        int p = n >> k;
        if (p == 1) {
            *f = Factorisation{n, 1, 0, 0, k};
            return true;
        }
        if (p > kMaxLargeOrder) return false;
        int kind, q;
        paley_kind(p, &kind, &q);
        if (kind) {
            *f = Factorisation{n, p, kind, q, k};
            return true;
        }
    }
    return false;
}

// Jacobsthal matrix of GF(q), row-major q x q: entry (i, j) = chi(a_i - a_j) - 0 on the diagonal, +1 for
// a non-zero square, -1 otherwise (section 2.3.3).  For a prime q the rows are the cyclic shifts of the
// Legendre symbols; for a prime power the difference of two elements is taken through element_diff.
static std::vector<int8_t> jacobsthal(int q) {
    std::vector<int8_t> m((size_t)q * q);
    if (is_prime(q)) {
        std::vector<int8_t> by_diff((size_t)q);
        for (int r = 0; r < q; ++r) by_diff[r] = (int8_t)legendre(r, q);
        for (int i = 0; i < q; ++i)
            for (int j = 0; j < q; ++j) m[(size_t)i * q + j] = by_diff[(i - j + q) % q];
        return m;
    }
    int fp = 0, fk = 0;
    prime_power(q, &fp, &fk);
    const std::vector<int8_t> chi = character_table(q);
    for (int i = 0; i < q; ++i)
        for (int j = 0; j < q; ++j) m[(size_t)i * q + j] = chi[element_diff(i, j, fp, fk)];
    return m;
}

std::vector<int8_t> build_block(const Factorisation& f) {
    const int p = f.p;
    std::vector<int8_t> h((size_t)p * p, 1);
    if (f.kind == 0) return h;
    const int q = f.q;
    const std::vector<int8_t> core = jacobsthal(q);
    if (f.kind == 1) {
        // order q + 1 (Appendix B, Algorithm 2): Q - I inside a border of -1 with a +1 corner
        std::fill(h.begin(), h.end(), (int8_t)-1);
        h[0] = 1;
        for (int i = 0; i < q; ++i)
            for (int j = 0; j < q; ++j)
                if (i != j) h[(size_t)(i + 1) * p + (j + 1)] = core[(size_t)i * q + j];
    } else {
        // order 2 (q + 1): the conference matrix C (Q inside a border of +1 with a 0 corner) spread over
        // 2 x 2 cells - C_ij [[1, 1], [1, -1]] off the diagonal, [[1, -1], [-1, -1]] on it
        const int m = q + 1;
        for (int i = 0; i < m; ++i)
            for (int j = 0; j < m; ++j) {
                const int c = (i == 0 || j == 0) ? 1 : core[(size_t)(i - 1) * q + (j - 1)];
                int8_t* cell = &h[(size_t)(2 * i) * p + 2 * j];
                const bool diag = i == j;
                cell[0] = (int8_t)(diag ? 1 : c);
                cell[1] = (int8_t)(diag ? -1 : c);
                cell[p] = (int8_t)(diag ? -1 : c);
                cell[p + 1] = (int8_t)(diag ? -1 : -c);
            }
    }
    return h;
}

}  // namespace rq
