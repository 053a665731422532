// Hadamard block construction on the host: Legendre symbols, the Paley construction of
// Appendix B (Algorithm 2) for q = 3 (mod 4), Paley II for q = 1 (mod 4), and the order
// factorisation n = p * 2^k (section 2.3.3).
#include "hadamard.h"

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

void paley_kind(int p, int* kind, int* q) {
    *kind = 0;
    *q = 0;
    if (p < 4) return;
    if (is_prime(p - 1) && (p - 1) % 4 == 3) {
        *kind = 1;
        *q = p - 1;
    } else if (p % 2 == 0 && is_prime(p / 2 - 1) && (p / 2 - 1) % 4 == 1) {
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

std::vector<int8_t> build_block(const Factorisation& f) {
    const int p = f.p;
    std::vector<int8_t> h((size_t)p * p, 1);
    if (f.kind == 1) {
        // order q+1: corner +1, rest of first row and column -1, diagonal -1, entry [i][j] the
        // Legendre symbol of i - j elsewhere
        for (int i = 1; i < p; ++i) {
            h[(size_t)i * p] = -1;
            h[i] = -1;
            for (int j = 1; j < p; ++j)
                h[(size_t)i * p + j] = (i == j) ? -1 : (int8_t)legendre((int64_t)i - j, f.q);
        }
    } else if (f.kind == 2) {
        // order 2(q+1): 2x2 blocks; off-diagonal block (i,j) is c_ij * [[1,1],[1,-1]] with c the
        // bordered symmetric conference matrix, diagonal blocks are [[1,-1],[-1,-1]]
        const int m = f.q + 1;
        for (int i = 0; i < m; ++i)
            for (int j = 0; j < m; ++j) {
                int8_t* b = &h[(size_t)(2 * i) * p + 2 * j];
                if (i == j) {
                    b[0] = 1; b[1] = -1; b[p] = -1; b[p + 1] = -1;
                } else {
                    int c = (i == 0 || j == 0) ? 1 : legendre((int64_t)i - j, f.q);
                    b[0] = (int8_t)c; b[1] = (int8_t)c; b[p] = (int8_t)c; b[p + 1] = (int8_t)-c;
                }
            }
    }
    return h;
}

}  // namespace rq
