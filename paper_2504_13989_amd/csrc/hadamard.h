// Host-side construction of the rotation's +-1 block (integer arithmetic only).
#pragma once
#include <cstdint>
#include <vector>

namespace rq {

struct Factorisation {
    int n = 0;       // order
    int p = 1;       // block order (1 = pure Sylvester)
    int kind = 0;    // 0 Sylvester, 1 Paley (Algorithm 2), 2 Paley II
    int q = 0;       // prime (or prime power) of the Paley construction
    int log2m = 0;   // k: n = p * 2^k
};

constexpr int kMaxPaleyOrder = 256;    // blocks the hot kernels and the expansion helper use
constexpr int kMaxLargeOrder = 4096;   // largest block at all (general kernel only)

bool is_prime(int v);
// q = p^k with p prime, k >= 1.
bool prime_power(int q, int* p, int* k);
// (a/q) for a prime q by Euler's criterion a^((q-1)/2) mod q; result in {-1, 0, 1}.
int legendre(int64_t a, int q);
// kind (1 or 2) and prime for a block order p, or kind 0 if p is not constructible.
void paley_kind(int p, int* kind, int* q);
// Largest 2^k with n / 2^k equal to 1 or a constructible block order <= kMaxLargeOrder.
bool factor_order(int n, Factorisation* f);
// Row-major p x p matrix of +-1.
std::vector<int8_t> build_block(const Factorisation& f);
// Entry of H_n = H_p (x) H_{2^k}.
inline int sylvester_entry(uint32_t i, uint32_t j) { return (__builtin_popcount(i & j) & 1) ? -1 : 1; }

}  // namespace rq
