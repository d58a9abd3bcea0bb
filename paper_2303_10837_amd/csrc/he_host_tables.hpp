// Host-side derivation of the public crypto context: prime chain, roots of unity, transform
// twiddles with their Shoup companions, rescale / CRT constants and the encoder's FFT tables.
#pragma once
#include <stdint.h>

#include <cmath>
#include <vector>

namespace he_host {

inline uint32_t mulmod(uint32_t a, uint32_t b, uint32_t q) { return (uint32_t)((uint64_t)a * b % q); }

inline uint32_t powmod(uint32_t a, uint64_t e, uint32_t q) {
  uint32_t r = 1 % q;
  while (e) {
    if (e & 1) r = mulmod(r, a, q);
    a = mulmod(a, a, q);
    e >>= 1;
  }
  return r;
}

inline uint32_t invmod(uint32_t a, uint32_t q) { return powmod(a % q, q - 2, q); }  // q prime

// Deterministic Miller-Rabin; the bases 2, 3, 5, 7 are sufficient below 3,215,031,751.
inline bool is_prime_u32(uint32_t n) {
  if (n < 2) return false;
  const uint32_t small[] = {2, 3, 5, 7, 11, 13};
  for (uint32_t p : small) {
    if (n % p == 0) return n == p;
  }
  uint32_t d = n - 1;
  int r = 0;
  while ((d & 1) == 0) {
    d >>= 1;
    ++r;
  }
  for (uint32_t a : {2u, 3u, 5u, 7u}) {
    uint32_t x = powmod(a, d, n);
    if (x == 1 || x == n - 1) continue;
    bool composite = true;
    for (int i = 1; i < r; ++i) {
      x = mulmod(x, x, n);
      if (x == n - 1) {
        composite = false;
        break;
      }
    }
    if (composite) return false;
  }
  return true;
}

// The `count` largest primes below 2^31 with q = 1 (mod 2N), descending.
inline bool find_primes(uint32_t log2_n, uint32_t count, std::vector<uint32_t>* out) {
  const uint64_t two_n = 2ull << log2_n;
  uint64_t q = ((1ull << 31) - 1) / two_n * two_n + 1;
  if (q >= (1ull << 31)) q -= two_n;
  out->clear();
  while (out->size() < count) {
    if (q <= two_n) return false;
    if (is_prime_u32((uint32_t)q)) out->push_back((uint32_t)q);
    q -= two_n;
  }
  return true;
}

// Smallest psi with psi^N = -1 (mod q): take any primitive 2N-th root c = x^((q-1)/2N) and
// minimise over its odd powers (these are all the primitive 2N-th roots).
inline uint32_t smallest_primitive_2n_root(uint32_t q, uint32_t log2_n) {
  const uint64_t n_ring = 1ull << log2_n;
  uint32_t c = 0;
  for (uint32_t x = 2; x < q; ++x) {
    c = powmod(x, (q - 1) / (2 * n_ring), q);
    if (powmod(c, n_ring, q) == q - 1) break;
  }
  uint32_t best = c, cur = c;
  const uint32_t c2 = mulmod(c, c, q);
  for (uint64_t i = 1; i < n_ring; ++i) {
    cur = mulmod(cur, c2, q);
    if (cur < best) best = cur;
  }
  return best;
}

inline uint32_t bitrev(uint32_t x, int bits) {
  uint32_t r = 0;
  for (int i = 0; i < bits; ++i) {
    r = (r << 1) | (x & 1);
    x >>= 1;
  }
  return r;
}

struct U2 {
  uint32_t w, wp;  // value and floor(value * 2^32 / q)
};

inline U2 shoup(uint32_t w, uint32_t q) { return U2{w, (uint32_t)(((uint64_t)w << 32) / q)}; }

// table[k] = root^bitrev(k) for k < N, with Shoup companions.
inline void power_table_bitrev(uint32_t q, uint32_t root, uint32_t log2_n, U2* table) {
  const uint32_t n_ring = 1u << log2_n;
  std::vector<uint32_t> pw(n_ring);
  pw[0] = 1;
  for (uint32_t k = 1; k < n_ring; ++k) pw[k] = mulmod(pw[k - 1], root, q);
  for (uint32_t k = 0; k < n_ring; ++k) table[k] = shoup(pw[bitrev(k, (int)log2_n)], q);
}

// 5^j mod 2N and the FFT bin t_j = (5^j mod 2N - 1) / 4 of slot j.
inline void slot_bins(uint32_t log2_n, std::vector<uint32_t>* bins) {
  const uint32_t n = 1u << (log2_n - 1);
  const uint64_t two_n = 2ull << log2_n;
  bins->resize(n);
  uint64_t g = 1;
  for (uint32_t j = 0; j < n; ++j) {
    (*bins)[j] = (uint32_t)((g - 1) / 4);
    g = g * 5 % two_n;
  }
}

struct D2 {
  double x, y;
};

// exp(2 pi i * num / den), den a power of two: the turn fraction num / den is exact, the angle and cosl / sinl are
// evaluated in long double (64-bit mantissa) and rounded once to double, so an entry is off by at most about one unit
// in the last place of a double.
inline D2 unit_root(uint64_t num, uint64_t den) {
  const long double pi = 3.14159265358979323846264338327950288L;
  num %= den;
  long double frac = (long double)num / (long double)den;  // exact: den is a power of two
  long double ang = 2.0L * pi * frac;
  return D2{(double)cosl(ang), (double)sinl(ang)};
}

// Little-endian 32-bit words of the product of primes[0..level), and of (product - 1) / 2.
inline void modulus_words(const uint32_t* primes, uint32_t level, uint32_t* q_words, uint32_t* half_words) {
  std::vector<uint32_t> v(level + 1, 0);
  v[0] = 1;
  for (uint32_t j = 0; j < level; ++j) {
    uint64_t carry = 0;
    for (uint32_t i = 0; i <= level; ++i) {
      uint64_t t = (uint64_t)v[i] * primes[j] + carry;
      v[i] = (uint32_t)t;
      carry = t >> 32;
    }
  }
  for (uint32_t i = 0; i < level; ++i) q_words[i] = v[i];
  // (Q - 1) / 2: Q is odd, so this is Q >> 1
  for (uint32_t i = 0; i < level; ++i) {
    uint32_t hi = (i + 1 <= level) ? v[i + 1] : 0;
    half_words[i] = (v[i] >> 1) | (hi << 31);
  }
}

}  // namespace he_host
