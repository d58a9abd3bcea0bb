// Register-blocked fp64 complex FFT over LDS for the CKKS encoder / decoder (n = N/2 points).
//
// Radix-2 butterflies, R stages per pass on 2^R register-resident points of one group (same
// group geometry as the NTT passes: group g of the pass starting at stage s0 owns the points
// b*(n >> s0) + o + i*stride).  The twiddle of the pair (i, i + h) at stage s0 + k is
// e_tab[(o + (i mod h)*stride) << (s0 + k)], e_tab[r] = exp(-2 pi i r / n): 2^R - 1 distinct
// values per group and pass.
//   decimation in frequency (natural in, bit-reversed out): passes in plan order;
//   decimation in time      (bit-reversed in, natural out): passes in reverse order.
// LDS layout: no padding but an XOR swizzle of the low five index bits (the bank of an 8-byte
// element).  With lanes taking the lowest index bits that a pass leaves free, the 32 lanes of a
// half-wave vary index bits {0..4} in the wide-stride passes, {0,1,2} plus two higher bits in
// the stride-8 pass and {3..7} in the contiguous pass; the swizzle below makes the map from
// each of those bit sets to the five bank bits one-to-one (full rank over GF(2)).
//   n = 8192 (passes over bits 12-10, 9-7, 6-5, 4-3, 2-0): b5 -> x0^x3, b6 -> x1^x4, b7 -> x2
//   n = 4096 (passes over bits 11-9, 8-6, 5-3, 2-0):       b5 -> x0, b6 -> x1^x3, b7 -> x2^x4
//   n = 2048 (passes over bits 10-8, 7-5, 4-2, 1-0):       b5 -> x0^x2, b6 -> x1^x3, b7 -> x4
// The shorter transforms (n = 1024, 512: the half-length transforms of N = 2^12, 2^11) reuse the last map: any of them
// is a permutation of the low five bits for fixed higher bits, so the layout is valid at every length of at least 256.
#pragma once
#include "he_ntt_static.hpp"

namespace he {

template <int LOGn>
__host__ __device__ __forceinline__ constexpr int fswz(int a) {
  const int t = (a >> 5) & 7;
  return LOGn == 13 ? (a ^ t ^ ((t & 3) << 3)) : LOGn == 12 ? (a ^ t ^ ((t & 6) << 2)) : (a ^ (t & 3) ^ (t << 2));
}
__host__ __device__ __forceinline__ constexpr int fpad(int a) { return a; }  // array extent

template <int LOGn>
struct FftPlan;
template <>
struct FftPlan<13> {  // n = 8192: strides 1024, 128, 32, 8, 1
  static constexpr int kPasses = 5;
  static constexpr int R[5] = {3, 3, 2, 2, 3};
  static constexpr int S[5] = {0, 3, 6, 8, 10};
  static constexpr int NT = 1024;
};
template <>
struct FftPlan<11> {  // n = 2048: strides 256, 32, 4, 1
  static constexpr int kPasses = 4;
  static constexpr int R[5] = {3, 3, 3, 2, 0};
  static constexpr int S[5] = {0, 3, 6, 9, 11};
  static constexpr int NT = 256;
};
template <>
struct FftPlan<10> {  // n = 1024: strides 128, 16, 4, 1
  static constexpr int kPasses = 4;
  static constexpr int R[5] = {3, 3, 2, 2, 0};
  static constexpr int S[5] = {0, 3, 6, 8, 10};
  static constexpr int NT = 128;
};
template <>
struct FftPlan<9> {  // n = 512: strides 64, 16, 4, 1
  static constexpr int kPasses = 4;
  static constexpr int R[5] = {3, 2, 2, 2, 0};
  static constexpr int S[5] = {0, 3, 5, 7, 9};
  static constexpr int NT = 64;
};
template <>
struct FftPlan<12> {  // n = 4096: strides 512, 64, 8, 1
  static constexpr int kPasses = 4;
  static constexpr int R[5] = {3, 3, 3, 3, 0};
  static constexpr int S[5] = {0, 3, 6, 9, 12};
  static constexpr int NT = 512;
};

// R stages on one group.  DIT = false: (a, b) -> (a + b, (a - b) w), stages ascending;
// DIT = true: (a, b) -> (a + b w, a - b w), stages descending.  POS conjugates the twiddles.
// TSHIFT: e_tab holds the roots of a transform 2^TSHIFT times longer (index scaled accordingly).
template <int LOGn, int S0, int R, bool DIT, bool POS, int TSHIFT = 0>
__device__ __forceinline__ void fft_stages(double (&xr)[1 << R], double (&xi)[1 << R], int o,
                                           const double2* __restrict__ e_tab) {
  constexpr int E = 1 << R;
  constexpr int LSTRIDE = LOGn - S0 - R;
#pragma unroll
  for (int kk = 0; kk < R; ++kk) {
    const int k = DIT ? (R - 1 - kk) : kk;
    const int half = E >> (k + 1);
#pragma unroll
    for (int i = 0; i < E; ++i) {
      if (i & half) continue;
      const int r = (o + ((i & (half - 1)) << LSTRIDE)) << (S0 + k);
      double2 w = e_tab[r << TSHIFT];
      if (POS) w.y = -w.y;
      if (!DIT) {
        const double ar = xr[i], ai = xi[i], br = xr[i + half], bi = xi[i + half];
        xr[i] = ar + br;
        xi[i] = ai + bi;
        const double dr = ar - br, di = ai - bi;
        xr[i + half] = dr * w.x - di * w.y;
        xi[i + half] = dr * w.y + di * w.x;
      } else {
        const double br = xr[i + half], bi = xi[i + half];
        const double tr = br * w.x - bi * w.y, ti = br * w.y + bi * w.x;
        const double ar = xr[i], ai = xi[i];
        xr[i] = ar + tr;
        xi[i] = ai + ti;
        xr[i + half] = ar - tr;
        xi[i + half] = ai - ti;
      }
    }
  }
}

// One pass with caller-supplied load / store (index = natural position in the n-point array).
template <int LOGn, int PASS, bool DIT, bool POS, int TSHIFT = 0, class LoadF, class StoreF>
__device__ __forceinline__ void fft_pass(const double2* __restrict__ e_tab, LoadF ld, StoreF st) {
  using P = FftPlan<LOGn>;
  constexpr int S0 = P::S[PASS], R = P::R[PASS];
  using G = PassGeom<LOGn, S0, R>;
  for (int g = threadIdx.x; g < G::GROUPS; g += P::NT) {
    const int base = G::base(g);
    const int o = g & (G::STRIDE - 1);
    double xr[1 << R], xi[1 << R];
#pragma unroll
    for (int i = 0; i < G::E; ++i) ld(base + (i << G::LSTRIDE), xr[i], xi[i]);
    fft_stages<LOGn, S0, R, DIT, POS, TSHIFT>(xr, xi, o, e_tab);
#pragma unroll
    for (int i = 0; i < G::E; ++i) st(base + (i << G::LSTRIDE), xr[i], xi[i]);
  }
}

}  // namespace he
