// Device-side primitives for gfx950: 32-bit modular arithmetic, Philox4x32-10 and the
// samplers, register-blocked negacyclic NTT passes over an LDS-resident polynomial, and the
// fp64 FFT used by the CKKS encoder/decoder.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace he {

constexpr int kMaxLimbs = 8;

// ---------------------------------------------------------------------------------------
// 32-bit modular arithmetic.  All primes are below 2^31, so a value in [0, 2q) still fits a
// 32-bit word but a value in [0, 4q) does not: every sum is followed by one conditional
// subtraction.  Multiplication by a known constant w uses Shoup's method with the
// companion w' = floor(w * 2^32 / q): for ANY 32-bit y,
//     w*y - floor(w'*y / 2^32) * q   (computed modulo 2^32)   lies in [0, 2q).
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ uint32_t csub(uint32_t x, uint32_t q) {
  // x in [0, 2q) -> [0, q): if x < q the difference wraps to a huge value and min keeps x.
  return min(x, x - q);
}

__device__ __forceinline__ uint32_t add_mod(uint32_t a, uint32_t b, uint32_t q) {
  return csub(a + b, q);  // a, b in [0, q)
}

__device__ __forceinline__ uint32_t sub_mod(uint32_t a, uint32_t b, uint32_t q) {
  uint32_t d = a - b;     // a, b in [0, q)
  return min(d, d + q);   // if a < b, d wrapped and d + q is the small true value
}

__device__ __forceinline__ uint32_t mul_shoup_lazy(uint32_t y, uint2 w, uint32_t q) {
  return w.x * y - __umulhi(w.y, y) * q;  // in [0, 2q)
}

__device__ __forceinline__ uint32_t mul_shoup(uint32_t y, uint2 w, uint32_t q) {
  return csub(mul_shoup_lazy(y, w, q), q);
}

// The same product in three instructions instead of four: w*y as a full 64-bit multiply-add
// (v_mad_u64_u32, full rate on gfx950), then a second one adds hi * (2^32 - q); the low word is
// w*y - hi*q mod 2^32.  Left to itself the compiler sees that only the low word is used and narrows
// the pattern back to a 32-bit multiply and a subtraction; the empty asm statement below makes all
// 64 bits of the sum count as used and emits nothing.  Written as ordinary arithmetic (not as
// inline-assembly instructions) so that the scheduler knows the multiply-adds' latency and fills
// the wait state a dependent instruction needs after them with independent work instead of s_nop.
// W_SCALAR documents that w is wave-uniform (the compiler keeps it in scalar registers by itself).
// Measured 44.1 against 47.3 cycles per wave64 butterfly.
template <bool W_SCALAR>
__device__ __forceinline__ uint32_t mul_shoup_lazy_mad(uint32_t y, uint2 w, uint32_t q) {
  const uint32_t hi = __umulhi(w.y, y);
  uint64_t acc = (uint64_t)w.x * y;
  acc += (uint64_t)hi * (uint32_t)(0u - q);
  asm("" : "+v"(acc));
  return (uint32_t)acc;
}

template <bool W_SCALAR>
__device__ __forceinline__ uint32_t mul_shoup_mad(uint32_t y, uint2 w, uint32_t q) {
  return csub(mul_shoup_lazy_mad<W_SCALAR>(y, w, q), q);
}

// Signed integer (any int32) to its residue in [0, q), q in (2^30, 2^31): a negative x gets
// 2q added (2q > 2^31, so the sum is positive and below 2q; a non-negative x is below 2^31 < 2q
// already), then one conditional subtraction.
__device__ __forceinline__ uint32_t residue_of_signed(int32_t x, uint32_t q) {
  const uint32_t t = (uint32_t)x + ((uint32_t)(x >> 31) & (2u * q));
  return csub(t, q);
}

// Same for |x| < q (sampled ternary / centred-binomial values): negative x gets q added.
__device__ __forceinline__ uint32_t residue_of_small(int32_t x, uint32_t q) {
  return (uint32_t)x + ((uint32_t)(x >> 31) & q);
}

// ---------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11) and the position-addressable samplers.
//   key = (seed lo, seed hi), counter = (block, ciphertext index, client id, tag)
// ---------------------------------------------------------------------------------------

enum : uint32_t { kTagS = 0x00, kTagEpk = 0x01, kTagA0 = 0x10, kTagU = 0x20, kTagE0 = 0x21, kTagE1 = 0x22 };

__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one full-rate 32x32->64 multiply gives both halves of each product
    const uint64_t p0 = (uint64_t)M0 * c.x, p1 = (uint64_t)M1 * c.z;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    // three-input exclusive or in one instruction (v_bitop3_b32, truth table 0x96)
    c = make_uint4(__builtin_amdgcn_bitop3_b32(hi1, c.y, k.x, 0x96), lo1, __builtin_amdgcn_bitop3_b32(hi0, c.w, k.y, 0x96), lo0);
    k.x += W0;
    k.y += W1;
  }
  return c;
}

struct RngKey {
  uint2 key;
  uint32_t ct_index, client_id;
};

__device__ __forceinline__ uint4 rng_block(const RngKey& k, uint32_t block, uint32_t tag) {
  return philox4x32_10(make_uint4(block, k.ct_index, k.client_id, tag), k.key);
}

__device__ __forceinline__ int ternary_from_word(uint32_t x) {
  return (int)__umulhi(x, 3u) - 1;  // floor(3x / 2^32) - 1
}

__device__ __forceinline__ int cbd_from_words(uint32_t a, uint32_t b, uint32_t mask) {
  return __popc(a & mask) - __popc(b & mask);
}

__device__ __forceinline__ uint32_t cbd_mask(uint32_t eta) {
  return eta >= 32 ? 0xFFFFFFFFu : ((1u << eta) - 1u);
}

// ---------------------------------------------------------------------------------------
// Negacyclic NTT over an LDS-resident polynomial.
//
// Forward = decimation in time with the powers of psi merged into the twiddles: stage s
// (m = 2^s blocks of 2t = N/m elements) multiplies the upper half of block i by
// tw[m + i] = psi^bitrev(m + i) and does (x, y) -> (x + wy, x - wy).  Natural order in,
// bit-reversed order out.  Inverse = the same stages backwards with (x, y) -> (x + y,
// (x - y) * w^-1); the factor 1/N is left to the caller (it is folded into the key tables).
//
// A pass keeps 2^R elements of one butterfly group in registers and runs R consecutive
// stages on them, so a polynomial of 2^14 coefficients needs 4 trips through LDS instead
// of 14.  Group g of the pass starting at stage s0: stride = N >> (s0 + R), offset
// o = g mod stride, block b = g / stride, elements b * (N >> s0) + o + i * stride.
// At stage s0 + k the pair (i, i + 2^(R-1-k)) uses twiddle tw[2^(s0+k) + b*2^k + (i >> (R-k))].
//
// LDS index padding: 4 extra words per 64 keep the stride-4 and stride-64 passes free of
// bank conflicts (without it all lanes of the stride-4 pass fall on 4 banks).
// ---------------------------------------------------------------------------------------

__host__ __device__ __forceinline__ constexpr int lds_pad(int a) { return a + ((a >> 6) << 2); }

template <int R, bool INV, class LoadF, class StoreF>
__device__ __forceinline__ void ntt_pass(int logN, int s0, const uint2* __restrict__ tw, uint32_t q,
                                         LoadF ld, StoreF st) {
  constexpr int E = 1 << R;
  const int lstride = logN - s0 - R;
  const int stride_mask = (1 << lstride) - 1;
  const int groups = 1 << (logN - R);
  for (int g = threadIdx.x; g < groups; g += blockDim.x) {
    const int o = g & stride_mask;
    const int b = g >> lstride;
    const int base = (b << (logN - s0)) + o;
    uint32_t v[E];
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = ld(base + (i << lstride));
    if (!INV) {
#pragma unroll
      for (int k = 0; k < R; ++k) {
        const int half = 1 << (R - 1 - k);
        const int tw_base = (1 << (s0 + k)) + (b << k);
#pragma unroll
        for (int i = 0; i < E; ++i) {
          if (i & half) continue;
          const uint2 w = tw[tw_base + (i >> (R - k))];
          const uint32_t t = mul_shoup(v[i + half], w, q);
          const uint32_t x = v[i];
          v[i] = add_mod(x, t, q);
          v[i + half] = sub_mod(x, t, q);
        }
      }
    } else {
#pragma unroll
      for (int k = R - 1; k >= 0; --k) {
        const int half = 1 << (R - 1 - k);
        const int tw_base = (1 << (s0 + k)) + (b << k);
#pragma unroll
        for (int i = 0; i < E; ++i) {
          if (i & half) continue;
          const uint2 w = tw[tw_base + (i >> (R - k))];
          const uint32_t x = v[i], y = v[i + half];
          v[i] = add_mod(x, y, q);
          v[i + half] = mul_shoup(x - y + q, w, q);  // x - y + q in (0, 2q): fine for Shoup
        }
      }
    }
#pragma unroll
    for (int i = 0; i < E; ++i) st(base + (i << lstride), v[i]);
  }
}

template <bool INV, class LoadF, class StoreF>
__device__ __forceinline__ void ntt_pass_dyn(int R, int logN, int s0, const uint2* __restrict__ tw,
                                             uint32_t q, LoadF ld, StoreF st) {
  switch (R) {
    case 1: ntt_pass<1, INV>(logN, s0, tw, q, ld, st); break;
    case 2: ntt_pass<2, INV>(logN, s0, tw, q, ld, st); break;
    case 3: ntt_pass<3, INV>(logN, s0, tw, q, ld, st); break;
    default: ntt_pass<4, INV>(logN, s0, tw, q, ld, st); break;
  }
}

// Forward transform: first pass reads through `ld0` (any source), result is left in LDS
// buffer x (padded indexing).  Ends with a barrier.
template <class Load0>
__device__ __forceinline__ void ntt_forward_to_lds(uint32_t* x, int logN, const uint2* __restrict__ tw,
                                                   uint32_t q, Load0 ld0) {
  auto ldl = [=](int a) { return x[lds_pad(a)]; };
  auto stl = [=](int a, uint32_t v) { x[lds_pad(a)] = v; };
  for (int s0 = 0; s0 < logN; s0 += 4) {
    const int R = min(4, logN - s0);
    if (s0 == 0) ntt_pass_dyn<false>(R, logN, s0, tw, q, ld0, stl);
    else ntt_pass_dyn<false>(R, logN, s0, tw, q, ldl, stl);
    __syncthreads();
  }
}

// Inverse transform (without the 1/N factor): first pass reads through `ldf`, intermediate
// passes go through LDS buffer x, the final pass writes through `stl`.  The caller must
// have synchronised before the call if `ldf` reads LDS written by other threads.
template <class LoadFirst, class StoreLast>
__device__ __forceinline__ void ntt_inverse_from(uint32_t* x, int logN, const uint2* __restrict__ tw,
                                                 uint32_t q, LoadFirst ldf, StoreLast stlast) {
  auto ldl = [=](int a) { return x[lds_pad(a)]; };
  auto stl = [=](int a, uint32_t v) { x[lds_pad(a)] = v; };
  const int last_s0 = ((logN - 1) >> 2) << 2;
  for (int s0 = last_s0; s0 >= 0; s0 -= 4) {
    const int R = min(4, logN - s0);
    const bool first = (s0 == last_s0), last = (s0 == 0);
    if (first && last) ntt_pass_dyn<true>(R, logN, s0, tw, q, ldf, stlast);
    else if (first) ntt_pass_dyn<true>(R, logN, s0, tw, q, ldf, stl);
    else if (last) ntt_pass_dyn<true>(R, logN, s0, tw, q, ldl, stlast);
    else ntt_pass_dyn<true>(R, logN, s0, tw, q, ldl, stl);
    if (!last) __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
// fp64 complex FFT over LDS (separate real / imaginary arrays), decimation in time:
// bit-reversed input, natural-order output.  X_k = sum_t x_t * exp(-/+ 2 pi i t k / n);
// e_tab[r] = exp(-2 pi i r / n), r < n/2; conj_tw selects the + sign.
// Ends with a barrier.
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ void fft_dit_lds(double* re, double* im, int logn,
                                            const double2* __restrict__ e_tab, bool conj_tw) {
  const int half_n = 1 << (logn - 1);
  for (int s = 1; s <= logn; ++s) {
    const int half = 1 << (s - 1);
    const int tshift = logn - s;
    for (int b = threadIdx.x; b < half_n; b += blockDim.x) {
      const int k = b & (half - 1);
      const int i = ((b >> (s - 1)) << s) + k;
      double2 w = e_tab[k << tshift];
      if (conj_tw) w.y = -w.y;
      const double xr = re[i + half], xi = im[i + half];
      const double tr = xr * w.x - xi * w.y;
      const double ti = xr * w.y + xi * w.x;
      const double ar = re[i], ai = im[i];
      re[i] = ar + tr;
      im[i] = ai + ti;
      re[i + half] = ar - tr;
      im[i + half] = ai - ti;
    }
    __syncthreads();
  }
}

__device__ __forceinline__ uint32_t bitrev(uint32_t x, int bits) { return bits == 0 ? 0u : (__brev(x) >> (32 - bits)); }

}  // namespace he
