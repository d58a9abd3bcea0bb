// MI355X (gfx950) library for HE-based federated aggregation: kernels and C ABI.
// See include/he_fedavg.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "he_device.hpp"
#include "he_fedavg.h"
#include "he_host_tables.hpp"
#include "he_fft_static.hpp"
#include "he_ntt_static.hpp"
#include "he_select.hpp"

using namespace he;

namespace {

// =========================================================================================
// Device-visible descriptors (passed to kernels by value)
// =========================================================================================

struct RingDev {
  uint32_t logN, N, L, scale_bits, eta;
  uint32_t q[kMaxLimbs];
  uint2 ninv[kMaxLimbs];     // N^-1 mod q_j (+ Shoup companion)
  uint2 ninv_w1[kMaxLimbs];  // psi_j^-bitrev(1) * N^-1 mod q_j: last-stage twiddle of a standalone inverse transform
  const uint2* tw_fwd;       // [L][N]  psi^bitrev(k)
  const uint2* tw_inv;       // [L][N]  psi^-bitrev(k)
  const double2* fft_e;      // [n/2]   exp(-2 pi i r / n)
  const double2* twist;      // [n]     exp(+i pi k / N)
  const uint32_t* perm_enc;  // [n]     bitrev(t_j): where slot j enters the encoder FFT
  const uint32_t* perm_dec;  // [n]     t_j: where slot j leaves the decoder FFT
  const uint32_t* perm_half; // [n]     (bitrev_{log2(n)-1}(t_j >> 1) << 1) | (t_j & 1): half-length encoder input
  const uint2* garner_inv;   // [kMaxLimbs * kMaxLimbs]: entry i*kMaxLimbs+j = q_i^-1 mod q_j, i < j
};

struct MaskDev {
  const uint64_t* start;    // [n_runs]     first parameter index of each masked run
  const uint64_t* prefix;   // [n_runs + 1] packed offset of each masked run
  const uint64_t* cstart;   // [n_cruns]    complement runs
  const uint64_t* cprefix;  // [n_cruns + 1]
  uint32_t n_runs, n_cruns;
  uint64_t P, P_enc;
  // Only for masks whose complement is fragmented (see build_mask_bits); nullptr otherwise.
  const uint32_t* bits;     // bit i of the array = parameter i is masked; padded with ones to whole chunks of kBitChunk
  const uint64_t* cchunk;   // [P / kBitChunk + 2] unmasked parameters before parameter c * kBitChunk
  const uint32_t* ptab;     // [P_enc / 64 + 2] index of the masked run that holds packed position 64 k (the last entries: n_runs - 1)
  const uint64_t* ident;    // {0, 0, P_enc}: run tables of the mask "the first P_enc entries of a vector of P_enc" (see k_merge_bits)
};

constexpr uint32_t kBitChunk = 4096;  // parameters per workgroup of the bit-mask compaction (256 threads x 16)

struct CrtArgs {
  uint32_t qw[kMaxLimbs];  // little-endian words of Q' = prod_{j<level} q_j
  uint32_t hw[kMaxLimbs];  // words of (Q' - 1) / 2
};

constexpr int kAggClients = 64;  // clients folded per aggregation launch (their pointers and weights travel as kernel arguments: 2.5 KiB)

struct AggArgs {
  const uint32_t* ct[kAggClients];
  uint32_t w[kAggClients][kMaxLimbs];  // w_i mod q_j
  uint32_t K;
};

struct AggConst {
  uint32_t q[kMaxLimbs];
  uint2 c32[kMaxLimbs];    // 2^32 mod q_j
  uint2 qlinv[kMaxLimbs];  // q_{L-1}^-1 mod q_j
  uint32_t qdiff[kMaxLimbs];  // q_j - q_{L-1}
  uint32_t half_last;      // (q_{L-1} - 1) / 2
};

struct PlainArgs {
  const float* w[kAggClients];
  double alpha[kAggClients];
  uint32_t K;
};

// =========================================================================================
// Kernels
// =========================================================================================

__device__ __forceinline__ uint64_t run_lookup(const uint64_t* __restrict__ start,
                                               const uint64_t* __restrict__ prefix, uint32_t n_runs,
                                               uint64_t t) {
  uint32_t lo = 0, hi = n_runs;
  while (hi - lo > 1) {
    const uint32_t mid = (lo + hi) >> 1;
    if (prefix[mid] <= t) lo = mid;
    else hi = mid;
  }
  return start[lo] + (t - prefix[lo]);
}

// Index of the run that holds packed position t (prefix[r] <= t < prefix[r+1]).
__device__ __forceinline__ uint32_t run_find(const uint64_t* __restrict__ prefix, uint32_t n_runs, uint64_t t) {
  uint32_t lo = 0, hi = n_runs;
  while (hi - lo > 1) {
    const uint32_t mid = (lo + hi) >> 1;
    if (prefix[mid] <= t) lo = mid;
    else hi = mid;
  }
  return lo;
}

// Index of the run that holds packed position t when it is known to lie in [lo, hi] (the bounds are found once per
// workgroup with uniform loads).  Block-structured masks leave 0-2 steps to walk; under a fragmented mask (a top-p
// selection over per-parameter sensitivities has runs of one or two entries) a workgroup's positions span hundreds or
// thousands of runs, and the search inside the bounds is a bisection.
__device__ __forceinline__ uint32_t run_find_in(const uint64_t* __restrict__ prefix, uint32_t lo, uint32_t hi, uint64_t t) {
  if (hi - lo <= 4) {
    uint32_t r = lo;
    while (r < hi && prefix[r + 1] <= t) ++r;
    return r;
  }
  uint32_t a = lo, b = hi + 1;  // invariant: prefix[a] <= t < prefix[b] (prefix[hi + 1] > t by the caller's bound)
  while (b - a > 1) {
    const uint32_t mid = (a + b) >> 1;
    if (prefix[mid] <= t) a = mid;
    else b = mid;
  }
  return a;
}

__device__ __forceinline__ uint64_t run_lookup_in(const uint64_t* __restrict__ start, const uint64_t* __restrict__ prefix,
                                                  uint32_t lo, uint32_t hi, uint64_t t) {
  const uint32_t r = run_find_in(prefix, lo, hi, t);
  return start[r] + (t - prefix[r]);
}

// Lookup of packed position t of a ciphertext whose positions span the runs [lo, hi]: with the table of a fragmented mask
// (the run of every 64th position) the bounds shrink to the at most 65 runs around t before the bisection.
__device__ __forceinline__ uint64_t run_lookup_ct(const MaskDev& mk, uint32_t lo, uint32_t hi, uint64_t t) {
  if (mk.ptab && hi - lo > 8) {
    lo = mk.ptab[t >> 6];
    hi = mk.ptab[(t >> 6) + 1];
  }
  return run_lookup_in(mk.start, mk.prefix, lo, hi, t);
}

// ---- a1 + a2: gather under the mask and encode one ciphertext's slots -------------------
// m_k + i m_{k+n} = Delta * zeta^-k * (1/n) * sum_j z_j exp(-2 pi i t_j k / n)
__global__ void __launch_bounds__(1024)
k_encode(RingDev rg, MaskDev mk, const float* __restrict__ w, const float* __restrict__ slots_direct,
         uint64_t first_ct, int32_t* __restrict__ m_out, double pre_scale) {
  extern __shared__ double lds_d[];
  const int logn = (int)rg.logN - 1;
  const int n = 1 << logn;
  double* re = lds_d;
  double* im = lds_d + n;
  const uint64_t c_local = blockIdx.x;
  const uint64_t c = first_ct + c_local;
  for (int j = threadIdx.x; j < n; j += blockDim.x) {
    double z = 0.0;
    if (slots_direct) {
      z = (double)slots_direct[c_local * n + j];
    } else {
      const uint64_t t = c * (uint64_t)n + (uint64_t)j;
      if (t < mk.P_enc) z = (double)w[run_lookup(mk.start, mk.prefix, mk.n_runs, t)];
    }
    const uint32_t pos = rg.perm_enc[j];
    re[pos] = z * pre_scale;  // client-side weighting (1.0 otherwise: exact)
    im[pos] = 0.0;
  }
  __syncthreads();
  fft_dit_lds(re, im, logn, rg.fft_e, false);
  const double scale = ldexp(1.0, (int)rg.scale_bits - logn);
  int32_t* out = m_out + c_local * rg.N;
  for (int k = threadIdx.x; k < n; k += blockDim.x) {
    const double2 tw = rg.twist[k];
    const double ar = re[k], ai = im[k];
    const double cr = (ar * tw.x + ai * tw.y) * scale;
    const double ci = (ai * tw.x - ar * tw.y) * scale;
    out[k] = __double2int_rn(cr);
    out[k + n] = __double2int_rn(ci);
  }
}

// ---- a3: ephemeral randomness of one ciphertext -----------------------------------------
// u (ternary), e0 and e1 (centred binomial), each as int8 [N].  Called by all NT threads of a
// workgroup; every Philox block is drawn exactly once.
template <int NT>
__device__ __forceinline__ void sample_ct(const RngKey& rk, uint32_t N, uint32_t eta, int8_t* __restrict__ u_out,
                                          int8_t* __restrict__ e0_out, int8_t* __restrict__ e1_out, uint32_t it0 = 0,
                                          uint32_t it1 = 0xFFFFFFFFu) {
  const uint32_t mask = eta == 0 ? 0u : cbd_mask(eta);
  uint32_t* u32 = reinterpret_cast<uint32_t*>(u_out);
  uint32_t* e0w = reinterpret_cast<uint32_t*>(e0_out);
  uint32_t* e1w = reinterpret_cast<uint32_t*>(e1_out);
  auto pack4 = [](int a, int b, int c, int d) {
    return (uint32_t)(uint8_t)a | ((uint32_t)(uint8_t)b << 8) | ((uint32_t)(uint8_t)c << 16) | ((uint32_t)(uint8_t)d << 24);
  };
  // 4 coefficients per iteration and stream; iterations [it0, it1) of the N / (4 NT) a thread owns
  for (uint32_t it = it0, b = threadIdx.x + it0 * NT; it < it1 && b < N / 4; ++it, b += NT) {
    const uint4 r = rng_block(rk, b, kTagU);
    u32[b] = pack4(ternary_from_word(r.x), ternary_from_word(r.y), ternary_from_word(r.z), ternary_from_word(r.w));
    const uint4 a0 = rng_block(rk, 2 * b, kTagE0), a1 = rng_block(rk, 2 * b + 1, kTagE0);
    e0w[b] = pack4(cbd_from_words(a0.x, a0.y, mask), cbd_from_words(a0.z, a0.w, mask), cbd_from_words(a1.x, a1.y, mask),
                   cbd_from_words(a1.z, a1.w, mask));
    const uint4 b0 = rng_block(rk, 2 * b, kTagE1), b1 = rng_block(rk, 2 * b + 1, kTagE1);
    e1w[b] = pack4(cbd_from_words(b0.x, b0.y, mask), cbd_from_words(b0.z, b0.w, mask), cbd_from_words(b1.x, b1.y, mask),
                   cbd_from_words(b1.z, b1.w, mask));
  }
}

__global__ void __launch_bounds__(256)
k_sample(RingDev rg, uint2 key, uint32_t client, uint64_t first_ct, int8_t* __restrict__ u_out, int8_t* __restrict__ e0_out,
         int8_t* __restrict__ e1_out) {
  const uint64_t c_local = blockIdx.x;
  const RngKey rk{key, (uint32_t)(first_ct + c_local), client};
  sample_ct<256>(rk, rg.N, rg.eta, u_out + c_local * rg.N, e0_out + c_local * rg.N, e1_out + c_local * rg.N);
}

// ---- specialised encoder: the slot vector is real, so its n-point transform comes from one
// n/2-point complex FFT of z_s = Y_{2s} + i Y_{2s+1} (Y = slots placed at their bins) and a
// split step:  E_k = (Z_k + conj Z_{h-k})/2,  O_k = (Z_k - conj Z_{h-k})/(2i),
//              A_k = E_k + w^k O_k,  A_{k+h} = E_k - w^k O_k,  w = exp(-2 pi i / n),  h = n/2.
// Half the flops and half the LDS (two workgroups per CU) of the full-length transform.
template <int LOGN>
__global__ void __launch_bounds__(FftPlan<LOGN - 2>::NT)
k_encode_r(RingDev rg, MaskDev mk, const float* __restrict__ w, const float* __restrict__ slots_direct,
           uint64_t first_ct, int32_t* __restrict__ m_out, uint2 key, uint32_t client, int8_t* __restrict__ u_out,
           int8_t* __restrict__ e0_out, int8_t* __restrict__ e1_out, double pre_scale) {
  constexpr int LOGh = LOGN - 2, h = 1 << LOGh, n = 2 * h, N = 4 * h;
  using P = FftPlan<LOGh>;
  extern __shared__ double lds_d[];
  double* re = lds_d;
  double* im = lds_d + h;
  const uint64_t c_local = blockIdx.x;
  const uint64_t c = first_ct + c_local;
  // Gather: all loads of a thread are issued before any is consumed (U per thread, fixed).
  constexpr int U = n / P::NT;
  uint32_t code[U];
  float z[U];
#pragma unroll
  for (int u = 0; u < U; ++u) code[u] = rg.perm_half[threadIdx.x + u * P::NT];  // (bitrev(bin >> 1) << 1) | (bin & 1)
  if (slots_direct) {
    const float* sc = slots_direct + c_local * n;
#pragma unroll
    for (int u = 0; u < U; ++u) z[u] = sc[threadIdx.x + u * P::NT];
  } else {
    // runs that this ciphertext's packed range [c*n, (c+1)*n) touches
    const uint64_t t_first = c * (uint64_t)n;
    const uint32_t r_lo = run_find(mk.prefix, mk.n_runs, t_first);
    const uint32_t r_hi = run_find(mk.prefix, mk.n_runs, min(t_first + n, mk.P_enc) - 1);
    if (r_lo == r_hi) {  // common case: one run, a plain shifted copy
      const float* wc = w + (mk.start[r_lo] + (t_first - mk.prefix[r_lo]));
      const uint64_t live = min((uint64_t)n, mk.P_enc - t_first);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t j = threadIdx.x + u * P::NT;
        z[u] = j < live ? wc[j] : 0.f;
      }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t t = t_first + threadIdx.x + u * P::NT;
        z[u] = t < mk.P_enc ? w[run_lookup_ct(mk, r_lo, r_hi, t)] : 0.f;
      }
    }
  }
  // The ciphertext's randomness (u, e0, e1) is drawn in this kernel too, in slices placed where the encoder waits:
  // behind the gather loads and in front of every barrier.  The sampler is pure integer arithmetic, the transform
  // waits on LDS, twiddle loads and barriers, and the slices of one wavefront fill the waits of the others.
  static_assert(N / 4 / P::NT == 8, "eight sampler iterations per thread");
  const RngKey rk{key, (uint32_t)c, client};
  auto sample = [&](uint32_t it0, uint32_t it1) {
    if (u_out) sample_ct<P::NT>(rk, N, rg.eta, u_out + c_local * N, e0_out + c_local * N, e1_out + c_local * N, it0, it1);
  };
  sample(0, 3);
#pragma unroll
  for (int u = 0; u < U; ++u) ((code[u] & 1) ? im : re)[fswz<LOGh>((int)(code[u] >> 1))] = (double)z[u] * pre_scale;
  __syncthreads();
  const double2* e_tab = rg.fft_e;  // roots of the n-point transform: the h-point one uses every other entry
  auto ldl = [=](int a, double& r, double& i) { r = re[fswz<LOGh>(a)]; i = im[fswz<LOGh>(a)]; };
  auto stl = [=](int a, double r, double i) { re[fswz<LOGh>(a)] = r; im[fswz<LOGh>(a)] = i; };
  fft_pass<LOGh, 3, true, false, 1>(e_tab, ldl, stl);
  sample(3, 4);
  __syncthreads();
  fft_pass<LOGh, 2, true, false, 1>(e_tab, ldl, stl);
  sample(4, 5);
  __syncthreads();
  fft_pass<LOGh, 1, true, false, 1>(e_tab, ldl, stl);
  sample(5, 6);
  __syncthreads();
  fft_pass<LOGh, 0, true, false, 1>(e_tab, ldl, stl);
  sample(6, 7);
  __syncthreads();
  static_assert(P::kPasses == 4, "plans of the half-length transforms have four passes");
  const double scale = ldexp(1.0, (int)rg.scale_bits - LOGh - 2);  // Delta / n, and the 1/2 of the split step
  int32_t* out = m_out + c_local * N;
  const double2* twist = rg.twist;
#pragma unroll
  for (int ku = 0; ku < h / P::NT; ++ku) {
    const int k = threadIdx.x + ku * P::NT;
    const int kp = (h - k) & (h - 1);
    const double zr = re[fswz<LOGh>(k)], zi = im[fswz<LOGh>(k)];
    const double pr = re[fswz<LOGh>(kp)], pi = im[fswz<LOGh>(kp)];
    const double er = zr + pr, ei = zi - pi;          // 2 E_k
    const double o_r = zi + pi, o_i = pr - zr;        // 2 O_k
    const double2 wk = e_tab[k];
    const double tr = o_r * wk.x - o_i * wk.y, ti = o_r * wk.y + o_i * wk.x;
    const double a0r = er + tr, a0i = ei + ti;        // 2 A_k
    const double a1r = er - tr, a1i = ei - ti;        // 2 A_{k+h}
    const double2 t0 = twist[k], t1 = twist[k + h];
    out[k] = __double2int_rn((a0r * t0.x + a0i * t0.y) * scale);
    out[k + n] = __double2int_rn((a0i * t0.x - a0r * t0.y) * scale);
    out[k + h] = __double2int_rn((a1r * t1.x + a1i * t1.y) * scale);
    out[k + h + n] = __double2int_rn((a1i * t1.x - a1r * t1.y) * scale);
  }
  sample(7, 8);
}

// ---- a4: public-key encryption of one (ciphertext, limb) --------------------------------
// c0 = INTT(b^ . NTT(u)) + (m + e0),  c1 = INTT(a^ . NTT(u)) + e1   (mod q_j)
// pk holds b^ and a^ premultiplied by 1/N, with Shoup companions; m + e0 must fit 32 bits.
__global__ void __launch_bounds__(1024)
k_encrypt(RingDev rg, const uint2* __restrict__ pk, const int8_t* __restrict__ u, const int32_t* __restrict__ m,
          const int8_t* __restrict__ e0, const int8_t* __restrict__ e1, uint32_t* __restrict__ ct_out) {
  extern __shared__ uint32_t lds_u[];
  const int logN = (int)rg.logN;
  const uint32_t N = rg.N, L = rg.L;
  const uint32_t j = blockIdx.x;
  const uint64_t c = blockIdx.y;
  const uint32_t q = rg.q[j];
  uint32_t* bufU = lds_u;
  uint32_t* bufW = lds_u + lds_pad((int)N);
  const int8_t* uc = u + c * N;
  ntt_forward_to_lds(bufU, logN, rg.tw_fwd + (size_t)j * N, q, [=](int a) {
    const int v = uc[a];
    return (uint32_t)(v < 0 ? v + (int)q : v);
  });
  const int32_t* mc = m + c * N;
  const int8_t* e0c = e0 + c * N;
  const int8_t* ec = e1 + c * N;
  for (uint32_t p = 0; p < 2; ++p) {
    const uint2* key = pk + ((size_t)p * L + j) * N;
    uint32_t* out = ct_out + ((c * 2 + p) * L + j) * N;
    if (p == 0) {
      ntt_inverse_from(
          bufW, logN, rg.tw_inv + (size_t)j * N, q, [=](int a) { return mul_shoup(bufU[lds_pad(a)], key[a], q); },
          [=](int a, uint32_t v) { out[a] = add_mod(v, residue_of_signed(mc[a] + (int32_t)e0c[a], q), q); });
    } else {
      ntt_inverse_from(
          bufW, logN, rg.tw_inv + (size_t)j * N, q, [=](int a) { return mul_shoup(bufU[lds_pad(a)], key[a], q); },
          [=](int a, uint32_t v) { out[a] = add_mod(v, residue_of_signed((int32_t)ec[a], q), q); });
    }
    __syncthreads();
  }
}

// ---- a8: decryption of one (ciphertext, limb): d = c0 + INTT(s^ . NTT(c1)) ----------------
__global__ void __launch_bounds__(1024)
k_decrypt(RingDev rg, const uint2* __restrict__ sk, const uint32_t* __restrict__ ct, uint32_t level,
          uint32_t* __restrict__ d_out) {
  extern __shared__ uint32_t lds_u[];
  const int logN = (int)rg.logN;
  const uint32_t N = rg.N;
  const uint32_t j = blockIdx.x;
  const uint64_t c = blockIdx.y;
  const uint32_t q = rg.q[j];
  const uint32_t* c0 = ct + ((c * 2 + 0) * level + j) * N;
  const uint32_t* c1 = ct + ((c * 2 + 1) * level + j) * N;
  uint32_t* out = d_out + (c * level + j) * N;
  const uint2* key = sk + (size_t)j * N;
  uint32_t* buf = lds_u;
  ntt_forward_to_lds(buf, logN, rg.tw_fwd + (size_t)j * N, q, [=](int a) { return c1[a]; });
  ntt_inverse_from(
      buf, logN, rg.tw_inv + (size_t)j * N, q, [=](int a) { return mul_shoup(buf[lds_pad(a)], key[a], q); },
      [=](int a, uint32_t v) { out[a] = add_mod(v, c0[a], q); });
}

// ---- compile-time specialised versions of the three transform kernels (N = 2^11 ... 2^14) ----
// Same results as k_encrypt / k_decrypt / k_ntt_batch; see he_ntt_static.hpp for the plan.

__device__ __forceinline__ void load_key8(const uint2* __restrict__ key, int base, uint2 (&k)[8]) {
  const uint4* p = reinterpret_cast<const uint4*>(key + base);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint4 t = p[i];
    k[2 * i] = make_uint2(t.x, t.y);
    k[2 * i + 1] = make_uint2(t.z, t.w);
  }
}

// w_i = v_i * key[base + i] mod q for 8 consecutive table entries, four at a time (16-byte loads; eight entries
// at once would hold 16 registers the kernel does not have).
__device__ __forceinline__ void key_product8(const uint2* __restrict__ key, int base, const uint32_t (&v)[8], uint32_t (&w)[8],
                                             uint32_t q) {
  const uint4* p = reinterpret_cast<const uint4*>(key + base);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint4 t0 = p[2 * h], t1 = p[2 * h + 1];
    w[4 * h + 0] = mul_shoup_mad<false>(v[4 * h + 0], make_uint2(t0.x, t0.y), q);
    w[4 * h + 1] = mul_shoup_mad<false>(v[4 * h + 1], make_uint2(t0.z, t0.w), q);
    w[4 * h + 2] = mul_shoup_mad<false>(v[4 * h + 2], make_uint2(t1.x, t1.y), q);
    w[4 * h + 3] = mul_shoup_mad<false>(v[4 * h + 3], make_uint2(t1.z, t1.w), q);
  }
}

// One LDS buffer per workgroup (two workgroups per CU) and at most 64 registers per thread (8
// waves per SIMD): the kernel waits on table loads from L2 most of the time it is not computing,
// and resident waves are what hides that.  The two inverse transforms (c0, c1) run one after the
// other through the same buffer; after the fused middle pass the second polynomial waits in
// registers (16 per thread), so the kernel's only global traffic is its inputs, tables and outputs.
template <int LOGN>
__global__ void __launch_bounds__(NttPlan<LOGN>::NT, 8)
k_encrypt_s(RingDev rg, const uint2* __restrict__ pk, const int8_t* __restrict__ u, const int32_t* __restrict__ m,
            const int8_t* __restrict__ e0, const int8_t* __restrict__ e1, uint32_t* __restrict__ ct_out, uint32_t n_ct) {
  using P = NttPlan<LOGN>;
  constexpr int N = 1 << LOGN, NT = P::NT;
  extern __shared__ uint32_t lds_u[];
  uint32_t* A = lds_u;
  const uint32_t L = rg.L;
  // Workgroups are dealt to the 8 XCDs round-robin by linear id (id = slot * 8 + xcd), and each XCD has its own L2.
  // The L limb-workgroups of a ciphertext sit on ONE XCD at consecutive slots, so that the ciphertext's inputs
  // (u, m, e0, e1: 7 N bytes) leave HBM once and the other L - 1 workgroups find them in that XCD's L2: measured
  // 1.10 x the algorithmic bytes, against 1.5 x when every XCD works on one limb (which keeps less table data per L2,
  // 512 KiB instead of 2 MiB at N = 2^14, L = 4, but reads the inputs on L XCDs) and 2 % faster.
  const uint32_t slot = blockIdx.x >> 3, xcd = blockIdx.x & 7;
  const uint32_t j = slot % L;
  const uint64_t c_lin = (uint64_t)(slot / L) * 8 + xcd;
  if (c_lin >= n_ct) return;  // whole workgroup leaves before any barrier
  // Last ciphertext first: the encoder has just written this launch's inputs in ascending order (235 MB per 2048
  // ciphertexts at N = 2^14, about what the last-level cache holds), so the ones written last are the ones still cached
  // when this kernel starts; going through them in the encoder's order measured 1.8 % slower.
  const uint64_t c = n_ct - 1 - c_lin;
  const uint32_t q = rg.q[j];
  const uint2* twf = rg.tw_fwd + (size_t)j * N;
  const uint2* twi = rg.tw_inv + (size_t)j * N;
  const int8_t* uc = u + c * N;
  uint32_t* const out0 = ct_out + ((c * 2 + 0) * L + j) * N;
  uint32_t* const out1 = ct_out + ((c * 2 + 1) * L + j) * N;
  fwd_head<LOGN, NT>(A, twf, q, [=](int a) { return residue_of_small((int32_t)uc[a], q); });
  constexpr int S3 = P::S[3], R3 = P::R[3];
  static_assert(R3 == 3, "the fused middle pass works on groups of 8");
  constexpr int IT3 = OwnedIters<LOGN, 3, NT>::value;
  // Forward pass 3, product with b^ / a^, inverse pass 3: all on the same 8 coefficients.  The first polynomial goes
  // back to LDS; the second one (16 words per thread) waits in registers until the first has left the buffer.
  uint32_t parked[IT3][8];
  {
    const uint2* kb = pk + ((size_t)0 * L + j) * N;
    const uint2* ka = pk + ((size_t)1 * L + j) * N;
#pragma unroll
    for (int it = 0; it < IT3; ++it) {
      const int g = owned_group<LOGN, 3, NT>(it);
      uint32_t v[1][8];
      lds_load_group<LOGN, S3, R3>(A, g, v[0]);
      bfly_stages<LOGN, S3, R3, false, 1, true>(v, g, twf, q);
      uint32_t w[1][8];
      key_product8(kb, g << 3, v[0], w[0], q);
      bfly_stages<LOGN, S3, R3, true, 1>(w, g, twi, q);
      lds_store_group<LOGN, S3, R3>(A, g, w[0]);
      key_product8(ka, g << 3, v[0], w[0], q);
      bfly_stages<LOGN, S3, R3, true, 1>(w, g, twi, q);
#pragma unroll
      for (int i = 0; i < 8; ++i) parked[it][i] = w[0][i];
    }
  }
  uint32_t* const xs[1] = {A};
  constexpr int R0 = P::R[0];
  using G0 = PassGeom<LOGN, 0, R0>;
  const int32_t* mc = m + c * N;
  const int8_t* e0c = e0 + c * N;
  const int8_t* e1c = e1 + c * N;
#pragma unroll
  for (int poly = 0; poly < 2; ++poly) {
    if (poly == 1) {
      __syncthreads();  // every wave's reads of the first polynomial are done
#pragma unroll
      for (int it = 0; it < IT3; ++it) lds_store_group<LOGN, S3, R3>(A, owned_group<LOGN, 3, NT>(it), parked[it]);
    }
    inv_middle<LOGN, 1, NT>(xs, twi, q);
    uint32_t* out = poly == 0 ? out0 : out1;
    // inverse pass 0, + (m + e0) or + e1, streaming store (kept from evicting the key / twiddle
    // tables that every workgroup shares)
#pragma unroll
    for (int g = threadIdx.x; g < G0::GROUPS; g += NT) {
      uint32_t v[1][1 << R0];
      lds_load_group<LOGN, 0, R0>(A, g, v[0]);
      bfly_stages<LOGN, 0, R0, true, 1>(v, 0, twi, q);
#pragma unroll
      for (int i = 0; i < G0::E; ++i) {
        const int a = g + (i << G0::LSTRIDE);
        const uint32_t r = poly == 0 ? residue_of_signed(mc[a] + (int32_t)e0c[a], q) : residue_of_small((int32_t)e1c[a], q);
        __builtin_nontemporal_store(add_mod(v[0][i], r, q), out + a);
      }
    }
  }
}

template <int LOGN>
__global__ void __launch_bounds__(NttPlan<LOGN>::NT, 8)  // two workgroups per CU, 8 waves per SIMD
k_decrypt_s(RingDev rg, const uint2* __restrict__ sk, const uint32_t* __restrict__ ct, uint32_t level,
            uint32_t* __restrict__ d_out) {
  using P = NttPlan<LOGN>;
  constexpr int N = 1 << LOGN, NT = P::NT;
  extern __shared__ uint32_t lds_u[];
  uint32_t* A = lds_u;
  const uint32_t j = blockIdx.x;
  const uint64_t c = blockIdx.y;
  const uint32_t q = rg.q[j];
  const uint2* twf = rg.tw_fwd + (size_t)j * N;
  const uint2* twi = rg.tw_inv + (size_t)j * N;
  const uint32_t* c0 = ct + ((c * 2 + 0) * level + j) * N;
  const uint32_t* c1 = ct + ((c * 2 + 1) * level + j) * N;
  uint32_t* out = d_out + (c * level + j) * N;
  const uint2* key = sk + (size_t)j * N;
  fwd_head<LOGN, NT>(A, twf, q, [=](int a) { return c1[a]; });
  {
    constexpr int S0 = P::S[3], R = P::R[3];
    static_assert(R == 3, "the fused middle pass works on groups of 8");
#pragma unroll
    for (int it = 0; it < OwnedIters<LOGN, 3, NT>::value; ++it) {
      const int g = owned_group<LOGN, 3, NT>(it);
      uint32_t v[1][8];
      lds_load_group<LOGN, S0, R>(A, g, v[0]);
      bfly_stages<LOGN, S0, R, false, 1, true>(v, g, twf, q);
      uint2 k0[8];
      load_key8(key, g << 3, k0);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[0][i] = mul_shoup_mad<false>(v[0][i], k0[i], q);
      bfly_stages<LOGN, S0, R, true, 1>(v, g, twi, q);
      lds_store_group<LOGN, S0, R>(A, g, v[0]);
    }
  }
  uint32_t* const xs[1] = {A};
  inv_middle<LOGN, 1, NT>(xs, twi, q);
  {
    constexpr int R = P::R[0];
    using G = PassGeom<LOGN, 0, R>;
#pragma unroll
    for (int g = threadIdx.x; g < G::GROUPS; g += NT) {
      uint32_t v[1][1 << R];
      lds_load_group<LOGN, 0, R>(A, g, v[0]);
      bfly_stages<LOGN, 0, R, true, 1>(v, 0, twi, q);
#pragma unroll
      for (int i = 0; i < G::E; ++i) {
        const int a = g + (i << G::LSTRIDE);
        out[a] = add_mod(v[0][i], c0[a], q);
      }
    }
  }
}

template <int LOGN, bool INV>
__global__ void __launch_bounds__(NttPlan<LOGN>::NT, 8)
k_ntt_batch_s(RingDev rg, int limb, uint32_t* __restrict__ polys) {
  using P = NttPlan<LOGN>;
  constexpr int N = 1 << LOGN;
  extern __shared__ uint32_t lds_u[];
  uint32_t* A = lds_u;
  const uint32_t j = limb >= 0 ? (uint32_t)limb : (uint32_t)(blockIdx.x % rg.L);
  const uint32_t q = rg.q[j];
  uint32_t* x = polys + (size_t)blockIdx.x * N;
  constexpr int S3 = P::S[3], R3 = P::R[3];
  if (!INV) {
    const uint2* twf = rg.tw_fwd + (size_t)j * N;
    fwd_head<LOGN>(A, twf, q, [=](int a) { return x[a]; });
#pragma unroll
    for (int it = 0; it < OwnedIters<LOGN, 3, P::NT>::value; ++it) {
      const int g = owned_group<LOGN, 3, P::NT>(it);
      uint32_t v[1][1 << R3];
      lds_load_group<LOGN, S3, R3>(A, g, v[0]);
      bfly_stages<LOGN, S3, R3, false, 1>(v, g, twf, q);
      uint4* o = reinterpret_cast<uint4*>(x + (g << R3));
#pragma unroll
      for (int i = 0; i < (1 << R3); i += 4) o[i >> 2] = make_uint4(v[0][i], v[0][i + 1], v[0][i + 2], v[0][i + 3]);
    }
  } else {
    const uint2* twi = rg.tw_inv + (size_t)j * N;
    const uint2 ninv = rg.ninv[j], ninv_w1 = rg.ninv_w1[j];
#pragma unroll
    for (int it = 0; it < OwnedIters<LOGN, 3, P::NT>::value; ++it) {
      const int g = owned_group<LOGN, 3, P::NT>(it);
      uint32_t v[1][1 << R3];
      const uint4* in = reinterpret_cast<const uint4*>(x + (g << R3));
#pragma unroll
      for (int i = 0; i < (1 << R3); i += 4) {
        const uint4 t = in[i >> 2];
        v[0][i] = t.x; v[0][i + 1] = t.y; v[0][i + 2] = t.z; v[0][i + 3] = t.w;
      }
      bfly_stages<LOGN, S3, R3, true, 1>(v, g, twi, q);
      lds_store_group<LOGN, S3, R3>(A, g, v[0]);
    }
    uint32_t* const xs[1] = {A};
    inv_middle<LOGN, 1>(xs, twi, q);
    constexpr int R0 = P::R[0];
    using G0 = PassGeom<LOGN, 0, R0>;
    for (int g = threadIdx.x; g < G0::GROUPS; g += P::NT) {
      uint32_t v[1][1 << R0];
      lds_load_group<LOGN, 0, R0>(A, g, v[0]);
      bfly_stages<LOGN, 0, R0, true, 1, false, true>(v, 0, twi, q, ninv, ninv_w1);
#pragma unroll
      for (int i = 0; i < G0::E; ++i) x[g + (i << G0::LSTRIDE)] = v[0][i];
    }
  }
}

// ---- a9: CRT lift (Garner), exact centring, conversion to fp64 ---------------------------
template <int LEVEL>
__device__ __forceinline__ double crt_centered(const RingDev& rg, const CrtArgs& ca, const uint32_t (&res)[LEVEL]) {
  uint32_t x[LEVEL];  // mixed-radix digits: v = x0 + q0 (x1 + q1 (x2 + ...))
#pragma unroll
  for (int j = 0; j < LEVEL; ++j) {
    const uint32_t qj = rg.q[j];
    uint32_t t = res[j];
#pragma unroll
    for (int i = 0; i < j; ++i) {
      t = sub_mod(t, csub(x[i], qj), qj);
      t = mul_shoup(t, rg.garner_inv[i * kMaxLimbs + j], qj);
    }
    x[j] = t;
  }
  uint32_t wds[LEVEL];
#pragma unroll
  for (int i = 0; i < LEVEL; ++i) wds[i] = 0;
  wds[0] = x[LEVEL - 1];
#pragma unroll
  for (int j = LEVEL - 2; j >= 0; --j) {
    uint64_t carry = x[j];
#pragma unroll
    for (int i = 0; i < LEVEL; ++i) {
      const uint64_t t = (uint64_t)wds[i] * rg.q[j] + carry;
      wds[i] = (uint32_t)t;
      carry = t >> 32;
    }
  }
  // v > (Q'-1)/2 ?  compare from the top word down
  bool greater = false, decided = false;
#pragma unroll
  for (int i = LEVEL - 1; i >= 0; --i) {
    if (!decided && wds[i] != ca.hw[i]) {
      greater = wds[i] > ca.hw[i];
      decided = true;
    }
  }
  if (greater) {  // v - Q' is negative: magnitude Q' - v
    uint64_t borrow = 0;
#pragma unroll
    for (int i = 0; i < LEVEL; ++i) {
      const uint64_t t = (uint64_t)ca.qw[i] - wds[i] - borrow;
      wds[i] = (uint32_t)t;
      borrow = (t >> 32) & 1;
    }
  }
  double r = 0.0;
#pragma unroll
  for (int i = LEVEL - 1; i >= 0; --i) r = r * 4294967296.0 + (double)wds[i];
  return greater ? -r : r;
}

// ---- a9 + a10: lift, decode, scatter one ciphertext ---------------------------------------
// z_j = Re( sum_k (v_k + i v_{k+n}) zeta^k exp(+2 pi i t_j k / n) ) / Delta
template <int LEVEL>
__global__ void __launch_bounds__(1024)
k_decode(RingDev rg, CrtArgs ca, MaskDev mk, const uint32_t* __restrict__ d, uint64_t first_ct,
         float* __restrict__ w_out, double* __restrict__ slots_out) {
  extern __shared__ double lds_d[];
  const int logn = (int)rg.logN - 1;
  const int n = 1 << logn;
  const uint32_t N = rg.N;
  double* re = lds_d;
  double* im = lds_d + n;
  const uint64_t c_local = blockIdx.x;
  const uint32_t* dc = d + c_local * LEVEL * N;
  for (int k = threadIdx.x; k < n; k += blockDim.x) {
    uint32_t ra[LEVEL], rb[LEVEL];
#pragma unroll
    for (int j = 0; j < LEVEL; ++j) {
      ra[j] = dc[(size_t)j * N + k];
      rb[j] = dc[(size_t)j * N + k + n];
    }
    const double vr = crt_centered<LEVEL>(rg, ca, ra);
    const double vi = crt_centered<LEVEL>(rg, ca, rb);
    const double2 tw = rg.twist[k];
    const uint32_t pos = bitrev((uint32_t)k, logn);
    re[pos] = vr * tw.x - vi * tw.y;
    im[pos] = vr * tw.y + vi * tw.x;
  }
  __syncthreads();
  fft_dit_lds(re, im, logn, rg.fft_e, true);
  const double inv_delta = ldexp(1.0, -(int)rg.scale_bits);
  for (int j = threadIdx.x; j < n; j += blockDim.x) {
    const double z = re[rg.perm_dec[j]] * inv_delta;
    if (slots_out) {
      slots_out[c_local * n + j] = z;
    } else {
      const uint64_t t = (first_ct + c_local) * (uint64_t)n + (uint64_t)j;
      if (t < mk.P_enc) w_out[run_lookup(mk.start, mk.prefix, mk.n_runs, t)] = (float)z;
    }
  }
}

// ---- half-length decoder (the tuned sizes): only the REAL part of the n-point transform is wanted, so it is the
// inverse real transform of the Hermitian part of the input and comes from one n/2-point complex FFT (the encoder's
// network transposed).  With d_k = (v_k + i v_{k+n}) zeta^k, h = n/2, w = exp(+2 pi i / n):
//     X_k = (d_k + conj d_{n-k}) / 2,            Y_k = conj X_{h-k} = (conj d_{h-k} + d_{h+k}) / 2,
//     Z_k = (X_k + Y_k) + i w^k (X_k - Y_k),     Z_{h-k} = conj(X_k + Y_k) + i conj(w^k (X_k - Y_k)),
//     z_s = sum_{k<h} Z_k exp(+2 pi i s k / h),  Re D[2s] = Re z_s,  Re D[2s+1] = Im z_s.
// One thread lifts the four inputs of a pair (k, h-k); half the LDS (two workgroups per CU) and half the flops of
// the full-length form.  The factor 1/2 of X and Y goes into the final scale.
template <int LOGN, int LEVEL>
__global__ void __launch_bounds__(FftPlan<LOGN - 2>::NT)
k_decode_h(RingDev rg, CrtArgs ca, MaskDev mk, const uint32_t* __restrict__ d, uint64_t first_ct,
           float* __restrict__ w_out, double* __restrict__ slots_out) {
  constexpr int LOGh = LOGN - 2, h = 1 << LOGh, n = 2 * h, N = 4 * h;
  using P = FftPlan<LOGh>;
  extern __shared__ double lds_d[];
  double* re = lds_d;
  double* im = lds_d + h;
  const uint64_t c_local = blockIdx.x;
  const uint32_t* dc = d + c_local * LEVEL * N;
  const double2* e_tab = rg.fft_e;  // exp(-2 pi i r / n), r < h
  const double2* twist = rg.twist;
  auto ldl = [=](int a, double& r, double& i) { r = re[fswz<LOGh>(a)]; i = im[fswz<LOGh>(a)]; };
  auto stl = [=](int a, double r, double i) { re[fswz<LOGh>(a)] = r; im[fswz<LOGh>(a)] = i; };
  auto lift = [&](int k, double& r, double& i) {  // d_k
    uint32_t ra[LEVEL], rb[LEVEL];
#pragma unroll
    for (int j = 0; j < LEVEL; ++j) {
      ra[j] = dc[(size_t)j * N + k];
      rb[j] = dc[(size_t)j * N + k + n];
    }
    const double vr = crt_centered<LEVEL>(rg, ca, ra);
    const double vi = crt_centered<LEVEL>(rg, ca, rb);
    const double2 tw = twist[k];
    r = vr * tw.x - vi * tw.y;
    i = vr * tw.y + vi * tw.x;
  };
  static_assert((h / 2) % P::NT == 0, "whole iterations over the pairs");
  for (int k = threadIdx.x; k < h / 2; k += P::NT) {
    // pair (k, h-k); k = 0 stands for the two self-paired indices 0 and h/2
    const int ka = k, kb = k ? h - k : h / 2;
    double ar, ai, br, bi, cr, ci, er, ei;
    lift(ka, ar, ai);                       // d_k
    lift((n - ka) & (n - 1), br, bi);       // d_{n-k}
    if (k) {
      lift(h - k, cr, ci);                  // d_{h-k}
      lift(h + k, er, ei);                  // d_{h+k}
    } else {
      lift(h / 2, cr, ci);                  // second self-pair: d_{h/2} and d_{3h/2}
      lift(h + h / 2, er, ei);
    }
    if (k) {
      const double xr = ar + br, xi = ai - bi;            // 2 X_k
      const double yr = cr + er, yi = ei - ci;            // 2 Y_k
      const double sr = xr + yr, si = xi + yi;            // 2 (X + Y)
      const double dr = xr - yr, di = xi - yi;            // 2 (X - Y)
      const double2 w = e_tab[k];                         // conj(w^k)
      const double tr = dr * w.x + di * w.y, ti = di * w.x - dr * w.y;   // 2 w^k (X - Y)
      stl(ka, sr - ti, si + tr);                          // S + i T
      stl(kb, sr + ti, tr - si);                          // conj S + i conj T
    } else {
      // k = 0: d_{n-0} = d_0 and d_{h-0} = d_{h+0} = d_h (here: a = b = d_0 is loaded twice; c, e are the second pair)
      double hr, hi;
      lift(h, hr, hi);                                    // d_h
      stl(0, 2.0 * (ar + hr), 2.0 * (ar - hr));           // Z_0 = (Re d_0 + Re d_h) + i (Re d_0 - Re d_h), doubled
      // Z_{h/2}: X = (d_{h/2} + conj d_{3h/2}) / 2, S = 2 Re X, T = -2 Im X, doubled like the rest
      stl(h / 2, 2.0 * (cr + er), -2.0 * (ci - ei));
    }
  }
  __syncthreads();
  fft_pass<LOGh, 0, false, true, 1>(e_tab, ldl, stl);
  __syncthreads();
  fft_pass<LOGh, 1, false, true, 1>(e_tab, ldl, stl);
  __syncthreads();
  fft_pass<LOGh, 2, false, true, 1>(e_tab, ldl, stl);
  __syncthreads();
  fft_pass<LOGh, 3, false, true, 1>(e_tab, ldl, stl);
  __syncthreads();
  static_assert(P::kPasses == 4, "plans of the half-length transforms have four passes");
  const double scale = ldexp(1.0, -(int)rg.scale_bits - 1);  // 1 / Delta and the 1/2 of X, Y
  uint32_t r_lo = 0, r_hi = 0;
  const uint64_t c = first_ct + c_local;
  if (!slots_out) {
    r_lo = run_find(mk.prefix, mk.n_runs, c * (uint64_t)n);
    r_hi = run_find(mk.prefix, mk.n_runs, min((c + 1) * (uint64_t)n, mk.P_enc) - 1);
  }
  for (int j = threadIdx.x; j < n; j += P::NT) {
    const uint32_t code = rg.perm_half[j];  // (bitrev(bin >> 1) << 1) | (bin & 1): bin 2s at Re z_s, bin 2s+1 at Im z_s
    const double z = ((code & 1) ? im : re)[fswz<LOGh>((int)(code >> 1))] * scale;
    if (slots_out) {
      slots_out[c_local * n + j] = z;
    } else {
      const uint64_t t = c * (uint64_t)n + (uint64_t)j;
      if (t < mk.P_enc) w_out[run_lookup_ct(mk, r_lo, r_hi, t)] = (float)z;
    }
  }
}

// ---- plaintext remainder: compaction (client, before sending) and scatter (after) -------
// A workgroup moves kMoveChunk consecutive compacted positions; lanes take consecutive positions
// so both sides are unit-stride streams inside a run.
constexpr uint32_t kMoveChunk = 256 * 16;
typedef float v4f_a16 __attribute__((ext_vector_type(4)));               // 16-byte aligned
typedef float v4f_a4 __attribute__((ext_vector_type(4), aligned(4)));    // element-aligned only

// VEC: the compacted buffer is 16-byte aligned, so a thread moves 4 consecutive compacted
// positions with one 16-byte access on each side when they fall into one run (the model side
// is then only 4-byte aligned, which the hardware's unaligned access mode handles).
template <bool SCATTER, bool VEC>
__global__ void __launch_bounds__(256)
k_plain_move(MaskDev mk, const float* __restrict__ src, float* __restrict__ dst) {
  const uint64_t n_plain = mk.P - mk.P_enc;
  const uint64_t t0 = (uint64_t)blockIdx.x * kMoveChunk;
  const uint64_t t1 = min(t0 + kMoveChunk, n_plain);
  if (t0 >= t1) return;
  const uint32_t lo = run_find(mk.cprefix, mk.n_cruns, t0);
  const uint32_t hi = run_find(mk.cprefix, mk.n_cruns, t1 - 1);
  if (VEC && lo == hi && t1 - t0 == kMoveChunk) {
    // The whole chunk lies in one run (all but a few chunks of a block-structured mask): a shifted copy, the four
    // 16-byte loads of a thread issued before its stores.
    const uint64_t shift = mk.cstart[lo] - mk.cprefix[lo];  // model index = compacted position + shift
    const float* model_in = SCATTER ? nullptr : src + shift;
    float* model_out = SCATTER ? dst + shift : nullptr;
    v4f_a16 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint64_t t = t0 + 4 * ((uint64_t)threadIdx.x + 256 * k);
      if (SCATTER) v[k] = __builtin_nontemporal_load(reinterpret_cast<const v4f_a16*>(src + t));
      else v[k] = __builtin_nontemporal_load(reinterpret_cast<const v4f_a4*>(model_in + t));
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint64_t t = t0 + 4 * ((uint64_t)threadIdx.x + 256 * k);
      if (SCATTER) *reinterpret_cast<v4f_a4*>(model_out + t) = v[k];
      else __builtin_nontemporal_store(v[k], reinterpret_cast<v4f_a16*>(dst + t));
    }
    return;
  }
  if (VEC) {
#pragma unroll 4
    for (uint64_t t = t0 + 4 * (uint64_t)threadIdx.x; t < t1; t += 4 * 256) {
      const uint32_t r = run_find_in(mk.cprefix, lo, hi, t);
      const uint64_t idx = mk.cstart[r] + (t - mk.cprefix[r]);
      if (t + 4 <= t1 && t + 4 <= mk.cprefix[r + 1]) {  // 4 positions, one run
        if (SCATTER) *reinterpret_cast<v4f_a4*>(dst + idx) = __builtin_nontemporal_load(reinterpret_cast<const v4f_a16*>(src + t));
        else __builtin_nontemporal_store(*reinterpret_cast<const v4f_a4*>(src + idx), reinterpret_cast<v4f_a16*>(dst + t));
      } else {
        for (uint64_t e = t; e < min(t + 4, t1); ++e) {
          const uint64_t ie = run_lookup_in(mk.cstart, mk.cprefix, r, hi, e);
          if (SCATTER) dst[ie] = src[e];
          else dst[e] = src[ie];
        }
      }
    }
  } else {
#pragma unroll 4
    for (uint64_t t = t0 + threadIdx.x; t < t1; t += 256) {
      const uint64_t idx = run_lookup_in(mk.cstart, mk.cprefix, lo, hi, t);
      if (SCATTER) dst[idx] = src[t];
      else dst[t] = src[idx];
    }
  }
}

// ---- the same two moves under a FRAGMENTED mask ------------------------------------------------
// When the complement of the mask comes in runs of a few parameters (a top-p selection over per-parameter
// sensitivities), a position-ordered walk pays a run lookup per 16 bytes.  These kernels go through the model in
// PARAMETER order instead: a workgroup takes kBitChunk consecutive parameters, a thread 16 of them with their 16 mask
// bits; the compacted position of an unmasked parameter is the chunk's offset (cchunk) + an exclusive scan of the
// threads' counts + its rank among the thread's bits.  The model side is a plain unit-stride stream whatever the
// mask looks like (masked parameters are read and dropped).

// bits from the run list: one thread per 32-bit word; parameters at and beyond P count as masked.
__global__ void __launch_bounds__(256)
k_mask_bits(const uint64_t* __restrict__ start, const uint64_t* __restrict__ prefix, uint32_t n_runs, uint64_t P,
            uint64_t n_words, uint32_t* __restrict__ bits) {
  const uint64_t wd = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (wd >= n_words) return;
  const uint64_t i0 = wd * 32;
  uint32_t out = 0;
  if (i0 >= P) {
    out = 0xFFFFFFFFu;
  } else {
    // first run that ends after i0 (runs are sorted by start; run r covers [start[r], start[r] + prefix[r+1] - prefix[r]))
    uint32_t a = 0, b = n_runs;  // answer in [a, b]; b == n_runs means none
    while (a < b) {
      const uint32_t mid = (a + b) >> 1;
      const uint64_t end = start[mid] + (prefix[mid + 1] - prefix[mid]);
      if (end > i0) b = mid;
      else a = mid + 1;
    }
    for (uint32_t r = a; r < n_runs; ++r) {
      const uint64_t s0 = start[r];
      if (s0 >= i0 + 32) break;
      const uint64_t e0 = s0 + (prefix[r + 1] - prefix[r]);
      const uint32_t lo = s0 > i0 ? (uint32_t)(s0 - i0) : 0u, hi = e0 < i0 + 32 ? (uint32_t)(e0 - i0) : 32u;  // bits [lo, hi)
      const uint32_t m_hi = hi >= 32 ? 0xFFFFFFFFu : ((1u << hi) - 1u);
      out |= m_hi & ~((1u << lo) - 1u);
    }
    if (P - i0 < 32) out |= ~((1u << (uint32_t)(P - i0)) - 1u);
  }
  bits[wd] = out;
}

// ptab[k] = masked run that holds packed position 64 k; entries at and beyond P_enc: the last run
__global__ void __launch_bounds__(256)
k_mask_ptab(const uint64_t* __restrict__ prefix, uint32_t n_runs, uint64_t P_enc, uint64_t n_entries, uint32_t* __restrict__ ptab) {
  const uint64_t k = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (k >= n_entries) return;
  ptab[k] = 64 * k < P_enc ? run_find(prefix, n_runs, 64 * k) : n_runs - 1;
}

// unmasked parameters per chunk of kBitChunk (128 words): one wavefront per chunk
__global__ void __launch_bounds__(64)
k_chunk_unmasked(const uint32_t* __restrict__ bits, uint32_t* __restrict__ counts) {
  const uint32_t* w = bits + (uint64_t)blockIdx.x * (kBitChunk / 32);
  uint32_t c = __popc(~w[threadIdx.x]) + __popc(~w[threadIdx.x + 64]);
  for (int d = 32; d > 0; d >>= 1) c += __shfl_down(c, d, 64);
  if (threadIdx.x == 0) counts[blockIdx.x] = c;
}

template <bool SCATTER>
__global__ void __launch_bounds__(256)
k_plain_move_bits(MaskDev mk, const float* __restrict__ src, float* __restrict__ dst) {
  // The chunk's unmasked values pass through LDS in compacted order, so that the compacted side is read / written with
  // consecutive lanes on consecutive words; the model side moves 16 bytes per lane (scalar where a quad has a masked one).
  __shared__ float stage[kBitChunk];
  const uint64_t chunk = blockIdx.x;
  const uint32_t word = mk.bits[chunk * (kBitChunk / 32) + (threadIdx.x >> 1)];
  const uint32_t um = ~(word >> (16 * (threadIdx.x & 1))) & 0xFFFFu;  // this thread's 16 parameters: bit set = unmasked
  uint32_t total;
  uint32_t r = he_sel::block_exclusive_scan((uint32_t)__popc(um), &total);  // rank of the thread's first unmasked one
  if (total == 0) return;  // uniform: every thread sees the same total
  const uint64_t cbase = mk.cchunk[chunk];                              // compacted position of the chunk's first one
  const uint64_t i0 = chunk * kBitChunk + (uint64_t)threadIdx.x * 16;  // the thread's first parameter
  if (!SCATTER) {
    const float* model = src + i0;
    float x[16];
    if (i0 + 16 <= mk.P && (reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const v4f_a16 q4 = __builtin_nontemporal_load(reinterpret_cast<const v4f_a16*>(model) + v);
        x[4 * v] = q4.x; x[4 * v + 1] = q4.y; x[4 * v + 2] = q4.z; x[4 * v + 3] = q4.w;
      }
    } else {
#pragma unroll
      for (int b = 0; b < 16; ++b) x[b] = ((um >> b) & 1u) ? model[b] : 0.f;  // unmasked bits are below P
    }
#pragma unroll
    for (int b = 0; b < 16; ++b)
      if ((um >> b) & 1u) stage[r++] = x[b];
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < total; j += 256) __builtin_nontemporal_store(stage[j], dst + cbase + j);
  } else {
    for (uint32_t j = threadIdx.x; j < total; j += 256) stage[j] = __builtin_nontemporal_load(src + cbase + j);
    __syncthreads();
    float* model = dst + i0;
    const bool wide = (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const uint32_t quad = (um >> (4 * v)) & 0xFu;
      if (quad == 0xFu && wide) {
        v4f_a16 q4;
        q4.x = stage[r]; q4.y = stage[r + 1]; q4.z = stage[r + 2]; q4.w = stage[r + 3];
        *(reinterpret_cast<v4f_a16*>(model) + v) = q4;
        r += 4;
      } else {
#pragma unroll
        for (int b = 0; b < 4; ++b)
          if ((quad >> b) & 1u) model[4 * v + b] = stage[r++];
      }
    }
  }
}

// Both halves of a model vector in one pass (encrypt side of a fragmented mask): the unmasked parameters go to the
// compacted remainder, the masked ones to the packed slot vector that the encoder then reads as a plain array.  Same
// walk as k_plain_move_bits; the masked values fill the staging array from its end.  MERGE is the inverse (decrypt side):
// the decoded slot vector and the aggregated remainder are woven back into the model, every parameter written once.
template <bool MERGE>
__global__ void __launch_bounds__(256)
k_split_bits(MaskDev mk, const float* __restrict__ model_in, float* __restrict__ model_out, const float* __restrict__ packed_in,
             float* __restrict__ packed_out, const float* __restrict__ plain_in, float* __restrict__ plain_out) {
  __shared__ float stage[kBitChunk];
  const uint64_t chunk = blockIdx.x;
  const uint64_t i0 = chunk * kBitChunk + (uint64_t)threadIdx.x * 16;  // the thread's first parameter
  const uint32_t word = mk.bits[chunk * (kBitChunk / 32) + (threadIdx.x >> 1)];
  const uint32_t half = (word >> (16 * (threadIdx.x & 1))) & 0xFFFFu;
  const uint32_t valid = i0 >= mk.P ? 0u : (mk.P - i0 >= 16 ? 0xFFFFu : ((1u << (uint32_t)(mk.P - i0)) - 1u));
  const uint32_t um = ~half & 0xFFFFu, mm = half & valid;  // unmasked / masked among the thread's parameters (padding is neither)
  uint32_t totals;
  const uint32_t excl = he_sel::block_exclusive_scan((uint32_t)__popc(um) | ((uint32_t)__popc(mm) << 16), &totals);  // both counts <= 4096
  uint32_t ru = excl & 0xFFFFu, rm = excl >> 16;
  const uint32_t total_u = totals & 0xFFFFu, total_m = totals >> 16;
  const uint64_t cbase = mk.cchunk[chunk], mbase = chunk * kBitChunk - cbase;  // every parameter before the chunk is below P
  const bool wide = i0 + 16 <= mk.P && (reinterpret_cast<uintptr_t>(MERGE ? (const void*)model_out : (const void*)model_in) & 15u) == 0;
  if (!MERGE) {
    float x[16];
    if (wide) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const v4f_a16 q4 = __builtin_nontemporal_load(reinterpret_cast<const v4f_a16*>(model_in + i0) + v);
        x[4 * v] = q4.x; x[4 * v + 1] = q4.y; x[4 * v + 2] = q4.z; x[4 * v + 3] = q4.w;
      }
    } else {
#pragma unroll
      for (int b = 0; b < 16; ++b) x[b] = ((valid >> b) & 1u) ? model_in[i0 + b] : 0.f;
    }
#pragma unroll
    for (int b = 0; b < 16; ++b) {
      if ((um >> b) & 1u) stage[ru++] = x[b];
      else if ((mm >> b) & 1u) stage[kBitChunk - 1 - rm++] = x[b];
    }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < total_u; j += 256) __builtin_nontemporal_store(stage[j], plain_out + cbase + j);
    for (uint32_t j = threadIdx.x; j < total_m; j += 256) packed_out[mbase + j] = stage[kBitChunk - 1 - j];  // read again soon: keep in L2
  } else {
    for (uint32_t j = threadIdx.x; j < total_u; j += 256) stage[j] = __builtin_nontemporal_load(plain_in + cbase + j);
    for (uint32_t j = threadIdx.x; j < total_m; j += 256) stage[kBitChunk - 1 - j] = packed_in[mbase + j];
    __syncthreads();
    float x[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) {
      x[b] = 0.f;
      if ((um >> b) & 1u) x[b] = stage[ru++];
      else if ((mm >> b) & 1u) x[b] = stage[kBitChunk - 1 - rm++];
    }
    if (wide) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        v4f_a16 q4;
        q4.x = x[4 * v]; q4.y = x[4 * v + 1]; q4.z = x[4 * v + 2]; q4.w = x[4 * v + 3];
        *(reinterpret_cast<v4f_a16*>(model_out + i0) + v) = q4;
      }
    } else {
#pragma unroll
      for (int b = 0; b < 16; ++b)
        if ((valid >> b) & 1u) model_out[i0 + b] = x[b];
    }
  }
}

template <bool SCATTER>
void launch_plain_move(const MaskDev& mk, const float* src, float* dst, hipStream_t st) {
  if (mk.bits) {
    const uint64_t n_pchunks = (mk.P + kBitChunk - 1) / kBitChunk;
    hipLaunchKernelGGL((k_plain_move_bits<SCATTER>), dim3((uint32_t)n_pchunks), dim3(256), 0, st, mk, src, dst);
    return;
  }
  const uint64_t n_plain = mk.P - mk.P_enc;
  const dim3 grid((uint32_t)((n_plain + kMoveChunk - 1) / kMoveChunk)), block(256);
  const bool aligned = reinterpret_cast<uintptr_t>(SCATTER ? (const void*)src : (const void*)dst) % 16 == 0;
  if (aligned) hipLaunchKernelGGL((k_plain_move<SCATTER, true>), grid, block, 0, st, mk, src, dst);
  else hipLaunchKernelGGL((k_plain_move<SCATTER, false>), grid, block, 0, st, mk, src, dst);
}

// ---- a5 + a6: sum_i w_i ct_i (mod q_j) over clients, then rescale by q_{L-1} ---------------
// One thread owns 4 consecutive coefficients of one (ciphertext, poly) in all L limbs.
// Products w*x < 2^62 are accumulated in 64 bits and folded back below q every 4 terms.
__device__ __forceinline__ uint32_t reduce64(uint64_t x, uint2 c32, uint32_t q) {
  const uint32_t hi = (uint32_t)(x >> 32), lo = (uint32_t)x;
  const uint32_t t = mul_shoup(hi, c32, q);          // hi * 2^32 mod q
  return add_mod(t, csub(csub(lo, q), q), q);        // lo < 2^32 < 3q
}

// Ciphertext streams are touched exactly once: mark them non-temporal so they do not displace
// what other kernels keep in L2.
__device__ __forceinline__ uint4 stream_load(const uint4* p) {
  typedef uint32_t v4u __attribute__((ext_vector_type(4)));
  const v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void stream_store(uint4* p, uint4 v) {
  typedef uint32_t v4u __attribute__((ext_vector_type(4)));
  v4u t;
  t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
  __builtin_nontemporal_store(t, reinterpret_cast<v4u*>(p));
}

template <int L, bool HAS_ACC, bool FINAL>
__global__ void __launch_bounds__(256)
k_aggregate(AggArgs a, AggConst k, uint32_t log_n4, uint64_t n_vec, const uint4* acc_in, uint4* out) {
  // acc_in and out may be the same buffer (in-place accumulation): a thread reads and writes only its own elements.
  const uint64_t gid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= n_vec) return;
  const uint64_t cp = gid >> log_n4;                 // ciphertext * 2 + poly
  const uint64_t kk = gid & ((1ull << log_n4) - 1);  // which group of 4 coefficients
  uint32_t res[L][4];
  if constexpr (L <= 4) {
    // Short chains: the L limb loads of four clients are issued together (16 L x 16 B in flight per thread instead
    // of 16 B, at 5 waves per SIMD: 5.9 -> 6.3 TB/s at K = 8, L = 4); longer chains would not keep L accumulators
    // in registers and go limb by limb, client by client.
    uint64_t acc[L][4];
#pragma unroll
    for (int j = 0; j < L; ++j) {
      const uint64_t off = ((cp * L + j) << log_n4) + kk;
      if (HAS_ACC) {
        const uint4 v = acc_in[off];
        acc[j][0] = v.x; acc[j][1] = v.y; acc[j][2] = v.z; acc[j][3] = v.w;
      } else {
        acc[j][0] = acc[j][1] = acc[j][2] = acc[j][3] = 0;
      }
    }
    uint32_t i = 0;
    constexpr int CB = 4;  // clients whose loads are in flight together (2, 4 and 8 measured alike, 1 slower)
    for (; i + CB <= a.K; i += CB) {
      uint4 x[CB][L];
#pragma unroll
      for (int c2 = 0; c2 < CB; ++c2)
#pragma unroll
        for (int j = 0; j < L; ++j) x[c2][j] = stream_load(reinterpret_cast<const uint4*>(a.ct[i + c2]) + (((cp * L + j) << log_n4) + kk));
#pragma unroll
      for (int c2 = 0; c2 < CB; ++c2) {
#pragma unroll
        for (int j = 0; j < L; ++j) {
          const uint64_t w = a.w[i + c2][j];
          acc[j][0] += w * x[c2][j].x; acc[j][1] += w * x[c2][j].y; acc[j][2] += w * x[c2][j].z; acc[j][3] += w * x[c2][j].w;
        }
        if (((i + c2) & 3) == 3) {
#pragma unroll
          for (int j = 0; j < L; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][e] = reduce64(acc[j][e], k.c32[j], k.q[j]);
        }
      }
    }
    for (; i < a.K; ++i) {
      uint4 x[L];
#pragma unroll
      for (int j = 0; j < L; ++j) x[j] = stream_load(reinterpret_cast<const uint4*>(a.ct[i]) + (((cp * L + j) << log_n4) + kk));
#pragma unroll
      for (int j = 0; j < L; ++j) {
        const uint64_t w = a.w[i][j];
        acc[j][0] += w * x[j].x; acc[j][1] += w * x[j].y; acc[j][2] += w * x[j].z; acc[j][3] += w * x[j].w;
      }
      if ((i & 3) == 3) {
#pragma unroll
        for (int j = 0; j < L; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[j][e] = reduce64(acc[j][e], k.c32[j], k.q[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < L; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) res[j][e] = reduce64(acc[j][e], k.c32[j], k.q[j]);
      if (!FINAL) out[((cp * L + j) << log_n4) + kk] = make_uint4(res[j][0], res[j][1], res[j][2], res[j][3]);
    }
  } else {
#pragma unroll
    for (int j = L - 1; j >= 0; --j) {
      const uint64_t off = ((cp * L + j) << log_n4) + kk;
      const uint32_t q = k.q[j];
      uint64_t acc[4] = {0, 0, 0, 0};
      if (HAS_ACC) {
        const uint4 v = acc_in[off];
        acc[0] = v.x; acc[1] = v.y; acc[2] = v.z; acc[3] = v.w;
      }
      // One client at a time: batching 2 or 4 clients' loads per thread measured 2-3 % slower (the stream is
      // HBM-limited, occupancy supplies the loads in flight).
      for (uint32_t i = 0; i < a.K; ++i) {
        const uint4 x = stream_load(reinterpret_cast<const uint4*>(a.ct[i]) + off);
        const uint64_t w = a.w[i][j];
        acc[0] += w * x.x; acc[1] += w * x.y; acc[2] += w * x.z; acc[3] += w * x.w;
        if ((i & 3) == 3) {
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[e] = reduce64(acc[e], k.c32[j], q);
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) res[j][e] = reduce64(acc[e], k.c32[j], q);
      if (!FINAL) out[off] = make_uint4(res[j][0], res[j][1], res[j][2], res[j][3]);
    }
  }
  if (FINAL) {
#pragma unroll
    for (int j = 0; j < L - 1; ++j) {
      const uint32_t q = k.q[j];
      uint32_t o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t r = res[L - 1][e];
        const uint32_t rj = r > k.half_last ? r + k.qdiff[j] : r;  // centred residue, reduced mod q_j
        o[e] = mul_shoup(sub_mod(res[j][e], rj, q), k.qlinv[j], q);
      }
      stream_store(out + (((cp * (L - 1) + j) << log_n4) + kk), make_uint4(o[0], o[1], o[2], o[3]));
    }
  }
}

// ---- a7: plain FedAvg of the unmasked remainder -------------------------------------------
// acc <- acc + alpha_i * w_i in float64, product and sum rounded separately, client order.
// VEC = 4: one thread owns 4 consecutive parameters (16-byte loads; all client pointers and
// the outputs must be 16-byte aligned); the tail and unaligned calls use VEC = 1.
template <bool HAS_ACC, bool FINAL, int VEC>
__global__ void __launch_bounds__(256)
k_plain_fedavg(PlainArgs a, uint64_t first, uint64_t n_groups, const double* acc_in, double* acc_out, float* out) {
  // acc_in / acc_out, and out / a client's input, may be the same buffer: a thread reads and writes only its own elements.
  // The product and the sum must round separately (no fused multiply-add), or the result
  // depends on the compiler's contraction choices.
#pragma clang fp contract(off)
  const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  const uint64_t t = first + g * VEC;
  double acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = HAS_ACC ? acc_in[t + e] : 0.0;
  for (uint32_t i = 0; i < a.K; ++i) {
    const double al = a.alpha[i];
    float x[VEC];
    if (VEC == 4) {
      typedef float v4f __attribute__((ext_vector_type(4)));
      const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(a.w[i] + t));
      x[0] = v.x; x[1 % VEC] = v.y; x[2 % VEC] = v.z; x[3 % VEC] = v.w;
    } else {
      x[0] = a.w[i][t];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const double prod = al * (double)x[e];
      acc[e] = acc[e] + prod;
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    if (FINAL) out[t + e] = (float)acc[e];
    else acc_out[t + e] = acc[e];
  }
}

__global__ void __launch_bounds__(256) k_fill_u32(uint32_t* p, uint64_t n, uint32_t v) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += stride) p[t] = v;
}

// ---- standalone batched transform (debug export, key generation) ------------------------
// limb < 0: polynomial b uses limb b % L (for [..][L][N] layouts).
template <bool INV>
__global__ void __launch_bounds__(1024)
k_ntt_batch(RingDev rg, int limb, uint32_t* __restrict__ polys) {
  extern __shared__ uint32_t lds_u[];
  const int logN = (int)rg.logN;
  const uint32_t N = rg.N;
  const uint32_t j = limb >= 0 ? (uint32_t)limb : (uint32_t)(blockIdx.x % rg.L);
  const uint32_t q = rg.q[j];
  uint32_t* x = polys + (size_t)blockIdx.x * N;
  uint32_t* buf = lds_u;
  if (!INV) {
    ntt_forward_to_lds(buf, logN, rg.tw_fwd + (size_t)j * N, q, [=](int a) { return x[a]; });
    for (uint32_t a = threadIdx.x; a < N; a += blockDim.x) x[a] = buf[lds_pad((int)a)];
  } else {
    const uint2 ninv = rg.ninv[j];
    ntt_inverse_from(
        buf, logN, rg.tw_inv + (size_t)j * N, q, [=](int a) { return x[a]; },
        [=](int a, uint32_t v) { x[a] = mul_shoup(v, ninv, q); });
  }
}

// ---- key generation ---------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_keygen_sample(RingDev rg, uint2 key, int8_t* __restrict__ s_coeff, uint32_t* __restrict__ s_res,
                uint32_t* __restrict__ e_res, uint32_t* __restrict__ a_res) {
  const uint32_t kidx = blockIdx.x * blockDim.x + threadIdx.x;
  if (kidx >= rg.N) return;
  const RngKey rk{key, 0u, 0u};
  const uint32_t mask = rg.eta == 0 ? 0u : cbd_mask(rg.eta);
  const uint4 rs = rng_block(rk, kidx >> 2, kTagS);
  const uint32_t ws[4] = {rs.x, rs.y, rs.z, rs.w};
  const int s = ternary_from_word(ws[kidx & 3]);
  const uint4 re = rng_block(rk, kidx >> 1, kTagEpk);
  const int e = (kidx & 1) ? cbd_from_words(re.z, re.w, mask) : cbd_from_words(re.x, re.y, mask);
  s_coeff[kidx] = (int8_t)s;
  for (uint32_t j = 0; j < rg.L; ++j) {
    const uint32_t q = rg.q[j];
    s_res[(size_t)j * rg.N + kidx] = residue_of_signed(s, q);
    e_res[(size_t)j * rg.N + kidx] = residue_of_signed(e, q);
    const uint4 ra = rng_block(rk, kidx >> 1, kTagA0 + j);
    const uint64_t x = (kidx & 1) ? (((uint64_t)ra.w << 32) | ra.z) : (((uint64_t)ra.y << 32) | ra.x);
    a_res[(size_t)j * rg.N + kidx] = (uint32_t)(x % q);
  }
}

// b^ = e^ - a^ . s^ ; tables premultiplied by 1/N with Shoup companions.
__global__ void __launch_bounds__(256)
k_keygen_combine(RingDev rg, const uint32_t* __restrict__ s_hat, const uint32_t* __restrict__ e_hat,
                 const uint32_t* __restrict__ a_hat, uint32_t* __restrict__ pk_raw, uint2* __restrict__ pk_tab,
                 uint2* __restrict__ sk_tab) {
  const uint32_t kidx = blockIdx.x * blockDim.x + threadIdx.x;
  if (kidx >= rg.N) return;
  const uint32_t N = rg.N, L = rg.L;
  for (uint32_t j = 0; j < L; ++j) {
    const uint32_t q = rg.q[j];
    const size_t o = (size_t)j * N + kidx;
    const uint32_t s = s_hat[o], a = a_hat[o], e = e_hat[o];
    const uint32_t as = (uint32_t)((uint64_t)a * s % q);
    const uint32_t b = sub_mod(e, as, q);
    pk_raw[o] = b;
    pk_raw[(size_t)L * N + o] = a;
    const uint32_t bn = mul_shoup(b, rg.ninv[j], q), an = mul_shoup(a, rg.ninv[j], q), sn = mul_shoup(s, rg.ninv[j], q);
    pk_tab[o] = make_uint2(bn, (uint32_t)(((uint64_t)bn << 32) / q));
    pk_tab[(size_t)L * N + o] = make_uint2(an, (uint32_t)(((uint64_t)an << 32) / q));
    sk_tab[o] = make_uint2(sn, (uint32_t)(((uint64_t)sn << 32) / q));
  }
}

__global__ void __launch_bounds__(256) k_widen_i8(const int8_t* __restrict__ in, int32_t* __restrict__ out, uint32_t n) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = in[i];
}

// Counts the parameters the encoder cannot carry: not finite, or |x| * Delta >= 2^31 - 32 (m + e0 would leave int32).
__global__ void __launch_bounds__(256)
k_count_out_of_range(const float* __restrict__ w, uint64_t n, double delta, unsigned long long* __restrict__ count) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  uint32_t bad = 0;
  for (uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += stride) {
    const double x = (double)w[t];
    if (!(fabs(x) * delta < 2147483616.0)) ++bad;  // exact in float64; NaN compares false: counted
  }
  for (int d = 32; d > 0; d >>= 1) bad += __shfl_down(bad, d, 64);
  if ((threadIdx.x & 63) == 0 && bad) atomicAdd(count, (unsigned long long)bad);
}

// Counts the words of ciphertext rows [rows][N] (row r belongs to limb r % level) that are not below their prime.
__global__ void __launch_bounds__(256)
k_count_noncanonical(RingDev rg, const uint32_t* __restrict__ ct, uint64_t n_words, uint32_t level,
                     unsigned long long* __restrict__ count) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  uint32_t bad = 0;
  for (uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n_words; t += stride) {
    const uint32_t j = (uint32_t)((t >> rg.logN) % level);
    if (ct[t] >= rg.q[j]) ++bad;
  }
  for (int d = 32; d > 0; d >>= 1) bad += __shfl_down(bad, d, 64);
  if ((threadIdx.x & 63) == 0 && bad) atomicAdd(count, (unsigned long long)bad);
}

// =========================================================================================
// Host side
// =========================================================================================

thread_local std::string g_last_error;

he_status fail(he_status code, const std::string& msg) {
  g_last_error = msg;
  return code;
}

// No exception leaves the library: host containers may throw std::bad_alloc, which every entry point turns into
// HE_ERR_NOMEM (the message fits the string's inline buffer, so setting it allocates nothing).
he_status on_exception() {
  try {
    g_last_error.assign("out of memory");
  } catch (...) {
  }
  return HE_ERR_NOMEM;
}

#define HIP_TRY(expr)                                                                         \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      return fail(e_ == hipErrorOutOfMemory ? HE_ERR_NOMEM : HE_ERR_HIP,                      \
                  std::string(#expr) + ": " + hipGetErrorString(e_));                         \
  } while (0)

constexpr uint64_t kCtChunk = 2048;  // ciphertexts per scratch chunk (m+e0, u, e1: 192 MiB at N = 2^14)

}  // namespace

// Scratch of he_encrypt_masked_static, the entry point for callers that cannot allocate: part of the code object, so
// every GPU the library runs on holds its own copy from module load to process end.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels, memsets and copies get the per-device address kept in g_static_scratch.
static __device__ __align__(256) unsigned char scratch[HE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices] = {};  // device address of `scratch` on each GPU, resolved by he_ctx_create
}  // namespace

enum KernelId : int {
  KID_ENCODE = 0, KID_SAMPLE, KID_ENCRYPT, KID_AGGREGATE, KID_PLAIN_FEDAVG, KID_DECRYPT, KID_DECODE, KID_PLAIN_MOVE,
  KID_NTT, KID_COUNT
};
static const char* const kKernelNames[KID_COUNT] = {"encode", "sample", "encrypt", "aggregate", "plain_fedavg",
                                                    "decrypt", "decode", "plain_move", "ntt"};

struct TimedSpan {
  int kid;
  hipEvent_t start, stop;
};

struct he_ctx {
  bool timing_on = false;
  std::vector<TimedSpan> spans;       // recorded, not yet read
  std::vector<hipEvent_t> event_pool; // recycled events
  int device = 0;
  RingDev ring{};
  std::vector<uint32_t> primes;
  std::vector<void*> dev_allocs;
  AggConst agg{};
  void* ws = nullptr;  // scratch, grown on demand
  size_t ws_bytes = 0;
  void* static_scratch = nullptr;  // this GPU's copy of the file-scope array `scratch`
  int max_lds = 0;
};

struct he_pk {
  he_ctx* ctx;
  uint2* tab;     // [2][L][N] (b^, a^) * 1/N with Shoup companions
  uint32_t* raw;  // [2][L][N] (b^, a^) as they are
};

struct he_sk {
  he_ctx* ctx;
  uint2* tab;     // [L][N] s^ * 1/N with Shoup companions
  int8_t* coeff;  // [N] s in {-1,0,1}
};

struct he_mask {
  he_ctx* ctx;
  MaskDev dev{};
  void* dev_block = nullptr;
  void* bits_block = nullptr;  // bit mask and per-chunk offsets of a fragmented mask (build_mask_bits)
  uint64_t n_runs = 0;
  // host copy of the run list; masks built on the device (he_mask_from_bytes, he_mask_select_top) fetch it on first use
  mutable std::vector<uint64_t> starts, lens;
  mutable bool host_runs_valid = true;
};

namespace {

// Brackets the launches issued during its lifetime with a pair of events on their stream
// when per-kernel timing is enabled (measurement only; no effect otherwise).
class KernelTimer {
 public:
  KernelTimer(he_ctx* ctx, int kid, hipStream_t st) : ctx_(ctx), st_(st) {
    if (!ctx_->timing_on) return;
    span_.kid = kid;
    span_.start = take();
    span_.stop = take();
    live_ = span_.start && span_.stop && hipEventRecord(span_.start, st_) == hipSuccess;
  }
  ~KernelTimer() {
    if (!live_ || hipEventRecord(span_.stop, st_) != hipSuccess) return;
    try {
      ctx_->spans.push_back(span_);
    } catch (...) {  // a destructor must not throw: this span is dropped from the measurement
    }
  }

 private:
  hipEvent_t take() {
    if (!ctx_->event_pool.empty()) {
      hipEvent_t e = ctx_->event_pool.back();
      ctx_->event_pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    return hipEventCreate(&e) == hipSuccess ? e : nullptr;
  }
  he_ctx* ctx_;
  hipStream_t st_;
  TimedSpan span_{};
  bool live_ = false;
};

he_status ensure_ws(he_ctx* ctx, size_t bytes) {
  if (ctx->ws_bytes >= bytes) return HE_OK;
  if (ctx->ws) {
    HIP_TRY(hipDeviceSynchronize());  // earlier launches may still use the old block
    HIP_TRY(hipFree(ctx->ws));
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
  }
  HIP_TRY(hipMalloc(&ctx->ws, bytes));
  ctx->ws_bytes = bytes;
  return HE_OK;
}

template <class T>
he_status upload(he_ctx* ctx, const std::vector<T>& host, const T** dev_out) {
  void* p = nullptr;
  HIP_TRY(hipMalloc(&p, std::max<size_t>(host.size() * sizeof(T), 16)));
  ctx->dev_allocs.push_back(p);
  if (!host.empty()) HIP_TRY(hipMemcpy(p, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
  *dev_out = static_cast<const T*>(p);
  return HE_OK;
}

int ntt_threads(uint32_t N) { return (int)std::min<uint32_t>(1024, std::max<uint32_t>(64, N >> 4)); }
int fft_threads(uint32_t n) { return (int)std::min<uint32_t>(1024, std::max<uint32_t>(64, n >> 2)); }
size_t ntt_lds_bytes(uint32_t N, int bufs) { return (size_t)bufs * lds_pad((int)N) * sizeof(uint32_t); }
size_t fft_lds_bytes(uint32_t n) { return (size_t)2 * n * sizeof(double); }
size_t static_fft_lds_bytes(int logn) { return (size_t)2 * fpad(1 << logn) * sizeof(double); }
size_t static_lds_bytes(int logN, int bufs) { return (size_t)bufs * spad(1 << logN) * sizeof(uint32_t); }

// Batched standalone transform: specialised kernels for the tuned sizes, generic otherwise.
void launch_ntt_batch(const RingDev& rg, bool inverse, int limb, uint32_t* polys, uint32_t batch, hipStream_t st);

template <class K>
he_status allow_lds(K kernel, size_t bytes) {
  HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return HE_OK;
}

uint32_t grid_for(uint64_t n, uint32_t block, uint32_t cap = 1u << 20) {
  return (uint32_t)std::min<uint64_t>(cap, std::max<uint64_t>(1, (n + block - 1) / block));
}

he_status check_ctx(const he_ctx* ctx) {
  if (!ctx) return fail(HE_ERR_INVALID_ARG, "context is null");
  HIP_TRY(hipSetDevice(ctx->device));
  return HE_OK;
}

// ---- shared launch helpers ---------------------------------------------------------------

void launch_ntt_batch(const RingDev& rg, bool inverse, int limb, uint32_t* polys, uint32_t batch, hipStream_t st) {
  const dim3 grid(batch);
  if (rg.logN == 14) {
    if (inverse) hipLaunchKernelGGL((k_ntt_batch_s<14, true>), grid, dim3(NttPlan<14>::NT), static_lds_bytes(14, 1), st, rg, limb, polys);
    else hipLaunchKernelGGL((k_ntt_batch_s<14, false>), grid, dim3(NttPlan<14>::NT), static_lds_bytes(14, 1), st, rg, limb, polys);
  } else if (rg.logN == 13) {
    if (inverse) hipLaunchKernelGGL((k_ntt_batch_s<13, true>), grid, dim3(NttPlan<13>::NT), static_lds_bytes(13, 1), st, rg, limb, polys);
    else hipLaunchKernelGGL((k_ntt_batch_s<13, false>), grid, dim3(NttPlan<13>::NT), static_lds_bytes(13, 1), st, rg, limb, polys);
  } else if (rg.logN == 12) {
    if (inverse) hipLaunchKernelGGL((k_ntt_batch_s<12, true>), grid, dim3(NttPlan<12>::NT), static_lds_bytes(12, 1), st, rg, limb, polys);
    else hipLaunchKernelGGL((k_ntt_batch_s<12, false>), grid, dim3(NttPlan<12>::NT), static_lds_bytes(12, 1), st, rg, limb, polys);
  } else if (rg.logN == 11) {
    if (inverse) hipLaunchKernelGGL((k_ntt_batch_s<11, true>), grid, dim3(NttPlan<11>::NT), static_lds_bytes(11, 1), st, rg, limb, polys);
    else hipLaunchKernelGGL((k_ntt_batch_s<11, false>), grid, dim3(NttPlan<11>::NT), static_lds_bytes(11, 1), st, rg, limb, polys);
  } else {
    if (inverse) hipLaunchKernelGGL(k_ntt_batch<true>, grid, dim3(ntt_threads(rg.N)), ntt_lds_bytes(rg.N, 1), st, rg, limb, polys);
    else hipLaunchKernelGGL(k_ntt_batch<false>, grid, dim3(ntt_threads(rg.N)), ntt_lds_bytes(rg.N, 1), st, rg, limb, polys);
  }
}

// Scratch of one chunk of ciphertexts: plaintext m (int32) and the randomness u, e0, e1 (int8).
struct EncScratch {
  int32_t* m;
  int8_t *u, *e0, *e1;
};
constexpr size_t kEncScratchBytesPerCoeff = 7;

EncScratch carve_enc_scratch(void* ws, uint64_t chunk, size_t N) {
  EncScratch s;
  s.m = static_cast<int32_t*>(ws);
  s.u = reinterpret_cast<int8_t*>(s.m + chunk * N);
  s.e0 = s.u + chunk * N;
  s.e1 = s.e0 + chunk * N;
  return s;
}

// Encode n_ct ciphertexts' slots into m_out; when `rnd` is given, also draw their randomness
// (specialised sizes do it inside the encoder kernel, the generic path with k_sample).
he_status launch_encode(he_ctx* ctx, const MaskDev& mk, const float* w, const float* slots, uint64_t first_ct,
                        uint64_t n_ct, int32_t* m_out, const EncScratch* rnd, uint64_t seed, uint32_t client, hipStream_t st,
                        double pre_scale = 1.0) {
  const RingDev& rg = ctx->ring;
  const uint32_t n = rg.N / 2;
  const uint2 key = make_uint2((uint32_t)seed, (uint32_t)(seed >> 32));
  int8_t* u = rnd ? rnd->u : nullptr;
  int8_t* e0 = rnd ? rnd->e0 : nullptr;
  int8_t* e1 = rnd ? rnd->e1 : nullptr;
  bool sampled = false;
  {
    KernelTimer timer_(ctx, KID_ENCODE, st);
    if (rg.logN == 14) {
      hipLaunchKernelGGL(k_encode_r<14>, dim3((uint32_t)n_ct), dim3(FftPlan<12>::NT), static_fft_lds_bytes(12), st, rg, mk, w, slots,
                         first_ct, m_out, key, client, u, e0, e1, pre_scale);
      sampled = true;
    } else if (rg.logN == 13) {
      hipLaunchKernelGGL(k_encode_r<13>, dim3((uint32_t)n_ct), dim3(FftPlan<11>::NT), static_fft_lds_bytes(11), st, rg, mk, w, slots,
                         first_ct, m_out, key, client, u, e0, e1, pre_scale);
      sampled = true;
    } else if (rg.logN == 12) {
      hipLaunchKernelGGL(k_encode_r<12>, dim3((uint32_t)n_ct), dim3(FftPlan<10>::NT), static_fft_lds_bytes(10), st, rg, mk, w, slots,
                         first_ct, m_out, key, client, u, e0, e1, pre_scale);
      sampled = true;
    } else if (rg.logN == 11) {
      hipLaunchKernelGGL(k_encode_r<11>, dim3((uint32_t)n_ct), dim3(FftPlan<9>::NT), static_fft_lds_bytes(9), st, rg, mk, w, slots,
                         first_ct, m_out, key, client, u, e0, e1, pre_scale);
      sampled = true;
    } else {
      hipLaunchKernelGGL(k_encode, dim3((uint32_t)n_ct), dim3(fft_threads(n)), fft_lds_bytes(n), st, rg, mk, w, slots, first_ct, m_out,
                         pre_scale);
    }
  }
  HIP_TRY(hipGetLastError());
  if (rnd && !sampled) {
    KernelTimer timer_(ctx, KID_SAMPLE, st);
    hipLaunchKernelGGL(k_sample, dim3((uint32_t)n_ct), dim3(256), 0, st, rg, key, client, first_ct, rnd->u, rnd->e0, rnd->e1);
    HIP_TRY(hipGetLastError());
  }
  return HE_OK;
}

he_status launch_sample(he_ctx* ctx, uint64_t seed, uint32_t client, uint64_t first_ct, uint64_t n_ct, const EncScratch& rnd,
                        hipStream_t st) {
  const uint2 key = make_uint2((uint32_t)seed, (uint32_t)(seed >> 32));
  KernelTimer timer_(ctx, KID_SAMPLE, st);
  hipLaunchKernelGGL(k_sample, dim3((uint32_t)n_ct), dim3(256), 0, st, ctx->ring, key, client, first_ct, rnd.u, rnd.e0, rnd.e1);
  HIP_TRY(hipGetLastError());
  return HE_OK;
}

he_status launch_encrypt(he_ctx* ctx, const he_pk* pk, uint64_t n_ct, const int32_t* m, const EncScratch& rnd, uint32_t* ct_out,
                         hipStream_t st) {
  const RingDev& rg = ctx->ring;
  KernelTimer timer_(ctx, KID_ENCRYPT, st);
  const dim3 grid(rg.L, (uint32_t)n_ct);
  // XCD-aware linear grid, see k_encrypt_s: 8 ciphertexts (one per XCD) x L limbs per group of 8 L workgroups
  const dim3 grid_x((uint32_t)((n_ct + 7) / 8) * 8 * rg.L);
  if (rg.logN == 14)
    hipLaunchKernelGGL(k_encrypt_s<14>, grid_x, dim3(NttPlan<14>::NT), static_lds_bytes(14, 1), st, rg, pk->tab, rnd.u, m, rnd.e0, rnd.e1,
                       ct_out, (uint32_t)n_ct);
  else if (rg.logN == 13)
    hipLaunchKernelGGL(k_encrypt_s<13>, grid_x, dim3(NttPlan<13>::NT), static_lds_bytes(13, 1), st, rg, pk->tab, rnd.u, m, rnd.e0, rnd.e1,
                       ct_out, (uint32_t)n_ct);
  else if (rg.logN == 12)
    hipLaunchKernelGGL(k_encrypt_s<12>, grid_x, dim3(NttPlan<12>::NT), static_lds_bytes(12, 1), st, rg, pk->tab, rnd.u, m, rnd.e0, rnd.e1,
                       ct_out, (uint32_t)n_ct);
  else if (rg.logN == 11)
    hipLaunchKernelGGL(k_encrypt_s<11>, grid_x, dim3(NttPlan<11>::NT), static_lds_bytes(11, 1), st, rg, pk->tab, rnd.u, m, rnd.e0, rnd.e1,
                       ct_out, (uint32_t)n_ct);
  else
    hipLaunchKernelGGL(k_encrypt, grid, dim3(ntt_threads(rg.N)), ntt_lds_bytes(rg.N, 2), st, rg, pk->tab, rnd.u, m, rnd.e0, rnd.e1, ct_out);
  HIP_TRY(hipGetLastError());
  return HE_OK;
}

he_status launch_decrypt(he_ctx* ctx, const he_sk* sk, const uint32_t* ct, uint64_t n_ct, uint32_t level, uint32_t* d_out,
                         hipStream_t st) {
  const RingDev& rg = ctx->ring;
  {
    KernelTimer timer_(ctx, KID_DECRYPT, st);
    const dim3 grid(level, (uint32_t)n_ct);
    if (rg.logN == 14)
      hipLaunchKernelGGL(k_decrypt_s<14>, grid, dim3(NttPlan<14>::NT), static_lds_bytes(14, 1), st, rg, sk->tab, ct, level, d_out);
    else if (rg.logN == 13)
      hipLaunchKernelGGL(k_decrypt_s<13>, grid, dim3(NttPlan<13>::NT), static_lds_bytes(13, 1), st, rg, sk->tab, ct, level, d_out);
    else if (rg.logN == 12)
      hipLaunchKernelGGL(k_decrypt_s<12>, grid, dim3(NttPlan<12>::NT), static_lds_bytes(12, 1), st, rg, sk->tab, ct, level, d_out);
    else if (rg.logN == 11)
      hipLaunchKernelGGL(k_decrypt_s<11>, grid, dim3(NttPlan<11>::NT), static_lds_bytes(11, 1), st, rg, sk->tab, ct, level, d_out);
    else
      hipLaunchKernelGGL(k_decrypt, grid, dim3(ntt_threads(rg.N)), ntt_lds_bytes(rg.N, 1), st, rg, sk->tab, ct, level, d_out);
  }
  HIP_TRY(hipGetLastError());
  return HE_OK;
}

template <int LEVEL>
void launch_decode_t(he_ctx* ctx, const CrtArgs& ca, const MaskDev& mk, const uint32_t* d, uint64_t first_ct, uint64_t n_ct,
                     float* w_out, double* slots_out, hipStream_t st) {
  const uint32_t n = ctx->ring.N / 2;
  if (ctx->ring.logN == 14)
    hipLaunchKernelGGL((k_decode_h<14, LEVEL>), dim3((uint32_t)n_ct), dim3(FftPlan<12>::NT), static_fft_lds_bytes(12), st, ctx->ring,
                       ca, mk, d, first_ct, w_out, slots_out);
  else if (ctx->ring.logN == 13)
    hipLaunchKernelGGL((k_decode_h<13, LEVEL>), dim3((uint32_t)n_ct), dim3(FftPlan<11>::NT), static_fft_lds_bytes(11), st, ctx->ring,
                       ca, mk, d, first_ct, w_out, slots_out);
  else if (ctx->ring.logN == 12)
    hipLaunchKernelGGL((k_decode_h<12, LEVEL>), dim3((uint32_t)n_ct), dim3(FftPlan<10>::NT), static_fft_lds_bytes(10), st, ctx->ring,
                       ca, mk, d, first_ct, w_out, slots_out);
  else if (ctx->ring.logN == 11)
    hipLaunchKernelGGL((k_decode_h<11, LEVEL>), dim3((uint32_t)n_ct), dim3(FftPlan<9>::NT), static_fft_lds_bytes(9), st, ctx->ring,
                       ca, mk, d, first_ct, w_out, slots_out);
  else
    hipLaunchKernelGGL(k_decode<LEVEL>, dim3((uint32_t)n_ct), dim3(fft_threads(n)), fft_lds_bytes(n), st, ctx->ring, ca, mk, d,
                       first_ct, w_out, slots_out);
}

he_status launch_decode(he_ctx* ctx, uint32_t level, const MaskDev& mk, const uint32_t* d, uint64_t first_ct, uint64_t n_ct,
                        float* w_out, double* slots_out, hipStream_t st) {
  CrtArgs ca{};
  he_host::modulus_words(ctx->primes.data(), level, ca.qw, ca.hw);
  KernelTimer timer_(ctx, KID_DECODE, st);
  switch (level) {
    case 1: launch_decode_t<1>(ctx, ca, mk, d, first_ct, n_ct, w_out, slots_out, st); break;
    case 2: launch_decode_t<2>(ctx, ca, mk, d, first_ct, n_ct, w_out, slots_out, st); break;
    case 3: launch_decode_t<3>(ctx, ca, mk, d, first_ct, n_ct, w_out, slots_out, st); break;
    case 4: launch_decode_t<4>(ctx, ca, mk, d, first_ct, n_ct, w_out, slots_out, st); break;
    case 5: launch_decode_t<5>(ctx, ca, mk, d, first_ct, n_ct, w_out, slots_out, st); break;
    case 6: launch_decode_t<6>(ctx, ca, mk, d, first_ct, n_ct, w_out, slots_out, st); break;
    case 7: launch_decode_t<7>(ctx, ca, mk, d, first_ct, n_ct, w_out, slots_out, st); break;
    case 8: launch_decode_t<8>(ctx, ca, mk, d, first_ct, n_ct, w_out, slots_out, st); break;
    default: return fail(HE_ERR_LEVEL, "level out of range");
  }
  HIP_TRY(hipGetLastError());
  return HE_OK;
}

template <int L, bool HAS_ACC, bool FINAL>
void launch_agg_t(const AggArgs& a, const AggConst& k, uint32_t log_n4, uint64_t n_vec, const uint32_t* acc_in, uint32_t* out,
                  hipStream_t st) {
  hipLaunchKernelGGL((k_aggregate<L, HAS_ACC, FINAL>), dim3((uint32_t)((n_vec + 255) / 256)), dim3(256), 0, st, a, k, log_n4,
                     n_vec, reinterpret_cast<const uint4*>(acc_in), reinterpret_cast<uint4*>(out));
}

template <int L>
void launch_agg_l(bool has_acc, bool fin, const AggArgs& a, const AggConst& k, uint32_t log_n4, uint64_t n_vec,
                  const uint32_t* acc_in, uint32_t* out, hipStream_t st) {
  if (has_acc && fin) launch_agg_t<L, true, true>(a, k, log_n4, n_vec, acc_in, out, st);
  else if (has_acc) launch_agg_t<L, true, false>(a, k, log_n4, n_vec, acc_in, out, st);
  else if (fin) launch_agg_t<L, false, true>(a, k, log_n4, n_vec, acc_in, out, st);
  else launch_agg_t<L, false, false>(a, k, log_n4, n_vec, acc_in, out, st);
}

he_status launch_agg(he_ctx* ctx, bool has_acc, bool fin, const AggArgs& a, uint64_t n_ct, const uint32_t* acc_in,
                     uint32_t* out, hipStream_t st) {
  if (n_ct == 0) return HE_OK;
  const RingDev& rg = ctx->ring;
  const uint32_t log_n4 = rg.logN - 2;
  const uint64_t n_vec = (n_ct * 2) << log_n4;
  if (((n_vec + 255) / 256) > 0x7FFFFFFFull) return fail(HE_ERR_INVALID_ARG, "too many ciphertexts for one launch");
  uintptr_t align_bits = reinterpret_cast<uintptr_t>(acc_in) | reinterpret_cast<uintptr_t>(out);
  for (uint32_t i = 0; i < a.K; ++i) align_bits |= reinterpret_cast<uintptr_t>(a.ct[i]);
  if (align_bits % 16 != 0) return fail(HE_ERR_INVALID_ARG, "ciphertext buffers must be 16-byte aligned");
  KernelTimer timer_(ctx, KID_AGGREGATE, st);
  switch (rg.L) {
    case 2: launch_agg_l<2>(has_acc, fin, a, ctx->agg, log_n4, n_vec, acc_in, out, st); break;
    case 3: launch_agg_l<3>(has_acc, fin, a, ctx->agg, log_n4, n_vec, acc_in, out, st); break;
    case 4: launch_agg_l<4>(has_acc, fin, a, ctx->agg, log_n4, n_vec, acc_in, out, st); break;
    case 5: launch_agg_l<5>(has_acc, fin, a, ctx->agg, log_n4, n_vec, acc_in, out, st); break;
    case 6: launch_agg_l<6>(has_acc, fin, a, ctx->agg, log_n4, n_vec, acc_in, out, st); break;
    case 7: launch_agg_l<7>(has_acc, fin, a, ctx->agg, log_n4, n_vec, acc_in, out, st); break;
    case 8: launch_agg_l<8>(has_acc, fin, a, ctx->agg, log_n4, n_vec, acc_in, out, st); break;
    default: return fail(HE_ERR_INVALID_ARG, "unsupported limb count");
  }
  HIP_TRY(hipGetLastError());
  return HE_OK;
}

template <int VEC>
void launch_plain_v(bool has_acc, bool fin, const PlainArgs& a, uint64_t first, uint64_t n_groups, const double* acc_in,
                    double* acc_out, float* out, hipStream_t st) {
  if (n_groups == 0) return;
  const dim3 grid((uint32_t)((n_groups + 255) / 256)), block(256);
  if (has_acc && fin) hipLaunchKernelGGL((k_plain_fedavg<true, true, VEC>), grid, block, 0, st, a, first, n_groups, acc_in, acc_out, out);
  else if (has_acc) hipLaunchKernelGGL((k_plain_fedavg<true, false, VEC>), grid, block, 0, st, a, first, n_groups, acc_in, acc_out, out);
  else if (fin) hipLaunchKernelGGL((k_plain_fedavg<false, true, VEC>), grid, block, 0, st, a, first, n_groups, acc_in, acc_out, out);
  else hipLaunchKernelGGL((k_plain_fedavg<false, false, VEC>), grid, block, 0, st, a, first, n_groups, acc_in, acc_out, out);
}

he_status launch_plain(he_ctx* ctx, bool has_acc, bool fin, const PlainArgs& a, uint64_t n_plain, const double* acc_in,
                       double* acc_out, float* out, hipStream_t st) {
  if (n_plain == 0) return HE_OK;
  if (n_plain > (1ull << 40)) return fail(HE_ERR_INVALID_ARG, "plaintext part too long for one launch");
  bool aligned = (reinterpret_cast<uintptr_t>(acc_in) | reinterpret_cast<uintptr_t>(acc_out) | reinterpret_cast<uintptr_t>(out)) % 16 == 0;
  for (uint32_t i = 0; i < a.K; ++i) aligned = aligned && reinterpret_cast<uintptr_t>(a.w[i]) % 16 == 0;
  const uint64_t n_vec = aligned ? n_plain / 4 : 0;
  KernelTimer timer_(ctx, KID_PLAIN_FEDAVG, st);
  launch_plain_v<4>(has_acc, fin, a, 0, n_vec, acc_in, acc_out, out, st);
  launch_plain_v<1>(has_acc, fin, a, n_vec * 4, n_plain - n_vec * 4, acc_in, acc_out, out, st);
  HIP_TRY(hipGetLastError());
  return HE_OK;
}

// Integer weights w_i = rint(alpha_i * q_{L-1}) (ties to even), validated.
he_status integer_weights(const he_ctx* ctx, uint32_t K, const double* alpha, bool check_sum, std::vector<uint32_t>* w) {
  const double q_last = (double)ctx->primes.back();
  double sum = 0.0;
  w->resize(K);
  for (uint32_t i = 0; i < K; ++i) {
    if (!(alpha[i] > 0.0) || !std::isfinite(alpha[i])) return fail(HE_ERR_INVALID_ARG, "aggregation weight must be positive and finite");
    const double r = std::nearbyint(alpha[i] * q_last);  // default rounding mode: to nearest, ties to even
    if (r < 1.0 || r > q_last) return fail(HE_ERR_INVALID_ARG, "aggregation weight rounds to 0 or exceeds 1");
    (*w)[i] = (uint32_t)r;
    sum += alpha[i];
  }
  if (check_sum && std::fabs(sum - 1.0) > 1e-9) return fail(HE_ERR_INVALID_ARG, "aggregation weights must sum to 1");
  return HE_OK;
}

// Folds K clients into (acc_ct, acc_plain) or, when `fin`, writes the final outputs.
he_status aggregate_impl(he_ctx* ctx, uint32_t K, const double* alpha, const std::vector<uint32_t>& w,
                         const uint32_t* const* ct_in, const float* const* plain_in, uint64_t n_ct, uint64_t n_plain,
                         bool has_acc, bool fin, uint32_t* acc_ct, double* acc_plain, uint32_t* ct_out, float* plain_out,
                         hipStream_t st) {
  const uint32_t L = ctx->ring.L;
  uint32_t done = 0;
  bool acc_live = has_acc;
  do {
    const uint32_t kc = std::min<uint32_t>(kAggClients, K - done);
    const bool last = (done + kc == K);
    AggArgs a{};
    PlainArgs pa{};
    a.K = pa.K = kc;
    for (uint32_t i = 0; i < kc; ++i) {
      a.ct[i] = n_ct ? ct_in[done + i] : nullptr;
      for (uint32_t j = 0; j < L; ++j) a.w[i][j] = w[done + i] % ctx->primes[j];
      pa.w[i] = n_plain ? plain_in[done + i] : nullptr;
      pa.alpha[i] = alpha[done + i];
    }
    const bool do_fin = fin && last;
    he_status s = launch_agg(ctx, acc_live, do_fin, a, n_ct, acc_ct, do_fin ? ct_out : acc_ct, st);
    if (s != HE_OK) return s;
    s = launch_plain(ctx, acc_live, do_fin, pa, n_plain, acc_plain, acc_plain, plain_out, st);
    if (s != HE_OK) return s;
    acc_live = true;
    done += kc;
  } while (done < K);
  return HE_OK;
}

// A mask whose complement comes in short runs gets a bit mask and per-chunk offsets beside its run tables, and its
// remainder is then compacted / scattered in parameter order (k_plain_move_bits).  Set-up path: synchronises `st`.
// Failing to allocate the tables is not an error: the run tables serve every mask.
// Measured on 400 M parameters (compaction, GB/s of the bytes it has to move): complement runs of 32 / 512 / 2048 / 8192 /
// 65536 parameters give 2.2 / 3.4 / 4.2 / 4.9 / 5.3 TB/s walking the run list and 3.5 / 4.5 / 4.6 / 4.6 / 4.5 TB/s in parameter order.
constexpr uint64_t kFragmentedBelow = 4096;  // average complement run (parameters) under which the bit mask is built
he_status build_mask_bits(he_mask* mk, hipStream_t st) {
  MaskDev& d = mk->dev;
  const uint64_t n_plain = d.P - d.P_enc;
  if (n_plain == 0 || d.n_cruns == 0 || n_plain / d.n_cruns >= kFragmentedBelow) return HE_OK;  // long runs: the run-ordered walk is faster
  const uint64_t n_pchunks = (d.P + kBitChunk - 1) / kBitChunk;
  if (n_pchunks >= (1ull << 31)) return HE_OK;
  const uint64_t n_words = n_pchunks * (kBitChunk / 32);
  const size_t bits_bytes = n_words * sizeof(uint32_t);
  const size_t cnt_bytes = ((n_pchunks * sizeof(uint32_t) + 255) / 256) * 256;
  const size_t off_bytes = (((n_pchunks + 2) * sizeof(uint64_t) + 255) / 256) * 256;
  const uint64_t n_ptab = d.n_runs ? d.P_enc / 64 + 2 : 0;  // the run of every 64th packed position, for gather and scatter
  const size_t ptab_bytes = ((n_ptab * sizeof(uint32_t) + 255) / 256) * 256;
  if (hipMalloc(&mk->bits_block, bits_bytes + cnt_bytes + off_bytes + ptab_bytes + 3 * sizeof(uint64_t)) != hipSuccess) {
    (void)hipGetLastError();
    mk->bits_block = nullptr;
    return HE_OK;
  }
  char* base = static_cast<char*>(mk->bits_block);
  uint32_t* bits = reinterpret_cast<uint32_t*>(base);
  uint32_t* counts = reinterpret_cast<uint32_t*>(base + bits_bytes);
  uint64_t* cchunk = reinterpret_cast<uint64_t*>(base + bits_bytes + cnt_bytes);
  hipLaunchKernelGGL(k_mask_bits, dim3((uint32_t)((n_words + 255) / 256)), dim3(256), 0, st, d.start, d.prefix, d.n_runs, d.P, n_words, bits);
  hipLaunchKernelGGL(k_chunk_unmasked, dim3((uint32_t)n_pchunks), dim3(64), 0, st, bits, counts);
  hipLaunchKernelGGL(he_sel::k_scan_counts, dim3(1), dim3(1024), 0, st, counts, n_pchunks, cchunk, (uint64_t)0, (uint64_t)0);
  uint32_t* ptab = reinterpret_cast<uint32_t*>(base + bits_bytes + cnt_bytes + off_bytes);
  if (n_ptab)
    hipLaunchKernelGGL(k_mask_ptab, dim3((uint32_t)((n_ptab + 255) / 256)), dim3(256), 0, st, d.prefix, d.n_runs, d.P_enc, n_ptab, ptab);
  HIP_TRY(hipGetLastError());
  uint64_t* ident = reinterpret_cast<uint64_t*>(base + bits_bytes + cnt_bytes + off_bytes + ptab_bytes);
  const uint64_t ident_host[3] = {0, 0, d.P_enc};
  HIP_TRY(hipMemcpyAsync(ident, ident_host, sizeof(ident_host), hipMemcpyHostToDevice, st));
  HIP_TRY(hipStreamSynchronize(st));
  d.bits = bits;
  d.cchunk = cchunk;
  d.ptab = n_ptab ? ptab : nullptr;
  d.ident = ident;
  return HE_OK;
}

}  // namespace

// =========================================================================================
// C ABI
// =========================================================================================

extern "C" {

const char* he_last_error(void) { return g_last_error.c_str(); }

he_status he_ctx_create(const he_params* params, int device, he_ctx** out) try {
  if (!params || !out) return fail(HE_ERR_INVALID_ARG, "params/out is null");
  *out = nullptr;
  if (params->log2_n < 3 || params->log2_n > 14) return fail(HE_ERR_INVALID_ARG, "log2_n must be in 3..14");
  if (params->n_limbs < 2 || params->n_limbs > (uint32_t)kMaxLimbs) return fail(HE_ERR_INVALID_ARG, "n_limbs must be in 2..8");
  if (params->scale_bits < 1 || params->scale_bits > 30) return fail(HE_ERR_INVALID_ARG, "scale_bits must be in 1..30");
  if (params->cbd_eta > 32) return fail(HE_ERR_INVALID_ARG, "cbd_eta must be in 0..32");
  HIP_TRY(hipSetDevice(device));
  if (device < 0 || device >= kMaxDevices) return fail(HE_ERR_INVALID_ARG, "device index out of range");
  if (!g_static_scratch[device]) {  // once per device, with that device current: each GPU has its own copy
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(HE_ERR_HIP, "the static scratch array has no device address");
    g_static_scratch[device] = ptr;
  }
  he_ctx* ctx = new (std::nothrow) he_ctx();
  if (!ctx) return fail(HE_ERR_NOMEM, "host allocation failed");
  ctx->device = device;
  ctx->static_scratch = g_static_scratch[device];
  const uint32_t logN = params->log2_n, N = 1u << logN, n = N / 2, L = params->n_limbs;
  if (params->primes) {
    ctx->primes.assign(params->primes, params->primes + L);
    for (uint32_t j = 0; j < L; ++j) {
      const uint32_t q = ctx->primes[j];
      if (q <= (1u << 30) || q >= (1u << 31) || (q - 1) % (2 * N) != 0 || !he_host::is_prime_u32(q) ||
          (j > 0 && q >= ctx->primes[j - 1])) {
        he_ctx_destroy(ctx);
        return fail(HE_ERR_INVALID_ARG, "primes must be descending primes in (2^30, 2^31) with q = 1 mod 2N");
      }
    }
  } else if (!he_host::find_primes(logN, L, &ctx->primes) || ctx->primes.back() <= (1u << 30)) {
    he_ctx_destroy(ctx);
    return fail(HE_ERR_INVALID_ARG, "not enough primes below 2^31 for this ring");
  }
  RingDev& rg = ctx->ring;
  rg.logN = logN; rg.N = N; rg.L = L; rg.scale_bits = params->scale_bits; rg.eta = params->cbd_eta;

  std::vector<uint2> twf((size_t)L * N), twi((size_t)L * N);
  static_assert(sizeof(he_host::U2) == sizeof(uint2), "layout");
  for (uint32_t j = 0; j < L; ++j) {
    const uint32_t q = ctx->primes[j];
    const uint32_t psi = he_host::smallest_primitive_2n_root(q, logN);
    he_host::power_table_bitrev(q, psi, logN, reinterpret_cast<he_host::U2*>(twf.data() + (size_t)j * N));
    he_host::power_table_bitrev(q, he_host::invmod(psi, q), logN, reinterpret_cast<he_host::U2*>(twi.data() + (size_t)j * N));
    rg.q[j] = q;
    const he_host::U2 ni = he_host::shoup(he_host::invmod(N % q, q), q);
    rg.ninv[j] = make_uint2(ni.w, ni.wp);
    const he_host::U2 niw = he_host::shoup((uint32_t)((uint64_t)ni.w * twi[(size_t)j * N + 1].x % q), q);
    rg.ninv_w1[j] = make_uint2(niw.w, niw.wp);
    const uint32_t q_last = ctx->primes[L - 1];
    ctx->agg.q[j] = q;
    const he_host::U2 c32 = he_host::shoup((uint32_t)((1ull << 32) % q), q);
    ctx->agg.c32[j] = make_uint2(c32.w, c32.wp);
    if (j + 1 < L) {
      const he_host::U2 qi = he_host::shoup(he_host::invmod(q_last % q, q), q);
      ctx->agg.qlinv[j] = make_uint2(qi.w, qi.wp);
      ctx->agg.qdiff[j] = q - q_last;
    }
  }
  ctx->agg.half_last = (ctx->primes[L - 1] - 1) / 2;

  std::vector<uint2> garner((size_t)kMaxLimbs * kMaxLimbs, make_uint2(0, 0));
  for (uint32_t i = 0; i < L; ++i)
    for (uint32_t j = i + 1; j < L; ++j) {
      const he_host::U2 v = he_host::shoup(he_host::invmod(ctx->primes[i] % ctx->primes[j], ctx->primes[j]), ctx->primes[j]);
      garner[i * kMaxLimbs + j] = make_uint2(v.w, v.wp);
    }

  std::vector<double2> fe(std::max<uint32_t>(1, n / 2)), tws(n);
  for (uint32_t r = 0; r < n / 2; ++r) {
    const he_host::D2 v = he_host::unit_root(r, n);
    fe[r] = make_double2(v.x, -v.y);
  }
  for (uint32_t k = 0; k < n; ++k) {
    const he_host::D2 v = he_host::unit_root(k, 4ull * n);
    tws[k] = make_double2(v.x, v.y);
  }
  std::vector<uint32_t> bins, penc(n), pdec(n), phalf(n);
  he_host::slot_bins(logN, &bins);
  for (uint32_t j = 0; j < n; ++j) {
    pdec[j] = bins[j];
    penc[j] = he_host::bitrev(bins[j], (int)logN - 1);
    phalf[j] = (he_host::bitrev(bins[j] >> 1, (int)logN - 2) << 1) | (bins[j] & 1);
  }

  he_status s = HE_OK;
  if (s == HE_OK) s = upload(ctx, twf, &rg.tw_fwd);
  if (s == HE_OK) s = upload(ctx, twi, &rg.tw_inv);
  if (s == HE_OK) s = upload(ctx, fe, &rg.fft_e);
  if (s == HE_OK) s = upload(ctx, tws, &rg.twist);
  if (s == HE_OK) s = upload(ctx, penc, &rg.perm_enc);
  if (s == HE_OK) s = upload(ctx, pdec, &rg.perm_dec);
  if (s == HE_OK) s = upload(ctx, phalf, &rg.perm_half);
  if (s == HE_OK) s = upload(ctx, garner, &rg.garner_inv);
  // kernels that need more than the default dynamic LDS
  if (s == HE_OK) s = allow_lds(k_encode, fft_lds_bytes(n));
  if (s == HE_OK) s = allow_lds(k_encrypt, ntt_lds_bytes(N, 2));
  if (s == HE_OK) s = allow_lds(k_decrypt, ntt_lds_bytes(N, 1));
  if (s == HE_OK) s = allow_lds(k_ntt_batch<false>, ntt_lds_bytes(N, 1));
  if (s == HE_OK) s = allow_lds(k_ntt_batch<true>, ntt_lds_bytes(N, 1));
  if (s == HE_OK && logN == 14) s = allow_lds(k_encrypt_s<14>, static_lds_bytes(14, 1));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decrypt_s<14>, static_lds_bytes(14, 1));
  if (s == HE_OK && logN == 14) s = allow_lds(k_ntt_batch_s<14, false>, static_lds_bytes(14, 1));
  if (s == HE_OK && logN == 14) s = allow_lds(k_ntt_batch_s<14, true>, static_lds_bytes(14, 1));
  if (s == HE_OK && logN == 13) s = allow_lds(k_encrypt_s<13>, static_lds_bytes(13, 1));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decrypt_s<13>, static_lds_bytes(13, 1));
  if (s == HE_OK && logN == 13) s = allow_lds(k_ntt_batch_s<13, false>, static_lds_bytes(13, 1));
  if (s == HE_OK && logN == 13) s = allow_lds(k_ntt_batch_s<13, true>, static_lds_bytes(13, 1));
  if (s == HE_OK && logN == 14) s = allow_lds(k_encode_r<14>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decode_h<14, 1>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decode_h<14, 2>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decode_h<14, 3>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decode_h<14, 4>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decode_h<14, 5>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decode_h<14, 6>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decode_h<14, 7>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 14) s = allow_lds(k_decode_h<14, 8>, static_fft_lds_bytes(12));
  if (s == HE_OK && logN == 13) s = allow_lds(k_encode_r<13>, static_fft_lds_bytes(11));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decode_h<13, 1>, static_fft_lds_bytes(11));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decode_h<13, 2>, static_fft_lds_bytes(11));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decode_h<13, 3>, static_fft_lds_bytes(11));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decode_h<13, 4>, static_fft_lds_bytes(11));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decode_h<13, 5>, static_fft_lds_bytes(11));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decode_h<13, 6>, static_fft_lds_bytes(11));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decode_h<13, 7>, static_fft_lds_bytes(11));
  if (s == HE_OK && logN == 13) s = allow_lds(k_decode_h<13, 8>, static_fft_lds_bytes(11));
  if (s == HE_OK) s = allow_lds(k_decode<1>, fft_lds_bytes(n));
  if (s == HE_OK) s = allow_lds(k_decode<2>, fft_lds_bytes(n));
  if (s == HE_OK) s = allow_lds(k_decode<3>, fft_lds_bytes(n));
  if (s == HE_OK) s = allow_lds(k_decode<4>, fft_lds_bytes(n));
  if (s == HE_OK) s = allow_lds(k_decode<5>, fft_lds_bytes(n));
  if (s == HE_OK) s = allow_lds(k_decode<6>, fft_lds_bytes(n));
  if (s == HE_OK) s = allow_lds(k_decode<7>, fft_lds_bytes(n));
  if (s == HE_OK) s = allow_lds(k_decode<8>, fft_lds_bytes(n));
  if (s != HE_OK) {
    he_ctx_destroy(ctx);
    return s;
  }
  *out = ctx;
  return HE_OK;
} catch (...) {
  return on_exception();
}

void he_ctx_destroy(he_ctx* ctx) {
  if (!ctx) return;
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  for (void* p : ctx->dev_allocs) (void)hipFree(p);
  if (ctx->ws) (void)hipFree(ctx->ws);
  for (const TimedSpan& sp : ctx->spans) {
    (void)hipEventDestroy(sp.start);
    (void)hipEventDestroy(sp.stop);
  }
  for (hipEvent_t e : ctx->event_pool) (void)hipEventDestroy(e);
  delete ctx;
}

he_status he_ctx_primes(const he_ctx* ctx, uint32_t* primes_host) try {
  if (!ctx || !primes_host) return fail(HE_ERR_INVALID_ARG, "null argument");
  std::copy(ctx->primes.begin(), ctx->primes.end(), primes_host);
  return HE_OK;
} catch (...) {
  return on_exception();
}

uint32_t he_ctx_ring_degree(const he_ctx* ctx) { return ctx ? ctx->ring.N : 0; }
uint32_t he_ctx_n_limbs(const he_ctx* ctx) { return ctx ? ctx->ring.L : 0; }
uint64_t he_ct_bytes(const he_ctx* ctx, uint32_t level) { return ctx ? 2ull * level * ctx->ring.N * 4ull : 0; }

// ---- keys ------------------------------------------------------------------------------

he_status he_keygen(he_ctx* ctx, uint64_t seed, he_pk** pk_out, he_sk** sk_out, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!pk_out || !sk_out) return fail(HE_ERR_INVALID_ARG, "pk/sk out pointer is null");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const RingDev& rg = ctx->ring;
  const size_t LN = (size_t)rg.L * rg.N;
  he_pk* pk = new (std::nothrow) he_pk{ctx, nullptr, nullptr};
  he_sk* sk = new (std::nothrow) he_sk{ctx, nullptr, nullptr};
  if (!pk || !sk) {
    delete pk;
    delete sk;
    return fail(HE_ERR_NOMEM, "host allocation failed");
  }
  uint32_t* tmp = nullptr;  // s_res, e_res, a_res: 3 x [L][N]
  auto cleanup = [&]() {
    if (tmp) (void)hipFree(tmp);
    he_pk_destroy(pk);
    he_sk_destroy(sk);
  };
#define KG_TRY(expr)                      \
  do {                                    \
    hipError_t e_ = (expr);               \
    if (e_ != hipSuccess) {               \
      cleanup();                          \
      return fail(HE_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    }                                     \
  } while (0)
  KG_TRY(hipMalloc(&pk->tab, 2 * LN * sizeof(uint2)));
  KG_TRY(hipMalloc(&pk->raw, 2 * LN * sizeof(uint32_t)));
  KG_TRY(hipMalloc(&sk->tab, LN * sizeof(uint2)));
  KG_TRY(hipMalloc(&sk->coeff, std::max<size_t>(rg.N, 16)));
  KG_TRY(hipMalloc(&tmp, 3 * LN * sizeof(uint32_t)));
  uint32_t *s_res = tmp, *e_res = tmp + LN, *a_res = tmp + 2 * LN;
  const uint2 key = make_uint2((uint32_t)seed, (uint32_t)(seed >> 32));
  const dim3 g1((rg.N + 255) / 256), b1(256);
  hipLaunchKernelGGL(k_keygen_sample, g1, b1, 0, st, rg, key, sk->coeff, s_res, e_res, a_res);
  KG_TRY(hipGetLastError());
  // forward transform of all 3L polynomials: polynomial index b -> limb b % L
  launch_ntt_batch(rg, false, -1, tmp, 3 * rg.L, st);
  KG_TRY(hipGetLastError());
  hipLaunchKernelGGL(k_keygen_combine, g1, b1, 0, st, rg, s_res, e_res, a_res, pk->raw, pk->tab, sk->tab);
  KG_TRY(hipGetLastError());
  KG_TRY(hipStreamSynchronize(st));  // tmp is freed below
  KG_TRY(hipFree(tmp));
  tmp = nullptr;
#undef KG_TRY
  *pk_out = pk;
  *sk_out = sk;
  return HE_OK;
} catch (...) {
  return on_exception();
}

void he_pk_destroy(he_pk* pk) {
  if (!pk) return;
  if (pk->tab) (void)hipFree(pk->tab);
  if (pk->raw) (void)hipFree(pk->raw);
  delete pk;
}

void he_sk_destroy(he_sk* sk) {
  if (!sk) return;
  if (sk->tab) (void)hipFree(sk->tab);
  if (sk->coeff) (void)hipFree(sk->coeff);
  delete sk;
}

// ---- mask ------------------------------------------------------------------------------

he_status he_mask_create(he_ctx* ctx, uint64_t P, const uint64_t* starts, const uint64_t* lens, uint64_t n_runs,
                         he_mask** out) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!out || (n_runs && (!starts || !lens))) return fail(HE_ERR_INVALID_ARG, "null argument");
  if (n_runs >= (1ull << 31)) return fail(HE_ERR_INVALID_ARG, "too many runs");
  // validate and build prefix sums + complement runs on the host
  std::vector<uint64_t> block;  // start | prefix | cstart | cprefix
  std::vector<uint64_t> st_v, pf_v, cs_v, cp_v;
  uint64_t pos = 0, packed = 0, cpacked = 0;
  for (uint64_t r = 0; r < n_runs; ++r) {
    if (lens[r] == 0 || starts[r] < pos || starts[r] > P || lens[r] > P - starts[r])
      return fail(HE_ERR_INVALID_ARG, "mask runs must be sorted, disjoint, non-empty and inside [0, P)");
    if (starts[r] > pos) {
      cs_v.push_back(pos);
      cp_v.push_back(cpacked);
      cpacked += starts[r] - pos;
    }
    st_v.push_back(starts[r]);
    pf_v.push_back(packed);
    packed += lens[r];
    pos = starts[r] + lens[r];
  }
  if (pos < P) {
    cs_v.push_back(pos);
    cp_v.push_back(cpacked);
    cpacked += P - pos;
  }
  pf_v.push_back(packed);
  cp_v.push_back(cpacked);
  const size_t o_st = 0, o_pf = o_st + st_v.size() + 1, o_cs = o_pf + pf_v.size(), o_cp = o_cs + cs_v.size() + 1;
  block.assign(o_cp + cp_v.size(), 0);
  he_mask* mk = new (std::nothrow) he_mask();
  if (!mk) return fail(HE_ERR_NOMEM, "host allocation failed");
  mk->ctx = ctx;
  try {  // the host copy of the run list is the last thing that can throw
    mk->starts.assign(starts, starts + n_runs);
    mk->lens.assign(lens, lens + n_runs);
    mk->n_runs = n_runs;
  } catch (...) {
    he_mask_destroy(mk);
    return on_exception();
  }
  std::copy(st_v.begin(), st_v.end(), block.begin() + o_st);
  std::copy(pf_v.begin(), pf_v.end(), block.begin() + o_pf);
  std::copy(cs_v.begin(), cs_v.end(), block.begin() + o_cs);
  std::copy(cp_v.begin(), cp_v.end(), block.begin() + o_cp);
  hipError_t e = hipMalloc(&mk->dev_block, block.size() * sizeof(uint64_t));
  if (e == hipSuccess) e = hipMemcpy(mk->dev_block, block.data(), block.size() * sizeof(uint64_t), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    he_mask_destroy(mk);
    return fail(HE_ERR_HIP, std::string("mask upload: ") + hipGetErrorString(e));
  }
  const uint64_t* base = static_cast<const uint64_t*>(mk->dev_block);
  mk->dev.start = base + o_st;
  mk->dev.prefix = base + o_pf;
  mk->dev.cstart = base + o_cs;
  mk->dev.cprefix = base + o_cp;
  mk->dev.n_runs = (uint32_t)st_v.size();
  mk->dev.n_cruns = (uint32_t)cs_v.size();
  mk->dev.P = P;
  mk->dev.P_enc = packed;
  const he_status sb = build_mask_bits(mk, nullptr);
  if (sb != HE_OK) {
    he_mask_destroy(mk);
    return sb;
  }
  *out = mk;
  return HE_OK;
} catch (...) {
  return on_exception();
}

// Mask object of a device byte mask (non-zero = selected), built on the GPU: per-chunk counts of run starts, run ends
// and set bytes, three exclusive scans, and an emit pass that writes the object's device tables (masked and complement
// runs with their packed offsets) in place.  Only five words travel to the host; the run list itself follows when
// he_mask_runs asks for it.
static he_status mask_from_device_bytes(he_ctx* ctx, uint64_t P, const uint8_t* mask_dev, he_mask** out, hipStream_t st) try {
  using namespace he_sel;
  if (P == 0) return he_mask_create(ctx, 0, nullptr, nullptr, 0, out);
  const uint64_t n_chunks = (P + kChunk - 1) / kChunk;
  if (n_chunks > 0x7FFFFFFFull) return fail(HE_ERR_INVALID_ARG, "vector too long");
  char* tmp = nullptr;
  he_mask* mk = nullptr;
  const size_t cnt_bytes = ((n_chunks * sizeof(uint32_t) + 255) / 256) * 256;
  const size_t off_bytes = (((n_chunks + 1) * sizeof(uint64_t) + 255) / 256) * 256;
  auto cleanup = [&]() {
    if (tmp) (void)hipFree(tmp);
    he_mask_destroy(mk);
  };
#define MK_TRY(expr)                                                                 \
  do {                                                                               \
    hipError_t e_ = (expr);                                                          \
    if (e_ != hipSuccess) {                                                          \
      cleanup();                                                                     \
      return fail(e_ == hipErrorOutOfMemory ? HE_ERR_NOMEM : HE_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    }                                                                                \
  } while (0)
  MK_TRY(hipMalloc(&tmp, 3 * cnt_bytes + 3 * off_bytes));
  uint32_t* n_start = reinterpret_cast<uint32_t*>(tmp);
  uint32_t* n_end = reinterpret_cast<uint32_t*>(tmp + cnt_bytes);
  uint32_t* n_set = reinterpret_cast<uint32_t*>(tmp + 2 * cnt_bytes);
  uint64_t* off_start = reinterpret_cast<uint64_t*>(tmp + 3 * cnt_bytes);
  uint64_t* off_end = reinterpret_cast<uint64_t*>(tmp + 3 * cnt_bytes + off_bytes);
  uint64_t* off_set = reinterpret_cast<uint64_t*>(tmp + 3 * cnt_bytes + 2 * off_bytes);
  hipLaunchKernelGGL(k_runs<false>, dim3((uint32_t)n_chunks), dim3(kThreads), 0, st, mask_dev, P, n_start, n_end, n_set, nullptr, nullptr,
                     nullptr, nullptr, nullptr, nullptr, nullptr);
  hipLaunchKernelGGL(k_scan_counts, dim3(3), dim3(1024), 0, st, n_start, n_chunks, off_start, (uint64_t)(cnt_bytes / sizeof(uint32_t)),
                     (uint64_t)(off_bytes / sizeof(uint64_t)));  // the three arrays, one workgroup each
  MK_TRY(hipGetLastError());
  uint64_t totals[3] = {0, 0, 0};
  uint8_t edge[2] = {0, 0};  // first and last byte of the mask
  MK_TRY(hipMemcpyAsync(&totals[0], off_start + n_chunks, sizeof(uint64_t), hipMemcpyDeviceToHost, st));
  MK_TRY(hipMemcpyAsync(&totals[1], off_end + n_chunks, sizeof(uint64_t), hipMemcpyDeviceToHost, st));
  MK_TRY(hipMemcpyAsync(&totals[2], off_set + n_chunks, sizeof(uint64_t), hipMemcpyDeviceToHost, st));
  MK_TRY(hipMemcpyAsync(&edge[0], mask_dev, 1, hipMemcpyDeviceToHost, st));
  MK_TRY(hipMemcpyAsync(&edge[1], mask_dev + (P - 1), 1, hipMemcpyDeviceToHost, st));
  MK_TRY(hipStreamSynchronize(st));
  const uint64_t R = totals[0], P_enc = totals[2];
  if (totals[1] != R || P_enc > P) {
    cleanup();
    return fail(HE_ERR_HIP, "run extraction: starts and ends disagree");
  }
  if (R == 0) {
    cleanup();
    return he_mask_create(ctx, P, nullptr, nullptr, 0, out);
  }
  if (R >= (1ull << 31)) {
    cleanup();
    return fail(HE_ERR_INVALID_ARG, "too many runs");
  }
  const uint64_t n_cruns = R + 1 - (edge[0] ? 1 : 0) - (edge[1] ? 1 : 0);
  mk = new (std::nothrow) he_mask();
  if (!mk) {
    cleanup();
    return fail(HE_ERR_NOMEM, "host allocation failed");
  }
  mk->ctx = ctx;
  mk->n_runs = R;
  mk->host_runs_valid = false;
  // same layout as he_mask_create: start | prefix | cstart | cprefix, one spare word after start and cstart
  const size_t o_st = 0, o_pf = o_st + R + 1, o_cs = o_pf + R + 1, o_cp = o_cs + n_cruns + 1, n_words = o_cp + n_cruns + 1;
  MK_TRY(hipMalloc(&mk->dev_block, n_words * sizeof(uint64_t)));
  uint64_t* base = static_cast<uint64_t*>(mk->dev_block);
  hipLaunchKernelGGL(k_runs<true>, dim3((uint32_t)n_chunks), dim3(kThreads), 0, st, mask_dev, P, nullptr, nullptr, nullptr, off_start, off_end,
                     off_set, base + o_st, base + o_pf, base + o_cs, base + o_cp);
  MK_TRY(hipGetLastError());
  const uint64_t tail[3] = {P_enc, P - P_enc, 0};  // prefix[R] and cprefix[n_cruns]: the totals; the spare words: 0
  MK_TRY(hipMemcpyAsync(base + o_pf + R, &tail[0], sizeof(uint64_t), hipMemcpyHostToDevice, st));
  MK_TRY(hipMemcpyAsync(base + o_cp + n_cruns, &tail[1], sizeof(uint64_t), hipMemcpyHostToDevice, st));
  MK_TRY(hipMemcpyAsync(base + o_st + R, &tail[2], sizeof(uint64_t), hipMemcpyHostToDevice, st));
  MK_TRY(hipMemcpyAsync(base + o_cs + n_cruns, &tail[2], sizeof(uint64_t), hipMemcpyHostToDevice, st));
  MK_TRY(hipStreamSynchronize(st));  // tmp is freed below, and tail[] leaves scope
  (void)hipFree(tmp);
  tmp = nullptr;
#undef MK_TRY
  mk->dev.start = base + o_st;
  mk->dev.prefix = base + o_pf;
  mk->dev.cstart = base + o_cs;
  mk->dev.cprefix = base + o_cp;
  mk->dev.n_runs = (uint32_t)R;
  mk->dev.n_cruns = (uint32_t)n_cruns;
  mk->dev.P = P;
  mk->dev.P_enc = P_enc;
  const he_status sb = build_mask_bits(mk, st);
  if (sb != HE_OK) {
    he_mask_destroy(mk);
    return sb;
  }
  *out = mk;
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_mask_from_bytes(he_ctx* ctx, uint64_t P, const uint8_t* mask_dev, he_mask** out, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!out || (P && !mask_dev)) return fail(HE_ERR_INVALID_ARG, "null argument");
  return mask_from_device_bytes(ctx, P, mask_dev, out, static_cast<hipStream_t>(stream));
} catch (...) {
  return on_exception();
}

he_status he_mask_select_top(he_ctx* ctx, uint64_t P, const float* s_dev, double ratio, he_mask** out, void* stream) try {
  using namespace he_sel;
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!out || (P && !s_dev)) return fail(HE_ERR_INVALID_ARG, "null argument");
  if (!(ratio >= 0.0) || !(ratio <= 1.0)) return fail(HE_ERR_INVALID_ARG, "ratio must be in [0, 1]");
  if (P >= (1ull << 40)) return fail(HE_ERR_INVALID_ARG, "vector too long");
  const uint64_t k = (uint64_t)std::nearbyint(ratio * (double)P);  // ties to even, as everywhere else
  if (k == 0) return he_mask_create(ctx, P, nullptr, nullptr, 0, out);
  if (k >= P) {
    const uint64_t zero = 0;
    return he_mask_create(ctx, P, &zero, &P, 1, out);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint64_t n_chunks = (P + kChunk - 1) / kChunk;
  if (n_chunks > 0x7FFFFFFFull) return fail(HE_ERR_INVALID_ARG, "vector too long");
  constexpr size_t kHistBytes = 3 * 2048 * sizeof(unsigned long long);
  const size_t cnt_bytes = ((n_chunks * sizeof(uint32_t) + 255) / 256) * 256;
  const size_t off_bytes = (((n_chunks + 1) * sizeof(uint64_t) + 255) / 256) * 256;
  const size_t mask_bytes = ((P + 255) / 256) * 256;
  char* tmp = nullptr;
  HIP_TRY(hipMalloc(&tmp, 256 + kHistBytes + cnt_bytes + off_bytes + mask_bytes));
  SelState* state = reinterpret_cast<SelState*>(tmp);
  unsigned long long* hist = reinterpret_cast<unsigned long long*>(tmp + 256);
  uint32_t* eq_count = reinterpret_cast<uint32_t*>(tmp + 256 + kHistBytes);
  uint64_t* eq_off = reinterpret_cast<uint64_t*>(tmp + 256 + kHistBytes + cnt_bytes);
  uint8_t* mask_dev = reinterpret_cast<uint8_t*>(tmp + 256 + kHistBytes + cnt_bytes + off_bytes);
#define SEL_TRY(expr)                                                                \
  do {                                                                               \
    hipError_t e_ = (expr);                                                          \
    if (e_ != hipSuccess) {                                                          \
      (void)hipFree(tmp);                                                            \
      return fail(HE_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));    \
    }                                                                                \
  } while (0)
  SelState init{0u, 0u, k, 0u};
  SEL_TRY(hipMemcpyAsync(state, &init, sizeof(init), hipMemcpyHostToDevice, st));
  hipLaunchKernelGGL(k_fill_u32, dim3(24), dim3(256), 0, st, reinterpret_cast<uint32_t*>(hist), (uint64_t)(kHistBytes / 4), 0u);
  const dim3 hgrid((uint32_t)std::min<uint64_t>(8192, (P + kThreads - 1) / kThreads));
  hipLaunchKernelGGL((k_hist<21, 11>), hgrid, dim3(kThreads), 0, st, s_dev, P, state, 0u, hist);
  hipLaunchKernelGGL((k_pick<21, 11>), dim3(1), dim3(64), 0, st, hist, state);
  hipLaunchKernelGGL((k_hist<10, 11>), hgrid, dim3(kThreads), 0, st, s_dev, P, state, 0xFFE00000u, hist + 2048);
  hipLaunchKernelGGL((k_pick<10, 11>), dim3(1), dim3(64), 0, st, hist + 2048, state);
  hipLaunchKernelGGL((k_hist<0, 10>), hgrid, dim3(kThreads), 0, st, s_dev, P, state, 0xFFFFFC00u, hist + 4096);
  hipLaunchKernelGGL((k_pick<0, 10>), dim3(1), dim3(64), 0, st, hist + 4096, state);
  SEL_TRY(hipGetLastError());
  SelState fin{};
  SEL_TRY(hipMemcpyAsync(&fin, state, sizeof(fin), hipMemcpyDeviceToHost, st));
  SEL_TRY(hipStreamSynchronize(st));
  const bool rank_ties = fin.k_rem < fin.cnt_eq;  // only some of the elements equal to the threshold are taken
  if (rank_ties) {
    hipLaunchKernelGGL(k_count_eq, dim3((uint32_t)n_chunks), dim3(kThreads), 0, st, s_dev, P, state, eq_count);
    hipLaunchKernelGGL(k_scan_counts, dim3(1), dim3(1024), 0, st, eq_count, n_chunks, eq_off, (uint64_t)0, (uint64_t)0);
  }
  hipLaunchKernelGGL(k_mark, dim3((uint32_t)n_chunks), dim3(kThreads), 0, st, s_dev, P, state, rank_ties ? eq_off : nullptr, mask_dev);
  SEL_TRY(hipGetLastError());
#undef SEL_TRY
  s = mask_from_device_bytes(ctx, P, mask_dev, out, st);  // synchronises the stream before it returns
  (void)hipFree(tmp);
  return s;
} catch (...) {
  return on_exception();
}

void he_mask_destroy(he_mask* mask) {
  if (!mask) return;
  if (mask->dev_block) (void)hipFree(mask->dev_block);
  if (mask->bits_block) (void)hipFree(mask->bits_block);
  delete mask;
}

uint64_t he_mask_n_runs(const he_mask* mask) { return mask ? mask->n_runs : 0; }

he_status he_mask_runs(const he_mask* mask, uint64_t* starts_host, uint64_t* lens_host) try {
  if (!mask || ((!starts_host || !lens_host) && mask->n_runs)) return fail(HE_ERR_INVALID_ARG, "null argument");
  if (!mask->host_runs_valid) {  // built on the device: fetch the run list now (synchronous), lengths from the packed offsets
    const uint64_t R = mask->n_runs;
    HIP_TRY(hipSetDevice(mask->ctx->device));
    mask->starts.resize(R);
    mask->lens.resize(R + 1);
    HIP_TRY(hipMemcpy(mask->starts.data(), mask->dev.start, R * sizeof(uint64_t), hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(mask->lens.data(), mask->dev.prefix, (R + 1) * sizeof(uint64_t), hipMemcpyDeviceToHost));
    for (uint64_t r = 0; r < R; ++r) mask->lens[r] = mask->lens[r + 1] - mask->lens[r];
    mask->lens.resize(R);
    mask->host_runs_valid = true;
  }
  std::copy(mask->starts.begin(), mask->starts.end(), starts_host);
  std::copy(mask->lens.begin(), mask->lens.end(), lens_host);
  return HE_OK;
} catch (...) {
  return on_exception();
}

uint64_t he_mask_n_params(const he_mask* mask) { return mask ? mask->dev.P : 0; }
uint64_t he_mask_n_enc(const he_mask* mask) { return mask ? mask->dev.P_enc : 0; }
uint64_t he_n_ct(const he_ctx* ctx, const he_mask* mask) {
  if (!ctx || !mask) return 0;
  const uint64_t n = ctx->ring.N / 2;
  return (mask->dev.P_enc + n - 1) / n;
}

// ---- client: encrypt -------------------------------------------------------------------

// fixed_scratch: when given (he_encrypt_masked_static), the per-ciphertext scratch lives there and the call
// allocates nothing; the call is refused unless that block holds the scratch of all n_ct ciphertexts.
static he_status encrypt_masked_impl(he_ctx* ctx, const he_pk* pk, const he_mask* mask, uint64_t seed, uint32_t client_id,
                                     double pre_scale, const float* w_dev, uint32_t* ct_out_dev, float* plain_out_dev,
                                     void* stream, void* fixed_scratch = nullptr, size_t fixed_bytes = 0) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!pk || !mask || pk->ctx != ctx || mask->ctx != ctx) return fail(HE_ERR_INVALID_ARG, "key/mask missing or from another context");
  const MaskDev& mk = mask->dev;
  const uint64_t n_ct = he_n_ct(ctx, mask), n_plain = mk.P - mk.P_enc;
  if ((mk.P && !w_dev) || (n_ct && !ct_out_dev) || (n_plain && !plain_out_dev)) return fail(HE_ERR_INVALID_ARG, "null data pointer");
  if (n_ct >= (1ull << 32)) return fail(HE_ERR_INVALID_ARG, "too many ciphertexts");
  if (reinterpret_cast<uintptr_t>(ct_out_dev) % 16 != 0) return fail(HE_ERR_INVALID_ARG, "ciphertext buffers must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const RingDev& rg = ctx->ring;
  const size_t N = rg.N;
  uint64_t chunk = std::min<uint64_t>(kCtChunk, n_ct);
  if (fixed_scratch) {
    if (n_ct * N * kEncScratchBytesPerCoeff > fixed_bytes)
      return fail(HE_ERR_INVALID_ARG, "too many ciphertexts for the static scratch: n_ct * N * 7 bytes must not exceed HE_STATIC_SCRATCH_BYTES");
  } else if (chunk) {
    s = ensure_ws(ctx, chunk * N * kEncScratchBytesPerCoeff);
    if (s != HE_OK) return s;
  }
  // Under a fragmented mask one pass in parameter order fills the remainder and the packed slot vector (n_ct * n floats,
  // zero-padded), which the encoder then reads as a plain array; the static-scratch form keeps the gather.
  const uint64_t n_slots = N / 2;
  const size_t enc_scratch_bytes = ((chunk * N * kEncScratchBytesPerCoeff + 255) / 256) * 256;
  const bool split = mk.bits && !fixed_scratch && n_ct > 0;
  float* packed = nullptr;
  if (split) {
    s = ensure_ws(ctx, enc_scratch_bytes + n_ct * n_slots * sizeof(float));
    if (s != HE_OK) return s;
    packed = reinterpret_cast<float*>(static_cast<char*>(ctx->ws) + enc_scratch_bytes);
  }
  const EncScratch sc = carve_enc_scratch(fixed_scratch ? fixed_scratch : ctx->ws, chunk, N);
  // The remainder is compacted first, on the same stream: an HBM-bound copy beside the transform kernels (tried on a
  // second stream, and on a disjoint set of compute units) lengthens them by as much as it saves, because it evicts
  // their twiddle and key tables from L2.
  if (n_plain) {
    {
      KernelTimer timer_(ctx, KID_PLAIN_MOVE, st);
      if (split) {
        const uint64_t n_pchunks = (mk.P + kBitChunk - 1) / kBitChunk, pad = n_ct * n_slots - mk.P_enc;
        hipLaunchKernelGGL(k_split_bits<false>, dim3((uint32_t)n_pchunks), dim3(256), 0, st, mk, w_dev, (float*)nullptr,
                           (const float*)nullptr, packed, (const float*)nullptr, plain_out_dev);
        if (pad) hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(pad, 256, 64)), dim3(256), 0, st, reinterpret_cast<uint32_t*>(packed + mk.P_enc), pad, 0u);
      } else {
        launch_plain_move<false>(mk, w_dev, plain_out_dev, st);
      }
      HIP_TRY(hipGetLastError());
    }
    if (pre_scale != 1.0) {  // weigh the compacted remainder in place: float32(alpha * x), product in float64
      PlainArgs pa{};
      pa.K = 1;
      pa.w[0] = plain_out_dev;
      pa.alpha[0] = pre_scale;
      s = launch_plain(ctx, false, true, pa, n_plain, nullptr, nullptr, plain_out_dev, st);
      if (s != HE_OK) return s;
    }
  }
  for (uint64_t c0 = 0; c0 < n_ct; c0 += chunk) {
    const uint64_t cn = std::min<uint64_t>(chunk, n_ct - c0);
    s = launch_encode(ctx, mk, w_dev, split ? packed + c0 * n_slots : nullptr, c0, cn, sc.m, &sc, seed, client_id, st, pre_scale);
    if (s != HE_OK) return s;
    s = launch_encrypt(ctx, pk, cn, sc.m, sc, ct_out_dev + c0 * 2 * rg.L * N, st);
    if (s != HE_OK) return s;
  }
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_encrypt_masked(he_ctx* ctx, const he_pk* pk, const he_mask* mask, uint64_t seed, uint32_t client_id,
                            const float* w_dev, uint32_t* ct_out_dev, float* plain_out_dev, void* stream) try {
  return encrypt_masked_impl(ctx, pk, mask, seed, client_id, 1.0, w_dev, ct_out_dev, plain_out_dev, stream);
} catch (...) {
  return on_exception();
}

he_status he_encrypt_masked_static(he_ctx* ctx, const he_pk* pk, const he_mask* mask, uint64_t seed, uint32_t client_id,
                                   const float* w_dev, uint32_t* ct_out_dev, float* plain_out_dev, void* stream) try {
  if (!ctx) return fail(HE_ERR_INVALID_ARG, "context is null");
  if (!ctx->static_scratch) return fail(HE_ERR_HIP, "the static scratch array was not resolved on this device");
  // Per-kernel timing takes events from a pool that it grows on demand: off for this call, which must create nothing.
  const bool timing = ctx->timing_on;
  ctx->timing_on = false;
  const he_status s = encrypt_masked_impl(ctx, pk, mask, seed, client_id, 1.0, w_dev, ct_out_dev, plain_out_dev, stream,
                                          ctx->static_scratch, HE_STATIC_SCRATCH_BYTES);
  ctx->timing_on = timing;
  return s;
} catch (...) {
  return on_exception();
}

he_status he_encrypt_masked_weighted(he_ctx* ctx, const he_pk* pk, const he_mask* mask, uint64_t seed, uint32_t client_id,
                                     double alpha, const float* w_dev, uint32_t* ct_out_dev, float* plain_out_dev,
                                     void* stream) try {
  if (!(alpha > 0.0) || !(alpha <= 1.0)) return fail(HE_ERR_INVALID_ARG, "aggregation weight must be in (0, 1]");
  return encrypt_masked_impl(ctx, pk, mask, seed, client_id, alpha, w_dev, ct_out_dev, plain_out_dev, stream);
} catch (...) {
  return on_exception();
}

// ---- server: aggregate -----------------------------------------------------------------

he_status he_aggregate(he_ctx* ctx, uint32_t K, const double* alpha_host, const uint32_t* const* ct_in_dev,
                       const float* const* plain_in_dev, uint64_t n_ct, uint64_t n_plain, uint32_t* ct_out_dev,
                       float* plain_out_dev, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (K == 0 || K > HE_MAX_CLIENTS_PER_CALL) return fail(HE_ERR_INVALID_ARG, "K must be in 1..HE_MAX_CLIENTS_PER_CALL");
  if (!alpha_host || (n_ct && (!ct_in_dev || !ct_out_dev)) || (n_plain && (!plain_in_dev || !plain_out_dev)))
    return fail(HE_ERR_INVALID_ARG, "null argument");
  for (uint32_t i = 0; i < K; ++i)
    if ((n_ct && !ct_in_dev[i]) || (n_plain && !plain_in_dev[i])) return fail(HE_ERR_INVALID_ARG, "null client buffer");
  std::vector<uint32_t> w;
  s = integer_weights(ctx, K, alpha_host, true, &w);
  if (s != HE_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint32_t* acc_ct = nullptr;
  double* acc_plain = nullptr;
  if (K > (uint32_t)kAggClients) {  // more clients than one launch folds: internal accumulators
    const size_t ct_bytes = (size_t)n_ct * 2 * ctx->ring.L * ctx->ring.N * 4;
    const size_t ct_bytes_al = (ct_bytes + 255) & ~(size_t)255;
    s = ensure_ws(ctx, ct_bytes_al + n_plain * sizeof(double));
    if (s != HE_OK) return s;
    acc_ct = static_cast<uint32_t*>(ctx->ws);
    acc_plain = reinterpret_cast<double*>(static_cast<char*>(ctx->ws) + ct_bytes_al);
  }
  return aggregate_impl(ctx, K, alpha_host, w, ct_in_dev, plain_in_dev, n_ct, n_plain, false, true, acc_ct, acc_plain,
                        ct_out_dev, plain_out_dev, st);
} catch (...) {
  return on_exception();
}

he_status he_aggregate_sum(he_ctx* ctx, uint32_t K, const uint32_t* const* ct_in_dev, const float* const* plain_in_dev,
                           uint64_t n_ct, uint64_t n_plain, uint32_t* ct_out_dev, float* plain_out_dev, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (K == 0 || K > HE_MAX_CLIENTS_PER_CALL) return fail(HE_ERR_INVALID_ARG, "K must be in 1..HE_MAX_CLIENTS_PER_CALL");
  if ((n_ct && (!ct_in_dev || !ct_out_dev)) || (n_plain && (!plain_in_dev || !plain_out_dev)))
    return fail(HE_ERR_INVALID_ARG, "null argument");
  for (uint32_t i = 0; i < K; ++i)
    if ((n_ct && !ct_in_dev[i]) || (n_plain && !plain_in_dev[i])) return fail(HE_ERR_INVALID_ARG, "null client buffer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint32_t L = ctx->ring.L;
  double* acc_plain = nullptr;
  if (K > (uint32_t)kAggClients && n_plain) {  // float64 partial sums of the plaintext part between launches
    s = ensure_ws(ctx, n_plain * sizeof(double));
    if (s != HE_OK) return s;
    acc_plain = static_cast<double*>(ctx->ws);
  }
  uint32_t done = 0;
  do {  // unit weights, no rescale: the sum of residues in all L limbs IS the result (accumulated in place)
    const uint32_t kc = std::min<uint32_t>(kAggClients, K - done);
    const bool first = done == 0, last = done + kc == K;
    AggArgs a{};
    PlainArgs pa{};
    a.K = pa.K = kc;
    for (uint32_t i = 0; i < kc; ++i) {
      a.ct[i] = n_ct ? ct_in_dev[done + i] : nullptr;
      for (uint32_t j = 0; j < L; ++j) a.w[i][j] = 1;
      pa.w[i] = n_plain ? plain_in_dev[done + i] : nullptr;
      pa.alpha[i] = 1.0;
    }
    s = launch_agg(ctx, !first, false, a, n_ct, ct_out_dev, ct_out_dev, st);
    if (s != HE_OK) return s;
    s = launch_plain(ctx, !first, last, pa, n_plain, acc_plain, acc_plain, plain_out_dev, st);
    if (s != HE_OK) return s;
    done += kc;
  } while (done < K);
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_aggregate_begin(he_ctx* ctx, uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev, double* acc_plain_dev,
                             void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if ((n_ct && !acc_ct_dev) || (n_plain && !acc_plain_dev)) return fail(HE_ERR_INVALID_ARG, "null accumulator");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint64_t n_words = n_ct * 2 * ctx->ring.L * ctx->ring.N;
  if (n_words) {
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(n_words, 256, 1u << 16)), dim3(256), 0, st, acc_ct_dev, n_words, 0u);
    HIP_TRY(hipGetLastError());
  }
  if (n_plain) {
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(n_plain * 2, 256, 1u << 16)), dim3(256), 0, st,
                       reinterpret_cast<uint32_t*>(acc_plain_dev), n_plain * 2, 0u);
    HIP_TRY(hipGetLastError());
  }
  return HE_OK;
} catch (...) {
  return on_exception();
}

// One fold of the streaming form.  has_acc: the accumulators hold earlier clients (otherwise they are only written);
// fin: the outputs are written instead of the accumulators.
static he_status aggregate_fold(he_ctx* ctx, uint32_t K_chunk, const double* alpha_host, const uint32_t* const* ct_in_dev,
                                const float* const* plain_in_dev, uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev,
                                double* acc_plain_dev, bool has_acc, bool fin, uint32_t* ct_out_dev, float* plain_out_dev,
                                void* stream) {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (K_chunk == 0 || K_chunk > HE_MAX_CLIENTS_PER_CALL) return fail(HE_ERR_INVALID_ARG, "K_chunk must be in 1..HE_MAX_CLIENTS_PER_CALL");
  // a fold of more clients than one launch takes keeps its partial sums in the accumulators, whatever it ends with
  const bool needs_acc = has_acc || !fin || K_chunk > (uint32_t)kAggClients;
  if (!alpha_host || (n_ct && (!ct_in_dev || (needs_acc && !acc_ct_dev))) || (n_plain && (!plain_in_dev || (needs_acc && !acc_plain_dev))))
    return fail(HE_ERR_INVALID_ARG, "null argument");
  if (fin && ((n_ct && !ct_out_dev) || (n_plain && !plain_out_dev))) return fail(HE_ERR_INVALID_ARG, "null output");
  for (uint32_t i = 0; i < K_chunk; ++i)
    if ((n_ct && !ct_in_dev[i]) || (n_plain && !plain_in_dev[i])) return fail(HE_ERR_INVALID_ARG, "null client buffer");
  std::vector<uint32_t> w;
  s = integer_weights(ctx, K_chunk, alpha_host, false, &w);
  if (s != HE_OK) return s;
  return aggregate_impl(ctx, K_chunk, alpha_host, w, ct_in_dev, plain_in_dev, n_ct, n_plain, has_acc, fin, acc_ct_dev,
                        acc_plain_dev, ct_out_dev, plain_out_dev, static_cast<hipStream_t>(stream));
}

he_status he_aggregate_add(he_ctx* ctx, uint32_t K_chunk, const double* alpha_host, const uint32_t* const* ct_in_dev,
                           const float* const* plain_in_dev, uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev,
                           double* acc_plain_dev, void* stream) try {
  return aggregate_fold(ctx, K_chunk, alpha_host, ct_in_dev, plain_in_dev, n_ct, n_plain, acc_ct_dev, acc_plain_dev, true, false,
                        nullptr, nullptr, stream);
} catch (...) {
  return on_exception();
}

he_status he_aggregate_add_first(he_ctx* ctx, uint32_t K_chunk, const double* alpha_host, const uint32_t* const* ct_in_dev,
                                 const float* const* plain_in_dev, uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev,
                                 double* acc_plain_dev, void* stream) try {
  return aggregate_fold(ctx, K_chunk, alpha_host, ct_in_dev, plain_in_dev, n_ct, n_plain, acc_ct_dev, acc_plain_dev, false, false,
                        nullptr, nullptr, stream);
} catch (...) {
  return on_exception();
}

he_status he_aggregate_add_last(he_ctx* ctx, uint32_t K_chunk, const double* alpha_host, const uint32_t* const* ct_in_dev,
                                const float* const* plain_in_dev, uint64_t n_ct, uint64_t n_plain, uint32_t* acc_ct_dev,
                                double* acc_plain_dev, uint32_t* ct_out_dev, float* plain_out_dev, void* stream) try {
  return aggregate_fold(ctx, K_chunk, alpha_host, ct_in_dev, plain_in_dev, n_ct, n_plain, acc_ct_dev, acc_plain_dev, true, true,
                        ct_out_dev, plain_out_dev, stream);
} catch (...) {
  return on_exception();
}

he_status he_aggregate_finalize(he_ctx* ctx, uint64_t n_ct, uint64_t n_plain, const uint32_t* acc_ct_dev,
                                const double* acc_plain_dev, uint32_t* ct_out_dev, float* plain_out_dev, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if ((n_ct && (!acc_ct_dev || !ct_out_dev)) || (n_plain && (!acc_plain_dev || !plain_out_dev)))
    return fail(HE_ERR_INVALID_ARG, "null argument");
  hipStream_t st = static_cast<hipStream_t>(stream);
  AggArgs a{};
  PlainArgs pa{};
  s = launch_agg(ctx, true, true, a, n_ct, acc_ct_dev, ct_out_dev, st);
  if (s != HE_OK) return s;
  return launch_plain(ctx, true, true, pa, n_plain, acc_plain_dev, nullptr, plain_out_dev, st);
} catch (...) {
  return on_exception();
}

// ---- client: decrypt + merge -----------------------------------------------------------

static he_status decrypt_merge_impl(he_ctx* ctx, const he_sk* sk, const he_mask* mask, uint32_t level,
                                    const uint32_t* ct_glob_dev, const float* plain_glob_dev, float* w_out_dev, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!sk || !mask || sk->ctx != ctx || mask->ctx != ctx) return fail(HE_ERR_INVALID_ARG, "key/mask missing or from another context");
  const MaskDev& mk = mask->dev;
  const uint64_t n_ct = he_n_ct(ctx, mask), n_plain = mk.P - mk.P_enc;
  if ((mk.P && !w_out_dev) || (n_ct && !ct_glob_dev) || (n_plain && !plain_glob_dev)) return fail(HE_ERR_INVALID_ARG, "null data pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const RingDev& rg = ctx->ring;
  if (level < 1 || level > rg.L) return fail(HE_ERR_LEVEL, "level must be in 1..L");
  const uint64_t chunk = std::min<uint64_t>(kCtChunk, n_ct);
  const size_t N = rg.N;
  // Under a fragmented mask the decoder writes the packed slot vector (as under the mask "the first P_enc entries"),
  // and one pass in parameter order weaves it and the remainder into the model.
  const bool weave = mk.bits && n_ct > 0 && n_plain > 0;
  const size_t d_bytes = ((chunk * level * N * 4 + 255) / 256) * 256;
  if (chunk) {
    s = ensure_ws(ctx, d_bytes + (weave ? mk.P_enc * sizeof(float) : 0));
    if (s != HE_OK) return s;
  }
  uint32_t* d = static_cast<uint32_t*>(ctx->ws);
  float* packed = weave ? reinterpret_cast<float*>(static_cast<char*>(ctx->ws) + d_bytes) : nullptr;
  MaskDev first_entries{};
  if (weave) {
    first_entries.start = mk.ident;
    first_entries.prefix = mk.ident + 1;
    first_entries.n_runs = 1;
    first_entries.P = first_entries.P_enc = mk.P_enc;
  }
  if (n_plain && !weave) {  // the scatter of the remainder writes other entries than the decoder does
    KernelTimer timer_(ctx, KID_PLAIN_MOVE, st);
    launch_plain_move<true>(mk, plain_glob_dev, w_out_dev, st);
    HIP_TRY(hipGetLastError());
  }
  for (uint64_t c0 = 0; c0 < n_ct; c0 += chunk) {
    const uint64_t cn = std::min<uint64_t>(chunk, n_ct - c0);
    s = launch_decrypt(ctx, sk, ct_glob_dev + c0 * 2 * level * N, cn, level, d, st);
    if (s != HE_OK) return s;
    s = launch_decode(ctx, level, weave ? first_entries : mk, d, c0, cn, weave ? packed : w_out_dev, nullptr, st);
    if (s != HE_OK) return s;
  }
  if (weave) {
    KernelTimer timer_(ctx, KID_PLAIN_MOVE, st);
    const uint64_t n_pchunks = (mk.P + kBitChunk - 1) / kBitChunk;
    hipLaunchKernelGGL(k_split_bits<true>, dim3((uint32_t)n_pchunks), dim3(256), 0, st, mk, (const float*)nullptr, w_out_dev,
                       (const float*)packed, (float*)nullptr, plain_glob_dev, (float*)nullptr);
    HIP_TRY(hipGetLastError());
  }
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_decrypt_merge(he_ctx* ctx, const he_sk* sk, const he_mask* mask, const uint32_t* ct_glob_dev,
                           const float* plain_glob_dev, float* w_out_dev, void* stream) try {
  if (!ctx) return fail(HE_ERR_INVALID_ARG, "context is null");
  return decrypt_merge_impl(ctx, sk, mask, ctx->ring.L - 1, ct_glob_dev, plain_glob_dev, w_out_dev, stream);
} catch (...) {
  return on_exception();
}

he_status he_decrypt_merge_level(he_ctx* ctx, const he_sk* sk, const he_mask* mask, uint32_t level,
                                 const uint32_t* ct_glob_dev, const float* plain_glob_dev, float* w_out_dev, void* stream) try {
  return decrypt_merge_impl(ctx, sk, mask, level, ct_glob_dev, plain_glob_dev, w_out_dev, stream);
} catch (...) {
  return on_exception();
}

// ---- test / measurement exports ---------------------------------------------------------

he_status he_debug_encode(he_ctx* ctx, const float* slots_dev, uint64_t n_ct, int32_t* m_out_dev, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (n_ct == 0) return HE_OK;
  if (!slots_dev || !m_out_dev) return fail(HE_ERR_INVALID_ARG, "null argument");
  if (n_ct >= (1ull << 31)) return fail(HE_ERR_INVALID_ARG, "too many ciphertexts");
  MaskDev mk{};
  return launch_encode(ctx, mk, nullptr, slots_dev, 0, n_ct, m_out_dev, nullptr, 0, 0, static_cast<hipStream_t>(stream));
} catch (...) {
  return on_exception();
}

he_status he_debug_encrypt_plain(he_ctx* ctx, const he_pk* pk, uint64_t seed, uint32_t client_id, uint64_t first_ct,
                                 const int32_t* m_dev, uint64_t n_ct, uint32_t* ct_out_dev, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (n_ct == 0) return HE_OK;
  if (!pk || pk->ctx != ctx || !m_dev || !ct_out_dev) return fail(HE_ERR_INVALID_ARG, "null argument or key from another context");
  if (first_ct + n_ct > (1ull << 32)) return fail(HE_ERR_INVALID_ARG, "ciphertext index out of range");
  if (reinterpret_cast<uintptr_t>(ct_out_dev) % 16 != 0) return fail(HE_ERR_INVALID_ARG, "ciphertext buffers must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const RingDev& rg = ctx->ring;
  const size_t N = rg.N;
  const uint64_t chunk = std::min<uint64_t>(kCtChunk, n_ct);
  s = ensure_ws(ctx, chunk * N * kEncScratchBytesPerCoeff);
  if (s != HE_OK) return s;
  const EncScratch sc = carve_enc_scratch(ctx->ws, chunk, N);
  for (uint64_t c0 = 0; c0 < n_ct; c0 += chunk) {
    const uint64_t cn = std::min<uint64_t>(chunk, n_ct - c0);
    s = launch_sample(ctx, seed, client_id, first_ct + c0, cn, sc, st);
    if (s != HE_OK) return s;
    s = launch_encrypt(ctx, pk, cn, m_dev + c0 * N, sc, ct_out_dev + c0 * 2 * rg.L * N, st);
    if (s != HE_OK) return s;
  }
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_debug_decrypt_residues(he_ctx* ctx, const he_sk* sk, const uint32_t* ct_dev, uint64_t n_ct, uint32_t level,
                                    uint32_t* d_out_dev, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (n_ct == 0) return HE_OK;
  if (!sk || sk->ctx != ctx || !ct_dev || !d_out_dev) return fail(HE_ERR_INVALID_ARG, "null argument or key from another context");
  if (level < 1 || level > ctx->ring.L) return fail(HE_ERR_LEVEL, "level must be in 1..L");
  if (n_ct >= 65536) {  // grid y limit: go chunk by chunk
    const size_t N = ctx->ring.N;
    for (uint64_t c0 = 0; c0 < n_ct; c0 += 32768) {
      const uint64_t cn = std::min<uint64_t>(32768, n_ct - c0);
      s = launch_decrypt(ctx, sk, ct_dev + c0 * 2 * level * N, cn, level, d_out_dev + c0 * level * N, static_cast<hipStream_t>(stream));
      if (s != HE_OK) return s;
    }
    return HE_OK;
  }
  return launch_decrypt(ctx, sk, ct_dev, n_ct, level, d_out_dev, static_cast<hipStream_t>(stream));
} catch (...) {
  return on_exception();
}

he_status he_debug_decode(he_ctx* ctx, const uint32_t* d_dev, uint64_t n_ct, uint32_t level, double* slots_out_dev,
                          void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (n_ct == 0) return HE_OK;
  if (!d_dev || !slots_out_dev) return fail(HE_ERR_INVALID_ARG, "null argument");
  if (level < 1 || level > ctx->ring.L) return fail(HE_ERR_LEVEL, "level must be in 1..L");
  if (n_ct >= (1ull << 31)) return fail(HE_ERR_INVALID_ARG, "too many ciphertexts");
  MaskDev mk{};
  return launch_decode(ctx, level, mk, d_dev, 0, n_ct, nullptr, slots_out_dev, static_cast<hipStream_t>(stream));
} catch (...) {
  return on_exception();
}

he_status he_debug_ntt(he_ctx* ctx, int inverse, uint32_t limb, uint32_t* polys_dev, uint64_t batch, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (batch == 0) return HE_OK;
  if (!polys_dev) return fail(HE_ERR_INVALID_ARG, "null argument");
  if (limb >= ctx->ring.L) return fail(HE_ERR_INVALID_ARG, "limb out of range");
  if (batch >= (1ull << 31)) return fail(HE_ERR_INVALID_ARG, "batch too large");
  const RingDev& rg = ctx->ring;
  hipStream_t st = static_cast<hipStream_t>(stream);
  KernelTimer timer_(ctx, KID_NTT, st);
  launch_ntt_batch(rg, inverse != 0, (int)limb, polys_dev, (uint32_t)batch, st);
  HIP_TRY(hipGetLastError());
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_debug_export_keys(he_ctx* ctx, const he_pk* pk, const he_sk* sk, uint32_t* pk_coeff_dev, int32_t* sk_coeff_dev,
                               void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const RingDev& rg = ctx->ring;
  if (pk_coeff_dev) {
    if (!pk || pk->ctx != ctx) return fail(HE_ERR_INVALID_ARG, "public key missing or from another context");
    HIP_TRY(hipMemcpyAsync(pk_coeff_dev, pk->raw, 2ull * rg.L * rg.N * 4, hipMemcpyDeviceToDevice, st));
    launch_ntt_batch(rg, true, -1, pk_coeff_dev, 2 * rg.L, st);
    HIP_TRY(hipGetLastError());
  }
  if (sk_coeff_dev) {
    if (!sk || sk->ctx != ctx) return fail(HE_ERR_INVALID_ARG, "secret key missing or from another context");
    hipLaunchKernelGGL(k_widen_i8, dim3((rg.N + 255) / 256), dim3(256), 0, st, sk->coeff, sk_coeff_dev, rg.N);
    HIP_TRY(hipGetLastError());
  }
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_debug_count_out_of_range(he_ctx* ctx, const float* w_dev, uint64_t n, uint64_t* count_host, void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!count_host || (n && !w_dev)) return fail(HE_ERR_INVALID_ARG, "null argument");
  *count_host = 0;
  if (n == 0) return HE_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  s = ensure_ws(ctx, 256);
  if (s != HE_OK) return s;
  unsigned long long* cnt = static_cast<unsigned long long*>(ctx->ws);
  hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, reinterpret_cast<uint32_t*>(cnt), (uint64_t)2, 0u);
  hipLaunchKernelGGL(k_count_out_of_range, dim3(grid_for(n, 256, 4096)), dim3(256), 0, st, w_dev, n,
                     std::ldexp(1.0, (int)ctx->ring.scale_bits), cnt);
  HIP_TRY(hipGetLastError());
  unsigned long long host = 0;
  HIP_TRY(hipMemcpyAsync(&host, cnt, sizeof(host), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  *count_host = host;
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_debug_count_noncanonical(he_ctx* ctx, const uint32_t* ct_dev, uint64_t n_ct, uint32_t level, uint64_t* count_host,
                                      void* stream) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!count_host || (n_ct && !ct_dev)) return fail(HE_ERR_INVALID_ARG, "null argument");
  if (level < 1 || level > ctx->ring.L) return fail(HE_ERR_LEVEL, "level must be in 1..L");
  *count_host = 0;
  if (n_ct == 0) return HE_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  s = ensure_ws(ctx, 256);
  if (s != HE_OK) return s;
  unsigned long long* cnt = static_cast<unsigned long long*>(ctx->ws);
  const uint64_t n_words = n_ct * 2 * level * ctx->ring.N;
  hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, reinterpret_cast<uint32_t*>(cnt), (uint64_t)2, 0u);
  hipLaunchKernelGGL(k_count_noncanonical, dim3(grid_for(n_words, 256, 8192)), dim3(256), 0, st, ctx->ring, ct_dev, n_words, level, cnt);
  HIP_TRY(hipGetLastError());
  unsigned long long host = 0;
  HIP_TRY(hipMemcpyAsync(&host, cnt, sizeof(host), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  *count_host = host;
  return HE_OK;
} catch (...) {
  return on_exception();
}

he_status he_debug_timing_enable(he_ctx* ctx, int on) try {
  if (!ctx) return fail(HE_ERR_INVALID_ARG, "context is null");
  ctx->timing_on = on != 0;
  return HE_OK;
} catch (...) {
  return on_exception();
}

uint32_t he_debug_timing_kernels(void) { return KID_COUNT; }

const char* he_debug_timing_name(uint32_t kernel_id) { return kernel_id < KID_COUNT ? kKernelNames[kernel_id] : ""; }

he_status he_debug_timing_read(he_ctx* ctx, double* ms_host, uint64_t* launches_host) try {
  he_status s = check_ctx(ctx);
  if (s != HE_OK) return s;
  if (!ms_host || !launches_host) return fail(HE_ERR_INVALID_ARG, "null argument");
  for (int k = 0; k < KID_COUNT; ++k) {
    ms_host[k] = 0.0;
    launches_host[k] = 0;
  }
  for (const TimedSpan& sp : ctx->spans) {
    HIP_TRY(hipEventSynchronize(sp.stop));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, sp.start, sp.stop));
    ms_host[sp.kid] += ms;
    launches_host[sp.kid] += 1;
    ctx->event_pool.push_back(sp.start);
    ctx->event_pool.push_back(sp.stop);
  }
  ctx->spans.clear();
  return HE_OK;
} catch (...) {
  return on_exception();
}

}  // extern "C"
