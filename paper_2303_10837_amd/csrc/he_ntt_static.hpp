// Compile-time specialised negacyclic NTT passes for the tuned ring sizes (N = 2^13, 2^14).
//
// Same mathematics as the generic passes in he_device.hpp; what changes is that the ring
// size, the pass plan and the workgroup size are template parameters, so that
//   * every LDS access is `group base + immediate offset` (no per-element index arithmetic),
//   * passes whose twiddles are the same for a whole wavefront fetch them with scalar loads,
//   * the last forward pass, the pointwise key product and the first inverse pass of the
//     encrypt / decrypt pipelines run back to back in registers (same group geometry), and
//   * several polynomials that share twiddles (c0 and c1 of one ciphertext) go through the
//     inverse passes together.
//
// Plan: N = 2^14 -> stages 4+4+3+3 (strides 1024, 64, 8, 1); N = 2^13 -> 4+3+3+3 (512, 64, 8, 1).
// Every thread owns 16 coefficients per pass (one group of 16 or two groups of 8).
#pragma once
#include "he_device.hpp"

namespace he {

// 8 pad words per 64: the stride-8 pass then maps 8 consecutive groups (64 lanes) onto 64
// distinct banks, and the other passes stay unit-stride across lanes.
constexpr int kSPad = 8;
__host__ __device__ __forceinline__ constexpr int spad(int a) { return a + ((a >> 6) * kSPad); }

template <int LOGN>
struct NttPlan;
template <>
struct NttPlan<14> {
  static constexpr int kPasses = 4;
  static constexpr int R[4] = {4, 4, 3, 3};
  static constexpr int S[4] = {0, 4, 8, 11};
  static constexpr int NT = 1024;
};
template <>
struct NttPlan<13> {
  static constexpr int kPasses = 4;
  static constexpr int R[4] = {4, 3, 3, 3};
  static constexpr int S[4] = {0, 4, 7, 10};
  static constexpr int NT = 512;
};

template <int LOGN, int S0, int R>
struct PassGeom {
  static constexpr int E = 1 << R;
  static constexpr int LSTRIDE = LOGN - S0 - R;
  static constexpr int STRIDE = 1 << LSTRIDE;
  static constexpr int GROUPS = 1 << (LOGN - R);
  static constexpr bool UNIFORM = LSTRIDE >= 6;  // one twiddle set per wavefront
  __device__ static __forceinline__ int block(int g) { return g >> LSTRIDE; }
  __device__ static __forceinline__ int base(int g) { return ((g >> LSTRIDE) << (LOGN - S0)) + (g & (STRIDE - 1)); }
};

// R butterfly stages on NP register-resident groups that share their twiddles.
template <int LOGN, int S0, int R, bool INV, int NP>
__device__ __forceinline__ void bfly_stages(uint32_t (&v)[NP][1 << R], int b, const uint2* __restrict__ tw, uint32_t q) {
  using G = PassGeom<LOGN, S0, R>;
  constexpr int E = 1 << R;
  const int bb = (S0 == 0) ? 0 : (G::UNIFORM ? __builtin_amdgcn_readfirstlane(b) : b);
  if (!INV) {
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const int half = E >> (k + 1);
      const uint2* twk = tw + (1 << (S0 + k)) + (bb << k);
#pragma unroll
      for (int i = 0; i < E; ++i) {
        if (i & half) continue;
        const uint2 w = twk[i >> (R - k)];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const uint32_t t = mul_shoup(v[p][i + half], w, q);
          const uint32_t x = v[p][i];
          v[p][i] = add_mod(x, t, q);
          v[p][i + half] = sub_mod(x, t, q);
        }
      }
    }
  } else {
#pragma unroll
    for (int k = R - 1; k >= 0; --k) {
      const int half = E >> (k + 1);
      const uint2* twk = tw + (1 << (S0 + k)) + (bb << k);
#pragma unroll
      for (int i = 0; i < E; ++i) {
        if (i & half) continue;
        const uint2 w = twk[i >> (R - k)];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const uint32_t x = v[p][i], y = v[p][i + half];
          v[p][i] = add_mod(x, y, q);
          v[p][i + half] = mul_shoup(x - y + q, w, q);
        }
      }
    }
  }
}

template <int LOGN, int S0, int R>
__device__ __forceinline__ void lds_load_group(const uint32_t* x, int g, uint32_t (&v)[1 << R]) {
  using G = PassGeom<LOGN, S0, R>;
  const uint32_t* p = x + spad(G::base(g));
  if constexpr (G::STRIDE == 1 && (G::E % 4) == 0) {
#pragma unroll
    for (int i = 0; i < G::E; i += 4) {
      const uint4 t = *reinterpret_cast<const uint4*>(p + i);
      v[i] = t.x; v[i + 1] = t.y; v[i + 2] = t.z; v[i + 3] = t.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < G::E; ++i) v[i] = p[spad(i << G::LSTRIDE)];
  }
}

template <int LOGN, int S0, int R>
__device__ __forceinline__ void lds_store_group(uint32_t* x, int g, const uint32_t (&v)[1 << R]) {
  using G = PassGeom<LOGN, S0, R>;
  uint32_t* p = x + spad(G::base(g));
  if constexpr (G::STRIDE == 1 && (G::E % 4) == 0) {
#pragma unroll
    for (int i = 0; i < G::E; i += 4) *reinterpret_cast<uint4*>(p + i) = make_uint4(v[i], v[i + 1], v[i + 2], v[i + 3]);
  } else {
#pragma unroll
    for (int i = 0; i < G::E; ++i) p[spad(i << G::LSTRIDE)] = v[i];
  }
}

// One LDS -> LDS pass over NP buffers that share twiddles.  No barrier inside.
template <int LOGN, int PASS, bool INV, int NP>
__device__ __forceinline__ void lds_pass(uint32_t* const (&x)[NP], const uint2* __restrict__ tw, uint32_t q) {
  using P = NttPlan<LOGN>;
  constexpr int S0 = P::S[PASS], R = P::R[PASS];
  using G = PassGeom<LOGN, S0, R>;
  for (int g = threadIdx.x; g < G::GROUPS; g += P::NT) {
    uint32_t v[NP][1 << R];
#pragma unroll
    for (int p = 0; p < NP; ++p) lds_load_group<LOGN, S0, R>(x[p], g, v[p]);
    bfly_stages<LOGN, S0, R, INV, NP>(v, G::block(g), tw, q);
#pragma unroll
    for (int p = 0; p < NP; ++p) lds_store_group<LOGN, S0, R>(x[p], g, v[p]);
  }
}

// Forward transform of one polynomial: first pass reads through ld0(index), passes 0..2 end
// in LDS buffer x (each followed by a barrier).  The LAST pass is left to the caller (it is
// fused with whatever follows); use fwd_last_group() for it.
template <int LOGN, class Load0>
__device__ __forceinline__ void fwd_head(uint32_t* x, const uint2* __restrict__ tw, uint32_t q, Load0 ld0) {
  using P = NttPlan<LOGN>;
  {
    constexpr int R = P::R[0];
    using G = PassGeom<LOGN, 0, R>;
    for (int g = threadIdx.x; g < G::GROUPS; g += P::NT) {
      uint32_t v[1][1 << R];
#pragma unroll
      for (int i = 0; i < G::E; ++i) v[0][i] = ld0(g + (i << G::LSTRIDE));
      bfly_stages<LOGN, 0, R, false, 1>(v, 0, tw, q);
      lds_store_group<LOGN, 0, R>(x, g, v[0]);
    }
  }
  __syncthreads();
  uint32_t* const xs[1] = {x};
  lds_pass<LOGN, 1, false, 1>(xs, tw, q);
  __syncthreads();
  lds_pass<LOGN, 2, false, 1>(xs, tw, q);
  __syncthreads();
}

// Inverse passes 2 and 1 over NP buffers (each followed by a barrier); the caller does the
// inverse of pass 3 before (fused) and of pass 0 after (fused with the store).
template <int LOGN, int NP>
__device__ __forceinline__ void inv_middle(uint32_t* const (&x)[NP], const uint2* __restrict__ tw, uint32_t q) {
  lds_pass<LOGN, 2, true, NP>(x, tw, q);
  __syncthreads();
  lds_pass<LOGN, 1, true, NP>(x, tw, q);
  __syncthreads();
}

}  // namespace he
