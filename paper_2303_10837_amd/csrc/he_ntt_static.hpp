// Compile-time specialised negacyclic NTT passes for the tuned ring sizes (N = 2^11 ... 2^14).
//
// Same mathematics as the generic passes in he_device.hpp; what changes is that the ring
// size, the pass plan and the workgroup size are template parameters, so that
//   * every LDS access is `group base + immediate offset` (no per-element index arithmetic),
//   * passes whose twiddles are the same for a whole wavefront fetch them with scalar loads,
//   * the last forward pass, the pointwise key product and the first inverse pass of the
//     encrypt / decrypt pipelines run back to back in registers (same group geometry),
//   * passes 1..3 work on blocks that one wavefront owns, so only pass 0 needs workgroup
//     barriers (see owned_group), and
//   * the Shoup products take three instructions (mul_shoup_mad).
//
// Plan: N = 2^14 -> stages 4+4+3+3 (strides 1024, 64, 8, 1); N = 2^13 -> 4+3+3+3 (512, 64, 8, 1);
// N = 2^12 -> 2+4+3+3 (1024, 64, 8, 1); N = 2^11 -> 1+4+3+3 (1024, 64, 8, 1).  The last pass always works on groups of
// 8 (the fused middle of the encrypt / decrypt pipelines), and the blocks that passes 1..3 stay inside hold at least
// 1024 coefficients, so that every pass has whole wavefronts of groups per block.
// N/16 threads per workgroup: every thread owns 16 coefficients per pass.
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

template <>
struct NttPlan<12> {
  static constexpr int kPasses = 4;
  static constexpr int R[4] = {2, 4, 3, 3};
  static constexpr int S[4] = {0, 2, 6, 9};
  static constexpr int NT = 256;
};
template <>
struct NttPlan<11> {
  static constexpr int kPasses = 4;
  static constexpr int R[4] = {1, 4, 3, 3};
  static constexpr int S[4] = {0, 1, 5, 8};
  static constexpr int NT = 128;
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
//
// Forward stages leave an output in [0, 2q) instead of [0, q) when its only next use is as the
// multiplicand of a Shoup product (which accepts any 32-bit value): inside a pass that is
// every element whose index has the next stage's pairing bit set (both outputs of a butterfly
// share that bit); after the last stage of a pass only when the caller says so (LAZY_LAST: the
// pass is followed by a pointwise key product).  Such a butterfly costs 8 instructions, not 11.
//
// SCALE_LAST (inverse, pass 0 only): the factor 1/N of a standalone inverse transform rides on the last stage, whose
// twiddle is then psi^-bitrev(1) / N and whose sum output takes a Shoup product by 1/N in place of its conditional
// subtraction (13 instructions for that butterfly instead of 10 and a separate product on both outputs).
template <int LOGN, int S0, int R, bool INV, int NP, bool LAZY_LAST = false, bool SCALE_LAST = false>
__device__ __forceinline__ void bfly_stages(uint32_t (&v)[NP][1 << R], int b, const uint2* __restrict__ tw, uint32_t q,
                                            uint2 n_inv = uint2{0, 0}, uint2 w1_n_inv = uint2{0, 0}) {
  static_assert(!SCALE_LAST || (INV && S0 == 0), "the scaled last stage is stage 0 of the inverse");
  using G = PassGeom<LOGN, S0, R>;
  constexpr int E = 1 << R;
  const int bb = (S0 == 0) ? 0 : (G::UNIFORM ? __builtin_amdgcn_readfirstlane(b) : b);
  constexpr bool WS = (S0 == 0) || G::UNIFORM;  // twiddles are wave-uniform: scalar registers
  if (!INV) {
#pragma unroll
    for (int k = 0; k < R; ++k) {
      const int half = E >> (k + 1);
      const uint2* twk = tw + (1 << (S0 + k)) + (bb << k);
#pragma unroll
      for (int i = 0; i < E; ++i) {
        if (i & half) continue;
        const uint2 w = twk[i >> (R - k)];
        const bool lazy = (k + 1 < R) ? ((i & (half >> 1)) != 0) : LAZY_LAST;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const uint32_t t = mul_shoup_mad<WS>(v[p][i + half], w, q);
          const uint32_t x = v[p][i];
          if (lazy) {
            v[p][i] = x + t;             // [0, 2q)
            v[p][i + half] = x - t + q;  // (0, 2q)
          } else {
            v[p][i] = add_mod(x, t, q);
            v[p][i + half] = sub_mod(x, t, q);
          }
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
        const uint2 w = (SCALE_LAST && k == 0) ? w1_n_inv : twk[i >> (R - k)];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const uint32_t x = v[p][i], y = v[p][i + half];
          if (SCALE_LAST && k == 0) v[p][i] = mul_shoup_mad<true>(x + y, n_inv, q);  // x + y < 2q: any 32-bit value is fine
          else v[p][i] = add_mod(x, y, q);
          v[p][i + half] = mul_shoup_mad<WS>(x - y + q, w, q);
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

// Passes 1..3 never leave a block of N >> S[1] consecutive coefficients (pass 1 starts at stage S[1]: N/16 coefficients
// for N = 2^13 and 2^14, 1024 for the smaller rings), and one such block is a whole number of wavefronts of groups in
// each of these passes.  Wave w of a workgroup of NT
// threads therefore OWNS blocks w, w + NT/64, ... through passes 1, 2 and 3 of the forward
// transform and 3, 2, 1 of the inverse: the data it reads in one of these passes was written by
// itself in the previous one, so those passes are separated by a wavefront-level ordering point
// only, and a workgroup barrier is needed just around pass 0 (stride N/16, the whole polynomial).
// owned_group(it) is the group index of this thread's it-th group of pass PASS.
template <int LOGN, int PASS, int NT>
__device__ __forceinline__ int owned_group(int it) {
  using P = NttPlan<LOGN>;
  static_assert(PASS >= 1, "blocks start at pass 1");
  constexpr int GPB = ((1 << LOGN) >> P::S[1]) >> P::R[PASS];  // groups per block in this pass
  constexpr int NW = NT / 64;
  static_assert(NT % 64 == 0 && (1 << P::S[1]) % NW == 0 && GPB % 64 == 0, "whole wavefronts per block");
  const int local = it * 64 + (int)(threadIdx.x & 63);
  return ((int)(threadIdx.x >> 6) + NW * (local / GPB)) * GPB + (local % GPB);
}
template <int LOGN, int PASS, int NT>
struct OwnedIters {
  static constexpr int value = (1 << (LOGN - NttPlan<LOGN>::R[PASS])) / NT;
  static_assert((1 << (LOGN - NttPlan<LOGN>::R[PASS])) % NT == 0, "whole iterations");
};

// Ordering point between two passes that stay inside wave-owned blocks: this wavefront's LDS
// writes are ordered before its later LDS reads.  No other wave is involved, so no s_barrier; the
// fence is restricted to LDS so that global loads and stores stay in flight across it.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup", "local");
  __builtin_amdgcn_wave_barrier();
}

// One LDS -> LDS pass (1, 2 or 3) over NP buffers that share twiddles, on the groups this
// wavefront owns.  No barrier inside.
template <int LOGN, int PASS, bool INV, int NP, int NT = NttPlan<LOGN>::NT>
__device__ __forceinline__ void lds_pass(uint32_t* const (&x)[NP], const uint2* __restrict__ tw, uint32_t q) {
  using P = NttPlan<LOGN>;
  constexpr int S0 = P::S[PASS], R = P::R[PASS];
  using G = PassGeom<LOGN, S0, R>;
#pragma unroll
  for (int it = 0; it < OwnedIters<LOGN, PASS, NT>::value; ++it) {
    const int g = owned_group<LOGN, PASS, NT>(it);
    uint32_t v[NP][1 << R];
#pragma unroll
    for (int p = 0; p < NP; ++p) lds_load_group<LOGN, S0, R>(x[p], g, v[p]);
    bfly_stages<LOGN, S0, R, INV, NP>(v, G::block(g), tw, q);
#pragma unroll
    for (int p = 0; p < NP; ++p) lds_store_group<LOGN, S0, R>(x[p], g, v[p]);
  }
}

// Forward transform of one polynomial: first pass reads through ld0(index), passes 0..2 end
// in LDS buffer x.  The LAST pass is left to the caller (it is fused with whatever follows);
// it must run on the caller's owned groups of pass 3, after which no barrier is needed either.
template <int LOGN, int NT = NttPlan<LOGN>::NT, class Load0>
__device__ __forceinline__ void fwd_head(uint32_t* x, const uint2* __restrict__ tw, uint32_t q, Load0 ld0) {
  using P = NttPlan<LOGN>;
  {
    constexpr int R = P::R[0];
    using G = PassGeom<LOGN, 0, R>;
#pragma unroll
    for (int g = threadIdx.x; g < G::GROUPS; g += NT) {
      uint32_t v[1][1 << R];
#pragma unroll
      for (int i = 0; i < G::E; ++i) v[0][i] = ld0(g + (i << G::LSTRIDE));
      bfly_stages<LOGN, 0, R, false, 1>(v, 0, tw, q);
      lds_store_group<LOGN, 0, R>(x, g, v[0]);
    }
  }
  __syncthreads();
  uint32_t* const xs[1] = {x};
  lds_pass<LOGN, 1, false, 1, NT>(xs, tw, q);
  wave_lds_sync();
  lds_pass<LOGN, 2, false, 1, NT>(xs, tw, q);
  wave_lds_sync();
}

// Inverse passes 2 and 1 over NP buffers, on owned groups; the caller does the inverse of pass
// 3 before (fused, on its owned groups, no barrier in between) and of pass 0 after (fused with
// the store).  Ends with the workgroup barrier that pass 0 needs.
template <int LOGN, int NP, int NT = NttPlan<LOGN>::NT>
__device__ __forceinline__ void inv_middle(uint32_t* const (&x)[NP], const uint2* __restrict__ tw, uint32_t q) {
  wave_lds_sync();
  lds_pass<LOGN, 2, true, NP, NT>(x, tw, q);
  wave_lds_sync();
  lds_pass<LOGN, 1, true, NP, NT>(x, tw, q);
  __syncthreads();
}

}  // namespace he
