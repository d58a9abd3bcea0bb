// Issue-rate measurements on gfx950 (see include/he_issue_rates.h): what one wave64 vector instruction, and one
// modular butterfly in several instruction selections, costs a SIMD when 8 waves are resident.  These numbers are the
// evidence behind the integer-ALU peak (one instruction per 4 cycles per SIMD) of the transform kernels' rooflines
// and behind the choice of the min-based conditional subtraction over the carry-based one.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "he_issue_rates.h"

namespace {

constexpr int kIter = 1024;
constexpr uint32_t kQ = 2147352577u;  // a 31-bit prime of the library's chain (only its size matters here)

enum Op : int {
  OP_ADD, OP_SUB, OP_AND, OP_LSHR, OP_LSHL, OP_MIN, OP_ADD_SGPR, OP_CNDMASK_PAIR, OP_SUBMIN_PAIR, OP_ADD3, OP_BITOP3,
  OP_MUL_LO, OP_MUL_HI, OP_MAD64, OP_FMA64, OP_ALT_SUB_MIN, OP_COUNT_SINGLE
};

#define A1(s) asm volatile(s : "+v"(a[i]) : "v"(m), "v"(b[i]))
template <int OP>
__global__ void __launch_bounds__(256) k_single(uint32_t* out, uint32_t seed) {
  uint32_t a[8], b[8];
  uint64_t l[8];
  double d[8];
  for (int i = 0; i < 8; ++i) {
    a[i] = seed + threadIdx.x * 7 + i;
    b[i] = a[i] * 3 + 1;
    l[i] = a[i];
    d[i] = a[i] * 1e-3;
  }
  const uint32_t m = seed | 1;
  const double dm = 1.0000001, dc = 0.5;
  for (int it = 0; it < kIter; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (OP == OP_ADD) A1("v_add_u32 %0, %0, %1");
      if (OP == OP_SUB) A1("v_sub_u32 %0, %0, %1");
      if (OP == OP_AND) A1("v_and_b32 %0, %0, %1");
      if (OP == OP_LSHR) A1("v_lshrrev_b32 %0, 1, %0");
      if (OP == OP_LSHL) A1("v_lshlrev_b32 %0, 1, %0");
      if (OP == OP_MIN) A1("v_min_u32 %0, %0, %1");
      if (OP == OP_ADD_SGPR) asm volatile("v_add_u32 %0, %0, %1" : "+v"(a[i]) : "s"(m));
      if (OP == OP_CNDMASK_PAIR) asm volatile("v_sub_co_u32 %1, vcc, %0, %2\n\tv_cndmask_b32 %0, %1, %0, vcc" : "+v"(a[i]), "=&v"(b[i]) : "v"(m) : "vcc");
      if (OP == OP_SUBMIN_PAIR) asm volatile("v_sub_u32 %1, %0, %2\n\tv_min_u32 %0, %0, %1" : "+v"(a[i]), "=&v"(b[i]) : "v"(m));
      if (OP == OP_ADD3) A1("v_add3_u32 %0, %0, %1, %2");
      if (OP == OP_BITOP3) A1("v_bitop3_b32 %0, %0, %1, %2 bitop3:0x96");
      if (OP == OP_MUL_LO) A1("v_mul_lo_u32 %0, %0, %1");
      if (OP == OP_MUL_HI) A1("v_mul_hi_u32 %0, %0, %1");
      if (OP == OP_MAD64) asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %0" : "+v"(l[i]) : "v"(a[i]), "v"(m) : "vcc");
      if (OP == OP_FMA64) asm volatile("v_fma_f64 %0, %0, %1, %2" : "+v"(d[i]) : "v"(dm), "v"(dc));
      if (OP == OP_ALT_SUB_MIN) {  // a fast-class and a full-rate instruction alternating, independent of each other
        A1("v_sub_u32 %0, %0, %1");
        asm volatile("v_min_u32 %0, %0, %1" : "+v"(b[i]) : "v"(m));
      }
    }
  }
  uint32_t r = 0;
  for (int i = 0; i < 8; ++i) r ^= a[i] ^ b[i] ^ (uint32_t)l[i] ^ (uint32_t)d[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// ---- butterflies: 8 independent ones per loop iteration ----
__device__ __forceinline__ uint32_t csub_min(uint32_t x, uint32_t q) { return min(x, x - q); }
__device__ __forceinline__ uint32_t csub_carry(uint32_t x, uint32_t q) {
  uint32_t t;
  return __builtin_usub_overflow(x, q, &t) ? x : t;
}
__device__ __forceinline__ uint32_t shoup_lazy(uint32_t y, uint32_t w, uint32_t wp, uint32_t q) {
  const uint32_t hi = __umulhi(wp, y);
  uint64_t acc = (uint64_t)w * y;
  acc += (uint64_t)hi * (uint32_t)(0u - q);
  asm("" : "+v"(acc));
  return (uint32_t)acc;
}
// CARRY: conditional subtraction by borrow and select, modulus in a vector register; otherwise subtraction and
// minimum, modulus in a scalar register (the library's form).
template <bool INV, bool CARRY>
__global__ void __launch_bounds__(256) k_bfly(uint32_t* out, uint32_t seed, uint32_t q_s, uint32_t w, uint32_t wp) {
  uint32_t x[8], y[8];
  for (int i = 0; i < 8; ++i) {
    x[i] = (seed + threadIdx.x * 7919u + i * 104729u + blockIdx.x) % q_s;
    y[i] = (x[i] * 3u + 12345u) % q_s;
  }
  uint32_t q = q_s;
  if (CARRY) asm volatile("v_mov_b32 %0, %1" : "=v"(q) : "s"(q_s));
  for (int it = 0; it < kIter; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (!INV) {
        const uint32_t t0 = shoup_lazy(y[i], w, wp, q);
        const uint32_t t = CARRY ? csub_carry(t0, q) : csub_min(t0, q);
        const uint32_t a = x[i];
        if (CARRY) {
          x[i] = csub_carry(a + t, q);
          uint32_t d;
          y[i] = __builtin_usub_overflow(a, t, &d) ? d + q : d;
        } else {
          x[i] = csub_min(a + t, q);
          const uint32_t d = a - t;
          y[i] = min(d, d + q);
        }
      } else {
        const uint32_t a = x[i], b = y[i];
        x[i] = CARRY ? csub_carry(a + b, q) : csub_min(a + b, q);
        const uint32_t t0 = shoup_lazy(a - b + q, w, wp, q);
        y[i] = CARRY ? csub_carry(t0, q) : csub_min(t0, q);
      }
    }
  }
  uint32_t r = 0;
  for (int i = 0; i < 8; ++i) r = r * 31u + x[i] + 7u * y[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

struct Entry {
  const char* name;
  uint32_t instructions;  // vector instructions per unit
  uint32_t units_per_iter;
  void (*launch)(uint32_t*, int);
};

constexpr int kBlocks = 4096;  // x 4 waves: every SIMD keeps its 8 wave slots full for the whole run
template <int OP>
void launch_single(uint32_t* out, int) { hipLaunchKernelGGL(k_single<OP>, dim3(kBlocks), dim3(256), 0, 0, out, 12345u); }
template <bool INV, bool CARRY>
void launch_bfly(uint32_t* out, int) {
  const uint32_t w = 1234567891u % kQ, wp = (uint32_t)(((uint64_t)w << 32) / kQ);
  hipLaunchKernelGGL((k_bfly<INV, CARRY>), dim3(kBlocks), dim3(256), 0, 0, out, 99u, kQ, w, wp);
}

const Entry kEntries[] = {
    {"v_add_u32", 1, 8, launch_single<OP_ADD>},
    {"v_sub_u32", 1, 8, launch_single<OP_SUB>},
    {"v_and_b32", 1, 8, launch_single<OP_AND>},
    {"v_lshrrev_b32", 1, 8, launch_single<OP_LSHR>},
    {"v_lshlrev_b32", 1, 8, launch_single<OP_LSHL>},
    {"v_min_u32", 1, 8, launch_single<OP_MIN>},
    {"v_add_u32 with a scalar-register operand", 1, 8, launch_single<OP_ADD_SGPR>},
    {"v_sub_co_u32 + v_cndmask_b32 (conditional subtraction by borrow)", 2, 8, launch_single<OP_CNDMASK_PAIR>},
    {"v_sub_u32 + v_min_u32 (conditional subtraction by minimum)", 2, 8, launch_single<OP_SUBMIN_PAIR>},
    {"v_add3_u32", 1, 8, launch_single<OP_ADD3>},
    {"v_bitop3_b32", 1, 8, launch_single<OP_BITOP3>},
    {"v_mul_lo_u32", 1, 8, launch_single<OP_MUL_LO>},
    {"v_mul_hi_u32", 1, 8, launch_single<OP_MUL_HI>},
    {"v_mad_u64_u32", 1, 8, launch_single<OP_MAD64>},
    {"v_fma_f64", 1, 8, launch_single<OP_FMA64>},
    {"v_sub_u32 and v_min_u32 alternating (independent)", 2, 8, launch_single<OP_ALT_SUB_MIN>},
    {"butterfly forward, min-based, modulus scalar (library form)", 11, 8, launch_bfly<false, false>},
    {"butterfly forward, borrow-based, modulus vector", 11, 8, launch_bfly<false, true>},
    {"butterfly inverse, min-based, modulus scalar (library form)", 10, 8, launch_bfly<true, false>},
    {"butterfly inverse, borrow-based, modulus vector", 10, 8, launch_bfly<true, true>},
};
constexpr uint32_t kCount = sizeof(kEntries) / sizeof(kEntries[0]);

}  // namespace

extern "C" {

uint32_t he_issue_rates_count(void) { return kCount; }
const char* he_issue_rates_name(uint32_t i) { return i < kCount ? kEntries[i].name : ""; }
uint32_t he_issue_rates_instructions(uint32_t i) { return i < kCount ? kEntries[i].instructions : 0; }

int he_issue_rates_run(int device, double* ns_per_unit_host, uint32_t* n_simd_host) {
  if (!ns_per_unit_host || !n_simd_host) return (int)hipErrorInvalidValue;
  hipError_t e = hipSetDevice(device);
  if (e != hipSuccess) return (int)e;
  hipDeviceProp_t prop;
  if ((e = hipGetDeviceProperties(&prop, device)) != hipSuccess) return (int)e;
  const uint32_t n_simd = 4u * (uint32_t)prop.multiProcessorCount;
  *n_simd_host = n_simd;
  uint32_t* out = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if ((e = hipMalloc(&out, (size_t)kBlocks * 256 * 4)) != hipSuccess) return (int)e;
  if ((e = hipEventCreate(&e0)) == hipSuccess) e = hipEventCreate(&e1);
  for (uint32_t i = 0; e == hipSuccess && i < kCount; ++i) {
    float best = 1e30f;
    for (int rep = 0; rep < 3 && e == hipSuccess; ++rep) {
      if ((e = hipEventRecord(e0, 0)) != hipSuccess) break;
      kEntries[i].launch(out, 0);
      if ((e = hipGetLastError()) != hipSuccess) break;
      if ((e = hipEventRecord(e1, 0)) != hipSuccess) break;
      if ((e = hipEventSynchronize(e1)) != hipSuccess) break;
      float ms = 0.f;
      if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) break;
      if (ms < best) best = ms;
    }
    const double units = (double)kBlocks * 4.0 * kIter * kEntries[i].units_per_iter;  // wave-level units issued chip-wide
    ns_per_unit_host[i] = (double)best * 1e6 * n_simd / units;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(out);
  return (int)e;
}

}  // extern "C"
