// Encryption-mask agreement on the GPU: Select(global privacy map, p) of Algorithm 1 ("Server
// Encryption Mask Aggregation"; Section "Selective Parameter Encryption", Step 2: the mask takes
// the ratio p of the most sensitive parameters), and the conversion of a selection into the run
// list that the mask object holds.
//
//   1. radix select: the k-th largest value of a float32 vector in three histogram passes over
//      order-preserving 32-bit keys (11 + 11 + 10 bits, most significant first);
//   2. mark: element i is selected iff key_i > T, or key_i == T and it is among the first r such
//      elements in index order (ties go to the lower index), written as a byte mask;
//   3. runs: starts and ends of the maximal runs of non-zero bytes, by per-chunk counts, an
//      exclusive scan over the chunks and an emit pass.
//
// Every pass is a unit-stride stream over the vector: 4 B per parameter for each of the three
// histogram passes and the mark pass (plus one more when ties must be ranked), 1 B per parameter
// for each of the two run passes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace he_sel {

constexpr int kThreads = 256, kItems = 8, kChunk = kThreads * kItems;  // elements per workgroup

struct SelState {
  uint32_t prefix;   // key bits fixed so far
  uint32_t pad;
  uint64_t k_rem;    // rank still to be resolved inside the current prefix (1-based, from the top)
  uint64_t cnt_eq;   // after the last pass: number of elements whose key equals the threshold
};

// Larger float <-> larger key; -0.0 and +0.0 share a key (x + 0.0f is +0.0 for both).
__device__ __forceinline__ uint32_t float_key(float x) {
  const uint32_t b = __float_as_uint(x + 0.0f);
  return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

template <int SHIFT, int BITS>
__global__ void __launch_bounds__(kThreads)
k_hist(const float* __restrict__ s, uint64_t P, const SelState* __restrict__ st, uint32_t prefix_mask,
       unsigned long long* __restrict__ hist) {
  __shared__ uint32_t lh[1 << BITS];
  for (int b = threadIdx.x; b < (1 << BITS); b += kThreads) lh[b] = 0;
  __syncthreads();
  const uint32_t prefix = st->prefix;
  const uint64_t stride = (uint64_t)gridDim.x * kThreads;
  for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < P; i += stride) {
    const uint32_t key = float_key(s[i]);
    if ((key & prefix_mask) == prefix) atomicAdd(&lh[(key >> SHIFT) & ((1u << BITS) - 1u)], 1u);
  }
  __syncthreads();
  for (int b = threadIdx.x; b < (1 << BITS); b += kThreads)
    if (lh[b]) atomicAdd(&hist[b], (unsigned long long)lh[b]);
}

// One thread: walks the digit histogram from the top until the remaining rank falls inside a bin.
template <int SHIFT, int BITS>
__global__ void k_pick(const unsigned long long* __restrict__ hist, SelState* st) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const uint64_t k = st->k_rem;
  uint64_t cum = 0;
  for (int d = (1 << BITS) - 1; d >= 0; --d) {
    const uint64_t c = hist[d];
    if (cum + c >= k) {
      st->prefix |= (uint32_t)d << SHIFT;
      st->k_rem = k - cum;
      st->cnt_eq = c;
      return;
    }
    cum += c;
  }
}

// Exclusive prefix sum inside a workgroup of kThreads threads (wave shuffles, then LDS across waves).
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* total) {
  __shared__ uint32_t wave_sum[kThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(inc, d, 64);
    if (lane >= d) inc += t;
  }
  __syncthreads();  // wave_sum may still be read from an earlier call
  if (lane == 63) wave_sum[wave] = inc;
  __syncthreads();
  uint32_t base = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) {
    if (w < wave) base += wave_sum[w];
    all += wave_sum[w];
  }
  *total = all;
  return base + inc - v;
}

// Per chunk: how many keys equal the threshold (only needed when not all of them are taken).
__global__ void __launch_bounds__(kThreads)
k_count_eq(const float* __restrict__ s, uint64_t P, const SelState* __restrict__ st, uint32_t* __restrict__ eq_count) {
  const uint32_t T = st->prefix;
  const uint64_t base = (uint64_t)blockIdx.x * kChunk + (uint64_t)threadIdx.x * kItems;
  uint32_t c = 0;
#pragma unroll
  for (int e = 0; e < kItems; ++e)
    if (base + e < P && float_key(s[base + e]) == T) ++c;
  uint32_t total;
  block_exclusive_scan(c, &total);
  if (threadIdx.x == 0) eq_count[blockIdx.x] = total;
}

// Exclusive scan of n 32-bit counts into 64-bit offsets; out[n] = grand total.  One workgroup.
__global__ void __launch_bounds__(1024)
k_scan_counts(const uint32_t* __restrict__ in, uint64_t n, uint64_t* __restrict__ out) {
  __shared__ uint64_t part[1024];
  const uint64_t per = (n + 1023) / 1024;
  const uint64_t lo = min(n, (uint64_t)threadIdx.x * per), hi = min(n, lo + per);
  uint64_t sum = 0;
  for (uint64_t i = lo; i < hi; ++i) sum += in[i];
  part[threadIdx.x] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint64_t run = 0;
    for (int t = 0; t < 1024; ++t) {
      const uint64_t v = part[t];
      part[t] = run;
      run += v;
    }
    out[n] = run;
  }
  __syncthreads();
  uint64_t run = part[threadIdx.x];
  for (uint64_t i = lo; i < hi; ++i) {
    out[i] = run;
    run += in[i];
  }
}

// Byte mask of the selection.  eq_off == nullptr: every element equal to the threshold is taken.
__global__ void __launch_bounds__(kThreads)
k_mark(const float* __restrict__ s, uint64_t P, const SelState* __restrict__ st, const uint64_t* __restrict__ eq_off,
       uint8_t* __restrict__ mask) {
  const uint32_t T = st->prefix;
  const uint64_t r = st->k_rem;
  const uint64_t base = (uint64_t)blockIdx.x * kChunk + (uint64_t)threadIdx.x * kItems;
  uint32_t keys[kItems];
  uint32_t c = 0;
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    keys[e] = base + e < P ? float_key(s[base + e]) : 0u;
    if (base + e < P && keys[e] == T) ++c;
  }
  uint64_t rank = 0;
  if (eq_off) {
    uint32_t total;
    rank = eq_off[blockIdx.x] + block_exclusive_scan(c, &total);
  }
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    if (base + e >= P) break;
    bool sel = keys[e] > T;
    if (keys[e] == T) {
      sel = eq_off ? rank < r : true;
      ++rank;
    }
    mask[base + e] = sel ? 1 : 0;
  }
}

// Run boundaries of a byte mask: a run starts at i if m[i] and not m[i-1], ends after i if m[i] and
// not m[i+1].  EMIT = false counts them per chunk, EMIT = true writes start / end positions at the
// chunk's offsets (exclusive scans of the counts).
template <bool EMIT>
__global__ void __launch_bounds__(kThreads)
k_runs(const uint8_t* __restrict__ m, uint64_t P, uint32_t* __restrict__ n_start, uint32_t* __restrict__ n_end,
       const uint64_t* __restrict__ off_start, const uint64_t* __restrict__ off_end, uint64_t* __restrict__ starts,
       uint64_t* __restrict__ ends) {
  const uint64_t base = (uint64_t)blockIdx.x * kChunk + (uint64_t)threadIdx.x * kItems;
  bool prev = base > 0 && base - 1 < P && m[base - 1] != 0;
  uint8_t v[kItems + 1];
#pragma unroll
  for (int e = 0; e <= kItems; ++e) v[e] = base + e < P ? m[base + e] : 0;
  uint32_t cs = 0, ce = 0;
  bool p = prev;
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    const bool cur = v[e] != 0, nxt = v[e + 1] != 0;
    if (cur && !p) ++cs;
    if (cur && !nxt) ++ce;
    p = cur;
  }
  uint32_t ts, te;
  const uint32_t xs = block_exclusive_scan(cs, &ts);
  const uint32_t xe = block_exclusive_scan(ce, &te);
  if (!EMIT) {
    if (threadIdx.x == 0) {
      n_start[blockIdx.x] = ts;
      n_end[blockIdx.x] = te;
    }
    return;
  }
  uint64_t ws = off_start[blockIdx.x] + xs, we = off_end[blockIdx.x] + xe;
  p = prev;
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    const bool cur = v[e] != 0, nxt = v[e + 1] != 0;
    if (cur && !p) starts[ws++] = base + e;
    if (cur && !nxt) ends[we++] = base + e + 1;
    p = cur;
  }
}

}  // namespace he_sel
