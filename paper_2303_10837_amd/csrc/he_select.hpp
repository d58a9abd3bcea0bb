// Encryption-mask agreement on the GPU: Select(global privacy map, p) of Algorithm 1 ("Server
// Encryption Mask Aggregation"; Section "Selective Parameter Encryption", Step 2: the mask takes
// the ratio p of the most sensitive parameters), and the conversion of a selection into the run
// list that the mask object holds.
//
//   1. radix select: the k-th largest value of a float32 vector in three histogram passes over
//      order-preserving 32-bit keys (11 + 11 + 10 bits, most significant first);
//   2. mark: element i is selected iff key_i > T, or key_i == T and it is among the first r such
//      elements in index order (ties go to the lower index), written as a byte mask;
//   3. runs: the maximal runs of non-zero bytes and of zero bytes with their packed offsets -- the tables of the
//      mask object -- by per-chunk counts, exclusive scans over the chunks and an emit pass, all on the device.
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

// Digit histogram of the keys that carry the prefix fixed so far.  Sensitivities of one layer share their leading key
// bits, so most lanes of a wavefront fall into one or two bins: the lanes that share the bin of the first live lane
// are counted with one ballot and added by that lane alone (twice), and only what is left takes an atomic per lane.
template <int SHIFT, int BITS>
__global__ void __launch_bounds__(kThreads)
k_hist(const float* __restrict__ s, uint64_t P, const SelState* __restrict__ st, uint32_t prefix_mask,
       unsigned long long* __restrict__ hist) {
  __shared__ uint32_t lh[1 << BITS];
  for (int b = threadIdx.x; b < (1 << BITS); b += kThreads) lh[b] = 0;
  __syncthreads();
  const uint32_t prefix = st->prefix;
  const uint32_t lane = threadIdx.x & 63;
  auto tally = [&](float x) {  // called by every lane that is still in the loop
    const uint32_t key = float_key(x);
    const uint32_t bin = (key >> SHIFT) & ((1u << BITS) - 1u);
    bool live = (key & prefix_mask) == prefix;
#pragma unroll
    for (int round = 0; round < 2; ++round) {
      const uint64_t live_mask = __ballot(live);
      if (live_mask == 0) break;  // wave-uniform
      const uint32_t lead = (uint32_t)__ffsll((long long)live_mask) - 1u;
      const uint32_t lead_bin = __shfl(bin, (int)lead, 64);
      const bool same = live && bin == lead_bin;
      const uint64_t same_mask = __ballot(same);
      if (lane == lead) atomicAdd(&lh[lead_bin], (uint32_t)__popcll(same_mask));
      live = live && !same;
    }
    if (live) atomicAdd(&lh[bin], 1u);
  };
  const uint64_t stride = (uint64_t)gridDim.x * kThreads, first = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if ((reinterpret_cast<uintptr_t>(s) & 15u) == 0) {  // 16-byte loads, then the last P mod 4 elements one by one
    const uint64_t n4 = P / 4;
    const float4* __restrict__ s4 = reinterpret_cast<const float4*>(s);
    for (uint64_t i = first; i < n4; i += stride) {
      const float4 x = s4[i];
      tally(x.x);
      tally(x.y);
      tally(x.z);
      tally(x.w);
    }
    for (uint64_t i = 4 * n4 + first; i < P; i += stride) tally(s[i]);
  } else {
    for (uint64_t i = first; i < P; i += stride) tally(s[i]);
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

// Keys of the kItems consecutive elements from `base` on (0 past the end of the vector, where `live` is false): two
// 16-byte loads when the thread's elements are all inside the vector and the vector is 16-byte aligned.
__device__ __forceinline__ void load_keys(const float* __restrict__ s, uint64_t P, uint64_t base, uint32_t (&keys)[kItems],
                                          bool (&live)[kItems]) {
  static_assert(kItems == 8, "two float4 loads");
  if (base + kItems <= P && (reinterpret_cast<uintptr_t>(s) & 15u) == 0) {
    const float4 a = *reinterpret_cast<const float4*>(s + base), b = *reinterpret_cast<const float4*>(s + base + 4);
    const float x[kItems] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      keys[e] = float_key(x[e]);
      live[e] = true;
    }
  } else {
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      live[e] = base + e < P;
      keys[e] = live[e] ? float_key(s[base + e]) : 0u;
    }
  }
}

// Per chunk: how many keys equal the threshold (only needed when not all of them are taken).
__global__ void __launch_bounds__(kThreads)
k_count_eq(const float* __restrict__ s, uint64_t P, const SelState* __restrict__ st, uint32_t* __restrict__ eq_count) {
  const uint32_t T = st->prefix;
  const uint64_t base = (uint64_t)blockIdx.x * kChunk + (uint64_t)threadIdx.x * kItems;
  uint32_t keys[kItems];
  bool live[kItems];
  load_keys(s, P, base, keys, live);
  uint32_t c = 0;
#pragma unroll
  for (int e = 0; e < kItems; ++e)
    if (live[e] && keys[e] == T) ++c;
  uint32_t total;
  block_exclusive_scan(c, &total);
  if (threadIdx.x == 0) eq_count[blockIdx.x] = total;
}

// Exclusive scan of n 32-bit counts into 64-bit offsets; out[n] = grand total.  One workgroup walks the array in tiles of
// 1024 consecutive counts (unit-stride loads and stores), a running 64-bit carry in front of each tile's block scan.
// Workgroup b of the launch scans the b-th array: in + b * in_stride words into out + b * out_stride words.
__global__ void __launch_bounds__(1024)
k_scan_counts(const uint32_t* __restrict__ in, uint64_t n, uint64_t* __restrict__ out, uint64_t in_stride, uint64_t out_stride) {
  __shared__ uint32_t wave_sum[16];
  in += blockIdx.x * in_stride;
  out += blockIdx.x * out_stride;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint64_t carry = 0;
  for (uint64_t t0 = 0; t0 < n; t0 += 1024) {
    const uint64_t i = t0 + threadIdx.x;
    const uint32_t v = i < n ? in[i] : 0u;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t t = __shfl_up(inc, d, 64);
      if (lane >= d) inc += t;
    }
    __syncthreads();  // wave_sum of the previous tile has been read
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    uint32_t base = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      if (w < wave) base += wave_sum[w];
      all += wave_sum[w];
    }
    if (i < n) out[i] = carry + base + inc - v;
    carry += all;
  }
  if (threadIdx.x == 0) out[n] = carry;
}

// Byte mask of the selection.  eq_off == nullptr: every element equal to the threshold is taken.
__global__ void __launch_bounds__(kThreads)
k_mark(const float* __restrict__ s, uint64_t P, const SelState* __restrict__ st, const uint64_t* __restrict__ eq_off,
       uint8_t* __restrict__ mask) {
  const uint32_t T = st->prefix;
  const uint64_t r = st->k_rem;
  const uint64_t base = (uint64_t)blockIdx.x * kChunk + (uint64_t)threadIdx.x * kItems;
  uint32_t keys[kItems];
  bool live[kItems];
  load_keys(s, P, base, keys, live);
  uint32_t c = 0;
#pragma unroll
  for (int e = 0; e < kItems; ++e)
    if (live[e] && keys[e] == T) ++c;
  uint64_t rank = 0;
  if (eq_off) {
    uint32_t total;
    rank = eq_off[blockIdx.x] + block_exclusive_scan(c, &total);
  }
  uint64_t bytes = 0;  // the thread's kItems mask bytes, lowest address in the lowest byte
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    bool sel = live[e] && keys[e] > T;
    if (live[e] && keys[e] == T) {
      sel = eq_off ? rank < r : true;
      ++rank;
    }
    bytes |= (uint64_t)(sel ? 1u : 0u) << (8 * e);
  }
  if (live[kItems - 1] && (reinterpret_cast<uintptr_t>(mask) & 7u) == 0) {
    *reinterpret_cast<uint64_t*>(mask + base) = bytes;
  } else {
#pragma unroll
    for (int e = 0; e < kItems; ++e)
      if (live[e]) mask[base + e] = (uint8_t)(bytes >> (8 * e));
  }
}

// Run boundaries of a byte mask: a run starts at i if m[i] and not m[i-1], ends after i if m[i] and
// not m[i+1].  EMIT = false counts run starts, run ends and set bytes per chunk; EMIT = true writes, at the chunk's
// offsets (exclusive scans of those counts), the tables a mask object keeps on the device:
//   start[r], prefix[r]    first position of masked run r and the number of masked positions before it,
//   cstart[c], cprefix[c]  the same for the runs of the complement (c counts from 1 when the vector starts unmasked:
//                          entry 0 is then the run at position 0, written by the first thread).
// A complement run starts where a masked run ends (unless that is the end of the vector).
template <bool EMIT>
__global__ void __launch_bounds__(kThreads)
k_runs(const uint8_t* __restrict__ m, uint64_t P, uint32_t* __restrict__ n_start, uint32_t* __restrict__ n_end,
       uint32_t* __restrict__ n_set, const uint64_t* __restrict__ off_start, const uint64_t* __restrict__ off_end,
       const uint64_t* __restrict__ off_set, uint64_t* __restrict__ start, uint64_t* __restrict__ prefix,
       uint64_t* __restrict__ cstart, uint64_t* __restrict__ cprefix) {
  const uint64_t base = (uint64_t)blockIdx.x * kChunk + (uint64_t)threadIdx.x * kItems;
  const bool prev = base > 0 && base - 1 < P && m[base - 1] != 0;
  uint8_t v[kItems + 1];
  static_assert(kItems == 8, "one 8-byte load");
  if (base + kItems < P && (reinterpret_cast<uintptr_t>(m) & 7u) == 0) {
    const uint64_t w = *reinterpret_cast<const uint64_t*>(m + base);
#pragma unroll
    for (int e = 0; e < kItems; ++e) v[e] = (uint8_t)(w >> (8 * e));
    v[kItems] = m[base + kItems];
  } else {
#pragma unroll
    for (int e = 0; e <= kItems; ++e) v[e] = base + e < P ? m[base + e] : 0;
  }
  uint32_t cs = 0, ce = 0, cn = 0;
  bool p = prev;
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    const bool cur = v[e] != 0, nxt = v[e + 1] != 0;
    if (cur && !p) ++cs;
    if (cur && !nxt) ++ce;
    if (cur) ++cn;
    p = cur;
  }
  uint32_t ts, te, tn;
  const uint32_t xs = block_exclusive_scan(cs, &ts);
  const uint32_t xe = block_exclusive_scan(ce, &te);
  const uint32_t xn = block_exclusive_scan(cn, &tn);
  if (!EMIT) {
    if (threadIdx.x == 0) {
      n_start[blockIdx.x] = ts;
      n_end[blockIdx.x] = te;
      n_set[blockIdx.x] = tn;
    }
    return;
  }
  const uint64_t c_first = m[0] != 0 ? 0 : 1;  // the complement's run at position 0, if the vector starts unmasked
  if (blockIdx.x == 0 && threadIdx.x == 0 && c_first) {
    cstart[0] = 0;
    cprefix[0] = 0;
  }
  uint64_t ws = off_start[blockIdx.x] + xs, we = off_end[blockIdx.x] + xe + c_first, set_before = off_set[blockIdx.x] + xn;
  p = prev;
#pragma unroll
  for (int e = 0; e < kItems; ++e) {
    const bool cur = v[e] != 0, nxt = v[e + 1] != 0;
    if (cur && !p) {
      start[ws] = base + e;
      prefix[ws] = set_before;
      ++ws;
    }
    if (cur) ++set_before;
    if (cur && !nxt) {
      if (base + e + 1 < P) {
        cstart[we] = base + e + 1;
        cprefix[we] = base + e + 1 - set_before;
      }
      ++we;
    }
    p = cur;
  }
}

}  // namespace he_sel
