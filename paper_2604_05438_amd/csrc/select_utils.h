// Workgroup-level pieces of the Top-K selection shared by the spill pipeline's kernels
// (topk_select.hip) and the fused select + gather kernel of the filtered pipeline
// (select_gather.hip): workgroup-wide prefix sums, the (score key, lower index first) composite and
// the radix search for the n-th largest composite.
#pragma once

#include "tkphi_internal.h"

namespace tkphi {

constexpr int kSelWaves = kSelThreads / 64;

// inclusive prefix sum over the threads of the workgroup; sh must hold one int per wavefront; two barriers (ordering LDS only)
__device__ __forceinline__ int sel_scan_incl(int v, int* sh) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int x = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int y = __shfl_up(x, o);
    if (lane >= o) x += y;
  }
  if (lane == 63) sh[w] = x;
  lds_barrier();
  int add = 0;
  for (int i = 0; i < w; ++i) add += sh[i];
  lds_barrier();
  return x + add;
}

__device__ __forceinline__ uint64_t composite(uint32_t key, uint32_t row) {
  return ((uint64_t)key << 32) | (uint64_t)(0xffffffffu - row);
}

// `want`-th largest (1-based) 64-bit composite among `count` elements delivered by
// get(j, &composite) -> bool (false: element does not take part).  8 radix passes of 8
// bits.  All threads must call; returns the composite in every thread.
template <typename Get>
__device__ uint64_t radix_select_desc(int count, int want, Get get, uint32_t* sh_hist /*[256]*/,
                                      int* sh_scan /*[16]*/, uint64_t* sh_prefix, int* sh_want) {
  const int tid = threadIdx.x;
  if (tid == 0) { *sh_prefix = 0ull; *sh_want = want; }
  __syncthreads();
  for (int shift = 56; shift >= 0; shift -= 8) {
    if (tid < 256) sh_hist[tid] = 0u;
    __syncthreads();
    const uint64_t prefix = *sh_prefix;
    const int w = *sh_want;
    const uint64_t himask = shift == 56 ? 0ull : (~0ull << (shift + 8));
    for (int j = tid; j < count; j += (int)blockDim.x) {
      uint64_t v;
      if (get(j, &v) && (v & himask) == prefix) atomicAdd(&sh_hist[(uint32_t)(v >> shift) & 255u], 1u);
    }
    __syncthreads();
    // thread t < 256 looks at digit 255 - t: prefix scan over t == suffix scan over digits
    const int digit = 255 - tid;
    const int c = tid < 256 ? (int)sh_hist[digit] : 0;
    const int incl = sel_scan_incl(c, sh_scan);
    const int excl = incl - c;
    if (tid < 256 && excl < w && w <= incl) {
      *sh_prefix = prefix | ((uint64_t)digit << shift);
      *sh_want = w - excl;
    }
    __syncthreads();
  }
  return *sh_prefix;
}


// monotone map of a score key to [0, kFineBins): sign, 16 exponents, 6 mantissa bits (four times the
// resolution of key_bin: the boundary bin of the fused select kernel holds ~100 candidates, not ~400)
constexpr int kFineBins = 2048;
__device__ __forceinline__ int fine_bin(uint32_t key) {
  const bool pos = (key & 0x80000000u) != 0;
  const uint32_t mag = pos ? (key & 0x7fffffffu) : (~key & 0x7fffffffu);
  const int e = (int)(mag >> 23);
  const int m6 = (int)((mag >> 17) & 63u);
  const int half = kFineBins / 2;
  const int mb = e < kExpLo ? 0 : e > kExpHi ? half - 1 : (e - kExpLo) * 64 + m6;
  return pos ? half + mb : half - 1 - mb;
}

// The binning the fused select kernel uses.  All candidates of a head have keys >= the head's sampled bound, and
// most lie within an octave above it: measured from the bound, 2^13 key units (1024 bins per octave of the score)
// per bin spread them over about a thousand bins, so the histogram's LDS atomics rarely collide and the
// boundary bin holds a handful of candidates instead of ~100.  Keys further up share the top bin.  Without a
// usable bound (no pruning, or after a rescan) the fixed map applies.  Monotone in the key either way.
struct SelBins {
  uint32_t edge;
  bool relative;
  __device__ __forceinline__ int operator()(uint32_t key) const {
    if (!relative) return fine_bin(key);
    return key >= edge ? (int)min((key - edge) >> 13, (uint32_t)(kFineBins - 1)) : 0;
  }
};

}  // namespace tkphi
