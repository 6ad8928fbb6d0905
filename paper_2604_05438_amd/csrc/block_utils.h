// Workgroup-level primitives for 256-thread workgroups (4 wavefronts of 64 lanes).
#pragma once

#include "tkphi_internal.h"

namespace tkphi {

// inclusive prefix sum over threadIdx.x; sh must hold >= 4 ints; contains two barriers
__device__ __forceinline__ int block_scan_incl(int v, int* sh) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int x = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int y = __shfl_up(x, o);
    if (lane >= o) x += y;
  }
  if (lane == 63) sh[w] = x;
  __syncthreads();
  int add = 0;
  for (int i = 0; i < w; ++i) add += sh[i];
  __syncthreads();
  return x + add;
}

// sum over the workgroup, result in every thread; sh must hold >= 4 floats; two barriers
__device__ __forceinline__ float block_sum(float v, float* sh) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  const float r = (sh[0] + sh[1]) + (sh[2] + sh[3]);
  __syncthreads();
  return r;
}

__device__ __forceinline__ int block_sum_int(int v, int* sh) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  const int r = sh[0] + sh[1] + sh[2] + sh[3];
  __syncthreads();
  return r;
}

__device__ __forceinline__ float block_max(float v, float* sh) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  const float r = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  __syncthreads();
  return r;
}

}  // namespace tkphi
