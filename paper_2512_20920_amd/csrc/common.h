// Shared device/host helpers for the RevFFN HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef long long i64;

#define WAVE 64

template <class T> __device__ __forceinline__ float to_f(T v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f(float v) { return (T)v; }

// xor-butterfly over the 64 lanes: every lane ends with the same, order-fixed sum
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// Block-wide sum for blockDim.x = 256 (4 waves); result valid in every thread.
// red must point at >= 4 floats of LDS.  Fixed combination order -> deterministic.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

__device__ __forceinline__ float sigmoid_f(float x) { return 1.0f / (1.0f + __expf(-x)); }

static inline int cdiv(i64 a, i64 b) { return (int)((a + b - 1) / b); }

// A kernel's dynamic-LDS limit is an attribute per device: `mask` (one per kernel instantiation) keeps one bit per
// device id.  attr_needed: the current device has not been marked yet (the caller sets the attribute, then calls
// attr_done; several threads may do so at once, which is harmless, and none launches before its own call returned).
#include <atomic>
static inline bool attr_needed(const std::atomic<unsigned long long>& mask) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return true;
  return (mask.load(std::memory_order_acquire) & (1ull << dev)) == 0;
}
static inline void attr_done(std::atomic<unsigned long long>& mask) {
  int dev = 0;
  if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev <= 63) mask.fetch_or(1ull << dev, std::memory_order_acq_rel);
}
