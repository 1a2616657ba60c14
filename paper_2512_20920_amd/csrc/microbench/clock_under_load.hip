// Core clock under load, and how matrix-core and vector work of ONE wave overlap.  A wave runs, per iteration, 16 MFMAs
// (v_mfma_f32_32x32x16_bf16), or 128 independent fused multiply-adds, or both interleaved (one MFMA, eight multiply-adds,
// sixteen times), or 32 independent exp2.  It reads the shader clock counter (s_memtime) and the constant 100 MHz counter
// (s_memrealtime) around the loop: their ratio is the clock the CU actually ran at.  With two waves per SIMD the span from
// the first wave's start to the last wave's end shows how much of the two waves' work the SIMD overlapped.  One workgroup alone and one on every
// CU, one and two waves per SIMD, random operand data.
// Build: make -C paper_2512_20920_amd/csrc microbench; run: paper_2512_20920_amd/csrc/_build/clock_under_load
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
#define FMA8 z0 = __builtin_fmaf(z0, 1.0001f, 0.5f); z1 = __builtin_fmaf(z1, 1.0001f, 0.5f); z2 = __builtin_fmaf(z2, 1.0001f, 0.5f); \
             z3 = __builtin_fmaf(z3, 1.0001f, 0.5f); z4 = __builtin_fmaf(z4, 1.0001f, 0.5f); z5 = __builtin_fmaf(z5, 1.0001f, 0.5f); \
             z6 = __builtin_fmaf(z6, 1.0001f, 0.5f); z7 = __builtin_fmaf(z7, 1.0001f, 0.5f);
template <int mode>
__global__ void __launch_bounds__(512) k(const unsigned* seed, float* out, unsigned long long* t, int iters) {
  unsigned h = (threadIdx.x + blockIdx.x * 256) * 2654435761u + seed[0];
  bf16x8 a[4], b[4];
  for (int i = 0; i < 4; i++) for (int q = 0; q < 8; q++) {
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    a[i][q] = (__bf16)(((int)(h & 0xffff) - 32768) / 32768.f);
    b[i][q] = (__bf16)(((int)(h >> 16) - 32768) / 32768.f);
  }
  f32x16 acc[4];
  for (int i = 0; i < 4; i++) for (int e = 0; e < 16; e++) acc[i][e] = 0.f;
  float x = (float)threadIdx.x * 1e-3f, y = 0.f;
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; it++) {
    float z0 = x, z1 = y, z2 = x + 1.f, z3 = y + 1.f, z4 = x + 2.f, z5 = y + 2.f, z6 = x + 3.f, z7 = y + 3.f;
    if constexpr (mode == 0) {
#pragma unroll
      for (int r = 0; r < 16; r++) acc[r & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r & 3], b[r & 3], acc[r & 3], 0, 0, 0);
    } else if constexpr (mode == 1) {
#pragma unroll
      for (int r = 0; r < 16; r++) { FMA8 }
    } else if constexpr (mode == 2) {
#pragma unroll
      for (int r = 0; r < 16; r++) {
        acc[r & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r & 3], b[r & 3], acc[r & 3], 0, 0, 0);
        FMA8
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 4; r++) {
        z0 = __builtin_amdgcn_exp2f(z0); z1 = __builtin_amdgcn_exp2f(z1); z2 = __builtin_amdgcn_exp2f(z2); z3 = __builtin_amdgcn_exp2f(z3);
        z4 = __builtin_amdgcn_exp2f(z4); z5 = __builtin_amdgcn_exp2f(z5); z6 = __builtin_amdgcn_exp2f(z6); z7 = __builtin_amdgcn_exp2f(z7);
      }
    }
    x = (z0 + z1 + z2 + z3) * 1e-9f; y = (z4 + z5 + z6 + z7) * 1e-9f;
  }
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float s = x + y;
  for (int i = 0; i < 4; i++) s += acc[i][0];
  if (s == 12345.678f) out[0] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) { t[0] = c1 - c0; t[1] = r1 - r0; }
  if (blockIdx.x == 0 && (threadIdx.x & 63) == 0) { t[2 + 2 * (threadIdx.x >> 6)] = c0; t[3 + 2 * (threadIdx.x >> 6)] = c1; }
}
int main() {
  unsigned* seed; float* out; unsigned long long* t; unsigned long long h[18];
  (void)hipMalloc(&seed, 4); (void)hipMalloc(&out, 4); (void)hipMalloc(&t, 18 * 8); (void)hipMemset(seed, 1, 4);
  const char* names[4] = {"16 MFMA", "128 FMA", "16 MFMA + 128 FMA interleaved", "32 exp2"};
  for (int blocks : {1, 256}) for (int threads : {256, 512}) for (int mode = 0; mode < 4; mode++) {
    const int iters = 20000;
    auto kern = mode == 0 ? k<0> : mode == 1 ? k<1> : mode == 2 ? k<2> : k<3>;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, seed, out, t, 200);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, seed, out, t, iters);
    (void)hipMemcpy(h, t, 18 * 8, hipMemcpyDeviceToHost);
    unsigned long long lo = ~0ull, hi = 0;
    for (int w = 0; w < threads / 64; w++) { lo = h[2 + 2 * w] < lo ? h[2 + 2 * w] : lo; hi = h[3 + 2 * w] > hi ? h[3 + 2 * w] : hi; }
    printf("workgroups %3d, waves per SIMD %d, %-30s: %6.0f clocks per iteration (first wave), %6.0f (first start to last end, all waves of the workgroup), clock %.2f GHz\n",
           blocks, threads / 256, names[mode], (double)h[0] / iters, (double)(hi - lo) / iters, (double)h[0] / (double)h[1] * 0.1);
    fflush(stdout);
  }
  return 0;
}
