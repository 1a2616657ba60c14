// Matrix-core issue rate on gfx950, nothing but v_mfma_f32_32x32x16_bf16 in the loop (operands stay in registers):
// one workgroup alone (1 or 2 waves per SIMD, 1/2/4 independent accumulators) and one workgroup on every CU, with zero
// and with random operand data.  Prints ns per MFMA per SIMD; 32 clocks at 2.4 GHz = 13.3 ns is the published peak
// (2.5 PFLOP/s over 256 CUs x 4 SIMDs).  With random data on all CUs the figure is what the power limit leaves.
// Build: make -C paper_2512_20920_amd/csrc microbench; run: paper_2512_20920_amd/csrc/_build/mfma_rate
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
template <int NACC>
__global__ void __launch_bounds__(512) mfma_k(const unsigned* seed, float* out, int iters, int random) {
  unsigned h = (threadIdx.x + blockIdx.x * 256) * 2654435761u + seed[0];
  bf16x8 a[NACC], b[NACC];
  for (int i = 0; i < NACC; i++) for (int q = 0; q < 8; q++) {
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    float fa = random ? ((int)(h & 0xffff) - 32768) / 32768.f : 0.f;
    float fb = random ? ((int)(h >> 16) - 32768) / 32768.f : 0.f;
    a[i][q] = (__bf16)fa; b[i][q] = (__bf16)fb;
  }
  f32x16 acc[NACC];
  for (int i = 0; i < NACC; i++) for (int e = 0; e < 16; e++) acc[i][e] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int r = 0; r < 8; r++)
#pragma unroll
      for (int i = 0; i < NACC; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < NACC; i++) s += acc[i][0];
  if (s == 12345.678f) out[0] = s;
}
template <int NACC> void run(int blocks, int threads, int random, unsigned* seed, float* out) {
  const int iters = 20000;
  hipEvent_t a, b; (void)hipEventCreate(&a); (void)hipEventCreate(&b);
  hipLaunchKernelGGL(mfma_k<NACC>, dim3(blocks), dim3(threads), 0, 0, seed, out, 100, random);
  (void)hipEventRecord(a, 0);
  hipLaunchKernelGGL(mfma_k<NACC>, dim3(blocks), dim3(threads), 0, 0, seed, out, iters, random);
  (void)hipEventRecord(b, 0); (void)hipEventSynchronize(b);
  float ms; (void)hipEventElapsedTime(&ms, a, b);
  const double per_simd = (double)iters * 8 * NACC * (threads / 256);     // MFMAs issued on one SIMD
  printf("blocks %4d threads %4d acc %2d %s: %8.1f us  %.2f ns per MFMA per SIMD = %.1f clk at 2.4 GHz\n", blocks, threads, NACC, random ? "random" : "zero  ", ms * 1e3, ms * 1e6 / per_simd, ms * 1e6 / per_simd * 2.4);
  fflush(stdout);
}
int main() {
  unsigned* seed; float* out; (void)hipMalloc(&seed, 4); (void)hipMalloc(&out, 4); (void)hipMemset(seed, 1, 4);
  for (int random = 0; random < 2; random++) {
    run<1>(1, 256, random, seed, out); run<2>(1, 256, random, seed, out); run<4>(1, 256, random, seed, out);
    run<1>(1, 512, random, seed, out); run<2>(1, 512, random, seed, out); run<4>(1, 512, random, seed, out);
    run<2>(256, 512, random, seed, out); run<4>(256, 512, random, seed, out);
  }
  return 0;
}
