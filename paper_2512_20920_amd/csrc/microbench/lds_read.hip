// LDS reads per CU: 1 to 16 waves, each issuing ds_read_b128 (or b64) one after the other, every read waited for before
// the next (lanes in address order, no bank conflicts).  With few waves the figure is the latency of one read
// (1 KiB / (B/clk of one wave)); with 16 waves it approaches what the LDS delivers per clock.
// Build: make -C paper_2512_20920_amd/csrc microbench; run: paper_2512_20920_amd/csrc/_build/lds_read
#include <hip/hip_runtime.h>
#include <stdio.h>
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
template <int MODE>
__global__ void __launch_bounds__(1024) rd_k(unsigned* sink, int iters) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  for (int i = threadIdx.x; i < 16384; i += blockDim.x) ((unsigned*)smem)[i] = i;
  __syncthreads();
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  unsigned acc = 0;
  unsigned off = (wv * 4096 + lane * 16) & 65535;
  for (int it = 0; it < iters; it++) {
    if (MODE == 0) {
#pragma unroll
      for (int u = 0; u < 8; u++) {
        u32x4 v = *(const u32x4*)(smem + ((off + u * 1024) & 65535));
        asm volatile("" :: "v"(v));
      }
    } else {
#pragma unroll
      for (int u = 0; u < 8; u++) {
        u32x2 v = *(const u32x2*)(smem + ((wv * 4096 + lane * 8 + u * 512) & 65535));
        asm volatile("" :: "v"(v));
      }
    }
  }
  if (acc == 0x1234567u) sink[0] = acc;
}
int main() {
  unsigned* sink; if (hipMalloc(&sink, 4)) return 1;
  hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  auto run = [&](const char* name, auto kern, int threads, int bytes_per_lane_iter) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
    const int iters = 20000;
    hipLaunchKernelGGL(kern, dim3(256), dim3(threads), 65536, 0, sink, 100);
    (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0);
    hipLaunchKernelGGL(kern, dim3(256), dim3(threads), 65536, 0, sink, iters);
    (void)hipEventRecord(e1); (void)hipEventSynchronize(e1);
    float ms; (void)hipEventElapsedTime(&ms, e0, e1);
    const double by = (double)threads * bytes_per_lane_iter * iters;      // per CU
    printf("%-18s %4d threads  %8.1f us  %6.1f B/clk/CU at 2.4 GHz  (%.1f GB/s/CU) err=%d\n", name, threads, ms * 1e3, by / (ms * 1e-3) / 2.4e9, by / (ms * 1e-3) / 1e9, (int)hipGetLastError());
    fflush(stdout);
  };
  for (int th : {64, 128, 256, 512, 1024}) run("ds_read_b128", rd_k<0>, th, 128);
  for (int th : {256, 512, 1024}) run("ds_read_b64", rd_k<1>, th, 64);
  return 0;
}
