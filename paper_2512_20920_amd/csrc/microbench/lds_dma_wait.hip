// One wave issues a global->LDS load of a cold address, then an LDS read of another location and waits on the LDS
// counter (lgkmcnt), then waits on the memory counter (vmcnt).  Prints s_memtime ticks to each point: the first is the
// latency of an LDS read (the LDS counter does not wait for the outstanding global->LDS load), the second the latency
// of the load from HBM.
// Build: make -C paper_2512_20920_amd/csrc microbench; run: paper_2512_20920_amd/csrc/_build/lds_dma_wait
#include <hip/hip_runtime.h>
#include <stdio.h>
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
__global__ void __launch_bounds__(64) k(const unsigned char* src, unsigned long long* out, int far) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[8192];
  const int lane = threadIdx.x;
  ((unsigned*)smem)[lane] = lane; ((unsigned*)smem)[1024 + lane] = 0;
  __syncthreads();
  const unsigned long long a = (unsigned long long)src;
  u32x4 d = {(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a), (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32)), 0x40000000u, 0x00020000u};
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  unsigned voff = (unsigned)far + lane * 16;
  unsigned long long t0, t1, t2; unsigned v;
  unsigned ldsaddr = lds0 + lane * 4;
  asm volatile(
    "s_waitcnt vmcnt(0) lgkmcnt(0)\n\t"
    "s_memtime %0\n\t"
    "s_waitcnt lgkmcnt(0)\n\t"
    "s_mov_b32 m0, %5\n\t"
    "buffer_load_dwordx4 %4, %6, 0 offen lds\n\t"
    "ds_read_b32 %3, %7\n\t"
    "s_waitcnt lgkmcnt(0)\n\t"
    "s_memtime %1\n\t"
    "s_waitcnt lgkmcnt(0)\n\t"
    "s_waitcnt vmcnt(0)\n\t"
    "s_memtime %2\n\t"
    "s_waitcnt lgkmcnt(0)\n\t"
    : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&v"(v)
    : "v"(voff), "s"(lds0 + 4096), "s"(d), "v"(ldsaddr) : "memory", "m0");
  if (lane == 0) { out[0] = t1 - t0; out[1] = t2 - t0; out[2] = v; }
}
int main() {
  unsigned char* src; unsigned long long* out; unsigned long long h[3];
  const size_t bytes = 1u << 30;
  if (hipMalloc(&src, bytes) || hipMalloc(&out, 24)) return 1;
  (void)hipMemset(src, 1, bytes);
  (void)hipDeviceSynchronize();
  for (int i = 0; i < 6; i++) {
    int far = (int)((size_t)(i + 1) * 150000000u % (bytes - 4096)) & ~1023;      // a different cold address every time
    hipLaunchKernelGGL(k, dim3(1), dim3(64), 0, 0, src, out, far);
    (void)hipMemcpy(h, out, 24, hipMemcpyDeviceToHost);
    printf("cold address %10d: after ds_read + lgkmcnt(0): %llu ticks; after vmcnt(0): %llu ticks (s_memtime)\n", far, h[0], h[1]);
  }
  return 0;
}
