// Rate of the direct global -> LDS path (buffer_load_dwordx4 ... lds) for the operand traffic of a 2048^3 GEMM with
// 128x128 tiles and k-step 64: 256 workgroups, each streaming its A and B tile k-slab by k-slab through NS LDS stages
// with one barrier per k-step and no arithmetic.  "strided": operands as row-major matrices (128 bytes per row per
// k-step, row stride 4 KiB); "packed": each tile's 16 KiB k-slab contiguous.  xcd=1: each XCD takes a 4 x 8 rectangle of
// tiles (operands shared inside one L2).  Prints bytes landed in LDS per second and per clock per CU.
// Build: make -C paper_2512_20920_amd/csrc microbench; run: paper_2512_20920_amd/csrc/_build/lds_stream
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
__device__ __forceinline__ void load_lds_b128(u32x4 desc, unsigned lds_addr, unsigned voff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(lds_addr), "v"(voff), "s"(desc) : "memory", "m0");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
__device__ __forceinline__ u32x4 make_desc(const void* p, unsigned bytes) {
  const unsigned long long a = (unsigned long long)p;
  u32x4 d = {(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a), (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32)), bytes, 0x00020000u};
  return d;
}
// mode 0: row-strided (row stride ld bytes, 128 B per row per k-tile); mode 1: packed panels (16 KiB per k-tile contiguous)
// grid: tiles_n x tiles_m workgroups (1-D, XCD round robin as the hardware does), 512 threads, NS stages of 32 KiB
template <int NS, int MODE>
__global__ void __launch_bounds__(512) stream_k(const unsigned char* A, const unsigned char* B, unsigned bytesA, unsigned bytesB,
                                                int tiles_n, int nk, unsigned ld, unsigned* sink, int xcd) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  int wg = blockIdx.x;
  if (xcd) {            // XCD x gets a rectangle of the tile grid: 4 tile rows x 8 tile columns (for 16 x 16 tiles)
    const int x = wg & 7, i = wg >> 3;        // i = 0..31 within the XCD
    const int by = (x >> 1) * 4 + (i >> 3), bx = (x & 1) * 8 + (i & 7);
    wg = by * tiles_n + bx;
  }
  const int bx = wg % tiles_n, by = wg / tiles_n;
  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const u32x4 da = make_desc(A, bytesA), db = make_desc(B, bytesB);
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  unsigned base[4];
  const bool isA = wv < 4;     // waves 0-3 load the A tile (16 wave-loads), 4-7 the B tile
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int j = (wv & 3) * 4 + i;           // wave-load 0..15 of the operand tile: rows 8j .. 8j+7
    const int pos = j * 64 + lane, r = pos >> 3, c = (pos & 7) ^ ((r >> 1) & 7);
    const int t = isA ? by : bx;
    if (MODE == 0) base[i] = (unsigned)(t * 128 + r) * ld + c * 16;
    else base[i] = (unsigned)t * (unsigned)nk * 16384u + r * 128 + c * 16;
  }
  const unsigned kstep = MODE == 0 ? 128u : 16384u;
  const unsigned lw = __builtin_amdgcn_readfirstlane(lds0 + (unsigned)wv * 4096u);
  auto issue = [&](int kt, int i) {
    const unsigned off = kt < nk ? base[i] + (unsigned)kt * kstep : 0x80000000u;
    load_lds_b128(isA ? da : db, lw + (unsigned)(kt % NS) * 32768u + i * 1024, off);
  };
#pragma unroll
  for (int p = 0; p < NS - 1; p++)
#pragma unroll
    for (int i = 0; i < 4; i++) issue(p, i);
  unsigned acc = 0;
  for (int kt = 0; kt < nk; kt++) {
    wait_vmcnt<4 * (NS - 2)>();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    acc += *(const unsigned*)(smem + (kt % NS) * 32768 + threadIdx.x * 64);
#pragma unroll
    for (int i = 0; i < 4; i++) issue(kt + NS - 1, i);
  }
  wait_vmcnt<0>();
  if (acc == 0x12345678u) sink[0] = acc;
}
int main(int argc, char** argv) {
  const int Mrows = 2048, K = 2048, tiles = 16, nk = K / 64;
  const size_t bytes = (size_t)Mrows * K * 2;
  unsigned char *A, *B; unsigned* sink;
  if (hipMalloc(&A, bytes) || hipMalloc(&B, bytes) || hipMalloc(&sink, 4)) return 1;
  hipMemset(A, 1, bytes); hipMemset(B, 2, bytes);
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  auto run = [&](const char* name, auto kern, int ns, int xcd) {
    hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, ns * 32768);
    for (int i = 0; i < 3; i++) hipLaunchKernelGGL(kern, dim3(tiles * tiles), dim3(512), ns * 32768, 0, A, B, (unsigned)bytes, (unsigned)bytes, tiles, nk, (unsigned)(K * 2), sink, xcd);
    hipDeviceSynchronize();
    const int it = 50;
    hipEventRecord(e0);
    for (int i = 0; i < it; i++) hipLaunchKernelGGL(kern, dim3(tiles * tiles), dim3(512), ns * 32768, 0, A, B, (unsigned)bytes, (unsigned)bytes, tiles, nk, (unsigned)(K * 2), sink, xcd);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    const double us = ms / it * 1e3, by = 256.0 * nk * 32768;
    printf("%-28s xcd=%d  %7.2f us  %6.2f TB/s into LDS  %5.1f B/clk/CU (2.4 GHz)  err=%d\n", name, xcd, us, by / us / 1e6, by / 256 / (us * 2400), (int)hipGetLastError());
    fflush(stdout);
  };
  for (int xcd = 0; xcd < 2; xcd++) {
    run("strided NS=4", stream_k<4, 0>, 4, xcd);
    run("packed  NS=4", stream_k<4, 1>, 4, xcd);
    run("strided NS=3", stream_k<3, 0>, 3, xcd);
    run("packed  NS=3", stream_k<3, 1>, 3, xcd);
    run("strided NS=5", stream_k<5, 0>, 5, xcd);
    run("packed  NS=5", stream_k<5, 1>, 5, xcd);
    run("strided NS=2", stream_k<2, 0>, 2, xcd);
    run("packed  NS=2", stream_k<2, 1>, 2, xcd);
  }
  return 0;
}
