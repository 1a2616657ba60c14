// HBM-side streaming rate of expert weight tiles through LDS (buffer_load_dwordx4 ... lds): 660 workgroups, each reads
// its own tile of 256 rows x 2048 bf16 columns (1 MiB; rows STRIDE bytes apart) once, 128 bytes of every row per k-step,
// 4 LDS stages, no arithmetic, nothing shared.  Variants: every workgroup starts at k-step 0; workgroup i starts at
// k-step (i * ROT) mod 32 and wraps around; rows padded by 128 or 256 bytes; the tile packed so that a k-step is
// contiguous.  With all workgroups in step at k = 0 their requests agree in the address bits above the cache-line
// offset (every row starts a multiple of 4 KiB from the tile), and those bits choose the memory channel.
// Build: make -C paper_2512_20920_amd/csrc microbench; run: paper_2512_20920_amd/csrc/_build/hbm_stream
#include <hip/hip_runtime.h>
#include <stdio.h>
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
// ROWB = bytes taken from one row per k-step; 0 = packed (a k-step's 32 KiB contiguous).  A k-step covers all 256
// rows x ROWB bytes, and there are 4096 / ROWB k-steps.
template <int NS, int ROWB, int ROT, int STRIDE>
__global__ void __launch_bounds__(512) stream_k(const unsigned char* W, unsigned* sink) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int RB = ROWB ? ROWB : 128;
  constexpr int STEP = 256 * RB;                 // bytes per k-step
  constexpr int LPW = STEP / 1024 / 8;           // wave-loads per wave per k-step
  constexpr int nk = 4096 / RB;
  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const u32x4 d = make_desc(W + (size_t)blockIdx.x * (256u * STRIDE), 256u * STRIDE);
  const int rot = ROT ? (int)((blockIdx.x * ROT) % nk) : 0;
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  unsigned base[LPW];
#pragma unroll
  for (int i = 0; i < LPW; i++) {
    const int pos = (wv * LPW + i) * 64 + lane;            // 16-byte chunk of the k-step
    if (ROWB == 0) base[i] = pos * 16;
    else { constexpr int CPR = RB / 16; base[i] = (pos / CPR) * STRIDE + (pos % CPR) * 16; }
  }
  const unsigned kstep = ROWB == 0 ? STEP : RB;
  const unsigned lw = __builtin_amdgcn_readfirstlane(lds0 + (unsigned)wv * LPW * 1024u);
  auto issue = [&](int kt, int i) {
    const int kr = kt + rot >= nk ? kt + rot - nk : kt + rot;
    const unsigned off = kt < nk ? base[i] + (unsigned)kr * kstep : 0x80000000u;
    load_lds_b128(d, lw + (unsigned)(kt % NS) * STEP + i * 1024, off);
  };
#pragma unroll
  for (int p = 0; p < NS - 1; p++)
#pragma unroll
    for (int i = 0; i < LPW; i++) issue(p, i);
  unsigned acc = 0;
  for (int kt = 0; kt < nk; kt++) {
    wait_vmcnt<LPW * (NS - 2)>();
    __builtin_amdgcn_s_barrier();
    acc += *(const unsigned*)(smem + (kt % NS) * STEP + threadIdx.x * 16);
#pragma unroll
    for (int i = 0; i < LPW; i++) issue(kt + NS - 1, i);
  }
  wait_vmcnt<0>();
  if (acc == 0x12345678u) sink[0] = acc;
}
int main() {
  const int WGS = 660; const size_t bytes = (size_t)WGS * 256 * 4352;
  unsigned char* W; unsigned* sink;
  if (hipMalloc(&W, bytes) || hipMalloc(&sink, 4)) return 1;
  (void)hipMemset(W, 1, bytes);
  hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  auto run = [&](const char* name, auto kern, int lds) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    for (int i = 0; i < 2; i++) hipLaunchKernelGGL(kern, dim3(WGS), dim3(512), lds, 0, W, sink);
    (void)hipDeviceSynchronize();
    const int it = 10;
    (void)hipEventRecord(e0);
    for (int i = 0; i < it; i++) hipLaunchKernelGGL(kern, dim3(WGS), dim3(512), lds, 0, W, sink);
    (void)hipEventRecord(e1); (void)hipEventSynchronize(e1);
    float ms; (void)hipEventElapsedTime(&ms, e0, e1);
    printf("%-34s %7.1f us  %5.2f TB/s  err=%d\n", name, ms / it * 1e3, (double)WGS * (1 << 20) / (ms / it * 1e-3) / 1e12, (int)hipGetLastError());
    fflush(stdout);
  };
  run("128 B/row stride 4096          ", stream_k<4, 128, 0, 4096>, 4 * 32768);
  run("128 B/row stride 4096 rot 1    ", stream_k<4, 128, 1, 4096>, 4 * 32768);
  run("128 B/row stride 4096 rot 5    ", stream_k<4, 128, 5, 4096>, 4 * 32768);
  run("128 B/row stride 4096 rot 13   ", stream_k<4, 128, 13, 4096>, 4 * 32768);
  run("128 B/row stride 4224 (pad 128)", stream_k<4, 128, 0, 4224>, 4 * 32768);
  run("128 B/row stride 4352 (pad 256)", stream_k<4, 128, 0, 4352>, 4 * 32768);
  run("packed                         ", stream_k<4, 0, 0, 4096>, 4 * 32768);
  return 0;
}
