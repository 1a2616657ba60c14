// Generic LDS-tiled GEMM on the vector ALUs (fp32 multiply-add, any shape, any of the
// operand layouts of GemmArgs).  It serves the float32 configuration, whose tolerance
// needs true fp32 products, and every bf16 problem whose shape the MFMA kernels do not
// take.  64x64 output tile per workgroup, 16x16 threads, 4x4 outputs per thread, BK = 16.
#include "kernels.h"

#define GT 64
#define GK 16

template <class TA, class TB, class TC, class TS>
__global__ void __launch_bounds__(256) gemm_generic_k(GemmArgs g) {
  __shared__ float As[GK][GT + 4];
  __shared__ float Bs[GK][GT + 4];
  const TA* A = (const TA*)g.A;
  const TB* Bm = (const TB*)g.B;
  TC* C = (TC*)g.C;
  int m0, m_end, k0 = 0, k_end = g.K;
  if (g.group_mode == 1) {
    int ti = blockIdx.y;
    int grp = g.tile_group[ti];
    if (grp < 0) return;
    m0 = g.tile_m0[ti];
    m_end = min(g.offsets[grp + 1], m0 + g.tile_bm);
    Bm += (i64)grp * g.b_group_stride;
  } else {
    m0 = blockIdx.y * GT;
    m_end = g.M;
    if (g.group_mode == 2) {
      int grp = blockIdx.z;
      k0 = g.offsets[grp];
      k_end = g.offsets[grp + 1];
      C += (i64)grp * g.c_group_stride;
    } else if (g.split_k > 1) {
      int per = ((g.K + g.split_k - 1) / g.split_k + GK - 1) / GK * GK;
      k0 = blockIdx.z * per;
      k_end = min(g.K, k0 + per);
    }
  }
  if (g.row_skip && g.group_mode == 0) {             // nothing to do if every row of the tile is marked as finished
    int live = 0;                                    // every wave checks all rows of the tile: same answer, no LDS
    for (int r = m0 + (int)(threadIdx.x & 63); r < min(m_end, m0 + GT); r += 64) live |= g.row_skip[r] == 0;
    if (!__any(live)) return;
  }
  const int n0 = blockIdx.x * GT;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = 0.f;

  // a 64x64 tile may be taller than a grouped m-tile of height tile_bm < 64 only if tile_bm == 64;
  // the host guarantees tile_bm == GT for this kernel.
  for (int kb = k0; kb < k_end; kb += GK) {
    // ---- A tile: As[kk][mm] = A(m0+mm, kb+kk)
    for (int e = threadIdx.x; e < GT * GK; e += 256) {
      int mm, kk;
      if (g.a_trans) { mm = e % GT; kk = e / GT; } else { kk = e % GK; mm = e / GK; }
      int m = m0 + mm, k = kb + kk;
      float v = 0.f;
      if (m < m_end && k < k_end) {
        if (!g.a_trans) {
          i64 r = g.a_gather ? (i64)(g.a_gather[m] / g.gather_div) : (i64)m;
          v = to_f(A[r * g.lda + k]);
        } else {
          i64 r = g.a_gather ? (i64)(g.a_gather[k] / g.gather_div) : (i64)k;
          v = to_f(A[r * g.lda + m]);
        }
      }
      As[kk][mm] = v;
    }
    // ---- B tile: Bs[kk][nn] = B(kb+kk, n0+nn)
    for (int e = threadIdx.x; e < GT * GK; e += 256) {
      int nn, kk;
      if (g.b_trans) { nn = e % GT; kk = e / GT; } else { kk = e % GK; nn = e / GK; }
      int n = n0 + nn, k = kb + kk;
      float v = 0.f;
      if (n < g.N && k < k_end) {
        if (!g.b_trans) {
          v = to_f(Bm[(i64)n * g.ldb + k]);
        } else {
          v = to_f(Bm[(i64)k * g.ldb + n]);
        }
      }
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; kk++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; j++) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  if (g.split_k > 1) {                       // raw partial sums; the epilogue runs in splitk_reduce_k
    float* ws = g.splitk_ws + (i64)blockIdx.z * g.M * g.N;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      int m = m0 + ty * 4 + i;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < 4; j++) {
        int n = n0 + tx * 4 + j;
        if (n < g.N) ws[(i64)m * g.N + n] = acc[i][j];
      }
    }
    return;
  }
  const TS* bias = (const TS*)g.bias;
  const TS* resid = (const TS*)g.resid;
  const TS* cscale = (const TS*)g.col_scale;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int m = m0 + ty * 4 + i;
    if (m >= m_end) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int n = n0 + tx * 4 + j;
      if (n >= g.N) continue;
      float v = acc[i][j];
      if (cscale) v *= to_f(cscale[n]);
      if (bias) v += to_f(bias[n]);
      if (g.tap) g.tap[(i64)m * g.ldtap + n] = v;
      if (resid) v = (g.resid_f32 ? ((const float*)g.resid)[(i64)m * g.ldr + n] : to_f(resid[(i64)m * g.ldr + n])) + g.resid_sign * v;
      C[(i64)m * g.ldc + n] = from_f<TC>(v);
    }
  }
}

// adds the split-k slices in index order, then the usual epilogue
template <class TC, class TS>
__global__ void __launch_bounds__(256) splitk_reduce_k(GemmArgs g) {
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  if (e >= (i64)g.M * g.N) return;
  int m = (int)(e / g.N), n = (int)(e % g.N);
  float v = 0.f;
  for (int z = 0; z < g.split_k; z++) v += g.splitk_ws[(i64)z * g.M * g.N + e];
  if (g.col_scale) v *= to_f(((const TS*)g.col_scale)[n]);
  if (g.bias) v += to_f(((const TS*)g.bias)[n]);
  if (g.tap) g.tap[(i64)m * g.ldtap + n] = v;
  if (g.resid) v = (g.resid_f32 ? ((const float*)g.resid)[(i64)m * g.ldr + n] : to_f(((const TS*)g.resid)[(i64)m * g.ldr + n])) + g.resid_sign * v;
  ((TC*)g.C)[(i64)m * g.ldc + n] = from_f<TC>(v);
}

template <class TA, class TB, class TC, class TS>
static void go(const GemmArgs& g, hipStream_t s) {
  dim3 grid;
  if (g.group_mode == 1) grid = dim3(cdiv(g.N, GT), g.max_tiles, 1);
  else grid = dim3(cdiv(g.N, GT), cdiv(g.M, GT), g.group_mode == 2 ? g.n_groups : (g.split_k > 1 ? g.split_k : 1));
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return;
  hipLaunchKernelGGL((gemm_generic_k<TA, TB, TC, TS>), grid, dim3(256), 0, s, g);
  if (g.group_mode == 0 && g.split_k > 1 && !g.splitk_raw)
    hipLaunchKernelGGL((splitk_reduce_k<TC, TS>), dim3(cdiv((i64)g.M * g.N, 256)), dim3(256), 0, s, g);
}

void launch_splitk_reduce(const GemmArgs& g, GemmTypes t, hipStream_t s) {
  dim3 grid(cdiv((i64)g.M * g.N, 256));
  if (t.tc == 0 && t.tside == 0) hipLaunchKernelGGL((splitk_reduce_k<float, float>), grid, dim3(256), 0, s, g);
  else if (t.tc == 0) hipLaunchKernelGGL((splitk_reduce_k<float, bf16>), grid, dim3(256), 0, s, g);
  else if (t.tside == 0) hipLaunchKernelGGL((splitk_reduce_k<bf16, float>), grid, dim3(256), 0, s, g);
  else hipLaunchKernelGGL((splitk_reduce_k<bf16, bf16>), grid, dim3(256), 0, s, g);
}

int launch_gemm_generic(const GemmArgs& g, GemmTypes t, hipStream_t s) {
  if (g.group_mode == 1 && g.tile_bm != GT) return -1;
  if (g.split_k > 1 && (g.group_mode != 0 || !g.splitk_ws)) return -1;
  int key = t.ta * 8 + t.tb * 4 + t.tc * 2 + t.tside;
  switch (key) {
    case 0: go<float, float, float, float>(g, s); break;            // fp32 everything
    case 15: go<bf16, bf16, bf16, bf16>(g, s); break;               // bf16 everything
    case 13: go<bf16, bf16, float, bf16>(g, s); break;              // bf16 in, fp32 out (router fold)
    case 7: go<float, bf16, bf16, bf16>(g, s); break;               // fp32 A (router logit gradients), bf16 B/C
    case 9: go<bf16, float, float, bf16>(g, s); break;              // bf16 A, fp32 B/C (router logits)
    case 1: go<float, float, float, bf16>(g, s); break;             // router logits from float32 residual streams
    case 5: go<float, bf16, float, bf16>(g, s); break;              // router weight gradient in float32
    default: return -1;
  }
  return 0;
}
