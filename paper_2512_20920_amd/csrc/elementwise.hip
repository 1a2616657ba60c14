// Memory-bound kernels of the RevFFN block: RMSNorm (Norm of Eq. 1-2) forward and
// backward, rotary encoding, SwiGLU, row gathers/copies, deterministic column sums.
#include "kernels.h"
#include <initializer_list>

#define DISPATCH_DT(dt, ...)                                  \
  do {                                                        \
    if ((dt) == 0) { typedef float T; __VA_ARGS__; }          \
    else { typedef bf16 T; __VA_ARGS__; }                     \
  } while (0)

// ---------------------------------------------------------------------------------
// RMSNorm forward: one wave per token row.
// ---------------------------------------------------------------------------------
// (blockIdx.y == 1: the second problem of the launch, same shape: x2, g2, out2)
template <class T, class TX>
__global__ void __launch_bounds__(256) rmsnorm_fwd_k(const TX* __restrict__ x, i64 ldx, const T* __restrict__ g,
                                                     T* __restrict__ out, i64 ldo, int rows, int h, float eps,
                                                     const unsigned char* __restrict__ row_skip,
                                                     const TX* __restrict__ x2, const T* __restrict__ g2, T* __restrict__ out2) {
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= rows || (row_skip && row_skip[row])) return;
  if (blockIdx.y) { x = x2; g = g2; out = out2; }
  const TX* xr = x + (i64)row * ldx;
  float ss = 0.f;
  for (int j = lane; j < h; j += 64) { float v = to_f(xr[j]); ss += v * v; }
  ss = wave_sum(ss);
  float r = 1.0f / sqrtf(ss / (float)h + eps);
  T* orow = out + (i64)row * ldo;
  for (int j = lane; j < h; j += 64) orow[j] = from_f<T>(to_f(xr[j]) * r * to_f(g[j]));
}

// bf16 rows of h % 8 == 0 elements at 16-byte aligned addresses: 16-byte accesses, 8 elements per lane
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_v;
static bool rows_vec8(int dt, int h, std::initializer_list<const void*> ptrs, std::initializer_list<i64> lds) {
  if (dt != 1 || (h & 7)) return false;
  for (const void* q : ptrs) if ((uintptr_t)q & 15) return false;
  for (i64 l : lds) if (l & 7) return false;
  return true;
}
// 8 consecutive elements of a bf16 or float32 row as floats (float32 rows: two 16-byte loads; p 16-byte aligned)
struct f32x8 { float v[8]; };
__device__ __forceinline__ f32x8 load8(const bf16* p) {
  const bf16x8_v t = *(const bf16x8_v*)p;
  f32x8 o;
#pragma unroll
  for (int q = 0; q < 8; q++) o.v[q] = (float)t[q];
  return o;
}
__device__ __forceinline__ f32x8 load8(const float* p) {
  const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
  return f32x8{{a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w}};
}
template <class TX>
__global__ void __launch_bounds__(256) rmsnorm_fwd_v8_k(const TX* __restrict__ x, i64 ldx, const bf16* __restrict__ g,
                                                        bf16* __restrict__ out, i64 ldo, int rows, int h, float eps,
                                                        const unsigned char* __restrict__ row_skip,
                                                        const TX* __restrict__ x2, const bf16* __restrict__ g2,
                                                        bf16* __restrict__ out2) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows || (row_skip && row_skip[row])) return;
  if (blockIdx.y) { x = x2; g = g2; out = out2; }
  const TX* xr = x + (i64)row * ldx;
  float ss = 0.f;
  for (int j = lane * 8; j < h; j += 512) {
    const f32x8 v = load8(xr + j);
#pragma unroll
    for (int q = 0; q < 8; q++) ss += v.v[q] * v.v[q];
  }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)h + eps);
  bf16* orow = out + (i64)row * ldo;
  for (int j = lane * 8; j < h; j += 512) {
    const f32x8 v = load8(xr + j);
    const bf16x8_v gv = *(const bf16x8_v*)(g + j);
    bf16x8_v o;
#pragma unroll
    for (int q = 0; q < 8; q++) o[q] = (__bf16)(v.v[q] * r * (float)gv[q]);
    *(bf16x8_v*)(orow + j) = o;
  }
}

void launch_rmsnorm_fwd(int dt, int tx, const void* x, i64 ldx, const void* g, void* out, i64 ldo, int rows, int h,
                        float eps, hipStream_t s, const unsigned char* row_skip, const void* x2, const void* g2,
                        void* out2) {
  if (rows <= 0) return;
  const dim3 grid(cdiv(rows, 4), x2 ? 2 : 1), block(256);
  if (rows_vec8(dt, h, {x, g, out, x2, g2, out2}, {ldx, ldo})) {
    if (tx == 0)
      hipLaunchKernelGGL(rmsnorm_fwd_v8_k<float>, grid, block, 0, s, (const float*)x, ldx, (const bf16*)g, (bf16*)out,
                         ldo, rows, h, eps, row_skip, (const float*)x2, (const bf16*)g2, (bf16*)out2);
    else
      hipLaunchKernelGGL(rmsnorm_fwd_v8_k<bf16>, grid, block, 0, s, (const bf16*)x, ldx, (const bf16*)g, (bf16*)out,
                         ldo, rows, h, eps, row_skip, (const bf16*)x2, (const bf16*)g2, (bf16*)out2);
    return;
  }
  if (dt == 1 && tx == 0) {
    hipLaunchKernelGGL((rmsnorm_fwd_k<bf16, float>), grid, block, 0, s, (const float*)x, ldx, (const bf16*)g,
                       (bf16*)out, ldo, rows, h, eps, row_skip, (const float*)x2, (const bf16*)g2, (bf16*)out2);
    return;
  }
  DISPATCH_DT(dt, hipLaunchKernelGGL((rmsnorm_fwd_k<T, T>), grid, block, 0, s, (const T*)x, ldx, (const T*)g, (T*)out,
                                     ldo, rows, h, eps, row_skip, (const T*)x2, (const T*)g2, (T*)out2));
}

// RMSNorm backward for the input:  dx = r*(g.dy) - x*r^3*mean_j(x_j g_j dy_j), plus an
// optional base term (the residual path of Eq. 1-2).  1/rms is kept per row.
template <class T, class TX>
__global__ void __launch_bounds__(256) rmsnorm_bwd_k(const T* __restrict__ dy, i64 ldd, const TX* __restrict__ x,
                                                     i64 ldx, const T* __restrict__ g, const T* base, i64 ldb,
                                                     T* dx, i64 ldo, float* __restrict__ rinv, int rows, int h,
                                                     float eps) {
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const TX* xr = x + (i64)row * ldx;
  const T* dr = dy + (i64)row * ldd;
  float ss = 0.f, sd = 0.f;
  for (int j = lane; j < h; j += 64) {
    float v = to_f(xr[j]);
    ss += v * v;
    sd += v * to_f(g[j]) * to_f(dr[j]);
  }
  ss = wave_sum(ss);
  sd = wave_sum(sd);
  float r = 1.0f / sqrtf(ss / (float)h + eps);
  float c = r * r * r * sd / (float)h;
  if (lane == 0) rinv[row] = r;
  for (int j = lane; j < h; j += 64) {
    float v = r * to_f(g[j]) * to_f(dr[j]) - to_f(xr[j]) * c;
    if (base) v += to_f(base[(i64)row * ldb + j]);
    dx[(i64)row * ldo + j] = from_f<T>(v);
  }
}

template <class TX>
__global__ void __launch_bounds__(256) rmsnorm_bwd_v8_k(const bf16* __restrict__ dy, i64 ldd, const TX* __restrict__ x,
                                                        i64 ldx, const bf16* __restrict__ g, const bf16* base, i64 ldb,
                                                        bf16* dx, i64 ldo, float* __restrict__ rinv, int rows, int h,
                                                        float eps) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const TX* xr = x + (i64)row * ldx;
  const bf16* dr = dy + (i64)row * ldd;
  float ss = 0.f, sd = 0.f;
  for (int j = lane * 8; j < h; j += 512) {
    const f32x8 v = load8(xr + j);
    const bf16x8_v gv = *(const bf16x8_v*)(g + j), d = *(const bf16x8_v*)(dr + j);
#pragma unroll
    for (int q = 0; q < 8; q++) { ss += v.v[q] * v.v[q]; sd += v.v[q] * (float)gv[q] * (float)d[q]; }
  }
  ss = wave_sum(ss);
  sd = wave_sum(sd);
  const float r = 1.0f / sqrtf(ss / (float)h + eps);
  const float c = r * r * r * sd / (float)h;
  if (lane == 0) rinv[row] = r;
  for (int j = lane * 8; j < h; j += 512) {
    // (dx may alias base or dy: every lane reads its 8 elements of all inputs before it writes them)
    const f32x8 v = load8(xr + j);
    const bf16x8_v gv = *(const bf16x8_v*)(g + j), d = *(const bf16x8_v*)(dr + j);
    bf16x8_v b;
    if (base) b = *(const bf16x8_v*)(base + (i64)row * ldb + j);
    bf16x8_v o;
#pragma unroll
    for (int q = 0; q < 8; q++) {
      float t = r * (float)gv[q] * (float)d[q] - v.v[q] * c;
      if (base) t += (float)b[q];
      o[q] = (__bf16)t;
    }
    *(bf16x8_v*)(dx + (i64)row * ldo + j) = o;
  }
}

void launch_rmsnorm_bwd(int dt, int tx, const void* dy, i64 ldd, const void* x, i64 ldx, const void* g,
                        const void* base, i64 ldb, void* dx, i64 ldo, float* rinv, int rows, int h, float eps,
                        hipStream_t s) {
  if (rows <= 0) return;
  const dim3 grid(cdiv(rows, 4)), block(256);
  if (rows_vec8(dt, h, {dy, x, g, base, dx}, {ldd, ldx, ldb, ldo})) {
    if (tx == 0)
      hipLaunchKernelGGL(rmsnorm_bwd_v8_k<float>, grid, block, 0, s, (const bf16*)dy, ldd, (const float*)x, ldx,
                         (const bf16*)g, (const bf16*)base, ldb, (bf16*)dx, ldo, rinv, rows, h, eps);
    else
      hipLaunchKernelGGL(rmsnorm_bwd_v8_k<bf16>, grid, block, 0, s, (const bf16*)dy, ldd, (const bf16*)x, ldx,
                         (const bf16*)g, (const bf16*)base, ldb, (bf16*)dx, ldo, rinv, rows, h, eps);
    return;
  }
  if (dt == 1 && tx == 0) {
    hipLaunchKernelGGL((rmsnorm_bwd_k<bf16, float>), grid, block, 0, s, (const bf16*)dy, ldd, (const float*)x, ldx,
                       (const bf16*)g, (const bf16*)base, ldb, (bf16*)dx, ldo, rinv, rows, h, eps);
    return;
  }
  DISPATCH_DT(dt, hipLaunchKernelGGL((rmsnorm_bwd_k<T, T>), grid, block, 0, s, (const T*)dy, ldd, (const T*)x, ldx,
                                     (const T*)g, (const T*)base, ldb, (T*)dx, ldo, rinv, rows, h, eps));
}

// ---------------------------------------------------------------------------------
// Deterministic column sum in two stages (used for gain, bias and router-bias gradients).
// Stage 1: block (column tile of 64, row chunk c) -> partial[c][col]; stage 2 adds the
// chunks in index order.
// ---------------------------------------------------------------------------------
#define COLSUM_CHUNKS 32
static int colsum_chunk_rows(int rows) { int c = cdiv(rows > 0 ? rows : 1, COLSUM_CHUNKS); return c < 32 ? 32 : c; }
size_t colsum_partial_floats(int rows, int cols) { return (size_t)COLSUM_BATCH * (COLSUM_CHUNKS + 1) * cols; }

// Up to COLSUM_BATCH problems of one shape and type go into one launch pair (blockIdx.z = problem).
struct ColsumBatch {
  const void* a[COLSUM_BATCH]; const void* b[COLSUM_BATCH]; const float* sc[COLSUM_BATCH]; void* out[COLSUM_BATCH];
  i64 lda[COLSUM_BATCH], ldb[COLSUM_BATCH];
};
template <class TA, class TB>
__global__ void __launch_bounds__(256) colsum1_k(ColsumBatch q, float* __restrict__ partial_all, int rows, int cols,
                                                 int chunk, int chunks) {
  __shared__ float red[4][64];
  const int z = blockIdx.z;
  const TA* __restrict__ a = (const TA*)q.a[z];
  const TB* __restrict__ b = (const TB*)q.b[z];
  const float* __restrict__ sc = q.sc[z];
  const i64 lda = q.lda[z], ldb = q.ldb[z];
  float* partial = partial_all + (i64)z * chunks * cols;
  int c = blockIdx.x * 64 + (threadIdx.x & 63);
  int qd = threadIdx.x >> 6;
  int r0 = blockIdx.y * chunk;
  int r1 = min(rows, r0 + chunk);
  float acc = 0.f;
  if (c < cols) {
    for (int t = r0 + qd; t < r1; t += 4) {
      float v = to_f(a[(i64)t * lda + c]);
      if (b) v *= to_f(b[(i64)t * ldb + c]);
      if (sc) v *= sc[t];
      acc += v;
    }
  }
  red[qd][threadIdx.x & 63] = acc;
  __syncthreads();
  if (qd == 0 && c < cols) {
    float v = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
    partial[(i64)blockIdx.y * cols + c] = v;
  }
}
// bf16 operands with 8 | cols at 16-byte aligned addresses: a thread owns 8 adjacent columns (16-byte loads) and every
// 8th row of the chunk; the 8 row lanes are added in lane order.  Same two-stage, fixed-order scheme.
__global__ void __launch_bounds__(256) colsum1_v8_k(ColsumBatch q, float* __restrict__ partial_all, int rows, int cols,
                                                    int chunk, int chunks) {
  __shared__ float red[8][256];
  const int z = blockIdx.z;
  const bf16* __restrict__ a = (const bf16*)q.a[z];
  const bf16* __restrict__ b = (const bf16*)q.b[z];
  const float* __restrict__ sc = q.sc[z];
  const i64 lda = q.lda[z], ldb = q.ldb[z];
  float* partial = partial_all + (i64)z * chunks * cols;
  const int cg = threadIdx.x & 31, qd = threadIdx.x >> 5;
  const int c = blockIdx.x * 256 + cg * 8;
  const int r0 = blockIdx.y * chunk, r1 = min(rows, r0 + chunk);
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; i++) acc[i] = 0.f;
  if (c < cols) {
#pragma unroll 4
    for (int t = r0 + qd; t < r1; t += 8) {
      const bf16x8_v av = *(const bf16x8_v*)(a + (i64)t * lda + c);
      const float w = sc ? sc[t] : 1.f;
      if (b) {
        const bf16x8_v bv = *(const bf16x8_v*)(b + (i64)t * ldb + c);
#pragma unroll
        for (int i = 0; i < 8; i++) acc[i] += (float)av[i] * (float)bv[i] * w;
      } else {
#pragma unroll
        for (int i = 0; i < 8; i++) acc[i] += (float)av[i] * w;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; i++) red[qd][cg * 8 + i] = acc[i];
  __syncthreads();
  const int cc = blockIdx.x * 256 + threadIdx.x;
  if (cc < cols) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < 8; j++) v += red[j][threadIdx.x];
    partial[(i64)blockIdx.y * cols + cc] = v;
  }
}
template <class TO>
__global__ void colsum2_k(const float* __restrict__ partial_all, ColsumBatch q, int chunks, int cols) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= cols) return;
  const float* partial = partial_all + (i64)blockIdx.z * chunks * cols;
  float acc = 0.f;
  for (int i = 0; i < chunks; i++) acc += partial[(i64)i * cols + c];
  ((TO*)q.out[blockIdx.z])[c] = from_f<TO>(acc);
}

template <class TA, class TB>
static void colsum_go(const ColsumBatch& q, int n, int tout, float* partial, int rows, int cols, hipStream_t s) {
  int chunk = colsum_chunk_rows(rows);
  int chunks = cdiv(rows > 0 ? rows : 1, chunk);
  constexpr bool both_bf16 = sizeof(TA) == 2 && sizeof(TB) == 2;
  bool v8 = both_bf16 && (cols & 7) == 0;
  for (int z = 0; z < n; z++)
    v8 = v8 && (q.lda[z] & 7) == 0 && (!q.b[z] || (q.ldb[z] & 7) == 0) && ((uintptr_t)q.a[z] & 15) == 0 && ((uintptr_t)q.b[z] & 15) == 0;
  if (v8) {
    hipLaunchKernelGGL(colsum1_v8_k, dim3(cdiv(cols, 256), chunks, n), dim3(256), 0, s, q, partial, rows, cols, chunk, chunks);
  } else {
    hipLaunchKernelGGL((colsum1_k<TA, TB>), dim3(cdiv(cols, 64), chunks, n), dim3(256), 0, s, q, partial, rows, cols, chunk, chunks);
  }
  if (tout == 0)
    hipLaunchKernelGGL(colsum2_k<float>, dim3(cdiv(cols, 256), 1, n), dim3(256), 0, s, partial, q, chunks, cols);
  else
    hipLaunchKernelGGL(colsum2_k<bf16>, dim3(cdiv(cols, 256), 1, n), dim3(256), 0, s, partial, q, chunks, cols);
}

void launch_colsum_batch(int n, int ta, const void* const* a, const i64* lda, int tb, const void* const* b, const i64* ldb,
                         const float* const* sc, int tout, void* const* out, float* partial, int rows, int cols,
                         hipStream_t s) {
  if (cols <= 0 || n <= 0 || n > COLSUM_BATCH) return;
  ColsumBatch q;
  for (int z = 0; z < COLSUM_BATCH; z++) {
    const int y = z < n ? z : 0;
    q.a[z] = a[y]; q.b[z] = b ? b[y] : nullptr; q.sc[z] = sc ? sc[y] : nullptr; q.out[z] = out[y];
    q.lda[z] = lda[y]; q.ldb[z] = ldb ? ldb[y] : 0;
  }
  if (ta == 0 && tb == 0) colsum_go<float, float>(q, n, tout, partial, rows, cols, s);
  else if (ta == 0 && tb == 1) colsum_go<float, bf16>(q, n, tout, partial, rows, cols, s);
  else if (ta == 1 && tb == 0) colsum_go<bf16, float>(q, n, tout, partial, rows, cols, s);
  else colsum_go<bf16, bf16>(q, n, tout, partial, rows, cols, s);
}
void launch_colsum(int ta, const void* a, i64 lda, int tb, const void* b, i64 ldb, const float* sc, int tout,
                   void* out, float* partial, int rows, int cols, hipStream_t s) {
  launch_colsum_batch(1, ta, &a, &lda, tb, &b, &ldb, &sc, tout, &out, partial, rows, cols, s);
}

// ---------------------------------------------------------------------------------
// Rotary encoding in place on buf[T, H*dh]; half-split pairing (i, i+dh/2); the angle of
// pair i at sequence position s comes from a host-built table cs[s][i] = (cos, sin).
// sign = -1 applies the inverse rotation (the backward of the forward rotation).
// ---------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(256) rope_k(T* __restrict__ buf, T* __restrict__ buf2, const float2* __restrict__ cs,
                                              i64 total, int S, int H, int half, float sign,
                                              const unsigned char* __restrict__ row_skip) {
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  if (blockIdx.y) buf = buf2;                // second tensor of the launch
  int i = (int)(e % half);
  i64 th = e / half;          // token*H + head
  i64 t = th / H;
  if (row_skip && row_skip[t]) return;
  int spos = (int)(t % S);
  float2 c = cs[(i64)spos * half + i];
  float sn = sign * c.y;
  T* p = buf + th * (2 * half);
  float a = to_f(p[i]), b = to_f(p[i + half]);
  p[i] = from_f<T>(a * c.x - b * sn);
  p[i + half] = from_f<T>(b * c.x + a * sn);
}

// bf16, half % 8 == 0: one lane rotates 8 consecutive pairs of one (token, head) with 16-byte accesses
__global__ void __launch_bounds__(256) rope_v8_k(bf16* __restrict__ buf, bf16* __restrict__ buf2,
                                                 const float2* __restrict__ cs, int total8, int S, int H, int half8,
                                                 float sign, const unsigned char* __restrict__ row_skip) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= total8) return;
  if (blockIdx.y) buf = buf2;                // second tensor of the launch
  const int i = (e % half8) * 8;
  const int th = e / half8;          // token*H + head
  if (row_skip && row_skip[th / H]) return;
  const int spos = (th / H) % S;
  const int half = half8 * 8;
  bf16* p = buf + (i64)th * (2 * half) + i;
  const bf16x8_v a = *(const bf16x8_v*)p, b = *(const bf16x8_v*)(p + half);
  const float2* c = cs + (i64)spos * half + i;
  bf16x8_v oa, ob;
#pragma unroll
  for (int q = 0; q < 8; q++) {
    const float2 cq = c[q];
    const float sn = sign * cq.y, av = (float)a[q], bv = (float)b[q];
    oa[q] = (__bf16)(av * cq.x - bv * sn);
    ob[q] = (__bf16)(bv * cq.x + av * sn);
  }
  *(bf16x8_v*)p = oa;
  *(bf16x8_v*)(p + half) = ob;
}

void launch_rope(int dt, void* buf, const float* cs_table, int Tn, int S, int H, int dh, float sign,
                 hipStream_t s, void* buf2, const unsigned char* row_skip) {
  i64 total = (i64)Tn * H * (dh / 2);
  if (total <= 0) return;
  const unsigned ny = buf2 ? 2 : 1;
  if (dt == 1 && (dh & 15) == 0 && (((uintptr_t)buf | (uintptr_t)buf2) & 15) == 0 && total / 8 < (i64)1 << 31) {
    hipLaunchKernelGGL(rope_v8_k, dim3(cdiv(total / 8, 256), ny), dim3(256), 0, s, (bf16*)buf, (bf16*)buf2,
                       (const float2*)cs_table, (int)(total / 8), S, H, dh / 16, sign, row_skip);
    return;
  }
  DISPATCH_DT(dt, hipLaunchKernelGGL(rope_k<T>, dim3(cdiv(total, 256), ny), dim3(256), 0, s, (T*)buf, (T*)buf2,
                                     (const float2*)cs_table, total, S, H, dh / 2, sign, row_skip));
}

// ---------------------------------------------------------------------------------
// SwiGLU: hh = silu(G) * U on gu[rows, 2I] = [G | U]; and its backward.
// ---------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(256) swiglu_fwd_k(const T* __restrict__ gu, T* __restrict__ hh, i64 total, int I) {
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  i64 r = e / I;
  int j = (int)(e % I);
  float g = to_f(gu[r * 2 * I + j]), u = to_f(gu[r * 2 * I + I + j]);
  hh[e] = from_f<T>(g * sigmoid_f(g) * u);
}
template <class T>
__global__ void __launch_bounds__(256) swiglu_bwd_k(const T* __restrict__ dhh, const T* __restrict__ gu,
                                                    T* __restrict__ dgu, i64 total, int I) {
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  i64 r = e / I;
  int j = (int)(e % I);
  float g = to_f(gu[r * 2 * I + j]), u = to_f(gu[r * 2 * I + I + j]);
  float dh = to_f(dhh[e]);
  float sg = sigmoid_f(g);
  dgu[r * 2 * I + j] = from_f<T>(dh * u * sg * (1.f + g * (1.f - sg)));
  dgu[r * 2 * I + I + j] = from_f<T>(dh * g * sg);
}
// bf16, I % 8 == 0: one thread handles 8 consecutive columns with 16-byte accesses
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
__global__ void __launch_bounds__(256) swiglu_fwd_v8_k(const bf16* __restrict__ gu, bf16* __restrict__ hh, i64 total8,
                                                       int I8) {
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  if (e >= total8) return;
  i64 r = e / I8;
  int j = (int)(e % I8) * 8;
  const int I = I8 * 8;
  bf16x8_t g = *(const bf16x8_t*)(gu + r * 2 * I + j), u = *(const bf16x8_t*)(gu + r * 2 * I + I + j), o;
#pragma unroll
  for (int q = 0; q < 8; q++) { float gv = (float)g[q]; o[q] = (__bf16)(gv * sigmoid_f(gv) * (float)u[q]); }
  *(bf16x8_t*)(hh + r * I + j) = o;
}
__global__ void __launch_bounds__(256) swiglu_bwd_v8_k(const bf16* __restrict__ dhh, const bf16* __restrict__ gu,
                                                       bf16* __restrict__ dgu, i64 total8, int I8) {
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  if (e >= total8) return;
  i64 r = e / I8;
  int j = (int)(e % I8) * 8;
  const int I = I8 * 8;
  bf16x8_t g = *(const bf16x8_t*)(gu + r * 2 * I + j), u = *(const bf16x8_t*)(gu + r * 2 * I + I + j);
  bf16x8_t dh = *(const bf16x8_t*)(dhh + r * I + j), og, ou;
#pragma unroll
  for (int q = 0; q < 8; q++) {
    float gv = (float)g[q], d = (float)dh[q], sg = sigmoid_f(gv);
    og[q] = (__bf16)(d * (float)u[q] * sg * (1.f + gv * (1.f - sg)));
    ou[q] = (__bf16)(d * gv * sg);
  }
  *(bf16x8_t*)(dgu + r * 2 * I + j) = og;
  *(bf16x8_t*)(dgu + r * 2 * I + I + j) = ou;
}

void launch_swiglu_fwd(int dt, const void* gu, void* hh, i64 rows, int I, hipStream_t s) {
  i64 total = rows * I;
  if (total <= 0) return;
  if (dt == 1 && (I & 7) == 0 && (((uintptr_t)gu | (uintptr_t)hh) & 15) == 0) {
    hipLaunchKernelGGL(swiglu_fwd_v8_k, dim3(cdiv(total / 8, 256)), dim3(256), 0, s, (const bf16*)gu, (bf16*)hh,
                       total / 8, I / 8);
    return;
  }
  DISPATCH_DT(dt, hipLaunchKernelGGL(swiglu_fwd_k<T>, dim3(cdiv(total, 256)), dim3(256), 0, s, (const T*)gu,
                                     (T*)hh, total, I));
}
void launch_swiglu_bwd(int dt, const void* dhh, const void* gu, void* dgu, i64 rows, int I, hipStream_t s) {
  i64 total = rows * I;
  if (total <= 0) return;
  if (dt == 1 && (I & 7) == 0 && (((uintptr_t)gu | (uintptr_t)dhh | (uintptr_t)dgu) & 15) == 0) {
    hipLaunchKernelGGL(swiglu_bwd_v8_k, dim3(cdiv(total / 8, 256)), dim3(256), 0, s, (const bf16*)dhh,
                       (const bf16*)gu, (bf16*)dgu, total / 8, I / 8);
    return;
  }
  DISPATCH_DT(dt, hipLaunchKernelGGL(swiglu_bwd_k<T>, dim3(cdiv(total, 256)), dim3(256), 0, s, (const T*)dhh,
                                     (const T*)gu, (T*)dgu, total, I));
}

// ---------------------------------------------------------------------------------
// Row gather (dst[r] = src[row_map[r] / div]) and strided row copy.
// ---------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(256) gather_rows_k(const T* __restrict__ src, const int* __restrict__ row_map,
                                                     int div, T* __restrict__ dst, int rows, int cols) {
  int r = blockIdx.x;
  if (r >= rows) return;
  const T* sp = src + (i64)(row_map[r] / div) * cols;
  T* dp = dst + (i64)r * cols;
  for (int c = threadIdx.x; c < cols; c += 256) dp[c] = sp[c];
}
void launch_gather_rows(int dt, const void* src, const int* row_map, int div, void* dst, int rows, int cols,
                        hipStream_t s) {
  if (rows <= 0) return;
  DISPATCH_DT(dt, hipLaunchKernelGGL(gather_rows_k<T>, dim3(rows), dim3(256), 0, s, (const T*)src, row_map, div,
                                     (T*)dst, rows, cols));
}
template <class T>
__global__ void __launch_bounds__(256) copy_rows_k(const T* __restrict__ src, i64 lds_, T* __restrict__ dst, i64 ldd,
                                                   int rows, int cols) {
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  if (e >= (i64)rows * cols) return;
  i64 r = e / cols;
  int c = (int)(e % cols);
  dst[r * ldd + c] = src[r * lds_ + c];
}
void launch_copy_rows(int dt, const void* src, i64 lds_, void* dst, i64 ldd, int rows, int cols, hipStream_t s) {
  i64 total = (i64)rows * cols;
  if (total <= 0) return;
  DISPATCH_DT(dt, hipLaunchKernelGGL(copy_rows_k<T>, dim3(cdiv(total, 256)), dim3(256), 0, s, (const T*)src, lds_,
                                     (T*)dst, ldd, rows, cols));
}

// dst rows [0, rows_a) = src_a rows, dst rows [rows_a, rows_a + rows_b) = src_b rows (the stacked router matrix)
template <class T>
__global__ void __launch_bounds__(256) copy_rows2_k(const T* __restrict__ src_a, i64 lds_a, int rows_a,
                                                    const T* __restrict__ src_b, i64 lds_b, int rows_b,
                                                    T* __restrict__ dst, i64 ldd, int cols) {
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  if (e >= (i64)(rows_a + rows_b) * cols) return;
  i64 r = e / cols;
  int c = (int)(e % cols);
  dst[r * ldd + c] = r < rows_a ? src_a[r * lds_a + c] : src_b[(r - rows_a) * lds_b + c];
}
void launch_copy_rows2(int dt, const void* src_a, i64 lds_a, int rows_a, const void* src_b, i64 lds_b, int rows_b,
                       void* dst, i64 ldd, int cols, hipStream_t s) {
  i64 total = (i64)(rows_a + rows_b) * cols;
  if (total <= 0) return;
  DISPATCH_DT(dt, hipLaunchKernelGGL(copy_rows2_k<T>, dim3(cdiv(total, 256)), dim3(256), 0, s, (const T*)src_a, lds_a,
                                     rows_a, (const T*)src_b, lds_b, rows_b, (T*)dst, ldd, cols));
}

template <class T>
__global__ void zero_k(T* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = from_f<T>(0.f);
}
void launch_zero(int dt, void* p, int n, hipStream_t s) {
  if (n <= 0) return;
  DISPATCH_DT(dt, hipLaunchKernelGGL(zero_k<T>, dim3(cdiv(n, 256)), dim3(256), 0, s, (T*)p, n));
}

__global__ void fill_u32_k(uint32_t* p, uint32_t v, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
void launch_fill_u32(uint32_t* p, uint32_t v, int n, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(fill_u32_k, dim3(cdiv(n, 256)), dim3(256), 0, s, p, v, n);
}

// res = max |a - b| over all elements (non-negative floats compare like their bit patterns, so
// an integer atomic max is exact and order-independent); then dst = a.
template <class T>
__global__ void __launch_bounds__(256) absdiff_max_copy_k(const T* __restrict__ a, i64 lda, const T* b, i64 ldb,
                                                          T* dst, i64 ldd, float* res, int rows, int cols) {
  __shared__ float red[4];
  i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
  float m = 0.f;
  if (e < (i64)rows * cols) {
    i64 r = e / cols;
    int c = (int)(e % cols);
    T av = a[r * lda + c];
    m = fabsf(to_f(av) - to_f(b[r * ldb + c]));
    dst[r * ldd + c] = av;
  }
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    atomicMax((unsigned int*)res, __float_as_uint(m));
  }
}
void launch_absdiff_max_copy(int dt, const void* a, i64 lda, const void* b, i64 ldb, void* dst, i64 ldd,
                             float* res, int rows, int cols, hipStream_t s) {
  i64 total = (i64)rows * cols;
  if (total <= 0) return;
  DISPATCH_DT(dt, hipLaunchKernelGGL(absdiff_max_copy_k<T>, dim3(cdiv(total, 256)), dim3(256), 0, s, (const T*)a,
                                     lda, (const T*)b, ldb, (T*)dst, ldd, res, rows, cols));
}

// ---------------------------------------------------------------------------------
// Stopping rule of the inverse's fixed-point iteration (x <- Y1 - attention branch(x, X2^)), decided on the device.
// Each query row's iterate depends on that row alone (keys and values come from X2^, which is fixed), so a block of
// rows can stop on its own: once max |x_n - x_(n-1)| over the block is <= tol its rows are marked, and the kernels of
// later iterations leave marked rows alone.  The host enqueues max_iters iterations and never waits.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ int conv_block_of(int row, int S, int bp, int nj) {
  if (bp <= 0) return 0;
  const int b = row / S;
  return b * nj + (row - b * S) / bp;
}
template <class T>
__global__ void __launch_bounds__(256) conv_update_k(const T* __restrict__ xn, i64 ldn, const T* xin, i64 ldi, T* dst,
                                                     i64 ldd, ConvState cs, int rows, int cols) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows || cs.row_done[row]) return;            // whole wave
  float m = 0.f;
  for (int c = lane; c < cols; c += 64) {
    const T a = xn[(i64)row * ldn + c];
    m = fmaxf(m, fabsf(to_f(a) - to_f(xin[(i64)row * ldi + c])));   // (dst may be xin: read before the write)
    dst[(i64)row * ldd + c] = a;
  }
  // fmaxf drops a NaN operand; a row with a non-finite difference must not look converged
  for (int c = lane; c < cols; c += 64) { const float a = to_f(xn[(i64)row * ldn + c]); if (!(a == a)) m = INFINITY; }
  m = wave_max(m);
  if (lane == 0) atomicMax(cs.blk_bits + conv_block_of(row, cs.S, cs.bp, cs.nj), __float_as_uint(m));
}
__global__ void __launch_bounds__(64) conv_decide_k(ConvState cs, int rows, float tol, int it) {
  const int blk = blockIdx.x;
  if (cs.blk_done[blk]) return;
  const float res = __uint_as_float(cs.blk_bits[blk]);
  const bool done = res <= tol;
  __syncthreads();                                        // every lane has read the running maximum
  if (threadIdx.x == 0) {
    cs.blk_iters[blk] = it;
    cs.blk_res[blk] = res;
    cs.blk_bits[blk] = 0u;
    if (done) cs.blk_done[blk] = 1;
  }
  if (!done) return;
  int r0, r1;
  if (cs.bp <= 0) { r0 = 0; r1 = rows; }
  else {
    const int b = blk / cs.nj, j = blk - b * cs.nj;
    r0 = b * cs.S + j * cs.bp;
    r1 = min(b * cs.S + min(cs.S, (j + 1) * cs.bp), rows);
  }
  for (int r = r0 + (int)threadIdx.x; r < r1; r += 64) cs.row_done[r] = 1;
}
__global__ void __launch_bounds__(256) conv_finalize_k(ConvState cs, float* residual_out) {
  __shared__ unsigned rb[4];
  __shared__ int ri[4];
  unsigned bits = 0;
  int iters = 0;
  for (int b = threadIdx.x; b < cs.nblk; b += 256) {
    bits = max(bits, __float_as_uint(cs.blk_res[b]));     // residuals are non-negative (or +inf / NaN, which rank above)
    iters = max(iters, cs.blk_iters[b]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { bits = max(bits, (unsigned)__shfl_xor((int)bits, o, WAVE)); iters = max(iters, __shfl_xor(iters, o, WAVE)); }
  if ((threadIdx.x & 63) == 0) { rb[threadIdx.x >> 6] = bits; ri[threadIdx.x >> 6] = iters; }
  __syncthreads();
  if (threadIdx.x == 0) {
    bits = max(max(rb[0], rb[1]), max(rb[2], rb[3]));
    iters = max(max(ri[0], ri[1]), max(ri[2], ri[3]));
    if (residual_out) *residual_out = __uint_as_float(bits);
    cs.stats[0] += 1;
    cs.stats[1] += iters;
    cs.stats[2] = iters;
    cs.stats[3] = (int)bits;
  }
}
void launch_conv_update(int dt, const void* xn, i64 ldn, const void* xin, i64 ldi, void* dst, i64 ldd,
                        const ConvState& cs, int rows, int cols, hipStream_t s) {
  if (rows <= 0) return;
  DISPATCH_DT(dt, hipLaunchKernelGGL(conv_update_k<T>, dim3(cdiv(rows, 4)), dim3(256), 0, s, (const T*)xn, ldn,
                                     (const T*)xin, ldi, (T*)dst, ldd, cs, rows, cols));
}
void launch_conv_decide(const ConvState& cs, int rows, float tol, int it, hipStream_t s) {
  hipLaunchKernelGGL(conv_decide_k, dim3(cs.nblk), dim3(64), 0, s, cs, rows, tol, it);
}
void launch_conv_finalize(const ConvState& cs, float* residual_out, hipStream_t s) {
  hipLaunchKernelGGL(conv_finalize_k, dim3(1), dim3(256), 0, s, cs, residual_out);
}
