// Generic softmax attention (Attn_pt of section 3.2) on the vector ALUs: any head_dim,
// any sequence length, float32 or bfloat16 storage with fp32 arithmetic.  It serves the
// float32 configuration and head dims the MFMA flash kernels do not take.
// Layout: q,k,v,o,do,dq,dk,dv are [T, H*dh] token-major (token t = b*S+s), head hh in
// columns hh*dh..hh*dh+dh-1.  lse and dvec are [B,H,S] float.
#include "kernels.h"

#define DISPATCH_DT(dt, ...)                                  \
  do {                                                        \
    if ((dt) == 0) { typedef float T; __VA_ARGS__; }          \
    else { typedef bf16 T; __VA_ARGS__; }                     \
  } while (0)

// One workgroup (256 threads) per (batch, head, query row).  Pass 1: row max of the scores.
// Pass 2: per chunk of 256 keys, p_j = exp(s_j - max) into LDS, then every thread adds its
// output columns.  lse = max + log(sum).
template <class T>
__global__ void __launch_bounds__(256) attn_fwd_generic_k(const T* __restrict__ q, const T* __restrict__ k,
                                                          const T* __restrict__ v, T* __restrict__ o,
                                                          float* __restrict__ lse, int S, int H, int dh,
                                                          int causal, float scale,
                                                          const unsigned char* __restrict__ row_skip) {
  extern __shared__ float sm[];            // qs[dh], ps[256], red[4]
  float* qs = sm;
  float* ps = sm + dh;
  float* red = ps + 256;
  const int i = blockIdx.x, hh = blockIdx.y, b = blockIdx.z;
  if (row_skip && row_skip[(i64)b * S + i]) return;       // a finished row of the inverse's iteration
  const i64 d = (i64)H * dh;
  const i64 base = (i64)b * S * d + (i64)hh * dh;
  const int nk = causal ? i + 1 : S;
  for (int c = threadIdx.x; c < dh; c += 256) qs[c] = to_f(q[base + (i64)i * d + c]) * scale;
  __syncthreads();
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < nk; j += 256) {
    const T* kr = k + base + (i64)j * d;
    float sc = 0.f;
    for (int c = 0; c < dh; c++) sc += qs[c] * to_f(kr[c]);
    mx = fmaxf(mx, sc);
  }
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float lsum = 0.f;
  const int ncol = (dh + 255) / 256;       // output columns per thread (1 for dh <= 256)
  float acc[4] = {0.f, 0.f, 0.f, 0.f};     // dh <= 1024
  for (int j0 = 0; j0 < nk; j0 += 256) {
    int j = j0 + threadIdx.x;
    float p = 0.f;
    if (j < nk) {
      const T* kr = k + base + (i64)j * d;
      float sc = 0.f;
      for (int c = 0; c < dh; c++) sc += qs[c] * to_f(kr[c]);
      p = __expf(sc - mx);
    }
    lsum += p;
    __syncthreads();                        // previous chunk's readers are done
    ps[threadIdx.x] = p;
    __syncthreads();
    int cnt = min(256, nk - j0);
    for (int cc = 0; cc < ncol; cc++) {
      int c = threadIdx.x + cc * 256;
      if (c < dh) {
        float a = acc[cc];
        for (int jj = 0; jj < cnt; jj++) a += ps[jj] * to_f(v[base + (i64)(j0 + jj) * d + c]);
        acc[cc] = a;
      }
    }
  }
  float tot = block_sum_256(lsum, red);
  float inv = 1.0f / tot;
  for (int cc = 0; cc < ncol; cc++) {
    int c = threadIdx.x + cc * 256;
    if (c < dh) o[base + (i64)i * d + c] = from_f<T>(acc[cc] * inv);
  }
  if (threadIdx.x == 0) lse[((i64)b * H + hh) * S + i] = mx + __logf(tot);
}

void launch_attn_fwd_generic(int dt, const void* q, const void* k, const void* v, void* o, float* lse, int B,
                             int S, int H, int dh, int causal, hipStream_t s, const unsigned char* row_skip) {
  if (B <= 0 || S <= 0) return;
  size_t smem = (size_t)(dh + 256 + 4) * sizeof(float);
  float scale = 1.0f / sqrtf((float)dh);
  DISPATCH_DT(dt, hipLaunchKernelGGL(attn_fwd_generic_k<T>, dim3(S, H, B), dim3(256), smem, s, (const T*)q,
                                     (const T*)k, (const T*)v, (T*)o, lse, S, H, dh, causal, scale, row_skip));
}

// dvec[b,h,i] = sum_c dO[i,c] * O[i,c]   (the row sum of dP.P in the softmax backward)
template <class T>
__global__ void __launch_bounds__(256) attn_dvec_k(const T* __restrict__ o, const T* __restrict__ d_o,
                                                   float* __restrict__ dvec, int S, int H, int dh, i64 rows) {
  i64 r = (i64)blockIdx.x * 4 + (threadIdx.x >> 6);   // r = (b*S + i)*H + hh
  int lane = threadIdx.x & 63;
  if (r >= rows) return;
  const T* op = o + r * dh;
  const T* dp = d_o + r * dh;
  float acc = 0.f;
  for (int c = lane; c < dh; c += 64) acc += to_f(op[c]) * to_f(dp[c]);
  acc = wave_sum(acc);
  if (lane == 0) {
    i64 t = r / H;
    int hh = (int)(r % H);
    i64 b = t / S;
    int i = (int)(t % S);
    dvec[(b * H + hh) * S + i] = acc;
  }
}

// dQ: one workgroup per (b, h, query i): dq_i = scale * sum_j ds_ij k_j,
//     ds_ij = p_ij (dp_ij - D_i), p_ij = exp(s_ij - lse_i), dp_ij = <dO_i, v_j>.
template <class T>
__global__ void __launch_bounds__(256) attn_bwd_dq_generic_k(const T* __restrict__ q, const T* __restrict__ k,
                                                             const T* __restrict__ v, const T* __restrict__ d_o,
                                                             const float* __restrict__ lse,
                                                             const float* __restrict__ dvec, T* __restrict__ dq,
                                                             int S, int H, int dh, int causal, float scale) {
  extern __shared__ float sm[];            // qs[dh], dos[dh], ds[256]
  float* qs = sm;
  float* dos = sm + dh;
  float* dss = dos + dh;
  const int i = blockIdx.x, hh = blockIdx.y, b = blockIdx.z;
  const i64 d = (i64)H * dh;
  const i64 base = (i64)b * S * d + (i64)hh * dh;
  const int nk = causal ? i + 1 : S;
  for (int c = threadIdx.x; c < dh; c += 256) {
    qs[c] = to_f(q[base + (i64)i * d + c]) * scale;
    dos[c] = to_f(d_o[base + (i64)i * d + c]);
  }
  const float L = lse[((i64)b * H + hh) * S + i];
  const float D = dvec[((i64)b * H + hh) * S + i];
  __syncthreads();
  const int ncol = (dh + 255) / 256;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 < nk; j0 += 256) {
    int j = j0 + threadIdx.x;
    float ds = 0.f;
    if (j < nk) {
      const T* kr = k + base + (i64)j * d;
      const T* vr = v + base + (i64)j * d;
      float sc = 0.f, dp = 0.f;
      for (int c = 0; c < dh; c++) { sc += qs[c] * to_f(kr[c]); dp += dos[c] * to_f(vr[c]); }
      ds = __expf(sc - L) * (dp - D);
    }
    __syncthreads();
    dss[threadIdx.x] = ds;
    __syncthreads();
    int cnt = min(256, nk - j0);
    for (int cc = 0; cc < ncol; cc++) {
      int c = threadIdx.x + cc * 256;
      if (c < dh) {
        float a = acc[cc];
        for (int jj = 0; jj < cnt; jj++) a += dss[jj] * to_f(k[base + (i64)(j0 + jj) * d + c]);
        acc[cc] = a;
      }
    }
  }
  for (int cc = 0; cc < ncol; cc++) {
    int c = threadIdx.x + cc * 256;
    if (c < dh) dq[base + (i64)i * d + c] = from_f<T>(acc[cc] * scale);
  }
}

// dK, dV: one workgroup per (b, h, key j): dv_j = sum_i p_ij dO_i ; dk_j = scale * sum_i ds_ij q_i
template <class T>
__global__ void __launch_bounds__(256) attn_bwd_dkv_generic_k(const T* __restrict__ q, const T* __restrict__ k,
                                                              const T* __restrict__ v, const T* __restrict__ d_o,
                                                              const float* __restrict__ lse,
                                                              const float* __restrict__ dvec, T* __restrict__ dk,
                                                              T* __restrict__ dv, int S, int H, int dh, int causal,
                                                              float scale) {
  extern __shared__ float sm[];            // ks[dh], vs[dh], ps[256], dss[256]
  float* ks = sm;
  float* vs = sm + dh;
  float* ps = vs + dh;
  float* dss = ps + 256;
  const int j = blockIdx.x, hh = blockIdx.y, b = blockIdx.z;
  const i64 d = (i64)H * dh;
  const i64 base = (i64)b * S * d + (i64)hh * dh;
  const int i_lo = causal ? j : 0;
  for (int c = threadIdx.x; c < dh; c += 256) {
    ks[c] = to_f(k[base + (i64)j * d + c]) * scale;
    vs[c] = to_f(v[base + (i64)j * d + c]);
  }
  __syncthreads();
  const int ncol = (dh + 255) / 256;
  float acck[4] = {0.f, 0.f, 0.f, 0.f}, accv[4] = {0.f, 0.f, 0.f, 0.f};
  for (int i0 = i_lo; i0 < S; i0 += 256) {
    int i = i0 + threadIdx.x;
    float p = 0.f, ds = 0.f;
    if (i < S) {
      const T* qr = q + base + (i64)i * d;
      const T* dr = d_o + base + (i64)i * d;
      float sc = 0.f, dp = 0.f;
      for (int c = 0; c < dh; c++) { sc += ks[c] * to_f(qr[c]); dp += vs[c] * to_f(dr[c]); }
      p = __expf(sc - lse[((i64)b * H + hh) * S + i]);
      ds = p * (dp - dvec[((i64)b * H + hh) * S + i]);
    }
    __syncthreads();
    ps[threadIdx.x] = p;
    dss[threadIdx.x] = ds;
    __syncthreads();
    int cnt = min(256, S - i0);
    for (int cc = 0; cc < ncol; cc++) {
      int c = threadIdx.x + cc * 256;
      if (c < dh) {
        float ak = acck[cc], av = accv[cc];
        for (int ii = 0; ii < cnt; ii++) {
          ak += dss[ii] * to_f(q[base + (i64)(i0 + ii) * d + c]);
          av += ps[ii] * to_f(d_o[base + (i64)(i0 + ii) * d + c]);
        }
        acck[cc] = ak;
        accv[cc] = av;
      }
    }
  }
  for (int cc = 0; cc < ncol; cc++) {
    int c = threadIdx.x + cc * 256;
    if (c < dh) {
      dk[base + (i64)j * d + c] = from_f<T>(acck[cc] * scale);
      dv[base + (i64)j * d + c] = from_f<T>(accv[cc]);
    }
  }
}

void launch_attn_dvec(int dt, const void* o, const void* d_o, float* dvec, int B, int S, int H, int dh,
                      hipStream_t s) {
  i64 rows = (i64)B * S * H;
  if (rows <= 0) return;
  DISPATCH_DT(dt, hipLaunchKernelGGL(attn_dvec_k<T>, dim3(cdiv(rows, 4)), dim3(256), 0, s, (const T*)o,
                                     (const T*)d_o, dvec, S, H, dh, rows));
}

void launch_attn_bwd_generic(int dt, const void* q, const void* k, const void* v, const void* o, const void* d_o,
                             const float* lse, float* dvec, void* dq, void* dk, void* dv, int B, int S, int H,
                             int dh, int causal, hipStream_t s) {
  if (B <= 0 || S <= 0) return;
  launch_attn_dvec(dt, o, d_o, dvec, B, S, H, dh, s);
  float scale = 1.0f / sqrtf((float)dh);
  size_t sm1 = (size_t)(2 * dh + 256) * sizeof(float);
  size_t sm2 = (size_t)(2 * dh + 512) * sizeof(float);
  DISPATCH_DT(dt, hipLaunchKernelGGL(attn_bwd_dq_generic_k<T>, dim3(S, H, B), dim3(256), sm1, s, (const T*)q,
                                     (const T*)k, (const T*)v, (const T*)d_o, lse, dvec, (T*)dq, S, H, dh, causal,
                                     scale));
  DISPATCH_DT(dt, hipLaunchKernelGGL(attn_bwd_dkv_generic_k<T>, dim3(S, H, B), dim3(256), sm2, s, (const T*)q,
                                     (const T*)k, (const T*)v, (const T*)d_o, lse, dvec, (T*)dk, (T*)dv, S, H, dh,
                                     causal, scale));
}
