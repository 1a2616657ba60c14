// Flash-style attention on the gfx950 matrix cores (bf16, head_dim 128, fp32 online softmax)
// for the cross-branch attention of Eq. 1: queries from stream 1, keys/values from stream 2.
//
// Layout: q,k,v,o,do,dq,dk,dv are [T, H*128] token-major, head hh in columns hh*128...
// All three kernels work on TRANSPOSED score tiles S^T[key, query] = K Q^T, so that in the
// MFMA result layout a lane owns one query (forward, dQ) or one key (dK/dV) column: softmax
// statistics and accumulator rescaling stay inside a lane, and the probability tile is
// already in the operand layout of the second product.  The operand that has to be read
// against its storage order (V^T, K^T, Q^T, dO^T) comes from LDS through the transposing
// read ds_read_b64_tr_b16.
#include "kernels.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

#define DH 128
#define BKV 64            // rows of the tile that is streamed through LDS
#define KST (DH + 8)      // LDS row stride (elements) of a tile read with 16-byte fragment reads
#define VST (DH + 32)     // LDS row stride of a tile read with transposing reads
#define BST (DH + 24)     // LDS row stride of a tile read both ways (backward: K; Q and dO): 76 dwords, i.e. rows 12
                          // banks apart, so that 16 rows x 16 bytes and 4 rows x 32 bytes both fall on distinct banks
#define LOG2E 1.4426950408889634f
#define LN2 0.6931471805599453f

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 16-byte fragment of a row-major LDS tile: rows r0 + (lane&31), columns kk*16 + (lane>>5)*8 ..
__device__ __forceinline__ bf16x8 frag_rows(const bf16* lds, int stride, int r0, int kk, int lane) {
  return *(const bf16x8*)(lds + (r0 + (lane & 31)) * stride + kk * 16 + (lane >> 5) * 8);
}
// Transposed fragment for a product whose contraction runs over the tile ROWS: operand row
// (MFMA row index) = tile column c0 + (lane&31); the 8 contraction slots u = 4*jp + i of half
// g = lane>>5 are tile rows rb + 8*jp + 4*g + i.  This matches a probability/score tile taken
// straight from the accumulator layout of a 32x32 MFMA (elements 8c..8c+7 of block c).
__device__ __forceinline__ bf16x8 frag_cols_tr(const bf16* lds, int stride, int rb, int c0, int lane) {
  int blk = lane >> 4, i16 = lane & 15;
  const bf16* p = lds + (rb + 4 * (blk >> 1) + (i16 >> 2)) * stride + c0 + 16 * (blk & 1) + 4 * (i16 & 3);
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * stride));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// elements 8c..8c+7 of an accumulator tile as a bf16 operand fragment
__device__ __forceinline__ bf16x8 acc_to_frag(const f32x16& a, int c) {
  bf16x8 r;
#pragma unroll
  for (int u = 0; u < 8; u++) r[u] = (__bf16)a[8 * c + u];
  return r;
}

// global [rows, DH] slice (row stride ld) -> registers: 64 rows x 16 chunks of 16 bytes, 4 per thread; rows at or
// past the sequence end are zero.  The loads are range-checked buffer loads: the descriptor covers the slice of one
// (batch, head) up to the last byte of row S - 1, so a row past the end is out of range and reads as zeros with no
// branch and no traffic, the address is one 32-bit offset per lane, and the loads of a tile issue back to back.
// (Predicated pointer loads put a branch and a full wait after every load and spilled their 64-bit addresses.)
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
struct RowSlice { __amdgpu_buffer_rsrc_t rs; unsigned ldb; };    // ldb = row stride in bytes
__device__ __forceinline__ RowSlice row_slice(const bf16* base, i64 ld, int S) {
  RowSlice r;
  r.rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, (short)0, (int)(((i64)S - 1) * ld * 2 + DH * 2), 0x00020000);
  r.ldb = (unsigned)(ld * 2);
  return r;
}
__device__ __forceinline__ void load_rows64(const RowSlice& sl, int row0, uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int c = threadIdx.x + 256 * i;
    const unsigned voff = (unsigned)(row0 + (c >> 4)) * sl.ldb + (unsigned)(c & 15) * 16u;
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(sl.rs, (int)voff, 0, 0);
    r[i] = make_uint4(v[0], v[1], v[2], v[3]);
  }
}
__device__ __forceinline__ void store_rows64(bf16* lds, int stride, const uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int c = threadIdx.x + 256 * i;
    *(uint4*)(lds + (c >> 4) * stride + (c & 15) * 8) = r[i];
  }
}

// ------------------------------------------------------------------------------------
// Forward.  Workgroup = 128 queries of one (batch, head); wave = 32 queries; keys/values
// streamed in tiles of 64.
// ------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256, 2) flash_fwd_k(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                   const bf16* __restrict__ v, bf16* __restrict__ o,
                                                   float* __restrict__ lse, int S, int H, int causal, float scale,
                                                   const unsigned char* __restrict__ row_skip) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* sK = (bf16*)smem_raw;               // 2 stages [64][KST]
  bf16* sV = sK + 2 * BKV * KST;            // 2 stages [64][VST]
  const int qt = gridDim.y - 1 - blockIdx.y;        // long (late) query tiles first, for every head
  const int hh = blockIdx.x, b = blockIdx.z;
  if (row_skip) {                           // every query of the tile is a finished row of the inverse's iteration
    int live = 0;                           // every wave checks all 128 rows of the tile: same answer, no LDS
    for (int r = qt * 128 + (int)(threadIdx.x & 63); r < min(S, qt * 128 + 128); r += 64) live |= row_skip[(i64)b * S + r] == 0;
    if (!__any(live)) return;
  }
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, g = lane >> 5;
  const i64 ld = (i64)H * DH;
  const bf16* qb = q + (i64)b * S * ld + hh * DH;
  const bf16* kb = k + (i64)b * S * ld + hh * DH;
  const bf16* vb = v + (i64)b * S * ld + hh * DH;
  const int q0 = qt * 128, qw = q0 + wv * 32;
  const int myq = qw + (lane & 31);
  const float sl2 = scale * LOG2E;

  bf16x8 qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; kk++) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (myq < S) t = *(const uint4*)(qb + (i64)myq * ld + kk * 16 + g * 8);
    qf[kk] = __builtin_bit_cast(bf16x8, t);
  }
  const int kv_lim = causal ? min(S, q0 + 128) : S;
  const int nt = (kv_lim + BKV - 1) / BKV;

  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) oacc[i][e] = 0.f;
  float m = -INFINITY, l = 0.f;

  uint4 rk[4], rv[4];
  const RowSlice slK = row_slice(kb, ld, S), slV = row_slice(vb, ld, S);
  load_rows64(slK, 0, rk);
  load_rows64(slV, 0, rv);
  store_rows64(sK, KST, rk);
  store_rows64(sV, VST, rv);
  __syncthreads();
  for (int t = 0; t < nt; t++) {
    const int cur = t & 1, kv0 = t * BKV;
    if (t + 1 < nt) {
      load_rows64(slK, kv0 + BKV, rk);
      load_rows64(slV, kv0 + BKV, rv);
    }
    const bf16* cK = sK + cur * BKV * KST;
    const bf16* cV = sV + cur * BKV * VST;
    if (!causal || kv0 <= qw + 31) {        // this wave has at least one unmasked key in the tile
      f32x16 sacc[2];
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) sacc[j][e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; kk++)
#pragma unroll
        for (int j = 0; j < 2; j++)
          sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(cK, KST, j * 32, kk, lane), qf[kk], sacc[j], 0, 0, 0);
      // scores in the log2 domain; keys past the sequence end or after the query are masked, which
      // only tiles on the diagonal or at the end of the sequence need
      const bool need_mask = (kv0 + BKV > S) || (causal && kv0 + BKV - 1 > qw);
      float mx = -INFINITY;
      if (need_mask) {
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
          for (int e = 0; e < 16; e++) {
            int kv = kv0 + j * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
            float sv = sacc[j][e] * sl2;
            if (kv >= S || (causal && kv > myq)) sv = -INFINITY;
            sacc[j][e] = sv;
            mx = fmaxf(mx, sv);
          }
      } else {
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
          for (int e = 0; e < 16; e++) {
            float sv = sacc[j][e] * sl2;
            sacc[j][e] = sv;
            mx = fmaxf(mx, sv);
          }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      const float mn = fmaxf(m, mx);
      const float msafe = (mn == -INFINITY) ? 0.f : mn;
      float rs = 0.f;
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          float p = fast_exp2(sacc[j][e] - msafe);
          sacc[j][e] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32, WAVE);
      // the running maximum settles after the first tiles: rescale the accumulator only when some
      // query of this wave actually raised it
      if (__any(mn > m)) {
        const float alpha = fast_exp2(m - msafe);
        l = l * alpha + rs;
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
          for (int e = 0; e < 16; e++) oacc[i][e] *= alpha;
      } else {
        l += rs;
      }
      m = mn;
      // O^T[dh, q] += V^T[dh, kv] P^T[kv, q]
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          bf16x8 pf = acc_to_frag(sacc[j], c);
#pragma unroll
          for (int dtile = 0; dtile < 4; dtile++)
            oacc[dtile] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_tr(cV, VST, j * 32 + c * 16, dtile * 32, lane),
                                                                  pf, oacc[dtile], 0, 0, 0);
        }
    }
    if (t + 1 < nt) {
      store_rows64(sK + (cur ^ 1) * BKV * KST, KST, rk);
      store_rows64(sV + (cur ^ 1) * BKV * VST, VST, rv);
    }
    __syncthreads();
  }
  if (myq < S) {
    const float inv = 1.0f / l;
    bf16* op = o + ((i64)b * S + myq) * ld + hh * DH;
#pragma unroll
    for (int dtile = 0; dtile < 4; dtile++)
#pragma unroll
      for (int jj = 0; jj < 4; jj++) {
        bf16x4 w;
#pragma unroll
        for (int i = 0; i < 4; i++) w[i] = (__bf16)(oacc[dtile][jj * 4 + i] * inv);
        *(bf16x4*)(op + dtile * 32 + jj * 8 + g * 4) = w;
      }
    if (g == 0) lse[((i64)b * H + hh) * S + myq] = (m + __log2f(l)) * LN2;
  }
}

int launch_attn_fwd_flash(const void* q, const void* k, const void* v, void* o, float* lse, int B, int S, int H,
                          int dh, int causal, hipStream_t s, const unsigned char* row_skip) {
  if (dh != DH || B <= 0 || S <= 0) return 1;
  if ((i64)S * H * DH * 2 >= ((i64)1 << 31)) return 1;      // one sequence of one tensor is addressed with 32-bit offsets
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return 1;
  size_t smem = (size_t)2 * BKV * (KST + VST) * sizeof(bf16);
  static std::atomic<unsigned long long> attr_mask{0};
  if (attr_needed(attr_mask)) {
    (void)hipFuncSetAttribute((const void*)flash_fwd_k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_done(attr_mask);
  }
  hipLaunchKernelGGL(flash_fwd_k, dim3(H, cdiv(S, 128), B), dim3(256), smem, s, (const bf16*)q, (const bf16*)k,
                     (const bf16*)v, (bf16*)o, lse, S, H, causal, 1.0f / sqrtf((float)dh), row_skip);
  return 0;
}

// ------------------------------------------------------------------------------------
// Backward, part 1: dQ.  Workgroup = 128 queries, wave = 32 queries (one per lane column);
// keys/values streamed in tiles of 64.  Per tile:
//   S^T = K Q^T,  P^T = exp(S^T*scale - lse),  dP^T = V dO^T,  dS^T = P^T (dP^T - D) scale,
//   dQ^T += K^T dS^T.
// ------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256, 2) flash_bwd_dq_k(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                      const bf16* __restrict__ v, const bf16* __restrict__ d_o,
                                                      const float* __restrict__ lse, const float* __restrict__ dvec,
                                                      bf16* __restrict__ dq, int S, int H, int causal, float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* sK = (bf16*)smem_raw;               // 2 stages [64][BST]
  bf16* sV = sK + 2 * BKV * BST;            // 2 stages [64][BST]
  const int qt = gridDim.y - 1 - blockIdx.y;
  const int hh = blockIdx.x, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, g = lane >> 5;
  const i64 ld = (i64)H * DH;
  const i64 boff = (i64)b * S * ld + hh * DH;
  const int q0 = qt * 128, qw = q0 + wv * 32;
  const int myq = qw + (lane & 31);
  const float sl2 = scale * LOG2E;

  bf16x8 qf[8], dof[8];
#pragma unroll
  for (int kk = 0; kk < 8; kk++) {
    uint4 t = make_uint4(0, 0, 0, 0), u = make_uint4(0, 0, 0, 0);
    if (myq < S) {
      t = *(const uint4*)(q + boff + (i64)myq * ld + kk * 16 + g * 8);
      u = *(const uint4*)(d_o + boff + (i64)myq * ld + kk * 16 + g * 8);
    }
    qf[kk] = __builtin_bit_cast(bf16x8, t);
    dof[kk] = __builtin_bit_cast(bf16x8, u);
  }
  const float mylse = (myq < S) ? lse[((i64)b * H + hh) * S + myq] * LOG2E : 0.f;
  const float myD = (myq < S) ? dvec[((i64)b * H + hh) * S + myq] : 0.f;
  const int kv_lim = causal ? min(S, q0 + 128) : S;
  const int nt = (kv_lim + BKV - 1) / BKV;

  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[i][e] = 0.f;

  uint4 rk[4], rv[4];
  const RowSlice slK = row_slice(k + boff, ld, S), slV = row_slice(v + boff, ld, S);
  load_rows64(slK, 0, rk);
  load_rows64(slV, 0, rv);
  store_rows64(sK, BST, rk);
  store_rows64(sV, BST, rv);
  __syncthreads();
  for (int t = 0; t < nt; t++) {
    const int cur = t & 1, kv0 = t * BKV;
    if (t + 1 < nt) {
      load_rows64(slK, kv0 + BKV, rk);
      load_rows64(slV, kv0 + BKV, rv);
    }
    const bf16* cK = sK + cur * BKV * BST;
    const bf16* cV = sV + cur * BKV * BST;
    if (!causal || kv0 <= qw + 31) {
      f32x16 sacc[2], dpacc[2];
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) { sacc[j][e] = 0.f; dpacc[j][e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 8; kk++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
          sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(cK, BST, j * 32, kk, lane), qf[kk], sacc[j], 0, 0, 0);
          dpacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(cV, BST, j * 32, kk, lane), dof[kk], dpacc[j], 0, 0, 0);
        }
      const bool need_mask = (kv0 + BKV > S) || (causal && kv0 + BKV - 1 > qw);
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          float p = fast_exp2(sacc[j][e] * sl2 - mylse);
          if (need_mask) {
            int kv = kv0 + j * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
            if (kv >= S || (causal && kv > myq)) p = 0.f;
          }
          sacc[j][e] = p * (dpacc[j][e] - myD) * scale;      // dS^T
        }
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          bf16x8 dsf = acc_to_frag(sacc[j], c);
#pragma unroll
          for (int dtile = 0; dtile < 4; dtile++)
            acc[dtile] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_tr(cK, BST, j * 32 + c * 16, dtile * 32, lane),
                                                                 dsf, acc[dtile], 0, 0, 0);
        }
    }
    if (t + 1 < nt) {
      store_rows64(sK + (cur ^ 1) * BKV * BST, BST, rk);
      store_rows64(sV + (cur ^ 1) * BKV * BST, BST, rv);
    }
    __syncthreads();
  }
  if (myq < S) {
    bf16* op = dq + boff + (i64)myq * ld;
#pragma unroll
    for (int dtile = 0; dtile < 4; dtile++)
#pragma unroll
      for (int jj = 0; jj < 4; jj++) {
        bf16x4 w;
#pragma unroll
        for (int i = 0; i < 4; i++) w[i] = (__bf16)acc[dtile][jj * 4 + i];
        *(bf16x4*)(op + dtile * 32 + jj * 8 + g * 4) = w;
      }
  }
}

// ------------------------------------------------------------------------------------
// Backward, part 2: dK and dV.  Workgroup = 128 keys, wave = 32 keys (one per lane column);
// queries (with dO, lse, D) streamed in tiles of 64, starting at the diagonal when causal.
//   S = Q K^T,  P = exp(S*scale - lse),  dP = dO V^T,  dS = P (dP - D) scale,
//   dV^T += dO^T P,   dK^T += Q^T dS.
// ------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) flash_bwd_dkv_k(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                       const bf16* __restrict__ v, const bf16* __restrict__ d_o,
                                                       const float* __restrict__ lse, const float* __restrict__ dvec,
                                                       bf16* __restrict__ dk, bf16* __restrict__ dv, int S, int H,
                                                       int causal, float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* sQ = (bf16*)smem_raw;               // 2 stages [64][BST]
  bf16* sO = sQ + 2 * BKV * BST;            // 2 stages [64][BST]  (dO)
  float* sL = (float*)(sO + 2 * BKV * BST); // 2 stages [64] lse (log2 domain), then 2 stages [64] D
  float* sD = sL + 2 * BKV;
  const int kt = blockIdx.y;                // early key tiles see the most queries when causal: first
  const int hh = blockIdx.x, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, g = lane >> 5;
  const i64 ld = (i64)H * DH;
  const i64 boff = (i64)b * S * ld + hh * DH;
  const i64 soff = ((i64)b * H + hh) * S;
  const int k0 = kt * 128, kw = k0 + wv * 32;
  const int mykv = kw + (lane & 31);
  const float sl2 = scale * LOG2E;

  bf16x8 kf[8], vf[8];
#pragma unroll
  for (int kk = 0; kk < 8; kk++) {
    uint4 t = make_uint4(0, 0, 0, 0), u = make_uint4(0, 0, 0, 0);
    if (mykv < S) {
      t = *(const uint4*)(k + boff + (i64)mykv * ld + kk * 16 + g * 8);
      u = *(const uint4*)(v + boff + (i64)mykv * ld + kk * 16 + g * 8);
    }
    kf[kk] = __builtin_bit_cast(bf16x8, t);
    vf[kk] = __builtin_bit_cast(bf16x8, u);
  }
  const int t_lo = causal ? k0 / BKV : 0;
  const int nt = (S + BKV - 1) / BKV;

  f32x16 dkacc[4], dvacc[4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) { dkacc[i][e] = 0.f; dvacc[i][e] = 0.f; }

  uint4 rq[4], ro[4];
  const RowSlice slQ = row_slice(q + boff, ld, S), slO = row_slice(d_o + boff, ld, S);
  float rl = 0.f, rd = 0.f;
  auto load_stats = [&](int q0) {
    if (threadIdx.x < BKV) {
      int qq = q0 + threadIdx.x;
      rl = (qq < S) ? lse[soff + qq] * LOG2E : INFINITY;    // +inf: probability 0 for rows past the end
      rd = (qq < S) ? dvec[soff + qq] : 0.f;
    }
  };
  auto store_stats = [&](int stage) {
    if (threadIdx.x < BKV) { sL[stage * BKV + threadIdx.x] = rl; sD[stage * BKV + threadIdx.x] = rd; }
  };
  if (t_lo < nt) {
    load_rows64(slQ, t_lo * BKV, rq);
    load_rows64(slO, t_lo * BKV, ro);
    load_stats(t_lo * BKV);
    store_rows64(sQ, BST, rq);
    store_rows64(sO, BST, ro);
    store_stats(0);
  }
  __syncthreads();
  for (int t = t_lo; t < nt; t++) {
    const int cur = (t - t_lo) & 1, q0 = t * BKV;
    if (t + 1 < nt) {
      load_rows64(slQ, q0 + BKV, rq);
      load_rows64(slO, q0 + BKV, ro);
      load_stats(q0 + BKV);
    }
    const bf16* cQ = sQ + cur * BKV * BST;
    const bf16* cO = sO + cur * BKV * BST;
    const float* cL = sL + cur * BKV;
    const float* cD = sD + cur * BKV;
    if (!causal || q0 + BKV - 1 >= kw) {     // some query of the tile can see some key of this wave
      f32x16 sacc[2], dpacc[2];
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) { sacc[j][e] = 0.f; dpacc[j][e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 8; kk++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
          sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(cQ, BST, j * 32, kk, lane), kf[kk], sacc[j], 0, 0, 0);
          dpacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(cO, BST, j * 32, kk, lane), vf[kk], dpacc[j], 0, 0, 0);
        }
      const bool need_mask = causal && (q0 < kw + 31);           // some query of the tile precedes some key of the wave
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int eb = 0; eb < 4; eb++) {
          const int r0 = j * 32 + eb * 8 + g * 4;                 // 4 consecutive query rows inside the tile
          const float4 l4 = *(const float4*)(cL + r0), d4 = *(const float4*)(cD + r0);
          const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int i = 0; i < 4; i++) {
            const int e = eb * 4 + i;
            float p = fast_exp2(sacc[j][e] * sl2 - lv[i]);
            if (need_mask && mykv > q0 + r0 + i) p = 0.f;
            dpacc[j][e] = p * (dpacc[j][e] - dv4[i]) * scale;     // dS
            sacc[j][e] = p;                                        // P
          }
        }
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          bf16x8 pf = acc_to_frag(sacc[j], c);
          bf16x8 dsf = acc_to_frag(dpacc[j], c);
#pragma unroll
          for (int dtile = 0; dtile < 4; dtile++) {
            dvacc[dtile] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_tr(cO, BST, j * 32 + c * 16, dtile * 32, lane),
                                                                   pf, dvacc[dtile], 0, 0, 0);
            dkacc[dtile] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_tr(cQ, BST, j * 32 + c * 16, dtile * 32, lane),
                                                                   dsf, dkacc[dtile], 0, 0, 0);
          }
        }
    }
    if (t + 1 < nt) {
      store_rows64(sQ + (cur ^ 1) * BKV * BST, BST, rq);
      store_rows64(sO + (cur ^ 1) * BKV * BST, BST, ro);
      store_stats(cur ^ 1);
    }
    __syncthreads();
  }
  if (mykv < S) {
    bf16* pk = dk + boff + (i64)mykv * ld;
    bf16* pv = dv + boff + (i64)mykv * ld;
#pragma unroll
    for (int dtile = 0; dtile < 4; dtile++)
#pragma unroll
      for (int jj = 0; jj < 4; jj++) {
        bf16x4 a, c2;
#pragma unroll
        for (int i = 0; i < 4; i++) { a[i] = (__bf16)dkacc[dtile][jj * 4 + i]; c2[i] = (__bf16)dvacc[dtile][jj * 4 + i]; }
        *(bf16x4*)(pk + dtile * 32 + jj * 8 + g * 4) = a;
        *(bf16x4*)(pv + dtile * 32 + jj * 8 + g * 4) = c2;
      }
  }
}

int launch_attn_bwd_flash(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                          const float* lse, float* dvec, void* dq, void* dk, void* dv, int B, int S, int H, int dh,
                          int causal, hipStream_t s) {
  if (dh != DH || B <= 0 || S <= 0) return 1;
  if ((i64)S * H * DH * 2 >= ((i64)1 << 31)) return 1;      // one sequence of one tensor is addressed with 32-bit offsets
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o | (uintptr_t)d_o | (uintptr_t)dq | (uintptr_t)dk |
       (uintptr_t)dv) & 15)
    return 1;
  launch_attn_dvec(1, o, d_o, dvec, B, S, H, dh, s);
  const float scale = 1.0f / sqrtf((float)dh);
  size_t sm1 = (size_t)4 * BKV * BST * sizeof(bf16);
  size_t sm2 = sm1 + 4 * BKV * sizeof(float);
  static std::atomic<unsigned long long> attr_mask{0};
  if (attr_needed(attr_mask)) {
    (void)hipFuncSetAttribute((const void*)flash_bwd_dq_k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm1);
    (void)hipFuncSetAttribute((const void*)flash_bwd_dkv_k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm2);
    attr_done(attr_mask);
  }
  dim3 grid(H, cdiv(S, 128), B);
  hipLaunchKernelGGL(flash_bwd_dq_k, grid, dim3(256), sm1, s, (const bf16*)q, (const bf16*)k, (const bf16*)v,
                     (const bf16*)d_o, lse, dvec, (bf16*)dq, S, H, causal, scale);
  hipLaunchKernelGGL(flash_bwd_dkv_k, grid, dim3(256), sm2, s, (const bf16*)q, (const bf16*)k, (const bf16*)v,
                     (const bf16*)d_o, lse, dvec, (bf16*)dk, (bf16*)dv, S, H, causal, scale);
  return 0;
}
