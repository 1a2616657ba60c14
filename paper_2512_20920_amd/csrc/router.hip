// Routing of the MoE half (MLP_pt of section 3.2 read as a Qwen2-MoE sparse block):
// router logits, softmax, top-k, per-expert offsets and the token permutation, the
// weighted combine, and the element-wise parts of their backward passes.
// Everything here is deterministic: integer results depend only on the logits' bits.
#include "kernels.h"
#include <initializer_list>

#define DISPATCH_DT(dt, ...)                                  \
  do {                                                        \
    if ((dt) == 0) { typedef float T; __VA_ARGS__; }          \
    else { typedef bf16 T; __VA_ARGS__; }                     \
  } while (0)

// ---------------------------------------------------------------------------------
// Router.  The logits are z = W_r (P_up_m Norm(Y1)) + b.  They are evaluated as
// (W_r P_up_m diag(gain)) Y1 / rms(Y1) with the product matrix held in fp32 and applied to the
// stored Y1 by an fp32 GEMM (zraw), so the selection depends only on the bits of Y1 and the
// weights, not on the rounding of the bf16 intermediate P_up_m Norm(Y1).  Column E of zraw
// (optional) is the shared expert's gate vector folded the same way.
// One wave per token.  Outputs: probs[T,E] (softmax over all experts), idx/wts[T,k] (slots
// by descending logit, equal logits -> lower expert index), gamma[T] = sigmoid(gate logit).
// ---------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(256) router_k(const T* __restrict__ y1, i64 ld, const float* __restrict__ zparts,
                                                int n_parts, const float* __restrict__ b_router,
                                                float* __restrict__ probs, int* __restrict__ idx,
                                                float* __restrict__ wts, float* __restrict__ gamma, int Tn, int h,
                                                int E, int k, int has_gate, int norm_topk, float eps) {
  extern __shared__ float sm[];          // per wave: z[E1]
  const int E1 = E + (has_gate ? 1 : 0);
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* z = sm + (size_t)wv * E1;
  const int t = blockIdx.x * 4 + wv;
  if (t >= Tn) return;                   // whole wave leaves; no block barriers below
  const T* yr = y1 + (i64)t * ld;
  float ss = 0.f;
  for (int j = lane; j < h; j += 64) { float v = to_f(yr[j]); ss += v * v; }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)h + eps);
  for (int e = lane; e < E1; e += 64) {
    float raw = 0.f;                     // the k-slices of the logit GEMM, added in slice order
    for (int p = 0; p < n_parts; p++) raw += zparts[((i64)p * Tn + t) * E1 + e];
    z[e] = raw * r + ((e < E && b_router) ? b_router[e] : 0.f);
  }
  __builtin_amdgcn_wave_barrier();       // LDS traffic of one wave is executed in order
  // softmax over the E routed logits
  float mx = -INFINITY;
  for (int e = lane; e < E; e += 64) mx = fmaxf(mx, z[e]);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int e = lane; e < E; e += 64) sum += __expf(z[e] - mx);
  sum = wave_sum(sum);
  const float inv = 1.0f / sum;
  for (int e = lane; e < E; e += 64) probs[(i64)t * E + e] = __expf(z[e] - mx) * inv;
  // top-k by k rounds of (value desc, index asc) arg-max over the experts not chosen yet.  A logit that is not a
  // number ranks as minus infinity, and a lane remembers which of its own experts (e = lane + 64 j, E <= 256) are
  // taken, so every round finds a valid expert that no earlier round has chosen, whatever the logits hold: a token
  // with a non-finite input cannot disturb the tables of other tokens.
  __builtin_amdgcn_wave_barrier();
  float wsum = 0.f;
  float myw = 0.f;                        // lane s keeps the weight of slot s
  unsigned taken = 0;                     // bit j: expert lane + 64 j has been chosen
  for (int s = 0; s < k; s++) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int e = lane, j = 0; e < E; e += 64, j++) {
      if ((taken >> j) & 1u) continue;
      float v = z[e];
      v = (v == v) ? v : -INFINITY;
      if (v > bv || (v == bv && e < bi)) { bv = v; bi = e; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      float ov = __shfl_xor(bv, o, WAVE);
      int oi = __shfl_xor(bi, o, WAVE);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    // the comparator is a total order (no NaN takes part), so every lane now holds the same (bv, bi); with
    // top_k <= E at least one expert was left, so bi < E (the clamp only guards the stores below)
    bi = min(bi, E - 1);
    if ((bi & 63) == lane) taken |= 1u << (bi >> 6);
    float p = __expf(bv - mx) * inv;
    wsum += p;
    if (lane == s) myw = p;
    if (lane == 0) idx[(i64)t * k + s] = bi;
  }
  if (lane < k) wts[(i64)t * k + lane] = norm_topk ? myw / wsum : myw;
  if (has_gate && lane == 0) gamma[t] = sigmoid_f(z[E]);
}

void launch_router(int dt, const void* y1, i64 ld, const float* zparts, int n_parts, const float* b_router, float* probs, int* idx,
                   float* wts, float* gamma, int Tn, int h, int E, int k, int has_gate, int norm_topk, float eps,
                   hipStream_t s) {
  if (Tn <= 0) return;
  size_t smem = (size_t)4 * (E + 1) * sizeof(float);
  DISPATCH_DT(dt, hipLaunchKernelGGL(router_k<T>, dim3(cdiv(Tn, 4)), dim3(256), smem, s, (const T*)y1, ld, zparts,
                                     n_parts, b_router, probs, idx, wts, gamma, Tn, h, E, k, has_gate, norm_topk, eps));
}

// ---------------------------------------------------------------------------------
// Permutation.  One workgroup of 16 waves; wave w owns the contiguous slice of the T*k
// (token, slot) entries [w*per, (w+1)*per).  Pass 1 counts per (wave, expert); the prefix
// over waves gives each wave its first row inside every expert; pass 2 hands out rows in
// entry order, which keeps (token, slot) order inside an expert (a stable grouping).
// Also emits the m-tile lists used by the grouped GEMMs: tile i covers rows
// [tile_m0[i], min(tile_m0[i]+bm, offsets[g+1])) of expert g = tile_group[i]; unused = -1.
// ---------------------------------------------------------------------------------
#define PERM_WAVES 16
#define PERM_UNROLL 8
__device__ __forceinline__ void same_expert_mask(int x, bool valid, int nbits, unsigned long long& same) {
  same = __ballot(valid);
  for (int b = 0; b < nbits; b++) {
    unsigned long long m = __ballot(valid && ((x >> b) & 1));
    same &= ((x >> b) & 1) ? m : ~m;
  }
}

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(v, o, WAVE);
    if (lane >= o) v += u;
  }
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}

__global__ void __launch_bounds__(PERM_WAVES * 64) permute_k(
    const int* __restrict__ idx, int N, int E, int* __restrict__ counts, int* __restrict__ offsets,
    int* __restrict__ row_map, int* __restrict__ inv_map, TileLists tl) {
  extern __shared__ int ism[];            // cnt[PERM_WAVES][E], off[E+1], tile counts [E+1]
  int* cnt = ism;
  int* off = ism + PERM_WAVES * E;
  const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  int nbits = 0;
  while ((1 << nbits) < E) nbits++;
  for (int i = threadIdx.x; i < PERM_WAVES * E; i += blockDim.x) cnt[i] = 0;
  __syncthreads();
  const int per = (N + PERM_WAVES - 1) / PERM_WAVES;
  const int lo = wv * per, hi = min(N, lo + per);
  int* mycnt = cnt + wv * E;
  for (int base0 = lo; base0 < hi; base0 += 64 * PERM_UNROLL) {
    int xs[PERM_UNROLL];                  // the loads of a batch are independent: one memory latency per batch
#pragma unroll
    for (int u = 0; u < PERM_UNROLL; u++) { int f = base0 + u * 64 + lane; xs[u] = f < hi ? idx[f] : 0; }
#pragma unroll
    for (int u = 0; u < PERM_UNROLL; u++) {
      int f = base0 + u * 64 + lane;
      bool valid = f < hi;
      int x = min(max(xs[u], 0), E - 1);    // an index outside [0, E) cannot reach the LDS tables
      unsigned long long same;
      same_expert_mask(x, valid, nbits, same);
      if (valid && (same & below) == 0) mycnt[x] += __popcll(same);   // group leader; groups are disjoint
      __builtin_amdgcn_wave_barrier();
    }
  }
  __syncthreads();
  // exclusive prefix over waves per expert, totals, offsets
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    int run = 0;
    for (int w = 0; w < PERM_WAVES; w++) { int c = cnt[w * E + e]; cnt[w * E + e] = run; run += c; }
    counts[e] = run;
    off[e + 1] = run;                     // totals for now
  }
  __syncthreads();
  if (wv == 0) {                          // offsets = prefix sums of the totals, 64 experts per step
    if (lane == 0) off[0] = 0;
    int carry = 0;
    for (int base = 0; base < E; base += 64) {
      const int e = base + lane;
      const int incl = carry + wave_inclusive_scan(e < E ? off[e + 1] : 0, lane);
      if (e < E) off[e + 1] = incl;
      carry = __shfl(incl, 63, WAVE);
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e <= E; e += blockDim.x) offsets[e] = off[e];
  // Waves 0-2 write one tile list each, wave 3 the evenness flag; none of them changes what the row pass below
  // reads (off, cnt), so nothing waits for them.
  if (wv < 3) {
    // tile lists: expert e owns the slots after the tiles of experts 0..e-1; slots past the last tile are marked
    // unused.  The number of tiles of an expert is an exact division: the fill loop below writes ceil(rows / bm)
    // slots per expert, and a count taken any other way (a shift, for a height that is not a power of two) would
    // leave slots of the list unwritten, with whatever the workspace held, for the GEMM to use as an expert index.
    const int pass = wv;
    const int bm = tl.bm[pass], mx = tl.max_tiles[pass];
    int* tg = tl.group[pass];
    int* tm = tl.m0[pass];
    int* tf = tl.first[pass];
    int total = 0;
    for (int base = 0; base < E; base += 64) {
      const int e = base + lane;
      const int m_lo = e < E ? off[e] : 0, m_hi = e < E ? off[e + 1] : 0;
      const int mine = (m_hi - m_lo + bm - 1) / bm;
      const int incl = wave_inclusive_scan(mine, lane);
      const int first = total + incl - mine;
      int i = first;
      for (int m = m_lo; m < m_hi; m += bm, i++)
        if (i < mx) { tg[i] = e; tm[i] = m; tf[i] = (first << 16) | mine; }
      total += __shfl(incl, 63, WAVE);
    }
    for (int i = total + lane; i < mx; i += 64) { tg[i] = -1; tm[i] = 0; tf[i] = (i << 16) | 1; }
    if (lane == 0) tl.count[pass] = min(total, mx);
  } else if (wv == 3) {
    // Is the routing even enough for the per-expert weight-gradient launches to give each expert to two XCDs?  Then
    // experts e = 4 r + q (q = 0..3) are worked on by XCD pair q in round r, and the pairs finish together only if
    // their experts cost about the same: a tile costs a fixed part (first loads, stores: about 5 k-steps' worth) plus
    // one k-step per 64 rows of the expert.  Even = no pair more than 6 % above the mean.
    int cost[4] = {0, 0, 0, 0};
    for (int base = 0; base < E; base += 64) {
      const int e = base + lane;
      const int mine = e < E ? 5 + (off[e + 1] - off[e] + 63) / 64 : 0;
#pragma unroll
      for (int q = 0; q < 4; q++) cost[q] += wave_sum((e & 3) == q ? mine : 0);
    }
    const int tot = cost[0] + cost[1] + cost[2] + cost[3];
    const int mx = max(max(cost[0], cost[1]), max(cost[2], cost[3]));
    if (lane == 0) tl.count[3] = (E >= 8 && 400 * mx <= 106 * tot) ? 1 : 0;
  }
  for (int base0 = lo; base0 < hi; base0 += 64 * PERM_UNROLL) {
    int xs[PERM_UNROLL];
#pragma unroll
    for (int u = 0; u < PERM_UNROLL; u++) { int f = base0 + u * 64 + lane; xs[u] = f < hi ? idx[f] : 0; }
#pragma unroll
    for (int u = 0; u < PERM_UNROLL; u++) {
      int f = base0 + u * 64 + lane;
      bool valid = f < hi;
      int x = min(max(xs[u], 0), E - 1);
      unsigned long long same;
      same_expert_mask(x, valid, nbits, same);
      int rank = __popcll(same & below);
      int start = valid ? mycnt[x] : 0;     // every lane of a group reads before its leader updates
      __builtin_amdgcn_wave_barrier();
      if (valid && rank == 0) mycnt[x] = start + __popcll(same);
      __builtin_amdgcn_wave_barrier();
      if (valid) {
        int pos = off[x] + start + rank;
        row_map[pos] = f;
        inv_map[f] = pos;
      }
    }
  }
}

void launch_permute(const int* idx, int Tn, int k, int E, int* counts, int* offsets, int* row_map, int* inv_map,
                    const TileLists& tl, hipStream_t s) {
  size_t smem = (size_t)(PERM_WAVES * E + 2 * (E + 1)) * sizeof(int);
  hipLaunchKernelGGL(permute_k, dim3(1), dim3(PERM_WAVES * 64), smem, s, idx, Tn * k, E, counts, offsets, row_map,
                     inv_map, tl);
}

// ---------------------------------------------------------------------------------
// Combine: rs[t] = sum_slot wts[t,slot] * yp[inv_map[t*k+slot]] + gamma[t] * ys[t], slots added
// in slot order (fixed order, no atomics).
// ---------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(256) combine_k(const T* __restrict__ yp, const int* __restrict__ inv_map,
                                                 const float* __restrict__ wts, const T* __restrict__ ys,
                                                 const float* __restrict__ gamma, T* __restrict__ rs, int d, int k) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x; c < d; c += 256) {
    float acc = 0.f;
    for (int s = 0; s < k; s++) {
      int pos = inv_map[(i64)t * k + s];
      acc += wts[(i64)t * k + s] * to_f(yp[(i64)pos * d + c]);
    }
    if (ys) acc += gamma[t] * to_f(ys[(i64)t * d + c]);
    rs[(i64)t * d + c] = from_f<T>(acc);
  }
}
// bf16, d % 8 == 0, 16-byte aligned rows: one lane handles 8 consecutive columns with 16-byte accesses
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
static bool vec8_ok(int dt, int d, std::initializer_list<const void*> ptrs) {
  if (dt != 1 || (d & 7)) return false;
  for (const void* q : ptrs) if ((uintptr_t)q & 15) return false;
  return true;
}
__global__ void __launch_bounds__(256) combine_v8_k(const bf16* __restrict__ yp, const int* __restrict__ inv_map,
                                                    const float* __restrict__ wts, const bf16* __restrict__ ys,
                                                    const float* __restrict__ gamma, bf16* __restrict__ rs, int d, int k) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; q++) acc[q] = 0.f;
    for (int s = 0; s < k; s++) {
      const int pos = inv_map[(i64)t * k + s];
      const float w = wts[(i64)t * k + s];
      const bf16x8_t v = *(const bf16x8_t*)(yp + (i64)pos * d + c);
#pragma unroll
      for (int q = 0; q < 8; q++) acc[q] += w * (float)v[q];
    }
    if (ys) {
      const float g = gamma[t];
      const bf16x8_t v = *(const bf16x8_t*)(ys + (i64)t * d + c);
#pragma unroll
      for (int q = 0; q < 8; q++) acc[q] += g * (float)v[q];
    }
    bf16x8_t o;
#pragma unroll
    for (int q = 0; q < 8; q++) o[q] = (__bf16)acc[q];
    *(bf16x8_t*)(rs + (i64)t * d + c) = o;
  }
}
void launch_combine(int dt, const void* yp, const int* inv_map, const float* wts, const void* ys,
                    const float* gamma, void* rs, int Tn, int d, int k, hipStream_t s) {
  if (Tn <= 0) return;
  if (vec8_ok(dt, d, {yp, ys, rs})) {
    hipLaunchKernelGGL(combine_v8_k, dim3(Tn), dim3(256), 0, s, (const bf16*)yp, inv_map, wts, (const bf16*)ys, gamma,
                       (bf16*)rs, d, k);
    return;
  }
  DISPATCH_DT(dt, hipLaunchKernelGGL(combine_k<T>, dim3(Tn), dim3(256), 0, s, (const T*)yp, inv_map, wts,
                                     (const T*)ys, gamma, (T*)rs, d, k));
}

// Combine in the half-width space of the streams (pre-merged down projections: expert outputs already have width h)
// with the coupling update of Eq. 2 / the first line of the inverse in the same pass:
//   branch[t] = sum_slot wts[t,slot] * yp[inv_map[t*k+slot]] + gamma[t] * ys[t]      (slot order, fp32)
//   dst[t] = resid[t] + sign * branch[t]   (rounded once to the stream type); tap (optional) keeps branch in fp32.
template <class T, class TS>
__global__ void __launch_bounds__(256) combine_couple_k(const T* __restrict__ yp, const int* __restrict__ inv_map,
                                                        const float* __restrict__ wts, const T* __restrict__ ys,
                                                        const float* __restrict__ gamma, const TS* resid, i64 ldr,
                                                        float sign, TS* dst, i64 ldd, float* __restrict__ tap, int h, int k) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x; c < h; c += 256) {
    float acc = 0.f;
    for (int s = 0; s < k; s++) {
      int pos = inv_map[(i64)t * k + s];
      acc += wts[(i64)t * k + s] * to_f(yp[(i64)pos * h + c]);
    }
    if (ys) acc += gamma[t] * to_f(ys[(i64)t * h + c]);
    if (tap) tap[(i64)t * h + c] = acc;
    dst[(i64)t * ldd + c] = from_f<TS>(to_f(resid[(i64)t * ldr + c]) + sign * acc);   // (dst may be resid: same element)
  }
}
void launch_combine_couple(int dt, int ts, const void* yp, const int* inv_map, const float* wts, const void* ys,
                           const float* gamma, const void* resid, i64 ldr, float sign, void* dst, i64 ldd, float* tap,
                           int Tn, int h, int k, hipStream_t s) {
  if (Tn <= 0) return;
  if (dt == 0)
    hipLaunchKernelGGL((combine_couple_k<float, float>), dim3(Tn), dim3(256), 0, s, (const float*)yp, inv_map, wts,
                       (const float*)ys, gamma, (const float*)resid, ldr, sign, (float*)dst, ldd, tap, h, k);
  else if (ts == 0)
    hipLaunchKernelGGL((combine_couple_k<bf16, float>), dim3(Tn), dim3(256), 0, s, (const bf16*)yp, inv_map, wts,
                       (const bf16*)ys, gamma, (const float*)resid, ldr, sign, (float*)dst, ldd, tap, h, k);
  else
    hipLaunchKernelGGL((combine_couple_k<bf16, bf16>), dim3(Tn), dim3(256), 0, s, (const bf16*)yp, inv_map, wts,
                       (const bf16*)ys, gamma, (const bf16*)resid, ldr, sign, (bf16*)dst, ldd, tap, h, k);
}

// ---------------------------------------------------------------------------------
// Backward of the combine, one workgroup per token:
//   dgamma = <drs, ys>, gate-logit gradient dzext[t,E] = dgamma*gamma*(1-gamma), dys = gamma*drs
//   dw[t,slot] = <drs, yp[pos]>,  dyp[pos] = wts[t,slot]*drs
// ---------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(256) moe_bwd_rows_k(const T* __restrict__ drs, const T* __restrict__ yp,
                                                      const T* __restrict__ ys, const int* __restrict__ inv_map,
                                                      const float* __restrict__ wts, const float* __restrict__ gamma,
                                                      T* __restrict__ dyp, T* __restrict__ dys, float* __restrict__ dw,
                                                      float* __restrict__ dzext, int d, int k, int E1, int has_gate) {
  __shared__ float red[4];
  const int t = blockIdx.x;
  const T* dr = drs + (i64)t * d;
  if (has_gate) {
    float g = gamma[t];
    float acc = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) {
      float v = to_f(dr[c]);
      acc += v * to_f(ys[(i64)t * d + c]);
      dys[(i64)t * d + c] = from_f<T>(g * v);
    }
    acc = block_sum_256(acc, red);
    if (threadIdx.x == 0) dzext[(i64)t * E1 + (E1 - 1)] = acc * g * (1.f - g);
  }
  for (int s = 0; s < k; s++) {
    int pos = inv_map[(i64)t * k + s];
    float w = wts[(i64)t * k + s];
    float acc = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) {
      float v = to_f(dr[c]);
      acc += v * to_f(yp[(i64)pos * d + c]);
      dyp[(i64)pos * d + c] = from_f<T>(w * v);
    }
    acc = block_sum_256(acc, red);
    if (threadIdx.x == 0) dw[(i64)t * k + s] = acc;
  }
}
__global__ void __launch_bounds__(256) moe_bwd_rows_v8_k(const bf16* __restrict__ drs, const bf16* __restrict__ yp,
                                                         const bf16* __restrict__ ys, const int* __restrict__ inv_map,
                                                         const float* __restrict__ wts, const float* __restrict__ gamma,
                                                         bf16* __restrict__ dyp, bf16* __restrict__ dys,
                                                         float* __restrict__ dw, float* __restrict__ dzext, int d, int k,
                                                         int E1, int has_gate) {
  __shared__ float red[4];
  const int t = blockIdx.x;
  const bf16* dr = drs + (i64)t * d;
  if (has_gate) {
    const float g = gamma[t];
    float acc = 0.f;
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
      const bf16x8_t v = *(const bf16x8_t*)(dr + c), y = *(const bf16x8_t*)(ys + (i64)t * d + c);
      bf16x8_t o;
#pragma unroll
      for (int q = 0; q < 8; q++) { acc += (float)v[q] * (float)y[q]; o[q] = (__bf16)(g * (float)v[q]); }
      *(bf16x8_t*)(dys + (i64)t * d + c) = o;
    }
    acc = block_sum_256(acc, red);
    if (threadIdx.x == 0) dzext[(i64)t * E1 + (E1 - 1)] = acc * g * (1.f - g);
  }
  for (int s = 0; s < k; s++) {
    const int pos = inv_map[(i64)t * k + s];
    const float w = wts[(i64)t * k + s];
    float acc = 0.f;
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
      const bf16x8_t v = *(const bf16x8_t*)(dr + c), y = *(const bf16x8_t*)(yp + (i64)pos * d + c);
      bf16x8_t o;
#pragma unroll
      for (int q = 0; q < 8; q++) { acc += (float)v[q] * (float)y[q]; o[q] = (__bf16)(w * (float)v[q]); }
      *(bf16x8_t*)(dyp + (i64)pos * d + c) = o;
    }
    acc = block_sum_256(acc, red);
    if (threadIdx.x == 0) dw[(i64)t * k + s] = acc;
  }
}
void launch_moe_bwd_rows(int dt, const void* drs, const void* yp, const void* ys, const int* inv_map,
                         const float* wts, const float* gamma, void* dyp, void* dys, float* dw, float* dzext,
                         int Tn, int d, int k, int E1, int has_gate, hipStream_t s) {
  if (Tn <= 0) return;
  if (vec8_ok(dt, d, {drs, yp, ys, dyp, dys})) {
    hipLaunchKernelGGL(moe_bwd_rows_v8_k, dim3(Tn), dim3(256), 0, s, (const bf16*)drs, (const bf16*)yp, (const bf16*)ys,
                       inv_map, wts, gamma, (bf16*)dyp, (bf16*)dys, dw, dzext, d, k, E1, has_gate);
    return;
  }
  DISPATCH_DT(dt, hipLaunchKernelGGL(moe_bwd_rows_k<T>, dim3(Tn), dim3(256), 0, s, (const T*)drs, (const T*)yp,
                                     (const T*)ys, inv_map, wts, gamma, (T*)dyp, (T*)dys, dw, dzext, d, k, E1,
                                     has_gate));
}

// ---------------------------------------------------------------------------------
// Backward of softmax + top-k weights (the selection itself carries no gradient):
//   dp_sel = dw                      (or (dw - sum dw*w) / sum_sel p with renormalisation)
//   dz_j   = p_j * ([j selected] dp_j - sum_sel dp_e p_e)        for every expert j
// One wave per token, lanes over the experts; writes columns 0..E-1 of dzext[T,E1].
// ---------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) router_bwd_k(const float* __restrict__ probs, const int* __restrict__ idx,
                                                    const float* __restrict__ wts, const float* __restrict__ dw,
                                                    float* __restrict__ dzext, int Tn, int E, int k, int E1,
                                                    int norm_topk, bf16* __restrict__ dzb, int E1p) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= Tn) return;                     // whole wave
  const float* p = probs + (i64)t * E;
  // slot s lives in lane s (k <= 16); sums over the slots run in slot order on every lane
  const int my_sel = lane < k ? idx[(i64)t * k + lane] : -1;
  const float my_dw = lane < k ? dw[(i64)t * k + lane] : 0.f;
  const float my_w = lane < k ? wts[(i64)t * k + lane] : 0.f;
  const float my_p = lane < k ? p[my_sel] : 0.f;
  float ssum = 0.f, dww = 0.f;
  for (int s = 0; s < k; s++) { ssum += __shfl(my_p, s, WAVE); dww += __shfl(my_dw, s, WAVE) * __shfl(my_w, s, WAVE); }
  const float my_dp = norm_topk ? (my_dw - dww) / ssum : my_dw;
  float inner = 0.f;
  for (int s = 0; s < k; s++) inner += __shfl(my_dp, s, WAVE) * __shfl(my_p, s, WAVE);
  for (int j = lane; j < E; j += 64) {
    float dp = 0.f;
    for (int s = 0; s < k; s++) { const int sel = __shfl(my_sel, s, WAVE); const float v = __shfl(my_dp, s, WAVE); if (sel == j) dp = v; }
    const float dz = p[j] * (dp - inner);
    dzext[(i64)t * E1 + j] = dz;
    if (dzb) dzb[(i64)t * E1p + j] = (bf16)dz;
  }
  // the remaining columns of the bf16 copy: the shared-gate column (written to dzext by an earlier kernel), zeros
  if (dzb)
    for (int j = E + lane; j < E1p; j += 64) dzb[(i64)t * E1p + j] = j < E1 ? (bf16)dzext[(i64)t * E1 + j] : (bf16)0.f;
}
void launch_router_bwd(const float* probs, const int* idx, const float* wts, const float* dw, float* dzext, int Tn,
                       int E, int k, int E1, int norm_topk, hipStream_t s, void* dzb, int E1p) {
  if (Tn <= 0) return;
  hipLaunchKernelGGL(router_bwd_k, dim3(cdiv(Tn, 4)), dim3(256), 0, s, probs, idx, wts, dw, dzext, Tn, E, k, E1,
                     norm_topk, (bf16*)dzb, E1p);
}

// ---------------------------------------------------------------------------------
// Gradient at the MoE input Um, all three sources added in a fixed order:
//   dum[t] = dum_sh[t] (shared expert) + sum_slot dxg[pos(t,slot)] (routed experts)
//          + sum_e dzext[t,e] * Wext[e]    (router rows, then the shared gate row)
// ---------------------------------------------------------------------------------
// dum[t] = dum_sh[t] + sum_slot dxg[pos(t,slot)] + router term, where the router term is either the
// precomputed dum_r[t] (bf16 path: a k = E1 GEMM on the matrix cores) or, when dum_r is null, is
// accumulated here from dzext and the router / shared-gate rows.
template <class T>
__global__ void __launch_bounds__(256) dum_finalize_k(const T* __restrict__ dxg, const int* __restrict__ inv_map,
                                                      const T* __restrict__ dum_sh, const T* __restrict__ dum_r,
                                                      const float* __restrict__ dzext,
                                                      const T* __restrict__ w_router, const T* __restrict__ ws_gate,
                                                      T* __restrict__ dum, int d, int k, int E, int E1) {
  extern __shared__ float dzs[];
  const int t = blockIdx.x;
  if (!dum_r) {
    for (int e = threadIdx.x; e < E1; e += 256) dzs[e] = dzext[(i64)t * E1 + e];
    __syncthreads();
  }
  for (int c = threadIdx.x; c < d; c += 256) {
    float acc = dum_sh ? to_f(dum_sh[(i64)t * d + c]) : 0.f;
    for (int s = 0; s < k; s++) acc += to_f(dxg[(i64)inv_map[(i64)t * k + s] * d + c]);
    if (dum_r) {
      acc += to_f(dum_r[(i64)t * d + c]);
    } else {
      for (int e = 0; e < E; e++) acc += dzs[e] * to_f(w_router[(i64)e * d + c]);
      if (E1 > E) acc += dzs[E] * to_f(ws_gate[c]);
    }
    dum[(i64)t * d + c] = from_f<T>(acc);
  }
}
__global__ void __launch_bounds__(256) dum_finalize_v8_k(const bf16* __restrict__ dxg, const int* __restrict__ inv_map,
                                                         const bf16* __restrict__ dum_sh, const bf16* __restrict__ dum_r,
                                                         bf16* __restrict__ dum, int d, int k) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; q++) acc[q] = 0.f;
    if (dum_sh) {
      const bf16x8_t v = *(const bf16x8_t*)(dum_sh + (i64)t * d + c);
#pragma unroll
      for (int q = 0; q < 8; q++) acc[q] = (float)v[q];
    }
    for (int s = 0; s < k; s++) {
      const bf16x8_t v = *(const bf16x8_t*)(dxg + (i64)inv_map[(i64)t * k + s] * d + c);
#pragma unroll
      for (int q = 0; q < 8; q++) acc[q] += (float)v[q];
    }
    const bf16x8_t r = *(const bf16x8_t*)(dum_r + (i64)t * d + c);
    bf16x8_t o;
#pragma unroll
    for (int q = 0; q < 8; q++) o[q] = (__bf16)(acc[q] + (float)r[q]);
    *(bf16x8_t*)(dum + (i64)t * d + c) = o;
  }
}
void launch_dum_finalize(int dt, const void* dxg, const int* inv_map, const void* dum_sh, const void* dum_r,
                         const float* dzext, const void* w_router, const void* ws_gate, void* dum, int Tn, int d,
                         int k, int E, int E1, hipStream_t s) {
  if (Tn <= 0) return;
  if (dum_r && vec8_ok(dt, d, {dxg, dum_sh, dum_r, dum})) {
    hipLaunchKernelGGL(dum_finalize_v8_k, dim3(Tn), dim3(256), 0, s, (const bf16*)dxg, inv_map, (const bf16*)dum_sh,
                       (const bf16*)dum_r, (bf16*)dum, d, k);
    return;
  }
  DISPATCH_DT(dt, hipLaunchKernelGGL(dum_finalize_k<T>, dim3(Tn), dim3(256), E1 * sizeof(float), s, (const T*)dxg,
                                     inv_map, (const T*)dum_sh, (const T*)dum_r, dzext, (const T*)w_router,
                                     (const T*)ws_gate, (T*)dum, d, k, E, E1));
}

