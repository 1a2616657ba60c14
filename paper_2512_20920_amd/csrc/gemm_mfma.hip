// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation) for
// every dense contraction of the block: adapters, Q/K/V/O projections, shared expert,
// grouped routed experts (forward, data gradient, weight gradient).
//
// Workgroup = 256 threads = 4 waves (2x2); workgroup tile BM x BN, k-step 64, two LDS
// stages.  Operand tiles are staged global -> registers -> LDS while the previous stage
// is multiplied.  An operand whose contraction index is contiguous in memory is read from
// LDS with 16-byte reads; an operand whose contraction index is the slow one (the
// "transposed" layouts of the data- and weight-gradient GEMMs) is kept as stored and read
// with the transposing LDS read ds_read_b64_tr_b16, whose lane mapping is: inside each
// block of 16 lanes, lane j receives element (j & 3) of the 8-byte words addressed by
// lanes 4*e + (j >> 2), e = 0..3.
#include "kernels.h"
#include <stdlib.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;


// LDS tile of one operand.  TR = 0: [ROWS][BK] with row stride BK+8 elements (144 B: the 16
// rows read together by a 16-byte fragment read start on distinct 16-byte bank groups).
// TR = 1: [BK][ROWS] with row stride ROWS+32 elements (the 4 k-rows x 64 B read together by a
// transposing read fall on disjoint banks).
template <bool TR, int ROWS, int BK, int NT>
struct Tile {
  static constexpr int stride = TR ? ROWS + 32 : BK + 8;
  static constexpr int elems = TR ? BK * stride : ROWS * stride;
  static constexpr int chunks = ROWS * (BK / 8) / NT;   // 16-byte chunks per thread per k-step
};

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Operands are read through raw buffer descriptors: a load whose byte offset is at or past
// num_records returns zeros.  Every matrix handed to this kernel spans less than 2 GiB from
// its base (checked on the host), so num_records = 2 GiB and the offset OOB below stand for
// "this chunk lies outside the k range / past the last row: give me zeros" without a branch,
// which keeps the loads of several k-tiles in flight together.
#define BUF_RECORDS 0x80000000u
#define OOB 0x80000000u

struct OperandSrc {
  __amdgpu_buffer_rsrc_t rsrc;   // matrix base (already offset by group)
  unsigned ld_bytes;             // row stride in bytes
  const int* gather;             // row indirection (non-transposed A only) or nullptr
  int div;
  int row0;                      // first tile row (m0 or n0) in the non-contraction index
  int row_lim;                   // exclusive bound of valid rows
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, BUF_RECORDS, 0x00020000);
}

// ---- global -> registers ----------------------------------------------------------
template <bool TR, int ROWS, int BK, int NT>
__device__ __forceinline__ void load_tile(const OperandSrc& s, int k0, int k_end,
                                          uint4 (&regs)[Tile<TR, ROWS, BK, NT>::chunks],
                                          const unsigned (&rowoff)[Tile<TR, ROWS, BK, NT>::chunks]) {
  constexpr int NC = Tile<TR, ROWS, BK, NT>::chunks;
#pragma unroll
  for (int i = 0; i < NC; i++) {
    int c = threadIdx.x + NT * i;
    unsigned off;
    if (!TR) {
      int k = k0 + (c % (BK / 8)) * 8;
      off = (k < k_end) ? rowoff[i] + (unsigned)k * 2u : OOB;
    } else {
      int k = k0 + c / (ROWS / 8);
      int m = s.row0 + (c % (ROWS / 8)) * 8;
      off = (k < k_end && m < s.row_lim) ? (unsigned)k * s.ld_bytes + (unsigned)m * 2u : OOB;
    }
    u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(s.rsrc, off, 0, 0);
    regs[i] = make_uint4(v[0], v[1], v[2], v[3]);
  }
}

// per-thread row byte offsets of the non-transposed operand (fixed over the k loop); rows past
// the limit are clamped to the last valid row (their products are never stored)
template <int ROWS, int BK, int NT>
__device__ __forceinline__ void row_offsets(const OperandSrc& s, unsigned (&rowoff)[ROWS * (BK / 8) / NT]) {
#pragma unroll
  for (int i = 0; i < ROWS * (BK / 8) / NT; i++) {
    int c = threadIdx.x + NT * i;
    int r = s.row0 + c / (BK / 8);
    const bool in = r < s.row_lim;
    if (!in) r = s.row_lim - 1;
    unsigned rr = s.gather ? (unsigned)(s.gather[r] / s.div) : (unsigned)r;
    rowoff[i] = in ? rr * s.ld_bytes : OOB;            // rows past the limit read as zeros, without traffic
  }
}

// ---- registers -> LDS -------------------------------------------------------------
template <bool TR, int ROWS, int BK, int NT>
__device__ __forceinline__ void store_tile(bf16* lds, const uint4 (&regs)[Tile<TR, ROWS, BK, NT>::chunks]) {
  constexpr int NC = Tile<TR, ROWS, BK, NT>::chunks;
  constexpr int ST = Tile<TR, ROWS, BK, NT>::stride;
#pragma unroll
  for (int i = 0; i < NC; i++) {
    int c = threadIdx.x + NT * i;
    int off;
    if (!TR) off = (c / (BK / 8)) * ST + (c % (BK / 8)) * 8;
    else off = (c / (ROWS / 8)) * ST + (c % (ROWS / 8)) * 8;
    *(uint4*)(lds + off) = regs[i];
  }
}

// ---- LDS -> MFMA operand fragment: 32 rows x 16 k, lane (r = lane & 31, g = lane >> 5)
// holds k = 8g..8g+7 of row r ---------------------------------------------------------
template <bool TR, int ROWS, int BK>
__device__ __forceinline__ bf16x8 load_frag(const bf16* lds, int r0, int kk, int lane) {
  constexpr int ST = Tile<TR, ROWS, BK, 256>::stride;
  if (!TR) {
    return *(const bf16x8*)(lds + (r0 + (lane & 31)) * ST + kk * 16 + (lane >> 5) * 8);
  } else {
    int blk = lane >> 4, i = lane & 15;
    int krow = kk * 16 + (blk >> 1) * 8 + (i >> 2);
    int mcol = r0 + (blk & 1) * 16 + (i & 3) * 4;
    const bf16* p = lds + krow * ST + mcol;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * ST));
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

// PD = number of k-tiles kept in flight in registers ahead of the one being multiplied
#define PD 3
template <int BM, int BN, int BK, int WGM, bool AT, bool BT, class TC, bool RB, int NW>
__global__ void __launch_bounds__(NW * 64, BK == 32 ? 3 : 1) gemm_mfma_k(GemmArgs g) {
  constexpr int NT = NW * 64;                       // threads per workgroup
  typedef Tile<AT, BM, BK, NT> TA_;
  typedef Tile<BT, BN, BK, NT> TB_;
  constexpr int WGN = NW / WGM;                      // waves along n
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be made of 32x32 blocks");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* sA = (bf16*)smem_raw;                       // 2 stages of A then 2 stages of B
  bf16* sB = sA + 2 * TA_::elems;

  const bf16* A = (const bf16*)g.A;
  const bf16* Bm = (const bf16*)g.B;
  TC* C = (TC*)g.C;
  // ---- which tile this workgroup computes (plain 2-D grid, or the XCD-aware placement of a 1-D grid)
  int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  if (g.xcd_m != 0 && !place_tile(g.group_mode, g.xcd_m, g.tiles_m, g.tiles_n, g.n_groups,
                                  g.group_mode == 1 ? g.tile_count[0] : 0, g.tile_first, (int)blockIdx.x, &bx, &by, &bz))
    return;
  int m0, m_end, k0 = 0, k_end = g.K;
  if (g.group_mode == 1) {
    int ti = by;
    int grp = g.tile_group[ti];
    if (grp < 0) return;
    m0 = g.tile_m0[ti];
    m_end = min(g.offsets[grp + 1], m0 + BM);
    Bm += (i64)grp * g.b_group_stride;
  } else {
    m0 = by * BM;
    m_end = g.M;
    if (g.group_mode == 2) {
      int grp = bz;
      k0 = g.offsets[grp];
      k_end = g.offsets[grp + 1];
      C += (i64)grp * g.c_group_stride;
    } else if (g.split_k > 1) {                      // k slices of whole k-tiles; partial sums go to splitk_ws
      int per = ((g.K + BK - 1) / BK + g.split_k - 1) / g.split_k * BK;
      k0 = min(g.K, bz * per);
      k_end = min(g.K, k0 + per);
    }
  }
  const int n0 = bx * BN;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int wm = (wv / WGN) * WM, wn = (wv % WGN) * WN;

  OperandSrc sa{make_rsrc(A), (unsigned)g.lda * 2u, g.a_gather, g.gather_div, m0, m_end};
  OperandSrc sb{make_rsrc(Bm), (unsigned)g.ldb * 2u, nullptr, 1, n0, g.N};
  unsigned offA[TA_::chunks], offB[TB_::chunks];
  if (!AT) row_offsets<BM, BK, NT>(sa, offA);
  if (!BT) row_offsets<BN, BK, NT>(sb, offB);

  // 32-row blocks of this wave's tile that hold at least one valid row (partial expert tiles)
  const int tm_eff = RB ? min(TM, max(0, (m_end - m0 - wm + 31) / 32)) : TM;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  // Software pipeline: register set u holds k-tile kt+PD while tile kt is multiplied from LDS and
  // tile kt+1 moves from its register set into the other LDS stage.  Loads and LDS stores are
  // unconditional (a tile past the end of the k range reads as zeros through the OOB offset), so
  // the loop body is straight-line code and the compiler can keep 2*PD-1 tile loads outstanding;
  // only the multiply is skipped for the padding tiles.
  uint4 ra[PD][TA_::chunks], rb[PD][TB_::chunks];
  const int nk = (k_end - k0 + BK - 1) / BK;
#pragma unroll
  for (int p = 0; p < PD; p++) {
    load_tile<AT, BM, BK, NT>(sa, k0 + p * BK, k_end, ra[p], offA);
    load_tile<BT, BN, BK, NT>(sb, k0 + p * BK, k_end, rb[p], offB);
  }
  store_tile<AT, BM, BK, NT>(sA, ra[0]);
  store_tile<BT, BN, BK, NT>(sB, rb[0]);
  __syncthreads();
  for (int kt0 = 0; kt0 < nk; kt0 += PD) {
#pragma unroll
    for (int u = 0; u < PD; u++) {
      const int kt = kt0 + u;
      const int cur = kt & 1;
      load_tile<AT, BM, BK, NT>(sa, k0 + (kt + PD) * BK, k_end, ra[u], offA);
      load_tile<BT, BN, BK, NT>(sb, k0 + (kt + PD) * BK, k_end, rb[u], offB);
      if (kt < nk) {                                  // uniform over the workgroup
        const bf16* cA = sA + cur * TA_::elems;
        const bf16* cB = sB + cur * TB_::elems;
        // fragments of k-step kk+1 are fetched from LDS while the MFMAs of k-step kk issue
        bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
        for (int i = 0; i < TM; i++)
          if (!RB || i < tm_eff) fa[0][i] = load_frag<AT, BM, BK>(cA, wm + i * 32, 0, lane);
#pragma unroll
        for (int j = 0; j < TN; j++) fb[0][j] = load_frag<BT, BN, BK>(cB, wn + j * 32, 0, lane);
#pragma unroll
        for (int kk = 0; kk < BK / 16; kk++) {
          if (kk + 1 < BK / 16) {
#pragma unroll
            for (int i = 0; i < TM; i++)
              if (!RB || i < tm_eff) fa[(kk + 1) & 1][i] = load_frag<AT, BM, BK>(cA, wm + i * 32, kk + 1, lane);
#pragma unroll
            for (int j = 0; j < TN; j++) fb[(kk + 1) & 1][j] = load_frag<BT, BN, BK>(cB, wn + j * 32, kk + 1, lane);
          }
#pragma unroll
          for (int i = 0; i < TM; i++)
            if (!RB || i < tm_eff) {
#pragma unroll
              for (int j = 0; j < TN; j++)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i], fb[kk & 1][j], acc[i][j], 0, 0, 0);
            }
        }
      }
      store_tile<AT, BM, BK, NT>(sA + (cur ^ 1) * TA_::elems, ra[(u + 1) % PD]);   // tile kt+1
      store_tile<BT, BN, BK, NT>(sB + (cur ^ 1) * TB_::elems, rb[(u + 1) % PD]);
      __syncthreads();
    }
  }

  // ---- epilogue: lane holds column n = lane & 31 and rows (e>>2)*8 + (lane>>5)*4 + (e&3)
  if (g.group_mode == 0 && g.split_k > 1) {
    float* ws = g.splitk_ws + (i64)bz * g.M * g.N;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn + j * 32 + (lane & 31);
      if (n >= g.N) continue;
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int m = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
          if (m < m_end) ws[(i64)m * g.N + n] = acc[i][j][e];
        }
    }
    return;
  }
  const bf16* bias = (const bf16*)g.bias;
  const bf16* resid = (const bf16*)g.resid;
  if (!g.row_scale && !bias && !g.tap && !resid) {
    // plain store (all weight gradients, most projections): no per-element epilogue work
    const bool full = (m0 + BM <= m_end) && (n0 + BN <= g.N);
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
      for (int i = 0; i < TM; i++) {
        TC* cp = C + (i64)(m0 + wm + i * 32 + (lane >> 5) * 4) * g.ldc + n;
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int dm = (e >> 2) * 8 + (e & 3);
          if (full || (n < g.N && m0 + wm + i * 32 + (lane >> 5) * 4 + dm < m_end)) cp[(i64)dm * g.ldc] = (TC)acc[i][j][e];
        }
      }
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int n = n0 + wn + j * 32 + (lane & 31);
    if (n >= g.N) continue;
    const float bv = bias ? (float)bias[n] : 0.f;
#pragma unroll
    for (int i = 0; i < TM; i++) {
#pragma unroll
      for (int e = 0; e < 16; e++) {
        const int m = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (m >= m_end) continue;
        float v = acc[i][j][e];
        if (g.row_scale) v *= g.row_scale[m];
        v += bv;
        if (g.tap) g.tap[(i64)m * g.ldtap + n] = v;
        if (resid) v = (float)resid[(i64)m * g.ldr + n] + g.resid_sign * v;
        C[(i64)m * g.ldc + n] = (TC)v;
      }
    }
  }
}

// REVFFN_XCD (tuning aid): 0 = plain 2-D grids, tiles land on the XCDs round-robin
static int xcd_enabled() {
  static int v = -1;
  if (v < 0) { const char* e = getenv("REVFFN_XCD"); v = e ? atoi(e) : 1; }
  return v;
}

template <int BM, int BN, int BK, int WGM, bool AT, bool BT, class TC, bool RB = false, int NW = 4>
static void go(const GemmArgs& g0, hipStream_t s) {
  GemmArgs g = g0;
  g.tiles_n = cdiv(g.N, BN);
  g.tiles_m = g.group_mode == 1 ? g.max_tiles : cdiv(g.M, BM);
  const int zdim = g.group_mode == 2 ? g.n_groups : (g.group_mode == 0 && g.split_k > 1 ? g.split_k : 1);
  if (g.tiles_n <= 0 || g.tiles_m <= 0 || zdim <= 0) return;
  dim3 grid(g.tiles_n, g.tiles_m, zdim);
  g.xcd_m = 0;
  if (xcd_enabled()) {
    if (g.group_mode == 1) {
      if (g.tile_count) { g.xcd_m = 1; grid = dim3(g.tiles_n * g.tiles_m, 1, 1); }
    } else if (g.group_mode == 2) {
      // whole experts per XCD: less traffic, but uneven expert sizes then leave XCDs idle (measured slower
      // under a skewed routing, equal under a balanced one), so only on request (REVFFN_XCD=2)
      if (xcd_enabled() == 2) { g.xcd_m = 1; grid = dim3(8 * cdiv(g.n_groups, 8) * g.tiles_n * g.tiles_m, 1, 1); }
    } else if ((i64)g.tiles_n * g.tiles_m >= 64) {
      g.xcd_m = pick_xcd_m(g.tiles_m, g.tiles_n, BM, BN);
      grid = dim3(dense_grid_x(g.xcd_m, g.tiles_m, g.tiles_n), 1, zdim);
    }
  }
  size_t smem = (size_t)2 * (Tile<AT, BM, BK, NW * 64>::elems + Tile<BT, BN, BK, NW * 64>::elems) * sizeof(bf16);
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)gemm_mfma_k<BM, BN, BK, WGM, AT, BT, TC, RB, NW>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_mfma_k<BM, BN, BK, WGM, AT, BT, TC, RB, NW>), grid, dim3(NW * 64), smem, s, g);
}

// REVFFN_GEMM_TILE (tuning aid): 1 = 128x128, 2 = 128x64, 3 = 64x128 for every non-grouped problem
static int tile_override() {
  static int v = -1;
  if (v < 0) { const char* e = getenv("REVFFN_GEMM_TILE"); v = e ? atoi(e) : 0; }
  return v;
}

template <bool AT, bool BT, class TC>
static void pick_tile(const GemmArgs& g, hipStream_t s) {
  if (g.group_mode != 1 && tile_override()) {
    switch (tile_override()) {
      case 1: go<128, 128, 64, 2, AT, BT, TC>(g, s); return;
      case 2: go<128, 64, 64, 2, AT, BT, TC>(g, s); return;
      case 3: go<64, 128, 64, 1, AT, BT, TC>(g, s); return;
      case 4: go<128, 128, 32, 2, AT, BT, TC>(g, s); return;
    }
  }
  if (g.group_mode == 1) {
    // expert tiles.  Variant 1 (waves split the weight columns and skip the 32-row blocks a short expert
    // does not fill) measured slightly slower than the plain 2x2 wave layout at ~137 rows per expert
    static int v = -1;                 // REVFFN_GROUPED_VARIANT (tuning aid): 0 = 2x2 waves, 1 = 1x4 waves + skipping
    if (v < 0) { const char* e = getenv("REVFFN_GROUPED_VARIANT"); v = e ? atoi(e) : 0; }
    if (g.tile_bm == 64) go<64, 128, 64, 1, AT, BT, TC>(g, s);
    else if (v == 0) go<128, 128, 64, 2, AT, BT, TC>(g, s);
    else go<128, 128, 64, 1, AT, BT, TC, true>(g, s);
    return;
  }
  if (g.group_mode == 2) {
    // per-expert weight gradients: the k range is one expert's rows; short ranges take the k-step 32 kernel
    // (less padding, smaller LDS footprint, more workgroups per CU to hide the load latency)
    static int v = -1;                 // REVFFN_WGRAD_BK32 (tuning aid)
    if (v < 0) { const char* e = getenv("REVFFN_WGRAD_BK32"); v = e ? atoi(e) : 1; }
    if (v && g.K < (i64)192 * g.n_groups) go<128, 128, 32, 2, AT, BT, TC>(g, s); else go<128, 128, 64, 2, AT, BT, TC>(g, s);
    return;
  }
  // small problems: narrower tiles so that every CU gets at least two workgroups
  i64 tiles = (i64)cdiv(g.M, 128) * cdiv(g.N, 128);
  if (tiles < 512 && g.N >= 128) go<128, 64, 64, 2, AT, BT, TC>(g, s);
  else go<128, 128, 64, 2, AT, BT, TC>(g, s);
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

int launch_gemm_mfma(const GemmArgs& g, GemmTypes t, hipStream_t s) {
  if (t.ta != 1 || t.tb != 1 || t.tside != 1) return 1;
  if (!aligned16(g.A) || !aligned16(g.B) || (g.lda & 7) || (g.ldb & 7)) return 1;
  if ((g.b_group_stride & 7) || (g.c_group_stride & 7)) return 1;
  if (!g.a_trans && (g.K & 7)) return 1;
  if (!g.b_trans && (g.K & 7)) return 1;
  if (g.a_trans && (g.M & 7)) return 1;
  if (g.b_trans && (g.N & 7)) return 1;
  if (g.a_trans && !g.b_trans) return 1;                 // layout not used by the block
  if (g.group_mode == 2 && !(g.a_trans && g.b_trans)) return 1;
  if (g.group_mode == 1 && (g.a_trans || (g.tile_bm != 128 && g.tile_bm != 64))) return 1;
  if (g.a_gather && g.a_trans) return 1;
  if (g.b_gather) return 1;                              // gather along k is not taken: materialise the rows
  if (g.group_mode != 1 && g.M <= 0) return 1;
  if (g.split_k > 1 && (g.group_mode != 0 || !g.splitk_ws)) return 1;
  if (g.col_scale && g.split_k <= 1) return 1;           // column scale lives in the split-k reduction only
  // every operand must span less than 2 GiB from its base (32-bit buffer offsets)
  {
    const i64 lim = (i64)1 << 30;                        // elements
    i64 a_rows = g.a_trans ? g.K : g.M, b_rows = g.b_trans ? g.K : g.N;
    if (a_rows * g.lda >= lim || b_rows * g.ldb >= lim) return 1;
  }
  const bool f32out = t.tc == 0;
  if (!g.a_trans && !g.b_trans) {
    if (f32out) pick_tile<false, false, float>(g, s); else pick_tile<false, false, bf16>(g, s);
  } else if (!g.a_trans && g.b_trans) {
    if (f32out) pick_tile<false, true, float>(g, s); else pick_tile<false, true, bf16>(g, s);
  } else {
    if (f32out) pick_tile<true, true, float>(g, s); else pick_tile<true, true, bf16>(g, s);
  }
  if (g.group_mode == 0 && g.split_k > 1) launch_splitk_reduce(g, t, s);
  return 0;
}
