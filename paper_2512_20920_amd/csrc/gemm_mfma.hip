// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation) for
// every dense contraction of the block: adapters, Q/K/V/O projections, shared expert,
// grouped routed experts (forward, data gradient, weight gradient).
//
// Workgroup = NW waves laid out WGM x (NW / WGM) over a BM x BN tile, k-step 64 (128 bytes per
// row), NS LDS stages.  Operand tiles go from global memory straight into LDS
// (buffer_load_dwordx4 ... lds: lane l of a wave-load lands at M0 + 16*l), NS-1 k-tiles ahead of
// the one being multiplied, and the loads of the next tile are issued between the MFMA groups of
// the current one, so that the load path and the matrix pipe run together instead of in turns.
// There is no register staging and no LDS store instruction.
//
// Because a wave-load fills 1 KiB of LDS in lane order, bank-conflict-free fragment reads cannot
// come from row padding; each lane instead fetches the 16-byte chunk that belongs in its slot
// under an XOR swizzle:
//  * operand with the contraction index contiguous in memory ("rows x k"): LDS row = 128 bytes =
//    8 chunks, chunk c of row r sits in slot c ^ ((r >> 1) & 7); fragments are 16-byte reads;
//  * operand with the contraction index as the slow one ("k x rows", the transposed layouts of
//    the data- and weight-gradient GEMMs): kept as stored, LDS row k = ROWS*2 bytes, and the
//    64-byte group G of row k sits in group G ^ (k & 3) (ROWS = 64: G ^ ((k >> 1) & 1)); fragments
//    come from the transposing read ds_read_b64_tr_b16, whose lane mapping is: inside each block
//    of 16 lanes, lane j receives element (j & 3) of the 8-byte words addressed by lanes
//    4*e + (j >> 2), e = 0..3.
#include "kernels.h"
#include <stdlib.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Operands are read through raw buffer descriptors with num_records = 2 GiB: a load whose byte
// offset is at or past that returns zeros (into LDS here) without traffic.  Every matrix handed
// to this kernel spans less than 2 GiB from its base (checked on the host), so the offset OOB
// stands for "outside the k range / past the last row" without a branch.
#define BUF_RECORDS 0x80000000u
#define OOB 0x80000000u
#define BK 64

// one wave-load: 64 lanes x 16 bytes from desc + voff (per lane) to LDS at lds_addr + 16 * lane
__device__ __forceinline__ void load_lds_b128(u32x4 desc, unsigned lds_addr, unsigned voff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(desc) : "memory", "m0");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

__device__ __forceinline__ u32x4 make_desc(const void* p) {
  // (operand bases are the same for every lane; saying so keeps the descriptor in scalar registers whatever the
  // compiler can prove about how the base was picked)
  const unsigned long long a = (unsigned long long)p;
  u32x4 d = {(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a),
             (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32)), BUF_RECORDS, 0x00020000u};
  return d;
}

// Where the 16-byte chunk at LDS position `pos` (in chunks, lane order of the wave-loads) of one operand tile
// comes from: byte offset of that chunk at k-tile 0 relative to the operand base, and the number of k-tiles for
// which it lies inside the k range (0 = never: a row past the limit).  krange = elements of the k range.
template <bool TR, int ROWS, int KB = BK>
__device__ __forceinline__ void chunk_source(int pos, int row0, int row_lim, unsigned ld_bytes, int k0, int krange,
                                             const int* gather, int div, unsigned* base, int* ntiles) {
  static_assert(KB == BK || TR, "rows x k tiles are laid out for 128-byte rows");
  if (!TR) {
    const int r = pos >> 3, slot = pos & 7;
    const int c = slot ^ ((r >> 1) & 7);                          // k-chunk of row r that lives in this slot
    int row = row0 + r;
    const bool in = row < row_lim;
    if (!in) row = row_lim - 1;
    const unsigned rr = gather ? (unsigned)(gather[row] / div) : (unsigned)row;
    *base = rr * ld_bytes + (unsigned)(k0 + c * 8) * 2u;
    *ntiles = in ? (krange - c * 8 + BK - 1) / BK : 0;
  } else {
    constexpr int CPR = ROWS / 8;                                 // chunks per LDS row (one k)
    const int kr = pos / CPR, slot = pos % CPR;
    const int gsw = (CPR >= 16) ? (kr & 3) : ((kr >> 1) & 1);
    const int c = (((slot >> 2) ^ gsw) << 2) | (slot & 3);        // 8-element column chunk that lives in this slot
    const int col = row0 + c * 8;
    *base = (unsigned)(k0 + kr) * ld_bytes + (unsigned)col * 2u;
    *ntiles = col < row_lim ? (krange - kr + KB - 1) / KB : 0;
  }
}

// The same for the weight tile of a gate/up GEMM with the SwiGLU epilogue: LDS row r of the tile holds weight row
// (r>>5 & 1) * half + col0 + (r>>6) * 32 + (r & 31), i.e. each wave's 64 rows are 32 gate rows and the 32 up rows of
// the same columns col0 + 32 w .. + 31 (col0 = first gate column of the tile; columns >= half are zeros).
__device__ __forceinline__ void chunk_source_gate_up(int pos, int col0, int half, unsigned ld_bytes, int k0, int krange,
                                                     unsigned* base, int* ntiles) {
  const int r = pos >> 3, slot = pos & 7;
  const int c = slot ^ ((r >> 1) & 7);
  int col = col0 + (r >> 6) * 32 + (r & 31);
  const bool in = col < half;
  if (!in) col = half - 1;
  const unsigned row = (unsigned)(((r >> 5) & 1) * half + col);
  *base = row * ld_bytes + (unsigned)(k0 + c * 8) * 2u;
  *ntiles = in ? (krange - c * 8 + BK - 1) / BK : 0;
}

// Per-lane LDS byte offset (inside the operand's tile, k-step kk = 0) of the MFMA fragment rows r0..r0+31:
// lane (r = lane & 31, g = lane >> 5) holds k = 16*kk + 8*g .. +7 of row r0 + r.
template <bool TR, int ROWS>
__device__ __forceinline__ unsigned frag_base(int r0, int lane) {
  if (!TR) return (unsigned)(r0 + (lane & 31)) * 128u;
  const int blk = lane >> 4, i = lane & 15;
  const int kr = (blk >> 1) * 8 + (i >> 2);
  const int col = r0 + (blk & 1) * 16 + (i & 3) * 4;
  constexpr int CPR = ROWS / 8;
  const int c = col >> 3;
  const int gsw = (CPR >= 16) ? (kr & 3) : ((kr >> 1) & 1);       // unchanged by + 4, + 8, + 16*kk
  const int slot = (((c >> 2) ^ gsw) << 2) | (c & 3);
  return (unsigned)kr * (ROWS * 2u) + (unsigned)slot * 16u + (unsigned)(col & 7) * 2u;
}
template <bool TR, int ROWS>
__device__ __forceinline__ bf16x8 load_frag(const unsigned char* tile, unsigned fb, int r0, int kk, int lane) {
  if (!TR) {
    const int sw = ((r0 + (lane & 31)) >> 1) & 7;
    return *(const bf16x8*)(tile + fb + ((((kk * 2) + (lane >> 5)) ^ sw) << 4));
  } else {
    const unsigned char* p = tile + fb + kk * 16 * (ROWS * 2);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * (ROWS * 2)));
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

// Two neighbouring lanes (columns n, n+1) hold values x0, x1 of rows r, r+1.  After the swap the even lane holds row r
// and the odd lane row r+1, each as (left column, right column): one 4-byte store of two 2-byte results per lane.
// Both lanes of a pair must be active.
__device__ __forceinline__ void pair_rows(bool odd, float x0, float x1, float* left, float* right) {
  const float send = odd ? x0 : x1;
  const float recv = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xf, 0xf, false));
  *left = odd ? recv : x0;
  *right = odd ? x1 : recv;
}

// One output tile; TE = 32-row blocks per wave.
template <int BM, int BN, int WGM, bool AT, bool BT, class TC, int NW, int NS, int TE, int KB = BK>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const bf16* A, const bf16* Bm, TC* C, const void* bias_ptr,
                                          int bx, int bz, int m0, int m_end, int k0, int k_end, int rot_seed) {
  constexpr int WGN = NW / WGM;                      // waves along n
  constexpr int WM = BM / WGM, WN = BN / WGN, TN = WN / 32;
  // KB: elements of k per LDS stage (64; 32 for the per-expert weight gradients, whose k range is a few dozen rows)
  constexpr int STAGE = (BM + BN) * KB * 2;          // bytes of one LDS stage: A tile, then B tile
  constexpr int ALOADS = BM * KB / 512;              // wave-loads (1 KiB) of the A tile
  constexpr int LPW = (BM + BN) * KB / 512 / NW;     // wave-loads per wave per stage
  constexpr int KS = KB / 16;                        // MFMA k-steps per stage
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be made of 32x32 blocks");
  static_assert(((BM + BN) * KB) % (512 * NW) == 0 && (BM * KB) % 512 == 0 && LPW % KS == 0 || KB == BK, "wave-loads must divide evenly");
  static_assert((BM + BN) % (8 * NW) == 0 && BM % 8 == 0, "wave-loads must divide evenly");
  static_assert(KB == BK || (AT && BT), "a shorter k-tile only for operands stored k x rows");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int n0 = bx * BN;
  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wv / WGN) * WM, wn = (wv % WGN) * WN;
  const int krange = k_end - k0;
  const int nk = (krange + KB - 1) / KB;

  // ---- this wave's loads: wave-load j = wv*LPW + i fills LDS chunks [64 j, 64 j + 64) of a stage; the first
  // BM/8 wave-loads are the A tile, the rest the B tile
  const u32x4 da = make_desc(A), db = make_desc(Bm);
  const unsigned lda_b = (unsigned)g.lda * 2u, ldb_b = (unsigned)g.ldb * 2u;
  const unsigned kstep_a = AT ? KB * lda_b : KB * 2u, kstep_b = BT ? KB * ldb_b : KB * 2u;
  unsigned base[LPW];
  int ntile[LPW];
#pragma unroll
  for (int i = 0; i < LPW; i++) {
    const int j = wv * LPW + i;
    if (j < ALOADS) chunk_source<AT, BM, KB>(j * 64 + lane, m0, m_end, lda_b, k0, krange, g.a_gather, g.gather_div, &base[i], &ntile[i]);
    else if (!AT && !BT && TN == 2 && g.act_half)
      chunk_source_gate_up((j - ALOADS) * 64 + lane, bx * (BN / 2), g.act_half, ldb_b, k0, krange, &base[i], &ntile[i]);
    else chunk_source<BT, BN, KB>((j - ALOADS) * 64 + lane, n0, g.N, ldb_b, k0, krange, nullptr, 1, &base[i], &ntile[i]);
  }
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned lw = __builtin_amdgcn_readfirstlane(lds0 + (unsigned)wv * LPW * 1024u);
  // The k-tiles are walked from a start that differs from workgroup to workgroup (and wraps around): workgroups
  // that stream weights from HBM otherwise all ask for the same address bits above the cache-line offset at the
  // same time (every tile row starts a multiple of 4 KiB from its operand's base), which lands on a few memory
  // channels at a time; staggered starts spread the requests over all of them.  The sum over k is the same set of
  // products in a rotated, per-tile fixed order.
  const int rot = __builtin_amdgcn_readfirstlane(nk > 0 ? rot_seed % nk : 0);
  auto issue = [&](int kt, int i) {                  // wave-load i of the kt-th k-tile walked, into stage kt % NS
    const bool isA = (wv * LPW + i) < ALOADS;        // wave-uniform
    const int kr = kt + rot >= nk ? kt + rot - nk : kt + rot;
    const unsigned off = (kt < nk && kr < ntile[i]) ? base[i] + (unsigned)kr * (isA ? kstep_a : kstep_b) : OOB;
    load_lds_b128(isA ? da : db, lw + (unsigned)(kt % NS) * STAGE + i * 1024, off);
  };

  f32x16 acc[TE][TN];
#pragma unroll
  for (int i = 0; i < TE; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;
  unsigned fba[TE], fbb[TN];
#pragma unroll
  for (int i = 0; i < TE; i++) fba[i] = frag_base<AT, BM>(wm + i * 32, lane);
#pragma unroll
  for (int j = 0; j < TN; j++) fbb[j] = BM * KB * 2u + frag_base<BT, BN>(wn + j * 32, lane);

  // ---- pipeline: tiles kt+1 .. kt+NS-1 are in flight while tile kt is multiplied.  A tile past the end of the
  // k range is loaded as zeros (OOB), so every iteration issues the same number of loads and the wait count
  // below is a constant.
#pragma unroll
  for (int p = 0; p < NS - 1; p++)
#pragma unroll
    for (int i = 0; i < LPW; i++) issue(p, i);
  for (int kt = 0; kt < nk; kt++) {
    wait_vmcnt<LPW * (NS - 2)>();                    // this wave's share of tile kt has landed in LDS
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // and its LDS reads of tile kt-1 have returned
    __builtin_amdgcn_s_barrier();                    // ... for every wave: stage (kt-1) % NS may be overwritten
    const unsigned char* st = smem + (kt % NS) * STAGE;
    // fragments of k-step kk+1 are fetched from LDS, and a share of the loads of tile kt+NS-1 issued, while the
    // MFMAs of k-step kk run
    bf16x8 fa[2][TE], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TE; i++) fa[0][i] = load_frag<AT, BM>(st, fba[i], wm + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; j++) fb[0][j] = load_frag<BT, BN>(st, fbb[j], wn + j * 32, 0, lane);
#pragma unroll
    for (int kk = 0; kk < KS; kk++) {
#pragma unroll
      for (int i = kk * LPW / KS; i < (kk + 1) * LPW / KS; i++) issue(kt + NS - 1, i);
      if (kk + 1 < KS) {
#pragma unroll
        for (int i = 0; i < TE; i++) fa[(kk + 1) & 1][i] = load_frag<AT, BM>(st, fba[i], wm + i * 32, kk + 1, lane);
#pragma unroll
        for (int j = 0; j < TN; j++) fb[(kk + 1) & 1][j] = load_frag<BT, BN>(st, fbb[j], wn + j * 32, kk + 1, lane);
      }
#pragma unroll
      for (int i = 0; i < TE; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i], fb[kk & 1][j], acc[i][j], 0, 0, 0);
    }
  }
  wait_vmcnt<0>();                                   // the zero-filled loads past the last tile

  // ---- epilogue: lane holds column n = lane & 31 and rows (e>>2)*8 + (lane>>5)*4 + (e&3)
  if (g.group_mode == 0 && g.split_k > 1) {
    float* ws = g.splitk_ws + (i64)bz * g.M * g.N;
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn + j * 32 + (lane & 31);
      if (n >= g.N) continue;
#pragma unroll
      for (int i = 0; i < TE; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int m = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
          if (m < m_end) ws[(i64)m * g.N + n] = acc[i][j][e];
        }
    }
    return;
  }
  if (g.act_half) {
    // gate/up GEMM with the SwiGLU epilogue: this wave's first 32-column block is gate columns, its second the up
    // columns of the same indices.  Both go to C (the backward pass needs them), and silu(gate) * up, from the
    // rounded values, to act_out.
    if constexpr (!AT && !BT && TN == 2) {
      TC* H = (TC*)g.act_out;
      const int half = g.act_half;
      const int col = bx * (BN / 2) + (wn >> 6) * 32 + (lane & 31);
      if constexpr (sizeof(TC) == 2) {
        // pairs of lanes store two columns of one row each (see the plain store below); rows past the end are masked
        // per lane after the swap, columns per pair (the width is even)
        if (!(g.ldc & 1) && !(g.ldact & 1) && !(half & 1) && !((uintptr_t)C & 3) && !((uintptr_t)H & 3) && !g.no_packed_stores) {
          const bool odd = lane & 1;
          const int colp = col - (odd ? 1 : 0);
          typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_v;
          if (colp < half) {
#pragma unroll
            for (int i = 0; i < TE; i++)
#pragma unroll
              for (int e = 0; e < 16; e += 2) {
                const int m = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3) + (odd ? 1 : 0);
                float gq[2], uq[2], hq[2];
#pragma unroll
                for (int p = 0; p < 2; p++) {
                  const TC gb = (TC)acc[i][0][e + p], ub = (TC)acc[i][1][e + p];
                  gq[p] = (float)gb; uq[p] = (float)ub;
                  hq[p] = (float)(TC)(gq[p] * sigmoid_f(gq[p]) * uq[p]);
                }
                float l, r;
                bf16x2_v wg, wu, wh;
                pair_rows(odd, gq[0], gq[1], &l, &r); wg[0] = (__bf16)l; wg[1] = (__bf16)r;
                pair_rows(odd, uq[0], uq[1], &l, &r); wu[0] = (__bf16)l; wu[1] = (__bf16)r;
                pair_rows(odd, hq[0], hq[1], &l, &r); wh[0] = (__bf16)l; wh[1] = (__bf16)r;
                if (m < m_end) {
                  *(bf16x2_v*)(C + (i64)m * g.ldc + colp) = wg;
                  *(bf16x2_v*)(C + (i64)m * g.ldc + half + colp) = wu;
                  *(bf16x2_v*)(H + (i64)m * g.ldact + colp) = wh;
                }
              }
          }
          return;
        }
      }
      if (col < half) {
#pragma unroll
        for (int i = 0; i < TE; i++)
#pragma unroll
          for (int e = 0; e < 16; e++) {
            const int m = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
            if (m < m_end) {
              const TC gb = (TC)acc[i][0][e], ub = (TC)acc[i][1][e];
              const float gv = (float)gb;
              C[(i64)m * g.ldc + col] = gb;
              C[(i64)m * g.ldc + half + col] = ub;
              H[(i64)m * g.ldact + col] = (TC)(gv * sigmoid_f(gv) * (float)ub);
            }
          }
      }
    }
    return;
  }
  const bf16* bias = (const bf16*)bias_ptr;
  const bf16* resid = (const bf16*)g.resid;
  if (!bias && !g.tap && !resid) {
    // plain store (all weight gradients, most projections): no per-element epilogue work
    // the column blocks of one row are stored back to back, so that the 64-byte pieces of a line reach L2 together.
    // (Staging the tile through LDS to store whole 128-byte lines, 16 bytes per lane, measured no faster: these
    // stores are not what bounds the weight-gradient kernels.)
    const bool full = (m0 + BM <= m_end) && (n0 + BN <= g.N);
    if constexpr (sizeof(TC) == 2) {
      // Whole tiles of 2-byte results: neighbouring lanes hold neighbouring columns of the same rows, so a pair of
      // lanes swaps one value per two rows (the even lane gives its value of the odd row and gets the neighbour's
      // value of the even row) and each lane stores 4 bytes, two columns of one row: half as many store
      // instructions, and the stores of a tile are bound by their number (per-expert weight gradients 10 % faster,
      // 1-2 % of a step).  Going on to a 4x4 transpose inside a quad and 8-byte stores is slower than no packing at
      // all: one instruction then touches eight rows.
      if (full && !(g.ldc & 1) && !((uintptr_t)C & 3) && !g.no_packed_stores) {
        const bool odd = lane & 1;
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_v;
#pragma unroll
        for (int i = 0; i < TE; i++) {
          // even lane: row of element e, its own column; odd lane: the row below, the column to its left
          TC* cp = C + (i64)(m0 + wm + i * 32 + (lane >> 5) * 4 + (odd ? 1 : 0)) * g.ldc + n0 + wn + (lane & 31) - (odd ? 1 : 0);
#pragma unroll
          for (int e = 0; e < 16; e += 2) {
            const int dm = (e >> 2) * 8 + (e & 3);
#pragma unroll
            for (int j = 0; j < TN; j++) {
              float l, r;
              pair_rows(odd, acc[i][j][e], acc[i][j][e + 1], &l, &r);
              bf16x2_v w;
              w[0] = (__bf16)l; w[1] = (__bf16)r;
              *(bf16x2_v*)(cp + (i64)dm * g.ldc + j * 32) = w;
            }
          }
        }
        return;
      }
    }
#pragma unroll
    for (int i = 0; i < TE; i++) {
      TC* cp = C + (i64)(m0 + wm + i * 32 + (lane >> 5) * 4) * g.ldc + n0 + wn + (lane & 31);
#pragma unroll
      for (int e = 0; e < 16; e++) {
        const int dm = (e >> 2) * 8 + (e & 3);
        const bool row_ok = full || (m0 + wm + i * 32 + (lane >> 5) * 4 + dm < m_end);
#pragma unroll
        for (int j = 0; j < TN; j++)
          if (row_ok && (full || n0 + wn + j * 32 + (lane & 31) < g.N)) cp[(i64)dm * g.ldc + j * 32] = (TC)acc[i][j][e];
      }
    }
    return;
  }
  // Two phases per 32-column block: every load (bias, residual) and all arithmetic on loaded values
  // first, then nothing but stores.  On this ISA one counter tracks loads and stores, and where a store may or may
  // not have been issued (rows and columns past the problem's edge are masked per lane) the compiler can only wait
  // for "everything": a use of a loaded value between two stores then waits for the earlier store to complete, and
  // the 16 * TE * TN stores of a lane run one after the other (the coupling GEMMs with a residual operand took
  // twice as long as the same GEMM with a plain store).  So loads are never masked (indices past the edge are
  // clamped to the last valid row / column instead), the finished values are pinned in registers before the first
  // store (the empty asm keeps the compiler from sinking the arithmetic into the masked store blocks), and the
  // store phase has nothing to wait for.  The residual operand may be the output itself (in-place coupling update):
  // it either is C, element for element, or does not overlap it, and each lane reads its elements before it writes.
  constexpr int GI = 1;                              // 32-row blocks whose loads are issued together (more would spill at TE = 2)
  const bool full = (m0 + BM <= m_end) && (n0 + BN <= g.N);
  const int m_last = m_end - 1, n_last = g.N - 1;
  auto row_of = [&](int i, int e) { return m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3); };
#pragma unroll
  for (int j = 0; j < TN; j++) {
    const int n = n0 + wn + j * 32 + (lane & 31);
    const bool n_ok = full || n < g.N;
    const int nn = min(n, n_last);
    const float bv = bias ? (float)bias[nn] : 0.f;
#pragma unroll
    for (int i0 = 0; i0 < TE; i0 += GI) {
      // ---- phase 1: loads and arithmetic
      float rv[GI][16];
      if (resid) {
        if (g.resid_f32) {
#pragma unroll
          for (int ii = 0; ii < GI; ii++)
#pragma unroll
            for (int e = 0; e < 16; e++)
              rv[ii][e] = ((const float*)g.resid)[(i64)min(row_of(i0 + ii, e), m_last) * g.ldr + nn];
        } else {
#pragma unroll
          for (int ii = 0; ii < GI; ii++)
#pragma unroll
            for (int e = 0; e < 16; e++) rv[ii][e] = (float)resid[(i64)min(row_of(i0 + ii, e), m_last) * g.ldr + nn];
        }
      } else {
#pragma unroll
        for (int ii = 0; ii < GI; ii++)
#pragma unroll
          for (int e = 0; e < 16; e++) rv[ii][e] = 0.f;
      }
#pragma unroll
      for (int ii = 0; ii < GI; ii++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          float v = acc[i0 + ii][j][e] + bv;                   // the value the tap records
          float o = resid ? rv[ii][e] + g.resid_sign * v : v;
          asm volatile("" : "+v"(v), "+v"(o));
          acc[i0 + ii][j][e] = v;
          rv[ii][e] = o;
        }
      // ---- phase 2: stores
      if constexpr (sizeof(TC) == 2) {
        // two columns of one row per lane (see the plain store above); the swap runs on every lane, the masks after it
        if (!g.tap && !(g.ldc & 1) && !(g.N & 1) && !((uintptr_t)C & 3) && !g.no_packed_stores) {
          const bool odd = lane & 1;
          typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_v;
#pragma unroll
          for (int ii = 0; ii < GI; ii++)
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
              float l, r;
              pair_rows(odd, rv[ii][e], rv[ii][e + 1], &l, &r);
              bf16x2_v w;
              w[0] = (__bf16)l; w[1] = (__bf16)r;
              const int m = row_of(i0 + ii, e) + (odd ? 1 : 0);
              if (n_ok && (full || m < m_end)) *(bf16x2_v*)(C + (i64)m * g.ldc + n - (odd ? 1 : 0)) = w;
            }
          continue;
        }
      }
#pragma unroll
      for (int ii = 0; ii < GI; ii++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int m = row_of(i0 + ii, e);
          if (n_ok && (full || m < m_end)) {
            if (g.tap) g.tap[(i64)m * g.ldtap + n] = acc[i0 + ii][j][e];
            C[(i64)m * g.ldc + n] = (TC)rv[ii][e];
          }
        }
    }
  }
}

template <int BM, int BN, int WGM, bool AT, bool BT, class TC, int NW, int NS, int KB = BK>
__global__ void __launch_bounds__(NW * 64) gemm_mfma_k(GemmArgs g) {
  constexpr int TM = BM / WGM / 32;
  const bf16* A = (const bf16*)g.A;
  const bf16* Bm = (const bf16*)g.B;
  TC* C = (TC*)g.C;
  const void* bias = g.bias;
  // ---- which tile this workgroup computes (plain 2-D grid, or the XCD-aware placement of a 1-D grid)
  int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  if (g.xcd_m != 0 && !place_tile(g.group_mode, g.xcd_m, g.tiles_m, g.tiles_n, g.n_groups,
                                  g.group_mode == 0 ? 0 : g.tile_count[0], g.tile_first, (int)blockIdx.x, &bx, &by, &bz))
    return;
  int m0, m_end, k0 = 0, k_end = g.K, rot_seed = 0;
  if (g.group_mode == 1) {
    if (!BT) rot_seed = by;     // per row tile (weights with k as the slow index are spread by their column tile already)
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
    } else if (g.n_sub > 1 && bz > 0) {              // one of several problems of one shape launched together
      // (constant indices: the argument block stays in scalar registers)
      if (bz == 1) { A = (const bf16*)g.subA[0]; Bm = (const bf16*)g.subB[0]; C = (TC*)g.subC[0]; bias = g.subBias[0]; }
      else { A = (const bf16*)g.subA[1]; Bm = (const bf16*)g.subB[1]; C = (TC*)g.subC[1]; bias = g.subBias[1]; }
    }
  }
  if (g.row_skip && g.group_mode == 0) {             // nothing to do if every row of the tile is marked as finished
    // every wave looks at all rows of the tile itself and reaches the same answer: no LDS, no barrier (a block-wide
    // vote adds 1 KiB of static LDS in front of the stages, which a tile that uses all 160 KiB for them cannot afford)
    int live = 0;
    for (int r = m0 + (int)(threadIdx.x & 63); r < min(m_end, m0 + BM); r += 64) live |= g.row_skip[r] == 0;
    if (!__any(live)) return;
  }
  gemm_tile<BM, BN, WGM, AT, BT, TC, NW, NS, TM, KB>(g, A, Bm, C, bias, bx, bz, m0, m_end, k0, k_end, rot_seed);
}

// REVFFN_XCD (tuning aid): 0 = plain 2-D grids, tiles land on the XCDs round-robin
static int xcd_enabled() {
  static int v = -1;
  if (v < 0) { const char* e = getenv("REVFFN_XCD"); v = e ? atoi(e) : 1; }
  return v;
}

template <int BM, int BN, int WGM, bool AT, bool BT, class TC, int NW, int NS, int KB = BK>
static void go(const GemmArgs& g0, hipStream_t s) {
  GemmArgs g = g0;
  { static int off = -1; if (off < 0) { const char* e = getenv("REVFFN_NO_PACKED_STORES"); off = e ? atoi(e) : 0; } g.no_packed_stores = off; }
  g.tiles_n = g.act_half ? cdiv(g.act_half, BN / 2) : cdiv(g.N, BN);
  g.tiles_m = g.group_mode == 1 ? g.max_tiles : cdiv(g.M, BM);
  const int zdim = g.group_mode == 2 ? g.n_groups : (g.group_mode == 0 && g.split_k > 1 ? g.split_k : (g.group_mode == 0 ? g.n_sub : 1));
  if (g.tiles_n <= 0 || g.tiles_m <= 0 || zdim <= 0) return;
  dim3 grid(g.tiles_n, g.tiles_m, zdim);
  g.xcd_m = 0;
  if (xcd_enabled()) {
    if (g.group_mode == 1) {
      if (g.tile_count) { g.xcd_m = 1; grid = dim3(g.tiles_n * g.tiles_m, 1, 1); }
    } else if (g.group_mode == 2) {
      // two XCDs per expert while the routing is even (decided on the device, by the permutation kernel): 3.1x fewer
      // operand bytes cross the fabric and these kernels are 6.5 % faster; whole experts per XCD fetch even less
      // but leave XCDs idle, four XCDs per expert split 1408 columns unevenly (both measured slower)
      if (g.tile_count) { g.xcd_m = 2; grid = dim3((unsigned)wgrad_grid_x(2, g.tiles_m, g.tiles_n, g.n_groups), 1, 1); }
    } else if ((i64)g.tiles_n * g.tiles_m >= 64) {
      g.xcd_m = pick_xcd_m(g.tiles_m, g.tiles_n, BM, BN);
      grid = dim3(dense_grid_x(g.xcd_m, g.tiles_m, g.tiles_n), 1, zdim);
    }
  }
  constexpr size_t smem = (size_t)NS * (BM + BN) * KB * 2;
  static_assert(smem <= 160 * 1024, "LDS stages exceed the CU's 160 KiB");
  static std::atomic<unsigned long long> attr_mask{0};
  if (attr_needed(attr_mask)) {
    (void)hipFuncSetAttribute((const void*)gemm_mfma_k<BM, BN, WGM, AT, BT, TC, NW, NS, KB>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_done(attr_mask);
  }
  hipLaunchKernelGGL((gemm_mfma_k<BM, BN, WGM, AT, BT, TC, NW, NS, KB>), grid, dim3(NW * 64), smem, s, g);
}

// The tile shapes: 256x128 and 128x256 (8 waves, one workgroup per CU), 256x256 (2 stages), 128x128 (8 waves of 32x64,
// 4 stages: with one workgroup per CU, two waves per SIMD hide each other's LDS and barrier waits; 10-17 % faster than
// 4 waves of 64x64 on the 2048^3 projections) and 128x64 (8 waves of 32x32, two workgroups per CU; 1.5 % of a step
// over 4 waves of 64x32, measured on one box with both builds).
template <bool AT, bool BT, class TC> static void go_256x128(const GemmArgs& g, hipStream_t s) { go<256, 128, 4, AT, BT, TC, 8, 3>(g, s); }
template <bool AT, bool BT, class TC> static void go_256x256(const GemmArgs& g, hipStream_t s) { go<256, 256, 2, AT, BT, TC, 8, 2>(g, s); }
template <bool AT, bool BT, class TC> static void go_128x128(const GemmArgs& g, hipStream_t s) { go<128, 128, 4, AT, BT, TC, 8, 4>(g, s); }
template <bool AT, bool BT, class TC> static void go_128x256(const GemmArgs& g, hipStream_t s) { go<128, 256, 2, AT, BT, TC, 8, 3>(g, s); }
template <bool AT, bool BT, class TC> static void go_128x64(const GemmArgs& g, hipStream_t s) { go<128, 64, 4, AT, BT, TC, 8, 3>(g, s); }
// 160x256 for the routed experts' forward GEMMs where one 160-row tile holds a typical expert: 4 waves side by side,
// each 160 rows x 64 columns (a gate and an up block for the SwiGLU epilogue), one wave per SIMD, 3 stages of 52 KiB
template <bool AT, bool BT, class TC> static void go_160x256(const GemmArgs& g, hipStream_t s) { go<160, 256, 1, AT, BT, TC, 4, 3>(g, s); }

template <bool AT, bool BT, class TC>
static void pick_tile(const GemmArgs& g, hipStream_t s) {
  // Dense problems: the tile whose rounds of workgroups over the 256 CUs cost least.  One tile of 256x128 takes about
  // 1.72 times, one of 256x256 about 3.05 times as long as one of 128x128 (measured on this block's shapes at 1024 to
  // 8192 tokens: larger tiles do more work per loaded byte, but a last, partly filled round costs a whole tile's time).
  auto dense_choice = [&]() {
    const int z = g.split_k > 1 ? g.split_k : g.n_sub;
    // (a launch that runs beside others on a helper stream fills only the CUs it needs: its cost is its tile count.
    // Not for a problem of fewer than 128 of the largest tiles: on a fraction of the CUs it takes several times as
    // long, and helper streams are chains too -- 32-tile weight gradients at the end of a call were the last thing
    // running, on an eighth of the chip.)
    const bool bulk = g.bulk && (i64)cdiv(g.M, 256) * cdiv(g.N, 256) * z >= 128;
    auto rounds = [&](int bm, int bn) {
      const i64 tiles = (i64)cdiv(g.M, bm) * cdiv(g.N, bn) * z;
      return bulk ? (double)tiles / 256.0 : (double)cdiv(tiles, 256);
    };
    const double c2 = rounds(128, 128), c3 = 1.72 * rounds(256, 128), c4 = 3.05 * rounds(256, 256);
    return (c4 < c3 && c4 < c2) ? 4 : (c3 < c2 ? 3 : 2);
  };
  if (g.act_half && g.group_mode == 0) {
    // SwiGLU epilogue: only tiles whose waves are 64 columns wide (a gate and an up block)
    switch (g.force_tile >= 2 ? g.force_tile : dense_choice()) {
      case 4: go_256x256<AT, BT, TC>(g, s); break;
      case 3: go_256x128<AT, BT, TC>(g, s); break;
      default: go_128x128<AT, BT, TC>(g, s);
    }
    return;
  }
  if (g.group_mode != 1 && g.force_tile) {           // a unit test asks for one of the shapes (dense problems)
    switch (g.force_tile) {
      case 1: go_128x64<AT, BT, TC>(g, s); return;
      case 2: go_128x128<AT, BT, TC>(g, s); return;
      case 3: go_256x128<AT, BT, TC>(g, s); return;
      case 4:
        if constexpr (AT && BT) go<256, 256, 2, AT, BT, TC, 8, 4, 32>(g, s);
        else go_256x256<AT, BT, TC>(g, s);
        return;
    }
  }
  if (g.group_mode == 1) {
    // expert tiles.  Skipping the MFMAs of the 32-row blocks past an expert's end (waves spanning all rows, a loop
    // specialised per block count) measured no gain, and neither did a fifth LDS stage.
    if constexpr (!AT) {
      if constexpr (!BT) { if (g.tile_bm == 160) { go_160x256<AT, BT, TC>(g, s); return; } }
      if (g.tile_bm == 256) go_256x128<AT, BT, TC>(g, s);
      else if (g.tile_bn == 256) go_128x256<AT, BT, TC>(g, s);
      else go_128x128<AT, BT, TC>(g, s);
    }
    return;
  }
  if (g.group_mode == 2) {
    // per-expert weight gradients: the k range is one expert's rows, a few k-tiles only, so a workgroup is mostly
    // fixed cost (start-up, first load latency) and output stores, none of which overlap on a CU that holds one
    // workgroup.  The largest tile, 256x256 (2 stages), spreads the fixed cost over the most output: 12 % faster than
    // 256x128 on these kernels and 1-1.6 % of a step, even where the last tile column is half empty (N = 1408).
    // Smaller tiles with two workgroups per CU (128x128 with 2 stages, 4 or 8 waves) were up to 7 % faster than
    // 256x128 alone but slower inside the step, next to the data-gradient chain on the main stream; a persistent
    // form of 256x128 (a workgroup walks over tiles and issues the next tile's first loads before it stores the
    // finished one) was 5 % faster alone and 3 % of a step slower.
    // With k-tiles of 32 rows (4 stages of 32 KiB) an expert of 137 rows is 5 k-tiles instead of 3 of 64 (17 % fewer
    // multiplied zero rows), and all but the last are in flight at once: these kernels 10 % faster, a step 1.1 %.
    // (5 stages: 8 % slower again; 3: the same.)
    if constexpr (AT && BT) { go<256, 256, 2, AT, BT, TC, 8, 4, 32>(g, s); return; }
    return;                                            // (launch_gemm_mfma admits this mode for that layout only)
  }
  // below ~200 tiles of 128x128: 128x64 (two workgroups per CU)
  const i64 t128 = (i64)cdiv(g.M, 128) * cdiv(g.N, 128) * (g.split_k > 1 ? g.split_k : g.n_sub);
  if (t128 < 200 && g.N >= 128) { go_128x64<AT, BT, TC>(g, s); return; }
  switch (dense_choice()) {
    case 4:
      // (weight gradients: four stages of 32 rows of k instead of two of 64 keep more loads in flight; 0.5-1.2 % of a
      // step on the skewed and long-sequence workloads)
      if constexpr (AT && BT) go<256, 256, 2, AT, BT, TC, 8, 4, 32>(g, s);
      else go_256x256<AT, BT, TC>(g, s);
      break;
    case 3:
      // (the same tile count either way; with k contiguous in both operands the wide tile measured 1-4 % faster)
      if (!AT && !BT && g.N % 256 == 0) go_128x256<AT, BT, TC>(g, s);
      else go_256x128<AT, BT, TC>(g, s);
      break;
    default: go_128x128<AT, BT, TC>(g, s);
  }
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
  if (g.group_mode == 1 && (g.a_trans || (g.tile_bm != 128 && g.tile_bm != 256 && !(g.tile_bm == 160 && !g.b_trans && g.tile_bn == 256)))) return 1;
  if (g.a_gather && g.a_trans) return 1;
  if (g.group_mode != 1 && g.M <= 0) return 1;
  if (g.split_k > 1 && (g.group_mode != 0 || !g.splitk_ws)) return 1;
  if (g.n_sub < 1 || g.n_sub > 3 || (g.n_sub > 1 && (g.group_mode != 0 || g.split_k > 1 || g.resid || g.tap || g.act_half))) return 1;
  for (int z = 1; z < g.n_sub; z++)
    if (!g.subA[z - 1] || !g.subB[z - 1] || !g.subC[z - 1] || !aligned16(g.subA[z - 1]) || !aligned16(g.subB[z - 1])) return 1;
  if (g.col_scale && g.split_k <= 1) return 1;           // column scale lives in the split-k reduction only
  if (g.act_half) {
    if (g.a_trans || g.b_trans || g.group_mode == 2 || g.split_k > 1 || g.bias || g.resid || g.tap || !g.act_out) return 1;
    if (g.N != 2 * g.act_half) return 1;
  }
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
