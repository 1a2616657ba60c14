// Internal launcher interface between the C-ABI layer and the HIP kernels.
// dt: 0 = float32, 1 = bfloat16 element type of streams / weights / activations.
#pragma once
#include "common.h"

// One GEMM problem  C[M,N] = epilogue( sum_k A(m,k) * B(k,n) ).
// Operands are row-major matrices RA / RB addressed through a transpose flag:
//   a_trans = 0: A(m,k) = RA[row(m)*lda + k]      a_trans = 1: A(m,k) = RA[row(k)*lda + m]
//   b_trans = 0: B(k,n) = RB[n*ldb + k]  ([out,in] weight)   b_trans = 1: B(k,n) = RB[k*ldb + n]
// row(i) = i, or a_gather[i] / gather_div when a gather list is given (it acts on the RA row index).
// Epilogue:  v = acc + (bias ? bias[n] : 0);
//            (generic kernel only: v *= col_scale[n] first, if col_scale is given)
//            if (tap) tap[m*ldtap+n] = v;
//            if (resid) v = resid[m*ldr+n] + resid_sign * v;      C[m*ldc+n] = v
// Grouping (routed experts):
//   group_mode 1: rows are partitioned by offsets[]; m-tiles come from a device tile
//                 list (tile_group/tile_m0, built for tile height tile_bm); B of group g is
//                 RB + g*b_group_stride.  M is ignored (rows are absolute permuted rows).
//   group_mode 2: the k range of group g is [offsets[g], offsets[g+1]); C of group g is
//                 C + g*c_group_stride (written with zeros when the range is empty).
struct GemmArgs {
  const void* A = nullptr; const void* B = nullptr; void* C = nullptr;
  int M = 0, N = 0, K = 0;
  i64 lda = 0, ldb = 0, ldc = 0;
  int a_trans = 0, b_trans = 0;
  const int* a_gather = nullptr; int gather_div = 1;
  const void* bias = nullptr;
  const void* resid = nullptr; i64 ldr = 0; float resid_sign = 1.f;
  int resid_f32 = 0;                     // resid holds float32 whatever the side type is (fp32 residual streams)
  float* tap = nullptr; i64 ldtap = 0;
  int group_mode = 0; int n_groups = 1; const int* offsets = nullptr;
  const int* tile_group = nullptr; const int* tile_m0 = nullptr; int max_tiles = 0; int tile_bm = 0;
  int no_packed_stores = 0;              // (tuning aid) 2-byte results stored one column per lane even in whole tiles
  int force_tile = 0;                    // MFMA kernel, dense problems: tile shape forced for this launch (unit tests), 0 = by size
  int tile_bn = 0;                       // MFMA expert tiles of height 128: 256 = 128x256 tiles, else 128x128
  i64 b_group_stride = 0, c_group_stride = 0;
  // MFMA kernel, [out,in] weights whose rows are [gate rows | up rows] (N = 2 * act_half): a tile holds matching gate
  // and up columns and also writes act_out[m*ldact + c] = silu(gate) * up, computed from the rounded outputs exactly
  // as the separate SwiGLU kernel does from C.  Ignored by the generic kernel (the caller runs that kernel instead).
  void* act_out = nullptr; i64 ldact = 0; int act_half = 0;
  // generic kernel only: the k range is cut into split_k slices whose fp32 partial tiles go to
  // splitk_ws[slice][M][N]; a second kernel adds the slices in index order and applies the epilogue
  int split_k = 1; float* splitk_ws = nullptr;
  int splitk_raw = 0;                    // generic kernel: leave the slices in splitk_ws, the consumer adds them
  const void* col_scale = nullptr;
  // group_mode 1: number of m-tiles of the list actually in use (device scalar written by the permutation kernel);
  // group_mode 2: the permutation kernel's flag that the routing is even (null: treated as uneven)
  const int* tile_count = nullptr;
  const int* tile_first = nullptr;       // per tile: (first tile of its expert) << 16 | tiles of that expert
  // MFMA kernel, dense problems without split-k: n_sub > 1 launches that many problems of one shape, layout and
  // strides together (grid z = problem); problem z >= 1 takes its operands, result and bias from sub*[z-1]
  int n_sub = 1;
  const void* subA[2] = {nullptr, nullptr}; const void* subB[2] = {nullptr, nullptr};
  void* subC[2] = {nullptr, nullptr}; const void* subBias[2] = {nullptr, nullptr};
  // dense problems: row_skip[m] != 0 marks an output row that is not wanted (a finished part of the fixed-point
  // iteration of the inverse); a workgroup whose rows are all marked exits at once, the others compute every row
  int bulk = 0;                           // 1: not on the caller's critical path (runs beside other kernels): least CU-time wins
  const unsigned char* row_skip = nullptr;
  // set by the MFMA launcher: XCD-aware placement of the tiles (0 = plain 2-D grid), tile counts of the problem
  int xcd_m = 0, tiles_m = 0, tiles_n = 0;
};

// ---- XCD-aware tile placement of the MFMA GEMM (1-D grid of `grid_x` workgroups) ------------------------
// Workgroups go to the 8 XCDs round-robin by linear id and every XCD has an L2 of its own, so workgroup `bid`
// (XCD bid & 7) is handed a tile that shares operands with the other tiles of its XCD:
//   dense (group_mode 0): one rectangle of an xcd_m x (8 / xcd_m) split of the tile grid, walked in bands of
//     8 m-tiles with m fastest, so that the ~64 workgroups an XCD runs together form an 8 x 8 block of tiles;
//   expert tiles (group_mode 1): a consecutive run of the (n-tile, m-tile) pairs of the tile list in use
//     (n_used entries); inside one expert the m-tiles are the fastest index (tile_first[t] = first tile of t's
//     expert << 16 | tiles of that expert), so the workgroups that read one weight tile run next to each other;
//   per-expert weight gradients (group_mode 2): n_used != 0 (the routing is even, see the permutation kernel):
//     xcd_m XCDs share an expert (bz), each taking a band of its column tiles, so that an operand panel is fetched
//     by xcd_m L2s instead of 8; n_used == 0: the plain walk, which spreads every expert over all XCDs (a hot expert
//     must not be left to two of them).
// Returns false for a workgroup that has no tile (it exits at once).  Host and device share this code so that
// the index arithmetic can be checked on the host.
__host__ __device__ inline bool place_tile(int group_mode, int xcd_m, int tiles_m, int tiles_n, int n_groups,
                                           int n_used, const int* tile_first, int bid, int* bx, int* by, int* bz) {
  const int c = bid & 7, loc = bid >> 3;
  if (group_mode == 1) {
    const int total = tiles_n * n_used;
    const int q = total >> 3, r = total & 7;
    if (loc >= q + (c < r ? 1 : 0)) return false;
    const int nl = c * q + (c < r ? c : r) + loc;
    *by = nl / tiles_n; *bx = nl - *by * tiles_n;
    if (tile_first) {
      const int pk = tile_first[*by], f = pk >> 16, cnt = pk & 0xffff;
      const int local = nl - f * tiles_n;
      *bx = local / cnt; *by = f + (local - *bx * cnt);
    }
    return true;
  }
  if (group_mode == 2) {
    if (!n_used) {                        // plain walk: n-tile fastest, then m-tile, then expert
      const int per = tiles_n * tiles_m;
      *bz = bid / per;
      if (*bz >= n_groups) return false;
      const int t = bid - *bz * per;
      *by = t / tiles_n; *bx = t - *by * tiles_n;
      return true;
    }
    // xcd_m XCDs share one expert, each taking a band of its column tiles; 8 / xcd_m experts are in flight at a time
    const int p = xcd_m, G = 8 / p, gi = c / p, mi = c - gi * p;
    const int cn = (tiles_n + p - 1) / p, per = cn * tiles_m;
    const int round = loc / per, t = loc - round * per;
    *bz = round * G + gi;
    if (*bz >= n_groups) return false;
    *by = t / cn; *bx = mi * cn + (t - *by * cn);
    return *bx < tiles_n;
  }
  const int xm = xcd_m, xn = 8 / xm;
  const int sm = (tiles_m + xm - 1) / xm, sn = (tiles_n + xn - 1) / xn;
  const int cm = c / xn, cn = c - cm * xn;
  const int band = loc / (8 * sn), r = loc - band * 8 * sn;
  const int bh = sm - band * 8 < 8 ? sm - band * 8 : 8;
  const int ln = r / bh, lm = band * 8 + (r - ln * bh);
  *by = cm * sm + lm; *bx = cn * sn + ln;
  return *by < tiles_m && *bx < tiles_n;
}
// the split of a dense problem's tiles over the XCDs that touches the fewest operand rows per XCD, and its grid
inline int pick_xcd_m(int tiles_m, int tiles_n, int bm, int bn) {
  long long best = -1; int pick = 1;
  for (int xm = 1; xm <= 8; xm *= 2) {
    long long cost = (long long)((tiles_m + xm - 1) / xm) * bm + (long long)((tiles_n + 8 / xm - 1) / (8 / xm)) * bn;
    if (best < 0 || cost < best) { best = cost; pick = xm; }
  }
  return pick;
}
// workgroups of a per-expert weight-gradient launch: enough for the plain walk and for the paired placement
inline long long wgrad_grid_x(int xcd_m, int tiles_m, int tiles_n, int n_groups) {
  const long long plain = (long long)n_groups * tiles_m * tiles_n;
  const int G = 8 / xcd_m;
  const long long paired = 8LL * ((n_groups + G - 1) / G) * ((tiles_n + xcd_m - 1) / xcd_m) * tiles_m;
  return plain > paired ? plain : paired;
}
inline int dense_grid_x(int xcd_m, int tiles_m, int tiles_n) {
  return 8 * ((tiles_m + xcd_m - 1) / xcd_m) * ((tiles_n + 8 / xcd_m - 1) / (8 / xcd_m));
}

// element types of A, B, C: 0 = f32, 1 = bf16.  bias and resid have C's... no: the
// storage dtype `dt` of the call (bias/resid are streams or weights).
struct GemmTypes { int ta, tb, tc, tside; };

int launch_gemm_generic(const GemmArgs& g, GemmTypes t, hipStream_t s);
// second stage of a split-k GEMM: adds the slices in splitk_ws in index order, applies the epilogue
void launch_splitk_reduce(const GemmArgs& g, GemmTypes t, hipStream_t s);
// bf16 x bf16 MFMA path; returns 1 if the problem does not meet its alignment rules
// (nothing launched), 0 if launched.
int launch_gemm_mfma(const GemmArgs& g, GemmTypes t, hipStream_t s);

// ---- normalisation / element-wise ------------------------------------------------
// tx: element type of x (0 float32, 1 bf16); gains, outputs and gradients have type dt
// row_skip (may be null): rows marked there are left alone (see GemmArgs::row_skip)
// x2 != null: a second problem of the same shape and strides (x2, g2 -> out2) in the same launch
void launch_rmsnorm_fwd(int dt, int tx, const void* x, i64 ldx, const void* g, void* out, i64 ldo,
                        int rows, int h, float eps, hipStream_t s, const unsigned char* row_skip = nullptr,
                        const void* x2 = nullptr, const void* g2 = nullptr, void* out2 = nullptr);
// dx = base + rmsnorm_bwd(dy; x, g);  rinv[rows] receives 1/rms per row (for the gain gradient)
void launch_rmsnorm_bwd(int dt, int tx, const void* dy, i64 ldd, const void* x, i64 ldx, const void* g,
                        const void* base, i64 ldb, void* dx, i64 ldo, float* rinv,
                        int rows, int h, float eps, hipStream_t s);
// out[j] = sum_t a[t*lda+j] * (b ? b[t*ldb+j] : 1) * (sc ? sc[t] : 1); ta/tb/tout element types.
// partial must hold >= colsum_partial_floats(rows, cols) floats.
#define COLSUM_BATCH 3
size_t colsum_partial_floats(int rows, int cols);
// n <= COLSUM_BATCH column sums of one shape and type in one launch pair (b, ldb, sc may be null arrays)
void launch_colsum_batch(int n, int ta, const void* const* a, const i64* lda, int tb, const void* const* b, const i64* ldb,
                         const float* const* sc, int tout, void* const* out, float* partial, int rows, int cols,
                         hipStream_t s);
void launch_colsum(int ta, const void* a, i64 lda, int tb, const void* b, i64 ldb, const float* sc,
                   int tout, void* out, float* partial, int rows, int cols, hipStream_t s);
// rotates buf (and, in the same launch, buf2 of the same shape when it is not null) in place
void launch_rope(int dt, void* buf, const float* cs_table, int T, int S, int H, int dh, float sign,
                 hipStream_t s, void* buf2 = nullptr, const unsigned char* row_skip = nullptr);
void launch_swiglu_fwd(int dt, const void* gu, void* hh, i64 rows, int I, hipStream_t s);
void launch_swiglu_bwd(int dt, const void* dhh, const void* gu, void* dgu, i64 rows, int I, hipStream_t s);
void launch_gather_rows(int dt, const void* src, const int* row_map, int div, void* dst, int rows, int cols,
                        hipStream_t s);
void launch_copy_rows(int dt, const void* src, i64 lds_, void* dst, i64 ldd, int rows, int cols, hipStream_t s);
void launch_copy_rows2(int dt, const void* src_a, i64 lds_a, int rows_a, const void* src_b, i64 lds_b, int rows_b,
                       void* dst, i64 ldd, int cols, hipStream_t s);
void launch_zero(int dt, void* p, int n, hipStream_t s);           // n elements of type dt set to zero
// res[0] = max |a - b| (bitwise max of non-negative floats; res must be zeroed first) ; dst = a
void launch_fill_u32(uint32_t* p, uint32_t v, int n, hipStream_t s);
void launch_absdiff_max_copy(int dt, const void* a, i64 lda, const void* b, i64 ldb, void* dst, i64 ldd,
                             float* res, int rows, int cols, hipStream_t s);
// ---- stopping rule of the fixed-point iteration, decided on the device per block of rows ----------------------
// Block of row t (token b*S + s): bp > 0: (b, s / bp), nj = ceil(S / bp) blocks per sequence; bp == 0: one block.
struct ConvState {
  unsigned char* row_done;    // [T]   1 = the row's block has met the tolerance: later kernels leave it alone
  unsigned char* blk_done;    // [nblk]
  unsigned* blk_bits;         // [nblk] running max |x_n - x_(n-1)| of the current iteration (float bits), 0 between
  int* blk_iters;             // [nblk] iterations the block has run
  float* blk_res;             // [nblk] its last residual
  int* stats;                 // calls, iterations summed (max over blocks per call), last call's iterations, its residual bits
  int S, bp, nj, nblk;
};
// rows not done: res[block] = max(res[block], max |xn - xin|), dst = xn
void launch_conv_update(int dt, const void* xn, i64 ldn, const void* xin, i64 ldi, void* dst, i64 ldd,
                        const ConvState& cs, int rows, int cols, hipStream_t s);
// blocks not done: record iteration `it` and the residual; residual <= tol marks the block and its rows done
void launch_conv_decide(const ConvState& cs, int rows, float tol, int it, hipStream_t s);
// end of one inverse: max over blocks -> residual_out (may be null) and the statistics
void launch_conv_finalize(const ConvState& cs, float* residual_out, hipStream_t s);

// ---- routing ---------------------------------------------------------------------
// zraw[T,E1] = Y1 . (gain * wrp)^T in fp32 (E1 = E (+1: shared gate row)); the kernel scales by 1/rms(Y1)
void launch_router(int dt, const void* y1, i64 ld, const float* zparts, int n_parts, const float* b_router,
                   float* probs, int* idx, float* wts, float* gamma, int T, int h, int E, int k, int has_gate,
                   int norm_topk, float eps, hipStream_t s);
// m-tile lists of the grouped GEMMs for three tile heights: list i covers every expert's rows with
// tiles of bm[i] rows (group[i][t] = expert or -1 for an unused slot, m0[i][t] = first row, first[i][t] = packed
// (first tile of t's expert) * 65536 + (tiles of that expert), count[i] = tiles in use)
// count[0..2]: tiles in use of the three lists; count[3]: 1 if the rows are spread evenly over the experts (place_tile)
struct TileLists { int* group[3]; int* m0[3]; int* first[3]; int max_tiles[3]; int bm[3]; int* count; };
// counts/offsets/row_map/inv_map and the tile lists
void launch_permute(const int* idx, int T, int k, int E, int* counts, int* offsets, int* row_map, int* inv_map,
                    const TileLists& tl, hipStream_t s);
void launch_combine(int dt, const void* yp, const int* inv_map, const float* wts, const void* ys,
                    const float* gamma, void* rs, int T, int d, int k, hipStream_t s);
// half-width combine + coupling update (pre-merged adapters): dst = resid + sign * (sum_slot w * yp[pos] + gamma * ys)
void launch_combine_couple(int dt, int ts, const void* yp, const int* inv_map, const float* wts, const void* ys,
                           const float* gamma, const void* resid, i64 ldr, float sign, void* dst, i64 ldd, float* tap,
                           int T, int h, int k, hipStream_t s);
void launch_moe_bwd_rows(int dt, const void* drs, const void* yp, const void* ys, const int* inv_map,
                         const float* wts, const float* gamma, void* dyp, void* dys, float* dw, float* dzext,
                         int T, int d, int k, int E1, int has_gate, hipStream_t s);
// dzb != null: also writes all E1 columns of dzext as bf16 rows of width E1p (zero padded) for the matrix-core GEMMs
void launch_router_bwd(const float* probs, const int* idx, const float* wts, const float* dw, float* dzext,
                       int T, int E, int k, int E1, int norm_topk, hipStream_t s, void* dzb = nullptr, int E1p = 0);
void launch_dum_finalize(int dt, const void* dxg, const int* inv_map, const void* dum_sh, const void* dum_r,
                         const float* dzext, const void* w_router, const void* ws_gate, void* dum, int T, int d,
                         int k, int E, int E1, hipStream_t s);

// ---- attention -------------------------------------------------------------------
// Q,K,V,O,dO,...: [T, H*dh] token-major, head hh occupies columns hh*dh..; lse/dvec: [B,H,S] float
void launch_attn_fwd_generic(int dt, const void* q, const void* k, const void* v, void* o, float* lse,
                             int B, int S, int H, int dh, int causal, hipStream_t s,
                             const unsigned char* row_skip = nullptr);
void launch_attn_dvec(int dt, const void* o, const void* d_o, float* dvec, int B, int S, int H, int dh,
                      hipStream_t s);
void launch_attn_bwd_generic(int dt, const void* q, const void* k, const void* v, const void* o,
                             const void* d_o, const float* lse, float* dvec, void* dq, void* dk, void* dv,
                             int B, int S, int H, int dh, int causal, hipStream_t s);
// MFMA flash kernels (bf16, dh = 128); return 1 if unsupported shape.
int launch_attn_fwd_flash(const void* q, const void* k, const void* v, void* o, float* lse,
                          int B, int S, int H, int dh, int causal, hipStream_t s,
                          const unsigned char* row_skip = nullptr);
int launch_attn_bwd_flash(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                          const float* lse, float* dvec, void* dq, void* dk, void* dv,
                          int B, int S, int H, int dh, int causal, hipStream_t s);
