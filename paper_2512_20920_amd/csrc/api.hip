// C ABI of the RevFFN block: argument validation, workspace, and the sequence of kernel
// launches for forward (Eq. 1-2), inverse (the display under them) and backward.
// No device synchronisation and no allocation happens outside create/destroy.
#include "../../include/revffn.h"
#include "kernels.h"

#include <math.h>
#include <mutex>
#include <new>
#include <stdlib.h>
#include <string.h>
#include <vector>

namespace {

struct Carver {            // hands out 256-byte aligned slices of one allocation (or just counts)
  char* base = nullptr;
  size_t off = 0;
  void* take(size_t bytes) {
    size_t a = (off + 255) & ~(size_t)255;
    off = a + bytes;
    return base ? (void*)(base + a) : nullptr;
  }
};

}  // namespace

// Kernel families of the per-launch timing.  The expert GEMMs (one weight matrix per expert, streamed once: bound by
// HBM) are kept apart from the dense GEMMs of the same operand layout (bound by the matrix cores).
enum { KID_GEMM_NT = 0, KID_GEMM_NN, KID_GEMM_TN, KID_GEMM_GENERIC, KID_ATTN_FWD_FLASH, KID_ATTN_BWD_FLASH,
       KID_ATTN_FWD_GENERIC, KID_ATTN_BWD_GENERIC, KID_GEMM_NT_EXPERTS, KID_GEMM_NN_EXPERTS, KID_GEMM_TN_EXPERTS,
       // the memory-bound kernels: algorithmic bytes only (every input read once, every output written once)
       KID_RMSNORM_FWD, KID_RMSNORM_BWD, KID_ROPE, KID_ROUTER, KID_PERMUTE, KID_COMBINE, KID_MOE_BWD_ROWS,
       KID_ROUTER_BWD, KID_DUM_FINALIZE, KID_SWIGLU_BWD, KID_COLSUM, KID_GATHER_ROWS, KID_COPY_ROWS,
       KID_COUNT };
static const char* const kid_names[KID_COUNT] = {"gemm_mfma_nt", "gemm_mfma_nn", "gemm_mfma_tn", "gemm_generic",
                                                 "attn_fwd_flash", "attn_bwd_flash", "attn_fwd_generic",
                                                 "attn_bwd_generic", "gemm_mfma_nt_experts", "gemm_mfma_nn_experts",
                                                 "gemm_mfma_tn_experts",
                                                 "rmsnorm_fwd", "rmsnorm_bwd", "rope", "router", "permute", "combine",
                                                 "moe_bwd_rows", "router_bwd", "dum_finalize", "swiglu_bwd", "colsum",
                                                 "gather_rows", "copy_rows"};
struct ProfRec { int kid; hipEvent_t a, b; double flops, bytes; };

struct revffn_ctx {
  bool prof_on = false;
  std::vector<ProfRec>* prof = nullptr;        // launches recorded since profiling was switched on
  std::vector<hipEvent_t>* ev_pool = nullptr;  // recycled events
  revffn_config cfg;
  int dt, es;                 // element type / size of weights, activations and gradients
  int sdt, ses;               // element type / size of the residual streams x1, x2, y1, y2 (float32 with fp32_streams)
  int gdt, ges;               // element type / size of the weight gradients (float32 with fp32_grads)
  int maxT;
  int mode = 0;               // 0 auto, 1 generic kernels only
  int taps = 0;
  int device = 0;
  void* slab = nullptr;
  size_t slab_bytes = 0;
  hipStream_t side[4] = {nullptr, nullptr, nullptr, nullptr};   // helper streams for independent branches of one call
  std::vector<hipEvent_t>* sync_ev = nullptr;  // ring of timing-free events for fork/join
  size_t sync_next = 0;
  bool use_streams = true;
  int lastT = 0;
  int lastT_rows = 0;         // lastT * top_k: permuted rows of the current routing
  // attention half
  void *n12, *U12, *Q, *K, *V, *O, *AO;
  float* lse;
  // moe half
  void *n3, *Um;
  float *wrp, *probs, *gamma, *wts;
  int *idx, *counts, *offsets, *row_map, *inv_map;
  int *tg_a, *tm_a, *tg_b, *tm_b, *tf_a, *tf_b, *tg_c, *tm_c, *tf_c;
  int max_tiles_a, max_tiles_b, max_tiles_c;
  int bm_b = 128;             // height of the tiles in list b for the routing in the workspace: 128, or 160 (see expert_rows_b)
  int expert_nt = 0, expert_nn = 0;
  bool no_fused_swiglu = false; // REVFFN_NO_FUSED_SWIGLU (tuning aid): SwiGLU as a kernel of its own after the gate/up GEMM
  int expert_tile = 0;        // m-tile height of the MFMA expert GEMMs forced to 128 or 256 (REVFFN_EXPERT_TILE), 0 = by rows per expert
  int* tile_cnt;              // tiles in use of the three lists, then the flag that the routing is even
  void *Xg, *GU, *Hh, *Yp, *GUs, *Hs, *Ys, *RS;
  float *tapA, *tapM;
  void *y1c, *xtmp;
  float* resid_dev;
  // tolerance-driven inverse: > 0 = every block of rows iterates until its max|x_n - x_(n-1)| <= inv_tol, at most
  // inv_max_iters times; inv_block = positions per block inside a sequence (0 = one block for the whole call).
  // The decision is taken on the device (conv_* kernels); conv holds its state.
  float inv_tol = 0.f;
  int inv_max_iters = 0;
  int inv_block = 0;
  ConvState conv;
  size_t conv_zero_words = 0;                     // 32-bit words from conv.row_done on that start every inverse at zero
  int conv_last_nblk = 0;
  // backward
  void *dRS, *dYp, *dYs, *dHs, *dGUs, *dUm_sh, *dHh, *dGU, *dXg, *dUm, *dn3, *g1;
  float *dw, *dzext, *rinv, *rinv3, *partial;
  float *splitk_ws, *splitk_ws_r;   // split-k slices: weight-gradient side, router side (fold, then logits)
  bool fold_queued = false;         // the router fold of this call is already enqueued on helper stream 2
  // the workspace still holds every activation of this revffn_forward call (stored-activation backward)
  const void *fwd_x1 = nullptr, *fwd_x2 = nullptr, *fwd_y1 = nullptr;
  int fwd_B = 0, fwd_S = 0;
  i64 fwd_ld = 0;
  void* dwr_tmp;
  void* wr_ext;               // [E1p, d]: router rows, shared-gate row, zero rows up to a multiple of 8
  void *dzb, *dUm_r;          // bf16 logit gradients [T, E1p] and the router term of dUm [T, d]
  void *dAO, *dO, *dQ, *dK, *dV, *dU12, *dn12;
  float* dvec;
  float* rope_cs;
};

namespace {

const int BM_A = 64;    // m-tile height of the generic grouped GEMM
const int BM_B = 128;   // m-tile heights of the MFMA grouped GEMM (list b is built 160 rows high instead where that
const int BM_C = 256;   // holds a typical expert, see expert_rows_b)
const int BM_B_MID = 160;
// k-slices of the small fp32 GEMMs around the router (each would otherwise run on a handful of CUs)
const int SPLIT_FOLD = 16, SPLIT_LOGITS = 16, SPLIT_DWR = 32;

int check_cfg(const revffn_config* c) {
  if (!c) return REVFFN_ENULL;
  if (c->d_model < 2 || (c->d_model & 1)) return REVFFN_EINVAL;
  if (c->n_heads < 1 || c->head_dim < 2 || (c->head_dim & 1) || c->head_dim > 1024) return REVFFN_EINVAL;
  if ((long long)c->n_heads * c->head_dim != c->d_model) return REVFFN_EINVAL;
  if (c->n_experts < 1 || c->n_experts > 256) return REVFFN_EINVAL;
  if (c->top_k < 1 || c->top_k > c->n_experts || c->top_k > 16) return REVFFN_EINVAL;
  if (c->d_expert < 1 || c->d_shared < 0) return REVFFN_EINVAL;
  if (c->dtype != REVFFN_F32 && c->dtype != REVFFN_BF16) return REVFFN_EINVAL;
  if (c->fp32_streams != 0 && c->fp32_streams != 1) return REVFFN_EINVAL;
  if (c->symmetric != 0 && c->symmetric != 1) return REVFFN_EINVAL;
  if (c->fp32_grads != 0 && c->fp32_grads != 1) return REVFFN_EINVAL;
  if (c->n_inv_iters < 0 || c->n_inv_iters > 1024) return REVFFN_EINVAL;
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return REVFFN_EINVAL;
  return REVFFN_OK;
}

// Lays out every workspace buffer; with c->slab == nullptr it only measures.
size_t carve(revffn_ctx* c, char* base) {
  const revffn_config& f = c->cfg;
  const size_t T = (size_t)c->maxT, d = f.d_model, h = d / 2, E = f.n_experts, k = f.top_k, I = f.d_expert,
               Is = f.d_shared, N = T * k, es = c->es, H = f.n_heads;
  const size_t E1 = E + (Is ? 1 : 0);
  Carver cv;
  cv.base = base;
  c->n12 = cv.take(2 * T * h * es);
  c->U12 = cv.take(2 * T * d * es);
  c->Q = cv.take(T * d * es);
  c->K = cv.take(T * d * es);
  c->V = cv.take(T * d * es);
  c->O = cv.take(T * d * es);
  c->AO = cv.take(T * d * es);
  c->lse = (float*)cv.take(T * H * 4);
  c->n3 = cv.take(T * h * es);
  c->Um = cv.take(T * d * es);
  c->wrp = (float*)cv.take(E1 * h * 4);
  c->probs = (float*)cv.take(T * E * 4);
  c->gamma = (float*)cv.take(T * 4);
  c->wts = (float*)cv.take(N * 4);
  c->idx = (int*)cv.take(N * 4);
  c->counts = (int*)cv.take(E * 4);
  c->offsets = (int*)cv.take((E + 1) * 4);
  c->row_map = (int*)cv.take(N * 4);
  c->inv_map = (int*)cv.take(N * 4);
  c->max_tiles_a = (int)(N / BM_A + E + 1);
  c->max_tiles_b = (int)(N / BM_B + E + 1);
  c->tg_a = (int*)cv.take(c->max_tiles_a * 4);
  c->tm_a = (int*)cv.take(c->max_tiles_a * 4);
  c->tg_b = (int*)cv.take(c->max_tiles_b * 4);
  c->tm_b = (int*)cv.take(c->max_tiles_b * 4);
  c->max_tiles_c = (int)(N / BM_C + E + 1);
  c->tg_c = (int*)cv.take(c->max_tiles_c * 4);
  c->tm_c = (int*)cv.take(c->max_tiles_c * 4);
  c->tf_c = (int*)cv.take(c->max_tiles_c * 4);
  c->tile_cnt = (int*)cv.take(4 * 4);
  c->tf_a = (int*)cv.take(c->max_tiles_a * 4);
  c->tf_b = (int*)cv.take(c->max_tiles_b * 4);
  c->Xg = cv.take(N * d * es);
  c->GU = cv.take(N * 2 * I * es);
  c->Hh = cv.take(N * I * es);
  c->Yp = cv.take(N * d * es);
  c->GUs = Is ? cv.take(T * 2 * Is * es) : nullptr;
  c->Hs = Is ? cv.take(T * Is * es) : nullptr;
  c->Ys = Is ? cv.take(T * d * es) : nullptr;
  c->RS = cv.take(T * d * es);
  c->tapA = (float*)cv.take(T * h * 4);
  c->tapM = (float*)cv.take(T * h * 4);
  c->y1c = cv.take(T * h * c->ses);
  c->xtmp = cv.take(T * h * c->ses);
  c->resid_dev = (float*)cv.take(256);
  {
    // state of the device-side stopping rule: the four arrays that start every inverse at zero are contiguous
    const size_t Tp = (T + 3) & ~(size_t)3;
    char* z = (char*)cv.take(Tp * (1 + 1 + 4 + 4));
    c->conv.row_done = (unsigned char*)z;
    c->conv.blk_done = (unsigned char*)(base ? z + Tp : nullptr);
    c->conv.blk_bits = (unsigned*)(base ? z + 2 * Tp : nullptr);
    c->conv.blk_iters = (int*)(base ? z + 6 * Tp : nullptr);
    c->conv_zero_words = Tp * 10 / 4;
    c->conv.blk_res = (float*)cv.take(Tp * 4);
    c->conv.stats = (int*)cv.take(256);
  }
  c->dRS = cv.take(T * d * es);
  c->dYp = cv.take(N * d * es);
  c->dYs = Is ? cv.take(T * d * es) : nullptr;
  c->dHs = Is ? cv.take(T * Is * es) : nullptr;
  c->dGUs = Is ? cv.take(T * 2 * Is * es) : nullptr;
  c->dUm_sh = Is ? cv.take(T * d * es) : nullptr;
  c->dHh = cv.take(N * I * es);
  c->dGU = cv.take(N * 2 * I * es);
  c->dXg = cv.take(N * d * es);
  c->dUm = cv.take(T * d * es);
  c->dn3 = cv.take(T * h * es);
  c->g1 = cv.take(T * h * es);
  c->dw = (float*)cv.take(N * 4);
  c->dzext = (float*)cv.take(T * E1 * 4);
  c->dwr_tmp = cv.take(E1 * d * c->ges);
  const size_t E1p = (E1 + 7) / 8 * 8;
  c->wr_ext = cv.take(E1p * d * es);
  c->dzb = cv.take(T * E1p * 2);
  c->dUm_r = cv.take(T * d * es);
  {
    size_t a = SPLIT_FOLD * E1 * h, b2 = SPLIT_LOGITS * T * E1, c3 = SPLIT_DWR * E1 * d;
    c->splitk_ws_r = (float*)cv.take((a > b2 ? a : b2) * 4);
    c->splitk_ws = (float*)cv.take(c3 * 4);
  }
  c->rinv = (float*)cv.take(2 * T * 4);
  c->rinv3 = (float*)cv.take(T * 4);
  size_t maxcols = d > E1 ? d : E1;
  c->partial = (float*)cv.take(colsum_partial_floats((int)(2 * T), (int)maxcols) * 4);
  c->dAO = cv.take(T * d * es);
  c->dO = cv.take(T * d * es);
  c->dQ = cv.take(T * d * es);
  c->dK = cv.take(T * d * es);
  c->dV = cv.take(T * d * es);
  c->dU12 = cv.take(2 * T * d * es);
  c->dn12 = cv.take(2 * T * h * es);
  c->dvec = (float*)cv.take(T * H * 4);
  c->rope_cs = (float*)cv.take(T * (f.head_dim / 2) * 8);
  return cv.off + 256;
}

inline char* at(void* p, size_t elems, int es) { return (char*)p + elems * (size_t)es; }
inline const char* at(const void* p, size_t elems, int es) { return (const char*)p + elems * (size_t)es; }

// ---- GEMM shorthands --------------------------------------------------------------
// C[M,N] = A[M,K] . W^T, W row-major [N,K]
GemmArgs nt(const void* A, i64 lda, const void* W, i64 ldw, void* C, i64 ldc, int M, int N, int K) {
  GemmArgs g;
  g.A = A; g.lda = lda; g.B = W; g.ldb = ldw; g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K;
  return g;
}
// C[M,N] = A[M,K] . W, W row-major [K,N]
GemmArgs nn(const void* A, i64 lda, const void* W, i64 ldw, void* C, i64 ldc, int M, int N, int K) {
  GemmArgs g = nt(A, lda, W, ldw, C, ldc, M, N, K);
  g.b_trans = 1;
  return g;
}
// C[M,N] = A^T . Bm, A row-major [K,M], Bm row-major [K,N]
GemmArgs tn(const void* A, i64 lda, const void* Bm, i64 ldb, void* C, i64 ldc, int M, int N, int K) {
  GemmArgs g = nt(A, lda, Bm, ldb, C, ldc, M, N, K);
  g.a_trans = 1;
  g.b_trans = 1;
  return g;
}

// ---- optional per-kernel timing with HIP events on the launch stream -----------------
hipEvent_t prof_event(revffn_ctx* c) {
  hipEvent_t e = nullptr;
  if (!c->ev_pool->empty()) { e = c->ev_pool->back(); c->ev_pool->pop_back(); }
  else (void)hipEventCreate(&e);
  return e;
}
struct ProfScope {
  revffn_ctx* c; hipStream_t s; ProfRec r; bool on;
  ProfScope(revffn_ctx* c_, hipStream_t s_, double flops, double bytes) : c(c_), s(s_), on(c_->prof_on) {
    if (!on) return;
    r.kid = -1; r.flops = flops; r.bytes = bytes; r.a = prof_event(c); r.b = prof_event(c);
    (void)hipEventRecord(r.a, s);
  }
  void done(int kid) {
    if (!on) return;
    r.kid = kid;
    (void)hipEventRecord(r.b, s);
    c->prof->push_back(r);
  }
};

// algorithmic work of one GEMM launch: 2*M*N*K flops; every operand and the result moved once
void gemm_work(const revffn_ctx* c, const GemmArgs& g, int ta, int tb, int tc, double* flops, double* bytes) {
  const double ea = ta ? 2 : 4, eb = tb ? 2 : 4, ec = tc ? 2 : 4;
  double M = g.M, N = g.N, K = g.K, G = g.n_groups;
  if (g.group_mode == 1) { *flops = 2 * M * N * K; *bytes = M * K * ea + G * N * K * eb + M * N * ec; }
  else if (g.group_mode == 2) { double R = K;                                     // rows summed over groups
    *flops = 2 * M * N * R; *bytes = R * M * ea + R * N * eb + G * M * N * ec; }
  else { *flops = 2 * M * N * K; *bytes = M * K * ea + N * K * eb + M * N * ec; }
  if (g.resid) *bytes += M * N * (g.resid_f32 ? 4 : c->es);
  if (g.act_half) *bytes += M * (double)g.act_half * ec;
}

int run_gemm(revffn_ctx* c, GemmArgs g, int ta, int tb, int tc, hipStream_t s) {
  GemmTypes t{ta, tb, tc, c->dt};
  double fl = 0, by = 0;
  if (c->prof_on) gemm_work(c, g, ta, tb, tc, &fl, &by);
  ProfScope ps(c, s, fl, by);
  // A gate/up GEMM asks for silu(gate) * up beside its output.  The matrix-core kernel does that in its epilogue;
  // on every other route the GEMM is followed by the SwiGLU kernel, which reads the output back.
  void* act_out = g.act_out;
  const int act_half = g.act_half;
  const i64 act_rows = g.group_mode == 1 ? c->lastT_rows : g.M;
  if (act_half && c->no_fused_swiglu) { g.act_out = nullptr; g.act_half = 0; }
  auto swiglu_after = [&]() { if (act_half && !g.act_half) launch_swiglu_fwd(c->dt, g.C, act_out, act_rows, act_half, s); };
  if (c->dt == 1 && c->mode == 0 && ta == 1 && tb == 1) {
    if (g.group_mode == 1) {
      // Expert tiles stream weights that nothing else reads, so what counts is weight bytes in flight per CU: a
      // 128x256 tile (3 stages) keeps 64 KiB of them in flight, 256x128 and 128x128 half of that.  Measured: 128x256
      // is 1.5-3 % of a step faster on every workload and both layouts, except the weights-as-[k,n] layout (data
      // gradients) while one 256-row tile holds a typical expert (96 < mean rows <= 192), where 256x128 is 3 % of
      // that kernel faster.  Shapes: 1 = 128x128, 2 = 256x128, 3 = 128x256 (REVFFN_EXPERT_NT / REVFFN_EXPERT_NN force one);
      // where list b was built 160 rows high (expert_rows_b), shape 3 is the 160x256 tile.
      const i64 rows = c->lastT_rows, E = c->cfg.n_experts;
      int shape = g.b_trans ? c->expert_nn : c->expert_nt;
      if (c->expert_tile) shape = c->expert_tile == 256 ? 2 : 1;
      if (!shape) shape = (g.b_trans && rows > 96 * E && rows <= 192 * E) ? 2 : 3;
      bool tall = shape == 2;
      g.tile_bn = shape == 3 ? 256 : 128;
      const bool mid = c->bm_b == BM_B_MID;              // list b holds 160-row tiles: for the 160x256 forward kernel only
      if (mid && !tall) { if (g.b_trans) tall = true; else g.tile_bn = 256; }
      if (tall && g.b_trans) g.tile_bn = 128;
      if (tall) {
        g.tile_group = c->tg_c; g.tile_m0 = c->tm_c; g.max_tiles = c->max_tiles_c; g.tile_bm = BM_C; g.tile_count = c->tile_cnt + 2;
        if (c->max_tiles_c < 32768) g.tile_first = c->tf_c;      // (the packed entry holds 15 + 16 bits)
      } else {
        g.tile_group = c->tg_b; g.tile_m0 = c->tm_b; g.max_tiles = c->max_tiles_b; g.tile_bm = c->bm_b; g.tile_count = c->tile_cnt + 1;
        if (c->max_tiles_b < 32768) g.tile_first = c->tf_b;
      }
    }
    if (launch_gemm_mfma(g, t, s) == 0) {
      if (g.group_mode) ps.done(g.a_trans ? KID_GEMM_TN_EXPERTS : (g.b_trans ? KID_GEMM_NN_EXPERTS : KID_GEMM_NT_EXPERTS));
      else ps.done(g.a_trans ? KID_GEMM_TN : (g.b_trans ? KID_GEMM_NN : KID_GEMM_NT));
      swiglu_after();
      return 0;
    }
  }
  if (g.group_mode == 1) { g.tile_group = c->tg_a; g.tile_m0 = c->tm_a; g.max_tiles = c->max_tiles_a; g.tile_bm = BM_A; g.tile_count = c->tile_cnt; }
  g.act_out = nullptr; g.act_half = 0;
  int e = launch_gemm_generic(g, t, s) == 0 ? 0 : REVFFN_EUNSUPPORTED;
  ps.done(KID_GEMM_GENERIC);
  if (!e) swiglu_after();
  return e;
}
int run_gemm(revffn_ctx* c, const GemmArgs& g, hipStream_t s) { return run_gemm(c, g, c->dt, c->dt, c->dt, s); }
// a GEMM whose result is a weight gradient: written in the gradient dtype (float32 with fp32_grads)
// (weight gradients run on helper streams beside the data-gradient chain: the tile with the least CU-time, see
// GemmArgs::bulk; measured 1.3 % of a headline step with the shared expert's forward GEMMs treated the same way)
int run_wgrad(revffn_ctx* c, const GemmArgs& g0, hipStream_t s) {
  GemmArgs g = g0;
  g.bulk = c->use_streams;
  return run_gemm(c, g, c->dt, c->dt, c->gdt, s);
}

// ---- the memory-bound kernels, timed like the GEMMs when profiling is on: algorithmic bytes = every input read
// once and every output written once (index arrays and per-row scalars included, gains and tables left out)
inline double esz(int dt) { return dt ? 2.0 : 4.0; }
void p_rmsnorm_fwd(revffn_ctx* c, int dt, int tx, const void* x, i64 ldx, const void* g, void* out, i64 ldo, int rows,
                   int h, float eps, hipStream_t s, const unsigned char* skip = nullptr, const void* x2 = nullptr,
                   const void* g2 = nullptr, void* out2 = nullptr) {
  ProfScope ps(c, s, 0, (x2 ? 2.0 : 1.0) * rows * h * (esz(tx) + esz(dt)));
  launch_rmsnorm_fwd(dt, tx, x, ldx, g, out, ldo, rows, h, eps, s, skip, x2, g2, out2);
  ps.done(KID_RMSNORM_FWD);
}
void p_rmsnorm_bwd(revffn_ctx* c, int dt, int tx, const void* dy, i64 ldd, const void* x, i64 ldx, const void* g,
                   const void* base, i64 ldb, void* dx, i64 ldo, float* rinv, int rows, int h, float eps, hipStream_t s) {
  ProfScope ps(c, s, 0, (double)rows * h * (esz(tx) + (base ? 3 : 2) * esz(dt)) + rows * 4.0);
  launch_rmsnorm_bwd(dt, tx, dy, ldd, x, ldx, g, base, ldb, dx, ldo, rinv, rows, h, eps, s);
  ps.done(KID_RMSNORM_BWD);
}
void p_rope(revffn_ctx* c, int dt, void* buf, const float* cs, int T, int S, int H, int dh, float sign, hipStream_t s,
            void* buf2 = nullptr, const unsigned char* skip = nullptr) {
  ProfScope ps(c, s, 0, (buf2 ? 2.0 : 1.0) * 2.0 * T * H * dh * esz(dt));
  launch_rope(dt, buf, cs, T, S, H, dh, sign, s, buf2, skip);
  ps.done(KID_ROPE);
}
void p_router(revffn_ctx* c, int dt, const void* y1, i64 ld, const float* zparts, int n_parts, const float* b_router,
              float* probs, int* idx, float* wts, float* gamma, int T, int h, int E, int k, int has_gate, int norm_topk,
              float eps, hipStream_t s) {
  ProfScope ps(c, s, 0, (double)T * (h * esz(dt) + (double)n_parts * (E + has_gate) * 4 + E * 4 + k * 8 + has_gate * 4));
  launch_router(dt, y1, ld, zparts, n_parts, b_router, probs, idx, wts, gamma, T, h, E, k, has_gate, norm_topk, eps, s);
  ps.done(KID_ROUTER);
}
void p_permute(revffn_ctx* c, const int* idx, int T, int k, int E, int* counts, int* offsets, int* row_map, int* inv_map,
               const TileLists& tl, hipStream_t s) {
  ProfScope ps(c, s, 0, (double)T * k * 4 * 4);                    // idx read twice, row_map and inv_map written
  launch_permute(idx, T, k, E, counts, offsets, row_map, inv_map, tl, s);
  ps.done(KID_PERMUTE);
}
void p_combine(revffn_ctx* c, int dt, const void* yp, const int* inv_map, const float* wts, const void* ys,
               const float* gamma, void* rs, int T, int d, int k, hipStream_t s) {
  ProfScope ps(c, s, 0, (double)T * d * esz(dt) * (k + (ys ? 2 : 1)) + (double)T * k * 8);
  launch_combine(dt, yp, inv_map, wts, ys, gamma, rs, T, d, k, s);
  ps.done(KID_COMBINE);
}
void p_moe_bwd_rows(revffn_ctx* c, int dt, const void* drs, const void* yp, const void* ys, const int* inv_map,
                    const float* wts, const float* gamma, void* dyp, void* dys, float* dw, float* dzext, int T, int d,
                    int k, int E1, int has_gate, hipStream_t s) {
  ProfScope ps(c, s, 0, (double)T * d * esz(dt) * (1 + 2 * k + (has_gate ? 2 : 0)) + (double)T * k * 12);
  launch_moe_bwd_rows(dt, drs, yp, ys, inv_map, wts, gamma, dyp, dys, dw, dzext, T, d, k, E1, has_gate, s);
  ps.done(KID_MOE_BWD_ROWS);
}
void p_router_bwd(revffn_ctx* c, const float* probs, const int* idx, const float* wts, const float* dw, float* dzext,
                  int T, int E, int k, int E1, int norm_topk, hipStream_t s, void* dzb = nullptr, int E1p = 0) {
  ProfScope ps(c, s, 0, (double)T * (E * 8.0 + k * 12.0 + (dzb ? E1p * 2.0 : 0.0)));
  launch_router_bwd(probs, idx, wts, dw, dzext, T, E, k, E1, norm_topk, s, dzb, E1p);
  ps.done(KID_ROUTER_BWD);
}
void p_dum_finalize(revffn_ctx* c, int dt, const void* dxg, const int* inv_map, const void* dum_sh, const void* dum_r,
                    const float* dzext, const void* w_router, const void* ws_gate, void* dum, int T, int d, int k, int E,
                    int E1, hipStream_t s) {
  ProfScope ps(c, s, 0, (double)T * d * esz(dt) * (k + 1 + (dum_sh ? 1 : 0) + (dum_r ? 1 : 0)) + (double)T * k * 4);
  launch_dum_finalize(dt, dxg, inv_map, dum_sh, dum_r, dzext, w_router, ws_gate, dum, T, d, k, E, E1, s);
  ps.done(KID_DUM_FINALIZE);
}
void p_swiglu_bwd(revffn_ctx* c, int dt, const void* dhh, const void* gu, void* dgu, i64 rows, int I, hipStream_t s) {
  ProfScope ps(c, s, 0, 5.0 * rows * I * esz(dt));
  launch_swiglu_bwd(dt, dhh, gu, dgu, rows, I, s);
  ps.done(KID_SWIGLU_BWD);
}
void p_colsum(revffn_ctx* c, int ta, const void* a, i64 lda, int tb, const void* b, i64 ldb, const float* sc, int tout,
              void* out, float* partial, int rows, int cols, hipStream_t s) {
  ProfScope ps(c, s, 0, (double)rows * cols * (esz(ta) + (b ? esz(tb) : 0.0)) + (sc ? rows * 4.0 : 0.0));
  launch_colsum(ta, a, lda, tb, b, ldb, sc, tout, out, partial, rows, cols, s);
  ps.done(KID_COLSUM);
}
void p_colsum_batch(revffn_ctx* c, int n, int ta, const void* const* a, const i64* lda, int tb, const void* const* b,
                    const i64* ldb, const float* const* sc, int tout, void* const* out, int rows, int cols, hipStream_t s) {
  if (n <= 0) return;
  ProfScope ps(c, s, 0, (double)n * ((double)rows * cols * (esz(ta) + (b ? esz(tb) : 0.0)) + (sc ? rows * 4.0 : 0.0)));
  launch_colsum_batch(n, ta, a, lda, tb, b, ldb, sc, tout, out, c->partial, rows, cols, s);
  ps.done(KID_COLSUM);
}
void p_gather_rows(revffn_ctx* c, int dt, const void* src, const int* row_map, int div, void* dst, int rows, int cols,
                   hipStream_t s) {
  ProfScope ps(c, s, 0, 2.0 * rows * cols * esz(dt) + rows * 4.0);
  launch_gather_rows(dt, src, row_map, div, dst, rows, cols, s);
  ps.done(KID_GATHER_ROWS);
}
void p_copy_rows(revffn_ctx* c, int dt, const void* src, i64 lds_, void* dst, i64 ldd, int rows, int cols, hipStream_t s) {
  ProfScope ps(c, s, 0, 2.0 * rows * cols * esz(dt));
  launch_copy_rows(dt, src, lds_, dst, ldd, rows, cols, s);
  ps.done(KID_COPY_ROWS);
}

// n <= 3 dense GEMMs of one shape, layout and strides as ONE launch of the matrix-core kernel (the 2048-wide
// projections are one round of workgroups each: together they fill the chip for several rounds); where that kernel
// does not take the problem they run one after the other.  tc: element type of the results.
int run_gemm_multi(revffn_ctx* c, const GemmArgs* subs, int n, int tc, hipStream_t s) {
  if (n <= 0) return 0;
  if (n > 1 && c->dt == 1 && c->mode == 0) {
    GemmArgs g = subs[0];
    g.n_sub = n;
    for (int z = 1; z < n; z++) {
      g.subA[z - 1] = subs[z].A; g.subB[z - 1] = subs[z].B; g.subC[z - 1] = subs[z].C; g.subBias[z - 1] = subs[z].bias;
    }
    GemmTypes t{c->dt, c->dt, tc, c->dt};
    double fl = 0, by = 0;
    if (c->prof_on) { gemm_work(c, subs[0], c->dt, c->dt, tc, &fl, &by); fl *= n; by *= n; }
    ProfScope ps(c, s, fl, by);
    if (launch_gemm_mfma(g, t, s) == 0) {
      ps.done(g.a_trans ? KID_GEMM_TN : (g.b_trans ? KID_GEMM_NN : KID_GEMM_NT));
      return 0;
    }
  }
  for (int z = 0; z < n; z++) {
    int e = run_gemm(c, subs[z], c->dt, c->dt, tc, s);
    if (e) return e;
  }
  return 0;
}

#define TRY(x) do { int _e = (x); if (_e) return _e; } while (0)

// ---- fork / join between the caller's stream and the context's helper streams ----------
// Independent branches of one call (K and V projections next to Q, the shared expert next to
// the routed experts, every weight-gradient GEMM next to the data-gradient chain) run on helper
// streams of default priority, so that launches too small to fill 256 CUs overlap.
hipEvent_t next_sync(revffn_ctx* c) {
  hipEvent_t e = (*c->sync_ev)[c->sync_next % c->sync_ev->size()];
  c->sync_next++;
  return e;
}
// stream `to` waits for everything enqueued so far on `from`
void after(revffn_ctx* c, hipStream_t from, hipStream_t to) {
  if (from == to) return;
  hipEvent_t e = next_sync(c);
  (void)hipEventRecord(e, from);
  (void)hipStreamWaitEvent(to, e, 0);
}
// the two halves of after(): an event that marks what `from` holds now, waited for later
hipEvent_t mark(revffn_ctx* c, hipStream_t from) {
  hipEvent_t e = next_sync(c);
  (void)hipEventRecord(e, from);
  return e;
}
void wait_for(hipStream_t to, hipEvent_t e) { (void)hipStreamWaitEvent(to, e, 0); }
// helper stream i, or the main stream when helper streams are switched off
hipStream_t side(revffn_ctx* c, hipStream_t main, int i) { return c->use_streams ? c->side[i] : main; }

// ---- attention half ---------------------------------------------------------------
// Query side of the attention half at x1: n12[0:T], U12[0:T], Q.
// skip (may be null): rows marked there are finished rows of the inverse's iteration and are left alone.
int attn_q(revffn_ctx* c, const revffn_weights* w, const void* x1, i64 ld1, int B, int S, hipStream_t s,
           const unsigned char* skip = nullptr) {
  const revffn_config& f = c->cfg;
  const int T = B * S, d = f.d_model, h = d / 2, dt = c->dt;
  p_rmsnorm_fwd(c, dt, c->sdt, x1, ld1, w->norm_a1, c->n12, h, T, h, f.rms_eps, s, skip);
  GemmArgs gu = nt(c->n12, h, w->pup_a, h, c->U12, d, T, d, h);
  gu.row_skip = skip;
  TRY(run_gemm(c, gu, s));
  GemmArgs gq = nt(c->U12, d, w->wq, d, c->Q, d, T, d, d);
  gq.bias = w->bq;
  gq.row_skip = skip;
  TRY(run_gemm(c, gq, s));
  if (f.use_rope) p_rope(c, dt, c->Q, c->rope_cs, T, S, f.n_heads, f.head_dim, 1.f, s, nullptr, skip);
  return 0;
}
// Recomputes n12, U12, Q, (K, V), O, lse, AO at streams (x1, x2).  q_done: attn_q(x1) has been enqueued already.
int attn_acts(revffn_ctx* c, const revffn_weights* w, const void* x1, i64 ld1, const void* x2, i64 ld2, int B, int S,
              bool do_kv, hipStream_t s, bool q_done = false, const unsigned char* skip = nullptr) {
  const revffn_config& f = c->cfg;
  const int T = B * S, d = f.d_model, h = d / 2, es = c->es, dt = c->dt;
  if (f.symmetric) {
    // comparison block: queries from stream 2 as well.  n2, U2 keep their places in the second halves of n12, U12.
    void* n2 = at(c->n12, (size_t)T * h, es);
    void* U2s = at(c->U12, (size_t)T * d, es);
    p_rmsnorm_fwd(c, dt, c->sdt, x2, ld2, w->norm_a2, n2, h, T, h, f.rms_eps, s);
    TRY(run_gemm(c, nt(n2, h, w->pup_a, h, U2s, d, T, d, h), s));
    GemmArgs gq = nt(U2s, d, w->wq, d, c->Q, d, T, d, d);
    gq.bias = w->bq;
    TRY(run_gemm(c, gq, s));
    if (f.use_rope) p_rope(c, dt, c->Q, c->rope_cs, T, S, f.n_heads, f.head_dim, 1.f, s);
    do_kv = true;
  } else if (q_done) {
    if (do_kv) {
      p_rmsnorm_fwd(c, dt, c->sdt, x2, ld2, w->norm_a2, at(c->n12, (size_t)T * h, es), h, T, h, f.rms_eps, s);
      TRY(run_gemm(c, nt(at(c->n12, (size_t)T * h, es), h, w->pup_a, h, at(c->U12, (size_t)T * d, es), d, T, d, h), s));
    }
  } else if (!do_kv) {
    TRY(attn_q(c, w, x1, ld1, B, S, s, skip));          // a later iterate of the inverse: query side only
  } else {
    // both streams in one launch (the two streams of a call share their row stride)
    if (do_kv && ld1 == ld2)
      p_rmsnorm_fwd(c, dt, c->sdt, x1, ld1, w->norm_a1, c->n12, h, T, h, f.rms_eps, s, nullptr, x2, w->norm_a2,
                    at(c->n12, (size_t)T * h, es));
    else {
      p_rmsnorm_fwd(c, dt, c->sdt, x1, ld1, w->norm_a1, c->n12, h, T, h, f.rms_eps, s);
      if (do_kv) p_rmsnorm_fwd(c, dt, c->sdt, x2, ld2, w->norm_a2, at(c->n12, (size_t)T * h, es), h, T, h, f.rms_eps, s);
    }
    // the same P_up serves both streams: one GEMM over the stacked rows
    TRY(run_gemm(c, nt(c->n12, h, w->pup_a, h, c->U12, d, do_kv ? 2 * T : T, d, h), s));
    if (do_kv) {
      // Q, K and V projections as one launch (three problems of one shape), then one rotary launch for Q and K
      const void* U2 = at(c->U12, (size_t)T * d, es);
      GemmArgs q3[3] = {nt(c->U12, d, w->wq, d, c->Q, d, T, d, d), nt(U2, d, w->wk, d, c->K, d, T, d, d),
                        nt(U2, d, w->wv, d, c->V, d, T, d, d)};
      q3[0].bias = w->bq; q3[1].bias = w->bk; q3[2].bias = w->bv;
      TRY(run_gemm_multi(c, q3, 3, dt, s));
      if (f.use_rope) p_rope(c, dt, c->Q, c->rope_cs, T, S, f.n_heads, f.head_dim, 1.f, s, c->K);
      do_kv = false;                                   // done here
    } else {
      GemmArgs gq = nt(c->U12, d, w->wq, d, c->Q, d, T, d, d);
      gq.bias = w->bq;
      TRY(run_gemm(c, gq, s));
      if (f.use_rope) p_rope(c, dt, c->Q, c->rope_cs, T, S, f.n_heads, f.head_dim, 1.f, s);
    }
  }
  if (do_kv) {
    // (the query side was enqueued earlier, or comes from stream 2 in the symmetric block): K and V as one launch
    const void* U2 = at(c->U12, (size_t)T * d, es);
    GemmArgs kv[2] = {nt(U2, d, w->wk, d, c->K, d, T, d, d), nt(U2, d, w->wv, d, c->V, d, T, d, d)};
    kv[0].bias = w->bk; kv[1].bias = w->bv;
    TRY(run_gemm_multi(c, kv, 2, dt, s));
    if (f.use_rope) p_rope(c, dt, c->K, c->rope_cs, T, S, f.n_heads, f.head_dim, 1.f, s);
  }
  {
    // algorithmic work of the attention core: QK^T and PV, halved by the causal mask
    double fl = 4.0 * B * (double)S * S * d * (f.causal ? 0.5 : 1.0), by = 4.0 * T * d * es;
    ProfScope ps(c, s, fl, by);
    bool done = false;
    if (dt == 1 && c->mode == 0)
      done = launch_attn_fwd_flash(c->Q, c->K, c->V, c->O, c->lse, B, S, f.n_heads, f.head_dim, f.causal, s, skip) == 0;
    if (!done) launch_attn_fwd_generic(dt, c->Q, c->K, c->V, c->O, c->lse, B, S, f.n_heads, f.head_dim, f.causal, s, skip);
    ps.done(done ? KID_ATTN_FWD_FLASH : KID_ATTN_FWD_GENERIC);
  }
  GemmArgs go = nt(c->O, d, w->wo, d, c->AO, d, T, d, d);
  go.row_skip = skip;
  TRY(run_gemm(c, go, s));
  return 0;
}
// dst = resid + sign * P_dn_a(AO)     (Eq. 1 and the second line of the inverse)
int attn_out(revffn_ctx* c, const revffn_weights* w, const void* resid, i64 ldr, float sign, void* dst, i64 ldd,
             int T, hipStream_t s, const unsigned char* skip = nullptr) {
  const int d = c->cfg.d_model, h = d / 2;
  GemmArgs g = nt(c->AO, d, w->pdn_a, d, dst, ldd, T, h, d);
  g.row_skip = skip;
  g.resid = resid; g.ldr = ldr; g.resid_sign = sign; g.resid_f32 = c->sdt == REVFFN_F32;
  if (c->taps) { g.tap = c->tapA; g.ldtap = h; }
  return run_gemm(c, g, c->dt, c->dt, c->sdt, s);
}

// ---- MoE half ---------------------------------------------------------------------
// Folded fp32 router matrix wrp = [W_r ; w_shared_gate] . P_up_m . diag(gain).  It depends on the weights only, so a
// call that starts with the attention half enqueues it at once on helper stream 2, next to that half.
// dst != null: the fold goes there (pre-merged weights) and runs on s itself.
void router_fold(revffn_ctx* c, const revffn_weights* w, hipStream_t s, float* dst = nullptr) {
  const revffn_config& f = c->cfg;
  const int d = f.d_model, h = d / 2, E = f.n_experts, Is = f.d_shared, dt = c->dt;
  hipStream_t sr = dst ? s : side(c, s, 2);
  after(c, s, sr);                        // everything that read wr_ext / wrp before is on s
  // [W_r ; w_shared_gate] stacked into one [E1, d] matrix so that the fold is a single GEMM
  {
    ProfScope ps(c, sr, 0, 2.0 * (E + (Is ? 1 : 0)) * d * esz(dt));
    launch_copy_rows2(dt, w->w_router, d, E, Is ? w->ws_gate : w->w_router, d, Is ? 1 : 0, c->wr_ext, d, d, sr);
    ps.done(KID_COPY_ROWS);
  }
  GemmArgs a = nn(c->wr_ext, d, w->pup_m, h, dst ? dst : c->wrp, h, E + (Is ? 1 : 0), h, d);
  a.split_k = SPLIT_FOLD; a.splitk_ws = c->splitk_ws_r; a.col_scale = w->norm_m;
  (void)run_gemm(c, a, dt, dt, 0, sr);
  if (!dst) c->fold_queued = true;
}

// Height of the tiles in list b (the routed experts' forward GEMMs) for N permuted rows over E experts.  An expert's
// rows are padded to whole tiles, its weight tile is fetched once per row tile, and with top-k of many small experts
// the mean expert (Qwen shape at 2048 tokens: 137 rows, standard deviation 12) is just above one 128-row tile: 77 %
// of the experts then take two tiles, the second nearly empty.  Tiles 160 rows high hold such experts in one (the
// forward kernels 7.5 % faster).  Only when the mean lies where that pays; a pure function of (N, E), so every call
// that reuses a routing sees the height its lists were built with.
static int expert_rows_b(const revffn_ctx* c, i64 N, i64 E) {
  if (c->expert_tile || c->expert_nt || c->expert_nn) return BM_B;          // a forced shape (tuning aid) keeps 128
  return (N > 118 * E && N <= 152 * E) ? BM_B_MID : BM_B;
}

// Recomputes n3, Um, routing, GU, Hh, Yp, shared expert and RS at y1.  q_x1 != null: the query side of the attention
// half at q_x1 (which must not depend on this MoE evaluation) is enqueued on s while the routing chain runs.
int moe_acts(revffn_ctx* c, const revffn_weights* w, const void* y1, i64 ld, int T, hipStream_t s,
             const void* q_x1 = nullptr, i64 q_ld = 0, int qB = 0, int qS = 0, const unsigned char* q_skip = nullptr) {
  const revffn_config& f = c->cfg;
  const int d = f.d_model, h = d / 2, E = f.n_experts, k = f.top_k, I = f.d_expert, Is = f.d_shared, dt = c->dt;
  const int N = T * k, E1 = E + (Is ? 1 : 0);
  c->lastT = T;
  c->lastT_rows = N;
  c->bm_b = expert_rows_b(c, N, E);
  // Routing needs Y1 and the weights only (the logits are Y1 . wrp^T in fp32, scaled by 1/rms(Y1) in the router
  // kernel), so fold, logits, top-k and the permutation run on helper stream 2 next to the norm and the up-projection.
  hipStream_t sr = side(c, s, 2);
  if (c->fold_queued) after(c, s, sr);    // y1 is complete on s
  else router_fold(c, w, s);              // (forks from s as well)
  c->fold_queued = false;
  {
    GemmArgs z = nt(y1, ld, c->wrp, h, c->splitk_ws_r, E1, T, E1, h);
    z.split_k = SPLIT_LOGITS; z.splitk_ws = c->splitk_ws_r; z.splitk_raw = 1;   // the router kernel adds the slices
    GemmTypes tz{c->sdt, 0, 0, dt};
    if (launch_gemm_generic(z, tz, sr)) return REVFFN_EUNSUPPORTED;
  }
  p_router(c, c->sdt, y1, ld, c->splitk_ws_r, SPLIT_LOGITS, w->b_router, c->probs, c->idx, c->wts, c->gamma, T, h, E, k,
                Is ? 1 : 0, f.norm_topk_prob, f.rms_eps, sr);
  TileLists tl{{c->tg_a, c->tg_b, c->tg_c}, {c->tm_a, c->tm_b, c->tm_c}, {c->tf_a, c->tf_b, c->tf_c},
               {c->max_tiles_a, c->max_tiles_b, c->max_tiles_c}, {BM_A, c->bm_b, BM_C}, c->tile_cnt};
  p_permute(c, c->idx, T, k, E, c->counts, c->offsets, c->row_map, c->inv_map, tl, sr);
  p_rmsnorm_fwd(c, dt, c->sdt, y1, ld, w->norm_m, c->n3, h, T, h, f.rms_eps, s);
  TRY(run_gemm(c, nt(c->n3, h, w->pup_m, h, c->Um, d, T, d, h), s));
  hipStream_t s0 = side(c, s, 0);
  if (Is) {                               // the shared expert needs Um only: next to routing + routed experts
    after(c, s, s0);
    GemmArgs gs = nt(c->Um, d, w->ws_gate_up, d, c->GUs, 2 * Is, T, 2 * Is, d);
    gs.act_out = c->Hs; gs.ldact = Is; gs.act_half = Is;      // Hs = silu(gate) * up with the GEMM
    gs.bulk = c->use_streams;                                 // beside the routed experts' GEMMs
    TRY(run_gemm(c, gs, s0));
    GemmArgs gd = nt(c->Hs, Is, w->ws_down, Is, c->Ys, d, T, d, Is);
    gd.bulk = gs.bulk;
    TRY(run_gemm(c, gd, s0));
  }
  if (q_x1) TRY(attn_q(c, w, q_x1, q_ld, qB, qS, s, q_skip));
  after(c, sr, s);                        // routing and permutation are ready
  // routed experts: GU = Xg . Wgu_e^T (rows gathered from Um through row_map), SwiGLU, Yp = Hh . Wd_e^T
  GemmArgs g1 = nt(c->Um, d, w->w_gate_up, d, c->GU, 2 * I, N, 2 * I, d);
  g1.group_mode = 1; g1.n_groups = E; g1.offsets = c->offsets; g1.b_group_stride = (i64)2 * I * d;
  g1.a_gather = c->row_map; g1.gather_div = k;
  g1.act_out = c->Hh; g1.ldact = I; g1.act_half = I;          // Hh = silu(gate) * up with the GEMM
  TRY(run_gemm(c, g1, s));
  GemmArgs g2 = nt(c->Hh, I, w->w_down, I, c->Yp, d, N, d, I);
  g2.group_mode = 1; g2.n_groups = E; g2.offsets = c->offsets; g2.b_group_stride = (i64)d * I;
  TRY(run_gemm(c, g2, s));
  if (Is) after(c, s0, s);
  p_combine(c, dt, c->Yp, c->inv_map, c->wts, Is ? c->Ys : nullptr, c->gamma, c->RS, T, d, k, s);
  c->lastT = T;
  return 0;
}
// dst = resid + sign * P_dn_m(RS)     (Eq. 2 and the first line of the inverse)
int moe_out(revffn_ctx* c, const revffn_weights* w, const void* resid, i64 ldr, float sign, void* dst, i64 ldd,
            int T, hipStream_t s) {
  const int d = c->cfg.d_model, h = d / 2;
  GemmArgs g = nt(c->RS, d, w->pdn_m, d, dst, ldd, T, h, d);
  g.resid = resid; g.ldr = ldr; g.resid_sign = sign; g.resid_f32 = c->sdt == REVFFN_F32;
  if (c->taps) { g.tap = c->tapM; g.ldtap = h; }
  return run_gemm(c, g, c->dt, c->dt, c->sdt, s);
}

// End of an entry point: a call that failed half way (REVFFN_EHIP / EUNSUPPORTED from a launch) may have forked work
// onto the helper streams; the caller's stream is made to wait for them, so that whatever was enqueued is ordered
// before the caller's next work.
int finish(revffn_ctx* c, hipStream_t s, int e) {
  if (e && c && c->use_streams)
    for (int i = 0; i < 4; i++) after(c, c->side[i], s);
  return e;
}

// ---- pre-merged adapters (section 3.2: Attn(.) = P_dn(Attn_pt(P_up .)), MLP(.) = P_dn(MLP_pt(P_up .))) ------------
// With static weights the products W . P_up and P_dn . W can be formed once; the forward and inverse passes then
// work on half-width inputs and outputs: no adapter GEMMs, Q/K/V projections and expert gate-up GEMMs with half the
// contraction length, expert down GEMMs with half the output width, and half the expert weight bytes to stream.
int merge_impl(revffn_ctx* c, const revffn_weights* w, const revffn_merged* m, hipStream_t s) {
  const revffn_config& f = c->cfg;
  const int d = f.d_model, h = d / 2, E = f.n_experts, I = f.d_expert, Is = f.d_shared, es = c->es;
  GemmArgs q3[3] = {nn(w->wq, d, w->pup_a, h, m->wq, h, d, h, d), nn(w->wk, d, w->pup_a, h, m->wk, h, d, h, d),
                    nn(w->wv, d, w->pup_a, h, m->wv, h, d, h, d)};
  TRY(run_gemm_multi(c, q3, 3, c->dt, s));
  TRY(run_gemm(c, nn(w->pdn_a, d, w->wo, d, m->wo, d, h, d, d), s));
  {
    // every expert's gate-up rows at once: [E * 2I, d] . [d, h]; in slices that keep 32-bit operand offsets valid
    const i64 rows = (i64)E * 2 * I, step = ((i64)1 << 29) / d;
    for (i64 r0 = 0; r0 < rows; r0 += step) {
      const int mrows = (int)((rows - r0) < step ? (rows - r0) : step);
      TRY(run_gemm(c, nn(at(w->w_gate_up, (size_t)r0 * d, es), d, w->pup_m, h, at(m->w_gate_up, (size_t)r0 * h, es), h, mrows, h, d), s));
    }
  }
  for (int e = 0; e < E; e++)
    TRY(run_gemm(c, nn(w->pdn_m, d, at(w->w_down, (size_t)e * d * I, es), I, at(m->w_down, (size_t)e * h * I, es), I, h, I, d), s));
  if (Is) {
    TRY(run_gemm(c, nn(w->ws_gate_up, d, w->pup_m, h, m->ws_gate_up, h, 2 * Is, h, d), s));
    TRY(run_gemm(c, nn(w->pdn_m, d, w->ws_down, Is, m->ws_down, Is, h, Is, d), s));
  }
  router_fold(c, w, s, m->w_router);
  return 0;
}

// n12, Q, (K, V), O, lse at streams (x1, x2) from merged projections.  do_kv = false: the query side only (a later
// iterate of the inverse).
int attn_acts_merged(revffn_ctx* c, const revffn_weights* w, const revffn_merged* m, const void* x1, i64 ld1,
                     const void* x2, i64 ld2, int B, int S, bool do_kv, hipStream_t s) {
  const revffn_config& f = c->cfg;
  const int T = B * S, d = f.d_model, h = d / 2, es = c->es, dt = c->dt;
  void* n2 = at(c->n12, (size_t)T * h, es);
  if (do_kv) {
    if (ld1 == ld2) p_rmsnorm_fwd(c, dt, c->sdt, x1, ld1, w->norm_a1, c->n12, h, T, h, f.rms_eps, s, nullptr, x2, w->norm_a2, n2);
    else {
      p_rmsnorm_fwd(c, dt, c->sdt, x1, ld1, w->norm_a1, c->n12, h, T, h, f.rms_eps, s);
      p_rmsnorm_fwd(c, dt, c->sdt, x2, ld2, w->norm_a2, n2, h, T, h, f.rms_eps, s);
    }
    GemmArgs q3[3] = {nt(c->n12, h, m->wq, h, c->Q, d, T, d, h), nt(n2, h, m->wk, h, c->K, d, T, d, h),
                      nt(n2, h, m->wv, h, c->V, d, T, d, h)};
    q3[0].bias = w->bq; q3[1].bias = w->bk; q3[2].bias = w->bv;
    TRY(run_gemm_multi(c, q3, 3, dt, s));
    if (f.use_rope) p_rope(c, dt, c->Q, c->rope_cs, T, S, f.n_heads, f.head_dim, 1.f, s, c->K);
  } else {
    p_rmsnorm_fwd(c, dt, c->sdt, x1, ld1, w->norm_a1, c->n12, h, T, h, f.rms_eps, s);
    GemmArgs gq = nt(c->n12, h, m->wq, h, c->Q, d, T, d, h);
    gq.bias = w->bq;
    TRY(run_gemm(c, gq, s));
    if (f.use_rope) p_rope(c, dt, c->Q, c->rope_cs, T, S, f.n_heads, f.head_dim, 1.f, s);
  }
  double fl = 4.0 * B * (double)S * S * d * (f.causal ? 0.5 : 1.0), by = 4.0 * T * d * es;
  ProfScope ps(c, s, fl, by);
  bool done = false;
  if (dt == 1 && c->mode == 0)
    done = launch_attn_fwd_flash(c->Q, c->K, c->V, c->O, c->lse, B, S, f.n_heads, f.head_dim, f.causal, s) == 0;
  if (!done) launch_attn_fwd_generic(dt, c->Q, c->K, c->V, c->O, c->lse, B, S, f.n_heads, f.head_dim, f.causal, s);
  ps.done(done ? KID_ATTN_FWD_FLASH : KID_ATTN_FWD_GENERIC);
  return 0;
}
// dst = resid + sign * O . (P_dn_a Wo)^T
int attn_out_merged(revffn_ctx* c, const revffn_merged* m, const void* resid, i64 ldr, float sign, void* dst, i64 ldd,
                    int T, hipStream_t s) {
  const int d = c->cfg.d_model, h = d / 2;
  GemmArgs g = nt(c->O, d, m->wo, d, dst, ldd, T, h, d);
  g.resid = resid; g.ldr = ldr; g.resid_sign = sign; g.resid_f32 = c->sdt == REVFFN_F32;
  if (c->taps) { g.tap = c->tapA; g.ldtap = h; }
  return run_gemm(c, g, c->dt, c->dt, c->sdt, s);
}
// dst = resid + sign * MoE branch at y1, everything from merged weights (routing from the stored fp32 fold)
int moe_merged(revffn_ctx* c, const revffn_weights* w, const revffn_merged* m, const void* y1, i64 ld, const void* resid,
               i64 ldr, float sign, void* dst, i64 ldd, int T, hipStream_t s) {
  const revffn_config& f = c->cfg;
  const int d = f.d_model, h = d / 2, E = f.n_experts, k = f.top_k, I = f.d_expert, Is = f.d_shared, dt = c->dt;
  const int N = T * k, E1 = E + (Is ? 1 : 0);
  c->lastT = T;
  c->lastT_rows = N;
  c->bm_b = expert_rows_b(c, N, E);
  hipStream_t sr = side(c, s, 2), s0 = side(c, s, 0);
  after(c, s, sr);
  {
    GemmArgs z = nt(y1, ld, m->w_router, h, c->splitk_ws_r, E1, T, E1, h);
    z.split_k = SPLIT_LOGITS; z.splitk_ws = c->splitk_ws_r; z.splitk_raw = 1;
    GemmTypes tz{c->sdt, 0, 0, dt};
    if (launch_gemm_generic(z, tz, sr)) return REVFFN_EUNSUPPORTED;
  }
  p_router(c, c->sdt, y1, ld, c->splitk_ws_r, SPLIT_LOGITS, w->b_router, c->probs, c->idx, c->wts, c->gamma, T, h, E, k,
           Is ? 1 : 0, f.norm_topk_prob, f.rms_eps, sr);
  TileLists tl{{c->tg_a, c->tg_b, c->tg_c}, {c->tm_a, c->tm_b, c->tm_c}, {c->tf_a, c->tf_b, c->tf_c},
               {c->max_tiles_a, c->max_tiles_b, c->max_tiles_c}, {BM_A, c->bm_b, BM_C}, c->tile_cnt};
  p_permute(c, c->idx, T, k, E, c->counts, c->offsets, c->row_map, c->inv_map, tl, sr);
  p_rmsnorm_fwd(c, dt, c->sdt, y1, ld, w->norm_m, c->n3, h, T, h, f.rms_eps, s);
  if (Is) {
    after(c, s, s0);
    GemmArgs gs = nt(c->n3, h, m->ws_gate_up, h, c->GUs, 2 * Is, T, 2 * Is, h);
    gs.act_out = c->Hs; gs.ldact = Is; gs.act_half = Is;
    gs.bulk = c->use_streams;
    TRY(run_gemm(c, gs, s0));
    GemmArgs gd = nt(c->Hs, Is, m->ws_down, Is, c->Ys, h, T, h, Is);
    gd.bulk = gs.bulk;
    TRY(run_gemm(c, gd, s0));
  }
  after(c, sr, s);
  GemmArgs g1 = nt(c->n3, h, m->w_gate_up, h, c->GU, 2 * I, N, 2 * I, h);
  g1.group_mode = 1; g1.n_groups = E; g1.offsets = c->offsets; g1.b_group_stride = (i64)2 * I * h;
  g1.a_gather = c->row_map; g1.gather_div = k;
  g1.act_out = c->Hh; g1.ldact = I; g1.act_half = I;
  TRY(run_gemm(c, g1, s));
  GemmArgs g2 = nt(c->Hh, I, m->w_down, I, c->Yp, h, N, h, I);
  g2.group_mode = 1; g2.n_groups = E; g2.offsets = c->offsets; g2.b_group_stride = (i64)h * I;
  TRY(run_gemm(c, g2, s));
  if (Is) after(c, s0, s);
  {
    ProfScope ps(c, s, 0, (double)T * h * esz(dt) * (k + (Is ? 1 : 0)) + 2.0 * T * h * esz(c->sdt));
    launch_combine_couple(dt, c->sdt, c->Yp, c->inv_map, c->wts, Is ? c->Ys : nullptr, c->gamma, resid, ldr, sign, dst, ldd,
                          c->taps ? c->tapM : nullptr, T, h, k, s);
    ps.done(KID_COMBINE);
  }
  return 0;
}
int check_merged(const revffn_ctx* c, const revffn_merged* m) {
  if (!m) return REVFFN_ENULL;
  if (c->cfg.symmetric) return REVFFN_EUNSUPPORTED;
  if (!m->wq || !m->wk || !m->wv || !m->wo || !m->w_gate_up || !m->w_down || !m->w_router) return REVFFN_ENULL;
  if (c->cfg.d_shared && (!m->ws_gate_up || !m->ws_down)) return REVFFN_ENULL;
  return 0;
}

int check_call(revffn_ctx* c, const revffn_weights* w, int B, int S, i64 ld) {
  if (!c || !w) return REVFFN_ENULL;
  c->fold_queued = false;
  c->fwd_x1 = nullptr;                    // any call invalidates the activations a forward call left behind
  if (B < 1 || S < 1) return REVFFN_ESHAPE;
  if ((i64)B * S > c->maxT) return REVFFN_ESHAPE;
  if (ld < c->cfg.d_model / 2) return REVFFN_ESHAPE;
  if (!w->norm_a1 || !w->norm_a2 || !w->norm_m || !w->pup_a || !w->pdn_a || !w->pup_m || !w->pdn_m || !w->wq ||
      !w->wk || !w->wv || !w->wo || !w->w_router || !w->w_gate_up || !w->w_down)
    return REVFFN_ENULL;
  if (c->cfg.d_shared && (!w->ws_gate_up || !w->ws_down || !w->ws_gate)) return REVFFN_ENULL;
  return 0;
}

int forward_impl(revffn_ctx* c, const revffn_weights* w, const void* x1, const void* x2, void* y1, void* y2, int B,
                 int S, i64 ld, hipStream_t s) {
  const int T = B * S;
  router_fold(c, w, s);
  TRY(attn_acts(c, w, x1, ld, x2, ld, B, S, true, s));
  TRY(attn_out(c, w, x1, ld, 1.f, y1, ld, T, s));                 // Eq. 1
  TRY(moe_acts(c, w, y1, ld, T, s));
  TRY(moe_out(c, w, x2, ld, 1.f, y2, ld, T, s));                  // Eq. 2
  return 0;
}

// y1k/ldk: where the exact Y1 stays readable during and after the call (== y1 unless in place)
int inverse_impl(revffn_ctx* c, const revffn_weights* w, const void* y1, const void* y2, void* x1, void* x2, int B,
                 int S, i64 ld, float* residual, hipStream_t s, const void** y1_kept, i64* ld_kept,
                 hipStream_t s_attn = nullptr, hipStream_t* s_attn_used = nullptr) {
  const int T = B * S, h = c->cfg.d_model / 2, dt = c->dt;
  const bool sym = c->cfg.symmetric != 0;  // closed-form inverse: one evaluation of the branch at X2^, no iteration
  const bool conv = !sym && c->inv_tol > 0.f;      // stop on the residual instead of after a fixed count
  const int n = sym ? 1 : conv ? c->inv_max_iters : c->cfg.n_inv_iters;
  const void* y1k = y1;
  i64 ldk = ld;
  if (x1 == y1 && (n >= 1)) {             // in place: Y1 is needed after x1 starts being overwritten
    p_copy_rows(c, c->sdt, y1, ld, c->y1c, h, T, h, s);
    y1k = c->y1c;
    ldk = h;
  }
  const unsigned char* skip = nullptr;
  if (conv) {
    // the stopping rule runs on the device: row marks, per-block residuals and counts start at zero (a fill kernel,
    // so that the call can be captured into a graph)
    c->conv.S = S;
    c->conv.bp = c->inv_block;
    c->conv.nj = c->inv_block > 0 ? (S + c->inv_block - 1) / c->inv_block : 1;
    c->conv.nblk = c->inv_block > 0 ? B * c->conv.nj : 1;
    c->conv_last_nblk = c->conv.nblk;
    launch_fill_u32((uint32_t*)c->conv.row_done, 0, (int)c->conv_zero_words, s);
    skip = c->conv.row_done;
  }
  // the first fixed-point iterate is Y1 itself, so its query side does not wait for X2^: it fills the main stream
  // while the routing chain runs
  TRY(moe_acts(c, w, y1k, ldk, T, s, (n >= 1 && !sym) ? y1k : nullptr, ldk, B, S, skip));
  TRY(moe_out(c, w, y2, ld, -1.f, x2, ld, T, s));                 // X2^ = Y2 - MoE branch(Y1)
  if (n == 0) {
    if (x1 != y1) p_copy_rows(c, c->sdt, y1, ld, x1, ld, T, h, s);
    if (residual) launch_fill_u32((uint32_t*)residual, 0, 1, s);
  }
  // The iteration needs X2^ and nothing else of the MoE half.  A caller that goes on with work that does not need X1^
  // (the fused sweep step: the MoE half's backward pass) hands over a stream of its own for it and joins that stream
  // itself, where X1^ is first needed.
  hipStream_t sa = s;
  if (s_attn && c->use_streams && n >= 1) { sa = s_attn; after(c, s, sa); }
  if (s_attn_used) *s_attn_used = sa;     // == s: nothing was left on another stream
  for (int it = 1; it <= n; it++) {
    const void* xin = (it == 1) ? y1k : x1;                       // iterate, started at Y1
    i64 ldin = (it == 1) ? ldk : ld;
    TRY(attn_acts(c, w, xin, ldin, x2, ld, B, S, it == 1, sa, it == 1 && !sym, skip));   // K, V depend on X2^ only: once
    if (sym && residual) launch_fill_u32((uint32_t*)residual, 0, 1, sa);    // nothing is iterated: residual 0
    if (conv) {
      // every iteration up to the cap is enqueued; workgroups whose rows have all met the tolerance exit at once,
      // and the update below touches the other rows only.  The host takes no part in the decision.
      TRY(attn_out(c, w, y1k, ldk, -1.f, c->xtmp, h, T, sa, skip));
      launch_conv_update(c->sdt, c->xtmp, h, xin, ldin, x1, ld, c->conv, T, h, sa);
      launch_conv_decide(c->conv, T, c->inv_tol, it, sa);
    } else if (!sym && it == n && residual) {
      TRY(attn_out(c, w, y1k, ldk, -1.f, c->xtmp, h, T, sa));
      launch_fill_u32((uint32_t*)residual, 0, 1, sa);
      launch_absdiff_max_copy(c->sdt, c->xtmp, h, xin, ldin, x1, ld, residual, T, h, sa);
    } else {
      TRY(attn_out(c, w, y1k, ldk, -1.f, x1, ld, T, sa));         // x <- Y1 - attention branch(x, X2^)
    }
  }
  if (conv) launch_conv_finalize(c->conv, residual, sa);
  if (y1_kept) { *y1_kept = y1k; *ld_kept = ldk; }
  return 0;
}

void* gfield(const revffn_grads* g, size_t off) { return g ? *(void* const*)((const char*)g + off) : nullptr; }
#define GF(name) gfield(g, offsetof(revffn_grads, name))

int backward_impl(revffn_ctx* c, const revffn_weights* w, const void* x1, const void* x2, const void* y1, i64 ldy,
                  const void* dy1, const void* dy2, void* dx1, void* dx2, const revffn_grads* g, int B, int S,
                  i64 ld, bool reuse_moe, bool reuse_kv, hipStream_t s, bool reuse_attn = false,
                  hipStream_t s_attn = nullptr) {
  const revffn_config& f = c->cfg;
  const int T = B * S, d = f.d_model, h = d / 2, E = f.n_experts, k = f.top_k, I = f.d_expert, Is = f.d_shared;
  const int N = T * k, E1 = E + (Is ? 1 : 0), dt = c->dt, es = c->es;
  // ---- recompute the attention half at (x1, x2)
  // (K, V and the normalised, lifted X2 are still those of the inverse when it ran in the same call: same X2 bits)
  // The MoE half's backward pass needs dY2, Y1 and the MoE activations only; the attention half is recomputed beside
  // it on a stream of its own (sa) and joined where its activations are first used.  (With y1 == NULL the MoE half
  // needs the recomputed Y1 first: one stream.)  s_attn: the stream the caller's inverse left X1^ on.
  hipStream_t sa = s;
  if (y1 && c->use_streams && !reuse_attn) {
    sa = s_attn ? s_attn : c->side[3];
    if (!s_attn) after(c, s, sa);
  } else if (s_attn && s_attn != s) {
    after(c, s_attn, s);                  // no overlap in this call: X1^ is needed on s from here on
  }
  if (!y1 || !reuse_moe) router_fold(c, w, s);
  if (!reuse_attn) TRY(attn_acts(c, w, x1, ld, x2, ld, B, S, !reuse_kv, sa));
  if (!y1) {
    TRY(attn_out(c, w, x1, ld, 1.f, c->y1c, h, T, s));
    y1 = c->y1c;
    ldy = h;
    reuse_moe = false;
  }
  // ---- recompute the MoE half at the exact y1
  if (!reuse_moe) TRY(moe_acts(c, w, y1, ldy, T, s));
  // ---- MoE half backward: Y2 = X2 + P_dn_m(RS)
  // sw: weight gradients of the MoE half (leaves of the graph, joined at the very end); s0: shared-expert branch,
  // then the weight gradients of the attention half
  hipStream_t sw = side(c, s, 1), s0 = side(c, s, 0);
  if (GF(pdn_m)) {
    // reads dy2: stays on the caller's stream when dx2 aliases dy2 (dx2 is written at the very end)
    hipStream_t sp = (dx2 == dy2) ? s : sw;
    after(c, s, sp);
    TRY(run_wgrad(c, tn(dy2, ld, c->RS, d, GF(pdn_m), d, h, d, T), sp));
  }
  TRY(run_gemm(c, nn(dy2, ld, w->pdn_m, d, c->dRS, d, T, d, h), s));
  p_moe_bwd_rows(c, dt, c->dRS, c->Yp, c->Ys, c->inv_map, c->wts, c->gamma, c->dYp, c->dYs, c->dw, c->dzext, T, d,
                      k, E1, Is ? 1 : 0, s);
  if (Is) {
    after(c, s, s0);
    if (GF(ws_down)) { after(c, s, sw); TRY(run_wgrad(c, tn(c->dYs, d, c->Hs, Is, GF(ws_down), Is, d, Is, T), sw)); }
    TRY(run_gemm(c, nn(c->dYs, d, w->ws_down, Is, c->dHs, Is, T, Is, d), s0));
    p_swiglu_bwd(c, dt, c->dHs, c->GUs, c->dGUs, T, Is, s0);
    if (GF(ws_gate_up)) {
      after(c, s0, sw);
      TRY(run_wgrad(c, tn(c->dGUs, 2 * Is, c->Um, d, GF(ws_gate_up), d, 2 * Is, d, T), sw));
    }
    TRY(run_gemm(c, nn(c->dGUs, 2 * Is, w->ws_gate_up, d, c->dUm_sh, d, T, d, 2 * Is), s0));
  }
  {
    if (GF(w_down)) {
      after(c, s, sw);
      GemmArgs b = tn(c->dYp, d, c->Hh, I, GF(w_down), I, d, I, N);        // dWd_e = dYp_e^T . Hh_e
      b.group_mode = 2; b.n_groups = E; b.offsets = c->offsets; b.tile_count = c->tile_cnt + 3; b.c_group_stride = (i64)d * I;
      TRY(run_wgrad(c, b, sw));
    }
    GemmArgs a = nn(c->dYp, d, w->w_down, I, c->dHh, I, N, I, d);          // dHh = dYp . Wd_e
    a.group_mode = 1; a.n_groups = E; a.offsets = c->offsets; a.b_group_stride = (i64)d * I;
    TRY(run_gemm(c, a, s));
    p_swiglu_bwd(c, dt, c->dHh, c->GU, c->dGU, N, I, s);
    if (GF(w_gate_up)) {
      // dWgu_e = dGU_e^T . Xg_e, with the permuted input rows Xg materialised once
      after(c, s, sw);
      p_gather_rows(c, dt, c->Um, c->row_map, k, c->Xg, N, d, sw);
      GemmArgs b = tn(c->dGU, 2 * I, c->Xg, d, GF(w_gate_up), d, 2 * I, d, N);
      b.group_mode = 2; b.n_groups = E; b.offsets = c->offsets; b.tile_count = c->tile_cnt + 3; b.c_group_stride = (i64)2 * I * d;
      TRY(run_wgrad(c, b, sw));
    }
    GemmArgs e = nn(c->dGU, 2 * I, w->w_gate_up, d, c->dXg, d, N, d, 2 * I);     // dXg = dGU . Wgu_e
    e.group_mode = 1; e.n_groups = E; e.offsets = c->offsets; e.b_group_stride = (i64)2 * I * d;
    TRY(run_gemm(c, e, s));
  }
  // (the bf16 copy of the logit gradients for the matrix-core router GEMM below is written by the same kernel)
  const bool dz_bf16 = dt == 1 && c->mode == 0;
  const int E1p = (E1 + 7) / 8 * 8;
  p_router_bwd(c, c->probs, c->idx, c->wts, c->dw, c->dzext, T, E, k, E1, f.norm_topk_prob, s,
                    dz_bf16 ? c->dzb : nullptr, E1p);
  // every column sum (bias and gain gradients) goes to helper stream 2: they share one scratch buffer, and the
  // weight-gradient GEMMs keep helper stream 1 to themselves.  The router weight gradient goes there too.
  hipStream_t sc = side(c, s, 2);
  if (GF(w_router) || (Is && GF(ws_gate)) || (g && g->b_router)) after(c, s, sc);
  if (GF(w_router) || (Is && GF(ws_gate))) {
    // [dW_r ; dw_shared_gate] = dzext^T . Um in one fp32-A split-k GEMM, then the rows go to their buffers
    GemmArgs a = tn(c->dzext, E1, c->Um, d, c->dwr_tmp, d, E1, d, T);
    a.split_k = SPLIT_DWR; a.splitk_ws = c->splitk_ws;
    GemmTypes t{0, dt, c->gdt, dt};
    if (launch_gemm_generic(a, t, sc)) return REVFFN_EUNSUPPORTED;
    if (GF(w_router)) p_copy_rows(c, c->gdt, c->dwr_tmp, d, GF(w_router), d, E, d, sc);
    if (Is && GF(ws_gate)) p_copy_rows(c, c->gdt, at(c->dwr_tmp, (size_t)E * d, c->ges), d, GF(ws_gate), d, 1, d, sc);
  }
  if (g && g->b_router) p_colsum(c, 0, c->dzext, E1, 0, nullptr, 0, nullptr, 0, g->b_router, c->partial, T, E, sc);
  if (Is) after(c, s0, s);
  const void* dum_r = nullptr;
  if (dz_bf16) {
    // router term of dUm on the matrix cores: dUm_r = dz . [W_r ; w_gate ; 0], contraction over E1p
    GemmArgs a = nn(c->dzb, E1p, c->wr_ext, d, c->dUm_r, d, T, d, E1p);
    GemmTypes tt{1, 1, 1, 1};
    if (launch_gemm_mfma(a, tt, s) == 0) dum_r = c->dUm_r;
  }
  p_dum_finalize(c, dt, c->dXg, c->inv_map, Is ? c->dUm_sh : nullptr, dum_r, c->dzext, w->w_router, w->ws_gate,
                      c->dUm, T, d, k, E, E1, s);
  if (GF(pup_m)) { after(c, s, sw); TRY(run_wgrad(c, tn(c->dUm, d, c->n3, h, GF(pup_m), h, d, h, T), sw)); }
  TRY(run_gemm(c, nn(c->dUm, d, w->pup_m, h, c->dn3, h, T, h, d), s));
  // g1 = dY1 + Norm'(dn3): total gradient at Y1
  p_rmsnorm_bwd(c, dt, c->sdt, c->dn3, h, y1, ldy, w->norm_m, dy1, ld, c->g1, h, c->rinv3, T, h, f.rms_eps, s);
  // ---- attention half backward: Y1 = X1 + P_dn_a(AO)
  if (sa != s) after(c, sa, s);           // the recomputed attention activations (and X1^ of a fused call)
  if (GF(norm_m)) { after(c, s, sc); p_colsum(c, c->sdt, y1, ldy, dt, c->dn3, h, c->rinv3, c->gdt, GF(norm_m), c->partial, T, h, sc); }
  if (GF(pdn_a)) { after(c, s, s0); TRY(run_wgrad(c, tn(c->g1, h, c->AO, d, GF(pdn_a), d, h, d, T), s0)); }
  TRY(run_gemm(c, nn(c->g1, h, w->pdn_a, d, c->dAO, d, T, d, h), s));
  if (GF(wo)) { after(c, s, s0); TRY(run_wgrad(c, tn(c->dAO, d, c->O, d, GF(wo), d, d, d, T), s0)); }
  TRY(run_gemm(c, nn(c->dAO, d, w->wo, d, c->dO, d, T, d, d), s));
  {
    // five S x S x dh products (scores, dP, dV, dQ, dK), halved by the causal mask
    double fl = 10.0 * B * (double)S * S * d * (f.causal ? 0.5 : 1.0), by = 8.0 * T * d * es;
    ProfScope ps(c, s, fl, by);
    bool done = false;
    if (dt == 1 && c->mode == 0)
      done = launch_attn_bwd_flash(c->Q, c->K, c->V, c->O, c->dO, c->lse, c->dvec, c->dQ, c->dK, c->dV, B, S,
                                   f.n_heads, f.head_dim, f.causal, s) == 0;
    if (!done)
      launch_attn_bwd_generic(dt, c->Q, c->K, c->V, c->O, c->dO, c->lse, c->dvec, c->dQ, c->dK, c->dV, B, S,
                              f.n_heads, f.head_dim, f.causal, s);
    ps.done(done ? KID_ATTN_BWD_FLASH : KID_ATTN_BWD_GENERIC);
  }
  if (f.use_rope) {
    p_rope(c, dt, c->dQ, c->rope_cs, T, S, f.n_heads, f.head_dim, -1.f, s, c->dK);   // both in one launch
  }
  const void* U1 = c->U12;
  const void* U2 = at(c->U12, (size_t)T * d, es);
  void* dU1 = c->dU12;
  void* dU2 = at(c->dU12, (size_t)T * d, es);
  const bool sym = f.symmetric != 0;
  after(c, s, s0);
  after(c, s, sc);
  // s0: dU1 next to dU2 on the main stream, then the projection weight gradients
  hipEvent_t du1_done = nullptr;
  if (!sym) {
    TRY(run_gemm(c, nn(c->dQ, d, w->wq, d, dU1, d, T, d, d), s0));
    du1_done = mark(c, s0);
  }
  {
    // the projection weight gradients asked for, as one launch (problems of one shape)
    GemmArgs wg[3];
    int nw = 0;
    if (GF(wq)) wg[nw++] = tn(c->dQ, d, sym ? U2 : U1, d, GF(wq), d, d, d, T);
    if (GF(wk)) wg[nw++] = tn(c->dK, d, U2, d, GF(wk), d, d, d, T);
    if (GF(wv)) wg[nw++] = tn(c->dV, d, U2, d, GF(wv), d, d, d, T);
    if (nw) wg[0].bulk = c->use_streams;
    TRY(run_gemm_multi(c, wg, nw, c->gdt, s0));
  }
  {
    // the three bias gradients (column sums of dQ, dK, dV) in one launch pair
    const void* ba[3]; void* bo[3]; i64 bl[3]; int nb = 0;
    if (GF(bq) && w->bq) { ba[nb] = c->dQ; bo[nb] = GF(bq); bl[nb++] = d; }
    if (GF(bk) && w->bk) { ba[nb] = c->dK; bo[nb] = GF(bk); bl[nb++] = d; }
    if (GF(bv) && w->bv) { ba[nb] = c->dV; bo[nb] = GF(bv); bl[nb++] = d; }
    p_colsum_batch(c, nb, dt, ba, bl, dt, nullptr, nullptr, nullptr, c->gdt, bo, T, d, sc);
  }
  TRY(run_gemm(c, nn(c->dK, d, w->wk, d, dU2, d, T, d, d), s));
  {
    GemmArgs a = nn(c->dV, d, w->wv, d, dU2, d, T, d, d);        // dU2 += dV . Wv
    a.resid = dU2; a.ldr = d; a.resid_sign = 1.f;
    TRY(run_gemm(c, a, s));
  }
  if (sym) {
    // the query path ends in stream 2 too: dU2 += dQ . Wq; stream 1 only carries the residual path
    GemmArgs a = nn(c->dQ, d, w->wq, d, dU2, d, T, d, d);
    a.resid = dU2; a.ldr = d; a.resid_sign = 1.f;
    TRY(run_gemm(c, a, s));
    void* n2 = at(c->n12, (size_t)T * h, es);
    void* dn2 = at(c->dn12, (size_t)T * h, es);
    if (GF(pup_a)) { after(c, s, s0); TRY(run_wgrad(c, tn(dU2, d, n2, h, GF(pup_a), h, d, h, T), s0)); }
    TRY(run_gemm(c, nn(dU2, d, w->pup_a, h, dn2, h, T, h, d), s));
    p_rmsnorm_bwd(c, dt, c->sdt, dn2, h, x2, ld, w->norm_a2, dy2, ld, dx2, ld, c->rinv + T, T, h, f.rms_eps, s);
    p_copy_rows(c, dt, c->g1, h, dx1, ld, T, h, s);              // dX1 = total gradient at Y1
    after(c, s, sc);
    if (GF(norm_a1)) launch_zero(c->gdt, GF(norm_a1), h, sc);          // stream 1 is not normalised in this block
    if (GF(norm_a2)) p_colsum(c, c->sdt, x2, ld, dt, dn2, h, c->rinv + T, c->gdt, GF(norm_a2), c->partial, T, h, sc);
    after(c, sw, s);
    after(c, s0, s);
    after(c, sc, s);
    return 0;
  }
  if (s0 != s) wait_for(s, du1_done);
  if (GF(pup_a)) { after(c, s, s0); TRY(run_wgrad(c, tn(c->dU12, d, c->n12, h, GF(pup_a), h, d, h, 2 * T), s0)); }
  TRY(run_gemm(c, nn(c->dU12, d, w->pup_a, h, c->dn12, h, 2 * T, h, d), s));
  // dX1 = g1 + Norm'(dn1);  dX2 = dY2 + Norm'(dn2)
  p_rmsnorm_bwd(c, dt, c->sdt, c->dn12, h, x1, ld, w->norm_a1, c->g1, h, dx1, ld, c->rinv, T, h, f.rms_eps, s);
  p_rmsnorm_bwd(c, dt, c->sdt, at(c->dn12, (size_t)T * h, es), h, x2, ld, w->norm_a2, dy2, ld, dx2, ld, c->rinv + T, T, h,
                     f.rms_eps, s);
  after(c, s, sc);
  {
    // the two gain gradients (sum over tokens of x * dn / rms) in one launch pair
    const void* ga[2]; const void* gb[2]; const float* gs[2]; void* go[2]; i64 gla[2], glb[2]; int ng = 0;
    if (GF(norm_a1)) { ga[ng] = x1; gb[ng] = c->dn12; gs[ng] = c->rinv; go[ng] = GF(norm_a1); gla[ng] = ld; glb[ng++] = h; }
    if (GF(norm_a2)) { ga[ng] = x2; gb[ng] = at(c->dn12, (size_t)T * h, es); gs[ng] = c->rinv + T; go[ng] = GF(norm_a2); gla[ng] = ld; glb[ng++] = h; }
    p_colsum_batch(c, ng, c->sdt, ga, gla, dt, gb, glb, gs, c->gdt, go, T, h, sc);
  }
  after(c, sw, s);                       // every weight gradient is complete for the caller's stream
  after(c, s0, s);
  after(c, sc, s);
  return 0;
}

}  // namespace

// ====================================================================================
extern "C" {

size_t revffn_workspace_bytes(const revffn_config* cfg, int32_t max_B, int32_t max_S) {
  if (check_cfg(cfg) || max_B < 1 || max_S < 1 || (long long)max_B * max_S > (1 << 24)) return 0;
  revffn_ctx tmp;
  tmp.cfg = *cfg;
  tmp.dt = cfg->dtype;
  tmp.es = cfg->dtype == REVFFN_BF16 ? 2 : 4;
  tmp.sdt = cfg->fp32_streams ? REVFFN_F32 : cfg->dtype;
  tmp.ses = tmp.sdt == REVFFN_BF16 ? 2 : 4;
  tmp.gdt = cfg->fp32_grads ? REVFFN_F32 : cfg->dtype;
  tmp.ges = tmp.gdt == REVFFN_BF16 ? 2 : 4;
  tmp.maxT = max_B * max_S;
  return carve(&tmp, nullptr);
}

void revffn_destroy(revffn_ctx* c);

int revffn_create(revffn_ctx** out, const revffn_config* cfg, int32_t max_B, int32_t max_S) {
  if (!out) return REVFFN_ENULL;
  *out = nullptr;
  int e = check_cfg(cfg);
  if (e) return e;
  if (max_B < 1 || max_S < 1 || (long long)max_B * max_S > (1 << 24)) return REVFFN_ESHAPE;
  revffn_ctx* c = new (std::nothrow) revffn_ctx;
  if (!c) return REVFFN_EWORKSPACE;
  memset(c, 0, sizeof(*c));
  c->prof = new (std::nothrow) std::vector<ProfRec>();
  c->ev_pool = new (std::nothrow) std::vector<hipEvent_t>();
  if (!c->prof || !c->ev_pool) { delete c->prof; delete c->ev_pool; delete c; return REVFFN_EWORKSPACE; }
  c->cfg = *cfg;
  c->dt = cfg->dtype;
  c->es = cfg->dtype == REVFFN_BF16 ? 2 : 4;
  c->sdt = cfg->fp32_streams ? REVFFN_F32 : cfg->dtype;
  c->ses = c->sdt == REVFFN_BF16 ? 2 : 4;
  c->gdt = cfg->fp32_grads ? REVFFN_F32 : cfg->dtype;
  c->ges = c->gdt == REVFFN_BF16 ? 2 : 4;
  c->maxT = max_B * max_S;
  c->slab_bytes = carve(c, nullptr);
  if (hipGetDevice(&c->device) != hipSuccess) { delete c->prof; delete c->ev_pool; delete c; return REVFFN_EHIP; }
  if (hipMalloc(&c->slab, c->slab_bytes) != hipSuccess) {
    (void)hipGetLastError();
    delete c->prof; delete c->ev_pool; delete c;
    return REVFFN_EWORKSPACE;
  }
  carve(c, (char*)c->slab);
  (void)hipMemset(c->wr_ext, 0, (size_t)((c->cfg.n_experts + (c->cfg.d_shared ? 1 : 0) + 7) / 8 * 8) * c->cfg.d_model * c->es);
  (void)hipMemset(c->conv.stats, 0, 4 * sizeof(int));
  c->use_streams = getenv("REVFFN_NO_STREAMS") == nullptr;
  { const char* e = getenv("REVFFN_EXPERT_TILE"); if (e && (atoi(e) == 256 || atoi(e) == 128)) c->expert_tile = atoi(e); }
  { const char* e = getenv("REVFFN_NO_FUSED_SWIGLU"); c->no_fused_swiglu = e && atoi(e) != 0; }
  { const char* e = getenv("REVFFN_EXPERT_NT"); if (e && atoi(e) >= 1 && atoi(e) <= 3) c->expert_nt = atoi(e); }
  { const char* e = getenv("REVFFN_EXPERT_NN"); if (e && atoi(e) >= 1 && atoi(e) <= 3) c->expert_nn = atoi(e); }
  c->sync_ev = new (std::nothrow) std::vector<hipEvent_t>();
  bool ok = c->sync_ev != nullptr;
  for (int i = 0; ok && i < 4; i++) ok = hipStreamCreateWithFlags(&c->side[i], hipStreamNonBlocking) == hipSuccess;
  for (int i = 0; ok && i < 96; i++) {
    hipEvent_t e;
    ok = hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
    if (ok) c->sync_ev->push_back(e);
  }
  if (!ok) { revffn_destroy(c); return REVFFN_EHIP; }
  // rotary table: cs[s][i] = (cos, sin)(s * theta^(-2i/dh)), built in double precision on the host.  One entry per
  // position a call may use: a call may put all maxT tokens into one sequence.
  const int half = cfg->head_dim / 2;
  std::vector<float> tab;
  try { tab.resize((size_t)c->maxT * half * 2); } catch (...) { revffn_destroy(c); return REVFFN_EWORKSPACE; }
  for (int sp = 0; sp < c->maxT; sp++)
    for (int i = 0; i < half; i++) {
      double ang = (double)sp * pow((double)cfg->rope_theta, -2.0 * i / (double)cfg->head_dim);
      tab[((size_t)sp * half + i) * 2 + 0] = (float)cos(ang);
      tab[((size_t)sp * half + i) * 2 + 1] = (float)sin(ang);
    }
  if (hipMemcpy(c->rope_cs, tab.data(), tab.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
    revffn_destroy(c);                      // streams, events and the workspace go with it
    return REVFFN_EHIP;
  }
  *out = c;
  return REVFFN_OK;
}

static void prof_clear(revffn_ctx* c) {
  for (auto& r : *c->prof) { c->ev_pool->push_back(r.a); c->ev_pool->push_back(r.b); }
  c->prof->clear();
}

void revffn_destroy(revffn_ctx* c) {
  if (!c) return;
  (void)hipDeviceSynchronize();          // helper streams may still hold work of the last call
  if (c->prof) {
    prof_clear(c);
    for (hipEvent_t e : *c->ev_pool) (void)hipEventDestroy(e);
    delete c->prof;
    delete c->ev_pool;
  }
  if (c->sync_ev) {
    for (hipEvent_t e : *c->sync_ev) (void)hipEventDestroy(e);
    delete c->sync_ev;
  }
  for (int i = 0; i < 4; i++) if (c->side[i]) (void)hipStreamDestroy(c->side[i]);
  if (c->slab) (void)hipFree(c->slab);
  delete c;
}

int revffn_profile_enable(revffn_ctx* c, int32_t on) {
  if (!c) return REVFFN_ENULL;
  prof_clear(c);
  c->prof_on = on != 0;
  return 0;
}

int revffn_profile_read(revffn_ctx* c, int32_t kid, double* ms_total, int64_t* launches, double* flops,
                        double* bytes) {
  if (!c) return REVFFN_ENULL;
  if (kid < 0 || kid >= KID_COUNT) return REVFFN_EINVAL;
  double ms = 0, fl = 0, by = 0;
  int64_t n = 0;
  for (auto& r : *c->prof) {
    if (r.kid != kid) continue;
    if (hipEventSynchronize(r.b) != hipSuccess) return REVFFN_EHIP;
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) return REVFFN_EHIP;
    ms += t; fl += r.flops; by += r.bytes; n++;
  }
  if (ms_total) *ms_total = ms;
  if (launches) *launches = n;
  if (flops) *flops = fl;
  if (bytes) *bytes = by;
  return 0;
}

const char* revffn_profile_kernel_name(int32_t kid) {
  return (kid >= 0 && kid < KID_COUNT) ? kid_names[kid] : nullptr;
}

int revffn_set_inv_iters(revffn_ctx* c, int32_t n) {
  if (!c) return REVFFN_ENULL;
  if (n < 0 || n > 1024) return REVFFN_EINVAL;
  c->cfg.n_inv_iters = n;
  return 0;
}
int revffn_set_inverse_tolerance_blocked(revffn_ctx* c, float tol, int32_t max_iters, int32_t block_positions) {
  if (!c) return REVFFN_ENULL;
  if (!(tol >= 0.f) || (tol > 0.f && (max_iters < 1 || max_iters > 1024)) || block_positions < 0) return REVFFN_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return REVFFN_EHIP;            // earlier inverses still update the statistics
  if (hipMemset(c->conv.stats, 0, 4 * sizeof(int)) != hipSuccess) return REVFFN_EHIP;
  c->inv_tol = tol;
  c->inv_max_iters = tol > 0.f ? max_iters : 0;
  c->inv_block = tol > 0.f ? block_positions : 0;
  c->conv_last_nblk = 0;
  return 0;
}
int revffn_set_inverse_tolerance(revffn_ctx* c, float tol, int32_t max_iters) {
  return revffn_set_inverse_tolerance_blocked(c, tol, max_iters, 0);
}
int revffn_get_inverse_stats(revffn_ctx* c, int64_t* calls, int64_t* iters_total, int32_t* last_iters,
                             float* last_residual) {
  if (!c) return REVFFN_ENULL;
  int st[4] = {0, 0, 0, 0};
  if (c->inv_tol > 0.f) {
    if (hipDeviceSynchronize() != hipSuccess) return REVFFN_EHIP;
    if (hipMemcpy(st, c->conv.stats, sizeof(st), hipMemcpyDeviceToHost) != hipSuccess) return REVFFN_EHIP;
  }
  float r;
  memcpy(&r, &st[3], sizeof(r));
  if (calls) *calls = st[0];
  if (iters_total) *iters_total = st[1];
  if (last_iters) *last_iters = st[2];
  if (last_residual) *last_residual = r;
  return 0;
}
int revffn_get_inverse_blocks(revffn_ctx* c, int32_t* iters, float* residuals, int32_t cap, int32_t* n_blocks) {
  if (!c) return REVFFN_ENULL;
  if (cap < 0) return REVFFN_EINVAL;
  const int n = c->inv_tol > 0.f ? c->conv_last_nblk : 0;
  if (n_blocks) *n_blocks = n;
  const int m = n < cap ? n : cap;
  if (m == 0) return 0;
  if (hipDeviceSynchronize() != hipSuccess) return REVFFN_EHIP;
  if (iters && hipMemcpy(iters, c->conv.blk_iters, (size_t)m * 4, hipMemcpyDeviceToHost) != hipSuccess) return REVFFN_EHIP;
  if (residuals && hipMemcpy(residuals, c->conv.blk_res, (size_t)m * 4, hipMemcpyDeviceToHost) != hipSuccess) return REVFFN_EHIP;
  return 0;
}
int revffn_enable_taps(revffn_ctx* c, int32_t on) {
  if (!c) return REVFFN_ENULL;
  c->taps = on ? 1 : 0;
  return 0;
}
int revffn_set_kernel_mode(revffn_ctx* c, int32_t mode) {
  if (!c) return REVFFN_ENULL;
  if (mode != 0 && mode != 1) return REVFFN_EINVAL;
  c->mode = mode;
  return 0;
}

int revffn_op_tile_placement(int32_t group_mode, int32_t tiles_m, int32_t tiles_n, int32_t bm, int32_t bn,
                             int32_t n_groups, const int32_t* tile_first, int32_t n_used, int32_t* out,
                             int32_t max_wg) {
  if (group_mode < 0 || group_mode > 2 || tiles_m < 1 || tiles_n < 1 || bm < 1 || bn < 1 || !out) return REVFFN_EINVAL;
  if (group_mode == 1 && (n_used < 0 || n_used > tiles_m)) return REVFFN_EINVAL;
  if (group_mode == 2 && n_groups < 1) return REVFFN_EINVAL;
  int xcd_m = 1;
  long long grid;
  if (group_mode == 0) { xcd_m = pick_xcd_m(tiles_m, tiles_n, bm, bn); grid = dense_grid_x(xcd_m, tiles_m, tiles_n); }
  else if (group_mode == 1) grid = (long long)tiles_n * tiles_m;
  else { xcd_m = 2; grid = wgrad_grid_x(xcd_m, tiles_m, tiles_n, n_groups); }
  if (grid > max_wg) return REVFFN_EINVAL;
  for (int i = 0; i < (int)grid; i++) {
    int bx = -1, by = -1, bz = 0;
    if (!place_tile(group_mode, xcd_m, tiles_m, tiles_n, n_groups, n_used, tile_first, i, &bx, &by, &bz)) bx = by = bz = -1;
    out[3 * i] = bx; out[3 * i + 1] = by; out[3 * i + 2] = bz;
  }
  return (int)grid;
}

int revffn_set_helper_streams(revffn_ctx* c, int32_t on) {
  if (!c) return REVFFN_ENULL;
  c->use_streams = on != 0;
  return 0;
}

int revffn_forward(revffn_ctx* c, const revffn_weights* w, const void* x1, const void* x2, void* y1, void* y2,
                   int32_t B, int32_t S, int64_t ld, void* stream) {
  TRY(check_call(c, w, B, S, ld));
  if (!x1 || !x2 || !y1 || !y2) return REVFFN_ENULL;
  TRY(finish(c, (hipStream_t)stream, forward_impl(c, w, x1, x2, y1, y2, B, S, ld, (hipStream_t)stream)));
  if (x1 != y1 && x2 != y2) { c->fwd_x1 = x1; c->fwd_x2 = x2; c->fwd_y1 = y1; c->fwd_B = B; c->fwd_S = S; c->fwd_ld = ld; }
  return 0;
}

int revffn_backward_stored(revffn_ctx* c, const revffn_weights* w, const void* x1, const void* x2, const void* y1,
                           const void* dy1, const void* dy2, void* dx1, void* dx2, const revffn_grads* g, int32_t B,
                           int32_t S, int64_t ld, void* stream) {
  if (!c) return REVFFN_ENULL;
  const bool match = c->fwd_x1 && c->fwd_x1 == x1 && c->fwd_x2 == x2 && c->fwd_y1 == y1 && c->fwd_B == B &&
                     c->fwd_S == S && c->fwd_ld == ld;
  TRY(check_call(c, w, B, S, ld));        // (also drops the stored state: it serves one backward call)
  if (!x1 || !x2 || !y1 || !dy1 || !dy2 || !dx1 || !dx2) return REVFFN_ENULL;
  if (!match) return REVFFN_EINVAL;
  if (dx1 == x1 || dx1 == x2 || dx2 == x1 || dx2 == x2 || dx1 == y1 || dx2 == y1) return REVFFN_EINVAL;
  return finish(c, (hipStream_t)stream,
                backward_impl(c, w, x1, x2, y1, ld, dy1, dy2, dx1, dx2, g, B, S, ld, true, true, (hipStream_t)stream, true));
}

int revffn_inverse(revffn_ctx* c, const revffn_weights* w, const void* y1, const void* y2, void* x1, void* x2,
                   int32_t B, int32_t S, int64_t ld, float* residual, void* stream) {
  TRY(check_call(c, w, B, S, ld));
  if (!x1 || !x2 || !y1 || !y2) return REVFFN_ENULL;
  return finish(c, (hipStream_t)stream,
                inverse_impl(c, w, y1, y2, x1, x2, B, S, ld, residual, (hipStream_t)stream, nullptr, nullptr));
}

int revffn_backward(revffn_ctx* c, const revffn_weights* w, const void* x1, const void* x2, const void* y1,
                    const void* dy1, const void* dy2, void* dx1, void* dx2, const revffn_grads* g, int32_t B,
                    int32_t S, int64_t ld, void* stream) {
  TRY(check_call(c, w, B, S, ld));
  if (!x1 || !x2 || !dy1 || !dy2 || !dx1 || !dx2) return REVFFN_ENULL;
  return finish(c, (hipStream_t)stream,
                backward_impl(c, w, x1, x2, y1, ld, dy1, dy2, dx1, dx2, g, B, S, ld, false, false, (hipStream_t)stream));
}

int revffn_inverse_backward(revffn_ctx* c, const revffn_weights* w, const void* y1, const void* y2, void* x1, void* x2,
                            const void* dy1, const void* dy2, void* dx1, void* dx2, const revffn_grads* g, int32_t B,
                            int32_t S, int64_t ld, float* residual, void* stream) {
  TRY(check_call(c, w, B, S, ld));
  if (!y1 || !y2 || !x1 || !x2 || !dy1 || !dy2 || !dx1 || !dx2) return REVFFN_ENULL;
  hipStream_t s = (hipStream_t)stream;
  const void* y1k = nullptr;
  i64 ldk = 0;
  hipStream_t sa = s;                     // the stream the inverse leaves X1^ on (helper stream 3 beside the MoE backward pass)
  TRY(finish(c, s, inverse_impl(c, w, y1, y2, x1, x2, B, S, ld, residual, s, &y1k, &ldk, c->side[3], &sa)));
  return finish(c, s, backward_impl(c, w, x1, x2, y1k, ldk, dy1, dy2, dx1, dx2, g, B, S, ld, true, c->cfg.n_inv_iters >= 1, s,
                                    false, sa == s ? nullptr : sa));
}

int revffn_merge_adapters(revffn_ctx* c, const revffn_weights* w, const revffn_merged* m, void* stream) {
  TRY(check_call(c, w, 1, 1, c ? c->cfg.d_model / 2 : 0));
  TRY(check_merged(c, m));
  return finish(c, (hipStream_t)stream, merge_impl(c, w, m, (hipStream_t)stream));
}

int revffn_forward_merged(revffn_ctx* c, const revffn_weights* w, const revffn_merged* m, const void* x1, const void* x2,
                          void* y1, void* y2, int32_t B, int32_t S, int64_t ld, void* stream) {
  TRY(check_call(c, w, B, S, ld));
  TRY(check_merged(c, m));
  if (!x1 || !x2 || !y1 || !y2) return REVFFN_ENULL;
  hipStream_t s = (hipStream_t)stream;
  const int T = B * S;
  TRY(finish(c, s, attn_acts_merged(c, w, m, x1, ld, x2, ld, B, S, true, s)));
  TRY(finish(c, s, attn_out_merged(c, m, x1, ld, 1.f, y1, ld, T, s)));                 // Eq. 1
  return finish(c, s, moe_merged(c, w, m, y1, ld, x2, ld, 1.f, y2, ld, T, s));         // Eq. 2
}

int revffn_inverse_merged(revffn_ctx* c, const revffn_weights* w, const revffn_merged* m, const void* y1, const void* y2,
                          void* x1, void* x2, int32_t B, int32_t S, int64_t ld, float* residual, void* stream) {
  TRY(check_call(c, w, B, S, ld));
  TRY(check_merged(c, m));
  if (!x1 || !x2 || !y1 || !y2) return REVFFN_ENULL;
  hipStream_t s = (hipStream_t)stream;
  const int T = B * S, h = c->cfg.d_model / 2, n = c->cfg.n_inv_iters;
  const void* y1k = y1;
  i64 ldk = ld;
  if (x1 == y1 && n >= 1) {               // in place: Y1 is needed after x1 starts being overwritten
    p_copy_rows(c, c->sdt, y1, ld, c->y1c, h, T, h, s);
    y1k = c->y1c;
    ldk = h;
  }
  TRY(finish(c, s, moe_merged(c, w, m, y1k, ldk, y2, ld, -1.f, x2, ld, T, s)));        // X2^ = Y2 - MoE branch(Y1)
  if (n == 0) {
    if (x1 != y1) p_copy_rows(c, c->sdt, y1, ld, x1, ld, T, h, s);
    if (residual) launch_fill_u32((uint32_t*)residual, 0, 1, s);
  }
  for (int it = 1; it <= n; it++) {
    const void* xin = (it == 1) ? y1k : x1;
    const i64 ldin = (it == 1) ? ldk : ld;
    TRY(finish(c, s, attn_acts_merged(c, w, m, xin, ldin, x2, ld, B, S, it == 1, s)));  // K, V depend on X2^ only: once
    if (it == n && residual) {
      TRY(finish(c, s, attn_out_merged(c, m, y1k, ldk, -1.f, c->xtmp, h, T, s)));
      launch_fill_u32((uint32_t*)residual, 0, 1, s);
      launch_absdiff_max_copy(c->sdt, c->xtmp, h, xin, ldin, x1, ld, residual, T, h, s);
    } else {
      TRY(finish(c, s, attn_out_merged(c, m, y1k, ldk, -1.f, x1, ld, T, s)));          // x <- Y1 - attention branch(x, X2^)
    }
  }
  return 0;
}

int revffn_stack_forward(revffn_ctx* c, const revffn_weights* w, int32_t n_blocks, const void* x1, const void* x2,
                         void* y1, void* y2, int32_t B, int32_t S, int64_t ld, void* stream) {
  if (n_blocks < 1) return REVFFN_EINVAL;
  if (!c || !w) return REVFFN_ENULL;
  for (int l = 0; l < n_blocks; l++) TRY(check_call(c, w + l, B, S, ld));
  if (!x1 || !x2 || !y1 || !y2) return REVFFN_ENULL;
  for (int l = 0; l < n_blocks; l++) {
    TRY(finish(c, (hipStream_t)stream, forward_impl(c, w + l, l == 0 ? x1 : y1, l == 0 ? x2 : y2, y1, y2, B, S, ld, (hipStream_t)stream)));
  }
  return 0;
}

int revffn_stack_backward(revffn_ctx* c, const revffn_weights* w, const revffn_grads* g, int32_t n_blocks, void* y1,
                          void* y2, void* dy1, void* dy2, int32_t B, int32_t S, int64_t ld, void* stream) {
  if (n_blocks < 1) return REVFFN_EINVAL;
  if (!c || !w) return REVFFN_ENULL;
  for (int l = 0; l < n_blocks; l++) TRY(check_call(c, w + l, B, S, ld));
  if (!y1 || !y2 || !dy1 || !dy2) return REVFFN_ENULL;
  hipStream_t s = (hipStream_t)stream;
  for (int l = n_blocks - 1; l >= 0; l--) {
    // rebuild this block's input in place; the exact Y1 survives in the workspace copy, and the MoE
    // activations computed at it by the inverse are reused by the backward pass
    const void* y1k = nullptr;
    i64 ldk = 0;
    hipStream_t sa = s;
    TRY(finish(c, s, inverse_impl(c, w + l, y1, y2, y1, y2, B, S, ld, nullptr, s, &y1k, &ldk, c->side[3], &sa)));
    TRY(finish(c, s, backward_impl(c, w + l, y1, y2, y1k, ldk, dy1, dy2, dy1, dy2, g ? g + l : nullptr, B, S, ld, true, c->cfg.n_inv_iters >= 1, s,
                                   false, sa == s ? nullptr : sa)));
  }
  return 0;
}

int revffn_get_routing(revffn_ctx* c, int32_t* idx, float* wts, int32_t* counts, int32_t* offsets, int32_t* row_map,
                       void* stream) {
  if (!c) return REVFFN_ENULL;
  if (c->lastT <= 0) return REVFFN_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const size_t N = (size_t)c->lastT * c->cfg.top_k, E = c->cfg.n_experts;
  hipError_t e = hipSuccess;
  if (idx && e == hipSuccess) e = hipMemcpyAsync(idx, c->idx, N * 4, hipMemcpyDeviceToDevice, s);
  if (wts && e == hipSuccess) e = hipMemcpyAsync(wts, c->wts, N * 4, hipMemcpyDeviceToDevice, s);
  if (counts && e == hipSuccess) e = hipMemcpyAsync(counts, c->counts, E * 4, hipMemcpyDeviceToDevice, s);
  if (offsets && e == hipSuccess) e = hipMemcpyAsync(offsets, c->offsets, (E + 1) * 4, hipMemcpyDeviceToDevice, s);
  if (row_map && e == hipSuccess) e = hipMemcpyAsync(row_map, c->row_map, N * 4, hipMemcpyDeviceToDevice, s);
  return e == hipSuccess ? 0 : REVFFN_EHIP;
}

int revffn_get_branch(revffn_ctx* c, int32_t which, float* dst, void* stream) {
  if (!c || !dst) return REVFFN_ENULL;
  if (!c->taps || c->lastT <= 0 || (which != 0 && which != 1)) return REVFFN_EINVAL;
  size_t bytes = (size_t)c->lastT * (c->cfg.d_model / 2) * 4;
  hipError_t e = hipMemcpyAsync(dst, which == 0 ? c->tapA : c->tapM, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream);
  return e == hipSuccess ? 0 : REVFFN_EHIP;
}

int revffn_op_gemm(int32_t dtype, int32_t kernel_mode, const void* a, const void* b, void* c, int32_t M, int32_t N,
                   int32_t K, int64_t lda, int64_t ldb, int64_t ldc, int32_t a_trans, int32_t b_trans,
                   int32_t out_f32, void* stream) {
  const int tile = kernel_mode >> 8;       // bits 8 and up: MFMA tile shape to force (1..4), 0 = chosen by size
  kernel_mode &= 0xff;
  if ((dtype != 0 && dtype != 1) || kernel_mode < 0 || kernel_mode > 2 || tile < 0 || tile > 4 || !a || !b || !c ||
      M < 1 || N < 1 || K < 0)
    return REVFFN_EINVAL;
  GemmArgs g = nt(a, lda, b, ldb, c, ldc, M, N, K);
  g.force_tile = tile;
  g.a_trans = a_trans ? 1 : 0;
  g.b_trans = b_trans ? 1 : 0;
  GemmTypes t{dtype, dtype, out_f32 ? 0 : dtype, dtype};
  if (dtype == 1 && kernel_mode != 1 && launch_gemm_mfma(g, t, (hipStream_t)stream) == 0) return 0;
  if (kernel_mode == 2) return REVFFN_EUNSUPPORTED;
  return launch_gemm_generic(g, t, (hipStream_t)stream) == 0 ? 0 : REVFFN_EUNSUPPORTED;
}

int revffn_op_attention_fwd(int32_t dtype, int32_t kernel_mode, const void* q, const void* k, const void* v, void* o,
                            float* lse, int32_t B, int32_t S, int32_t H, int32_t dh, int32_t causal, void* stream) {
  if ((dtype != 0 && dtype != 1) || kernel_mode < 0 || kernel_mode > 2 || !q || !k || !v || !o || !lse || B < 1 ||
      S < 1 || H < 1 || dh < 2 || dh > 1024)
    return REVFFN_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (dtype == 1 && kernel_mode != 1 && launch_attn_fwd_flash(q, k, v, o, lse, B, S, H, dh, causal, s) == 0) return 0;
  if (kernel_mode == 2) return REVFFN_EUNSUPPORTED;
  launch_attn_fwd_generic(dtype, q, k, v, o, lse, B, S, H, dh, causal, s);
  return 0;
}

int revffn_op_attention_bwd(int32_t dtype, int32_t kernel_mode, const void* q, const void* k, const void* v,
                            const void* o, const void* d_o, const float* lse, float* dvec, void* dq, void* dk, void* dv,
                            int32_t B, int32_t S, int32_t H, int32_t dh, int32_t causal, void* stream) {
  if ((dtype != 0 && dtype != 1) || kernel_mode < 0 || kernel_mode > 2 || !q || !k || !v || !o || !d_o || !lse ||
      !dvec || !dq || !dk || !dv || B < 1 || S < 1 || H < 1 || dh < 2 || dh > 1024)
    return REVFFN_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (dtype == 1 && kernel_mode != 1 &&
      launch_attn_bwd_flash(q, k, v, o, d_o, lse, dvec, dq, dk, dv, B, S, H, dh, causal, s) == 0)
    return 0;
  if (kernel_mode == 2) return REVFFN_EUNSUPPORTED;
  launch_attn_bwd_generic(dtype, q, k, v, o, d_o, lse, dvec, dq, dk, dv, B, S, H, dh, causal, s);
  return 0;
}

// ---- the entry point that allocates nothing -----------------------------------------------------------------
// The row-dot scratch of the attention backward (D[b, head, s] = <dO, O>, float) lives in a file-scope device array
// instead of a caller buffer.  In host code the array's name is only a handle: the device address is looked up once
// per device with hipGetSymbolAddress and kept, and only that pointer is ever handed to a kernel.
#define REVFFN_NOALLOC_MAX_ROWS (1 << 20)
static __device__ __align__(256) float scratch[REVFFN_NOALLOC_MAX_ROWS];
#define REVFFN_MAX_DEVICES 64
static float* scratch_ptr[REVFFN_MAX_DEVICES];          // per device: address of that device's copy of `scratch`
static std::mutex scratch_mu;

int revffn_op_attention_bwd_noalloc(int32_t dtype, int32_t kernel_mode, const void* q, const void* k, const void* v,
                                    const void* o, const void* d_o, const float* lse, void* dq, void* dk, void* dv,
                                    int32_t B, int32_t S, int32_t H, int32_t dh, int32_t causal, void* stream) {
  if ((dtype != 0 && dtype != 1) || kernel_mode < 0 || kernel_mode > 2 || !q || !k || !v || !o || !d_o || !lse ||
      !dq || !dk || !dv || B < 1 || S < 1 || H < 1 || dh < 2 || dh > 1024)
    return REVFFN_EINVAL;
  if ((long long)B * H * S > REVFFN_NOALLOC_MAX_ROWS) return REVFFN_ESHAPE;   // beyond the static scratch
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return REVFFN_EHIP;
  if (dev < 0 || dev >= REVFFN_MAX_DEVICES) return REVFFN_EUNSUPPORTED;
  float* dvec;
  {
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return REVFFN_EHIP; }
      scratch_ptr[dev] = (float*)p;
    }
    dvec = scratch_ptr[dev];
  }
  // every element of dvec that the kernels read is written first by the row-dot kernel of the same call, so nothing
  // of an earlier call's contents needs clearing
  return revffn_op_attention_bwd(dtype, kernel_mode, q, k, v, o, d_o, lse, dvec, dq, dk, dv, B, S, H, dh, causal, stream);
}

const char* revffn_strerror(int code) {
  switch (code) {
    case REVFFN_OK: return "ok";
    case REVFFN_EINVAL: return "invalid configuration value";
    case REVFFN_ESHAPE: return "batch, sequence length or row stride out of range for this context";
    case REVFFN_ENULL: return "required pointer is NULL";
    case REVFFN_EWORKSPACE: return "workspace allocation failed";
    case REVFFN_EHIP: return "HIP runtime call failed";
    case REVFFN_EUNSUPPORTED: return "request not implemented by this build";
    default: return "unknown error";
  }
}

}  // extern "C"
