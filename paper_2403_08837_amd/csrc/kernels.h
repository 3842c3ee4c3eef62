// Kernel-side interface of libcdp: problem descriptors handed to the grouped kernels by
// value (kernel arguments), and the host launch functions.  Device pointers only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstddef>
#include <string>

namespace cdp {

// Text for cdp_last_error(NULL) (thread-local), set by entry points that have no context.
void set_global_error(const std::string& msg);

enum DType : int { DT_F32 = 0, DT_BF16 = 1 };

// ---------------------------------------------------------------------------------
// Grouped GEMM.  Every contraction of a tick (Linear or convolution; forward, data
// gradient, weight gradient) is C[r][c] = sum_k A[r][k] * B[c][k] over *virtual*
// operand matrices.  An operand is either a plain matrix or an on-the-fly im2col view
// of an NHWC tensor, and is stored either k-contiguous or row-contiguous in memory.
// ---------------------------------------------------------------------------------
enum OperandMode : int {
  OP_PLAIN_K = 0,  // ptr[r*ld + k]                      (k contiguous)
  OP_PLAIN_R = 1,  // ptr[k*ld + r]                      (r contiguous)
  OP_CONV_FWD = 2, // r = (b,oh,ow), k = (kh,kw,c):  src[b][oh*s-p+kh][ow*s-p+kw][c]
  OP_CONV_DGRAD = 3, // r = (b,ih,iw), k = (kh,kw,o): src[b][(ih+p-kh)/s][(iw+p-kw)/s][o]
  OP_CONV_WGRAD = 4  // r = (kh,kw,c), k = (b,oh,ow): src[b][oh*s-p+kh][ow*s-p+kw][c]
};

struct ConvGeom {
  int H, W, C;    // gathered source tensor [*, H, W, C]
  int OH, OW;     // spatial extent of the position index (b, oh, ow)
  int KH, KW, stride, pad;
};

enum EpilogueKind : int {
  EPI_FWD = 0,    // out = act(acc + bias[c] + res[r][c])            -> T or f32
  EPI_DGRAD = 1,  // out = mask(acc + add[r][c] (+ out_old))         -> T
  EPI_WGRAD = 2   // G[r][c] (+)= gamma[r] * acc ; Ggamma[r] += sum_c acc * Wplain[r][c]
};

struct GemmProb {
  const void* A;
  const void* B;
  void* out;
  const void* aux0;  // FWD: bias f32[c]   DGRAD: add T[r][c]      WGRAD: gamma f32[r]
  const void* aux1;  // FWD: res T[r][c]   DGRAD: mask T[r][c]     WGRAD: Wplain T[r][c]
  void* aux2;        //                                            WGRAD: Ggamma f32[r]
  void* aux3;        //                                            WGRAD (conv fast path): partial dy column sums
  int M, N, K;       // C is M x N, reduction length K
  int lda, ldb, ldo; // leading dims for plain operands / output / aux matrices
  int a_mode, b_mode;
  int epi;
  int flags;         // bit0 relu, bit1 out_f32, bit2 accumulate (DGRAD: += out_old;
                     // WGRAD: beta = 1), bit3 atomic (WGRAD)
  int tiles_n;       // tiles along N
  int splits;        // split-K factor (WGRAD atomic only), >= 1
  int tile_begin;    // first block of this problem in the launch
  int upd;           // linear_tick_kernel, WGRAD: 1 + index into GemmBatch::upd of a fused SGD step, 0 = none
  ConvGeom g;        // geometry of the (single) gathered operand, if any
};
static_assert(sizeof(ConvGeom) >= 36, "group pointers of a deferred weight gradient are kept in the geometry block");

// Weight gradient of a Linear layer over a GROUP of micro-batches (GF_GROUP): G (+)= sum_m dY_m^T X_m in one
// pass over the accumulator, members m = 0 .. nmem-1 (nmem <= DW_GROUP_MAX) of `rows` rows each.  Member 0 is
// (A, B); the further members' (dY, X) pointers travel in fields a Linear weight gradient does not use:
// (aux0, aux1), then four pointers laid over the geometry block; g.pad holds `rows`.  P.K = nmem * rows.
constexpr int DW_GROUP_MAX = 4;
struct DwGroupView { const void* p[4]; int rows; };
static_assert(sizeof(DwGroupView) <= sizeof(ConvGeom) + 4 && offsetof(DwGroupView, rows) == offsetof(ConvGeom, pad), "layout of the overlay");
__host__ __device__ inline const void* dw_member(const GemmProb& P, int m, int which /*0: dY, 1: X*/) {
  if (m == 0) return which ? P.B : P.A;
  if (m == 1) return which ? P.aux1 : P.aux0;
  const void* const* q = reinterpret_cast<const void* const*>(&P.g);
  return q[(m - 2) * 2 + which];
}
__host__ inline void dw_set_member(GemmProb& P, int m, const void* dy, const void* x) {
  if (m == 0) { P.A = dy; P.B = x; }
  else if (m == 1) { P.aux0 = dy; P.aux1 = x; }
  else { const void** q = reinterpret_cast<const void**>(&P.g); q[(m - 2) * 2] = dy; q[(m - 2) * 2 + 1] = x; }
}

enum : int {
  GF_RELU = 1, GF_OUT_F32 = 2, GF_ACCUM = 4, GF_ATOMIC = 8,
  GF_THIN = 16,  // set by launch_linear_tick
  GF_A_F32 = 32, // linear_tick_kernel, forward: A holds fp32 values, rounded to the compute type on load
  GF_GROUP = 128, // linear_tick_kernel, WGRAD: operands of several micro-batches (DwGroupView)
  GF_CE = 64     // linear_tick_kernel, thin forward tile with N <= 32 classes: softmax cross-entropy in the epilogue
                 // (out = dlogits T[M][N], aux2 = int32 labels, aux3 = loss slots, g.H = rows per loss slot)
};

// SGD step on fp32 master parameters from the summed micro-batch gradients G (Eq. (CDP)),
// optionally with momentum and weight decay (the optimiser of Sec. 5 "Hyperparameters"):
//   g = G*inv_n + wd*w ;  v = momentum*v + g (when a velocity buffer is given) ;  w -= lr*v.
// apply == 0 leaves the parameters as they are (initial fill of the ring slots).
struct SgdParams { float lr, inv_n, momentum, wd; int apply; };

// SGD step of a Linear layer fused into the weight-gradient contraction that delivers the
// N-th micro-batch gradient of the step: the tile that completes sum_i g_i applies the step
// to its part of the fp32 master weights and writes the compute copies of the new version
// (forward layout wf[n][k] and data-gradient layout wt[k][n]) into the other ring slot.
// The accumulator is not written: the next step's first gradient overwrites it.
struct LinUpdate {
  float* master; float* V;                  // fp32 [N][K]; V = velocity or NULL
  void* wf; void* wt;                       // compute copies of the new version
  float* bmaster; float* bV; float* bcopy;  // bias: master, velocity or NULL, fp32 copy in the new slot (bmaster NULL: no bias)
  SgdParams sgd;
};

// Staging of a micro-batch that starts in this tick, carried by the tick's first Linear launch
// as extra tiles: fp32 -> T conversion of its rows, label copy, zeroing of its loss slots
// (what launch_stage_input does as a kernel of its own).
struct StageCopy {
  const float* x; const int32_t* y;  // caller's rows [rows][per_row] and labels [rows]
  void* xo; int32_t* yo;             // staged copies
  float* loss; int n_slots;          // loss slots to clear
  int rows; int64_t n;               // n = rows * per_row
};
constexpr int STAGE_COPY_ELEMS = 8192;  // elements per copy tile

constexpr int GEMM_MAX_PROBS = 24;
constexpr int LIN_UPD_MAX = 2;
struct GemmBatch {
  int n;
  int total_tiles;
  int head_tiles;  // linear_tick_kernel: tiles of the forward / data-gradient problems (listed first)
  int upd_tiles;   // linear_tick_kernel: tiles of the weight gradients with a fused SGD step (listed next)
  int n_upd;
  int copy_tiles;  // linear_tick_kernel: tiles of the staging copy `sc` (listed last), 0 = none
  // linear_tick_kernel: room for thin tiles that split a long reduction over several workgroups
  // (THIN_WS_SLOTS partial tiles of 32 x 32 floats and as many counters, which must be zero
  // before the launch and are zero again after it), or NULL: no thin tile is split.
  // conv_gemm_kernel: the same for the tiles of a small launch (CONV_SPLIT_WS_BYTES of partial
  // tiles, CONV_SPLIT_SLOTS counters)
  float* thin_ws;
  unsigned int* thin_cnt;
  int slot_floats;  // linear_tick_kernel: floats per partial-tile slot of this launch (set by launch_linear_tick)
  GemmProb p[GEMM_MAX_PROBS];
  LinUpdate upd[LIN_UPD_MAX];
  StageCopy sc;
};
static_assert(sizeof(GemmBatch) <= 4000, "kernel argument block must stay under 4 KiB");

// Tile shape variants (rows x cols of C per workgroup).
enum TileShape : int { TILE_128x128 = 0, TILE_64x128 = 1, TILE_64x64 = 2, TILE_COUNT = 3 };
void tile_dims(int shape, int* bm, int* bn);

// Fills tiles_n / tile_begin / total_tiles for the chosen tile shape and launches.
hipError_t launch_gemm_batch(GemmBatch& batch, int dtype, int tile_shape, hipStream_t stream);

// HBM-streaming variants for Linear layers with a small batch (plain operands only):
//   skinny: forward / data gradient, operands both k-contiguous; wide = 128-column tiles.
//   dw:     weight gradient G (+)= dY^T X with A = dY (OP_PLAIN_R), B = X (OP_PLAIN_R),
//           GF_ACCUM selects accumulate vs overwrite; aux2 = bias-gradient vector or NULL
//           (same accumulate/overwrite rule).
//   thin:   forward / data gradient of problems with at most 32 rows and 16-byte-chunked
//           operands (chosen per problem when allow_thin): no staging, split reduction.
// All kinds may be mixed in one batch (one launch per tick level).
hipError_t launch_linear_tick(GemmBatch& batch, int dtype, bool wide, bool allow_thin, hipStream_t stream);
constexpr int CONV_SPLIT_SLOTS = 2048;
constexpr int64_t CONV_SPLIT_WS_BYTES = 32ll << 20;
constexpr int THIN_WS_SLOTS = 1024;
constexpr int64_t THIN_WS_BYTES = (int64_t)THIN_WS_SLOTS * (32 * 32 * 4 + 4);  // partial tiles, then counters

// Implicit-GEMM convolution fast paths (channel counts that are multiples of the slab).
bool conv_fast_eligible(const GemmProb& p, int dtype);
void conv_gemm_tile(const GemmProb* p, int n, int* bm, int* bn);  // tile shape that keeps the chip busy for these problems
hipError_t launch_conv_gemm(GemmBatch& batch, int dtype, int bm, int bn, hipStream_t stream);  // forward / data gradient
// Large-tile variant (256 x 256 outputs, eight wavefronts, operands loaded straight into LDS) for bf16
// problems whose reduction slabs of 64 lie inside one tap; _wanted: enough mostly-full tiles to fill the chip.
bool conv_gemm256_eligible(const GemmProb& p, int dtype);
bool conv_gemm256_wanted(const GemmProb* p, int n, int dtype);
hipError_t launch_conv_gemm256(GemmBatch& batch, int dtype, hipStream_t stream, int tile = 256);  // tile: 256 or 128 (same kernel, four wavefronts)
// Weight gradient in two phases: launch_conv_wgrad writes per-range partial sums
// (out = f32 [splits][Cout][Ncol], aux3 = f32 [splits][Cout] or NULL; splits: any number of ranges from 1 to
// ceil(K / conv_wgrad_slab), conv_wgrad_splits gives what a problem launched on its own wants),
// launch_wgrad_reduce folds them into the accumulators.
int conv_wgrad_splits(const GemmProb& p, int dtype, int wanted);
int conv_wgrad_slab(int dtype);  // output positions per reduction slab; a problem takes 1 .. ceil(K / slab) ranges
hipError_t launch_conv_wgrad(GemmBatch& batch, int dtype, bool wide, hipStream_t stream);
// the same with the tile height chosen per problem (128 rows for matrices of 128 rows and more, 64 below)
hipError_t launch_conv_wgrad_mixed(GemmBatch& batch, int dtype, hipStream_t stream);
struct WReduceProb {
  const float* part; const float* part_beta;  // partial sums [splits][Cout][Ncol], [splits][Cout]
  float* G; float* Ggamma; float* Gbeta;      // accumulators (Ggamma / Gbeta may be NULL)
  const float* gamma; const void* wplain;     // gamma f32[Cout], plain weights T[Cout][Ncol] (or NULL)
  int Cout, Ncol, splits;
  int tile_begin;  // first workgroup of this problem in the launch (set by launch_wgrad_reduce)
  int rg;          // groups of 32 lanes that share one weight row (set by launch_wgrad_reduce)
  // d gamma of a row is a sum over the row's 128-column chunks, which different workgroups hold.  With gpart
  // (f32 [Cout][chunks]) and cnt (one zeroed counter per block of rows, left zero by the launch) the chunks'
  // shares are written there and the last workgroup of a row block adds them in chunk order (one writer per
  // row, fixed order); without them (or with one chunk) the shares meet in a float atomic add / a plain add.
  float* gpart;
  unsigned int* cnt;
};
constexpr int FOLD_COUNTERS = 1 << 16;  // counters the engine keeps for the fold launches
constexpr int WREDUCE_MAX_PROBS = 32;
struct WReduceBatch { int n; WReduceProb p[WREDUCE_MAX_PROBS]; };
hipError_t launch_wgrad_reduce(WReduceBatch& b, int dtype, hipStream_t stream);

// ---------------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------------
// Staging of one micro-batch: fp32 -> T conversion of its rows, label copy, and zeroing
// of the n_slots (<= 256) loss slots its head pass will add into.
hipError_t launch_stage_input(const float* x, const int32_t* y, void* x_out, int32_t* y_out, float* loss_slot, int n_slots,
                              int rows, int64_t per_row, int dtype, hipStream_t stream);

// Loss slots hold the micro-batch objective as a 32-bit fixed-point number (units of 1 / LOSS_SCALE): every
// row adds round(loss_row / rows_per_slot * LOSS_SCALE) with an integer atomic, so the sum does not depend
// on the order in which the rows arrive (a float atomic add would).  Range +-512, resolution 2.4e-7.
constexpr float LOSS_SCALE = 4194304.0f;  // 2^22

// Softmax cross-entropy of one batch: logits f32 [B][C] -> dlogits = (softmax - onehot)/B as
// T [B][C]; the mean loss of every group of rows_per_slot consecutive rows (a divisor of B) is
// added to loss_out[group] (zeroed by the staging kernel) in the fixed-point form above.
hipError_t launch_ce_head(const float* logits, const int32_t* labels, void* dlogits, float* loss_out,
                          int B, int C, int rows_per_slot, int dtype, hipStream_t stream);

// out[c] += sum_r src[r][c]  (fp32 atomics; out must hold the running sum).
struct ColsumProb { const void* src; float* out; int rows, cols, ld; };
constexpr int COLSUM_MAX_PROBS = 32;
struct ColsumBatch { int n; ColsumProb p[COLSUM_MAX_PROBS]; };
hipError_t launch_colsum_batch(const ColsumBatch& b, int dtype, hipStream_t stream);


// Vector parameters (bias, gamma, beta): SGD step ; G = 0 ; copy = master.  V may be NULL.
// All vectors of a stage go in one launch.
struct VecUpdate { float* master; float* G; float* V; float* copy; int64_t n; };
constexpr int VEC_UPDATE_MAX = 24;
struct VecUpdateBatch { int n; VecUpdate v[VEC_UPDATE_MAX]; };
hipError_t launch_update_vec_batch(const VecUpdateBatch& b, SgdParams sgd, hipStream_t stream);

// Matrix parameters W[O][T][C] (Linear: T = 1):  SGD step on master (V = velocity or NULL),
// G = 0 if zero_g, then write the compute copies of the new version:
//   wf[o][t][c] = T(gamma[o]*master)   forward layout
//   wt[c][t][o] = T(gamma[o]*master)   data-gradient layout
//   wp[o][t][c] = T(master)            plain copy (only when gamma != NULL)
// gamma points at the already updated fp32 copy in the new ring slot.  All matrices of a stage
// go in one launch.
struct RepackArgs {
  float* master; float* G; float* V; const float* gamma;
  void* wf; void* wt; void* wp;
  int O, T, C; SgdParams sgd; int zero_g;
  int ldf;         // row length of wf (T*C, or the zero-padded length of an im2col layer)
  int tile_begin;  // first workgroup of this matrix in the launch (set by launch_repack_batch)
};
constexpr int REPACK_MAX = 12;
struct RepackBatch { int n; RepackArgs a[REPACK_MAX]; };
hipError_t launch_repack_batch(RepackBatch& b, int dtype, hipStream_t stream);

// Explicit im2col for layers whose channel count is below one 16-byte chunk (the RGB stem):
// col[(b,oh,ow)][k] = x[b][oh*s-p+kh][ow*s-p+kw][c], k = (kh*KW+kw)*C+c, zero for k >= KH*KW*C.
hipError_t launch_im2col(const void* x, void* col, int B, const ConvGeom& g, int kpad, int dtype, hipStream_t stream);

// Max pool (NHWC) forward, and backward by gather (first maximum in (kh,kw) scan order
// receives the gradient); backward optionally masks with x > 0.
hipError_t launch_maxpool_fwd(const void* x, void* y, int B, int H, int W, int C, int k, int s, int p,
                              int dtype, hipStream_t stream);
// With a workspace of at least B*OH*OW*C bytes (and C a multiple of the 16-byte chunk) the
// backward first records every window's first maximum there, then gathers.
hipError_t launch_maxpool_bwd(const void* x, const void* dy, void* dx, int B, int H, int W, int C, int k,
                              int s, int p, int mask_relu, void* workspace, int64_t workspace_bytes, int dtype,
                              hipStream_t stream);
// Global average pool forward / backward (backward optionally masks with x > 0).
hipError_t launch_gap_fwd(const void* x, void* y, int B, int HW, int C, int dtype, hipStream_t stream);
hipError_t launch_gap_bwd(const void* x, const void* dy, void* dx, int B, int HW, int C, int mask_relu,
                          int dtype, hipStream_t stream);
// ViT-shaped stages (transformer_kernels.hip).  LayerNorm over the C channels of `rows` rows
// (C <= 1024), fp32 gamma / beta; the backward adds `add` (may be NULL) to dx and adds d gamma /
// d beta to the running sums Ggamma / Gbeta through row statistics and per-workgroup partial
// sums in `workspace` (layernorm_bwd_workspace_bytes) and a small fold kernel.
hipError_t launch_layernorm_fwd(const void* x, const float* gamma, const float* beta, void* y, int rows, int C, int dtype,
                                hipStream_t stream);
int64_t layernorm_bwd_workspace_bytes(int rows, int C);
// The same passes for up to LN_BATCH_MAX problems of one shape in one launch each (rows that are whole 16-byte
// chunks only: layernorm_batchable on every tensor of a problem; workspace as for launch_layernorm_bwd).
constexpr int LN_BATCH_MAX = 8;
struct LnFwdProb { const void* x; const float* gamma; const float* beta; void* y; };
struct LnFwdBatch { LnFwdProb p[LN_BATCH_MAX]; int n; };
struct LnBwdProb { const void* x; const void* dy; const void* add; const float* gamma; void* dx; float* Ggamma; float* Gbeta; float* workspace; };
struct LnBwdBatch { LnBwdProb p[LN_BATCH_MAX]; int n; };
bool layernorm_batchable(const void* a, const void* b, const void* c, const void* d, int C, int dtype);
hipError_t launch_layernorm_fwd_batch(const LnFwdBatch& b, int rows, int C, int dtype, hipStream_t stream);
hipError_t launch_layernorm_bwd_batch(const LnBwdBatch& b, int rows, int C, int dtype, hipStream_t stream);

hipError_t launch_layernorm_bwd(const void* x, const void* dy, const void* add, const float* gamma, void* dx, float* Ggamma,
                                float* Gbeta, float* workspace, int rows, int C, int dtype, hipStream_t stream);
// Exact GELU and its derivative, elementwise.
hipError_t launch_gelu_fwd(const void* x, void* y, int64_t n, int dtype, hipStream_t stream);
hipError_t launch_gelu_bwd(const void* x, const void* dy, void* dx, int64_t n, int dtype, hipStream_t stream);
// Self-attention core on qkv[B][T][3*D] (q | k | v per token; T <= 1024): P[B][heads][T][T] are the
// attention probabilities (written by the forward, read by the backward), out / dout [B][T][D];
// ws: fp32 [B][heads][T][T] scratch; ws_ds: T [B][heads][T][T] scratch.
hipError_t launch_attention_fwd(const void* qkv, void* P, void* out, float* ws, int B, int T, int D, int heads, int dtype,
                                hipStream_t stream);
hipError_t launch_attention_bwd(const void* qkv, const void* P, const void* dout, void* dqkv, float* ws_dp, void* ws_ds, int B,
                                int T, int D, int heads, int dtype, hipStream_t stream);
// Kernels one call of the above launches (the score rows take one kernel where attn_scores_kernel applies, else two).
int attention_launches(bool backward, int NT, int D, int heads, int dtype);

// T -> f32 copy (cdp_get_weights of a ring copy).
hipError_t launch_to_f32(const void* src, float* dst, int64_t n, int dtype, hipStream_t stream);
hipError_t launch_fill_f32(float* dst, int64_t n, float v, hipStream_t stream);

}  // namespace cdp
