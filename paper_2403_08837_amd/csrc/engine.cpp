// Host engine of libcdp: tick scheduler, weight-version ring, gradient-accumulator
// bookkeeping, activation pool, per-tick launch lists, and the C ABI of include/cdp.h.
//
// Timeline (Sec. 3.2 "Algorithmic description", Fig. 1): micro-batch i of step t starts at
// tick 2S*t + d*i and runs forward of stages 0..S-1 then backward of stages S-1..0, one
// stage per tick.  Version rule (Sec. 3.2 "Update rules"): the forward of stage j reads
//   DP: theta_t      v1: theta_{t-1}      v2: the freshest version in memory,
// and the backward reads the version its own forward used, so that the applied gradient
// is the gradient at one consistent point theta_hat_{i,t} as Eq. (CDP) states.  A stage
// is updated at the end of the tick in which it received its N-th gradient; the new
// version is written into the other ring slot and is visible from the next tick.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "../../include/cdp.h"
#include "kernels.h"
#include "plan.h"

using namespace cdp;

namespace {

constexpr int LOSS_LOG_STEPS = 1024;
constexpr size_t TRACE_CAP = 1u << 20;

thread_local std::string g_last_error;

struct Block {
  int64_t off = -1;
  int64_t bytes = 0;
  bool valid() const { return off >= 0; }
};

// Size-class slab pool over [base, base+cap) of the arena: one free list per block
// size, new slots carved from a bump pointer.  Every size class is bounded by its own
// peak live count, so the footprint stops growing after the first steady-state period.
struct Pool {
  int64_t base = 0, cap = 0, bump = 0, in_use = 0, peak = 0;
  std::map<int64_t, std::vector<int64_t>> free_lists;
  bool alloc(int64_t bytes, Block* out) {
    bytes = align_up(std::max<int64_t>(bytes, 1), 256);
    auto& fl = free_lists[bytes];
    int64_t off;
    if (!fl.empty()) {
      off = fl.back();
      fl.pop_back();
    } else {
      if (cap >= 0 && bump + bytes > cap) return false;
      off = bump;
      bump += bytes;
    }
    in_use += bytes;
    peak = std::max(peak, in_use);
    out->off = base + off;
    out->bytes = bytes;
    return true;
  }
  void release(const Block& b) {
    if (!b.valid()) return;
    free_lists[b.bytes].push_back(b.off - base);
    in_use -= b.bytes;
  }
};

struct VisitRecord {
  bool live = false;
  int version = 0;
  int64_t step = 0;
  std::vector<Block> t;  // per tensor of the stage
};

struct StageState {
  int64_t master = 0, G = 0, V = -1, slot[2] = {0, 0};  // V: velocity (momentum) or -1
  int ver = 0, cnt = 0;
  int ring_ver[2] = {0, 0};
};

enum ItemKind { IT_GEMM, IT_COLSUM, IT_WREDUCE, IT_IM2COL, IT_STAGE_IN, IT_CE, IT_MAXPOOL_F, IT_MAXPOOL_B, IT_GAP_F, IT_GAP_B,
                IT_LN_F, IT_LN_B, IT_GELU_F, IT_GELU_B, IT_ATTN_F, IT_ATTN_B };
struct Item {
  int kind;
  GemmProb g;
  ColsumProb c;
  WReduceProb r;
  const void* p0 = nullptr; const void* p1 = nullptr; void* p2 = nullptr; void* p3 = nullptr; void* p4 = nullptr;
  const void* p5 = nullptr; void* p6 = nullptr; void* p7 = nullptr;
  int64_t n0 = 0;
  int i[10] = {0};
  double flops = 0, bytes = 0;  // algorithmic work (contractions only)
  bool done = false;            // already carried by another launch of its level
  bool fused_update = false;    // IT_GEMM weight gradient of a Linear layer that also takes the SGD step (u)
  bool big_tile = false;        // IT_GEMM forward / data gradient that runs on the 256 x 256 tile in this launch
  LinUpdate u;
};
typedef std::vector<std::vector<Item>> Program;

}  // namespace

struct cdp_ctx {
  ModelPlan plan;
  int S = 0, N = 0, B = 0, d = 0, rule = 0;
  std::vector<uint8_t> fresh_mask;  // CDP_RULE_MASK: [micro-batch][stage]
  bool bwd_fresh = false;           // backward reads the freshest version
  int dw_group = 1;                 // micro-batches per pass over a Linear accumulator (cdp_opts.dw_group)
  // weight gradients deferred until their group is complete: per stage, the (dY, X) pointers of every Linear
  // layer of the passes waiting, and the blocks those passes would have released
  struct PendingPass { std::vector<std::pair<const void*, const void*>> ops; std::vector<Block> held; };
  std::vector<std::vector<PendingPass>> pending;  // [stage][waiting passes]
  double empty_pair_ms = 0.0;       // event-to-event time of an empty bracket (cdp_profile_gemm)
  int groups = 1;  // lock-step batched DP: the caller's micro-batches run as one batch of groups * (caller's B) rows (then N = 1)
  float lr = 0.f, momentum = 0.f, weight_decay = 0.f;
  bool dry = false;
  hipStream_t stream = nullptr;
  char* arena = nullptr;
  int64_t arena_bytes = 0;
  std::vector<StageState> st;
  int64_t labels_off = 0, loss_off = 0, thin_ws_off = 0, conv_ws_off = -1, fold_cnt_off = -1;
  Pool pool;
  int64_t scratch_base = 0, scratch_cap = -1, scratch_bump = 0;  // per-tick workspace (im2col buffers, partial sums)
  std::vector<std::vector<VisitRecord>> rec;  // [mb][stage]
  std::vector<Block> carry;                   // per micro-batch: activation / gradient between stages
  std::vector<Block> deferred;                // released when the tick's launches are enqueued
  int64_t tick = 0, origin_tick = 0, origin_step = 0, steps_enqueued = 0;
  bool weights_locked = false;
  bool poisoned = false;                      // a tick failed half-way: the timeline state is no longer consistent
  std::vector<int> heads_done;                // per logged step: head passes run
  std::vector<cdp_trace_rec> trace;
  std::vector<int32_t> live_counts;
  std::vector<int64_t> live_bytes[2];         // per tick: retained for a backward | everything the pool holds (in-tick)
  cdp_stats stats;
  int64_t in_features = 0;                    // per-sample input elements
  std::string err;
  // optional timing of the grouped contraction launches (HIP events on the work stream)
  bool profiling = false;
  struct ProfRec { hipEvent_t a, b; double flops, bytes; };
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> event_pool;

  void* ptr(int64_t off) const { return reinterpret_cast<void*>(reinterpret_cast<uintptr_t>(arena) + (uintptr_t)off); }
  float* fptr(int64_t off) const { return static_cast<float*>(ptr(off)); }
};

namespace {

}  // namespace

// Error text of calls that have no context (the kernel-level entry points); read by cdp_last_error(NULL).
namespace cdp {
void set_global_error(const std::string& msg) { g_last_error = msg; }
}  // namespace cdp

namespace {

int fail(cdp_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  g_last_error = msg;
  return code;
}

#define HIP_TRY(ctx, expr)                                                                     \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) return fail(ctx, CDP_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

int64_t tensor_bytes(const cdp_ctx* c, const TensorInfo& t) {
  return (int64_t)c->B * t.per_sample() * (t.f32 ? 4 : c->plan.elem_bytes);
}

bool pool_alloc(cdp_ctx* c, int64_t bytes, Block* b) {
  if (!c->pool.alloc(bytes, b)) return false;
  c->stats.peak_activation_bytes = std::max<int64_t>(c->stats.peak_activation_bytes, c->pool.in_use);
  c->stats.pool_span_bytes = std::max<int64_t>(c->stats.pool_span_bytes, c->pool.bump);
  return true;
}

// Workspace that lives for one tick only (reset when the tick's launches are enqueued).
bool scratch_alloc(cdp_ctx* c, int64_t bytes, Block* b) {
  bytes = align_up(std::max<int64_t>(bytes, 1), 256);
  if (c->scratch_cap >= 0 && c->scratch_bump + bytes > c->scratch_cap) return false;
  b->off = c->scratch_base + c->scratch_bump;
  b->bytes = bytes;
  c->scratch_bump += bytes;
  c->stats.scratch_bytes = std::max<int64_t>(c->stats.scratch_bytes, c->scratch_bump);
  return true;
}

// --------------------------------------------------------------------------- layouts
struct StaticLayout {
  std::vector<StageState> st;
  int64_t labels_off, loss_off, thin_ws_off, conv_ws_off, fold_cnt_off, pool_base, weight_bytes;
};

StaticLayout static_layout(const ModelPlan& plan, int N, int B, int groups, bool velocity) {
  StaticLayout L;
  int64_t off = 0;
  L.weight_bytes = 0;
  for (const StagePlan& sp : plan.stages) {
    StageState s;
    s.master = off; off = align_up(off + sp.n_params * 4, 256);
    s.G = off; off = align_up(off + sp.n_params * 4, 256);
    if (velocity) { s.V = off; off = align_up(off + sp.n_params * 4, 256); }
    s.slot[0] = off; off = align_up(off + sp.slot_bytes, 256);
    s.slot[1] = off; off = align_up(off + sp.slot_bytes, 256);
    L.st.push_back(s);
  }
  L.weight_bytes = off;
  L.labels_off = off; off = align_up(off + (int64_t)N * B * 4, 256);
  L.loss_off = off; off = align_up(off + (int64_t)LOSS_LOG_STEPS * N * groups * 4, 256);
  L.thin_ws_off = off; off = align_up(off + THIN_WS_BYTES, 256);
  L.conv_ws_off = -1;
  for (const StagePlan& sp : plan.stages)
    for (const Op& o : sp.ops)
      if (o.kind == OPK_GEMM && o.is_conv) L.conv_ws_off = 0;
  L.fold_cnt_off = -1;
  if (L.conv_ws_off == 0) {
    L.conv_ws_off = off; off = align_up(off + CONV_SPLIT_WS_BYTES + CONV_SPLIT_SLOTS * 4, 256);
    L.fold_cnt_off = off; off = align_up(off + (int64_t)FOLD_COUNTERS * 4, 256);  // zeroed at init, left zero by every fold launch
  }
  L.pool_base = off;
  return L;
}

// --------------------------------------------------------------------------- GEMM problems
void conv_geom(const Op& o, int mode, ConvGeom* g) {
  if (mode == OP_CONV_DGRAD) {
    g->H = o.Hout; g->W = o.Wout; g->C = o.Cout; g->OH = o.Hin; g->OW = o.Win;
  } else {
    g->H = o.Hin; g->W = o.Win; g->C = o.Cin; g->OH = o.Hout; g->OW = o.Wout;
  }
  g->KH = o.KH; g->KW = o.KW; g->stride = o.stride; g->pad = o.pad;
}

bool pointwise(const Op& o) { return !o.is_conv || (o.KH == 1 && o.KW == 1 && o.stride == 1 && o.pad == 0); }

GemmProb zero_prob() {
  GemmProb p;
  memset(&p, 0, sizeof(p));
  p.splits = 1;
  return p;
}

// x is the layer input, or its im2col buffer [rows][kpad] for a layer with o.kpad > 0.
GemmProb fwd_prob(const cdp_ctx* c, const Op& o, const void* x, void* y, const char* slot, const void* res) {
  GemmProb p = zero_prob();
  const int rows = c->B * o.Hout * o.Wout;
  p.A = x; p.B = slot + o.wf; p.out = y;
  p.aux0 = o.bias_c >= 0 ? slot + o.bias_c : nullptr;
  p.aux1 = res;
  p.M = rows; p.N = o.Cout; p.K = o.kpad ? o.kpad : (int)o.K();
  p.ldb = p.K; p.ldo = o.Cout;
  p.b_mode = OP_PLAIN_K;
  if (o.kpad) { p.a_mode = OP_PLAIN_K; p.lda = o.kpad; }
  else if (pointwise(o)) { p.a_mode = OP_PLAIN_K; p.lda = o.Cin; }
  else { p.a_mode = OP_CONV_FWD; conv_geom(o, OP_CONV_FWD, &p.g); }
  p.epi = EPI_FWD;
  p.flags = (o.relu ? GF_RELU : 0) | (o.out_f32 ? GF_OUT_F32 : 0);
  return p;
}

GemmProb dgrad_prob(const cdp_ctx* c, const Op& o, const void* dz, void* dx, const char* slot, const void* add,
                    const void* mask, bool accumulate) {
  GemmProb p = zero_prob();
  p.A = dz; p.B = slot + o.wt; p.out = dx; p.aux0 = add; p.aux1 = mask;
  p.M = c->B * o.Hin * o.Win; p.N = o.Cin; p.K = o.KH * o.KW * o.Cout;
  p.ldb = p.K; p.ldo = o.Cin;
  p.b_mode = OP_PLAIN_K;
  if (pointwise(o)) { p.a_mode = OP_PLAIN_K; p.lda = o.Cout; }
  else { p.a_mode = OP_CONV_DGRAD; conv_geom(o, OP_CONV_DGRAD, &p.g); }
  p.epi = EPI_DGRAD;
  p.flags = accumulate ? GF_ACCUM : 0;
  return p;
}

// slot: weight version the backward reads (gamma of the affine); slot_f: version the forward read (the plain
// weights that rebuild the pre-affine activation in the gamma gradient).
GemmProb wgrad_prob(const cdp_ctx* c, const Op& o, const void* dz, const void* x, const char* slot, const char* slot_f,
                    float* G, bool first) {
  GemmProb p = zero_prob();
  const int rows = c->B * o.Hout * o.Wout;
  p.A = dz; p.a_mode = OP_PLAIN_R; p.lda = o.Cout;
  p.B = x;  // the layer input, or its im2col buffer for o.kpad > 0
  if (o.kpad) { p.b_mode = OP_PLAIN_R; p.ldb = o.kpad; }
  else if (pointwise(o)) { p.b_mode = OP_PLAIN_R; p.ldb = o.Cin; }
  else { p.b_mode = OP_CONV_WGRAD; conv_geom(o, OP_CONV_WGRAD, &p.g); }
  p.M = o.Cout; p.N = (int)o.K(); p.K = rows;
  p.out = G + o.w_off; p.ldo = (int)o.K();
  p.epi = EPI_WGRAD;
  if (o.is_conv) {
    // accumulators of conv weights are kept zeroed by the update kernel; the long reduction
    // over output positions is split across workgroups
    p.flags = GF_ATOMIC;
    if (o.has_gamma) { p.aux0 = slot + o.gamma_c; p.aux1 = slot_f + o.wp; p.aux2 = G + o.g_off; }
    if (conv_fast_eligible(p, c->plan.dtype)) {
      // two-phase path: build_backward points out / aux3 at a partial-sum workspace
      const int to = p.M >= 128 ? 128 : 64;
      const int tiles = ((p.M + to - 1) / to) * ((p.N + 127) / 128);
      // enough ranges to fill the chip together with the other passes of the tick, but no more
      // partial-sum traffic than ~8 MB per layer
      const int64_t by_bytes = std::max<int64_t>(1, (8ll << 20) / (4 * o.w_count()));
      p.splits = conv_wgrad_splits(p, c->plan.dtype, (int)std::min<int64_t>((384 + tiles - 1) / tiles, by_bytes));
    } else {
      const int tiles = ((p.M + 127) / 128) * ((p.N + 127) / 128);
      const int ktiles = (p.K + 31) / 32;
      p.splits = std::min(std::max(1, std::min((1024 + tiles - 1) / tiles, ktiles / 8)), 256);
    }
  } else {
    p.flags = first ? 0 : GF_ACCUM;
    if (o.b_off >= 0) p.aux2 = G + o.b_off;  // bias gradient is folded into the weight-gradient kernel
  }
  return p;
}

// Algorithmic work of one contraction of a layer: 2 * multiply-adds as the layer defines
// them (the same count for forward, data gradient and weight gradient), and bytes with
// every operand read once and the result written once (a read-modify-write counts twice).
void op_work(const cdp_ctx* c, const Op& o, int pass, bool rmw, bool extra_in, Item* it) {
  const double eb = c->plan.elem_bytes;
  const double rows = (double)c->B * o.Hout * o.Wout;
  const double x = (double)c->B * o.Hin * o.Win * o.Cin, y = rows * o.Cout, w = (double)o.w_count();
  it->flops = 2.0 * rows * o.Cout * (double)o.K();
  if (pass == 0) it->bytes = x * eb + w * eb + y * (o.out_f32 ? 4 : eb) + (o.res >= 0 ? y * eb : 0);
  else if (pass == 1) it->bytes = y * eb + w * eb + x * eb * (rmw ? 2 : 1) + (extra_in ? x * eb : 0);
  else it->bytes = y * eb + x * eb + w * 4 * (rmw ? 2 : 1) + (o.has_gamma ? w * eb : 0);
}

// Linear layers whose weight gradient runs in the HBM-streaming kernel can take their SGD
// step inside that kernel (LinUpdate).
bool linear_update_fusable(const Op& o) {
  return o.kind == OPK_GEMM && !o.is_conv && !o.has_gamma && o.kpad == 0;
}

// Launch class of a contraction: which kernel family and tile shape runs it.
enum LaunchClass {
  LC_LINEAR = 0, LC_CONV_NARROW, LC_CONV_WIDE, LC_CWGRAD_64, LC_CWGRAD_128,
  LC_GEN_FIRST,  // LC_GEN_FIRST + 2*shape + wgrad
  LC_CONV_256 = LC_GEN_FIRST + 2 * TILE_COUNT  // chosen per launch (launch_level), never by launch_class
};

int launch_class(const GemmProb& p, int dtype) {
  (void)dtype;
  if (p.epi != EPI_WGRAD && p.a_mode == OP_PLAIN_K && p.b_mode == OP_PLAIN_K && p.M <= 128) return LC_LINEAR;
  if (p.epi == EPI_WGRAD && p.a_mode == OP_PLAIN_R && p.b_mode == OP_PLAIN_R && !(p.flags & GF_ATOMIC) &&
      ((p.flags & GF_GROUP) || (!p.aux0 && !p.aux1)))
    return LC_LINEAR;
  if (conv_fast_eligible(p, dtype)) {
    if (p.epi == EPI_WGRAD) return p.M >= 128 ? LC_CWGRAD_128 : LC_CWGRAD_64;
    return p.N > 64 ? LC_CONV_WIDE : LC_CONV_NARROW;
  }
  int shape;
  if (p.M <= 64) shape = p.N >= 128 ? TILE_64x128 : TILE_64x64;
  else shape = p.N <= 64 ? TILE_64x64 : TILE_128x128;
  return LC_GEN_FIRST + 2 * shape + (p.epi == EPI_WGRAD ? 1 : 0);
}

// --------------------------------------------------------------------------- programs
int build_forward(cdp_ctx* c, int i, int64_t t, int j, int version, const float* x_dev, const int32_t* y_dev, Program* prog) {
  const StagePlan& sp = c->plan.stages[j];
  VisitRecord& r = c->rec[i][j];
  r.live = true; r.version = version; r.step = t;
  r.t.assign(sp.tensors.size(), Block());
  const char* slot = static_cast<const char*>(c->ptr(c->st[j].slot[version & 1]));
  size_t level = 0;
  bool first_reads_f32 = false;
  auto at = [&](size_t l) -> std::vector<Item>& { if (prog->size() <= l) prog->resize(l + 1); return (*prog)[l]; };
  if (j == 0) {
    if (!pool_alloc(c, tensor_bytes(c, sp.tensors[0]), &r.t[0])) return fail(c, CDP_ENOMEM, "activation pool exhausted");
    Item it; it.kind = IT_STAGE_IN;
    it.p0 = x_dev + (int64_t)i * c->B * c->in_features;
    it.p1 = y_dev + (int64_t)i * c->B;
    it.p2 = c->ptr(r.t[0].off);
    it.p3 = static_cast<int32_t*>(c->ptr(c->labels_off)) + (int64_t)i * c->B;
    it.p4 = c->fptr(c->loss_off) + ((t % LOSS_LOG_STEPS) * c->N + i) * c->groups;
    it.i[0] = c->B; it.i[1] = c->groups; it.n0 = c->in_features;
    at(level).push_back(it);
    // A first Linear layer that runs in the streaming kernel reads the caller's fp32 rows itself
    // (rounding them as the staging kernel does), so it shares the level with the staging; the
    // staged copy is what the backward pass and any other consumer read.
    const Op& o0 = sp.ops.front();
    first_reads_f32 = o0.kind == OPK_GEMM && !o0.is_conv && o0.kpad == 0 && o0.in == 0 && c->B <= 128 &&
                      reinterpret_cast<uintptr_t>(it.p0) % 16 == 0;
    if (!first_reads_f32) ++level;
  } else {
    r.t[0] = c->carry[i];
    c->carry[i] = Block();
  }
  bool ce_fused = false;
  for (size_t oi = 0; oi < sp.ops.size(); ++oi) {
    const Op& o = sp.ops[oi];
    if (o.kind == OPK_CE && ce_fused) continue;  // computed in the epilogue of the classifier's contraction
    if (!pool_alloc(c, tensor_bytes(c, sp.tensors[o.out]), &r.t[o.out])) return fail(c, CDP_ENOMEM, "activation pool exhausted");
    Item it;
    if (o.kind == OPK_GEMM) {
      it.kind = IT_GEMM;
      const void* a_src = c->ptr(r.t[o.in].off);
      if (o.kpad) {  // explicit im2col into a buffer that lives for this tick only
        Block col;
        if (!scratch_alloc(c, (int64_t)c->B * o.Hout * o.Wout * o.kpad * c->plan.elem_bytes, &col)) return fail(c, CDP_ENOMEM, "tick workspace exhausted");
        Item ic; ic.kind = IT_IM2COL;
        ic.p0 = a_src; ic.p2 = c->ptr(col.off); ic.i[0] = c->B; ic.i[1] = o.kpad;
        conv_geom(o, OP_CONV_FWD, &ic.g.g);
        at(level++).push_back(ic);
        a_src = c->ptr(col.off);
      }
      it.g = fwd_prob(c, o, a_src, c->ptr(r.t[o.out].off), slot, o.res >= 0 ? c->ptr(r.t[o.res].off) : nullptr);
      if (first_reads_f32 && &o == &sp.ops.front()) {
        it.g.A = x_dev + (int64_t)i * c->B * c->in_features;
        it.g.flags |= GF_A_F32;
      }
      op_work(c, o, 0, false, false, &it);
      // A classifier of at most 32 classes on at most 32 rows is a single thin tile of the
      // streaming kernel, which then applies the loss head in its epilogue: the logits are
      // never stored, the tile writes dlogits and adds the row losses to their slots.
      const int vec = 16 / c->plan.elem_bytes;
      if (o.out_f32 && !o.is_conv && oi + 1 < sp.ops.size() && sp.ops[oi + 1].kind == OPK_CE && sp.ops[oi + 1].in == o.out &&
          c->B <= 32 && o.Cout <= 32 && o.Cin % vec == 0) {
        const Op& ce = sp.ops[oi + 1];
        if (!pool_alloc(c, tensor_bytes(c, sp.tensors[ce.out]), &r.t[ce.out])) return fail(c, CDP_ENOMEM, "activation pool exhausted");
        it.g.out = c->ptr(r.t[ce.out].off);
        it.g.flags = (it.g.flags & ~GF_OUT_F32) | GF_CE;
        it.g.aux2 = static_cast<int32_t*>(c->ptr(c->labels_off)) + (int64_t)i * c->B;
        it.g.aux3 = c->fptr(c->loss_off) + ((t % LOSS_LOG_STEPS) * c->N + i) * c->groups;
        it.g.g.H = c->B / c->groups;
        ce_fused = true;
      }
    } else if (o.kind == OPK_MAXPOOL) {
      it.kind = IT_MAXPOOL_F;
      it.p0 = c->ptr(r.t[o.in].off); it.p2 = c->ptr(r.t[o.out].off);
      it.i[0] = c->B; it.i[1] = o.Hin; it.i[2] = o.Win; it.i[3] = o.Cin; it.i[4] = o.pk; it.i[5] = o.ps; it.i[6] = o.pp;
    } else if (o.kind == OPK_GAP) {
      it.kind = IT_GAP_F;
      it.p0 = c->ptr(r.t[o.in].off); it.p2 = c->ptr(r.t[o.out].off);
      it.i[0] = c->B; it.i[1] = o.Hin * o.Win; it.i[2] = o.Cin;
    } else if (o.kind == OPK_LN) {
      it.kind = IT_LN_F;
      it.p0 = c->ptr(r.t[o.in].off); it.p2 = c->ptr(r.t[o.out].off);
      it.p1 = slot + o.gamma_c; it.p5 = slot + o.bias_c;
      it.i[0] = c->B * o.Hin * o.Win; it.i[1] = o.Cin;
    } else if (o.kind == OPK_GELU) {
      it.kind = IT_GELU_F;
      it.p0 = c->ptr(r.t[o.in].off); it.p2 = c->ptr(r.t[o.out].off);
      it.n0 = (int64_t)c->B * o.Hin * o.Win * o.Cin;
    } else if (o.kind == OPK_ATTN) {
      // scores of all (sample, head) pairs in fp32: tick workspace
      if (!pool_alloc(c, tensor_bytes(c, sp.tensors[o.aux]), &r.t[o.aux])) return fail(c, CDP_ENOMEM, "activation pool exhausted");
      Block ws;
      if (!scratch_alloc(c, (int64_t)c->B * o.heads * o.Win * o.Win * 4, &ws)) return fail(c, CDP_ENOMEM, "tick workspace exhausted");
      it.kind = IT_ATTN_F;
      it.p0 = c->ptr(r.t[o.in].off); it.p2 = c->ptr(r.t[o.out].off); it.p3 = c->ptr(r.t[o.aux].off); it.p4 = c->ptr(ws.off);
      it.i[0] = c->B; it.i[1] = o.Win; it.i[2] = o.Cout; it.i[3] = o.heads;
    } else {  // OPK_CE
      it.kind = IT_CE;
      it.p0 = c->ptr(r.t[o.in].off);
      it.p1 = static_cast<int32_t*>(c->ptr(c->labels_off)) + (int64_t)i * c->B;
      it.p2 = c->ptr(r.t[o.out].off);
      it.p3 = c->fptr(c->loss_off) + ((t % LOSS_LOG_STEPS) * c->N + i) * c->groups;
      it.i[0] = c->B; it.i[1] = o.classes; it.i[2] = c->B / c->groups;
    }
    at(level++).push_back(it);
  }
  // keep what the backward pass reads; hand the stage output to the next stage
  const int last = (int)sp.tensors.size() - 1;
  for (int k = 0; k <= last; ++k) {
    const TensorInfo& ti = sp.tensors[k];
    bool keep = ti.consumed && !ti.f32;            // logits feed only the loss head
    if (k == last) keep = sp.has_head;             // dlogits stay; other outputs travel on
    if (k == last && !sp.has_head) { c->carry[i] = r.t[k]; r.t[k] = Block(); continue; }
    if (!keep) { c->deferred.push_back(r.t[k]); r.t[k] = Block(); }
  }
  if (sp.has_head) c->heads_done[t % LOSS_LOG_STEPS]++;
  return CDP_OK;
}

int build_backward(cdp_ctx* c, int i, int j, int version, Program* prog, bool first_grad, bool fuse_update) {
  const StagePlan& sp = c->plan.stages[j];
  VisitRecord& r = c->rec[i][j];
  if (!r.live) return fail(c, CDP_ESTATE, "backward without a matching forward");
  const StageState& ss = c->st[j];
  const char* slot = static_cast<const char*>(c->ptr(ss.slot[version & 1]));      // parameters the backward reads
  const char* slot_f = static_cast<const char*>(c->ptr(ss.slot[r.version & 1]));  // parameters its forward read
  float* G = c->fptr(ss.G);
  const int nt = (int)sp.tensors.size(), last = nt - 1;
  std::vector<const void*> g(nt, nullptr), addend(nt, nullptr);
  std::vector<Block> owned(nt);
  Block incoming;
  if (sp.has_head) {
    g[last] = c->ptr(r.t[last].off);
  } else {
    incoming = c->carry[i];
    c->carry[i] = Block();
    if (!incoming.valid()) return fail(c, CDP_ESTATE, "missing upstream gradient");
    g[last] = c->ptr(incoming.off);
  }
  // Deferred weight gradients (dw_group > 1): the Linear layers of this pass only note their (dY, X) until the
  // group is complete (or the step's last gradient arrives); the completing pass contracts all members in one
  // pass over the accumulator, members in arrival order.
  const int waiting = (int)c->pending[j].size();
  const bool grouping = c->dw_group > 1;
  const bool flush = !grouping || waiting + 1 == c->dw_group || ss.cnt == c->N - 1;
  cdp_ctx::PendingPass mine;
  size_t lin_idx = 0;
  size_t level = 0;
  auto at = [&](size_t l) -> std::vector<Item>& { if (prog->size() <= l) prog->resize(l + 1); return (*prog)[l]; };
  for (int oi = (int)sp.ops.size() - 1; oi >= 0; --oi) {
    const Op& o = sp.ops[oi];
    const void* dz = g[o.out];
    if (!dz && addend[o.out] && !sp.tensors[o.out].relu) dz = addend[o.out];  // tensor used only as a residual operand
    if (!dz) return fail(c, CDP_ESTATE, "internal: gradient of a tensor was never produced");
    if (o.kind == OPK_CE) { g[o.in] = dz; continue; }
    const bool need_dx = !(j == 0 && o.in == 0);
    const TensorInfo& tin = sp.tensors[o.in];
    void* dx = nullptr;
    bool accumulate = false;
    if (need_dx) {
      if (g[o.in]) {
        dx = const_cast<void*>(g[o.in]);
        accumulate = true;
      } else {
        if (!pool_alloc(c, tensor_bytes(c, tin), &owned[o.in])) return fail(c, CDP_ENOMEM, "activation pool exhausted");
        dx = c->ptr(owned[o.in].off);
        g[o.in] = dx;
      }
    }
    const void* xin = c->ptr(r.t[o.in].off);
    const void* mask = tin.relu ? xin : nullptr;
    if (o.kind == OPK_GEMM) {
      if (o.res >= 0) {
        if (g[o.res] || addend[o.res]) return fail(c, CDP_EINVAL, "residual operand with an earlier gradient is not supported");
        addend[o.res] = dz;
      }
      if (need_dx) {
        Item it; it.kind = IT_GEMM;
        it.g = dgrad_prob(c, o, dz, dx, slot, accumulate ? nullptr : addend[o.in], mask, accumulate);
        op_work(c, o, 1, accumulate, mask != nullptr, &it);
        at(level).push_back(it);
      }
      Item w; w.kind = IT_GEMM;
      const void* w_src = xin;
      size_t wl = level;  // level of the weight-gradient contraction
      if (o.kpad) {       // rebuild the im2col buffer (cheaper than keeping it between the passes)
        Block col;
        if (!scratch_alloc(c, (int64_t)c->B * o.Hout * o.Wout * o.kpad * c->plan.elem_bytes, &col)) return fail(c, CDP_ENOMEM, "tick workspace exhausted");
        Item ic; ic.kind = IT_IM2COL;
        ic.p0 = xin; ic.p2 = c->ptr(col.off); ic.i[0] = c->B; ic.i[1] = o.kpad;
        conv_geom(o, OP_CONV_FWD, &ic.g.g);
        at(level).push_back(ic);
        w_src = c->ptr(col.off);
        wl = level + 1;
      }
      const bool groupable = grouping && linear_update_fusable(o);
      if (groupable && !flush) {  // noted; contracted by the pass that completes the group
        mine.ops.push_back({dz, w_src});
        ++lin_idx;
        ++level;
        continue;
      }
      const bool first_of_step = groupable ? (ss.cnt - waiting == 0) : first_grad;
      w.g = wgrad_prob(c, o, dz, w_src, slot, slot_f, G, first_of_step);
      op_work(c, o, 2, o.is_conv || !first_of_step, false, &w);
      if (groupable && waiting > 0) {
        const int rows = c->B;
        for (int m = 0; m < waiting; ++m) dw_set_member(w.g, m, c->pending[j][m].ops[lin_idx].first, c->pending[j][m].ops[lin_idx].second);
        dw_set_member(w.g, waiting, dz, w_src);
        w.g.flags |= GF_GROUP;
        w.g.g.pad = rows;
        w.g.K = (waiting + 1) * rows;
        w.flops *= (waiting + 1);
        w.bytes += (double)waiting * rows * (o.Cin + o.Cout) * c->plan.elem_bytes;
      }
      if (groupable) ++lin_idx;
      if (fuse_update && linear_update_fusable(o)) {
        // this gradient is the N-th of the step: its contraction also takes the SGD step and
        // writes the new version into the other ring slot (which no pass of this tick reads)
        char* nslot = static_cast<char*>(c->ptr(ss.slot[(ss.ver + 1) & 1]));
        float* master = c->fptr(ss.master);
        float* V = ss.V >= 0 ? c->fptr(ss.V) : nullptr;
        w.fused_update = true;
        w.u.master = master + o.w_off; w.u.V = V ? V + o.w_off : nullptr;
        w.u.wf = nslot + o.wf; w.u.wt = nslot + o.wt;
        w.u.bmaster = o.b_off >= 0 ? master + o.b_off : nullptr;
        w.u.bV = (o.b_off >= 0 && V) ? V + o.b_off : nullptr;
        w.u.bcopy = o.b_off >= 0 ? reinterpret_cast<float*>(nslot + o.bias_c) : nullptr;
        w.u.sgd = SgdParams{c->lr, 1.0f / (float)c->N, c->momentum, c->weight_decay, 1};
        // master read + write, both compute copies written, accumulator not written back
        w.bytes += (double)o.w_count() * (4 + 2 * c->plan.elem_bytes + (V ? 8 : 0));
      }
      bool two_phase = false;
      if (o.is_conv && conv_fast_eligible(w.g, c->plan.dtype)) {
        // partial sums of every reduction range, folded into the accumulators one level later
        two_phase = true;
        const int64_t wn = (int64_t)w.g.splits * o.w_count(), bn = (int64_t)w.g.splits * o.Cout;
        Block ws;
        if (!scratch_alloc(c, (wn + bn) * 4, &ws)) return fail(c, CDP_ENOMEM, "tick workspace exhausted");
        float* part = c->fptr(ws.off);
        Item rd; rd.kind = IT_WREDUCE;
        rd.r.part = part; rd.r.part_beta = o.b_off >= 0 ? part + wn : nullptr;
        rd.r.G = G + o.w_off; rd.r.Ggamma = o.has_gamma ? G + o.g_off : nullptr; rd.r.Gbeta = o.b_off >= 0 ? G + o.b_off : nullptr;
        rd.r.gamma = static_cast<const float*>(w.g.aux0); rd.r.wplain = w.g.aux1;
        rd.r.Cout = o.Cout; rd.r.Ncol = (int)o.K(); rd.r.splits = w.g.splits;
        rd.r.gpart = nullptr; rd.r.cnt = nullptr;
        const int chunks = ((int)o.K() + 127) / 128;
        if (o.has_gamma && chunks > 1) {  // shares of d gamma per 128-column chunk, added in chunk order by the fold
          Block gp;
          if (!scratch_alloc(c, (int64_t)o.Cout * chunks * 4, &gp)) return fail(c, CDP_ENOMEM, "tick workspace exhausted");
          rd.r.gpart = c->fptr(gp.off);
        }
        w.g.out = part; w.g.aux0 = nullptr; w.g.aux1 = nullptr; w.g.aux2 = nullptr;
        w.g.aux3 = o.b_off >= 0 ? part + wn : nullptr;
        at(wl + 1).push_back(rd);
      }
      at(wl).push_back(w);
      if (o.b_off >= 0 && o.is_conv && !two_phase) {
        Item b; b.kind = IT_COLSUM;
        b.c.src = dz; b.c.out = G + o.b_off; b.c.rows = c->B * o.Hout * o.Wout; b.c.cols = o.Cout; b.c.ld = o.Cout;
        at(wl).push_back(b);
      }
    } else if (o.kind == OPK_LN) {
      // d gamma / d beta are needed even when the input gradient is not; the input may also be
      // the residual operand of a later layer, whose gradient is added here
      if (accumulate) return fail(c, CDP_EINVAL, "layernorm input with an earlier gradient is not supported");
      Block tmp;
      if (!need_dx) {
        if (!scratch_alloc(c, tensor_bytes(c, tin), &tmp)) return fail(c, CDP_ENOMEM, "tick workspace exhausted");
        dx = c->ptr(tmp.off);
      }
      Item it; it.kind = IT_LN_B;
      it.p0 = xin; it.p1 = dz; it.p2 = dx; it.p5 = need_dx ? addend[o.in] : nullptr;
      it.p3 = const_cast<char*>(slot + o.gamma_c); it.p4 = G + o.g_off; it.p6 = G + o.b_off;
      it.i[0] = c->B * o.Hin * o.Win; it.i[1] = o.Cin;
      Block part;  // per-workgroup partial sums of d gamma / d beta
      if (!scratch_alloc(c, layernorm_bwd_workspace_bytes(it.i[0], it.i[1]), &part)) return fail(c, CDP_ENOMEM, "tick workspace exhausted");
      it.p7 = c->ptr(part.off);
      at(level).push_back(it);
    } else if (need_dx && (o.kind == OPK_GELU || o.kind == OPK_ATTN)) {
      if (accumulate || addend[o.in]) return fail(c, CDP_EINVAL, "gelu / attention input with another use is not supported");
      Item it;
      it.p0 = xin; it.p1 = dz; it.p2 = dx;
      if (o.kind == OPK_GELU) {
        it.kind = IT_GELU_B;
        it.n0 = (int64_t)c->B * o.Hin * o.Win * o.Cin;
      } else {
        const int64_t tt = (int64_t)c->B * o.heads * o.Win * o.Win;
        Block w1, w2;
        if (!scratch_alloc(c, tt * 4, &w1) || !scratch_alloc(c, tt * c->plan.elem_bytes, &w2))
          return fail(c, CDP_ENOMEM, "tick workspace exhausted");
        it.kind = IT_ATTN_B;
        it.p5 = c->ptr(r.t[o.aux].off); it.p3 = c->ptr(w1.off); it.p4 = c->ptr(w2.off);
        it.i[0] = c->B; it.i[1] = o.Win; it.i[2] = o.Cout; it.i[3] = o.heads;
      }
      at(level).push_back(it);
    } else if (need_dx) {
      if (accumulate) return fail(c, CDP_EINVAL, "pooling input with several consumers is not supported");
      Item it;
      it.kind = (o.kind == OPK_MAXPOOL) ? IT_MAXPOOL_B : IT_GAP_B;
      it.p0 = xin; it.p1 = dz; it.p2 = dx;
      if (o.kind == OPK_MAXPOOL) {
        it.i[0] = c->B; it.i[1] = o.Hin; it.i[2] = o.Win; it.i[3] = o.Cin; it.i[4] = o.pk; it.i[5] = o.ps; it.i[6] = o.pp;
        it.i[7] = tin.relu ? 1 : 0;
        // tick workspace for the windows' argmax indices (one byte per pooled element)
        Block ws;
        const int64_t nb = (int64_t)c->B * o.Hout * o.Wout * o.Cout;
        if (!scratch_alloc(c, nb, &ws)) return fail(c, CDP_ENOMEM, "tick workspace exhausted");
        it.p3 = c->ptr(ws.off);
        it.n0 = nb;
      } else {
        it.i[0] = c->B; it.i[1] = o.Hin * o.Win; it.i[2] = o.Cin; it.i[3] = tin.relu ? 1 : 0;
      }
      at(level).push_back(it);
    }
    ++level;
  }
  // release everything the pass held; the gradient of the stage input travels on
  // (a pass whose weight gradients wait for their group keeps what it would release: dY and X are in there)
  std::vector<Block>& sink = flush ? c->deferred : mine.held;
  for (int k = 0; k < nt; ++k) {
    if (r.t[k].valid()) sink.push_back(r.t[k]);
    if (owned[k].valid()) {
      if (k == 0 && j > 0) c->carry[i] = owned[k];
      else sink.push_back(owned[k]);
    }
  }
  if (incoming.valid()) sink.push_back(incoming);
  if (!flush) {
    c->pending[j].push_back(std::move(mine));
  } else if (waiting > 0) {
    for (auto& pp : c->pending[j]) c->deferred.insert(c->deferred.end(), pp.held.begin(), pp.held.end());
    c->pending[j].clear();
  }
  r.live = false;
  r.t.clear();
  return CDP_OK;
}

// --------------------------------------------------------------------------- launching
int launch_level(cdp_ctx* c, std::vector<Item>& items) {
  // The wide forward / data-gradient problems that the 256 x 256 tile takes move to a launch of their
  // own when together they fill the chip with mostly-full tiles.
  {
    std::vector<Item*> big;
    std::vector<GemmProb> probs;
    for (Item& it : items) {
      it.big_tile = false;
      if (it.kind == IT_GEMM && launch_class(it.g, c->plan.dtype) == LC_CONV_WIDE && conv_gemm256_eligible(it.g, c->plan.dtype) &&
          it.g.N >= 192 && it.g.M >= 512) {
        big.push_back(&it);
        probs.push_back(it.g);
      }
    }
    if (!big.empty() && conv_gemm256_wanted(probs.data(), (int)probs.size(), c->plan.dtype))
      for (Item* it : big) it->big_tile = true;
  }
  // grouped contractions, one launch per tile shape (and per GEMM_MAX_PROBS problems)
  // convolution weight gradients of both tile heights share one launch (each height alone is short of workgroups
  // on the small configurations): they are all listed under the taller class
  // Forward / data-gradient problems with at most 64 output columns have a launch of their own (128 x 64 tiles).
  // Where the level's wide problems fill a launch of 128 x 128 tiles by themselves, the narrow ones join it
  // instead, half of each of their tiles empty: they are bound by their operand traffic, not by the matrix
  // cores, and one launch fewer per level is worth more than the idle half (cfg4 22.8 -> 22.0 ms per step; on
  // the small launches of cfg3, which run on 64 x 64 tiles with shared reductions, the same costs 19 %).
  bool narrow_joins_wide = false;
  {
    std::vector<GemmProb> wide;
    for (const Item& it : items)
      if (it.kind == IT_GEMM && !it.big_tile && launch_class(it.g, c->plan.dtype) == LC_CONV_WIDE) wide.push_back(it.g);
    if (!wide.empty() && wide.size() < (size_t)GEMM_MAX_PROBS) {
      int bm = 0, bn = 0;
      conv_gemm_tile(wide.data(), (int)wide.size(), &bm, &bn);
      narrow_joins_wide = bm == 128 && bn == 128;
    }
  }
  auto item_class = [&](const Item& it) {
    if (it.big_tile) return (int)LC_CONV_256;
    const int lc = launch_class(it.g, c->plan.dtype);
    if (lc == LC_CONV_NARROW && narrow_joins_wide) return (int)LC_CONV_WIDE;
    return lc == LC_CWGRAD_64 ? (int)LC_CWGRAD_128 : lc;
  };
  for (int key = 0; key <= LC_CONV_256; ++key) {
    std::vector<const Item*> sel;
    for (const Item& it : items)
      if (it.kind == IT_GEMM && item_class(it) == key) sel.push_back(&it);
    // longest reductions first so the tail of the launch is made of short tiles
    std::stable_sort(sel.begin(), sel.end(),
                     [](const Item* a, const Item* b) { return a->g.K / a->g.splits > b->g.K / b->g.splits; });
    for (size_t k = 0; k < sel.size(); k += GEMM_MAX_PROBS) {
      GemmBatch batch;
      batch.n = (int)std::min<size_t>(GEMM_MAX_PROBS, sel.size() - k);
      batch.n_upd = 0;
      batch.copy_tiles = 0;
      batch.thin_ws = c->fptr(c->thin_ws_off);  // zeroed at init, left zero by every launch
      batch.thin_cnt = reinterpret_cast<unsigned int*>(c->fptr(c->thin_ws_off) + (int64_t)THIN_WS_SLOTS * 1024);
      if (key == LC_LINEAR && k == 0) {
        // a micro-batch that starts in this tick: its staging rides on this launch
        for (Item& si : items)
          if (si.kind == IT_STAGE_IN && !si.done && (int64_t)si.i[0] * si.n0 < (1ll << 40)) {
            batch.sc = StageCopy{static_cast<const float*>(si.p0), static_cast<const int32_t*>(si.p1), si.p2,
                                 static_cast<int32_t*>(si.p3), static_cast<float*>(si.p4), si.i[1], si.i[0],
                                 (int64_t)si.i[0] * si.n0};
            batch.copy_tiles = (int)((batch.sc.n + STAGE_COPY_ELEMS - 1) / STAGE_COPY_ELEMS);
            si.done = true;
            break;
          }
      }
      for (int q = 0; q < batch.n; ++q) {
        batch.p[q] = sel[k + q]->g;
        batch.p[q].upd = 0;
        if (sel[k + q]->fused_update) {
          if (batch.n_upd == LIN_UPD_MAX) return fail(c, CDP_ESTATE, "internal: too many fused updates in one launch");
          batch.upd[batch.n_upd] = sel[k + q]->u;
          batch.p[q].upd = ++batch.n_upd;
        }
      }
      cdp_ctx::ProfRec pr{nullptr, nullptr, 0, 0};
      const bool timed = c->profiling && c->prof.size() < (1u << 18);
      if (timed) {
        for (hipEvent_t* e : {&pr.a, &pr.b}) {
          if (!c->event_pool.empty()) { *e = c->event_pool.back(); c->event_pool.pop_back(); }
          else HIP_TRY(c, hipEventCreate(e));
        }
        for (int q = 0; q < batch.n; ++q) { pr.flops += sel[k + q]->flops; pr.bytes += sel[k + q]->bytes; }
        HIP_TRY(c, hipEventRecord(pr.a, c->stream));
      }
      if (key == LC_LINEAR) {
        // wide column tiles when the forward / data-gradient problems are large enough to fill the chip with them
        int64_t skinny_cols = 0;
        for (int q = 0; q < batch.n; ++q)
          if (batch.p[q].epi != EPI_WGRAD) skinny_cols += batch.p[q].N;
        HIP_TRY(c, launch_linear_tick(batch, c->plan.dtype, skinny_cols >= 32768, true, c->stream));
      } else if (key == LC_CONV_NARROW || key == LC_CONV_WIDE) {
        if (c->conv_ws_off >= 0) {  // zeroed at init, counters left zero by every launch
          batch.thin_ws = c->fptr(c->conv_ws_off);
          batch.thin_cnt = reinterpret_cast<unsigned int*>(static_cast<char*>(c->ptr(c->conv_ws_off)) + CONV_SPLIT_WS_BYTES);
        } else {
          batch.thin_ws = nullptr;
          batch.thin_cnt = nullptr;
        }
        int bm, bn;
        conv_gemm_tile(batch.p, batch.n, &bm, &bn);
        HIP_TRY(c, launch_conv_gemm(batch, c->plan.dtype, bm, bn, c->stream));
      }
      else if (key == LC_CONV_256) HIP_TRY(c, launch_conv_gemm256(batch, c->plan.dtype, c->stream));
      else if (key == LC_CWGRAD_128) HIP_TRY(c, launch_conv_wgrad_mixed(batch, c->plan.dtype, c->stream));
      else HIP_TRY(c, launch_gemm_batch(batch, c->plan.dtype, (key - LC_GEN_FIRST) / 2, c->stream));
      if (timed) {
        HIP_TRY(c, hipEventRecord(pr.b, c->stream));
        c->prof.push_back(pr);
      }
      c->stats.kernel_launches++;
    }
  }
  ColsumBatch cb;
  cb.n = 0;
  for (const Item& it : items) {
    if (it.kind != IT_COLSUM) continue;
    cb.p[cb.n++] = it.c;
    if (cb.n == COLSUM_MAX_PROBS) {
      HIP_TRY(c, launch_colsum_batch(cb, c->plan.dtype, c->stream));
      c->stats.kernel_launches++;
      cb.n = 0;
    }
  }
  if (cb.n) {
    HIP_TRY(c, launch_colsum_batch(cb, c->plan.dtype, c->stream));
    c->stats.kernel_launches++;
  }
  // folds of the convolution weight-gradient partial sums: part of the contraction (timed with it)
  WReduceBatch rb;
  rb.n = 0;
  auto flush_folds = [&]() -> int {
    if (!rb.n) return CDP_OK;
    cdp_ctx::ProfRec pr{nullptr, nullptr, 0, 0};
    const bool timed = c->profiling && c->prof.size() < (1u << 18);
    if (timed) {
      for (hipEvent_t* e : {&pr.a, &pr.b}) {
        if (!c->event_pool.empty()) { *e = c->event_pool.back(); c->event_pool.pop_back(); }
        else HIP_TRY(c, hipEventCreate(e));
      }
      // no algorithmic work of its own: the accumulator's read-modify-write is already counted with the
      // weight-gradient contraction, the partial sums are this implementation's traffic
      HIP_TRY(c, hipEventRecord(pr.a, c->stream));
    }
    {
      // one counter per block of rows of every problem that orders its d gamma shares
      int64_t used = 0;
      unsigned int* base = c->fold_cnt_off >= 0 ? reinterpret_cast<unsigned int*>(c->ptr(c->fold_cnt_off)) : nullptr;
      for (int q = 0; q < rb.n; ++q) {
        WReduceProb& r = rb.p[q];
        if (!r.gpart) continue;
        const int rg = r.splits <= 8 ? 1 : r.splits <= 16 ? 2 : r.splits <= 32 ? 4 : 8;  // as launch_wgrad_reduce
        const int blocks = (r.Cout + 8 / rg - 1) / (8 / rg);
        if (base && used + blocks <= FOLD_COUNTERS) { r.cnt = base + used; used += blocks; }
        else r.gpart = nullptr;  // no counters left: the shares meet in atomic adds
      }
    }
    HIP_TRY(c, launch_wgrad_reduce(rb, c->plan.dtype, c->stream));
    if (timed) {
      HIP_TRY(c, hipEventRecord(pr.b, c->stream));
      c->prof.push_back(pr);
    }
    c->stats.kernel_launches++;
    rb.n = 0;
    return CDP_OK;
  };
  for (const Item& it : items) {
    if (it.kind != IT_WREDUCE) continue;
    rb.p[rb.n++] = it.r;
    if (rb.n == WREDUCE_MAX_PROBS) { int rc = flush_folds(); if (rc) return rc; }
  }
  { int rc = flush_folds(); if (rc) return rc; }
  const int dt = c->plan.dtype;
  // LayerNorm passes of one shape (the same layer of several stages / micro-batches) share their launches
  for (size_t a = 0; a < items.size(); ++a) {
    Item& first = items[a];
    if (first.done || (first.kind != IT_LN_F && first.kind != IT_LN_B)) continue;
    auto batchable = [&](const Item& it) {
      return it.kind == IT_LN_F ? layernorm_batchable(it.p0, it.p2, nullptr, nullptr, it.i[1], dt)
                                : layernorm_batchable(it.p0, it.p1, it.p5, it.p2, it.i[1], dt);
    };
    if (!batchable(first)) continue;
    std::vector<Item*> grp;
    for (size_t b = a; b < items.size() && grp.size() < (size_t)LN_BATCH_MAX; ++b) {
      Item& it = items[b];
      if (!it.done && it.kind == first.kind && it.i[0] == first.i[0] && it.i[1] == first.i[1] && batchable(it)) grp.push_back(&it);
    }
    if (grp.size() < 2) continue;
    if (first.kind == IT_LN_F) {
      LnFwdBatch fb;
      fb.n = (int)grp.size();
      for (int q = 0; q < fb.n; ++q)
        fb.p[q] = LnFwdProb{grp[q]->p0, static_cast<const float*>(grp[q]->p1), static_cast<const float*>(grp[q]->p5), grp[q]->p2};
      HIP_TRY(c, launch_layernorm_fwd_batch(fb, first.i[0], first.i[1], dt, c->stream));
      c->stats.kernel_launches += 1;
    } else {
      LnBwdBatch bb;
      bb.n = (int)grp.size();
      for (int q = 0; q < bb.n; ++q)
        bb.p[q] = LnBwdProb{grp[q]->p0, grp[q]->p1, grp[q]->p5, static_cast<const float*>(grp[q]->p3), grp[q]->p2,
                            static_cast<float*>(grp[q]->p4), static_cast<float*>(grp[q]->p6), static_cast<float*>(grp[q]->p7)};
      HIP_TRY(c, launch_layernorm_bwd_batch(bb, first.i[0], first.i[1], dt, c->stream));
      c->stats.kernel_launches += 3;
    }
    for (Item* it : grp) it->done = true;
  }
  for (const Item& it : items) {
    if (it.done && (it.kind == IT_LN_F || it.kind == IT_LN_B)) continue;
    switch (it.kind) {
      case IT_STAGE_IN:
        if (it.done) continue;
        HIP_TRY(c, launch_stage_input(static_cast<const float*>(it.p0), static_cast<const int32_t*>(it.p1), it.p2,
                                      static_cast<int32_t*>(it.p3), static_cast<float*>(it.p4), it.i[1], it.i[0], it.n0, dt, c->stream));
        break;
      case IT_IM2COL:
        HIP_TRY(c, launch_im2col(it.p0, it.p2, it.i[0], it.g.g, it.i[1], dt, c->stream));
        break;
      case IT_CE:
        HIP_TRY(c, launch_ce_head(static_cast<const float*>(it.p0), static_cast<const int32_t*>(it.p1), it.p2,
                                  static_cast<float*>(it.p3), it.i[0], it.i[1], it.i[2], dt, c->stream));
        break;
      case IT_MAXPOOL_F:
        HIP_TRY(c, launch_maxpool_fwd(it.p0, it.p2, it.i[0], it.i[1], it.i[2], it.i[3], it.i[4], it.i[5], it.i[6], dt, c->stream));
        break;
      case IT_MAXPOOL_B:
        HIP_TRY(c, launch_maxpool_bwd(it.p0, it.p1, it.p2, it.i[0], it.i[1], it.i[2], it.i[3], it.i[4], it.i[5], it.i[6],
                                      it.i[7], it.p3, it.n0, dt, c->stream));
        c->stats.kernel_launches += 2;  // three kernels
        break;
      case IT_GAP_F:
        HIP_TRY(c, launch_gap_fwd(it.p0, it.p2, it.i[0], it.i[1], it.i[2], dt, c->stream));
        break;
      case IT_LN_F:
        HIP_TRY(c, launch_layernorm_fwd(it.p0, static_cast<const float*>(it.p1), static_cast<const float*>(it.p5), it.p2, it.i[0],
                                        it.i[1], dt, c->stream));
        break;
      case IT_LN_B:
        HIP_TRY(c, launch_layernorm_bwd(it.p0, it.p1, it.p5, static_cast<const float*>(it.p3), it.p2, static_cast<float*>(it.p4),
                                        static_cast<float*>(it.p6), static_cast<float*>(it.p7), it.i[0], it.i[1], dt, c->stream));
        c->stats.kernel_launches += 2;  // three kernels
        break;
      case IT_GELU_F:
        HIP_TRY(c, launch_gelu_fwd(it.p0, it.p2, it.n0, dt, c->stream));
        break;
      case IT_GELU_B:
        HIP_TRY(c, launch_gelu_bwd(it.p0, it.p1, it.p2, it.n0, dt, c->stream));
        break;
      case IT_ATTN_F:
        HIP_TRY(c, launch_attention_fwd(it.p0, it.p3, it.p2, static_cast<float*>(it.p4), it.i[0], it.i[1], it.i[2], it.i[3], dt,
                                        c->stream));
        c->stats.kernel_launches += attention_launches(false, it.i[1], it.i[2], it.i[3], dt) - 1;
        break;
      case IT_ATTN_B:
        HIP_TRY(c, launch_attention_bwd(it.p0, it.p5, it.p1, it.p2, static_cast<float*>(it.p3), it.p4, it.i[0], it.i[1], it.i[2],
                                        it.i[3], dt, c->stream));
        c->stats.kernel_launches += attention_launches(true, it.i[1], it.i[2], it.i[3], dt) - 1;
        break;
      case IT_GAP_B:
        HIP_TRY(c, launch_gap_bwd(it.p0, it.p1, it.p2, it.i[0], it.i[1], it.i[2], it.i[3], dt, c->stream));
        break;
      default:
        continue;
    }
    c->stats.kernel_launches++;
  }
  return CDP_OK;
}

int launch_program(cdp_ctx* c, Program& prog) {
  for (auto& level : prog) {
    int rc = launch_level(c, level);
    if (rc) return rc;
  }
  return CDP_OK;
}

// Writes the compute copies of stage j's current master weights into ring slot `slot`;
// with apply first takes the SGD step of Eq. (CDP) on the master weights.
int refresh_slot(cdp_ctx* c, int j, int slot, bool apply, bool linear_done = false) {
  SgdParams sgd{c->lr, 1.0f / (float)c->N, c->momentum, c->weight_decay, apply ? 1 : 0};
  const StagePlan& sp = c->plan.stages[j];
  const StageState& ss = c->st[j];
  char* sl = static_cast<char*>(c->ptr(ss.slot[slot]));
  float* master = c->fptr(ss.master);
  float* G = c->fptr(ss.G);
  float* V = ss.V >= 0 ? c->fptr(ss.V) : nullptr;
  // two launches per stage: every vector parameter (the folded weights use the updated gamma),
  // then every weight matrix
  VecUpdateBatch vb;
  vb.n = 0;
  RepackBatch rb;
  rb.n = 0;
  auto flush_vec = [&]() -> int {
    if (vb.n) {
      HIP_TRY(c, launch_update_vec_batch(vb, sgd, c->stream));
      c->stats.kernel_launches++;
      vb.n = 0;
    }
    return CDP_OK;
  };
  auto flush_mat = [&]() -> int {
    if (rb.n) {
      HIP_TRY(c, launch_repack_batch(rb, c->plan.dtype, c->stream));
      c->stats.kernel_launches++;
      rb.n = 0;
    }
    return CDP_OK;
  };
  auto add_vec = [&](int64_t off, int64_t copy_off, int n) -> int {
    if (vb.n == VEC_UPDATE_MAX) { int rc = flush_vec(); if (rc) return rc; }
    vb.v[vb.n++] = VecUpdate{master + off, G + off, V ? V + off : nullptr, reinterpret_cast<float*>(sl + copy_off), n};
    return CDP_OK;
  };
  for (const Op& o : sp.ops) {
    if (o.kind != OPK_GEMM && o.kind != OPK_LN) continue;
    if (linear_done && linear_update_fusable(o)) continue;  // updated by its weight-gradient kernel
    if (o.g_off >= 0) { int rc = add_vec(o.g_off, o.gamma_c, o.Cout); if (rc) return rc; }
    if (o.b_off >= 0) { int rc = add_vec(o.b_off, o.bias_c, o.Cout); if (rc) return rc; }
  }
  { int rc = flush_vec(); if (rc) return rc; }
  for (const Op& o : sp.ops) {
    if (o.kind != OPK_GEMM) continue;
    if (linear_done && linear_update_fusable(o)) continue;
    if (rb.n == REPACK_MAX) { int rc = flush_mat(); if (rc) return rc; }
    RepackArgs& a = rb.a[rb.n++];
    a.master = master + o.w_off; a.G = G + o.w_off; a.V = V ? V + o.w_off : nullptr;
    a.gamma = o.has_gamma ? reinterpret_cast<const float*>(sl + o.gamma_c) : nullptr;
    a.wf = sl + o.wf; a.wt = sl + o.wt; a.wp = o.has_gamma ? sl + o.wp : nullptr;
    a.O = o.Cout; a.T = o.KH * o.KW; a.C = o.Cin; a.sgd = sgd;
    a.ldf = o.kpad ? o.kpad : a.T * a.C;
    a.zero_g = o.is_conv ? 1 : 0;  // conv accumulators are added into and must start at zero
    a.tile_begin = 0;
  }
  return flush_mat();
}

int inflight(const cdp_ctx* c) {
  int n = 0;
  for (int i = 0; i < c->N; ++i) {
    const int64_t rel = c->tick - c->origin_tick - (int64_t)c->d * i;
    if (rel < 0) continue;
    const int64_t t = c->origin_step + rel / (2 * c->S);
    if (t < c->steps_enqueued) ++n;
  }
  return n;
}

int run_tick(cdp_ctx* c, const float* x_dev, const int32_t* y_dev) {
  const int S = c->S, N = c->N, d = c->d;
  const int64_t rel_tick = c->tick - c->origin_tick;
  if (rel_tick % (2 * S) == 0) {
    const int64_t t_new = c->origin_step + rel_tick / (2 * S);
    if (t_new == c->steps_enqueued && x_dev != nullptr) {
      if (!y_dev) return fail(c, CDP_EINVAL, "labels missing");
      c->steps_enqueued++;
      c->heads_done[t_new % LOSS_LOG_STEPS] = 0;
    }
  }
  else if (x_dev != nullptr && c->origin_step + rel_tick / (2 * S) >= c->steps_enqueued) {
    // a mini-batch handed over in the middle of its step: its first micro-batches should have started already
    return fail(c, CDP_ESTATE, "the mini-batch of this step was not handed over at the step's first tick");
  }
  struct Visit { int i; int64_t t; int j; int dir; int version; };
  std::vector<Visit> act;
  int n_fwd = 0;
  for (int i = 0; i < N; ++i) {
    const int64_t rel = rel_tick - (int64_t)d * i;
    if (rel < 0) continue;
    const int64_t t = c->origin_step + rel / (2 * S);
    const int p = (int)(rel % (2 * S));
    if (t >= c->steps_enqueued) continue;
    Visit v{i, t, p < S ? p : 2 * S - 1 - p, p < S ? 0 : 1, 0};
    if (v.dir == 0 && v.j == 0 && x_dev == nullptr) return fail(c, CDP_EINVAL, "a micro-batch starts in this tick but x_dev is NULL");
    n_fwd += (v.dir == 0);
    act.push_back(v);
  }
  int live = n_fwd;
  for (int i = 0; i < N; ++i)
    for (int j = 0; j < S; ++j) live += c->rec[i][j].live ? 1 : 0;
  live *= c->groups;  // a batched pass holds the stage inputs of all the caller's micro-batches
  c->stats.last_live_stage_inputs = live;
  c->stats.peak_live_stage_inputs = std::max<int64_t>(c->stats.peak_live_stage_inputs, live);
  if (c->live_counts.size() < TRACE_CAP) c->live_counts.push_back(live);
  // bytes retained for a later backward by the passes of earlier ticks (a backward of this tick has
  // not released its record yet); the forwards of this tick are added below
  int64_t retained = 0;
  for (int i = 0; i < N; ++i)
    for (int j = 0; j < S; ++j)
      if (c->rec[i][j].live)
        for (const Block& b : c->rec[i][j].t) retained += b.valid() ? b.bytes : 0;
  for (int j = 0; j < S; ++j)  // passes whose weight gradients wait for their group (dw_group > 1)
    for (const auto& pp : c->pending[j])
      for (const Block& b : pp.held) retained += b.bytes;
  c->weights_locked = c->weights_locked || !act.empty();

  // weight version of every pass: forward by the update rule, backward as its own forward
  for (Visit& v : act) {
    const StageState& ss = c->st[v.j];
    if (v.dir == 0) {
      const bool freshest = c->rule == CDP_RULE_V2 || (c->rule == CDP_RULE_MASK && c->fresh_mask[(size_t)v.i * S + v.j]);
      if (freshest) v.version = ss.ver;
      else if (c->rule == CDP_RULE_DP) v.version = (int)v.t;
      else v.version = (int)std::max<int64_t>(v.t - 1, 0);
    } else {
      v.version = c->bwd_fresh ? ss.ver : c->rec[v.i][v.j].version;
    }
    if (ss.ring_ver[v.version & 1] != v.version)
      return fail(c, CDP_ESTATE, v.dir == 0 ? "internal: weight version left the ring before its forward"
                                            : "internal: weight version left the ring before its backward");
  }
  std::vector<Program> progs(act.size());
  std::vector<char> fused(S, 0);
  for (size_t a = 0; a < act.size(); ++a) {
    Visit& v = act[a];
    StageState& ss = c->st[v.j];
    int rc;
    if (v.dir == 0) {
      rc = build_forward(c, v.i, v.t, v.j, v.version, x_dev, y_dev, &progs[a]);
    } else {
      // The backward that brings the N-th gradient may take the SGD step inside its weight-
      // gradient kernels, provided no pass of this tick reads the ring slot the new version
      // goes to (under CDP-v1 the backward itself still reads it).
      bool fuse = ss.cnt == N - 1;
      for (const Visit& o : act)
        if (o.j == v.j && ((o.version ^ (ss.ver + 1)) & 1) == 0) fuse = false;
      rc = build_backward(c, v.i, v.j, v.version, &progs[a], ss.cnt == 0, fuse);
      if (fuse) fused[v.j] = 1;
      ss.cnt++;
    }
    if (rc) return rc;
    for (int q = 0; q < c->groups; ++q)
      if (c->trace.size() < TRACE_CAP)
        c->trace.push_back(cdp_trace_rec{(int32_t)c->tick, v.i * c->groups + q, (int32_t)v.t, v.j, v.dir, v.version});
  }
  for (const Visit& v : act)
    if (v.dir == 0)
      for (const Block& b : c->rec[v.i][v.j].t) retained += b.valid() ? b.bytes : 0;
  if (c->live_bytes[0].size() < TRACE_CAP) {
    c->live_bytes[0].push_back(retained);
    c->live_bytes[1].push_back(c->pool.in_use);  // nothing released during the tick has been returned yet
  }
  // The folds of the convolution weight-gradient partial sums feed nothing before the end-of-
  // tick update: they leave their levels and run together as the last launch of the program.
  auto defer_folds = [](Program& p) {
    std::vector<Item> folds;
    for (auto& level : p) {
      auto keep = std::stable_partition(level.begin(), level.end(), [](const Item& it) { return it.kind != IT_WREDUCE; });
      folds.insert(folds.end(), keep, level.end());
      level.erase(keep, level.end());
    }
    if (!folds.empty()) p.push_back(std::move(folds));
  };
  // Neither do the convolution weight gradients: nothing in the tick reads their partial sums but the folds, and
  // their operands (saved inputs, output gradients) stay untouched until the tick's blocks are released.  They
  // leave their levels too and run as one launch (tiles of both heights) in front of the folds, with the reduction
  // ranges chosen for the launch as a whole: several layers together fill the chip with fewer, longer ranges
  // than each layer would need on its own, and every range less is one partial tile less to write and fold.
  auto defer_wgrads = [c](Program& p) {
    constexpr int TARGET_WGS = 2048;  // workgroups the launch aims at (8 per CU: measured best of 1024 / 2048 / 4096)
    constexpr int MIN_CHUNK = 8;      // slabs per reduction range at least
    std::vector<Item> wg;
    auto is_cw = [c](const Item& it) {
      if (it.kind != IT_GEMM || it.g.epi != EPI_WGRAD) return false;
      const int lc = launch_class(it.g, c->plan.dtype);
      return lc == LC_CWGRAD_64 || lc == LC_CWGRAD_128;
    };
    for (auto& level : p) {
      auto keep = std::stable_partition(level.begin(), level.end(), [&](const Item& it) { return !is_cw(it); });
      wg.insert(wg.end(), keep, level.end());
      level.erase(keep, level.end());
    }
    if (wg.empty()) return;
    const int slab = conv_wgrad_slab(c->plan.dtype);
    int64_t work = 0;  // slabs of all tiles
    for (const Item& it : wg) {
      const int to = it.g.M >= 128 ? 128 : 64;
      work += (int64_t)((it.g.M + to - 1) / to) * ((it.g.N + 127) / 128) * ((it.g.K + slab - 1) / slab);
    }
    const int64_t chunk = std::max<int64_t>(MIN_CHUNK, (work + TARGET_WGS - 1) / TARGET_WGS);
    for (Item& it : wg) {
      // never more ranges than the pass asked for: its partial-sum buffer is sized for those
      const int nslab = (it.g.K + slab - 1) / slab;
      const int splits = (int)std::max<int64_t>(1, std::min<int64_t>(it.g.splits, (nslab + chunk - 1) / chunk));
      if (splits == it.g.splits) continue;
      for (auto& level : p)  // the fold of the same partial sums
        for (Item& f : level)
          if (f.kind == IT_WREDUCE && f.r.part == static_cast<const float*>(it.g.out)) f.r.splits = splits;
      it.g.splits = splits;
    }
    p.push_back(std::move(wg));
  };
  if (!c->dry) {
    if (c->rule == CDP_RULE_DP) {
      // lock-step: all micro-batches hit the same stage, so passes run one after another
      // (their weight gradients share one accumulator)
      for (auto& p : progs) {
        defer_wgrads(p);
        defer_folds(p);
        int rc = launch_program(c, p);
        if (rc) return rc;
      }
    } else {
      // cyclic: the passes of a tick touch distinct micro-batches and never two backwards of
      // one stage, so their launch lists merge level by level into grouped launches
      Program merged;
      for (auto& p : progs) {
        if (merged.size() < p.size()) merged.resize(p.size());
        for (size_t l = 0; l < p.size(); ++l) merged[l].insert(merged[l].end(), p[l].begin(), p[l].end());
      }
      defer_wgrads(merged);
      defer_folds(merged);
      int rc = launch_program(c, merged);
      if (rc) return rc;
    }
  }
  for (const Block& b : c->deferred) c->pool.release(b);
  c->deferred.clear();
  c->scratch_bump = 0;
  c->stats.cur_activation_bytes = c->pool.in_use;
  // SGD update of every stage that now holds N gradients (end of tick)
  for (int j = 0; j < S; ++j) {
    StageState& ss = c->st[j];
    if (ss.cnt != N) continue;
    const int nv = ss.ver + 1;
    if (!c->dry) {
      int rc = refresh_slot(c, j, nv & 1, true, fused[j] != 0);
      if (rc) return rc;
    }
    ss.ring_ver[nv & 1] = nv;
    ss.ver = nv;
    ss.cnt = 0;
  }
  c->tick++;
  c->stats.ticks_run = c->tick;
  c->stats.steps_enqueued = c->steps_enqueued;
  // a fully drained timeline restarts its cycle at the next tick
  if (inflight(c) == 0) {
    bool any = false;
    for (int i = 0; i < N && !any; ++i)
      for (int j = 0; j < S && !any; ++j) any = c->rec[i][j].live;
    if (!any) { c->origin_tick = c->tick; c->origin_step = c->steps_enqueued; }
  }
  return CDP_OK;
}

int check_args(const cdp_stage_desc* stages, int n_stages, int N, int B, int rule, const cdp_opts* opts, ModelPlan* plan) {
  if (!stages || !opts) return fail(nullptr, CDP_EINVAL, "stages/opts is NULL");
  if (N <= 0 || B <= 0) return fail(nullptr, CDP_EINVAL, "N and micro_batch must be positive");
  if (rule != CDP_RULE_DP && rule != CDP_RULE_V1 && rule != CDP_RULE_V2 && rule != CDP_RULE_MASK)
    return fail(nullptr, CDP_EINVAL, "unknown update rule");
  if ((rule == CDP_RULE_MASK) != (opts->fresh_mask != nullptr))
    return fail(nullptr, CDP_EINVAL, "fresh_mask is needed by, and only by, CDP_RULE_MASK");
  if (opts->bwd_fresh && opts->dp_batched) return fail(nullptr, CDP_EINVAL, "bwd_fresh cannot be combined with dp_batched");
  if (rule != CDP_RULE_DP && (2 * n_stages) % N != 0)
    return fail(nullptr, CDP_EINVAL, "the cyclic schedule needs N to divide 2S (uniform delay d = 2S/N)");
  std::string e = build_plan(stages, n_stages, opts, plan);
  if (!e.empty()) return fail(nullptr, CDP_EINVAL, e);
  if (!(opts->momentum >= 0.f && opts->momentum < 1.f) || !(opts->weight_decay >= 0.f))
    return fail(nullptr, CDP_EINVAL, "momentum must be in [0, 1) and weight_decay >= 0");
  if (opts->dp_batched && rule != CDP_RULE_DP) return fail(nullptr, CDP_EINVAL, "dp_batched needs CDP_RULE_DP");
  if (opts->dp_batched && N > 256) return fail(nullptr, CDP_EINVAL, "dp_batched supports at most 256 micro-batches");
  if (opts->dw_group < 0 || opts->dw_group > DW_GROUP_MAX || (opts->dw_group > 1 && (rule == CDP_RULE_DP || N % opts->dw_group != 0)))
    return fail(nullptr, CDP_EINVAL, "dw_group must be 0 or 1 (off) or a divisor of N up to 4, with a cyclic rule");
  if ((int64_t)B * (opts->dp_batched ? N : 1) > 1024 && plan->stages.back().has_head)
    return fail(nullptr, CDP_EINVAL, "a head pass over more than 1024 rows is not supported");
  return CDP_OK;
}

int make_ctx(cdp_ctx** out, const cdp_stage_desc* stages, int n_stages, int N, int B, float lr, int rule, const cdp_opts* opts,
             bool force_dry) {
  cdp_ctx* c = new cdp_ctx();
  int rc = check_args(stages, n_stages, N, B, rule, opts, &c->plan);
  if (rc) { delete c; return rc; }
  if (opts->dp_batched) {
    // lock-step executor: one pass per stage over all N*B rows; f = (1/N) sum_i f_i is the mean
    // loss over those rows, so the update of Eq. (DP) is that of a single micro-batch
    c->groups = N;
    B *= N;
    N = 1;
  }
  if (rule == CDP_RULE_MASK) c->fresh_mask.assign(opts->fresh_mask, opts->fresh_mask + (size_t)N * n_stages);
  c->bwd_fresh = opts->bwd_fresh != 0;
  c->dw_group = opts->dw_group > 1 ? opts->dw_group : 1;
  c->S = n_stages; c->N = N; c->B = B; c->rule = rule; c->lr = lr;
  c->d = rule == CDP_RULE_DP ? 0 : 2 * n_stages / N;
  c->dry = force_dry || opts->dry_run != 0;
  c->stream = static_cast<hipStream_t>(opts->hip_stream);
  // a dry run never touches memory; a non-null stand-in base keeps the address arithmetic of the
  // launch lists well defined
  c->arena = c->dry ? reinterpret_cast<char*>(uintptr_t(1) << 30) : static_cast<char*>(opts->arena);
  c->arena_bytes = (int64_t)opts->arena_bytes;
  c->momentum = opts->momentum; c->weight_decay = opts->weight_decay;
  StaticLayout L = static_layout(c->plan, N, B, c->groups, c->momentum != 0.f);
  c->st = L.st;
  c->labels_off = L.labels_off; c->loss_off = L.loss_off; c->thin_ws_off = L.thin_ws_off; c->conv_ws_off = L.conv_ws_off; c->fold_cnt_off = L.fold_cnt_off;
  c->pool.base = L.pool_base;
  c->pool.cap = c->dry ? -1 : c->arena_bytes - L.pool_base;
  c->rec.assign(N, std::vector<VisitRecord>(n_stages));
  c->carry.assign(N, Block());
  c->pending.assign(n_stages, {});
  c->heads_done.assign(LOSS_LOG_STEPS, 0);
  memset(&c->stats, 0, sizeof(c->stats));
  c->stats.weight_bytes = L.weight_bytes;
  const TensorInfo& t0 = c->plan.stages[0].tensors[0];
  c->in_features = t0.per_sample();
  // lock-step DP keeps every stage input of every micro-batch at the end of the forward pass
  int64_t dp = 0;
  for (const StagePlan& sp : c->plan.stages)
    for (size_t k = 0; k + 1 < sp.tensors.size(); ++k)
      if (sp.tensors[k].consumed && !sp.tensors[k].f32) dp += align_up(tensor_bytes(c, sp.tensors[k]), 256);
  c->stats.dp_activation_bytes = dp * N;
  *out = c;
  return CDP_OK;
}

}  // namespace

// =============================================================================== C ABI
extern "C" {

// Dry simulation of the timeline: the pool and the tick workspace are deterministic, so the
// footprint found here is the footprint of the real run.
static int simulate_footprint(const cdp_stage_desc* stages, int n_stages, int N, int B, int rule, const cdp_opts* opts,
                              int64_t* pool_base, int64_t* pool_span, int64_t* scratch_peak) {
  cdp_ctx* c = nullptr;
  int rc = make_ctx(&c, stages, n_stages, N, B, 0.f, rule, opts, true);
  if (rc) return rc;
  const float* fake_x = reinterpret_cast<const float*>(uintptr_t(256));
  const int32_t* fake_y = reinterpret_cast<const int32_t*>(uintptr_t(256));
  const int steps = 4;
  for (int t = 0; t < steps && rc == CDP_OK; ++t)
    for (int k = 0; k < 2 * n_stages && rc == CDP_OK; ++k) rc = run_tick(c, fake_x, fake_y);
  while (rc == CDP_OK && inflight(c) > 0) rc = run_tick(c, nullptr, nullptr);
  if (rc == CDP_OK) {
    *pool_base = c->pool.base;
    *pool_span = align_up(c->pool.bump, 256);
    *scratch_peak = align_up(c->stats.scratch_bytes, 256);
  } else {
    g_last_error = c->err;
  }
  delete c;
  return rc;
}

int cdp_arena_bytes(const cdp_stage_desc* stages, int n_stages, int N, int B, int rule, const cdp_opts* opts, size_t* bytes_out) {
  if (!bytes_out) return fail(nullptr, CDP_EINVAL, "bytes_out is NULL");
  int64_t base = 0, span = 0, scratch = 0;
  int rc = simulate_footprint(stages, n_stages, N, B, rule, opts, &base, &span, &scratch);
  if (rc == CDP_OK) *bytes_out = (size_t)(base + span + scratch + 256);
  return rc;
}

int cdp_init(cdp_ctx** out, const cdp_stage_desc* stages, int n_stages, int N, int B, float lr, int rule, const cdp_opts* opts) {
  if (!out) return fail(nullptr, CDP_EINVAL, "out is NULL");
  *out = nullptr;
  cdp_ctx* c = nullptr;
  int rc = make_ctx(&c, stages, n_stages, N, B, lr, rule, opts, false);
  if (rc) return rc;
  if (!c->dry) {
    int64_t base = 0, span = 0, scratch = 0;
    rc = simulate_footprint(stages, n_stages, N, B, rule, opts, &base, &span, &scratch);
    if (rc) { delete c; return rc; }
    const size_t need = (size_t)(base + span + scratch + 256);
    c->pool.cap = span;
    c->scratch_base = base + span;
    c->scratch_cap = scratch;
    if (!opts->arena || (reinterpret_cast<uintptr_t>(opts->arena) & 255) != 0) {
      delete c;
      return fail(nullptr, CDP_EINVAL, "arena must be a 256-byte aligned device pointer");
    }
    if (opts->arena_bytes < need) {
      delete c;
      return fail(nullptr, CDP_ENOMEM, "arena too small: need " + std::to_string(need) + " bytes");
    }
    // accumulators and the loss log start at zero; weights are zero until cdp_set_weights
    hipError_t e = hipMemsetAsync(c->arena, 0, (size_t)c->pool.base, c->stream);
    if (e != hipSuccess) {
      std::string m = std::string("hipMemsetAsync: ") + hipGetErrorString(e);
      delete c;
      return fail(nullptr, CDP_EHIP, m);
    }
  }
  *out = c;
  return CDP_OK;
}

int cdp_param_count(const cdp_ctx* c, int stage, size_t* n_out) {
  if (!c || !n_out || stage < 0 || stage >= c->S) return fail(nullptr, CDP_EINVAL, "bad argument");
  *n_out = (size_t)c->plan.stages[stage].n_params;
  return CDP_OK;
}

int cdp_set_weights(cdp_ctx* c, int stage, const float* host, size_t n) {
  if (!c) return fail(nullptr, CDP_EINVAL, "ctx is NULL");
  if (stage < 0 || stage >= c->S || !host) return fail(c, CDP_EINVAL, "bad stage or NULL weights");
  if (n != (size_t)c->plan.stages[stage].n_params) return fail(c, CDP_EINVAL, "weight count does not match the stage");
  if (c->weights_locked) return fail(c, CDP_ESTATE, "weights can only be set before the first tick");
  if (c->dry) return CDP_OK;
  HIP_TRY(c, hipMemcpyAsync(c->fptr(c->st[stage].master), host, n * 4, hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int s = 0; s < 2; ++s) {
    int rc = refresh_slot(c, stage, s, false);
    if (rc) return rc;
  }
  return CDP_OK;
}

// A tick that fails after it has started to change the timeline state (counters, records, pool) cannot be
// retried: the context refuses further ticks.  A failure before any change leaves the context as it was.
static int guarded_tick(cdp_ctx* c, const float* x_dev, const int32_t* y_dev) {
  if (c->poisoned) return fail(c, CDP_ESTATE, "an earlier tick failed half-way; the context can only be read and destroyed");
  const int64_t enq = c->steps_enqueued;
  const size_t ticks_logged = c->live_counts.size();
  const int rc = run_tick(c, x_dev, y_dev);
  if (rc != CDP_OK && (c->steps_enqueued != enq || c->live_counts.size() != ticks_logged)) c->poisoned = true;
  return rc;
}

int cdp_tick(cdp_ctx* c, const float* x_dev, const int32_t* y_dev) {
  if (!c) return fail(nullptr, CDP_EINVAL, "ctx is NULL");
  return guarded_tick(c, x_dev, y_dev);
}

int cdp_step(cdp_ctx* c, const float* x_dev, const int32_t* y_dev) {
  if (!c) return fail(nullptr, CDP_EINVAL, "ctx is NULL");
  if (!x_dev || !y_dev) return fail(c, CDP_EINVAL, "x_dev / y_dev is NULL");
  if ((c->tick - c->origin_tick) % (2 * c->S) != 0) return fail(c, CDP_ESTATE, "cdp_step must start on a step boundary");
  for (int k = 0; k < 2 * c->S; ++k) {
    int rc = guarded_tick(c, x_dev, y_dev);
    if (rc) return rc;
  }
  return CDP_OK;
}

int cdp_drain(cdp_ctx* c) {
  if (!c) return fail(nullptr, CDP_EINVAL, "ctx is NULL");
  // finish the started step boundary bookkeeping: no new mini-batch is enqueued, so the
  // remaining passes are exactly those of micro-batches already in flight
  int guard = 4 * c->S + c->d * c->N + 4;
  while (inflight(c) > 0 && guard-- > 0) {
    int rc = guarded_tick(c, nullptr, nullptr);
    if (rc) return rc;
  }
  return CDP_OK;
}

int cdp_get_weights(cdp_ctx* c, int stage, int version, float* host, size_t cap, size_t* n_out) {
  if (!c) return fail(nullptr, CDP_EINVAL, "ctx is NULL");
  if (stage < 0 || stage >= c->S || !host) return fail(c, CDP_EINVAL, "bad stage or NULL buffer");
  const StagePlan& sp = c->plan.stages[stage];
  const StageState& ss = c->st[stage];
  if (n_out) *n_out = (size_t)sp.n_params;
  if (cap < (size_t)sp.n_params) return fail(c, CDP_EINVAL, "buffer too small");
  if (version < 0) version = ss.ver;
  if (c->dry) return fail(c, CDP_ESTATE, "no weights in a dry run");
  if (version == ss.ver) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(host, c->fptr(ss.master), (size_t)sp.n_params * 4, hipMemcpyDeviceToHost));
    return CDP_OK;
  }
  if (version != ss.ver - 1 || ss.ring_ver[version & 1] != version) return fail(c, CDP_ESTATE, "that weight version is no longer in the ring");
  if (sp.has_gamma) return fail(c, CDP_ESTATE, "ring copies of stages with affine layers are folded and cannot be read back");
  for (const Op& o : sp.ops)
    if (o.kpad) return fail(c, CDP_ESTATE, "ring copies of im2col layers are padded and cannot be read back");
  float* tmp = nullptr;
  HIP_TRY(c, hipMalloc(reinterpret_cast<void**>(&tmp), (size_t)sp.n_params * 4));
  const char* sl = static_cast<const char*>(c->ptr(ss.slot[version & 1]));
  hipError_t e = hipSuccess;
  for (const Op& o : sp.ops) {
    if (o.kind != OPK_GEMM) continue;
    if (e == hipSuccess) e = launch_to_f32(sl + o.wf, tmp + o.w_off, o.w_count(), c->plan.dtype, c->stream);
    if (e == hipSuccess && o.b_off >= 0)
      e = hipMemcpyAsync(tmp + o.b_off, sl + o.bias_c, (size_t)o.Cout * 4, hipMemcpyDeviceToDevice, c->stream);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e == hipSuccess) e = hipMemcpy(host, tmp, (size_t)sp.n_params * 4, hipMemcpyDeviceToHost);
  (void)hipFree(tmp);
  if (e != hipSuccess) return fail(c, CDP_EHIP, std::string("cdp_get_weights: ") + hipGetErrorString(e));
  return CDP_OK;
}

int cdp_get_losses(cdp_ctx* c, int64_t step, float* host, size_t cap) {
  if (!c || !host) return fail(c, CDP_EINVAL, "bad argument");
  const size_t n_loss = (size_t)c->N * c->groups;
  if (cap < n_loss) return fail(c, CDP_EINVAL, "buffer too small");
  if (step < 0 || step >= c->steps_enqueued || step + LOSS_LOG_STEPS <= c->steps_enqueued - 1)
    return fail(c, CDP_ESTATE, "step is not in the loss log");
  if (c->heads_done[step % LOSS_LOG_STEPS] < c->N) return fail(c, CDP_ESTATE, "not every micro-batch of that step has reached the head yet");
  if (c->dry) return fail(c, CDP_ESTATE, "no losses in a dry run");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  std::vector<int32_t> fixed(n_loss);  // the slots hold fixed-point sums (LOSS_SCALE)
  HIP_TRY(c, hipMemcpy(fixed.data(), c->fptr(c->loss_off) + (step % LOSS_LOG_STEPS) * n_loss, n_loss * 4, hipMemcpyDeviceToHost));
  for (size_t k = 0; k < n_loss; ++k) host[k] = (float)((double)fixed[k] / (double)LOSS_SCALE);
  return CDP_OK;
}

int cdp_get_trace(const cdp_ctx* c, cdp_trace_rec* out, size_t cap, size_t* n_out) {
  if (!c) return fail(nullptr, CDP_EINVAL, "ctx is NULL");
  if (n_out) *n_out = c->trace.size();
  if (out) memcpy(out, c->trace.data(), std::min(cap, c->trace.size()) * sizeof(cdp_trace_rec));
  return CDP_OK;
}

int cdp_get_live_counts(const cdp_ctx* c, int32_t* out, size_t cap, size_t* n_out) {
  if (!c) return fail(nullptr, CDP_EINVAL, "ctx is NULL");
  if (n_out) *n_out = c->live_counts.size();
  if (out) memcpy(out, c->live_counts.data(), std::min(cap, c->live_counts.size()) * sizeof(int32_t));
  return CDP_OK;
}

int cdp_get_live_bytes(const cdp_ctx* c, int kind, int64_t* out, size_t cap, size_t* n_out) {
  if (!c || kind < 0 || kind > 1) return fail(nullptr, CDP_EINVAL, "bad argument");
  const std::vector<int64_t>& v = c->live_bytes[kind];
  if (n_out) *n_out = v.size();
  if (out) memcpy(out, v.data(), std::min(cap, v.size()) * sizeof(int64_t));
  return CDP_OK;
}

int cdp_get_stats(const cdp_ctx* c, cdp_stats* out) {
  if (!c || !out) return fail(nullptr, CDP_EINVAL, "bad argument");
  *out = c->stats;
  return CDP_OK;
}

int cdp_profile_gemm(cdp_ctx* c, int enable) {
  if (!c) return fail(nullptr, CDP_EINVAL, "ctx is NULL");
  if (c->dry) return fail(c, CDP_ESTATE, "nothing to time in a dry run");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (auto& r : c->prof) { c->event_pool.push_back(r.a); c->event_pool.push_back(r.b); }
  c->prof.clear();
  c->profiling = enable != 0;
  if (c->profiling) {
    // the bracket's own cost: event pairs with nothing between them, median of 32
    constexpr int PAIRS = 32;
    hipEvent_t ev[2 * PAIRS];
    for (int k = 0; k < 2 * PAIRS; ++k) {
      if (!c->event_pool.empty()) { ev[k] = c->event_pool.back(); c->event_pool.pop_back(); }
      else HIP_TRY(c, hipEventCreate(&ev[k]));
    }
    for (int k = 0; k < 2 * PAIRS; ++k) HIP_TRY(c, hipEventRecord(ev[k], c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    std::vector<float> gap(PAIRS);
    for (int k = 0; k < PAIRS; ++k) HIP_TRY(c, hipEventElapsedTime(&gap[k], ev[2 * k], ev[2 * k + 1]));
    std::sort(gap.begin(), gap.end());
    c->empty_pair_ms = gap[PAIRS / 2];
    for (int k = 0; k < 2 * PAIRS; ++k) c->event_pool.push_back(ev[k]);
  }
  return CDP_OK;
}

int cdp_get_gemm_profile(cdp_ctx* c, cdp_gemm_profile* out) {
  if (!c || !out) return fail(c, CDP_EINVAL, "bad argument");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  memset(out, 0, sizeof(*out));
  for (auto& r : c->prof) {
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, r.a, r.b));
    out->launches++;
    out->total_ms += ms;
    out->flops += r.flops;
    out->bytes += r.bytes;
  }
  out->empty_pair_ms = c->empty_pair_ms;
  return CDP_OK;
}

const char* cdp_last_error(const cdp_ctx* c) { return c ? c->err.c_str() : g_last_error.c_str(); }

void cdp_destroy(cdp_ctx* c) {
  if (!c) return;
  for (auto& r : c->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
  delete c;
}

}  // extern "C"
