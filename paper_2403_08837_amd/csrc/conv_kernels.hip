// Implicit-GEMM convolution passes of a CDP tick on gfx950, for channel counts that are a
// multiple of the reduction slab (bf16: 32, fp32: 16); other shapes (the 3-channel stem)
// run on the generic kernel of gemm.hip.
//
//   conv_gemm_kernel   forward   y[(b,oh,ow)][o]  = sum_{tap,c} x[b][oh*s-p+kh][ow*s-p+kw][c] * wf[o][tap][c]
//                      data grad dx[(b,ih,iw)][c] = sum_{tap,o} dy[b][(ih+p-kh)/s][(iw+p-kw)/s][o] * wt[c][tap][o]
//     A slab of the reduction lies inside one tap, so the tap and its address delta are
//     wavefront-uniform; each thread keeps, per tile row it loads, one base offset and one
//     bit per tap (inside the image / on the stride lattice).  No division in the k-loop.
//   conv_wgrad_kernel  part[range][o][(tap,c)] = sum_{m in range} dy[m][o] * x[pos(m)+tap][c]
//     reduction over output positions, cut into ranges that write partial tiles with plain
//     stores; operands are staged as they lie in memory ([m][channels]) and MFMA fragments are
//     read transposed out of LDS; the per-position address decode is done once per workgroup
//     into an LDS table.  wgrad_reduce_kernel folds the ranges into G (scaled by gamma) and
//     produces d gamma and d beta.
#include <algorithm>

#include "elem.h"
#include "kernels.h"
#include "mfma_frag.h"

namespace cdp {

// Consecutive logical tiles that one XCD takes in a row (xcd_block_cyclic); measured on the ResNet-50 and ViT-B/16
// shaped workloads: 4, 8 and 16 within 0.5 % of each other in time, L2 misses of the forward / data-gradient
// kernel 26 % below the round-robin order.
constexpr int XCD_RUN = 8;

// ---------------------------------------------------------------------------------
// forward / data gradient: 128 x BN tile, waves 2 x 2, reduction slab BK (a divisor of the
// channel count).  The epilogue goes through LDS so that results, residuals and masks move
// as 16-byte vectors along the channel dimension.
template <typename T, int BM, int BN, int BK, bool DB>
__global__ __launch_bounds__(256) void conv_gemm_kernel(const GemmBatch batch) {
  using E = Elem<T>;
  constexpr int VEC = E::VEC, LDP = BK + VEC;
  constexpr int WTM = BM / 2, MI = WTM / 32;   // wave tile WTM x WTN
  constexpr int CPR = BK / VEC;                // chunks per tile row
  constexpr int NA = BM * CPR / 256;           // A chunks per thread
  constexpr int NB = BN * CPR / 256;           // B chunks per thread
  constexpr int WTN = BN / 2, NI = WTN / 32;
  constexpr int SP = WTN + 4;                  // pitch (floats) of a wave's 32-row staging area
  // one or two (DB) operand buffers; the epilogue staging reuses the space.
  // Size: conv_gemm_lds_bytes<T, BM, BN, BK, DB>().
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int BUF = (BM + BN) * LDP;  // elements per operand buffer
  T* const As0 = reinterpret_cast<T*>(smem);

  // runs of XCD_RUN neighbouring tiles (same rows, next columns; then the next rows, whose 3x3 halo they share) on one XCD
  const int tile = xcd_block_cyclic((int)blockIdx.x, batch.total_tiles, XCD_RUN);
  const GemmProb& P = batch.p[find_problem(batch, tile)];
  // a long reduction of a small launch is shared by P.splits workgroups (neighbours in the
  // tile list); the last of them to finish adds the partial tiles and runs the epilogue
  constexpr bool SPLIT = BM == 64 && BN == 64;  // the launcher splits only launches of the smallest tiles
  const int ks = SPLIT ? P.splits : 1, split = (tile - P.tile_begin) % ks;
  const int local = (tile - P.tile_begin) / ks;
  const int tn = local % P.tiles_n, tm = local / P.tiles_n;
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const T* __restrict__ Ap = static_cast<const T*>(P.A);
  const T* __restrict__ Bp = static_cast<const T*>(P.B);
  const ConvGeom g = P.g;
  const int mode = P.a_mode;
  const int C = (mode == OP_PLAIN_K) ? P.K : g.C;  // channels per tap of the gathered tensor

  // per-row state of the A chunks this thread loads
  const int arow = tid / CPR, akc = (tid % CPR) * VEC;
  int abase[NA];
  unsigned amask[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int r = row0 + arow + i * (256 / CPR);
    abase[i] = 0;
    amask[i] = 0;
    if (r < P.M) {
      if (mode == OP_PLAIN_K) {
        abase[i] = r * P.lda;
        amask[i] = 1u;
      } else {
        const int b = r / (g.OH * g.OW);
        const int rem = r - b * (g.OH * g.OW);
        const int oh = rem / g.OW, ow = rem - oh * g.OW;
        if (mode == OP_CONV_FWD) {
          const int ih0 = oh * g.stride - g.pad, iw0 = ow * g.stride - g.pad;
          abase[i] = ((b * g.H + ih0) * g.W + iw0) * g.C;
          // taps inside the image: the columns kw with 0 <= iw0 + kw < W, for every row kh with 0 <= ih0 + kh < H
          const int kw_lo = max(0, -iw0), kw_hi = min(g.KW, g.W - iw0);
          const unsigned cols = kw_hi > kw_lo ? ((1u << kw_hi) - 1u) & ~((1u << kw_lo) - 1u) : 0u;
          for (int kh = max(0, -ih0); kh < min(g.KH, g.H - ih0); ++kh) amask[i] |= cols << (kh * g.KW);
        } else {  // OP_CONV_DGRAD: (oh, ow) is an input position, the gathered tensor is dy
          const int qh = (oh + g.pad) / g.stride, eh = (oh + g.pad) - qh * g.stride;
          const int qw = (ow + g.pad) / g.stride, ew = (ow + g.pad) - qw * g.stride;
          abase[i] = ((b * g.H + qh) * g.W + qw) * g.C;
          for (int kh = 0; kh < g.KH; ++kh)
            for (int kw = 0; kw < g.KW; ++kw) {
              const int uh = kh / g.stride, uw = kw / g.stride;
              if (kh - uh * g.stride == eh && kw - uw * g.stride == ew && qh - uh >= 0 && qh - uh < g.H && qw - uw >= 0 &&
                  qw - uw < g.W)
                amask[i] |= 1u << (kh * g.KW + kw);
            }
        }
      }
    }
  }
  const int brow = tid / CPR;
  int boff[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int r = col0 + brow + i * (256 / CPR);
    boff[i] = r < P.N ? r * P.ldb + akc : -1;
  }

  uint4 ra[NA], rb[NB];
  // wavefront-uniform position of the current slab: tap index, channel offset inside the tap
  const int nslab_all = P.K / BK, per = (nslab_all + ks - 1) / ks;
  const int s_begin = split * per, nslab = max(0, min(nslab_all, s_begin + per) - s_begin);
  const int kbeg = s_begin * BK;
  int tap = kbeg / C, c0 = kbeg - tap * C, kh = 0, kw = 0;
  if (mode != OP_PLAIN_K) { kh = tap / g.KW; kw = tap - kh * g.KW; }
  auto fetch = [&](int k0) {
    int delta;
    if (mode == OP_PLAIN_K) delta = c0;
    else if (mode == OP_CONV_FWD) delta = (kh * g.W + kw) * g.C + c0;
    else delta = -((kh / g.stride) * g.W + (kw / g.stride)) * g.C + c0;
#pragma unroll
    for (int i = 0; i < NA; ++i)
      ra[i] = ((amask[i] >> tap) & 1u) ? *reinterpret_cast<const uint4*>(Ap + abase[i] + delta + akc) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < NB; ++i) rb[i] = boff[i] >= 0 ? *reinterpret_cast<const uint4*>(Bp + boff[i] + k0) : make_uint4(0, 0, 0, 0);
    c0 += BK;
    if (c0 == C) {
      c0 = 0;
      ++tap;
      if (++kw == g.KW) { kw = 0; ++kh; }
    }
  };

  v16f_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  auto stash = [&](int buf) {  // registers -> operand buffer `buf`
    T* As = As0 + buf * BUF;
    T* Bs = As + BM * LDP;
#pragma unroll
    for (int i = 0; i < NA; ++i) *reinterpret_cast<uint4*>(As + (arow + i * (256 / CPR)) * LDP + akc) = ra[i];
#pragma unroll
    for (int i = 0; i < NB; ++i) *reinterpret_cast<uint4*>(Bs + (brow + i * (256 / CPR)) * LDP + akc) = rb[i];
  };
  auto contract = [&](const T* As) {
    const T* Bs = As + BM * LDP;
    const int kg = (lane >> 5) * E::KPL;
    const T* ap = As + (wm * WTM + (lane & 31)) * LDP + kg;
    const T* bp = Bs + (wn * WTN + (lane & 31)) * LDP + kg;
#pragma unroll
    for (int kk = 0; kk < BK; kk += E::MFMA_K) {
      if constexpr (sizeof(T) == 2) {
        uint4 a[MI], b[NI];
#pragma unroll
        for (int i = 0; i < MI; ++i) a[i] = *reinterpret_cast<const uint4*>(ap + i * 32 * LDP + kk);
#pragma unroll
        for (int j = 0; j < NI; ++j) b[j] = *reinterpret_cast<const uint4*>(bp + j * 32 * LDP + kk);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j) acc[i][j] = mfma_bf16(a[i], b[j], acc[i][j]);
      } else {
        float a[MI], b[NI];
#pragma unroll
        for (int i = 0; i < MI; ++i) a[i] = ap[i * 32 * LDP + kk];
#pragma unroll
        for (int j = 0; j < NI; ++j) b[j] = bp[j * 32 * LDP + kk];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    }
  };
  if constexpr (DB) {
    // Two operand buffers (small problems, whose k-loop is a chain of latencies): while slab
    // `it` is contracted out of one buffer the loads of slab it+1 are in flight; they are
    // written to the other buffer after the contraction and the loads of slab it+2 are
    // issued.  One barrier per slab.
    if (nslab > 0) {
      fetch(kbeg);
      stash(0);
    }
    if (nslab > 1) fetch(kbeg + BK);
    __syncthreads();
    for (int it = 0; it < nslab; ++it) {
      contract(As0 + (it & 1) * BUF);
      if (it + 1 < nslab) {
        stash((it + 1) & 1);  // last read in iteration it-1, which every wave has left (barrier below)
        if (it + 2 < nslab) fetch(kbeg + (it + 2) * BK);
      }
      __syncthreads();
    }
  } else {
    // One operand buffer (large launches, where more workgroups per CU hide the latency):
    // the next slab's loads are in flight while the current one is contracted.
    if (nslab > 0) fetch(kbeg);
    for (int it = 0; it < nslab; ++it) {
      __syncthreads();
      stash(0);
      __syncthreads();
      if (it + 1 < nslab) fetch(kbeg + (it + 1) * BK);
      contract(As0);
    }
  }

  // The epilogue's own operand (forward: the residual, data gradient: the ReLU mask) for all of the tile's
  // staging passes is requested here in one go, into the registers the operand prefetch no longer needs: its
  // round trip to memory overlaps the staging of the first pass instead of being paid once per pass (what
  // counts for the short reductions of the 1x1 layers, whose tiles are a chain of memory latencies).
  constexpr int CPS = WTN / VEC;             // chunks per staged row of the epilogue
  constexpr int NCH = 32 * CPS / 64;         // chunks per lane and pass
  uint4 pa[MI][NCH];
  float bias[VEC];  // forward: the bias of this lane's columns (the same columns in every pass and chunk: CPS divides 64)
  static_assert(64 % CPS == 0, "a lane keeps its columns from chunk to chunk");
  if (P.epi == EPI_FWD && P.aux0) {
    const int c = col0 + wn * WTN + (lane % CPS) * VEC;
#pragma unroll
    for (int e = 0; e < VEC; ++e) bias[e] = c < P.N ? static_cast<const float*>(P.aux0)[c + e] : 0.f;
  }
  if (P.aux1) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int t = 0; t < NCH; ++t) {
        const int q = lane + 64 * t;
        const int r = row0 + wm * WTM + i * 32 + q / CPS, c = col0 + wn * WTN + (q % CPS) * VEC;
        pa[i][t] = (r < P.M && c < P.N) ? *reinterpret_cast<const uint4*>(static_cast<const T*>(P.aux1) + (int64_t)r * P.ldo + c)
                                        : make_uint4(0, 0, 0, 0);
      }
  }

  if (SPLIT && ks > 1) {
    // Partial tile -> this workgroup's slot of the workspace, in register order (lane-contiguous).
    // Partials and counter are device-scope atomics (they bypass the per-XCD L2) ordered by
    // waiting for the stores; the last arrival sums the slots in a fixed order.
    float* slot = batch.thin_ws + (int64_t)tile * (BM * BN);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          __hip_atomic_store(slot + ((i * NI + j) * 16 + v) * 256 + tid, acc[i][j][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // every store above has been acknowledged before this wavefront reaches the barrier (a
    // workgroup-scope fence alone does not wait for global stores)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();  // also: the operand tiles are no longer read
    unsigned int* cnt = batch.thin_cnt + (tile - split);
    int* flag = reinterpret_cast<int*>(smem);
    if (tid == 0) {
      const unsigned int arrived = atomicAdd(cnt, 1u);
      *flag = arrived == (unsigned)(ks - 1);
      if (arrived == (unsigned)(ks - 1)) atomicExch(cnt, 0u);  // ready for the next launch
    }
    __syncthreads();
    if (!*flag) return;
    const float* first = batch.thin_ws + (int64_t)(tile - split) * (BM * BN);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    // one round trip per group of four slots: all their loads are issued together, then added in slot order
    constexpr int GS = 4, PE = MI * NI * 16;
    for (int sp = 0; sp < ks; sp += GS) {
      float part[GS][PE];
#pragma unroll
      for (int u = 0; u < GS; ++u) {
        const float* src = first + (int64_t)min(sp + u, ks - 1) * (BM * BN) + tid;  // (past the last slot: a harmless re-read)
#pragma unroll
        for (int e = 0; e < PE; ++e) part[u][e] = __hip_atomic_load(src + e * 256, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
#pragma unroll
      for (int u = 0; u < GS; ++u)
        if (sp + u < ks) {
#pragma unroll
          for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
              for (int v = 0; v < 16; ++v) acc[i][j][v] += part[u][(i * NI + j) * 16 + v];
        }
    }
  }

  // ---- epilogue: 32 rows of the wave tile at a time through LDS (fp32), then 16-byte rows
  const int flags = P.flags;
  const bool fwd = P.epi == EPI_FWD;
  float* stage = reinterpret_cast<float*>(smem) + wave * (32 * SP);
  T* outp = static_cast<T*>(P.out);
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    __syncthreads();  // operand tiles (first pass) or the previous staging pass are consumed
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) stage[((v >> 2) * 8 + (lane >> 5) * 4 + (v & 3)) * SP + j * 32 + (lane & 31)] = acc[i][j][v];
    __syncthreads();
#pragma unroll
    for (int t = 0; t < NCH; ++t) {
      const int q = lane + 64 * t;
      const int sr = q / CPS, sc = (q % CPS) * VEC;
      const int r = row0 + wm * WTM + i * 32 + sr, c = col0 + wn * WTN + sc;
      if (r >= P.M || c >= P.N) continue;  // N is a multiple of VEC on this path
      const int64_t o = (int64_t)r * P.ldo + c;
      float val[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) val[e] = stage[sr * SP + sc + e];
      Chunk16<T> x0, x1, x2, res;
      if (fwd) {
        if (P.aux0) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] += bias[e];
        }
        if (P.aux1) {
          x1.v = pa[i][t];
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] += E::to_f32(x1.e[e]);
        }
        if (flags & GF_RELU) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] = fmaxf(val[e], 0.f);
        }
      } else {
        if (P.aux0) {
          x0.v = *reinterpret_cast<const uint4*>(static_cast<const T*>(P.aux0) + o);
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] += E::to_f32(x0.e[e]);
        }
        if (flags & GF_ACCUM) {
          x2.v = *reinterpret_cast<const uint4*>(outp + o);
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] += E::to_f32(x2.e[e]);
        }
        if (P.aux1) {
          x1.v = pa[i][t];
#pragma unroll
          for (int e = 0; e < VEC; ++e)
            if (!(E::to_f32(x1.e[e]) > 0.f)) val[e] = 0.f;
        }
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) res.e[e] = E::from_f32(val[e]);
      *reinterpret_cast<uint4*>(outp + o) = res.v;
    }
  }
}

// ---------------------------------------------------------------------------------
// weight gradient.  Batch entry convention (as for the generic kernel): A = dy [Mpos][Cout]
// (OP_PLAIN_R, lda = Cout), B = x (OP_CONV_WGRAD geometry, or OP_PLAIN_R with ldb = Cin for a
// 1x1/stride-1 layer), out = G [Cout][taps*Cin] (ldo = taps*Cin), P.M = Cout, P.N = taps*Cin,
// P.K = Mpos, splits = number of reduction ranges.  Each range writes its partial tile with plain
// stores: out = partial sums f32 [splits][Cout][taps*Cin], aux3 = partial column sums of dy
// f32 [splits][Cout] or NULL.  wgrad_reduce_kernel folds the partials into the accumulators
// (device-wide atomics on a small hot array are an order of magnitude slower than this).
constexpr int WG_MAX_SLABS = 16;  // slabs per chunk of a workgroup's range (size of the LDS position table)
template <typename T> struct WgSlab { static constexpr int MB = sizeof(T) == 2 ? 64 : 32; };  // positions per slab
static inline int wg_slab(int dtype) { return dtype == DT_BF16 ? 64 : 32; }

// One tile (TO rows of the weight matrix x 128 columns, one reduction range) of problem P; Ds [MB][TO + PAD],
// Xs [MB][128 + PAD] and the two position tables [WG_MAX_SLABS * MB] are the workgroup's LDS.
template <typename T, int TO>
__device__ __forceinline__ void conv_wgrad_body(const GemmProb& P, int tile, T* __restrict__ Ds, T* __restrict__ Xs,
                                                int* __restrict__ pos_base, int* __restrict__ pos_hw) {
  using E = Elem<T>;
  constexpr int TC = 128, VEC = E::VEC, MB = WgSlab<T>::MB;
  constexpr int PAD = (sizeof(T) == 2) ? 16 : 4;  // bf16: pitch of 32 bytes modulo 128 for the transposing LDS read
  constexpr int PD = TO + PAD, PX = TC + PAD;  // LDS pitches (elements)
  constexpr int WAVES_O = TO / 64;             // 1 or 2
  constexpr int WAVES_C = 4 / WAVES_O;         // 4 or 2
  constexpr int WTC = TC / WAVES_C;            // 32 or 64 columns per wave
  constexpr int NI = WTC / 32;                 // 1 or 2
  int local = tile - P.tile_begin;
  const int split = local % P.splits;
  local /= P.splits;
  const int tc = local % P.tiles_n, to = local / P.tiles_n;
  const int o0 = to * TO, col0 = tc * TC;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wo = wave / WAVES_C, wc = wave % WAVES_C;
  const int Cout = P.M, Ncol = P.N, Mpos = P.K;
  const ConvGeom g = P.g;
  const bool gather = P.b_mode == OP_CONV_WGRAD;
  const int Cin = gather ? g.C : P.ldb;

  const int nslab_total = (Mpos + MB - 1) / MB;
  const int per = (nslab_total + P.splits - 1) / P.splits;
  const int s0 = split * per, s1 = min(nslab_total, s0 + per);
  const int nslab = max(0, s1 - s0);  // an empty range still writes its (zero) partial tile
  const int m_begin = s0 * MB, m_count = max(0, min(Mpos, s1 * MB) - m_begin);

  // this thread's chunks: dy columns (o) and x columns (tap, c) are fixed, rows advance
  constexpr int DCH = TO / VEC, XCH = TC / VEC;  // chunks per staged row
  constexpr int ND = MB * DCH / 256, NX = MB * XCH / 256;
  const int d_c = (tid % DCH) * VEC, d_m = tid / DCH;   // rows d_m + i * (256 / DCH)
  const int x_c = (tid % XCH) * VEC, x_m = tid / XCH;   // rows x_m + i * (256 / XCH)
  const int xcol = col0 + x_c;
  int x_kh = 0, x_kw = 0, x_delta = 0;
  const bool xcol_ok = xcol < Ncol;
  if (xcol_ok) {
    const int tap = xcol / Cin, c = xcol - tap * Cin;
    if (gather) {
      x_kh = tap / g.KW;
      x_kw = tap - x_kh * g.KW;
      x_delta = (x_kh * g.W + x_kw) * g.C + c;
    } else {
      x_delta = c;
    }
  }
  const T* __restrict__ Dp = static_cast<const T*>(P.A);
  const T* __restrict__ Xp = static_cast<const T*>(P.B);
  const bool dcol_ok = o0 + d_c < Cout;  // Cout is a multiple of VEC on this path

  uint4 rd[ND], rx[NX];
  int chunk_q0 = 0;  // first position (relative to m_begin) of the chunk the table describes
  auto fetch = [&](int s) {  // s = slab index inside the chunk; positions s*MB .. s*MB+MB-1 of the table
#pragma unroll
    for (int i = 0; i < ND; ++i) {
      const int q = chunk_q0 + s * MB + d_m + i * (256 / DCH);
      rd[i] = (dcol_ok && q < m_count) ? *reinterpret_cast<const uint4*>(Dp + (int64_t)(m_begin + q) * P.lda + o0 + d_c)
                                       : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int q = s * MB + x_m + i * (256 / XCH);
      const int hw = pos_hw[q];
      const int ih = (hw >> 16) + x_kh, iw = (int)(short)(hw & 0xffff) + x_kw;
      const bool ok = xcol_ok && (!gather || (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W)) && hw != (int)0x80008000u;
      rx[i] = ok ? *reinterpret_cast<const uint4*>(Xp + pos_base[q] + x_delta) : make_uint4(0, 0, 0, 0);
    }
  };

  v16f_t acc[2][NI];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  float bsum = 0.f;
  const bool do_beta = (tc == 0) && P.aux3 != nullptr && tid < TO;

  // The range is walked in chunks of at most WG_MAX_SLABS slabs; per chunk the positions are
  // decoded once into the LDS table.
  for (int cs = 0; cs < nslab; cs += WG_MAX_SLABS) {
  const int cn = min(WG_MAX_SLABS, nslab - cs);
  chunk_q0 = cs * MB;
  __syncthreads();  // the previous chunk's table and operand tiles are consumed
  // position table: element offset of x[b][oh*s-p][ow*s-p][0] and the packed (ih0, iw0)
  for (int q = tid; q < cn * MB; q += 256) {
    int base = 0, hw = (int)0x80008000u;  // (ih0, iw0) = (-32768, -32768): every tap out of range
    if (chunk_q0 + q < m_count) {
      const int m = m_begin + chunk_q0 + q;
      if (gather) {
        const int b = m / (g.OH * g.OW);
        const int rem = m - b * (g.OH * g.OW);
        const int oh = rem / g.OW, ow = rem - oh * g.OW;
        const int ih0 = oh * g.stride - g.pad, iw0 = ow * g.stride - g.pad;
        base = ((b * g.H + ih0) * g.W + iw0) * g.C;
        hw = (int)(((unsigned)(ih0 & 0xffff) << 16) | (unsigned)(iw0 & 0xffff));
      } else {
        base = m * P.ldb;
        hw = 0;
      }
    }
    pos_base[q] = base;
    pos_hw[q] = hw;
  }
  __syncthreads();  // position table complete
  fetch(0);
  for (int s = 0; s < cn; ++s) {
    if (s > 0) __syncthreads();
#pragma unroll
    for (int i = 0; i < ND; ++i) {
      Chunk16<T> c;
      c.v = rd[i];
      uint2* dst = reinterpret_cast<uint2*>(Ds + (d_m + i * (256 / DCH)) * PD + d_c);
      dst[0] = c.h[0];
      dst[1] = c.h[1];
    }
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      Chunk16<T> c;
      c.v = rx[i];
      uint2* dst = reinterpret_cast<uint2*>(Xs + (x_m + i * (256 / XCH)) * PX + x_c);
      dst[0] = c.h[0];
      dst[1] = c.h[1];
    }
    __syncthreads();
    if (s + 1 < cn) fetch(s + 1);
    const int gq = lane >> 5, l31 = lane & 31;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int kk = 0; kk < MB; kk += 16) {
        uint4 a[2], b[NI];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = frag_tr_bf16(Ds, PD, kk, wo * 64 + i * 32, lane);
#pragma unroll
        for (int j = 0; j < NI; ++j) b[j] = frag_tr_bf16(Xs, PX, kk, wc * WTC + j * 32, lane);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j) acc[i][j] = mfma_bf16(a[i], b[j], acc[i][j]);
      }
    } else {
#pragma unroll 8
      for (int kk = 0; kk < MB; kk += 2) {
        float a[2], b[NI];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = Ds[(kk + gq) * PD + wo * 64 + i * 32 + l31];
#pragma unroll
        for (int j = 0; j < NI; ++j) b[j] = Xs[(kk + gq) * PX + wc * WTC + j * 32 + l31];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    }
    if (do_beta)
      for (int m = 0; m < MB; ++m) bsum += E::to_f32(Ds[m * PD + tid]);
  }
  }

  // epilogue: acc rows = o, cols = (tap, c); plain stores into this range's partial buffer
  float* __restrict__ part = static_cast<float*>(P.out) + (int64_t)split * Cout * Ncol;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = o0 + wo * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      if (r >= Cout) continue;
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int c = col0 + wc * WTC + j * 32 + (lane & 31);
        if (c < Ncol) part[(int64_t)r * Ncol + c] = acc[i][j][v];
      }
    }
  if (do_beta && o0 + tid < Cout) static_cast<float*>(P.aux3)[(int64_t)split * Cout + o0 + tid] = bsum;
}

template <typename T, int TO>
__global__ __launch_bounds__(256) void conv_wgrad_kernel(const GemmBatch batch) {
  constexpr int MB = WgSlab<T>::MB, PAD = (sizeof(T) == 2) ? 16 : 4;
  __shared__ __attribute__((aligned(16))) T Ds[MB * (TO + PAD)];
  __shared__ __attribute__((aligned(16))) T Xs[MB * (128 + PAD)];
  __shared__ int pos_base[WG_MAX_SLABS * MB];
  __shared__ int pos_hw[WG_MAX_SLABS * MB];
  const int tile = (int)blockIdx.x;
  conv_wgrad_body<T, TO>(batch.p[find_problem(batch, tile)], tile, Ds, Xs, pos_base, pos_hw);
}
// Tiles of both heights in one launch (the height is the problem's: 128 rows for matrices of 128 rows and more, 64
// below): the weight gradients of a tick are one launch instead of one per height, each of which alone is short
// of workgroups on the small ResNet configurations.
__host__ __device__ inline int conv_wgrad_rows(const GemmProb& p) { return p.M >= 128 ? 128 : 64; }
template <typename T>
__global__ __launch_bounds__(256) void conv_wgrad_mixed_kernel(const GemmBatch batch) {
  constexpr int MB = WgSlab<T>::MB, PAD = (sizeof(T) == 2) ? 16 : 4;
  __shared__ __attribute__((aligned(16))) T Ds[MB * (128 + PAD)];
  __shared__ __attribute__((aligned(16))) T Xs[MB * (128 + PAD)];
  __shared__ int pos_base[WG_MAX_SLABS * MB];
  __shared__ int pos_hw[WG_MAX_SLABS * MB];
  const int tile = (int)blockIdx.x;
  const GemmProb& P = batch.p[find_problem(batch, tile)];
  if (conv_wgrad_rows(P) == 128) conv_wgrad_body<T, 128>(P, tile, Ds, Xs, pos_base, pos_hw);
  else conv_wgrad_body<T, 64>(P, tile, Ds, Xs, pos_base, pos_hw);
}

// Fold of the partial sums.  A workgroup is 8 groups of 32 lanes; a lane owns 4 of the 128
// columns of its group's weight row.  Depending on the number of ranges, `rg` = 1, 2, 4 or 8
// groups share one row (each summing every rg-th range) and the workgroup covers 8/rg rows,
// so layers with few ranges still give every lane work and layers with hundreds of ranges
// still split the long sum.  The workgroups of all problems form one flat list.
//   s[c] = sum_ranges part[.][o][c];  G[o][c] += gamma[o]*s[c];
//   d gamma[o] += sum_c s[c]*Wplain[o][c]  (one atomic per 128 columns);
//   d beta[o]  += sum_ranges part_beta[.][o]  (first column chunk only).
template <typename T>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const WReduceBatch batch) {
  using E = Elem<T>;
  __shared__ float4 red[8][32];
  int pi = 0;
  for (int q = 1; q < batch.n; ++q)
    if ((int)blockIdx.x >= batch.p[q].tile_begin) pi = q;
  const WReduceProb& P = batch.p[pi];
  const int rg = P.rg, rows_per_wg = 8 / rg;
  const int chunks = (P.Ncol + 127) >> 7;
  const int local = (int)blockIdx.x - P.tile_begin;
  const int ob = local / chunks, c0 = (local - ob * chunks) * 128;
  const int cl = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int o = ob * rows_per_wg + grp / rg, q0 = grp % rg;
  const int c = c0 + cl * 4;
  const bool row_ok = o < P.Cout;
  const int64_t row = (int64_t)o * P.Ncol, stride = (int64_t)P.Cout * P.Ncol;
  const bool vec4 = (P.Ncol & 3) == 0;  // rows of the partial buffers are 16-byte aligned
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  if (row_ok && vec4) {
    if (c < P.Ncol) {
      // four independent loads in flight per lane
      const float* src = P.part + row + c;
      float4 s1 = sum, s2 = sum, s3 = sum;
      int q = q0;
      for (; q + 3 * rg < P.splits; q += 4 * rg) {
        const float4 v0 = *reinterpret_cast<const float4*>(src + q * stride);
        const float4 v1 = *reinterpret_cast<const float4*>(src + (q + rg) * stride);
        const float4 v2 = *reinterpret_cast<const float4*>(src + (q + 2 * rg) * stride);
        const float4 v3 = *reinterpret_cast<const float4*>(src + (q + 3 * rg) * stride);
        sum.x += v0.x; sum.y += v0.y; sum.z += v0.z; sum.w += v0.w;
        s1.x += v1.x; s1.y += v1.y; s1.z += v1.z; s1.w += v1.w;
        s2.x += v2.x; s2.y += v2.y; s2.z += v2.z; s2.w += v2.w;
        s3.x += v3.x; s3.y += v3.y; s3.z += v3.z; s3.w += v3.w;
      }
      for (; q < P.splits; q += rg) {
        const float4 v = *reinterpret_cast<const float4*>(src + q * stride);
        sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
      }
      sum.x += (s1.x + s2.x) + s3.x; sum.y += (s1.y + s2.y) + s3.y;
      sum.z += (s1.z + s2.z) + s3.z; sum.w += (s1.w + s2.w) + s3.w;
    }
  } else if (row_ok) {
    for (int q = q0; q < P.splits; q += rg) {
      const float* src = P.part + q * stride + row;
      if (c + 0 < P.Ncol) sum.x += src[c + 0];
      if (c + 1 < P.Ncol) sum.y += src[c + 1];
      if (c + 2 < P.Ncol) sum.z += src[c + 2];
      if (c + 3 < P.Ncol) sum.w += src[c + 3];
    }
  }
  red[grp][cl] = sum;
  __syncthreads();
  const bool owner = row_ok && q0 == 0;  // this group of 32 lanes finishes row o
  float dg = 0.f;
  if (owner) {
    float tot[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < rg; ++k) {
      const float4 v = red[grp + k][cl];
      tot[0] += v.x; tot[1] += v.y; tot[2] += v.z; tot[3] += v.w;
    }
    const float gam = P.gamma ? P.gamma[o] : 1.f;
    // loads before stores (which may alias them for all the compiler knows: one round trip instead of four)
    float gold[4], wpl[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      gold[e] = wpl[e] = 0.f;
      if (c + e < P.Ncol) {
        gold[e] = P.G[row + c + e];
        if (P.wplain) wpl[e] = E::to_f32(static_cast<const T*>(P.wplain)[row + c + e]);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (c + e < P.Ncol) {
        P.G[row + c + e] = gold[e] + gam * tot[e];
        dg += tot[e] * wpl[e];
      }
    if (c0 == 0 && P.Gbeta) {
      float sb = 0.f;
      for (int q = cl; q < P.splits; q += 32) sb += P.part_beta[(int64_t)q * P.Cout + o];
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) sb += __shfl_xor(sb, off, 64);
      if (cl == 0) P.Gbeta[o] += sb;
    }
  }
  if (!P.Ggamma) return;  // uniform over the workgroup
  // the 32 lanes of a group (shuffles stay inside a half wavefront; lanes of other groups carry zeros)
#pragma unroll
  for (int off = 16; off >= 1; off >>= 1) dg += __shfl_xor(dg, off, 64);
  const int chunk = c0 >> 7;
  if (chunks == 1) {
    if (owner && cl == 0) P.Ggamma[o] += dg;
    return;
  }
  if (!P.gpart || !P.cnt) {
    if (owner && cl == 0) atomicAdd(P.Ggamma + o, dg);
    return;
  }
  // share of this chunk -> workspace; the last workgroup of the row block to get here adds the shares of
  // every row of the block in chunk order.  Shares and counter are device-scope atomics ordered by waiting
  // for the stores' acknowledgement before the barrier (as in the split contraction tiles).
  if (owner && cl == 0) __hip_atomic_store(P.gpart + (int64_t)o * chunks + chunk, dg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  __shared__ int last;
  if (threadIdx.x == 0) {
    const unsigned int arrived = atomicAdd(P.cnt + ob, 1u);
    last = arrived == (unsigned)(chunks - 1);
    if (last) atomicExch(P.cnt + ob, 0u);  // ready for the next launch
  }
  __syncthreads();
  if (!last) return;
  if ((int)threadIdx.x < rows_per_wg) {
    const int orow = ob * rows_per_wg + (int)threadIdx.x;
    if (orow < P.Cout) {
      float total = 0.f;
      for (int k = 0; k < chunks; ++k)
        total += __hip_atomic_load(P.gpart + (int64_t)orow * chunks + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      P.Ggamma[orow] += total;
    }
  }
}

// The same fold for layers with at most 8 ranges and rows of whole 16-byte groups, by rows: a group of 32 lanes
// walks all 128-column chunks of one weight row (eight rows per workgroup), so a row's d gamma is complete inside
// its group - no shares in a workspace, no counters, no barriers - and a workgroup moves 8 whole rows instead of
// 4 KB of the accumulator.  Every sum is associated as wgrad_reduce_kernel associates it (ranges: groups of four
// into four running sums, the rest into the first; a chunk's d gamma share: the lane's four products in order,
// then the 32-lane exchange tree; shares in chunk order), so the two kernels give the same bits.
template <typename T>
__global__ __launch_bounds__(256) void wgrad_fold_rows_kernel(const WReduceBatch batch) {
  using E = Elem<T>;
  int pi = 0;
  for (int q = 1; q < batch.n; ++q)
    if ((int)blockIdx.x >= batch.p[q].tile_begin) pi = q;
  const WReduceProb& P = batch.p[pi];
  const int cl = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int o = ((int)blockIdx.x - P.tile_begin) * 8 + grp;
  if (o >= P.Cout) return;  // whole 32-lane groups leave: the exchanges below stay inside a group
  const int splits = P.splits, chunks = (P.Ncol + 127) >> 7;
  const int64_t row = (int64_t)o * P.Ncol, stride = (int64_t)P.Cout * P.Ncol;
  const float gam = P.gamma ? P.gamma[o] : 1.f;
  const T* __restrict__ wplain = static_cast<const T*>(P.wplain);
  float dgsum = 0.f;
  for (int chunk = 0; chunk < chunks; ++chunk) {
    const int c = chunk * 128 + cl * 4;
    float dg = 0.f;
    if (c < P.Ncol) {
      const float* src = P.part + row + c;
      float4 v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = q < splits ? *reinterpret_cast<const float4*>(src + q * stride) : make_float4(0.f, 0.f, 0.f, 0.f);
      const float4 gold = *reinterpret_cast<const float4*>(P.G + row + c);
      float wpl[4] = {0.f, 0.f, 0.f, 0.f};
      if (wplain) {
#pragma unroll
        for (int e = 0; e < 4; ++e) wpl[e] = E::to_f32(wplain[row + c + e]);
      }
      float4 sum = make_float4(0.f, 0.f, 0.f, 0.f), s1 = sum, s2 = sum, s3 = sum;
      const int full = splits & ~3;
#pragma unroll
      for (int q = 0; q < 8; q += 4)
        if (q + 3 < splits) {
          sum.x += v[q].x; sum.y += v[q].y; sum.z += v[q].z; sum.w += v[q].w;
          s1.x += v[q + 1].x; s1.y += v[q + 1].y; s1.z += v[q + 1].z; s1.w += v[q + 1].w;
          s2.x += v[q + 2].x; s2.y += v[q + 2].y; s2.z += v[q + 2].z; s2.w += v[q + 2].w;
          s3.x += v[q + 3].x; s3.y += v[q + 3].y; s3.z += v[q + 3].z; s3.w += v[q + 3].w;
        }
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (q >= full && q < splits) { sum.x += v[q].x; sum.y += v[q].y; sum.z += v[q].z; sum.w += v[q].w; }
      sum.x += (s1.x + s2.x) + s3.x; sum.y += (s1.y + s2.y) + s3.y;
      sum.z += (s1.z + s2.z) + s3.z; sum.w += (s1.w + s2.w) + s3.w;
      const float tot[4] = {0.f + sum.x, 0.f + sum.y, 0.f + sum.z, 0.f + sum.w};
      *reinterpret_cast<float4*>(P.G + row + c) =
          make_float4(gold.x + gam * tot[0], gold.y + gam * tot[1], gold.z + gam * tot[2], gold.w + gam * tot[3]);
#pragma unroll
      for (int e = 0; e < 4; ++e) dg += tot[e] * wpl[e];
    }
    if (chunk == 0 && P.Gbeta) {
      float sb = 0.f;
      for (int q = cl; q < splits; q += 32) sb += P.part_beta[(int64_t)q * P.Cout + o];
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) sb += __shfl_xor(sb, off, 64);
      if (cl == 0) P.Gbeta[o] += sb;
    }
    if (P.Ggamma) {
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) dg += __shfl_xor(dg, off, 64);
      dgsum += dg;
    }
  }
  if (P.Ggamma && cl == 0) P.Ggamma[o] += dgsum;
}

hipError_t launch_wgrad_reduce(WReduceBatch& b, int dtype, hipStream_t stream) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > WREDUCE_MAX_PROBS) return hipErrorInvalidValue;
  {
    // by rows where every problem allows it and the launch still has a few workgroups per compute unit
    bool rows_ok = true;
    int64_t wgs = 0;
    for (int i = 0; i < b.n && rows_ok; ++i) {
      const WReduceProb& p = b.p[i];
      rows_ok = p.splits >= 1 && p.splits <= 8 && p.Cout > 0 && p.Ncol > 0 && p.Ncol % 4 == 0 &&
                reinterpret_cast<uintptr_t>(p.part) % 16 == 0 && reinterpret_cast<uintptr_t>(p.G) % 16 == 0 && (!p.Gbeta || p.part_beta);
      wgs += (p.Cout + 7) / 8;
    }
    if (rows_ok && wgs >= 512 && wgs < (1ll << 31)) {
      int total = 0;
      for (int i = 0; i < b.n; ++i) {
        b.p[i].tile_begin = total;
        total += (b.p[i].Cout + 7) / 8;
      }
      if (dtype == DT_BF16) hipLaunchKernelGGL((wgrad_fold_rows_kernel<uint16_t>), dim3((unsigned)total), dim3(256), 0, stream, b);
      else hipLaunchKernelGGL((wgrad_fold_rows_kernel<float>), dim3((unsigned)total), dim3(256), 0, stream, b);
      return hipGetLastError();
    }
  }
  int64_t total = 0;
  for (int i = 0; i < b.n; ++i) {
    WReduceProb& p = b.p[i];
    if (p.Cout <= 0 || p.Ncol <= 0 || p.splits <= 0) return hipErrorInvalidValue;
    if ((p.gpart == nullptr) != (p.cnt == nullptr)) return hipErrorInvalidValue;
    p.rg = p.splits <= 8 ? 1 : p.splits <= 16 ? 2 : p.splits <= 32 ? 4 : 8;
    const int rows_per_wg = 8 / p.rg;
    p.tile_begin = (int)total;
    total += (int64_t)((p.Cout + rows_per_wg - 1) / rows_per_wg) * ((p.Ncol + 127) / 128);
    if (total >= (1ll << 31)) return hipErrorInvalidValue;
  }
  dim3 grid((unsigned)total), block(256);
  if (dtype == DT_BF16) hipLaunchKernelGGL((wgrad_reduce_kernel<uint16_t>), grid, block, 0, stream, b);
  else hipLaunchKernelGGL((wgrad_reduce_kernel<float>), grid, block, 0, stream, b);
  return hipGetLastError();
}

int conv_wgrad_slab(int dtype) { return wg_slab(dtype); }

int conv_wgrad_splits(const GemmProb& p, int dtype, int wanted) {
  // Short ranges (one per WG_MAX_SLABS slabs) measured faster than few long ones as long as the
  // launch is short of workgroups, even though they write more partial sums; a layer with
  // enough tiles of its own does not need them.
  const int nslab = (p.K + wg_slab(dtype) - 1) / wg_slab(dtype);
  const int to = p.M >= 128 ? 128 : 64;
  const int tiles = ((p.M + to - 1) / to) * ((p.N + 127) / 128);
  const int min_splits = std::min((nslab + WG_MAX_SLABS - 1) / WG_MAX_SLABS, (1024 + tiles - 1) / tiles);
  return std::max(1, std::min(nslab, std::max(wanted, min_splits)));
}

// ---------------------------------------------------------------------------------
bool conv_fast_eligible(const GemmProb& p, int dtype) {
  const int bk = dtype == DT_BF16 ? 32 : 16, vec = dtype == DT_BF16 ? 8 : 4;
  if (p.epi == EPI_WGRAD) {
    if (p.a_mode != OP_PLAIN_R) return false;
    if (p.b_mode == OP_CONV_WGRAD) {
      if (p.g.C % vec || p.g.KH * p.g.KW > 32 || p.g.H >= 32768 || p.g.W >= 32768) return false;
    } else if (p.b_mode == OP_PLAIN_R) {
      if (p.ldb % vec || p.N > p.ldb) return false;
    } else {
      return false;
    }
    return (p.M % vec) == 0 && (p.lda % vec) == 0;
  }
  if (p.b_mode != OP_PLAIN_K || p.ldb != p.K || (p.K % bk)) return false;
  if ((p.flags & GF_OUT_F32) || (p.N % vec) || (p.ldo % vec)) return false;
  if (p.a_mode == OP_PLAIN_K) return p.lda == p.K;
  if (p.a_mode == OP_CONV_FWD || p.a_mode == OP_CONV_DGRAD) return (p.g.C % bk) == 0 && p.g.KH * p.g.KW <= 32;
  return false;
}

template <typename T, int BM, int BN, int BK, bool DB>
constexpr int conv_gemm_lds_bytes() {
  constexpr int oper = (DB ? 2 : 1) * (BM + BN) * (BK + 16 / (int)sizeof(T)) * (int)sizeof(T);
  constexpr int stage = 4 * 32 * (BN / 2 + 4) * 4;
  return oper > stage ? oper : stage;
}

template <typename T, int BM, int BN, int BK, bool DB>
static hipError_t launch_conv_gemm_inst(const GemmBatch& b, dim3 grid, hipStream_t stream) {
  constexpr int lds = conv_gemm_lds_bytes<T, BM, BN, BK, DB>();
  static_assert(lds <= 64 * 1024, "stays within the default dynamic LDS limit");
  hipLaunchKernelGGL((conv_gemm_kernel<T, BM, BN, BK, DB>), grid, dim3(256), lds, stream, b);
  return hipGetLastError();
}

template <typename T, int BK>
static hipError_t launch_conv_gemm_typed(const GemmBatch& b, int bm, int bn, dim3 grid, hipStream_t stream) {
  if (bm == 128 && bn == 128) return launch_conv_gemm_inst<T, 128, 128, BK, false>(b, grid, stream);
  if (bm == 128) return launch_conv_gemm_inst<T, 128, 64, BK, false>(b, grid, stream);
  if (bn == 128) return launch_conv_gemm_inst<T, 64, 128, BK, true>(b, grid, stream);
  return launch_conv_gemm_inst<T, 64, 64, BK, true>(b, grid, stream);
}

// Tile shape for the forward / data-gradient problems of one launch: the largest of
// 128x128, 64x128, 64x64 (128x64, 64x64 when every output is at most 64 wide) that still
// yields enough workgroups over the whole launch.
void conv_gemm_tile(const GemmProb* p, int n, int* bm, int* bn) {
  const int want = 384;
  bool narrow = true;
  for (int i = 0; i < n; ++i) narrow = narrow && p[i].N <= 64;
  auto tiles = [&](int tm, int tn) {
    int t = 0;
    for (int i = 0; i < n; ++i) t += ((p[i].M + tm - 1) / tm) * ((p[i].N + tn - 1) / tn);
    return t;
  };
  if (narrow) {
    *bn = 64;
    *bm = tiles(128, 64) >= want ? 128 : 64;
  } else if (tiles(128, 128) >= want) {
    *bm = 128; *bn = 128;
  } else if (tiles(64, 128) >= want) {
    *bm = 64; *bn = 128;
  } else {
    *bm = 64; *bn = 64;
  }
}

hipError_t launch_conv_gemm(GemmBatch& b, int dtype, int bm, int bn, hipStream_t stream) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > GEMM_MAX_PROBS) return hipErrorInvalidValue;
  if ((bm != 64 && bm != 128) || (bn != 64 && bn != 128)) return hipErrorInvalidValue;
  const int bk = dtype == DT_BF16 ? 32 : 16;
  int total = 0;
  bool deep = true;  // every problem allows the double-depth slab
  for (int i = 0; i < b.n; ++i) {
    GemmProb& p = b.p[i];
    if (p.M <= 0 || p.N <= 0 || p.K <= 0 || p.epi == EPI_WGRAD || !conv_fast_eligible(p, dtype)) return hipErrorInvalidValue;
    const int C = p.a_mode == OP_PLAIN_K ? p.K : p.g.C;
    if (C % (2 * bk)) deep = false;
    p.splits = 1;
    p.tiles_n = (p.N + bn - 1) / bn;
    p.tile_begin = total;
    total += ((p.M + bm - 1) / bm) * p.tiles_n;
  }
  // A launch short of workgroups shares its long reductions: about 640 workgroups in all,
  // ranges of at least 4 slabs, at most 8 per tile, while the partial tiles fit the workspace.
  // (64 x 64 tiles only: the partial tile of a larger one costs more than the shorter chain saves)
  if (b.thin_ws && b.thin_cnt && total < 512 && bm == 64 && bn == 64) {
    const int slab = deep ? 2 * bk : bk, want = (640 + total - 1) / total;
    int split_total = 0;
    for (int i = 0; i < b.n; ++i) {
      GemmProb& p = b.p[i];
      p.splits = std::max(1, std::min(std::min(want, 8), p.K / slab / 4));
      split_total += ((p.M + bm - 1) / bm) * p.tiles_n * p.splits;
    }
    if (split_total <= CONV_SPLIT_SLOTS && (int64_t)split_total * bm * bn * 4 <= CONV_SPLIT_WS_BYTES) {
      total = 0;
      for (int i = 0; i < b.n; ++i) {
        b.p[i].tile_begin = total;
        total += ((b.p[i].M + bm - 1) / bm) * b.p[i].tiles_n * b.p[i].splits;
      }
    } else {
      for (int i = 0; i < b.n; ++i) b.p[i].splits = 1;
    }
  }
  b.total_tiles = total;
  dim3 grid(total);
  if (dtype == DT_BF16) return deep ? launch_conv_gemm_typed<uint16_t, 64>(b, bm, bn, grid, stream)
                                    : launch_conv_gemm_typed<uint16_t, 32>(b, bm, bn, grid, stream);
  return deep ? launch_conv_gemm_typed<float, 32>(b, bm, bn, grid, stream)
              : launch_conv_gemm_typed<float, 16>(b, bm, bn, grid, stream);
}

hipError_t launch_conv_wgrad_mixed(GemmBatch& b, int dtype, hipStream_t stream) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > GEMM_MAX_PROBS) return hipErrorInvalidValue;
  int total = 0;
  for (int i = 0; i < b.n; ++i) {
    GemmProb& p = b.p[i];
    if (p.M <= 0 || p.N <= 0 || p.K <= 0 || p.epi != EPI_WGRAD || !conv_fast_eligible(p, dtype)) return hipErrorInvalidValue;
    if (p.splits < 1 || p.splits > (p.K + wg_slab(dtype) - 1) / wg_slab(dtype)) return hipErrorInvalidValue;  // the caller sized the partial buffer
    const int to = conv_wgrad_rows(p);
    p.tiles_n = (p.N + 127) / 128;
    p.tile_begin = total;
    total += ((p.M + to - 1) / to) * p.tiles_n * p.splits;
  }
  b.total_tiles = total;
  if (dtype == DT_BF16) hipLaunchKernelGGL((conv_wgrad_mixed_kernel<uint16_t>), dim3(total), dim3(256), 0, stream, b);
  else hipLaunchKernelGGL((conv_wgrad_mixed_kernel<float>), dim3(total), dim3(256), 0, stream, b);
  return hipGetLastError();
}

hipError_t launch_conv_wgrad(GemmBatch& b, int dtype, bool wide, hipStream_t stream) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > GEMM_MAX_PROBS) return hipErrorInvalidValue;
  const int to = wide ? 128 : 64;
  int total = 0;
  for (int i = 0; i < b.n; ++i) {
    GemmProb& p = b.p[i];
    if (p.M <= 0 || p.N <= 0 || p.K <= 0 || p.epi != EPI_WGRAD || !conv_fast_eligible(p, dtype)) return hipErrorInvalidValue;
    if (p.splits < 1 || p.splits > (p.K + wg_slab(dtype) - 1) / wg_slab(dtype)) return hipErrorInvalidValue;  // the caller sized the partial buffer
    p.tiles_n = (p.N + 127) / 128;
    p.tile_begin = total;
    total += ((p.M + to - 1) / to) * p.tiles_n * p.splits;
  }
  b.total_tiles = total;
  dim3 grid(total), block(256);
  if (dtype == DT_BF16) {
    if (wide) hipLaunchKernelGGL((conv_wgrad_kernel<uint16_t, 128>), grid, block, 0, stream, b);
    else hipLaunchKernelGGL((conv_wgrad_kernel<uint16_t, 64>), grid, block, 0, stream, b);
  } else {
    if (wide) hipLaunchKernelGGL((conv_wgrad_kernel<float, 128>), grid, block, 0, stream, b);
    else hipLaunchKernelGGL((conv_wgrad_kernel<float, 64>), grid, block, 0, stream, b);
  }
  return hipGetLastError();
}

}  // namespace cdp
