// Large-tile implicit-GEMM convolution / token-wise linear pass for bf16 on gfx950: 256 x 256 outputs per
// workgroup, 64-deep reduction slabs, eight wavefronts (two per SIMD, wave tile 128 x 64).
//
// What is different from conv_gemm_kernel (128 x 128, four wavefronts):
//   * operands go from global memory straight into LDS (global_load_lds_dwordx4, 16 bytes per lane, no
//     register round trip and no LDS store instructions); a lane whose chunk is a structural zero (a tap
//     outside the image, a row past the matrix) reads 16 zero bytes from a small device array instead;
//   * one such instruction fills 1 KB of LDS lane by lane, so a tile row is 128 unpadded bytes and bank
//     conflicts are avoided by an XOR swizzle: 16-byte chunk c of tile row r sits in slot c ^ ((r >> 1) & 7)
//     (the loading lane picks the global chunk that belongs in its slot); a fragment read of 16 rows x
//     16 bytes then covers all 64 banks once;
//   * two LDS stages (2 x 64 KB): the loads of slab t+1 are in flight while slab t is contracted, one
//     barrier per slab.  The stages are two separate __shared__ arrays on purpose: the compiler orders an
//     LDS read after every outstanding LDS-writing load it cannot prove disjoint, and a single array would
//     make it wait for the prefetch before the first fragment read;
//   * operand bytes per flop through the CU's vector-memory path are half those of the 128 x 128 tile.
// Same problem descriptors, same epilogues (bias, residual, ReLU; data gradient: addend, accumulate, mask).
#include <algorithm>

#include "elem.h"
#include "kernels.h"

namespace cdp {

namespace {

constexpr int BK = 64;

__device__ uint4 g_zero_chunk[4];  // zero-initialised; source of structural zeros

typedef __attribute__((address_space(3))) void* lds_ptr;

}  // namespace

// BM x BN outputs per workgroup, WAVES_M x WAVES_N wavefronts: 256 x 256 with 2 x 4 (wave tile 128 x 64, one
// workgroup per CU), 128 x 128 with 2 x 2 (wave tile 64 x 64, two workgroups per CU).
template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void conv_gemm_dl_kernel(const GemmBatch batch) {
  constexpr int NWAVE = WAVES_M * WAVES_N;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
  constexpr int MI = WTM / 32, NI = WTN / 32;            // MFMA tiles per wave
  constexpr int STAGE_BYTES = (BM + BN) * BK * 2;        // one LDS stage
  constexpr int LPA = BM / 8 / NWAVE, LPB = BN / 8 / NWAVE;  // 1 KB blocks (8 rows) a wave loads per operand and slab
  static_assert(LPA * 8 * NWAVE == BM && LPB * 8 * NWAVE == BN && BM == BN, "tile rows are dealt to the waves in blocks of 8");
  constexpr int LPW = LPA;
  __shared__ __attribute__((aligned(1024))) unsigned char smem0[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char smem1[STAGE_BYTES];
  using E = Elem<uint16_t>;
  constexpr int VEC = 8;
  const int tile = (int)blockIdx.x;
  const GemmProb& P = batch.p[find_problem(batch, tile)];
  const int local = tile - P.tile_begin;
  const int tn = local % P.tiles_n, tm = local / P.tiles_n;
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const uint16_t* __restrict__ Ap = static_cast<const uint16_t*>(P.A);
  const uint16_t* __restrict__ Bp = static_cast<const uint16_t*>(P.B);
  const uint16_t* const zero = reinterpret_cast<const uint16_t*>(g_zero_chunk);
  const ConvGeom g = P.g;
  const int mode = P.a_mode;
  const int C = (mode == OP_PLAIN_K) ? P.K : g.C;  // channels per tap of the gathered tensor

  // rows this lane loads: block (wave * LPW + i) of 8 rows, row lane / 8 of it, slot lane % 8
  const int lr = lane >> 3, ls = lane & 7;
  int abase[LPW], boff[LPW];
  unsigned amask[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int tr = (wave * LPW + i) * 8 + lr;     // tile row
    const int chunk = ls ^ ((tr >> 1) & 7);       // the global chunk whose place is slot ls
    const int r = row0 + tr;
    abase[i] = 0;
    amask[i] = 0;
    if (r < P.M) {
      if (mode == OP_PLAIN_K) {
        abase[i] = r * P.lda + chunk * VEC;
        amask[i] = 1u;
      } else {
        const int b = r / (g.OH * g.OW);
        const int rem = r - b * (g.OH * g.OW);
        const int oh = rem / g.OW, ow = rem - oh * g.OW;
        if (mode == OP_CONV_FWD) {
          const int ih0 = oh * g.stride - g.pad, iw0 = ow * g.stride - g.pad;
          abase[i] = ((b * g.H + ih0) * g.W + iw0) * g.C + chunk * VEC;
          const int kw_lo = max(0, -iw0), kw_hi = min(g.KW, g.W - iw0);
          const unsigned cols = kw_hi > kw_lo ? ((1u << kw_hi) - 1u) & ~((1u << kw_lo) - 1u) : 0u;
          for (int kh = max(0, -ih0); kh < min(g.KH, g.H - ih0); ++kh) amask[i] |= cols << (kh * g.KW);
        } else {  // OP_CONV_DGRAD: (oh, ow) is an input position, the gathered tensor is dy
          const int qh = (oh + g.pad) / g.stride, eh = (oh + g.pad) - qh * g.stride;
          const int qw = (ow + g.pad) / g.stride, ew = (ow + g.pad) - qw * g.stride;
          abase[i] = ((b * g.H + qh) * g.W + qw) * g.C + chunk * VEC;
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
    const int c = col0 + tr;
    boff[i] = c < P.N ? c * P.ldb + chunk * VEC : -1;
  }

  // wavefront-uniform position of the next slab to load: tap index, channel offset inside the tap
  int tap = 0, c0 = 0, kh = 0, kw = 0, kload = 0;
  auto issue = [&](unsigned char* stage) {
    int delta;
    if (mode == OP_PLAIN_K) delta = c0;
    else if (mode == OP_CONV_FWD) delta = (kh * g.W + kw) * g.C + c0;
    else delta = -((kh / g.stride) * g.W + (kw / g.stride)) * g.C + c0;
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      const uint16_t* pa = ((amask[i] >> tap) & 1u) ? Ap + abase[i] + delta : zero;
      const uint16_t* pb = boff[i] >= 0 ? Bp + boff[i] + kload : zero;
      __builtin_amdgcn_global_load_lds(pa, (lds_ptr)(stage + (wave * LPW + i) * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(pb, (lds_ptr)(stage + BM * BK * 2 + (wave * LPW + i) * 1024), 16, 0, 0);
    }
    kload += BK;
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

  // fragments: row = base + lane % 32, chunk = 2 * kk + lane / 32, slot = chunk ^ ((row >> 1) & 7)
  const int l31 = lane & 31, hi = lane >> 5;
  int offa[MI], offb[NI], swa[MI], swb[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) { const int r = wm * WTM + i * 32 + l31; offa[i] = r * 128; swa[i] = (r >> 1) & 7; }
#pragma unroll
  for (int j = 0; j < NI; ++j) { const int r = wn * WTN + j * 32 + l31; offb[j] = BM * BK * 2 + r * 128; swb[j] = (r >> 1) & 7; }
  auto contract = [&](const unsigned char* stage) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      uint4 a[MI], b[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) a[i] = *reinterpret_cast<const uint4*>(stage + offa[i] + (((kk * 2 + hi) ^ swa[i]) << 4));
#pragma unroll
      for (int j = 0; j < NI; ++j) b[j] = *reinterpret_cast<const uint4*>(stage + offb[j] + (((kk * 2 + hi) ^ swb[j]) << 4));
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = mfma_bf16(a[i], b[j], acc[i][j]);
    }
  };

  const int nslab = P.K / BK;
  issue(smem0);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  for (int t = 0; t < nslab; t += 2) {
    if (t + 1 < nslab) issue(smem1);
    contract(smem0);
    __builtin_amdgcn_s_waitcnt(0);  // the next slab has landed (every outstanding load of this wave)
    __syncthreads();
    if (t + 1 >= nslab) break;
    if (t + 2 < nslab) issue(smem0);
    contract(smem1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  }

  // ---- epilogue: 32 rows of the wave tile at a time through a staging area of the wave's own (fp32),
  // then 16-byte rows.  No load is outstanding and every wave has passed the last barrier: both stages are free.
  constexpr int SP = WTN + 4;
  constexpr int HALF = NWAVE / 2;
  static_assert(HALF * 32 * SP * 4 <= STAGE_BYTES, "half of the waves' staging areas per LDS stage");
  float* stage = reinterpret_cast<float*>(wave < HALF ? smem0 : smem1) + (wave % HALF) * (32 * SP);
  const int flags = P.flags;
  const bool fwd = P.epi == EPI_FWD;
  uint16_t* outp = static_cast<uint16_t*>(P.out);
  constexpr int CPS = WTN / VEC;      // chunks per staged row
  constexpr int NCH = 32 * CPS / 64;  // chunks per lane
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the previous pass's reads are done
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) stage[((v >> 2) * 8 + hi * 4 + (v & 3)) * SP + j * 32 + l31] = acc[i][j][v];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
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
      Chunk16<uint16_t> x0, x1, x2, res;
      if (fwd) {
        if (P.aux0) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] += static_cast<const float*>(P.aux0)[c + e];
        }
        if (P.aux1) {
          x1.v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(P.aux1) + o);
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] += E::to_f32(x1.e[e]);
        }
        if (flags & GF_RELU) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] = fmaxf(val[e], 0.f);
        }
      } else {
        if (P.aux0) {
          x0.v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(P.aux0) + o);
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] += E::to_f32(x0.e[e]);
        }
        if (flags & GF_ACCUM) {
          x2.v = *reinterpret_cast<const uint4*>(outp + o);
#pragma unroll
          for (int e = 0; e < VEC; ++e) val[e] += E::to_f32(x2.e[e]);
        }
        if (P.aux1) {
          x1.v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(P.aux1) + o);
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

// A forward / data-gradient problem the large tile takes: bf16, every reduction slab of 64 inside one tap,
// 16-byte aligned operands, 32-bit element offsets.
bool conv_gemm256_eligible(const GemmProb& p, int dtype) {
  if (dtype != DT_BF16 || p.epi == EPI_WGRAD || !conv_fast_eligible(p, dtype)) return false;
  const int C = p.a_mode == OP_PLAIN_K ? p.K : p.g.C;
  if (p.K % BK || C % BK) return false;
  if ((reinterpret_cast<uintptr_t>(p.A) | reinterpret_cast<uintptr_t>(p.B) | reinterpret_cast<uintptr_t>(p.out)) & 15) return false;
  if ((p.aux1 && (reinterpret_cast<uintptr_t>(p.aux1) & 15)) || (p.epi == EPI_DGRAD && p.aux0 && (reinterpret_cast<uintptr_t>(p.aux0) & 15)))
    return false;
  const int64_t a_elems = p.a_mode == OP_PLAIN_K ? (int64_t)p.M * p.lda : (int64_t)(p.M / (p.g.OH * p.g.OW) + 1) * p.g.H * p.g.W * p.g.C;
  return a_elems < (1ll << 31) && (int64_t)p.N * p.ldb < (1ll << 31);
}

// Worth it (measured against the 128 x 128 tile of conv_gemm_kernel: 880 vs 720 TFLOP/s on a 3x3 convolution
// over 512 channels with 25088 rows, 1050 TFLOP/s on an 8192^3 product, but 705 vs 745 on 25088 x 2048 x 2048,
// where the 784 tiles make 3.06 rounds of one workgroup per CU): long reductions (the tile's prologue and
// epilogue are paid once per 256 x 256 outputs), mostly full tiles, and a tile count that rounds well to the CUs.
bool conv_gemm256_wanted(const GemmProb* p, int n, int dtype) {
  constexpr int BM = 256, BN = 256;
  int64_t tiles = 0;
  double useful = 0;
  for (int i = 0; i < n; ++i) {
    if (!conv_gemm256_eligible(p[i], dtype) || p[i].K < 32 * BK) return false;
    tiles += (int64_t)((p[i].M + BM - 1) / BM) * ((p[i].N + BN - 1) / BN);
    useful += (double)p[i].M * p[i].N;
  }
  if (tiles < 192) return false;
  const int64_t rounds = (tiles + 255) / 256;
  return useful / ((double)rounds * 256 * BM * BN) >= 0.75;
}

hipError_t launch_conv_gemm256(GemmBatch& b, int dtype, hipStream_t stream, int tile) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > GEMM_MAX_PROBS || (tile != 256 && tile != 128)) return hipErrorInvalidValue;
  int total = 0;
  for (int i = 0; i < b.n; ++i) {
    GemmProb& p = b.p[i];
    if (p.M <= 0 || p.N <= 0 || p.K <= 0 || !conv_gemm256_eligible(p, dtype)) return hipErrorInvalidValue;
    p.splits = 1;
    p.tiles_n = (p.N + tile - 1) / tile;
    p.tile_begin = total;
    total += ((p.M + tile - 1) / tile) * p.tiles_n;
  }
  b.total_tiles = total;
  if (tile == 256) hipLaunchKernelGGL((conv_gemm_dl_kernel<256, 256, 2, 4>), dim3(total), dim3(512), 0, stream, b);
  else hipLaunchKernelGGL((conv_gemm_dl_kernel<128, 128, 2, 2>), dim3(total), dim3(256), 0, stream, b);
  return hipGetLastError();
}

}  // namespace cdp
