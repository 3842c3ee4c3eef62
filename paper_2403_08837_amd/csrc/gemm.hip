// Grouped GEMM for one CDP tick on gfx950 (CDNA4): every (micro-batch, stage) pair
// active in the tick contributes forward / data-gradient / weight-gradient problems
// (Sec. 3.2: each stage processes one distinct micro-batch per time step, so the
// problems of a tick are independent and use distinct stage weights).  One launch walks
// a tile list over all problems.  Tiles are staged through LDS and contracted with
// MFMA (bf16: v_mfma_f32_32x32x16_bf16, fp32: v_mfma_f32_32x32x2_f32), fp32 accumulate.
#include "elem.h"
#include "kernels.h"

namespace cdp {

// Element offset of virtual operand entry (r, k), or -1 where the entry is a structural
// zero (padding, stride hole, out of range).
__device__ __forceinline__ int64_t operand_offset(int mode, int ld, const ConvGeom& g, int R, int K, int r, int k) {
  if (r >= R || k >= K) return -1;
  if (mode == OP_PLAIN_K) return (int64_t)r * ld + k;
  if (mode == OP_PLAIN_R) return (int64_t)k * ld + r;
  int pos = (mode == OP_CONV_WGRAD) ? k : r;
  int tc = (mode == OP_CONV_WGRAD) ? r : k;
  int b = pos / (g.OH * g.OW);
  int rem = pos - b * (g.OH * g.OW);
  int oh = rem / g.OW, ow = rem - oh * g.OW;
  int tap = tc / g.C, c = tc - tap * g.C;
  int kh = tap / g.KW, kw = tap - kh * g.KW;
  int ih, iw;
  if (mode == OP_CONV_DGRAD) {
    int th = oh + g.pad - kh, tw = ow + g.pad - kw;
    if (th < 0 || tw < 0) return -1;
    ih = th / g.stride;
    iw = tw / g.stride;
    if (ih * g.stride != th || iw * g.stride != tw) return -1;
  } else {
    ih = oh * g.stride - g.pad + kh;
    iw = ow * g.stride - g.pad + kw;
    if (ih < 0 || iw < 0) return -1;
  }
  if (ih >= g.H || iw >= g.W) return -1;
  return (((int64_t)b * g.H + ih) * g.W + iw) * g.C + c;
}

union Chunk {
  uint4 v;
  uint16_t h[8];
  float f[4];
};

// One 16-byte chunk of the operand tile.  Class-K modes: VEC consecutive k at row r.
// Class-R modes: VEC consecutive r at reduction index k.
template <typename T>
__device__ __forceinline__ uint4 fetch_chunk(const T* __restrict__ ptr, int mode, int ld, const ConvGeom& g, int R, int K,
                                             int r, int k, bool vec_ok) {
  constexpr int VEC = Elem<T>::VEC;
  const bool along_r = (mode == OP_PLAIN_R || mode == OP_CONV_WGRAD);
  Chunk c;
  c.v = make_uint4(0, 0, 0, 0);
  if (vec_ok && (along_r ? (r + VEC <= R && k < K) : (k + VEC <= K && r < R))) {
    int64_t off = operand_offset(mode, ld, g, R, K, r, k);
    if (off >= 0) c.v = *reinterpret_cast<const uint4*>(ptr + off);
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      int64_t off = along_r ? operand_offset(mode, ld, g, R, K, r + e, k) : operand_offset(mode, ld, g, R, K, r, k + e);
      if (off >= 0) {
        if constexpr (sizeof(T) == 2) c.h[e] = ptr[off]; else c.f[e] = ptr[off];
      }
    }
  }
  return c.v;
}

// A chunk is contiguous in memory (one aligned 16-byte load) under these conditions.
template <typename T>
__device__ __forceinline__ bool operand_vec_ok(int mode, int ld, const ConvGeom& g) {
  constexpr int VEC = Elem<T>::VEC;
  if (mode == OP_PLAIN_K || mode == OP_PLAIN_R) return (ld % VEC) == 0;
  return (g.C % VEC) == 0;
}

template <typename T, int ROWS, int BK>
struct TileLoader {
  static constexpr int VEC = Elem<T>::VEC;
  static constexpr int LDP = BK + VEC;  // padded LDS pitch (elements)
  static constexpr int NCH = ROWS * BK / VEC / 256;
  static_assert(NCH >= 1, "tile too small for 256 threads");
  uint4 regs[NCH];

  __device__ __forceinline__ void fetch(const T* ptr, int mode, int ld, const ConvGeom& g, int R, int K, int row0, int k0,
                                        bool vec_ok, int tid) {
    const bool along_r = (mode == OP_PLAIN_R || mode == OP_CONV_WGRAD);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int id = tid + i * 256;
      int r, k;
      if (along_r) {
        k = id / (ROWS / VEC);
        r = (id - k * (ROWS / VEC)) * VEC;
      } else {
        r = id / (BK / VEC);
        k = (id - r * (BK / VEC)) * VEC;
      }
      regs[i] = fetch_chunk<T>(ptr, mode, ld, g, R, K, row0 + r, k0 + k, vec_ok);
    }
  }

  // LDS layout is always [row][k] (k contiguous) so MFMA fragments are one LDS read.
  __device__ __forceinline__ void store(T* lds, int mode, int tid) const {
    const bool along_r = (mode == OP_PLAIN_R || mode == OP_CONV_WGRAD);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int id = tid + i * 256;
      if (along_r) {
        int k = id / (ROWS / VEC);
        int r = (id - k * (ROWS / VEC)) * VEC;
        Chunk c;
        c.v = regs[i];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          if constexpr (sizeof(T) == 2) lds[(r + e) * LDP + k] = c.h[e]; else lds[(r + e) * LDP + k] = c.f[e];
        }
      } else {
        int r = id / (BK / VEC);
        int k = (id - r * (BK / VEC)) * VEC;
        *reinterpret_cast<uint4*>(lds + r * LDP + k) = regs[i];
      }
    }
  }
};

template <typename T>
__device__ __forceinline__ v16f_t mfma_step(const T* a_lds, const T* b_lds, v16f_t acc);

template <>
__device__ __forceinline__ v16f_t mfma_step<uint16_t>(const uint16_t* a, const uint16_t* b, v16f_t acc) {
  uint4 av = *reinterpret_cast<const uint4*>(a);
  uint4 bv = *reinterpret_cast<const uint4*>(b);
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf16_t, av), __builtin_bit_cast(v8bf16_t, bv), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ v16f_t mfma_step<float>(const float* a, const float* b, v16f_t acc) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(*a, *b, acc, 0, 0, 0);
}

// EPIG selects the epilogue family at compile time: 0 = forward / data gradient (stores
// activations), 1 = weight gradient (accumulates into the fp32 gradient buffer; the old
// values of a non-atomic accumulate are fetched before the contraction starts so that
// their latency overlaps it).
template <typename T, int BM, int BN, int BK, int WAVES_M, int EPIG>
__global__ __launch_bounds__(256) void gemm_grouped_kernel(const GemmBatch batch) {
  using E = Elem<T>;
  constexpr int VEC = E::VEC, LDP = BK + VEC;
  constexpr int WAVES_N = 4 / WAVES_M;
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int MI = WTM / 32, NI = WTN / 32;
  static_assert(MI >= 1 && NI >= 1, "wave tile must hold a 32x32 MFMA tile");
  __shared__ __attribute__((aligned(16))) T As[BM * LDP];
  __shared__ __attribute__((aligned(16))) T Bs[BN * LDP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  int pi = 0;
  for (int q = 1; q < batch.n; ++q)
    if ((int)blockIdx.x >= batch.p[q].tile_begin) pi = q;
  const GemmProb& P = batch.p[pi];

  int local = (int)blockIdx.x - P.tile_begin;
  const int split = local % P.splits;
  local /= P.splits;
  const int tn = local % P.tiles_n, tm = local / P.tiles_n;
  const int row0 = tm * BM, col0 = tn * BN;
  const int ktiles = (P.K + BK - 1) / BK;
  const int per = (ktiles + P.splits - 1) / P.splits;
  const int kt0 = split * per;
  const int kt1 = min(ktiles, kt0 + per);
  if (kt0 >= kt1) return;

  const T* Ap = static_cast<const T*>(P.A);
  const T* Bp = static_cast<const T*>(P.B);
  const bool a_gather = P.a_mode >= OP_CONV_FWD;
  const bool a_vec = operand_vec_ok<T>(P.a_mode, P.lda, P.g);
  const bool b_vec = operand_vec_ok<T>(P.b_mode, P.ldb, P.g);
  (void)a_gather;

  TileLoader<T, BM, BK> la;
  TileLoader<T, BN, BK> lb;
  v16f_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  la.fetch(Ap, P.a_mode, P.lda, P.g, P.M, P.K, row0, kt0 * BK, a_vec, tid);
  lb.fetch(Bp, P.b_mode, P.ldb, P.g, P.N, P.K, col0, kt0 * BK, b_vec, tid);

  const int flags = P.flags;
  constexpr int NOLD = (EPIG == 1) ? MI * NI * 16 : 1;
  float gold[NOLD];
  const bool rmw = (EPIG == 1) && (flags & GF_ACCUM) && !(flags & GF_ATOMIC);
  if constexpr (EPIG == 1) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = row0 + wm * WTM + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          const int c = col0 + wn * WTN + j * 32 + (lane & 31);
          gold[(i * NI + j) * 16 + v] = (rmw && r < P.M && c < P.N) ? static_cast<const float*>(P.out)[(int64_t)r * P.ldo + c] : 0.f;
        }
  }

  for (int kt = kt0; kt < kt1; ++kt) {
    __syncthreads();  // previous tile fully consumed
    la.store(As, P.a_mode, tid);
    lb.store(Bs, P.b_mode, tid);
    __syncthreads();
    if (kt + 1 < kt1) {  // prefetch the next tile while this one is contracted
      la.fetch(Ap, P.a_mode, P.lda, P.g, P.M, P.K, row0, (kt + 1) * BK, a_vec, tid);
      lb.fetch(Bp, P.b_mode, P.ldb, P.g, P.N, P.K, col0, (kt + 1) * BK, b_vec, tid);
    }
    const int kg = (lane >> 5) * E::KPL;
#pragma unroll
    for (int kk = 0; kk < BK; kk += E::MFMA_K) {
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const T* ap = As + (wm * WTM + i * 32 + (lane & 31)) * LDP + kk + kg;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          const T* bp = Bs + (wn * WTN + j * 32 + (lane & 31)) * LDP + kk + kg;
          acc[i][j] = mfma_step<T>(ap, bp, acc[i][j]);
        }
      }
    }
  }

  // ---- epilogue.  acc[i][j][v]: row = 8*(v/4) + 4*(lane/32) + v%4, col = lane%32 of the 32x32 tile
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = row0 + wm * WTM + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      float gsum = 0.f;
      float gam = 1.f;
      if (EPIG == 1 && P.aux0 != nullptr && r < P.M) gam = static_cast<const float*>(P.aux0)[r];
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int c = col0 + wn * WTN + j * 32 + (lane & 31);
        if (r >= P.M || c >= P.N) continue;
        float val = acc[i][j][v];
        const int64_t o = (int64_t)r * P.ldo + c;
        if (EPIG == 0 && P.epi == EPI_FWD) {
          if (P.aux0) val += static_cast<const float*>(P.aux0)[c];
          if (P.aux1) val += E::to_f32(static_cast<const T*>(P.aux1)[o]);
          if (flags & GF_RELU) val = fmaxf(val, 0.f);
          if (flags & GF_OUT_F32) static_cast<float*>(P.out)[o] = val;
          else static_cast<T*>(P.out)[o] = E::from_f32(val);
        } else if (EPIG == 0) {  // EPI_DGRAD
          if (P.aux0) val += E::to_f32(static_cast<const T*>(P.aux0)[o]);
          if (flags & GF_ACCUM) val += E::to_f32(static_cast<T*>(P.out)[o]);
          if (P.aux1 && !(E::to_f32(static_cast<const T*>(P.aux1)[o]) > 0.f)) val = 0.f;
          static_cast<T*>(P.out)[o] = E::from_f32(val);
        } else {  // EPI_WGRAD
          if (P.aux1) gsum += val * E::to_f32(static_cast<const T*>(P.aux1)[o]);
          float* G = static_cast<float*>(P.out) + o;
          const float gv = gam * val;
          if (flags & GF_ATOMIC) atomicAdd(G, gv);
          else *G = gold[(EPIG == 1) ? (i * NI + j) * 16 + v : 0] + gv;
        }
      }
      if (EPIG == 1 && P.aux2 != nullptr) {  // d gamma[r] = sum_c acc[r][c] * Wplain[r][c]
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) gsum += __shfl_xor(gsum, off, 64);
        if ((lane & 31) == 0 && r < P.M) atomicAdd(static_cast<float*>(P.aux2) + r, gsum);
      }
    }
  }
}

void tile_dims(int shape, int* bm, int* bn) {
  switch (shape) {
    case TILE_128x128: *bm = 128; *bn = 128; break;
    case TILE_64x128: *bm = 64; *bn = 128; break;
    default: *bm = 64; *bn = 64; break;
  }
}

// Reduction depth of one LDS slab per tile shape.  The 64-row shapes serve the small-
// batch Linear contractions, which stream a weight matrix once (HBM-bound): a deep slab
// keeps ~50 KB of loads in flight per workgroup.  The square shape serves convolutions
// and weight gradients.
template <typename T> struct SlabK;
template <> struct SlabK<uint16_t> { static constexpr int BIG = 32, SKINNY = 128; };
template <> struct SlabK<float> { static constexpr int BIG = 16, SKINNY = 64; };

template <typename T, int EPIG>
static hipError_t launch_typed(const GemmBatch& b, int shape, hipStream_t s) {
  dim3 grid(b.total_tiles), block(256);
  switch (shape) {
    case TILE_128x128: hipLaunchKernelGGL((gemm_grouped_kernel<T, 128, 128, SlabK<T>::BIG, 2, EPIG>), grid, block, 0, s, b); break;
    case TILE_64x128: hipLaunchKernelGGL((gemm_grouped_kernel<T, 64, 128, SlabK<T>::SKINNY, 2, EPIG>), grid, block, 0, s, b); break;
    default: hipLaunchKernelGGL((gemm_grouped_kernel<T, 64, 64, SlabK<T>::SKINNY, 2, EPIG>), grid, block, 0, s, b); break;
  }
  return hipGetLastError();
}

hipError_t launch_gemm_batch(GemmBatch& b, int dtype, int shape, hipStream_t stream) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > GEMM_MAX_PROBS) return hipErrorInvalidValue;
  int bm, bn;
  tile_dims(shape, &bm, &bn);
  int total = 0;
  const bool wgrad = b.p[0].epi == EPI_WGRAD;
  for (int i = 0; i < b.n; ++i) {
    GemmProb& p = b.p[i];
    if (p.M <= 0 || p.N <= 0 || p.K <= 0 || p.splits < 1) return hipErrorInvalidValue;
    if ((p.epi == EPI_WGRAD) != wgrad) return hipErrorInvalidValue;  // one epilogue family per launch
    if (p.splits > 1 && !(p.epi == EPI_WGRAD && (p.flags & GF_ATOMIC))) return hipErrorInvalidValue;
    p.tiles_n = (p.N + bn - 1) / bn;
    p.tile_begin = total;
    total += ((p.M + bm - 1) / bm) * p.tiles_n * p.splits;
  }
  b.total_tiles = total;
  if (dtype == DT_BF16) return wgrad ? launch_typed<uint16_t, 1>(b, shape, stream) : launch_typed<uint16_t, 0>(b, shape, stream);
  return wgrad ? launch_typed<float, 1>(b, shape, stream) : launch_typed<float, 0>(b, shape, stream);
}

}  // namespace cdp
