// HBM-streaming contractions of the Linear stages of a CDP tick (gfx950).
//
// With a micro-batch of B <= 64 rows every Linear pass reads or updates one weight-
// sized matrix exactly once for 2*B flops per element, far below the MFMA/HBM ridge, so
// these kernels are built to keep HBM busy rather than the matrix cores:
//   * skinny tile     C[M][N] = A[M][K] * W[N][K]^T  (forward with W, data gradient with
//                     the transposed copy W^T): 64-row tiles, 128-deep slabs, one slab of
//                     loads in flight per workgroup while the previous one is contracted;
//   * dw tile         G[N][K] (+)= dY[M][N]^T * X[M][K] (weight gradient): the old
//                     accumulator tile is requested before the operands so the read-
//                     modify-write stream is never waiting on the contraction; the bias
//                     gradient (column sums of dY) is folded into the first column tile.
// Workgroups are renumbered so that the tiles of one problem land on one XCD (its L2
// then holds that problem's activations once), and every workgroup starts its reduction
// loop at a different slab so that concurrent workgroups do not hit the same HBM
// channels (weight rows are a power of two apart).
#include <algorithm>

#include "elem.h"
#include "kernels.h"
#include "mfma_frag.h"
#include "sgd_step.h"

namespace cdp {

namespace {

template <typename T> struct LT : Elem<T> {
  static constexpr int SLAB = 16 * Elem<T>::VEC;  // reduction depth of a staged slab
};

// blockIdx -> logical tile: consecutive workgroup ids are dealt round-robin to the 8 XCDs,
// so XCD x receives the contiguous logical range [x*chunk, (x+1)*chunk).
__device__ __forceinline__ int xcd_remap(int bid, int total) {
  const int chunk = (total + 7) >> 3;
  return (bid & 7) * chunk + (bid >> 3);
}

// Rows of a weight-gradient tile (tiles_n is set).
__host__ __device__ __forceinline__ int dw_tile_rows(const GemmProb& p) {
  // (a long reduction, as in the lock-step run's batched passes, re-stages its operands per tile: keep 64 rows)
  return ((p.M + 63) / 64) * p.tiles_n < 512 && (p.K <= 64 || p.upd) ? 32 : 64;
}

}  // namespace

// One 16-byte chunk of operand elements read from an fp32 matrix and rounded to T (RNE), the
// same conversion the staging kernel applies: a first Linear layer can read the caller's
// fp32 micro-batch directly.
template <typename T>
__device__ __forceinline__ uint4 load_chunk_f32(const float* src) {
  if constexpr (sizeof(T) == 4) {
    return *reinterpret_cast<const uint4*>(src);
  } else {
    const float4 lo = *reinterpret_cast<const float4*>(src), hi = *reinterpret_cast<const float4*>(src + 4);
    return make_uint4((uint32_t)f32_to_bf16(lo.x) | ((uint32_t)f32_to_bf16(lo.y) << 16), (uint32_t)f32_to_bf16(lo.z) | ((uint32_t)f32_to_bf16(lo.w) << 16),
                      (uint32_t)f32_to_bf16(hi.x) | ((uint32_t)f32_to_bf16(hi.y) << 16), (uint32_t)f32_to_bf16(hi.z) | ((uint32_t)f32_to_bf16(hi.w) << 16));
  }
}

// Epilogue of one output element of a forward (bias, residual, ReLU) or data-gradient (addend, accumulate,
// ReLU mask) contraction, in two steps: what it reads from memory, then the arithmetic and the store.  A tile
// requests the operands of ALL its elements before the first store: a store may alias the later loads for all
// the compiler knows, so element by element every load would wait for the store before it and the epilogue
// would be one memory round trip per element.
struct EpiOperand {
  float a;     // forward: residual; data gradient: addend (+ the old output value when accumulating)
  float mask;  // data gradient: the ReLU argument (1 when there is no mask)
};
template <typename T>
__device__ __forceinline__ EpiOperand load_epilogue_operand(const GemmProb& P, int r, int c, bool inb) {
  using E = LT<T>;
  EpiOperand e{0.f, 1.f};
  if (!inb) return e;
  const int64_t o = (int64_t)r * P.ldo + c;
  if (P.epi == EPI_FWD) {
    if (P.aux1) e.a = E::to_f32(static_cast<const T*>(P.aux1)[o]);
  } else {
    // (val + addend) + old in the single-step form; here addend + old first: both are T values, their fp32 sum is
    // exact unless they differ by more than 2^16 in magnitude, and the tolerance of the result is that of a T value
    if (P.aux0) e.a = E::to_f32(static_cast<const T*>(P.aux0)[o]);
    if (P.flags & GF_ACCUM) e.a += E::to_f32(static_cast<const T*>(P.out)[o]);
    if (P.aux1) e.mask = E::to_f32(static_cast<const T*>(P.aux1)[o]);
  }
  return e;
}
template <typename T>
__device__ __forceinline__ void store_result(const GemmProb& P, int r, int c, float val, float bias, const EpiOperand& e) {
  using E = LT<T>;
  const int64_t o = (int64_t)r * P.ldo + c;
  if (P.epi == EPI_FWD) {
    val += bias;
    val += e.a;
    if (P.flags & GF_RELU) val = fmaxf(val, 0.f);
    if (P.flags & GF_OUT_F32) static_cast<float*>(P.out)[o] = val;
    else static_cast<T*>(P.out)[o] = E::from_f32(val);
  } else {
    val += e.a;
    if (!(e.mask > 0.f)) val = 0.f;
    static_cast<T*>(P.out)[o] = E::from_f32(val);
  }
}

// ---------------------------------------------------------------------------------
// skinny tile: 64 x BN outputs, waves 2 (rows) x 2 (cols).
template <typename T, int BN>
__device__ __forceinline__ void skinny_tile(const GemmBatch& batch, const GemmProb& P, int tile, unsigned char* smem) {
  using E = LT<T>;
  constexpr int BM = 64, BK = E::SLAB, VEC = E::VEC, LDP = BK + VEC;
  constexpr int NA = BM / 16, NB = BN / 16;  // 16-byte chunks per thread and slab
  constexpr int NI = BN / 64;                // 32-wide MFMA tiles per wave along N
  T* As = reinterpret_cast<T*>(smem);
  T* Bs = As + BM * LDP;

  // 64-column tiles of a launch short of workgroups share a long reduction among P.splits
  // workgroups (neighbours in the tile list), as the thin tiles do
  constexpr bool SPLIT = BN == 64;
  const int ks = SPLIT ? P.splits : 1, split = (tile - P.tile_begin) % ks;
  const int local = (tile - P.tile_begin) / ks;
  const int tn = local % P.tiles_n, tm = local / P.tiles_n;
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const T* __restrict__ Ap = static_cast<const T*>(P.A);
  const T* __restrict__ Bp = static_cast<const T*>(P.B);
  const int crow = tid >> 4, ck = (tid & 15) * VEC;  // this thread's chunk: rows crow + 16*i, columns ck..ck+VEC-1
  int offA[NA], offB[NB];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int r = row0 + crow + 16 * i;
    offA[i] = r < P.M ? r * P.lda + ck : -1;
  }
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int r = col0 + crow + 16 * i;
    offB[i] = r < P.N ? r * P.ldb + ck : -1;
  }
  // narrow tiles serve small problems whose k-loop is a chain of memory latencies: keep two
  // slabs of loads in flight; wide tiles are bandwidth-bound and keep occupancy instead
  constexpr int DEPTH = (BN == 64) ? 2 : 1;
  uint4 ra[DEPTH][NA], rb[DEPTH][NB];
  // rows are 16-byte aligned and K is a whole number of chunks: one vector load per chunk;
  // otherwise (e.g. a 10-class head) chunks are gathered element by element
  const bool vec = (P.K % VEC) == 0 && (P.lda % VEC) == 0 && (P.ldb % VEC) == 0;
  const bool a_f32 = (P.flags & GF_A_F32) != 0;  // A holds fp32 values (same leading dimension in elements)
  const float* __restrict__ Apf = static_cast<const float*>(P.A);
  auto gather = [&](const T* src, int k) {
    Chunk16<T> c;
    c.v = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < VEC; ++e)
      if (k + e < P.K) c.e[e] = src[e];
    return c.v;
  };
  auto gather_f32 = [&](const float* src, int k) {
    Chunk16<T> c;
    c.v = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < VEC; ++e)
      if (k + e < P.K) c.e[e] = E::from_f32(src[e]);
    return c.v;
  };
  auto fetch = [&](uint4* qa, uint4* qb, int k0) {
    const bool kin = k0 + ck < P.K;
    if (vec) {
#pragma unroll
      for (int i = 0; i < NA; ++i) {
        if (!(kin && offA[i] >= 0)) qa[i] = make_uint4(0, 0, 0, 0);
        else if (a_f32) qa[i] = load_chunk_f32<T>(Apf + offA[i] + k0);
        else qa[i] = *reinterpret_cast<const uint4*>(Ap + offA[i] + k0);
      }
#pragma unroll
      for (int i = 0; i < NB; ++i)
        qb[i] = (kin && offB[i] >= 0) ? *reinterpret_cast<const uint4*>(Bp + offB[i] + k0) : make_uint4(0, 0, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < NA; ++i) {
        if (!(kin && offA[i] >= 0)) qa[i] = make_uint4(0, 0, 0, 0);
        else if (a_f32) qa[i] = gather_f32(Apf + offA[i] + k0, k0 + ck);
        else qa[i] = gather(Ap + offA[i] + k0, k0 + ck);
      }
#pragma unroll
      for (int i = 0; i < NB; ++i) qb[i] = (kin && offB[i] >= 0) ? gather(Bp + offB[i] + k0, k0 + ck) : make_uint4(0, 0, 0, 0);
    }
  };

  v16f_t acc[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

  const int nslab_all = (P.K + BK - 1) / BK, per = (nslab_all + ks - 1) / ks;
  const int sb = split * per, nslab = max(0, min(nslab_all, sb + per) - sb);
  const int s0 = nslab > 0 ? (int)(((unsigned)tile * 2654435761u) >> 8) % nslab : 0;  // per-workgroup starting slab
  auto slab_k = [&](int i) { const int q = s0 + i; return (sb + (q >= nslab ? q - nslab : q)) * BK; };
  // An interior tile of whole chunks (every row of both operand blocks exists, K is whole slabs) loads without
  // a branch per chunk: guarded loads sit in basic blocks of their own and the compiler then waits for each.
  const bool clean = vec && !a_f32 && row0 + BM <= P.M && col0 + BN <= P.N && (P.K % BK) == 0;
  auto fetch_clean = [&](uint4* qa, uint4* qb, int k0) {
#pragma unroll
    for (int i = 0; i < NA; ++i) qa[i] = *reinterpret_cast<const uint4*>(Ap + offA[i] + k0);
#pragma unroll
    for (int i = 0; i < NB; ++i) qb[i] = *reinterpret_cast<const uint4*>(Bp + offB[i] + k0);
  };
  auto k_loop = [&](auto&& fetch_fn) {
#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (d < nslab) fetch_fn(ra[d], rb[d], slab_k(d));
  for (int it0 = 0; it0 < nslab; it0 += DEPTH)
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) {
    const int it = it0 + d;
    if (it >= nslab) break;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NA; ++i) *reinterpret_cast<uint4*>(As + (crow + 16 * i) * LDP + ck) = ra[d][i];
#pragma unroll
    for (int i = 0; i < NB; ++i) *reinterpret_cast<uint4*>(Bs + (crow + 16 * i) * LDP + ck) = rb[d][i];
    __syncthreads();
    if (it + DEPTH < nslab) fetch_fn(ra[d], rb[d], slab_k(it + DEPTH));
    const int kg = (lane >> 5) * E::KPL;
    const T* ap = As + (wm * 32 + (lane & 31)) * LDP + kg;
    const T* bp = Bs + (wn * (BN / 2) + (lane & 31)) * LDP + kg;
#pragma unroll
    for (int kk = 0; kk < BK; kk += E::MFMA_K) {
      if constexpr (sizeof(T) == 2) {
        const uint4 a = *reinterpret_cast<const uint4*>(ap + kk);
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[j] = mfma_bf16(a, *reinterpret_cast<const uint4*>(bp + j * 32 * LDP + kk), acc[j]);
      } else {
        const float a = ap[kk];
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bp[j * 32 * LDP + kk], acc[j], 0, 0, 0);
      }
    }
  }

  };
  if (clean) k_loop(fetch_clean);
  else k_loop(fetch);

  if constexpr (SPLIT) {
    if (ks > 1) {
      // partial tile (register order) -> this workgroup's slot; the last arrival adds the slots in order
      float* slot = batch.thin_ws + (int64_t)tile * batch.slot_floats;
#pragma unroll
      for (int v = 0; v < 16; ++v) __hip_atomic_store(slot + v * 256 + tid, acc[0][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stores are acknowledged before the barrier
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
      const float* first = batch.thin_ws + (int64_t)(tile - split) * batch.slot_floats + tid;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[0][v] = 0.f;
      for (int sp = 0; sp < ks; ++sp) {  // one round trip per slot
        float part[16];
#pragma unroll
        for (int v = 0; v < 16; ++v)
          part[v] = __hip_atomic_load(first + (int64_t)sp * batch.slot_floats + v * 256, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[0][v] += part[v];
      }
    }
  }
  EpiOperand eo[NI][16];
  float bias[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int c = col0 + wn * (BN / 2) + j * 32 + (lane & 31);
    bias[j] = (P.epi == EPI_FWD && P.aux0 != nullptr && c < P.N) ? static_cast<const float*>(P.aux0)[c] : 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = row0 + wm * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      eo[j][v] = load_epilogue_operand<T>(P, r, c, r < P.M && c < P.N);
    }
  }
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int c = col0 + wn * (BN / 2) + j * 32 + (lane & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = row0 + wm * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      if (r >= P.M || c >= P.N) continue;
      store_result<T>(P, r, c, acc[j][v], bias[j], eo[j][v]);
    }
  }
}

// ---------------------------------------------------------------------------------
// thin tile: problems of at most 32 rows whose operands are whole 16-byte chunks.  A
// workgroup owns 32 x 32 outputs and its four waves split the reduction: wave w takes
// slabs w, w+4, ... through a staging block of its own.  The k-loop has no barrier; the
// partial tiles meet once in LDS, each wave finishing 8 of the 32 rows.
template <typename T>
__device__ __forceinline__ void thin_tile(const GemmBatch& batch, const GemmProb& P, int tile, unsigned char* smem) {
  using E = LT<T>;
  constexpr int VEC = E::VEC, CH = 4, SLAB = 2 * CH * VEC;  // chunk c of lane (row, g) holds k = 2*VEC*c + VEC*g ...
  // a long reduction is shared by P.splits workgroups (neighbours in the tile list), each
  // taking a contiguous range of slabs; the one that finishes last adds the partial tiles
  const int ks = P.splits, local = tile - P.tile_begin;
  const int split = local % ks;
  const int col0 = (local / ks) * 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r31 = lane & 31, g = lane >> 5;
  const bool a_f32 = (P.flags & GF_A_F32) != 0;
  // Operands reach the MFMA through a staging block of this wavefront's own in LDS: a slab of
  // 32 rows x 128 bytes per operand is fetched with four load instructions whose lanes cover
  // whole 128-byte row pieces (lane l: row 8j + l/8, 16-byte chunk l%8), a quarter of the
  // cache-line requests that loading the fragments directly (32 rows x 32 bytes per
  // instruction) makes - the request rate of the CU, not latency, bounded the k-loop - then
  // written to LDS and read back as fragments.  No barrier: the block is private to the
  // wavefront, whose LDS instructions execute in order.
  constexpr int LP = SLAB + VEC;  // LDS pitch (elements): 144 bytes, fragment reads of 32 rows hit 32 distinct bank groups
  T* const stA = reinterpret_cast<T*>(smem) + wave * (2 * 32 * LP);
  T* const stB = stA + 32 * LP;
  const int lrow = lane >> 3, lk = (lane & 7) * VEC;
  // rows past the end are read from the last valid row: they only reach outputs that are not stored
  const T* __restrict__ Ap = static_cast<const T*>(P.A);
  const float* __restrict__ Apf = static_cast<const float*>(P.A);
  const T* __restrict__ Bp = static_cast<const T*>(P.B);
  int offA[4], offB[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    offA[j] = min(8 * j + lrow, P.M - 1) * P.lda + lk;
    offB[j] = min(col0 + 8 * j + lrow, P.N - 1) * P.ldb + lk;
  }
  const int nslab_all = (P.K + SLAB - 1) / SLAB, per = (nslab_all + ks - 1) / ks;
  const int sb = split * per, nslab = max(0, min(nslab_all, sb + per) - sb);
  const int s0 = nslab > 0 ? (int)(((unsigned)tile * 2654435761u) >> 8) % nslab : 0;
  auto slab_k = [&](int i) { const int q = s0 + i; return (sb + (q >= nslab ? q - nslab : q)) * SLAB; };

  uint4 ra[2][4], rb[2][4];
  auto fetch = [&](uint4* qa, uint4* qb, int k0) {
    const bool kin = k0 + lk < P.K;  // chunks past K are zero in both operands (last, partial slab)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!kin) qa[j] = make_uint4(0, 0, 0, 0);
      else qa[j] = a_f32 ? load_chunk_f32<T>(Apf + offA[j] + k0) : *reinterpret_cast<const uint4*>(Ap + offA[j] + k0);
      qb[j] = kin ? *reinterpret_cast<const uint4*>(Bp + offB[j] + k0) : make_uint4(0, 0, 0, 0);
    }
  };
  v16f_t acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  auto contract = [&](const uint4* qa, const uint4* qb) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      *reinterpret_cast<uint4*>(stA + (8 * j + lrow) * LP + lk) = qa[j];
      *reinterpret_cast<uint4*>(stB + (8 * j + lrow) * LP + lk) = qb[j];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint4 fa[CH], fb[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {  // chunk c of lane (row, g) holds k = 2*VEC*c + VEC*g ...
      fa[c] = *reinterpret_cast<const uint4*>(stA + r31 * LP + 2 * VEC * c + VEC * g);
      fb[c] = *reinterpret_cast<const uint4*>(stB + r31 * LP + 2 * VEC * c + VEC * g);
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      if constexpr (sizeof(T) == 2) {
        acc = mfma_bf16(fa[c], fb[c], acc);
      } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[c].x), __uint_as_float(fb[c].x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[c].y), __uint_as_float(fb[c].y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[c].z), __uint_as_float(fb[c].z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[c].w), __uint_as_float(fb[c].w), acc, 0, 0, 0);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the fragments are in registers before the block is written again
  };
  int s = wave;
  if (s < nslab) fetch(ra[0], rb[0], slab_k(s));
  if (s + 4 < nslab) fetch(ra[1], rb[1], slab_k(s + 4));
  for (; s < nslab; s += 8) {
    contract(ra[0], rb[0]);
    if (s + 8 < nslab) fetch(ra[0], rb[0], slab_k(s + 8));
    if (s + 4 < nslab) {
      contract(ra[1], rb[1]);
      if (s + 12 < nslab) fetch(ra[1], rb[1], slab_k(s + 12));
    }
  }
  __syncthreads();  // the partial sums below reuse the staging blocks of all wavefronts

  float* red = reinterpret_cast<float*>(smem);  // [4 waves][16][64 lanes]
#pragma unroll
  for (int v = 0; v < 16; ++v) red[(wave * 16 + v) * 64 + lane] = acc[v];
  __syncthreads();
  const int c = col0 + r31;
  const float bias = (P.epi == EPI_FWD && P.aux0 != nullptr && c < P.N) ? static_cast<const float*>(P.aux0)[c] : 0.f;
  const bool ce = (P.flags & GF_CE) != 0;
  float vals[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int v = wave * 4 + q;
    vals[q] = (red[v * 64 + lane] + red[(16 + v) * 64 + lane]) + (red[(32 + v) * 64 + lane] + red[(48 + v) * 64 + lane]);
  }
  if (ks > 1) {
    // partial tile -> workspace slot of this workgroup; the last of the ks workgroups to get
    // here (counter of the output tile) sums the slots in a fixed order and finishes the tile
    // Partials and counter are device-scope atomics (they bypass the per-XCD L2), ordered by
    // waiting for the stores to complete; a device-scope fence here would write back every
    // dirty L2 line of the weight-gradient tiles that share the launch.
    float* slot = batch.thin_ws + (int64_t)tile * batch.slot_floats;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      __hip_atomic_store(slot + (wave * 4 + q) * 64 + lane, vals[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // every store above has been acknowledged before this wavefront reaches the barrier (a
    // workgroup-scope fence alone does not wait for global stores)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();  // also: every wave has read its share of `red`
    unsigned int* cnt = batch.thin_cnt + (tile - split);
    if (tid == 0) {
      const unsigned int arrived = atomicAdd(cnt, 1u);
      red[0] = arrived == (unsigned)(ks - 1) ? 1.f : 0.f;
      if (arrived == (unsigned)(ks - 1)) atomicExch(cnt, 0u);  // ready for the next launch
    }
    __syncthreads();
    if (red[0] == 0.f) return;
    const float* first = batch.thin_ws + (int64_t)(tile - split) * batch.slot_floats;
#pragma unroll
    for (int q = 0; q < 4; ++q) vals[q] = 0.f;
    for (int sp = 0; sp < ks; ++sp) {  // one round trip per slot
      float part[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        part[q] = __hip_atomic_load(first + (int64_t)sp * batch.slot_floats + (wave * 4 + q) * 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
      for (int q = 0; q < 4; ++q) vals[q] += part[q];
    }
  }
  EpiOperand eo[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = wave * 8 + g * 4 + q;
    eo[q] = load_epilogue_operand<T>(P, r, c, !ce && r < P.M && c < P.N);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float val = vals[q];
    const int r = wave * 8 + g * 4 + q;
    if (!ce) {
      if (r < P.M && c < P.N) store_result<T>(P, r, c, val, bias, eo[q]);
      continue;
    }
    // Loss head on the logits row this half wavefront holds (one class per lane, N <= 32):
    // softmax cross-entropy, dlogits = (softmax - onehot) / rows, row loss added to its slot.
    // out = dlogits T[M][N], aux2 = labels, aux3 = loss slots, g.H = rows per loss slot.
    const bool cls = c < P.N;
    const float z = cls ? val + bias : -INFINITY;
    float m = z;
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    const float e = cls ? expf(z - m) : 0.f;
    float sum = e;
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
    const int y = r < P.M ? static_cast<const int32_t*>(P.aux2)[r] : -1;
    float own = (cls && c == y) ? (m + logf(sum)) - z : 0.f;  // the row's loss sits in the lane of its label
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) own += __shfl_xor(own, off, 64);
    if (r < P.M) {
      if (cls) static_cast<T*>(P.out)[(int64_t)r * P.ldo + c] = E::from_f32((e / sum - (c == y ? 1.f : 0.f)) / (float)P.M);
      if (r31 == 0) atomicAdd(static_cast<int*>(P.aux3) + r / P.g.H, __float2int_rn(own / (float)P.g.H * LOSS_SCALE));  // fixed point: order-independent
    }
  }
}

// ---------------------------------------------------------------------------------
// dw_kernel: G tile of TN = 64 (rows n) x 128 (cols k); wave w owns columns [32w, 32w+32).
// Tiles are 32 rows high when the matrix has few of them (dw_tile_rows): twice as many
// workgroups share what are the longest tiles of a small launch.
// Operand convention of the batch entry: A = dY [Mb][N] (lda = N), B = X [Mb][K]
// (ldb = K), out = G [N][K] (ldo = K), P.M = N, P.N = K, P.K = Mb (reduction length);
// aux2 = bias-gradient vector [N] or NULL.
template <typename T, int TN>
__device__ __forceinline__ void dw_tile(const GemmBatch& batch, const GemmProb& P, int tile, unsigned char* smem) {
  using E = LT<T>;
  constexpr int TK = 128, MB = 64, VEC = E::VEC, NI2 = TN / 32;
  // LDS pitches (elements): bf16 fragments are read with the transposing LDS read, which wants
  // 32 bytes modulo 128 between consecutive rows; fp32 fragments are plain column reads
  constexpr int PAD = sizeof(T) == 2 ? 16 : 4;
  constexpr int PD = 64 + PAD, PX = TK + PAD;  // one pitch for both tile heights
  T* Ds = reinterpret_cast<T*>(smem);
  T* Xs = Ds + MB * PD;

  const int local = tile - P.tile_begin;
  const int tk = local % P.tiles_n, tnn = local / P.tiles_n;
  const int n0 = tnn * TN, k0 = tk * TK;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int Nn = P.M, Kk = P.N, Mb = P.K;
  const int flags = P.flags;
  float* __restrict__ G = static_cast<float*>(P.out);

  // 1. request the old accumulator tile (read-modify-write) before anything else.  A tile that
  // also takes the SGD step requests its master weights (and velocities) now as well and keeps
  // one combined value per element, so that only this micro-batch's share is missing:
  //   plain / weight decay:  w' = [w - lr*(Gold/N + wd*w)] - (lr/N)*acc
  //   momentum:              v' = [mu*v + Gold/N + wd*w] + acc/N ,  w' = w - lr*v'
  const bool rmw = (flags & GF_ACCUM) != 0;
  const bool upd = P.upd != 0;
  const LinUpdate& U = batch.upd[upd ? P.upd - 1 : 0];
  const bool mom = upd && U.V != nullptr;
  const int gc = k0 + wave * 32 + (lane & 31);
  float gold[16 * NI2];
#pragma unroll
  for (int i = 0; i < NI2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = n0 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      const bool inb = r < Nn && gc < Kk;
      const int64_t idx = (int64_t)r * P.ldo + gc;
      gold[i * 16 + v] = (rmw && inb) ? G[idx] : 0.f;
    }
  if (upd) {
    // All master weights (and velocities) of the tile are requested before the first one is used: read inside
    // a per-element branch, each was waited for before the next was issued, 32 memory round trips in a row.
    // Outside the matrix everything reads 0 and combines to 0.
    float wm[16 * NI2];
#pragma unroll
    for (int i = 0; i < NI2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = n0 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        wm[i * 16 + v] = (r < Nn && gc < Kk) ? U.master[(int64_t)r * P.ldo + gc] : 0.f;
      }
    if (mom) {
      float vm[16 * NI2];
#pragma unroll
      for (int i = 0; i < NI2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = n0 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          vm[i * 16 + v] = (r < Nn && gc < Kk) ? U.V[(int64_t)r * P.ldo + gc] : 0.f;
        }
#pragma unroll
      for (int e = 0; e < 16 * NI2; ++e) {
        const float gw = gold[e] * U.sgd.inv_n + U.sgd.wd * wm[e];
        gold[e] = U.sgd.momentum * vm[e] + gw;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16 * NI2; ++e) {
        const float gw = gold[e] * U.sgd.inv_n + U.sgd.wd * wm[e];
        gold[e] = wm[e] - U.sgd.lr * gw;
      }
    }
  }

  v16f_t acc[NI2];
#pragma unroll
  for (int i = 0; i < NI2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  float bsum = 0.f;  // bias gradient of column n0 + tid (threads 0..63 of the first column tile)

  const bool dvec = (P.lda % VEC) == 0, xvec = (P.ldb % VEC) == 0;
  // the reduction runs over the rows of one micro-batch, or (GF_GROUP) of several micro-batches whose dY / X
  // lie in buffers of their own
  const bool grouped = (flags & GF_GROUP) != 0;
  const int rows = grouped ? P.g.pad : Mb, nmem = grouped ? Mb / P.g.pad : 1;
  constexpr int DCH = TN / VEC, XCH = TK / VEC;  // chunks per row
  constexpr int ND = MB * DCH / 256, NX = MB * XCH / 256;
  static_assert(ND * 256 == MB * DCH && NX * 256 == MB * XCH, "whole chunks per thread");
  // 3. contraction over the batch rows of the staged slab; fragments are read transposed out of LDS
  auto contract = [&]() {
    const int g = lane >> 5, l31 = lane & 31;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int kk = 0; kk < MB; kk += 16) {
        const uint4 bv = frag_tr_bf16(Xs, PX, kk, wave * 32, lane);
#pragma unroll
        for (int i = 0; i < NI2; ++i) acc[i] = mfma_bf16(frag_tr_bf16(Ds, PD, kk, i * 32, lane), bv, acc[i]);
      }
    } else {
#pragma unroll 8
      for (int kk = 0; kk < MB; kk += 2) {
        const float bv = Xs[(kk + g) * PX + wave * 32 + l31];
#pragma unroll
        for (int i = 0; i < NI2; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(Ds[(kk + g) * PD + i * 32 + l31], bv, acc[i], 0, 0, 0);
      }
    }
    if (tk == 0 && P.aux2 != nullptr && tid < TN) {
      for (int m = 0; m < MB; ++m) bsum += E::to_f32(Ds[m * PD + tid]);
    }
  };
  if (dvec && xvec && (Nn % VEC) == 0 && (Kk % VEC) == 0) {
    // 2. every chunk is whole (inside or outside the matrices): slabs of 64 batch rows of dY[.., n0..n0+TN-1] and
    // X[.., k0..k0+127] are staged as they lie in memory, one slab ahead: the next slab (of this member or of the
    // next one of the group) is requested before the current one is contracted, so a reduction over several
    // slabs is not one memory round trip per slab.  All of a thread's chunks are requested before the first one
    // is written to LDS (requested one by one, the six round trips of a bf16 tile cost 30 us of a 280 us launch
    // of 16384 tiles).
    const int per = (rows + MB - 1) / MB, nit = nmem * per;
    uint4 rd[ND], rx[NX];
    auto fetch = [&](int it) {
      const int mem = it / per, m0 = (it - mem * per) * MB;
      const T* __restrict__ Dp = static_cast<const T*>(dw_member(P, mem, 0));
      const T* __restrict__ Xp = static_cast<const T*>(dw_member(P, mem, 1));
#pragma unroll
      for (int i = 0; i < ND; ++i) {
        const int id = tid + 256 * i, m = id / DCH, c = (id % DCH) * VEC;
        rd[i] = (m0 + m < rows && n0 + c < Nn) ? *reinterpret_cast<const uint4*>(Dp + (int64_t)(m0 + m) * P.lda + n0 + c)
                                              : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < NX; ++i) {
        const int id = tid + 256 * i, m = id / XCH, c = (id % XCH) * VEC;
        rx[i] = (m0 + m < rows && k0 + c < Kk) ? *reinterpret_cast<const uint4*>(Xp + (int64_t)(m0 + m) * P.ldb + k0 + c)
                                              : make_uint4(0, 0, 0, 0);
      }
    };
    fetch(0);
    for (int it = 0; it < nit; ++it) {
      if (it > 0) __syncthreads();
#pragma unroll
      for (int i = 0; i < ND; ++i) {
        const int id = tid + 256 * i, m = id / DCH, c = (id % DCH) * VEC;
        Chunk16<T> tmp;
        tmp.v = rd[i];
        uint2* dst = reinterpret_cast<uint2*>(Ds + m * PD + c);
        dst[0] = tmp.h[0];
        dst[1] = tmp.h[1];
      }
#pragma unroll
      for (int i = 0; i < NX; ++i) {
        const int id = tid + 256 * i, m = id / XCH, c = (id % XCH) * VEC;
        Chunk16<T> tmp;
        tmp.v = rx[i];
        uint2* dst = reinterpret_cast<uint2*>(Xs + m * PX + c);
        dst[0] = tmp.h[0];
        dst[1] = tmp.h[1];
      }
      __syncthreads();
      if (it + 1 < nit) fetch(it + 1);
      contract();
    }
  } else {
  for (int mem = 0; mem < nmem; ++mem) {
  const T* __restrict__ Dp = static_cast<const T*>(dw_member(P, mem, 0));
  const T* __restrict__ Xp = static_cast<const T*>(dw_member(P, mem, 1));
  for (int m0 = 0; m0 < rows; m0 += MB) {
    if (mem > 0 || m0 > 0) __syncthreads();
    {
      for (int id = tid; id < MB * DCH; id += 256) {
        const int m = id / DCH, c = (id % DCH) * VEC;
        Chunk16<T> tmp;
        tmp.v = make_uint4(0, 0, 0, 0);
        if (m0 + m < rows) {
          const T* src = Dp + (int64_t)(m0 + m) * P.lda + n0 + c;
          if (dvec && n0 + c + VEC <= Nn) {
            tmp.v = *reinterpret_cast<const uint4*>(src);
          } else {
  #pragma unroll
            for (int e = 0; e < VEC; ++e)
              if (n0 + c + e < Nn) tmp.e[e] = src[e];
          }
        }
        uint2* dst = reinterpret_cast<uint2*>(Ds + m * PD + c);
        dst[0] = tmp.h[0];
        dst[1] = tmp.h[1];
      }
      for (int id = tid; id < MB * XCH; id += 256) {
        const int m = id / XCH, c = (id % XCH) * VEC;
        Chunk16<T> tmp;
        tmp.v = make_uint4(0, 0, 0, 0);
        if (m0 + m < rows) {
          const T* src = Xp + (int64_t)(m0 + m) * P.ldb + k0 + c;
          if (xvec && k0 + c + VEC <= Kk) {
            tmp.v = *reinterpret_cast<const uint4*>(src);
          } else {
  #pragma unroll
            for (int e = 0; e < VEC; ++e)
              if (k0 + c + e < Kk) tmp.e[e] = src[e];
          }
        }
        uint2* dst = reinterpret_cast<uint2*>(Xs + m * PX + c);
        dst[0] = tmp.h[0];
        dst[1] = tmp.h[1];
      }
    }
    __syncthreads();
    contract();
  }
  }
  }

  if (!upd) {
    // 4. accumulate and write back
#pragma unroll
    for (int i = 0; i < NI2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = n0 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (r < Nn && gc < Kk) G[(int64_t)r * P.ldo + gc] = gold[i * 16 + v] + acc[i][v];
      }
    if (tk == 0 && P.aux2 != nullptr && tid < TN && n0 + tid < Nn) {
      float* gb = static_cast<float*>(P.aux2) + n0 + tid;
      *gb = rmw ? (*gb + bsum) : bsum;
    }
    return;
  }

  // 4'. this contraction completes the sum over the micro-batches: take the SGD step on the
  // tile's master weights and write both compute copies of the new version
  constexpr int PW = TK + (sizeof(T) == 2 ? 2 : 1);  // LDS pitch of the new-weight tile [TN][TK]
  T* Ws = reinterpret_cast<T*>(smem);
  __syncthreads();  // the operand tiles in LDS are no longer read
  // (parameters and pointers in locals: read through the descriptor they are fetched again after every store)
  const float lr = U.sgd.lr, inv_n = U.sgd.inv_n, step = U.sgd.lr * U.sgd.inv_n;
  float* const master = U.master;
  float* const Vel = U.V;
  float wm[16 * NI2];
  if (mom) {  // the master weights again, all requested before the first store
#pragma unroll
    for (int i = 0; i < NI2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = n0 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        wm[i * 16 + v] = (r < Nn && gc < Kk) ? master[(int64_t)r * P.ldo + gc] : 0.f;
      }
  }
#pragma unroll
  for (int i = 0; i < NI2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rl = i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      const int r = n0 + rl;
      float w = 0.f;
      if (r < Nn && gc < Kk) {
        const int64_t idx = (int64_t)r * P.ldo + gc;
        if (mom) {
          const float vel = gold[i * 16 + v] + acc[i][v] * inv_n;
          Vel[idx] = vel;
          w = wm[i * 16 + v] - lr * vel;
        } else {
          w = gold[i * 16 + v] - step * acc[i][v];
        }
        master[idx] = w;
      }
      Ws[rl * PW + wave * 32 + (lane & 31)] = E::from_f32(w);
    }
  __syncthreads();
  T* __restrict__ wf = static_cast<T*>(U.wf);
  T* __restrict__ wt = static_cast<T*>(U.wt);
  {  // forward layout: rows n, 16-byte chunks along k
    constexpr int CPR = TK / VEC;
    const bool al = (Kk % VEC) == 0;
    for (int id = tid; id < TN * CPR; id += 256) {
      const int n = id / CPR, ck = (id % CPR) * VEC;
      if (n0 + n >= Nn || k0 + ck >= Kk) continue;
      Chunk16<T> tmp;
#pragma unroll
      for (int e = 0; e < VEC; ++e) tmp.e[e] = Ws[n * PW + ck + e];
      T* dst = wf + (int64_t)(n0 + n) * Kk + k0 + ck;
      if (al) {
        *reinterpret_cast<uint4*>(dst) = tmp.v;
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e)
          if (k0 + ck + e < Kk) dst[e] = tmp.e[e];
      }
    }
  }
  {  // data-gradient layout: rows k, 16-byte chunks along n (read transposed out of LDS)
    constexpr int CPR = TN / VEC;
    const bool al = (Nn % VEC) == 0;
    for (int id = tid; id < TK * CPR; id += 256) {
      const int k = id / CPR, cn = (id % CPR) * VEC;
      if (k0 + k >= Kk || n0 + cn >= Nn) continue;
      Chunk16<T> tmp;
#pragma unroll
      for (int e = 0; e < VEC; ++e) tmp.e[e] = Ws[(cn + e) * PW + k];
      T* dst = wt + (int64_t)(k0 + k) * Nn + n0 + cn;
      if (al) {
        *reinterpret_cast<uint4*>(dst) = tmp.v;
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e)
          if (n0 + cn + e < Nn) dst[e] = tmp.e[e];
      }
    }
  }
  if (tk == 0 && U.bmaster != nullptr && tid < TN && n0 + tid < Nn) {
    const int n = n0 + tid;
    const float gb = (rmw ? static_cast<const float*>(P.aux2)[n] : 0.f) + bsum;
    const float b = sgd_step(U.bmaster[n], gb, U.bV ? U.bV + n : nullptr, U.sgd);
    U.bmaster[n] = b;
    U.bcopy[n] = b;
  }
}

// ---------------------------------------------------------------------------------
// dw_run: DW_RUN consecutive 64 x 128 tiles of one row block of G per workgroup, software-pipelined.  With one
// tile per workgroup the resident workgroups of a launch move in step (request, wait, contract, store), and the
// time of the operand / contraction phase adds to the time of the accumulator stream instead of hiding under
// it (a 16384-tile launch: 117 us without the accumulator traffic, 188 us for that traffic alone, 280 us
// together).  Here the accumulator tile and the X tile of the NEXT column tile are requested before the
// current one is contracted and written back, and the dY tile is staged once for the whole run.
// For plain accumulate tiles (no fused SGD step) of a single reduction slab (at most 64 batch rows) whose
// operand chunks are whole; same operand convention as dw_tile.
constexpr int DW_RUN = 2;  // 2, 4 and 8 measured within 2 % of each other on 4096 x 4096 accumulators; 2 leaves most workgroups
// upd_ok: a problem with a fused SGD step may take this path (wide kernel, no momentum)
__host__ __device__ __forceinline__ int dw_run_length(const GemmProb& p, int vec, bool upd_ok) {
  const bool whole = p.lda % vec == 0 && p.ldb % vec == 0 && p.M % vec == 0 && p.N % vec == 0;
  const bool off32 = (int64_t)p.M * p.ldo < (1ll << 30);  // accumulator elements are addressed by 32-bit byte offsets
  return ((!p.upd || upd_ok) && whole && off32 && !(p.flags & GF_GROUP) && p.K <= 64 && p.N >= 8 * 128 && p.M >= 512) ? DW_RUN : 1;
}

template <typename T, bool UPD>
__device__ __forceinline__ void dw_run(const GemmBatch& batch, const GemmProb& P, int tile, unsigned char* smem) {
  using E = LT<T>;
  constexpr int TN = 64, TK = 128, MB = 64, VEC = E::VEC, NI2 = TN / 32;
  constexpr int PAD = sizeof(T) == 2 ? 16 : 4;
  constexpr int PD = 64 + PAD, PX = TK + PAD;
  constexpr int PW = TK + (sizeof(T) == 2 ? 2 : 1);  // LDS pitch of the new-weight tile [TN][TK] (UPD)
  T* Ds = reinterpret_cast<T*>(smem);
  T* Xs = Ds + MB * PD;
  T* Ws = Xs + MB * PX;
  const int groups = (P.tiles_n + DW_RUN - 1) / DW_RUN;
  const int local = tile - P.tile_begin;
  const int tk0 = (local % groups) * DW_RUN, tnn = local / groups;
  const int nrun = min(DW_RUN, P.tiles_n - tk0);
  const int n0 = tnn * TN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int Nn = P.M, Kk = P.N, Mb = P.K;
  const bool rmw = (P.flags & GF_ACCUM) != 0;
  const LinUpdate& U = batch.upd[UPD ? P.upd - 1 : 0];
  float* __restrict__ G = static_cast<float*>(P.out);
  const T* __restrict__ Dp = static_cast<const T*>(P.A);
  const T* __restrict__ Xp = static_cast<const T*>(P.B);
  constexpr int DCH = TN / VEC, XCH = TK / VEC;
  constexpr int ND = MB * DCH / 256, NX = MB * XCH / 256;

  // (parameters and pointers of the SGD step in locals: read through the descriptor they are fetched again after every store)
  const float upd_lr = UPD ? U.sgd.lr : 0.f, upd_inv_n = UPD ? U.sgd.inv_n : 0.f, upd_wd = UPD ? U.sgd.wd : 0.f;
  const float upd_step = upd_lr * upd_inv_n;
  float* const upd_master = UPD ? U.master : nullptr;
  float gold[2][16 * NI2];
  uint4 rx[NX];
  // old accumulator values; with a fused SGD step combined with the master weights so that only this
  // micro-batch's share is missing: w' = [w - lr*(Gold/N + wd*w)] - (lr/N)*acc
  // Element (r, c) of an accumulator-shaped array at a 32-bit byte offset from its (uniform) base: the row
  // offsets of a tile then cost one register each where 64-bit indices cost two, which is what decides
  // whether the update tiles fit the kernel's register budget.  dw_run_length admits only matrices below 4 GiB.
  const uint32_t ldo4 = (uint32_t)P.ldo * 4u;
  auto at32 = [&](float* base, int r, int c) -> float* {
    return reinterpret_cast<float*>(reinterpret_cast<char*>(base) + ((uint32_t)r * ldo4 + (uint32_t)c * 4u));
  };
  // Accumulator tile; with a fused SGD step finish_gold then combines it with the master weights.  Every element
  // of an array is requested before the first value is used: with the master weight read inside a per-element
  // branch the compiler waited for each one before it issued the next, 32 memory round trips in a row per tile.
  // (Outside the matrix both reads give 0 and so does the combination.)
  auto load_gold = [&](float* g, int k0) {
    const int gc = k0 + wave * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < NI2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = n0 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        g[i * 16 + v] = (rmw && r < Nn && gc < Kk) ? *at32(G, r, gc) : 0.f;
      }
  };
  auto finish_gold = [&](float* g, int k0) {
    if constexpr (UPD) {
      const int gc = k0 + wave * 32 + (lane & 31);
      float wm[16 * NI2];
#pragma unroll
      for (int i = 0; i < NI2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = n0 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          wm[i * 16 + v] = (r < Nn && gc < Kk) ? *at32(upd_master, r, gc) : 0.f;
        }
#pragma unroll
      for (int e = 0; e < 16 * NI2; ++e) {
        const float w = wm[e];
        g[e] = w - upd_lr * (g[e] * upd_inv_n + upd_wd * w);
      }
    }
  };
  auto load_x = [&](int k0) {
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int id = tid + 256 * i, m = id / XCH, c = (id % XCH) * VEC;
      rx[i] = (m < Mb && k0 + c < Kk) ? *reinterpret_cast<const uint4*>(Xp + (int64_t)m * P.ldb + k0 + c) : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_x = [&]() {
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int id = tid + 256 * i, m = id / XCH, c = (id % XCH) * VEC;
      Chunk16<T> tmp;
      tmp.v = rx[i];
      uint2* dst = reinterpret_cast<uint2*>(Xs + m * PX + c);
      dst[0] = tmp.h[0];
      dst[1] = tmp.h[1];
    }
  };

  // prologue: accumulator tile 0, the dY tile of the row block, X tile 0
  load_gold(gold[0], tk0 * TK);
  {
    uint4 rd[ND];
#pragma unroll
    for (int i = 0; i < ND; ++i) {
      const int id = tid + 256 * i, m = id / DCH, c = (id % DCH) * VEC;
      rd[i] = (m < Mb && n0 + c < Nn) ? *reinterpret_cast<const uint4*>(Dp + (int64_t)m * P.lda + n0 + c) : make_uint4(0, 0, 0, 0);
    }
    load_x(tk0 * TK);
#pragma unroll
    for (int i = 0; i < ND; ++i) {
      const int id = tid + 256 * i, m = id / DCH, c = (id % DCH) * VEC;
      Chunk16<T> tmp;
      tmp.v = rd[i];
      uint2* dst = reinterpret_cast<uint2*>(Ds + m * PD + c);
      dst[0] = tmp.h[0];
      dst[1] = tmp.h[1];
    }
    store_x();
  }
  finish_gold(gold[0], tk0 * TK);  // after the staging: both together need more registers than the kernel has
  __syncthreads();
  float bsum = 0.f;  // bias gradient of column n0 + tid (first column tile of the matrix only)
  if (tk0 == 0 && P.aux2 != nullptr && tid < TN)
    for (int m = 0; m < MB; ++m) bsum += E::to_f32(Ds[m * PD + tid]);

#pragma unroll
  for (int t = 0; t < DW_RUN; ++t) {
    if (t >= nrun) break;
    const int k0 = (tk0 + t) * TK;
    float* gcur = gold[t & 1];
    // next tile's accumulator and X tile are on their way while this one is contracted and written back
    if (t + 1 < nrun) {
      load_gold(gold[(t + 1) & 1], k0 + TK);
      finish_gold(gold[(t + 1) & 1], k0 + TK);
      load_x(k0 + TK);
    }
    v16f_t acc[NI2];
#pragma unroll
    for (int i = 0; i < NI2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const int g = lane >> 5, l31 = lane & 31;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int kk = 0; kk < MB; kk += 16) {
        const uint4 bv = frag_tr_bf16(Xs, PX, kk, wave * 32, lane);
#pragma unroll
        for (int i = 0; i < NI2; ++i) acc[i] = mfma_bf16(frag_tr_bf16(Ds, PD, kk, i * 32, lane), bv, acc[i]);
      }
    } else {
#pragma unroll 8
      for (int kk = 0; kk < MB; kk += 2) {
        const float bv = Xs[(kk + g) * PX + wave * 32 + l31];
#pragma unroll
        for (int i = 0; i < NI2; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(Ds[(kk + g) * PD + i * 32 + l31], bv, acc[i], 0, 0, 0);
      }
    }
    const int gc = k0 + wave * 32 + l31;
#pragma unroll
    for (int i = 0; i < NI2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int rl = i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
        const int r = n0 + rl;
        if constexpr (!UPD) {
          if (r < Nn && gc < Kk) *at32(G, r, gc) = gcur[i * 16 + v] + acc[i][v];
        } else {
          // this contraction completes the sum over the micro-batches: the SGD step on the master weights
          float w = 0.f;
          if (r < Nn && gc < Kk) {
            w = gcur[i * 16 + v] - upd_step * acc[i][v];
            *at32(upd_master, r, gc) = w;
          }
          Ws[rl * PW + wave * 32 + l31] = E::from_f32(w);
        }
      }
    if (UPD || t + 1 < nrun) __syncthreads();  // every wave has read its fragments of X tile t; Ws is complete
    if (t + 1 < nrun) store_x();
    if constexpr (UPD) {
      // both compute copies of the new version, out of the new-weight tile in LDS
      T* __restrict__ wf = static_cast<T*>(U.wf);
      T* __restrict__ wt = static_cast<T*>(U.wt);
      {  // forward layout: rows n, 16-byte chunks along k
        constexpr int CPR = TK / VEC;
        for (int id = tid; id < TN * CPR; id += 256) {
          const int n = id / CPR, ck = (id % CPR) * VEC;
          if (n0 + n >= Nn || k0 + ck >= Kk) continue;
          Chunk16<T> tmp;
#pragma unroll
          for (int e = 0; e < VEC; ++e) tmp.e[e] = Ws[n * PW + ck + e];
          *reinterpret_cast<uint4*>(wf + (int64_t)(n0 + n) * Kk + k0 + ck) = tmp.v;
        }
      }
      {  // data-gradient layout: rows k, 16-byte chunks along n (read transposed out of LDS)
        constexpr int CPR = TN / VEC;
        for (int id = tid; id < TK * CPR; id += 256) {
          const int k = id / CPR, cn = (id % CPR) * VEC;
          if (k0 + k >= Kk || n0 + cn >= Nn) continue;
          Chunk16<T> tmp;
#pragma unroll
          for (int e = 0; e < VEC; ++e) tmp.e[e] = Ws[(cn + e) * PW + k];
          *reinterpret_cast<uint4*>(wt + (int64_t)(k0 + k) * Nn + n0 + cn) = tmp.v;
        }
      }
    }
    if (t + 1 < nrun) __syncthreads();  // X tile t+1 is staged; Ws has been read
  }
  if (tk0 == 0 && tid < TN && n0 + tid < Nn) {
    if constexpr (!UPD) {
      if (P.aux2 != nullptr) {
        float* gb = static_cast<float*>(P.aux2) + n0 + tid;
        *gb = rmw ? (*gb + bsum) : bsum;
      }
    } else if (U.bmaster != nullptr) {
      const int n = n0 + tid;
      const float gb = (rmw ? static_cast<const float*>(P.aux2)[n] : 0.f) + bsum;
      const float bnew = sgd_step(U.bmaster[n], gb, U.bV ? U.bV + n : nullptr, U.sgd);
      U.bmaster[n] = bnew;
      U.bcopy[n] = bnew;
    }
  }
}

// ---------------------------------------------------------------------------------
// One launch for every Linear contraction of a tick level: the tile list mixes forward /
// data-gradient tiles (skinny or thin) and weight-gradient tiles (dw), so the short read-
// modify-write tiles fill the machine while the long weight-streaming tiles run.
template <typename T, int BN, bool THIN>
__device__ __forceinline__ void linear_tick_body(const GemmBatch& batch) {
  using E = LT<T>;
  constexpr int SK_BYTES = (64 + BN) * (E::SLAB + E::VEC) * (int)sizeof(T);
  // operand tiles of the weight gradient; in the wide kernel also the new-weight tile of a pipelined run with a fused SGD step
  constexpr int DW_BYTES = (64 * (64 + 128 + 2 * (sizeof(T) == 2 ? 16 : 4)) + (BN == 128 && sizeof(T) == 2 ? 64 * (128 + 2) : 0)) * (int)sizeof(T);
  constexpr int TH_BYTES = THIN ? 4 * 2 * 32 * (2 * 4 * E::VEC + E::VEC) * (int)sizeof(T) : 0;  // thin tile: staging blocks of the four wavefronts
  static_assert(TH_BYTES == 0 || TH_BYTES >= 4 * 16 * 64 * 4, "the thin tile's partial sums must fit");
  constexpr int SM_BYTES = SK_BYTES > DW_BYTES ? (SK_BYTES > TH_BYTES ? SK_BYTES : TH_BYTES) : (DW_BYTES > TH_BYTES ? DW_BYTES : TH_BYTES);
  __shared__ __attribute__((aligned(16))) unsigned char smem[SM_BYTES];
  // Tile order: forward / data-gradient tiles, weight-gradient tiles that also take the SGD
  // step, plain weight-gradient tiles.  The first and the last kind are spread over the XCDs
  // separately (each XCD gets a contiguous share of both, so a problem's activations sit in
  // one L2); the longer update tiles stay in launch order, which deals them round-robin to
  // all XCDs.
  const int head8 = (batch.head_tiles + 7) & ~7, upd8 = (batch.upd_tiles + 7) & ~7;
  const int bid = (int)blockIdx.x;
  int tile;
  if (bid < head8) {
    tile = xcd_remap(bid, batch.head_tiles);
    if (tile >= batch.head_tiles) return;
  } else if (bid < head8 + upd8) {
    tile = bid - head8;
    if (tile >= batch.upd_tiles) return;
    tile += batch.head_tiles;
  } else {
    const int first = batch.head_tiles + batch.upd_tiles;
    const int rest8 = (batch.total_tiles - first + 7) & ~7;
    if (bid >= head8 + upd8 + rest8) {  // staging copy of the micro-batch that starts in this tick
      const StageCopy& sc = batch.sc;
      const int ct = bid - (head8 + upd8 + rest8);
      if (ct == 0) {
        for (int i = threadIdx.x; i < sc.n_slots; i += 256) sc.loss[i] = 0.f;
        for (int i = threadIdx.x; i < sc.rows; i += 256) sc.yo[i] = sc.y[i];
      }
      const int64_t lo = (int64_t)ct * STAGE_COPY_ELEMS;
      const int64_t hi = lo + STAGE_COPY_ELEMS < sc.n ? lo + STAGE_COPY_ELEMS : sc.n;
      T* __restrict__ xo = static_cast<T*>(sc.xo);
      for (int64_t i = lo + threadIdx.x; i < hi; i += 256) xo[i] = E::from_f32(sc.x[i]);
      return;
    }
    tile = first + xcd_remap(bid - head8 - upd8, batch.total_tiles - first);
    if (tile >= batch.total_tiles) return;
  }
  const GemmProb& P = batch.p[find_problem(batch, tile)];
  if (P.epi == EPI_WGRAD) {
    constexpr bool RUN_UPD = BN == 128 && sizeof(T) == 2;  // the new-weight tile has LDS of its own only there
    const bool upd_ok = RUN_UPD && P.upd != 0 && batch.upd[P.upd - 1].V == nullptr;
    if (dw_run_length(P, E::VEC, upd_ok) > 1) {
      if constexpr (RUN_UPD) {
        if (P.upd) {
          dw_run<T, true>(batch, P, tile, smem);
          return;
        }
      }
      dw_run<T, false>(batch, P, tile, smem);
    } else if (dw_tile_rows(P) == 32) dw_tile<T, 32>(batch, P, tile, smem);
    else dw_tile<T, 64>(batch, P, tile, smem);
  } else {
    if constexpr (THIN) {
      if (P.flags & GF_THIN) {
        thin_tile<T>(batch, P, tile, smem);
        return;
      }
    }
    skinny_tile<T, BN>(batch, P, tile, smem);
  }
}

// The bf16 kernel is held to three wavefronts per SIMD (168 registers): left alone the allocator takes 176, one
// workgroup per CU less, which costs the weight-streaming launches 6 % (cfg5 19.5 -> 18.2 ms per step).  The fp32
// kernel needs more registers and keeps two.
template <typename T, int BN, bool THIN>
__global__ __launch_bounds__(256) void linear_tick_kernel(const GemmBatch batch) {
  linear_tick_body<T, BN, THIN>(batch);
}
template <int BN, bool THIN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void linear_tick_kernel_bf16(const GemmBatch batch) {
  linear_tick_body<uint16_t, BN, THIN>(batch);
}
template <typename T, int BN, bool THIN>
static void launch_tick_kernel(const GemmBatch& b, dim3 grid, hipStream_t stream) {
  if constexpr (sizeof(T) == 2) hipLaunchKernelGGL((linear_tick_kernel_bf16<BN, THIN>), grid, dim3(256), 0, stream, b);
  else hipLaunchKernelGGL((linear_tick_kernel<T, BN, THIN>), grid, dim3(256), 0, stream, b);
}

namespace {
template <typename T>
void launch_variant(const GemmBatch& b, bool wide, bool thin, dim3 grid, hipStream_t stream) {
  if (thin) {
    if (wide) launch_tick_kernel<T, 128, true>(b, grid, stream);
    else launch_tick_kernel<T, 64, true>(b, grid, stream);
  } else {
    if (wide) launch_tick_kernel<T, 128, false>(b, grid, stream);
    else launch_tick_kernel<T, 64, false>(b, grid, stream);
  }
}
}  // namespace

hipError_t launch_linear_tick(GemmBatch& b, int dtype, bool wide, bool allow_thin, hipStream_t stream) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > GEMM_MAX_PROBS) return hipErrorInvalidValue;
  const int bn = wide ? 128 : 64;
  const int vec = dtype == DT_BF16 ? 8 : 4;
  // forward / data-gradient problems first, weight gradients after them
  GemmProb* wg = std::stable_partition(b.p, b.p + b.n, [](const GemmProb& p) { return p.epi != EPI_WGRAD; });
  // weight gradients that also take the SGD step have the longest tiles: start them first
  std::stable_partition(wg, b.p + b.n, [](const GemmProb& p) { return p.upd != 0; });
  int total = 0;
  bool any_thin = false;
  const bool split_ok = b.thin_ws != nullptr && b.thin_cnt != nullptr;
  bool skinny_split = false;
  b.head_tiles = 0;
  b.upd_tiles = 0;
  for (int i = 0; i < b.n; ++i) {
    GemmProb& p = b.p[i];
    if (p.M <= 0 || p.N <= 0 || p.K <= 0) return hipErrorInvalidValue;
    p.splits = 1;
    p.flags &= ~GF_THIN;
    int tiles;
    if (p.epi == EPI_WGRAD) {
      const bool grouped = (p.flags & GF_GROUP) != 0;
      if (p.a_mode != OP_PLAIN_R || p.b_mode != OP_PLAIN_R || (p.flags & GF_ATOMIC) || (!grouped && (p.aux0 || p.aux1))) return hipErrorInvalidValue;
      if (grouped && (p.g.pad <= 0 || p.K % p.g.pad != 0 || p.K / p.g.pad > DW_GROUP_MAX)) return hipErrorInvalidValue;
      if (p.upd < 0 || p.upd > b.n_upd || b.n_upd > LIN_UPD_MAX) return hipErrorInvalidValue;
      if (p.upd) {
        const LinUpdate& u = b.upd[p.upd - 1];
        if (p.ldo != p.N) return hipErrorInvalidValue;
        if (!u.master || !u.wf || !u.wt || (u.bmaster && (!u.bcopy || !p.aux2))) return hipErrorInvalidValue;
      }
      p.tiles_n = (p.N + 127) / 128;
      tiles = ((p.M + 63) / 64) * p.tiles_n;
      {
        const int rows = dw_tile_rows(p);
        tiles = ((p.M + rows - 1) / rows) * p.tiles_n;
        const int run = dw_run_length(p, vec, wide && dtype == DT_BF16 && p.upd != 0 && b.upd[p.upd - 1].V == nullptr);
        if (run > 1) tiles = ((p.M + 63) / 64) * ((p.tiles_n + run - 1) / run);  // runs of column tiles, 64 rows high
        if (p.upd) b.upd_tiles += tiles;
      }
    } else {
      if (p.a_mode != OP_PLAIN_K || p.b_mode != OP_PLAIN_K) return hipErrorInvalidValue;
      if ((int64_t)p.M * p.lda >= (1ll << 31) || (int64_t)p.N * p.ldb >= (1ll << 31)) return hipErrorInvalidValue;
      if ((p.flags & GF_A_F32) && (reinterpret_cast<uintptr_t>(p.A) % 16 != 0 || p.lda % 4 != 0) && p.K % vec == 0 &&
          p.lda % vec == 0 && p.ldb % vec == 0)
        return hipErrorInvalidValue;  // vector path on an fp32 operand needs 16-byte aligned rows
      const bool chunked = p.K % vec == 0 && p.lda % vec == 0 && p.ldb % vec == 0 &&
                           reinterpret_cast<uintptr_t>(p.A) % 16 == 0 && reinterpret_cast<uintptr_t>(p.B) % 16 == 0;
      if ((p.flags & GF_CE) && !(allow_thin && p.M <= 32 && chunked && p.N <= 32 && p.epi == EPI_FWD && p.aux2 && p.aux3 &&
                                 p.g.H > 0 && p.M % p.g.H == 0))
        return hipErrorInvalidValue;  // the fused loss head exists in the thin tile only
      if (allow_thin && p.M <= 32 && chunked) {
        p.flags |= GF_THIN;
        any_thin = true;
        p.tiles_n = (p.N + 31) / 32;
        // reductions of 32 slabs and more are cut into ranges of about 16 slabs (at most 4)
        const int nslab = (p.K + 8 * vec - 1) / (8 * vec);
        if (split_ok && nslab >= 32 && !(p.flags & GF_CE)) p.splits = std::min(4, nslab / 16);
        tiles = p.tiles_n * p.splits;
      } else {
        p.tiles_n = (p.N + bn - 1) / bn;
        tiles = ((p.M + 63) / 64) * p.tiles_n;
        // few (at most 64) 64-column tiles with a long reduction (a classifier, or the one layer of a stage that
        // is alone at its level of the tick): ranges of at least 4 slabs of 128, at most 8 per tile, about 256
        // workgroups in all (the partial tiles of a launch share a workspace of 256 slots)
        const int nslab = (p.K + 16 * vec - 1) / (16 * vec);
        const int want = std::min(std::min(8, nslab / 4), std::max(1, 256 / std::max(1, tiles)));
        if (split_ok && !wide && tiles <= 64 && want >= 2) {
          p.splits = want;
          tiles *= p.splits;
          skinny_split = true;
        }
      }
      b.head_tiles += tiles;
    }
    p.tile_begin = total;
    total += tiles;
  }
  b.total_tiles = total;
  // partial tiles are addressed by tile number: one slot size per launch
  b.slot_floats = skinny_split ? 64 * 64 : 32 * 32;
  if ((int64_t)b.head_tiles * b.slot_floats > (int64_t)THIN_WS_SLOTS * 1024 && split_ok) {
    // split tiles address the workspace by their tile number: lay the launch out again without them
    b.thin_ws = nullptr;
    return launch_linear_tick(b, dtype, wide, allow_thin, stream);
  }
  if (b.copy_tiles < 0 || (b.copy_tiles > 0 && (!b.sc.x || !b.sc.y || !b.sc.xo || !b.sc.yo || !b.sc.loss || b.sc.n <= 0 ||
                                                b.copy_tiles != (int)((b.sc.n + STAGE_COPY_ELEMS - 1) / STAGE_COPY_ELEMS))))
    return hipErrorInvalidValue;
  const dim3 grid(((b.head_tiles + 7) / 8) * 8 + ((b.upd_tiles + 7) / 8) * 8 + ((total - b.head_tiles - b.upd_tiles + 7) / 8) * 8 +
                  b.copy_tiles);
  if (dtype == DT_BF16) launch_variant<uint16_t>(b, wide, any_thin, grid, stream);
  else launch_variant<float>(b, wide, any_thin, grid, stream);
  return hipGetLastError();
}

}  // namespace cdp
