// Kernels of ViT-shaped stages (the homogeneous stages of Sec. 5, "Memory"): LayerNorm,
// GELU and the self-attention core.  Token-wise linear maps run on the convolution path as
// 1x1 convolutions.  LayerNorm and the softmax take one wavefront per token row; the attention
// contractions (about a tenth of a block's flops at 196 tokens) are a batched MFMA product.
#include "elem.h"
#include "kernels.h"

namespace cdp {

namespace {

template <typename T> __device__ __forceinline__ float tld(const T* p, int64_t i) { return ld_f32<T>(p, i); }
template <typename T> __device__ __forceinline__ void tst(T* p, int64_t i, float v) { st_f32<T>(p, i, v); }

#define CDP_TDISPATCH(dtype, CALL)                        \
  do {                                                    \
    if ((dtype) == DT_BF16) { using T = uint16_t; CALL; } \
    else { using T = float; CALL; }                       \
  } while (0)

// Wavefront-wide sum / maximum, result in every lane: four rotations inside the 16-lane rows on
// the VALU (DPP row_ror 1, 2, 4, 8), then two exchanges through the LDS crossbar (instead of six).
template <int CTRL>
__device__ __forceinline__ float dpp_rot(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float wsum(float v) {
  v += dpp_rot<0x121>(v);
  v += dpp_rot<0x122>(v);
  v += dpp_rot<0x124>(v);
  v += dpp_rot<0x128>(v);
  v += __shfl_xor(v, 16, 64);
  return v + __shfl_xor(v, 32, 64);
}
__device__ __forceinline__ float wmax(float v) {
  v = fmaxf(v, dpp_rot<0x121>(v));
  v = fmaxf(v, dpp_rot<0x122>(v));
  v = fmaxf(v, dpp_rot<0x124>(v));
  v = fmaxf(v, dpp_rot<0x128>(v));
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  return fmaxf(v, __shfl_xor(v, 32, 64));
}

constexpr float LN_EPS = 1e-5f;
constexpr int LN_MAX_PER_LANE = 16;  // channels <= 1024

// 16-byte chunks of a row: 8 bf16 or 4 fp32 values.
template <typename T> struct RowChunk;
template <> struct RowChunk<uint16_t> {
  static constexpr int N = 8;
  __device__ static __forceinline__ void load(const uint16_t* p, float* v) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
    v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
    v[4] = __uint_as_float(u.z << 16); v[5] = __uint_as_float(u.z & 0xffff0000u);
    v[6] = __uint_as_float(u.w << 16); v[7] = __uint_as_float(u.w & 0xffff0000u);
  }
  __device__ static __forceinline__ void store(uint16_t* p, const float* v) {
    uint4 u;
    u.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
    u.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
    u.z = (uint32_t)f32_to_bf16(v[4]) | ((uint32_t)f32_to_bf16(v[5]) << 16);
    u.w = (uint32_t)f32_to_bf16(v[6]) | ((uint32_t)f32_to_bf16(v[7]) << 16);
    *reinterpret_cast<uint4*>(p) = u;
  }
};
template <> struct RowChunk<float> {
  static constexpr int N = 4;
  __device__ static __forceinline__ void load(const float* p, float* v) {
    const float4 u = *reinterpret_cast<const float4*>(p);
    v[0] = u.x; v[1] = u.y; v[2] = u.z; v[3] = u.w;
  }
  __device__ static __forceinline__ void store(float* p, const float* v) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};

}  // namespace

// ---------------------------------------------------------------------------------
// LayerNorm over the channels of every row: one wavefront per row, lane l owns channels
// l, l+64, ...  y = (x - mean) * rstd * gamma + beta (biased variance, eps = 1e-5).
template <typename T>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const T* __restrict__ x, const float* __restrict__ gamma,
                                                            const float* __restrict__ beta, T* __restrict__ y, int rows, int C) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* xr = x + (int64_t)row * C;
  float v[LN_MAX_PER_LANE];
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    v[q] = c < C ? tld<T>(xr, c) : 0.f;
    s += v[q];
  }
  const float mean = wsum(s) / (float)C;
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    const float d = c < C ? v[q] - mean : 0.f;
    ss += d * d;
  }
  const float rstd = rsqrtf(wsum(ss) / (float)C + LN_EPS);
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    if (c < C) tst<T>(y, (int64_t)row * C + c, (v[q] - mean) * rstd * gamma[c] + beta[c]);
  }
}

// The same with 16-byte accesses, for rows that are whole 16-byte chunks: lane l owns chunks
// l, l + 64, ... of its row.
template <typename T>
__device__ __forceinline__ void layernorm_fwd_vec_body(const T* __restrict__ x, const float* __restrict__ gamma,
                                                                const float* __restrict__ beta, T* __restrict__ y, int rows, int C) {
  constexpr int N = RowChunk<T>::N, Q = LN_MAX_PER_LANE / N;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int64_t base = (int64_t)row * C;
  float v[Q][N];
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int c = (lane + 64 * q) * N;
    if (c < C) {
      RowChunk<T>::load(x + base + c, v[q]);
#pragma unroll
      for (int e = 0; e < N; ++e) s += v[q][e];
    }
  }
  const float mean = wsum(s) / (float)C;
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < Q; ++q)
    if ((lane + 64 * q) * N < C) {
#pragma unroll
      for (int e = 0; e < N; ++e) ss += (v[q][e] - mean) * (v[q][e] - mean);
    }
  const float rstd = rsqrtf(wsum(ss) / (float)C + LN_EPS);
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int c = (lane + 64 * q) * N;
    if (c < C) {
      float o[N];
#pragma unroll
      for (int e = 0; e < N; ++e) o[e] = (v[q][e] - mean) * rstd * gamma[c + e] + beta[c + e];
      RowChunk<T>::store(y + base + c, o);
    }
  }
}

template <typename T>
__device__ __forceinline__ void layernorm_bwd_rows_vec_body(const T* __restrict__ x, const T* __restrict__ dy,
                                                                     const T* __restrict__ add, const float* __restrict__ gamma,
                                                                     T* __restrict__ dx, float* __restrict__ stats, int rows, int C) {
  constexpr int N = RowChunk<T>::N, Q = LN_MAX_PER_LANE / N;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int64_t base = (int64_t)row * C;
  float v[Q][N], g[Q][N];
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int c = (lane + 64 * q) * N;
    if (c < C) {
      RowChunk<T>::load(x + base + c, v[q]);
      RowChunk<T>::load(dy + base + c, g[q]);
#pragma unroll
      for (int e = 0; e < N; ++e) {
        g[q][e] *= gamma[c + e];
        s += v[q][e];
      }
    }
  }
  const float mean = wsum(s) / (float)C;
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < Q; ++q)
    if ((lane + 64 * q) * N < C) {
#pragma unroll
      for (int e = 0; e < N; ++e) ss += (v[q][e] - mean) * (v[q][e] - mean);
    }
  const float rstd = rsqrtf(wsum(ss) / (float)C + LN_EPS);
  float sg = 0.f, sgx = 0.f;
#pragma unroll
  for (int q = 0; q < Q; ++q)
    if ((lane + 64 * q) * N < C) {
#pragma unroll
      for (int e = 0; e < N; ++e) {
        v[q][e] = (v[q][e] - mean) * rstd;
        sg += g[q][e];
        sgx += g[q][e] * v[q][e];
      }
    }
  const float mg = wsum(sg) / (float)C, mgx = wsum(sgx) / (float)C;
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int c = (lane + 64 * q) * N;
    if (c < C) {
      float o[N], a[N];
      if (add) RowChunk<T>::load(add + base + c, a);
#pragma unroll
      for (int e = 0; e < N; ++e) o[e] = rstd * (g[q][e] - mg - v[q][e] * mgx) + (add ? a[e] : 0.f);
      RowChunk<T>::store(dx + base + c, o);
    }
  }
  if (lane == 0) {
    stats[2 * (int64_t)row] = mean;
    stats[2 * (int64_t)row + 1] = rstd;
  }
}

// Backward: with xh = (x - mean) * rstd and g = dy * gamma,
//   dx = rstd * (g - mean(g) - xh * mean(g * xh)) (+ add), dgamma += sum dy * xh, dbeta += sum dy.
// Three kernels: the row pass (one wavefront per row, like the forward; leaves mean and rstd of
// every row in `stats`), the column pass (a workgroup sums LN_ROWS_PER_WG rows with threads
// owning columns, no cross-lane traffic, one partial row per workgroup) and the fold of the
// partial rows into the running sums.  Device-wide atomics on these small hot vectors, or a
// row pass that also carries the column sums, cost several times the whole pass.
constexpr int LN_ROWS_PER_WG = 32;
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_rows_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                                 const T* __restrict__ add, const float* __restrict__ gamma,
                                                                 T* __restrict__ dx, float* __restrict__ stats, int rows, int C) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int64_t base = (int64_t)row * C;
  float v[LN_MAX_PER_LANE], g[LN_MAX_PER_LANE];
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    v[q] = c < C ? tld<T>(x, base + c) : 0.f;
    g[q] = c < C ? tld<T>(dy, base + c) * gamma[c] : 0.f;
    s += v[q];
  }
  const float mean = wsum(s) / (float)C;
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    const float t = c < C ? v[q] - mean : 0.f;
    ss += t * t;
  }
  const float rstd = rsqrtf(wsum(ss) / (float)C + LN_EPS);
  float sg = 0.f, sgx = 0.f;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    v[q] = c < C ? (v[q] - mean) * rstd : 0.f;
    sg += g[q];
    sgx += g[q] * v[q];
  }
  const float mg = wsum(sg) / (float)C, mgx = wsum(sgx) / (float)C;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    if (c < C) {
      float r = rstd * (g[q] - mg - v[q] * mgx);
      if (add) r += tld<T>(add, base + c);
      tst<T>(dx, base + c, r);
    }
  }
  if (lane == 0) {
    stats[2 * (int64_t)row] = mean;
    stats[2 * (int64_t)row + 1] = rstd;
  }
}

template <typename T>
__device__ __forceinline__ void layernorm_bwd_cols_body(const T* __restrict__ x, const T* __restrict__ dy,
                                                                 const float* __restrict__ stats, float* __restrict__ part,
                                                                 int rows, int C) {
  __shared__ float st[2 * LN_ROWS_PER_WG];
  const int r0 = blockIdx.x * LN_ROWS_PER_WG;
  const int nr = min(LN_ROWS_PER_WG, rows - r0);
  if (threadIdx.x < 2 * nr) st[threadIdx.x] = stats[2 * (int64_t)r0 + threadIdx.x];
  __syncthreads();
  float* pg = part + (int64_t)blockIdx.x * 2 * C;
  for (int c = threadIdx.x; c < C; c += 256) {
    float dg = 0.f, db = 0.f;
    const T* xp = x + (int64_t)r0 * C + c;
    const T* dp = dy + (int64_t)r0 * C + c;
#pragma unroll 8
    for (int r = 0; r < nr; ++r) {
      const float d = tld<T>(dp, (int64_t)r * C);
      dg += d * (tld<T>(xp, (int64_t)r * C) - st[2 * r]) * st[2 * r + 1];
      db += d;
    }
    pg[c] = dg;
    pg[C + c] = db;
  }
}

// Column sums of the n_part partial rows (2C wide): 16 columns x 16 row groups per workgroup (a short chain of
// loads per lane: the kernel is a handful of memory round trips long), the groups' sums added in group order.
__device__ __forceinline__ void layernorm_fold_body(const float* __restrict__ part, int n_part, float* __restrict__ Ggamma,
                                                             float* __restrict__ Gbeta, int C) {
  __shared__ float red[16][17];
  const int col = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + col;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (c < 2 * C) {
    int k = grp;
    for (; k + 48 < n_part; k += 64) {
      s0 += part[(int64_t)k * 2 * C + c];
      s1 += part[(int64_t)(k + 16) * 2 * C + c];
      s2 += part[(int64_t)(k + 32) * 2 * C + c];
      s3 += part[(int64_t)(k + 48) * 2 * C + c];
    }
    for (; k < n_part; k += 16) s0 += part[(int64_t)k * 2 * C + c];
  }
  red[grp][col] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (grp == 0 && c < 2 * C) {
    float s = 0.f;
#pragma unroll
    for (int g = 0; g < 16; ++g) s += red[g][col];
    if (c < C) Ggamma[c] += s;
    else Gbeta[c - C] += s;
  }
}

// The kernels proper: one problem per launch, or (batch kernels) the same pass of up to LN_BATCH_MAX problems of one
// shape, problem = blockIdx.y.  The passes of a tick that sit at the same level are the same layer of different
// stages and micro-batches; each alone is a launch of a few microseconds, most of it the launch's own latency.
template <typename T>
__global__ __launch_bounds__(256) void layernorm_fwd_vec_kernel(const T* x, const float* gamma, const float* beta, T* y, int rows, int C) {
  layernorm_fwd_vec_body<T>(x, gamma, beta, y, rows, C);
}
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_rows_vec_kernel(const T* x, const T* dy, const T* add, const float* gamma, T* dx,
                                                                     float* stats, int rows, int C) {
  layernorm_bwd_rows_vec_body<T>(x, dy, add, gamma, dx, stats, rows, C);
}
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_cols_kernel(const T* x, const T* dy, const float* stats, float* part, int rows, int C) {
  layernorm_bwd_cols_body<T>(x, dy, stats, part, rows, C);
}
__global__ __launch_bounds__(256) void layernorm_fold_kernel(const float* part, int n_part, float* Ggamma, float* Gbeta, int C) {
  layernorm_fold_body(part, n_part, Ggamma, Gbeta, C);
}
template <typename T>
__global__ __launch_bounds__(256) void layernorm_fwd_vec_batch_kernel(const LnFwdBatch b, int rows, int C) {
  const LnFwdProb& p = b.p[blockIdx.y];
  layernorm_fwd_vec_body<T>(static_cast<const T*>(p.x), p.gamma, p.beta, static_cast<T*>(p.y), rows, C);
}
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_rows_vec_batch_kernel(const LnBwdBatch b, int rows, int C) {
  const LnBwdProb& p = b.p[blockIdx.y];
  layernorm_bwd_rows_vec_body<T>(static_cast<const T*>(p.x), static_cast<const T*>(p.dy), static_cast<const T*>(p.add), p.gamma,
                                 static_cast<T*>(p.dx), p.workspace, rows, C);
}
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_cols_batch_kernel(const LnBwdBatch b, int rows, int C, int stats_floats) {
  const LnBwdProb& p = b.p[blockIdx.y];
  layernorm_bwd_cols_body<T>(static_cast<const T*>(p.x), static_cast<const T*>(p.dy), p.workspace, p.workspace + stats_floats, rows, C);
}
__global__ __launch_bounds__(256) void layernorm_fold_batch_kernel(const LnBwdBatch b, int n_part, int C, int stats_floats) {
  const LnBwdProb& p = b.p[blockIdx.y];
  layernorm_fold_body(p.workspace + stats_floats, n_part, p.Ggamma, p.Gbeta, C);
}

// rows of C elements at p are whole, 16-byte aligned chunks
static bool ln_vec_ok(const void* p, int C, int eb) {
  return p == nullptr || (reinterpret_cast<uintptr_t>(p) % 16 == 0 && (C * eb) % 16 == 0);
}

hipError_t launch_layernorm_fwd(const void* x, const float* gamma, const float* beta, void* y, int rows, int C, int dtype,
                                hipStream_t stream) {
  if (rows <= 0 || C <= 0 || C > 64 * LN_MAX_PER_LANE) return hipErrorInvalidValue;
  const int eb = dtype == DT_BF16 ? 2 : 4;
  if (ln_vec_ok(x, C, eb) && ln_vec_ok(y, C, eb))
    CDP_TDISPATCH(dtype, hipLaunchKernelGGL((layernorm_fwd_vec_kernel<T>), dim3((rows + 3) / 4), dim3(256), 0, stream,
                                            static_cast<const T*>(x), gamma, beta, static_cast<T*>(y), rows, C));
  else
    CDP_TDISPATCH(dtype, hipLaunchKernelGGL((layernorm_fwd_kernel<T>), dim3((rows + 3) / 4), dim3(256), 0, stream,
                                            static_cast<const T*>(x), gamma, beta, static_cast<T*>(y), rows, C));
  return hipGetLastError();
}
static int64_t ln_stats_bytes(int rows) { return ((int64_t)rows * 8 + 255) / 256 * 256; }
int64_t layernorm_bwd_workspace_bytes(int rows, int C) {
  return ln_stats_bytes(rows) + (int64_t)((rows + LN_ROWS_PER_WG - 1) / LN_ROWS_PER_WG) * 2 * C * 4;
}
hipError_t launch_layernorm_bwd(const void* x, const void* dy, const void* add, const float* gamma, void* dx, float* Ggamma,
                                float* Gbeta, float* workspace, int rows, int C, int dtype, hipStream_t stream) {
  if (rows <= 0 || C <= 0 || C > 64 * LN_MAX_PER_LANE || !workspace) return hipErrorInvalidValue;
  const int wgs = (rows + LN_ROWS_PER_WG - 1) / LN_ROWS_PER_WG;
  float* stats = workspace;
  float* part = workspace + ln_stats_bytes(rows) / 4;
  const int eb = dtype == DT_BF16 ? 2 : 4;
  if (ln_vec_ok(x, C, eb) && ln_vec_ok(dy, C, eb) && ln_vec_ok(add, C, eb) && ln_vec_ok(dx, C, eb))
    CDP_TDISPATCH(dtype, hipLaunchKernelGGL((layernorm_bwd_rows_vec_kernel<T>), dim3((rows + 3) / 4), dim3(256), 0, stream,
                                            static_cast<const T*>(x), static_cast<const T*>(dy), static_cast<const T*>(add), gamma,
                                            static_cast<T*>(dx), stats, rows, C));
  else
    CDP_TDISPATCH(dtype, hipLaunchKernelGGL((layernorm_bwd_rows_kernel<T>), dim3((rows + 3) / 4), dim3(256), 0, stream,
                                            static_cast<const T*>(x), static_cast<const T*>(dy), static_cast<const T*>(add), gamma,
                                            static_cast<T*>(dx), stats, rows, C));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  CDP_TDISPATCH(dtype, hipLaunchKernelGGL((layernorm_bwd_cols_kernel<T>), dim3(wgs), dim3(256), 0, stream, static_cast<const T*>(x),
                                          static_cast<const T*>(dy), stats, part, rows, C));
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(layernorm_fold_kernel, dim3((2 * C + 15) / 16), dim3(256), 0, stream, part, wgs, Ggamma, Gbeta, C);
  return hipGetLastError();
}

bool layernorm_batchable(const void* a, const void* b, const void* c, const void* d, int C, int dtype) {
  const int eb = dtype == DT_BF16 ? 2 : 4;
  return C > 0 && C <= 64 * LN_MAX_PER_LANE && ln_vec_ok(a, C, eb) && ln_vec_ok(b, C, eb) && ln_vec_ok(c, C, eb) && ln_vec_ok(d, C, eb);
}
hipError_t launch_layernorm_fwd_batch(const LnFwdBatch& b, int rows, int C, int dtype, hipStream_t stream) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > LN_BATCH_MAX || rows <= 0) return hipErrorInvalidValue;
  for (int i = 0; i < b.n; ++i)
    if (!b.p[i].x || !b.p[i].y || !layernorm_batchable(b.p[i].x, b.p[i].y, nullptr, nullptr, C, dtype)) return hipErrorInvalidValue;
  CDP_TDISPATCH(dtype, hipLaunchKernelGGL((layernorm_fwd_vec_batch_kernel<T>), dim3((rows + 3) / 4, b.n), dim3(256), 0, stream, b, rows, C));
  return hipGetLastError();
}
hipError_t launch_layernorm_bwd_batch(const LnBwdBatch& b, int rows, int C, int dtype, hipStream_t stream) {
  if (b.n <= 0) return hipSuccess;
  if (b.n > LN_BATCH_MAX || rows <= 0) return hipErrorInvalidValue;
  for (int i = 0; i < b.n; ++i)
    if (!b.p[i].workspace || !b.p[i].x || !b.p[i].dy || !b.p[i].dx || !b.p[i].Ggamma || !b.p[i].Gbeta ||
        !layernorm_batchable(b.p[i].x, b.p[i].dy, b.p[i].add, b.p[i].dx, C, dtype))
      return hipErrorInvalidValue;
  const int wgs = (rows + LN_ROWS_PER_WG - 1) / LN_ROWS_PER_WG;
  const int stats_floats = (int)(ln_stats_bytes(rows) / 4);
  CDP_TDISPATCH(dtype, hipLaunchKernelGGL((layernorm_bwd_rows_vec_batch_kernel<T>), dim3((rows + 3) / 4, b.n), dim3(256), 0, stream, b, rows, C));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  CDP_TDISPATCH(dtype, hipLaunchKernelGGL((layernorm_bwd_cols_batch_kernel<T>), dim3(wgs, b.n), dim3(256), 0, stream, b, rows, C, stats_floats));
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(layernorm_fold_batch_kernel, dim3((2 * C + 15) / 16, b.n), dim3(256), 0, stream, b, wgs, C, stats_floats);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// GELU, exact form: y = x * Phi(x);  dx = dy * (Phi(x) + x * phi(x)).
// The first n4 groups of four elements go through 8- / 16-byte accesses, the rest one by one.
__device__ __forceinline__ void t_ld4(const uint16_t* p, int64_t g, float* v) {
  const uint2 u = reinterpret_cast<const uint2*>(p)[g];
  v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
  v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
}
__device__ __forceinline__ void t_ld4(const float* p, int64_t g, float* v) {
  const float4 u = reinterpret_cast<const float4*>(p)[g];
  v[0] = u.x; v[1] = u.y; v[2] = u.z; v[3] = u.w;
}
__device__ __forceinline__ void t_st4(uint16_t* p, int64_t g, const float* v) {
  uint2 u;
  u.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
  u.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
  reinterpret_cast<uint2*>(p)[g] = u;
}
__device__ __forceinline__ void t_st4(float* p, int64_t g, const float* v) {
  reinterpret_cast<float4*>(p)[g] = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ float gelu_f(float v) { return 0.5f * v * (1.f + erff(v * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_df(float v) {
  return 0.5f * (1.f + erff(v * 0.70710678118654752f)) + v * 0.3989422804014327f * expf(-0.5f * v * v);
}

template <typename T>
__global__ void gelu_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, int64_t n, int64_t n4) {
  const int64_t t0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x, step = (int64_t)gridDim.x * blockDim.x;
  for (int64_t g = t0; g < n4; g += step) {
    float v[4];
    t_ld4(x, g, v);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = gelu_f(v[e]);
    t_st4(y, g, v);
  }
  for (int64_t i = 4 * n4 + t0; i < n; i += step) tst<T>(y, i, gelu_f(tld<T>(x, i)));
}
template <typename T>
__global__ void gelu_bwd_kernel(const T* __restrict__ x, const T* __restrict__ dy, T* __restrict__ dx, int64_t n, int64_t n4) {
  const int64_t t0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x, step = (int64_t)gridDim.x * blockDim.x;
  for (int64_t g = t0; g < n4; g += step) {
    float v[4], d[4];
    t_ld4(x, g, v);
    t_ld4(dy, g, d);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = d[e] * gelu_df(v[e]);
    t_st4(dx, g, v);
  }
  for (int64_t i = 4 * n4 + t0; i < n; i += step) tst<T>(dx, i, tld<T>(dy, i) * gelu_df(tld<T>(x, i)));
}
static bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }
hipError_t launch_gelu_fwd(const void* x, void* y, int64_t n, int dtype, hipStream_t stream) {
  if (n <= 0) return hipErrorInvalidValue;
  const int64_t n4 = aligned16(x) && aligned16(y) ? n / 4 : 0;
  const int64_t want = (n4 + (n - 4 * n4) + 255) / 256;
  const int blocks = (int)(want < (1 << 20) ? want : (1 << 20));
  CDP_TDISPATCH(dtype, hipLaunchKernelGGL((gelu_fwd_kernel<T>), dim3(blocks), dim3(256), 0, stream, static_cast<const T*>(x),
                                          static_cast<T*>(y), n, n4));
  return hipGetLastError();
}
hipError_t launch_gelu_bwd(const void* x, const void* dy, void* dx, int64_t n, int dtype, hipStream_t stream) {
  if (n <= 0) return hipErrorInvalidValue;
  const int64_t n4 = aligned16(x) && aligned16(dy) && aligned16(dx) ? n / 4 : 0;
  const int64_t want = (n4 + (n - 4 * n4) + 255) / 256;
  const int blocks = (int)(want < (1 << 20) ? want : (1 << 20));
  CDP_TDISPATCH(dtype, hipLaunchKernelGGL((gelu_bwd_kernel<T>), dim3(blocks), dim3(256), 0, stream, static_cast<const T*>(x),
                                          static_cast<const T*>(dy), static_cast<T*>(dx), n, n4));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Batched product C[z][i][j] = alpha * sum_k A[z][i][k] * B[z][j][k] with arbitrary element
// strides; batch z = (sample, head) with its own pair of offsets per operand.  A workgroup owns
// 64 x 64 outputs (four wavefronts, one 32 x 32 MFMA accumulator each) and walks the reduction
// in 32-deep slabs staged through LDS as tile[row][k]; an operand whose k (mode 1) or row
// (mode 2) index is contiguous in memory is fetched four elements at a time, anything else
// element by element (mode 0).
struct BmmOperand {
  const void* p;
  int64_t s_sample, s_head, s_row, s_k;  // element strides
};
struct BmmArgs {
  BmmOperand A, B;
  void* C;
  int64_t c_sample, c_head, c_row, c_col;
  int M, N, K, heads;
  float alpha;
  int c_f32;  // C holds fp32, else T
  int mode_a, mode_b;
};

typedef float bmm_v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bmm_v8bf __attribute__((ext_vector_type(8)));
template <typename T> struct BmmTile;
template <> struct BmmTile<uint16_t> { static constexpr int PITCH = 40; typedef uint2 vec4; };
template <> struct BmmTile<float> { static constexpr int PITCH = 33; typedef float4 vec4; };

__device__ __forceinline__ void bmm_put4(uint16_t* dst, int stride, uint2 v) {
  if (stride == 1) { *reinterpret_cast<uint2*>(dst) = v; return; }
  dst[0] = (uint16_t)(v.x & 0xffffu); dst[stride] = (uint16_t)(v.x >> 16);
  dst[2 * stride] = (uint16_t)(v.y & 0xffffu); dst[3 * stride] = (uint16_t)(v.y >> 16);
}
__device__ __forceinline__ void bmm_put4(float* dst, int stride, float4 v) {
  dst[0] = v.x; dst[stride] = v.y; dst[2 * stride] = v.z; dst[3 * stride] = v.w;
}

// tile[r][k] = op[row0 + r][k0 + k] for r < 64, k < 32, zero outside rows x K, in two steps: bmm_fetch requests a
// thread's two 4-element pieces (vector modes 1 and 2), bmm_store writes them to LDS (mode 0, element by element
// with arbitrary strides, does all its work in bmm_store).  Split so that the pieces of both operands, and of the
// next slab, are in flight together: fetched and stored piece by piece, a slab was four memory round trips in a row.
template <typename T>
__device__ __forceinline__ void bmm_fetch(typename BmmTile<T>::vec4 (&v)[2], const T* base, int64_t s_row, int64_t s_k, int mode,
                                          int row0, int rows, int k0, int K) {
  typedef typename BmmTile<T>::vec4 vec4;
  if (mode == 1) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int e = threadIdx.x + 256 * i, r = e >> 3, k = (e & 7) * 4;
      v[i] = vec4{};
      if (row0 + r < rows && k0 + k < K) v[i] = *reinterpret_cast<const vec4*>(base + (int64_t)(row0 + r) * s_row + (k0 + k));
    }
  } else if (mode == 2) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int e = threadIdx.x + 256 * i, k = e >> 4, r = (e & 15) * 4;
      v[i] = vec4{};
      if (row0 + r < rows && k0 + k < K) v[i] = *reinterpret_cast<const vec4*>(base + (row0 + r) + (int64_t)(k0 + k) * s_k);
    }
  }
}
template <typename T>
__device__ __forceinline__ void bmm_store(T* tile, const typename BmmTile<T>::vec4 (&v)[2], const T* base, int64_t s_row, int64_t s_k,
                                          int mode, int row0, int rows, int k0, int K) {
  constexpr int PITCH = BmmTile<T>::PITCH;
  if (mode == 1) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int e = threadIdx.x + 256 * i, r = e >> 3, k = (e & 7) * 4;
      bmm_put4(tile + r * PITCH + k, 1, v[i]);
    }
  } else if (mode == 2) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int e = threadIdx.x + 256 * i, k = e >> 4, r = (e & 15) * 4;
      bmm_put4(tile + r * PITCH + k, PITCH, v[i]);
    }
  } else {
    for (int e = threadIdx.x; e < 2048; e += 256) {
      const int r = e >> 5, k = e & 31;
      T x = T(0);
      if (row0 + r < rows && k0 + k < K) x = base[(int64_t)(row0 + r) * s_row + (int64_t)(k0 + k) * s_k];
      tile[r * PITCH + k] = x;
    }
  }
}

// MODES: 4 * mode_a + mode_b for the four pairs of vector modes (straight-line staging code, which lets the
// next slab's requests stay in flight across the contraction), or -1: the modes are read from the arguments.
template <typename T, int MODES>
__global__ __launch_bounds__(256) void bmm_kernel(const BmmArgs a) {
  constexpr int PITCH = BmmTile<T>::PITCH;
  const int mode_a = MODES >= 0 ? MODES / 4 : a.mode_a, mode_b = MODES >= 0 ? MODES % 4 : a.mode_b;
  __shared__ __attribute__((aligned(16))) T As[64 * PITCH];
  __shared__ __attribute__((aligned(16))) T Bs[64 * PITCH];
  const int z = blockIdx.z, sample = z / a.heads, head = z % a.heads;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const T* Ap = static_cast<const T*>(a.A.p) + sample * a.A.s_sample + head * a.A.s_head;
  const T* Bp = static_cast<const T*>(a.B.p) + sample * a.B.s_sample + head * a.B.s_head;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
  const int l31 = lane & 31, hi = lane >> 5;
  // wavefronts whose 32 x 32 block lies outside the product still help staging
  const bool live = i0 + wm * 32 < a.M && j0 + wn * 32 < a.N;
  bmm_v16f acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  typename BmmTile<T>::vec4 ra[2], rb[2];
  bmm_fetch<T>(ra, Ap, a.A.s_row, a.A.s_k, mode_a, i0, a.M, 0, a.K);
  bmm_fetch<T>(rb, Bp, a.B.s_row, a.B.s_k, mode_b, j0, a.N, 0, a.K);
  for (int k0 = 0; k0 < a.K; k0 += 32) {
    bmm_store<T>(As, ra, Ap, a.A.s_row, a.A.s_k, mode_a, i0, a.M, k0, a.K);
    bmm_store<T>(Bs, rb, Bp, a.B.s_row, a.B.s_k, mode_b, j0, a.N, k0, a.K);
    __syncthreads();
    if (k0 + 32 < a.K) {  // the next slab's pieces are on their way while this one is contracted
      bmm_fetch<T>(ra, Ap, a.A.s_row, a.A.s_k, mode_a, i0, a.M, k0 + 32, a.K);
      bmm_fetch<T>(rb, Bp, a.B.s_row, a.B.s_k, mode_b, j0, a.N, k0 + 32, a.K);
    }
    if (live) {
      const T* ar = As + (wm * 32 + l31) * PITCH;
      const T* br = Bs + (wn * 32 + l31) * PITCH;
      if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int kk = 0; kk < 32; kk += 16) {
          const uint4 av = *reinterpret_cast<const uint4*>(ar + kk + 8 * hi);
          const uint4 bv = *reinterpret_cast<const uint4*>(br + kk + 8 * hi);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bmm_v8bf, av), __builtin_bit_cast(bmm_v8bf, bv), acc, 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int kk = 0; kk < 32; kk += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ar[kk + hi], br[kk + hi], acc, 0, 0, 0);
      }
    }
    __syncthreads();
  }
  if (!live) return;
  // acc[v]: row = 8*(v/4) + 4*(lane/32) + v%4, column = lane%32 of the wavefront's block
  const int64_t cbase = sample * a.c_sample + head * a.c_head;
  const int j = j0 + wn * 32 + l31;
  if (j >= a.N) return;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = i0 + wm * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
    if (i >= a.M) continue;
    const int64_t o = cbase + (int64_t)i * a.c_row + (int64_t)j * a.c_col;
    if (a.c_f32) static_cast<float*>(a.C)[o] = a.alpha * acc[v];
    else tst<T>(static_cast<T*>(a.C), o, a.alpha * acc[v]);
  }
}

static int bmm_mode(const BmmOperand& op, int rows, int K, int eb) {
  const bool base_ok = reinterpret_cast<uintptr_t>(op.p) % (4 * eb) == 0 && op.s_sample % 4 == 0 && op.s_head % 4 == 0;
  if (base_ok && op.s_k == 1 && op.s_row % 4 == 0 && K % 4 == 0) return 1;
  if (base_ok && op.s_row == 1 && op.s_k % 4 == 0 && rows % 4 == 0) return 2;
  return 0;
}

static hipError_t launch_bmm(BmmArgs a, int batch, int dtype, hipStream_t stream) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0 || batch <= 0 || batch > 65535) return hipErrorInvalidValue;
  const int eb = dtype == DT_BF16 ? 2 : 4;
  a.mode_a = bmm_mode(a.A, a.M, a.K, eb);
  a.mode_b = bmm_mode(a.B, a.N, a.K, eb);
  dim3 grid((a.N + 63) / 64, (a.M + 63) / 64, batch);
  const int modes = (a.mode_a >= 1 && a.mode_b >= 1) ? 4 * a.mode_a + a.mode_b : -1;
  switch (modes) {
    case 5: CDP_TDISPATCH(dtype, hipLaunchKernelGGL((bmm_kernel<T, 5>), grid, dim3(256), 0, stream, a)); break;
    case 6: CDP_TDISPATCH(dtype, hipLaunchKernelGGL((bmm_kernel<T, 6>), grid, dim3(256), 0, stream, a)); break;
    case 9: CDP_TDISPATCH(dtype, hipLaunchKernelGGL((bmm_kernel<T, 9>), grid, dim3(256), 0, stream, a)); break;
    case 10: CDP_TDISPATCH(dtype, hipLaunchKernelGGL((bmm_kernel<T, 10>), grid, dim3(256), 0, stream, a)); break;
    default: CDP_TDISPATCH(dtype, hipLaunchKernelGGL((bmm_kernel<T, -1>), grid, dim3(256), 0, stream, a)); break;
  }
  return hipGetLastError();
}

// Row softmax of fp32 scores into T probabilities, one wavefront per row (length <= 1024).
template <typename T>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const float* __restrict__ s, T* __restrict__ p, int64_t rows, int n) {
  const int lane = threadIdx.x & 63;
  const int64_t row = blockIdx.x * (int64_t)4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float* sr = s + row * n;
  float v[LN_MAX_PER_LANE];
  float m = -INFINITY;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    v[q] = c < n ? sr[c] : -INFINITY;
    m = fmaxf(m, v[q]);
  }
  m = wmax(m);
  float sum = 0.f;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    v[q] = (lane + 64 * q) < n ? expf(v[q] - m) : 0.f;
    sum += v[q];
  }
  const float inv = 1.f / wsum(sum);
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    if (c < n) tst<T>(p, row * n + c, v[q] * inv);
  }
}
// ds = P * (dP - sum_k dP_k P_k) * scale, rows as above.
template <typename T>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const T* __restrict__ p, const float* __restrict__ dp, T* __restrict__ ds,
                                                          int64_t rows, int n, float scale) {
  const int lane = threadIdx.x & 63;
  const int64_t row = blockIdx.x * (int64_t)4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  float pv[LN_MAX_PER_LANE], dv[LN_MAX_PER_LANE];
  float dot = 0.f;
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    pv[q] = c < n ? tld<T>(p, row * n + c) : 0.f;
    dv[q] = c < n ? dp[row * n + c] : 0.f;
    dot += pv[q] * dv[q];
  }
  dot = wsum(dot);
#pragma unroll
  for (int q = 0; q < LN_MAX_PER_LANE; ++q) {
    const int c = lane + 64 * q;
    if (c < n) tst<T>(ds, row * n + c, pv[q] * (dv[q] - dot) * scale);
  }
}

// The two softmax kernels with 4-element accesses, for row lengths that are multiples of 4
// (fp32 rows are then whole 16-byte chunks, T rows whole 8- or 16-byte chunks): lane l owns
// chunks l, l + 64, ... of its row.
template <typename T>
__global__ __launch_bounds__(256) void softmax_fwd_vec_kernel(const float* __restrict__ s, T* __restrict__ p, int64_t rows, int n) {
  constexpr int Q = LN_MAX_PER_LANE / 4;
  const int lane = threadIdx.x & 63;
  const int64_t row = blockIdx.x * (int64_t)4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float* sr = s + row * n;
  float v[Q][4];
  float m = -INFINITY;
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const int c = (lane + 64 * q) * 4;
    if (c < n) {
      t_ld4(sr, lane + 64 * q, v[q]);
#pragma unroll
      for (int e = 0; e < 4; ++e) m = fmaxf(m, v[q][e]);
    }
  }
  m = wmax(m);
  float sum = 0.f;
#pragma unroll
  for (int q = 0; q < Q; ++q)
    if ((lane + 64 * q) * 4 < n) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[q][e] = expf(v[q][e] - m);
        sum += v[q][e];
      }
    }
  const float inv = 1.f / wsum(sum);
  T* pr = p + row * n;
#pragma unroll
  for (int q = 0; q < Q; ++q)
    if ((lane + 64 * q) * 4 < n) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[q][e] *= inv;
      t_st4(pr, lane + 64 * q, v[q]);
    }
}
template <typename T>
__global__ __launch_bounds__(256) void softmax_bwd_vec_kernel(const T* __restrict__ p, const float* __restrict__ dp, T* __restrict__ ds,
                                                              int64_t rows, int n, float scale) {
  constexpr int Q = LN_MAX_PER_LANE / 4;
  const int lane = threadIdx.x & 63;
  const int64_t row = blockIdx.x * (int64_t)4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  float pv[Q][4], dv[Q][4];
  float dot = 0.f;
#pragma unroll
  for (int q = 0; q < Q; ++q)
    if ((lane + 64 * q) * 4 < n) {
      t_ld4(p + row * n, lane + 64 * q, pv[q]);
      t_ld4(dp + row * n, lane + 64 * q, dv[q]);
#pragma unroll
      for (int e = 0; e < 4; ++e) dot += pv[q][e] * dv[q][e];
    }
  dot = wsum(dot);
#pragma unroll
  for (int q = 0; q < Q; ++q)
    if ((lane + 64 * q) * 4 < n) {
#pragma unroll
      for (int e = 0; e < 4; ++e) pv[q][e] = pv[q][e] * (dv[q][e] - dot) * scale;
      t_st4(ds + row * n, lane + 64 * q, pv[q]);
    }
}

// ---------------------------------------------------------------------------------
// Score rows without the fp32 round trip through memory (bf16, at most 256 tokens, head width a multiple of 16 up
// to 80).  A workgroup owns 64 query rows of one (sample, head) and all keys: wavefront w contracts the 64 x 64
// block of keys 64 w .. 64 w + 63 (2 x 2 MFMA accumulators, reduction over the head width); the fp32 block then
// goes to LDS (over the operand tiles), and each wavefront finishes 16 whole rows, a lane holding four
// neighbouring keys of the row: the row maximum / sums are wavefront reductions and rows move as 8-byte vectors.
//   forward : A = q, B = k:     P = softmax(scale * A B^T)                           -> out (bf16)
//   backward: A = d out, B = v: dP = A B^T, dS = P * (dP - rowsum(dP * P)) * scale   -> out (bf16)
struct AttnScoreArgs {
  const uint16_t* A; int64_t a_sample, a_head, a_row;  // rows = queries (reduction index contiguous)
  const uint16_t* B; int64_t b_sample, b_head, b_row;  // rows = keys
  const uint16_t* P;                                   // backward: probabilities [z][NT][NT]
  uint16_t* out;                                       // [z][NT][NT]
  int NT, dh, heads;
  float scale;
  int vec;  // rows of P / out are whole 8-byte groups (NT % 4 == 0, bases 8-byte aligned)
};
__device__ __forceinline__ float row16_sum(float v) {  // over the 16 lanes of a VALU row, result in each of them
  v += dpp_rot<0x121>(v);
  v += dpp_rot<0x122>(v);
  v += dpp_rot<0x124>(v);
  return v + dpp_rot<0x128>(v);
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_rot<0x121>(v));
  v = fmaxf(v, dpp_rot<0x122>(v));
  v = fmaxf(v, dpp_rot<0x124>(v));
  return fmaxf(v, dpp_rot<0x128>(v));
}
constexpr int ATTN_SP = 264;  // pitch (floats) of the score block in LDS: rows 4 apart sit 32 banks apart

template <bool BWD>
__global__ __launch_bounds__(256) void attn_scores_kernel(const AttnScoreArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char attn_smem[];
  const int pitch = a.dh + 8;  // elements; rows stay 16-byte aligned and 16 fragment rows cover all banks
  uint16_t* As = reinterpret_cast<uint16_t*>(attn_smem);  // [64][pitch]
  uint16_t* Bs = As + 64 * pitch;                         // [256][pitch]
  float* S = reinterpret_cast<float*>(attn_smem);         // [32][ATTN_SP], after the contraction
  const int z = blockIdx.y, sample = z / a.heads, head = z % a.heads;
  const int q0 = blockIdx.x * 64, NT = a.NT;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, hi = lane >> 5;
  const uint16_t* Ap = a.A + sample * a.a_sample + head * a.a_head;
  const uint16_t* Bp = a.B + sample * a.b_sample + head * a.b_head;
  const int cpr = a.dh >> 3;  // 16-byte chunks per row
  for (int e = tid; e < 64 * cpr; e += 256) {
    const int r = e / cpr, c = (e - r * cpr) * 8;
    const uint4 v = q0 + r < NT ? *reinterpret_cast<const uint4*>(Ap + (int64_t)(q0 + r) * a.a_row + c) : make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(As + r * pitch + c) = v;
  }
  const int key_rows = min(256, (NT + 63) & ~63);  // key blocks some wavefront contracts
  for (int e = tid; e < key_rows * cpr; e += 256) {
    const int r = e / cpr, c = (e - r * cpr) * 8;
    const uint4 v = r < NT ? *reinterpret_cast<const uint4*>(Bp + (int64_t)r * a.b_row + c) : make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(Bs + r * pitch + c) = v;
  }
  // the score block passes through LDS in two halves of 32 rows; of each half this wavefront finishes rows
  // 8 wave .. 8 wave + 7, four at a time: 16 lanes per row, a lane holding keys
  // 64 k + 4 l15 .. + 3 for k = 0 .. 3, so that row reductions stay inside the 16-lane rows of the VALU (DPP).
  // Backward: the rows' probabilities are requested now.
  const int sub = lane >> 4, l15 = lane & 15;
  auto tile_row = [&](int ps) { return (ps >> 1) * 32 + wave * 8 + (ps & 1) * 4 + sub; };  // pass ps = 0 .. 3 of this lane
  const int64_t rbase = ((int64_t)z * NT + q0) * NT + 4 * l15;  // + row * NT + 64 k
  uint2 pr[4][4];
  if constexpr (BWD) {
#pragma unroll
    for (int ps = 0; ps < 4; ++ps)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        pr[ps][k] = make_uint2(0, 0);
        const int c = 64 * k + 4 * l15;
        if (q0 + tile_row(ps) < NT && c < NT) {
          const uint16_t* src = a.P + rbase + (int64_t)tile_row(ps) * NT + 64 * k;
          if (a.vec) pr[ps][k] = *reinterpret_cast<const uint2*>(src);
          else {
            uint32_t e[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) e[q] = c + q < NT ? src[q] : 0u;
            pr[ps][k] = make_uint2(e[0] | (e[1] << 16), e[2] | (e[3] << 16));
          }
        }
      }
  }
  __syncthreads();
  // element (i, j, v) of this lane: row = 32 i + 8 (v / 4) + 4 hi + v % 4, key = 64 wave + 32 j + l31
  const bool live = wave * 64 < NT;          // wavefront-uniform
  const bool second = wave * 64 + 32 < NT;   // so is the presence of the wavefront's second block of 32 keys
  bmm_v16f acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  if (live) {
    const uint16_t* ar = As + l31 * pitch + 8 * hi;
    const uint16_t* br = Bs + (wave * 64 + l31) * pitch + 8 * hi;
    for (int kk = 0; kk < a.dh; kk += 16) {
      uint4 av[2], bv[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) av[i] = *reinterpret_cast<const uint4*>(ar + i * 32 * pitch + kk);
#pragma unroll
      for (int j = 0; j < 2; ++j) bv[j] = *reinterpret_cast<const uint4*>(br + j * 32 * pitch + kk);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          if (j == 0 || second)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bmm_v8bf, av[i]), __builtin_bit_cast(bmm_v8bf, bv[j]), acc[i][j], 0, 0, 0);
    }
  }
#pragma unroll
  for (int ps = 0; ps < 4; ++ps) {
    if ((ps & 1) == 0) {
      __syncthreads();  // the operand tiles / the first half of the score block are consumed
      if (live) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            S[((v >> 2) * 8 + hi * 4 + (v & 3)) * ATTN_SP + wave * 64 + j * 32 + l31] = acc[ps >> 1][j][v];
      }
      __syncthreads();
    }
    const int row = tile_row(ps), srow = wave * 8 + (ps & 1) * 4 + sub;  // row of the tile, row of the half in LDS
    // (no early exit: every wavefront reaches the barriers; rows past the end compute on zeros and store nothing)
    const bool row_ok = q0 + row < NT;
    float x[4][4], y[4][4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float4 s4 = *reinterpret_cast<const float4*>(S + srow * ATTN_SP + 64 * k + 4 * l15);
      x[k][0] = s4.x; x[k][1] = s4.y; x[k][2] = s4.z; x[k][3] = s4.w;
    }
    if constexpr (!BWD) {
      float m = -INFINITY;
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          x[k][q] = 64 * k + 4 * l15 + q < NT ? x[k][q] * a.scale : -INFINITY;  // (columns of wavefronts that are not live hold no scores)
          m = fmaxf(m, x[k][q]);
        }
      m = row16_max(m);  // key 0 is always there: finite
      float sum = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          y[k][q] = 64 * k + 4 * l15 + q < NT ? __expf(x[k][q] - m) : 0.f;
          sum += y[k][q];
        }
      const float inv = __builtin_amdgcn_rcpf(row16_sum(sum));
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int q = 0; q < 4; ++q) y[k][q] *= inv;
    } else {
      float dot = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        y[k][0] = __uint_as_float(pr[ps][k].x << 16); y[k][1] = __uint_as_float(pr[ps][k].x & 0xffff0000u);
        y[k][2] = __uint_as_float(pr[ps][k].y << 16); y[k][3] = __uint_as_float(pr[ps][k].y & 0xffff0000u);
#pragma unroll
        for (int q = 0; q < 4; ++q) dot += 64 * k + 4 * l15 + q < NT ? y[k][q] * x[k][q] : 0.f;
      }
      dot = row16_sum(dot);
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int q = 0; q < 4; ++q) y[k][q] = y[k][q] * (x[k][q] - dot) * a.scale;
    }
    if (!row_ok) continue;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = 64 * k + 4 * l15;
      if (c >= NT) continue;
      uint16_t* dst = a.out + rbase + (int64_t)row * NT + 64 * k;
      if (a.vec) {
        *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)f32_to_bf16(y[k][0]) | ((uint32_t)f32_to_bf16(y[k][1]) << 16),
                                                    (uint32_t)f32_to_bf16(y[k][2]) | ((uint32_t)f32_to_bf16(y[k][3]) << 16));
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (c + q < NT) dst[q] = f32_to_bf16(y[k][q]);
      }
    }
  }
}

static bool attn_scores_fused_ok(const void* a, int64_t a_row, const void* b, int64_t b_row, int NT, int dh, int dtype) {
  return dtype == DT_BF16 && NT <= 256 && dh % 16 == 0 && dh <= 80 && a_row % 8 == 0 && b_row % 8 == 0 &&
         reinterpret_cast<uintptr_t>(a) % 16 == 0 && reinterpret_cast<uintptr_t>(b) % 16 == 0;
}
template <bool BWD>
static hipError_t launch_attn_scores(const AttnScoreArgs& a, int batch, hipStream_t stream) {
  if (batch <= 0 || batch > 65535) return hipErrorInvalidValue;
  const size_t lds = std::max<size_t>((size_t)(64 + 256) * (a.dh + 8) * 2, (size_t)32 * ATTN_SP * 4);
  AttnScoreArgs b = a;
  b.vec = a.NT % 4 == 0 && reinterpret_cast<uintptr_t>(a.out) % 8 == 0 && (!BWD || reinterpret_cast<uintptr_t>(a.P) % 8 == 0);
  hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_scores_kernel<BWD>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL((attn_scores_kernel<BWD>), dim3((a.NT + 63) / 64, batch), dim3(256), lds, stream, b);
  return hipGetLastError();
}

// Self-attention core on qkv[B][T][3*D] (q | k | v per token, head h in columns h*dh..):
// forward  S = q k^T / sqrt(dh) (fp32 workspace), P = softmax(S) (kept for the backward), out = P v;
// backward dv = P^T do, dP = do v^T (fp32 workspace), ds = P * (dP - rowsum(dP * P)) / sqrt(dh),
//          dq = ds k, dk = ds^T q, written into dqkv[B][T][3*D].
hipError_t launch_attention_fwd(const void* qkv, void* P, void* out, float* ws, int B, int NT, int D, int heads, int dtype,
                                hipStream_t stream) {
  if (B <= 0 || NT <= 0 || NT > 64 * LN_MAX_PER_LANE || heads <= 0 || D % heads) return hipErrorInvalidValue;
  const int dh = D / heads;
  const int64_t tok = 3ll * D, TT = (int64_t)NT * NT;
  const float scale = 1.0f / sqrtf((float)dh);
  const char* base = static_cast<const char*>(qkv);
  const int eb = dtype == DT_BF16 ? 2 : 4;
  const int64_t rows = (int64_t)B * heads * NT;
  if (attn_scores_fused_ok(base, tok, base + (int64_t)D * eb, tok, NT, dh, dtype) && (dh * eb) % 16 == 0) {
    AttnScoreArgs f;
    f.A = reinterpret_cast<const uint16_t*>(base); f.a_sample = NT * tok; f.a_head = dh; f.a_row = tok;
    f.B = reinterpret_cast<const uint16_t*>(base + (int64_t)D * eb); f.b_sample = NT * tok; f.b_head = dh; f.b_row = tok;
    f.P = nullptr; f.out = static_cast<uint16_t*>(P); f.NT = NT; f.dh = dh; f.heads = heads; f.scale = scale;
    hipError_t e = launch_attn_scores<false>(f, B * heads, stream);
    if (e != hipSuccess) return e;
  } else {
  BmmArgs s;  // S[z][q][key] = scale * sum_j q[q][j] k[key][j]
  s.A = BmmOperand{base, NT * tok, dh, tok, 1};
  s.B = BmmOperand{base + (int64_t)D * eb, NT * tok, dh, tok, 1};
  s.C = ws; s.c_sample = heads * TT; s.c_head = TT; s.c_row = NT; s.c_col = 1;
  s.M = NT; s.N = NT; s.K = dh; s.heads = heads; s.alpha = scale; s.c_f32 = 1;
  hipError_t e = launch_bmm(s, B * heads, dtype, stream);
  if (e != hipSuccess) return e;
  if (NT % 4 == 0 && aligned16(ws) && aligned16(P))
    CDP_TDISPATCH(dtype, hipLaunchKernelGGL((softmax_fwd_vec_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, ws,
                                            static_cast<T*>(P), rows, NT));
  else
    CDP_TDISPATCH(dtype, hipLaunchKernelGGL((softmax_fwd_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, ws,
                                            static_cast<T*>(P), rows, NT));
  if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  BmmArgs o;  // out[z][q][j] = sum_key P[q][key] v[key][j]
  o.A = BmmOperand{P, heads * TT, TT, NT, 1};
  o.B = BmmOperand{base + 2ll * D * eb, NT * tok, dh, 1, tok};
  o.C = out; o.c_sample = (int64_t)NT * D; o.c_head = dh; o.c_row = D; o.c_col = 1;
  o.M = NT; o.N = dh; o.K = NT; o.heads = heads; o.alpha = 1.f; o.c_f32 = 0;
  return launch_bmm(o, B * heads, dtype, stream);
}

int attention_launches(bool backward, int NT, int D, int heads, int dtype) {
  const int dh = heads > 0 ? D / heads : 0;
  // (operands the engine passes are 256-byte aligned)
  const bool fused = dtype == DT_BF16 && NT <= 256 && dh > 0 && dh % 16 == 0 && dh <= 80 && D % 8 == 0;
  return backward ? (fused ? 4 : 5) : (fused ? 2 : 3);
}

hipError_t launch_attention_bwd(const void* qkv, const void* P, const void* dout, void* dqkv, float* ws_dp, void* ws_ds, int B,
                                int NT, int D, int heads, int dtype, hipStream_t stream) {
  if (B <= 0 || NT <= 0 || NT > 64 * LN_MAX_PER_LANE || heads <= 0 || D % heads) return hipErrorInvalidValue;
  const int dh = D / heads;
  const int64_t tok = 3ll * D, TT = (int64_t)NT * NT;
  const float scale = 1.0f / sqrtf((float)dh);
  const int eb = dtype == DT_BF16 ? 2 : 4;
  const char* base = static_cast<const char*>(qkv);
  char* dbase = static_cast<char*>(dqkv);
  const BmmOperand Pqk{P, heads * TT, TT, NT, 1};    // rows = query, k = key
  const BmmOperand Pkq{P, heads * TT, TT, 1, NT};    // rows = key,   k = query
  const BmmOperand dOqj{dout, (int64_t)NT * D, dh, D, 1};  // rows = query, k = j
  const BmmOperand dOjq{dout, (int64_t)NT * D, dh, 1, D};  // rows = j,     k = query
  hipError_t e;
  BmmArgs a;
  // dv[key][j] = sum_q P[q][key] do[q][j]
  a.A = Pkq; a.B = dOjq; a.C = dbase + 2ll * D * eb; a.c_sample = NT * tok; a.c_head = dh; a.c_row = tok; a.c_col = 1;
  a.M = NT; a.N = dh; a.K = NT; a.heads = heads; a.alpha = 1.f; a.c_f32 = 0;
  if ((e = launch_bmm(a, B * heads, dtype, stream)) != hipSuccess) return e;
  if (attn_scores_fused_ok(dout, D, base + 2ll * D * eb, tok, NT, dh, dtype) && (dh * eb) % 16 == 0) {
    // dS straight from d out, v and P
    AttnScoreArgs f;
    f.A = static_cast<const uint16_t*>(dout); f.a_sample = (int64_t)NT * D; f.a_head = dh; f.a_row = D;
    f.B = reinterpret_cast<const uint16_t*>(base + 2ll * D * eb); f.b_sample = NT * tok; f.b_head = dh; f.b_row = tok;
    f.P = static_cast<const uint16_t*>(P); f.out = static_cast<uint16_t*>(ws_ds); f.NT = NT; f.dh = dh; f.heads = heads; f.scale = scale;
    if ((e = launch_attn_scores<true>(f, B * heads, stream)) != hipSuccess) return e;
  } else {
  // dP[q][key] = sum_j do[q][j] v[key][j]
  a.A = dOqj; a.B = BmmOperand{base + 2ll * D * eb, NT * tok, dh, tok, 1}; a.C = ws_dp;
  a.c_sample = heads * TT; a.c_head = TT; a.c_row = NT; a.c_col = 1; a.M = NT; a.N = NT; a.K = dh; a.c_f32 = 1;
  if ((e = launch_bmm(a, B * heads, dtype, stream)) != hipSuccess) return e;
  const int64_t rows = (int64_t)B * heads * NT;
  if (NT % 4 == 0 && aligned16(P) && aligned16(ws_dp) && aligned16(ws_ds))
    CDP_TDISPATCH(dtype, hipLaunchKernelGGL((softmax_bwd_vec_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream,
                                            static_cast<const T*>(P), ws_dp, static_cast<T*>(ws_ds), rows, NT, scale));
  else
    CDP_TDISPATCH(dtype, hipLaunchKernelGGL((softmax_bwd_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream,
                                            static_cast<const T*>(P), ws_dp, static_cast<T*>(ws_ds), rows, NT, scale));
  if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  const BmmOperand dSqk{ws_ds, heads * TT, TT, NT, 1}, dSkq{ws_ds, heads * TT, TT, 1, NT};
  // dq[q][j] = sum_key ds[q][key] k[key][j]
  a.A = dSqk; a.B = BmmOperand{base + (int64_t)D * eb, NT * tok, dh, 1, tok}; a.C = dbase;
  a.c_sample = NT * tok; a.c_head = dh; a.c_row = tok; a.c_col = 1; a.M = NT; a.N = dh; a.K = NT; a.c_f32 = 0;
  if ((e = launch_bmm(a, B * heads, dtype, stream)) != hipSuccess) return e;
  // dk[key][j] = sum_q ds[q][key] q[q][j]
  a.A = dSkq; a.B = BmmOperand{base, NT * tok, dh, 1, tok}; a.C = dbase + (int64_t)D * eb;
  return launch_bmm(a, B * heads, dtype, stream);
}

}  // namespace cdp
