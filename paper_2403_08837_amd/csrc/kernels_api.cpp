// C ABI of the kernel-level entry points (include/cdp_kernels.h).
#include <hip/hip_runtime.h>

#include <cstring>

#include "../../include/cdp.h"
#include "../../include/cdp_kernels.h"
#include "kernels.h"

using namespace cdp;

extern "C" {

int cdp_k_gemm(int dtype, int tile_shape, int a_kmajor, int b_kmajor, const void* A, const void* B, float* C, int M, int N,
               int K, int lda, int ldb, void* stream) {
  if (!A || !B || !C || M <= 0 || N <= 0 || K <= 0 || tile_shape < 0 || tile_shape >= TILE_COUNT + 3) return CDP_EINVAL;
  if (tile_shape >= TILE_COUNT && !(a_kmajor && b_kmajor)) return CDP_EINVAL;
  if (dtype != DT_F32 && dtype != DT_BF16) return CDP_EINVAL;
  GemmBatch b;
  memset(&b, 0, sizeof(b));
  b.n = 1;
  GemmProb& p = b.p[0];
  p.A = A; p.B = B; p.out = C;
  p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldo = N;
  p.a_mode = a_kmajor ? OP_PLAIN_K : OP_PLAIN_R;
  p.b_mode = b_kmajor ? OP_PLAIN_K : OP_PLAIN_R;
  p.epi = EPI_FWD;
  p.flags = GF_OUT_F32;
  p.splits = 1;
  if (tile_shape >= TILE_COUNT)
    return launch_linear_tick(b, dtype, tile_shape == TILE_COUNT + 1, tile_shape == TILE_COUNT + 2, static_cast<hipStream_t>(stream)) == hipSuccess ? CDP_OK : CDP_EHIP;
  return launch_gemm_batch(b, dtype, tile_shape, static_cast<hipStream_t>(stream)) == hipSuccess ? CDP_OK : CDP_EHIP;
}

int cdp_k_conv(int dtype, int which, const void* in0, const void* in1, void* out, int B, int H, int W, int Cin, int Cout,
               int ks, int stride, int pad, void* workspace, size_t workspace_bytes, void* stream) {
  if (!in0 || !in1 || !out || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || ks <= 0 || stride <= 0 || pad < 0)
    return CDP_EINVAL;
  if (dtype != DT_F32 && dtype != DT_BF16) return CDP_EINVAL;
  if (H + 2 * pad < ks || W + 2 * pad < ks) return CDP_EINVAL;
  const int Ho = (H + 2 * pad - ks) / stride + 1, Wo = (W + 2 * pad - ks) / stride + 1;
  GemmBatch b;
  memset(&b, 0, sizeof(b));
  b.n = 1;
  GemmProb& p = b.p[0];
  p.splits = 1;
  p.A = in0; p.B = in1; p.out = out;
  ConvGeom& g = p.g;
  g.KH = ks; g.KW = ks; g.stride = stride; g.pad = pad;
  const bool force256 = which >= 3 && which <= 6;  // the direct-to-LDS tile regardless of the launch heuristic
  const int forced_tile = which >= 5 ? 128 : 256;
  if (force256) which -= which >= 5 ? 5 : 3;
  if (which == 0) {
    p.M = B * Ho * Wo; p.N = Cout; p.K = ks * ks * Cin;
    p.a_mode = OP_CONV_FWD; p.b_mode = OP_PLAIN_K; p.ldb = p.K; p.ldo = Cout;
    g.H = H; g.W = W; g.C = Cin; g.OH = Ho; g.OW = Wo;
    p.epi = EPI_FWD;
  } else if (which == 1) {
    p.M = B * H * W; p.N = Cin; p.K = ks * ks * Cout;
    p.a_mode = OP_CONV_DGRAD; p.b_mode = OP_PLAIN_K; p.ldb = p.K; p.ldo = Cin;
    g.H = Ho; g.W = Wo; g.C = Cout; g.OH = H; g.OW = W;
    p.epi = EPI_DGRAD;
  } else if (which == 2) {
    p.M = Cout; p.N = ks * ks * Cin; p.K = B * Ho * Wo;
    p.a_mode = OP_PLAIN_R; p.lda = Cout; p.b_mode = OP_CONV_WGRAD; p.ldo = p.N;
    g.H = H; g.W = W; g.C = Cin; g.OH = Ho; g.OW = Wo;
    p.epi = EPI_WGRAD;
  } else {
    return CDP_EINVAL;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  // same kernel choice as the engine: the fast implicit-GEMM paths where the shape allows
  if (which == 2) {
    const int splits = conv_wgrad_splits(p, dtype, 3);
    if (conv_fast_eligible(p, dtype) && workspace && workspace_bytes >= (size_t)splits * p.M * p.N * 4) {
      // two phases as in the engine: partial sums per reduction range, then the fold
      WReduceBatch rb;
      memset(&rb, 0, sizeof(rb));
      rb.n = 1;
      rb.p[0].part = static_cast<const float*>(workspace);
      rb.p[0].G = static_cast<float*>(out);
      rb.p[0].Cout = p.M; rb.p[0].Ncol = p.N; rb.p[0].splits = splits;
      p.out = workspace;
      p.splits = splits;
      if (launch_fill_f32(static_cast<float*>(out), (int64_t)p.M * p.N, 0.f, st) != hipSuccess) return CDP_EHIP;
      if (launch_conv_wgrad(b, dtype, p.M >= 128, st) != hipSuccess) return CDP_EHIP;
      return launch_wgrad_reduce(rb, dtype, st) == hipSuccess ? CDP_OK : CDP_EHIP;
    }
  } else if (force256) {
    if (!conv_gemm256_eligible(p, dtype)) return CDP_EINVAL;
    return launch_conv_gemm256(b, dtype, st, forced_tile) == hipSuccess ? CDP_OK : CDP_EHIP;
  } else if (conv_fast_eligible(p, dtype)) {
    if (conv_gemm256_wanted(&p, 1, dtype)) return launch_conv_gemm256(b, dtype, st) == hipSuccess ? CDP_OK : CDP_EHIP;
    int bm, bn;
    conv_gemm_tile(&p, 1, &bm, &bn);
    return launch_conv_gemm(b, dtype, bm, bn, st) == hipSuccess ? CDP_OK : CDP_EHIP;
  }
  const int shape = p.M <= 64 ? (p.N >= 128 ? TILE_64x128 : TILE_64x64) : (p.N <= 64 ? TILE_64x64 : TILE_128x128);
  return launch_gemm_batch(b, dtype, shape, st) == hipSuccess ? CDP_OK : CDP_EHIP;
}

int cdp_k_layernorm(int dtype, int backward, const void* x, const void* dy, const void* add, const float* gamma,
                    const float* beta, void* out, float* dgamma, float* dbeta, void* workspace, size_t workspace_bytes,
                    int rows, int C, void* stream) {
  if (!x || !gamma || !out || rows <= 0 || C <= 0 || C > 1024 || (dtype != DT_F32 && dtype != DT_BF16)) return CDP_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!backward) {
    if (!beta) return CDP_EINVAL;
    return launch_layernorm_fwd(x, gamma, beta, out, rows, C, dtype, st) == hipSuccess ? CDP_OK : CDP_EHIP;
  }
  if (!dy || !dgamma || !dbeta || !workspace || (int64_t)workspace_bytes < layernorm_bwd_workspace_bytes(rows, C)) return CDP_EINVAL;
  return launch_layernorm_bwd(x, dy, add, gamma, out, dgamma, dbeta, static_cast<float*>(workspace), rows, C, dtype, st) == hipSuccess
             ? CDP_OK : CDP_EHIP;
}

int cdp_k_gelu(int dtype, int backward, const void* x, const void* dy, void* out, int64_t n, void* stream) {
  if (!x || !out || n <= 0 || (backward && !dy) || (dtype != DT_F32 && dtype != DT_BF16)) return CDP_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const hipError_t e = backward ? launch_gelu_bwd(x, dy, out, n, dtype, st) : launch_gelu_fwd(x, out, n, dtype, st);
  return e == hipSuccess ? CDP_OK : CDP_EHIP;
}

int cdp_k_attention(int dtype, int backward, const void* qkv, void* P, const void* dout, void* out, void* workspace,
                    size_t workspace_bytes, int B, int T, int D, int heads, void* stream) {
  if (!qkv || !P || !out || !workspace || B <= 0 || T <= 0 || T > 1024 || D <= 0 || heads <= 0 || D % heads ||
      (dtype != DT_F32 && dtype != DT_BF16))
    return CDP_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t tt = (int64_t)B * heads * T * T;
  if (!backward) {
    if ((int64_t)workspace_bytes < 4 * tt) return CDP_EINVAL;
    return launch_attention_fwd(qkv, P, out, static_cast<float*>(workspace), B, T, D, heads, dtype, st) == hipSuccess ? CDP_OK : CDP_EHIP;
  }
  const int64_t dp_bytes = (4 * tt + 255) / 256 * 256;
  if (!dout || (int64_t)workspace_bytes < dp_bytes + tt * (dtype == DT_BF16 ? 2 : 4)) return CDP_EINVAL;
  return launch_attention_bwd(qkv, P, dout, out, static_cast<float*>(workspace), static_cast<char*>(workspace) + dp_bytes, B, T, D,
                              heads, dtype, st) == hipSuccess ? CDP_OK : CDP_EHIP;
}

}  // extern "C"
