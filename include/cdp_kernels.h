/* libcdp kernel-level entry points: the contractions a CDP tick is made of, callable on
 * their own (unit parity tests against the CPU oracle, roofline micro-benchmarks).
 * All pointers are HIP device pointers owned by the caller; work is enqueued on
 * `stream` (hipStream_t, may be NULL) and the call returns without waiting.
 * Return value: 0 or a negative status code of cdp.h. */
#ifndef CDP_KERNELS_H
#define CDP_KERNELS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* C[M][N] (fp32, row-major, ldc = N) = A * B^T with fp32 accumulation, the tile
 * contraction used by every stage forward / backward of a tick (Sec. 3.1: the forward and
 * backward computation of a stage on one micro-batch).
 *   dtype      0 fp32, 1 bf16 (operand element type)
 *   tile_shape 0: 128x128, 1: 64x128, 2: 64x64 workgroup tile of the generic kernel;
 *              3: 64x64, 4: 64x128 tile of the weight-streaming kernel the Linear stages
 *              use; 5: the same kernel as launched by the engine, which gives problems of
 *              at most 32 rows with 16-byte-chunked operands 32x32 tiles whose waves split
 *              the reduction (3..5 need a_kmajor = b_kmajor = 1)
 *   a_kmajor   1: A[m][k] at A[m*lda + k]   0: A[m][k] at A[k*lda + m]
 *   b_kmajor   1: B[n][k] at B[n*ldb + k]   0: B[n][k] at B[k*ldb + n] */
int cdp_k_gemm(int dtype, int tile_shape, int a_kmajor, int b_kmajor, const void* A, const void* B,
               float* C, int M, int N, int K, int lda, int ldb, void* stream);

/* One NHWC convolution contraction as implicit GEMM (no affine, no activation).
 *   which 0: forward        y[B][Ho][Wo][Cout] (elem type) = conv(x, w),  w[Cout][k][k][Cin]
 *         1: data gradient  dx[B][H][W][Cin]   (elem type) from dy and wt[Cin][k][k][Cout]
 *         2: weight gradient dw[Cout][k][k][Cin] (fp32, overwritten) from dy and x
 *         3, 4: as 0, 1 on the direct-to-LDS kernel's 256 x 256 tile whatever the size (the engine and which =
 *               0, 1 choose by launch size); 5, 6: the same kernel's 128 x 128 tile; CDP_EINVAL unless bf16 with
 *               channel counts that are multiples of 64
 * in0/in1: (x, w) | (dy, wt) | (dy, x).  `out` must not alias the inputs.
 * workspace (device, may be NULL): scratch for the split weight-gradient kernel; with at
 * least 4 * Cout*k*k*Cin * (B*Ho*Wo / 512 + 4) bytes the two-phase path is used when the
 * shape allows, otherwise the generic single-pass kernel runs. */
int cdp_k_conv(int dtype, int which, const void* in0, const void* in1, void* out, int B, int H, int W,
               int Cin, int Cout, int ksize, int stride, int pad, void* workspace,
               size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the weight gradient of cdp_k_conv (which = 2, two-phase path) with the
 * partial sums of its reduction ranges in a device array that is part of the library image
 * (CDP_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of a caller's workspace.
 * dw[Cout][k][k][Cin] (fp32, overwritten) from dy[B][Ho][Wo][Cout] and x[B][H][W][Cin] (element type by
 * dtype).  Calls no hipMalloc / hipFree and no allocating library routine.
 * Errors: CDP_EINVAL for shapes the two-phase kernels do not take (channel counts that are not whole
 * 16-byte chunks, more than 32 taps); CDP_ENOMEM when the partial sums (4 * Cout*k*k*Cin * ranges bytes)
 * exceed the array - cdp_last_error(NULL) then says how many bytes were needed; CDP_EHIP.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams,
 * different threads) race.  Nothing in the array has to be cleared between calls. */
#define CDP_STATIC_SCRATCH_BYTES (16u << 20)
int cdp_k_conv_wgrad_static(int dtype, const void* dy, const void* x, float* dw, int B, int H, int W, int Cin,
                            int Cout, int ksize, int stride, int pad, void* stream);

/* The kernels of ViT-shaped stages (the homogeneous stages of Sec. 5 "Memory") on their own.
 * Element type of x / dy / out / qkv / P / dout by `dtype`; gamma, beta and their gradients fp32.
 *
 * LayerNorm over the last axis of x[rows][C] (C <= 1024, eps 1e-5, biased variance):
 *   backward 0: out = y = (x - mean) * rstd * gamma + beta       (dy, add, dgamma, dbeta, workspace unused)
 *   backward 1: out = dx (+ add, may be NULL); dgamma[C] += sum dy * xhat; dbeta[C] += sum dy;
 *               workspace: 8 * rows + 8 * C * ceil(rows / 32) + 256 bytes (CDP_EINVAL if smaller). */
int cdp_k_layernorm(int dtype, int backward, const void* x, const void* dy, const void* add, const float* gamma,
                    const float* beta, void* out, float* dgamma, float* dbeta, void* workspace,
                    size_t workspace_bytes, int rows, int C, void* stream);

/* Exact GELU on n elements: backward 0: out = x * Phi(x); backward 1: out = dy * (Phi(x) + x * phi(x)). */
int cdp_k_gelu(int dtype, int backward, const void* x, const void* dy, void* out, int64_t n, void* stream);

/* Multi-head self-attention core on qkv[B][T][3*D] (q | k | v per token, head h in columns
 * h*D/heads..; T <= 1024):
 *   backward 0: P[B][heads][T][T] = softmax(q k^T / sqrt(D/heads)) (written), out[B][T][D] = P v
 *   backward 1: out = dqkv[B][T][3*D] from P (read) and dout[B][T][D]
 * workspace: 4 * B*heads*T*T bytes (forward), (4 + element size) * B*heads*T*T + 256 bytes (backward). */
int cdp_k_attention(int dtype, int backward, const void* qkv, void* P, const void* dout, void* out, void* workspace,
                    size_t workspace_bytes, int B, int T, int D, int heads, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CDP_KERNELS_H */
