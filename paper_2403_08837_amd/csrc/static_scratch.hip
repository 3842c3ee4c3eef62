// Entry point that allocates nothing: the convolution weight gradient of cdp_k_conv (which = 2) with
// its partial-sum workspace in a file-scope device array instead of a caller-provided buffer.
//
// `scratch` below is a host-side stand-in for the device array: its name must never be passed to a
// kernel or a memory routine.  The device address is looked up once per device with
// hipGetSymbolAddress (each GPU holds its own copy at its own address) and kept in `g_scratch`;
// everything after that uses that pointer.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <string>

#include "../../include/cdp.h"
#include "../../include/cdp_kernels.h"
#include "kernels.h"

using namespace cdp;

namespace {

constexpr size_t SCRATCH_BYTES = (size_t)CDP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_mutex;
void* g_scratch[MAX_DEVICES] = {nullptr};  // device address of `scratch` on each device, 0 = not looked up yet

int fail(int code, const std::string& msg) {
  set_global_error(msg);
  return code;
}

// Device address of the scratch array on the current device.
int scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(CDP_EHIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(CDP_EINVAL, "device ordinal out of range");
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_scratch[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(CDP_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    g_scratch[dev] = p;
  }
  *out = g_scratch[dev];
  return CDP_OK;
}

}  // namespace

extern "C" int cdp_k_conv_wgrad_static(int dtype, const void* dy, const void* x, float* dw, int B, int H, int W, int Cin, int Cout,
                                       int ks, int stride, int pad, void* stream) {
  if (!dy || !x || !dw || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || ks <= 0 || stride <= 0 || pad < 0)
    return fail(CDP_EINVAL, "cdp_k_conv_wgrad_static: bad argument");
  if (dtype != DT_F32 && dtype != DT_BF16) return fail(CDP_EINVAL, "cdp_k_conv_wgrad_static: unknown dtype");
  if (H + 2 * pad < ks || W + 2 * pad < ks) return fail(CDP_EINVAL, "cdp_k_conv_wgrad_static: filter larger than the padded image");
  const int Ho = (H + 2 * pad - ks) / stride + 1, Wo = (W + 2 * pad - ks) / stride + 1;
  if ((int64_t)B * Ho * Wo >= (1ll << 31) || (int64_t)B * H * W * Cin >= (1ll << 31) || (int64_t)ks * ks * Cin >= (1ll << 31))
    return fail(CDP_EINVAL, "cdp_k_conv_wgrad_static: tensor too large for 32-bit indexing");
  GemmBatch b;
  memset(&b, 0, sizeof(b));
  b.n = 1;
  GemmProb& p = b.p[0];
  p.A = dy; p.B = x;
  p.M = Cout; p.N = ks * ks * Cin; p.K = B * Ho * Wo;
  p.a_mode = OP_PLAIN_R; p.lda = Cout; p.b_mode = OP_CONV_WGRAD; p.ldo = p.N;
  p.g.KH = ks; p.g.KW = ks; p.g.stride = stride; p.g.pad = pad;
  p.g.H = H; p.g.W = W; p.g.C = Cin; p.g.OH = Ho; p.g.OW = Wo;
  p.epi = EPI_WGRAD;
  if (!conv_fast_eligible(p, dtype))
    return fail(CDP_EINVAL, "cdp_k_conv_wgrad_static: shape not supported by the two-phase weight-gradient kernels "
                            "(channel counts must be whole 16-byte chunks, at most 32 taps)");
  const int splits = conv_wgrad_splits(p, dtype, 3);
  const size_t need = (size_t)splits * (size_t)p.M * (size_t)p.N * 4;
  if (need > SCRATCH_BYTES)
    return fail(CDP_ENOMEM, "cdp_k_conv_wgrad_static: needs " + std::to_string(need) + " bytes of partial sums, the static scratch holds " +
                                std::to_string(SCRATCH_BYTES) + "; use cdp_k_conv with a workspace");
  void* ws = nullptr;
  int rc = scratch_ptr(&ws);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // every range writes its whole partial tile (an empty range writes zeros), so nothing in the scratch
  // has to start at zero; the output does, because the fold adds into it
  WReduceBatch rb;
  memset(&rb, 0, sizeof(rb));
  rb.n = 1;
  rb.p[0].part = static_cast<const float*>(ws);
  rb.p[0].G = dw;
  rb.p[0].Cout = p.M; rb.p[0].Ncol = p.N; rb.p[0].splits = splits;
  p.out = ws;
  p.splits = splits;
  hipError_t e = launch_fill_f32(dw, (int64_t)p.M * p.N, 0.f, st);
  if (e == hipSuccess) e = launch_conv_wgrad(b, dtype, p.M >= 128, st);
  if (e == hipSuccess) e = launch_wgrad_reduce(rb, dtype, st);
  if (e != hipSuccess) return fail(CDP_EHIP, std::string("cdp_k_conv_wgrad_static: ") + hipGetErrorString(e));
  return CDP_OK;
}
