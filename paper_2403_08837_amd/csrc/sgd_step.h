// Device-side SGD step shared by the update kernels and the fused weight-gradient tile.
#pragma once
#include "kernels.h"

namespace cdp {

// One parameter: g = gsum/N + wd*w ; with a velocity v = momentum*v + g (stored back) ; returns w - lr*v.
// (Eq. (CDP) for plain SGD; Sec. 5 "Hyperparameters" for momentum and weight decay.)
__device__ __forceinline__ float sgd_step(float w, float gsum, float* v, const SgdParams& p) {
  float g = gsum * p.inv_n + p.wd * w;
  if (v) {
    g = p.momentum * (*v) + g;
    *v = g;
  }
  return w - p.lr * g;
}

}  // namespace cdp
