// Host-side model plan: layer descriptors of a stage are fused into kernel-sized ops,
// tensor shapes and parameter/ring layouts are derived once at cdp_init.
#pragma once
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/cdp.h"

namespace cdp {

inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct TensorInfo {
  int H = 1, W = 1, C = 1;     // per-sample shape (vectors: 1 x 1 x features)
  bool f32 = false;            // logits are kept in fp32, everything else in the compute type
  bool relu = false;           // produced by an op that ends in ReLU (values >= 0)
  bool consumed = false;       // read as the input of some op (must survive until backward)
  bool is_residual = false;    // read as the residual operand of some op
  int n_consumers = 0;         // ops that read it as input
  int producer = -1;           // op index, -1 for the stage input
  int64_t per_sample() const { return (int64_t)H * W * C; }
};

enum OpKind { OPK_GEMM = 0, OPK_MAXPOOL = 1, OPK_GAP = 2, OPK_CE = 3, OPK_LN = 4, OPK_GELU = 5, OPK_ATTN = 6 };

struct Op {
  int kind = OPK_GEMM;
  int in = 0, out = 0, res = -1;  // tensor ids within the stage
  bool relu = false, is_conv = false, has_gamma = false, out_f32 = false;
  int Cin = 0, Cout = 0, KH = 1, KW = 1, stride = 1, pad = 0;  // Linear: 1x1 conv on a 1x1 image
  int Hin = 1, Win = 1, Hout = 1, Wout = 1;
  int pk = 0, ps = 0, pp = 0;     // pooling window / stride / pad
  int classes = 0;
  int heads = 0;                  // OPK_ATTN
  int aux = -1;                   // OPK_ATTN: tensor id of the attention probabilities kept for the backward
  int kpad = 0;                   // > 0: the forward weights are stored with this (zero-padded) row length and the
                                  // layer runs on an explicit im2col buffer (channel counts below one 16-byte chunk)
  // float offsets inside the stage's flat fp32 parameter block (-1: absent)
  int64_t w_off = -1, b_off = -1, g_off = -1;
  // byte offsets inside one ring slot
  int64_t wf = -1, wt = -1, wp = -1, bias_c = -1, gamma_c = -1;
  int64_t K() const { return (int64_t)KH * KW * Cin; }
  int64_t w_count() const { return (int64_t)Cout * K(); }
};

struct StagePlan {
  std::vector<TensorInfo> tensors;
  std::vector<Op> ops;
  int64_t n_params = 0;      // fp32 parameters (user-visible flat block)
  int64_t slot_bytes = 0;    // one ring slot (compute copies of one weight version)
  bool has_gamma = false;
  bool has_head = false;
};

struct ModelPlan {
  std::vector<StagePlan> stages;
  int elem_bytes = 4;
  int dtype = 0;
};

// Returns "" on success, else a description of the unsupported pattern.
std::string build_plan(const cdp_stage_desc* stages, int n_stages, const cdp_opts* opts, ModelPlan* out);

}  // namespace cdp
