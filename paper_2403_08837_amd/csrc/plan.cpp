#include "plan.h"

#include <sstream>

namespace cdp {

namespace {

std::string err(int stage, int layer, const char* what) {
  std::ostringstream o;
  o << "stage " << stage << " layer " << layer << ": " << what;
  return o.str();
}

bool follows(const cdp_layer_desc& l, int idx) { return l.src == -1 || l.src == idx; }

}  // namespace

std::string build_plan(const cdp_stage_desc* stages, int n_stages, const cdp_opts* opts, ModelPlan* out) {
  if (!stages || n_stages <= 0) return "no stages";
  if (!opts) return "opts is NULL";
  if (opts->dtype != CDP_F32 && opts->dtype != CDP_BF16) return "unknown dtype";
  out->dtype = opts->dtype;
  out->elem_bytes = opts->dtype == CDP_BF16 ? 2 : 4;
  out->stages.clear();

  TensorInfo cur;
  if (opts->in_rank == 1) {
    cur.C = opts->in_dims[0];
  } else if (opts->in_rank == 3) {
    cur.H = opts->in_dims[0];
    cur.W = opts->in_dims[1];
    cur.C = opts->in_dims[2];
  } else {
    return "in_rank must be 1 or 3";
  }
  if (cur.H <= 0 || cur.W <= 0 || cur.C <= 0) return "input dims must be positive";

  for (int s = 0; s < n_stages; ++s) {
    const cdp_stage_desc& sd = stages[s];
    if (!sd.layers || sd.n_layers <= 0) return err(s, 0, "empty stage");
    StagePlan sp;
    TensorInfo t0 = cur;
    t0.producer = -1;
    t0.consumed = false;
    t0.is_residual = false;
    t0.n_consumers = 0;
    sp.tensors.push_back(t0);
    std::vector<int> map(sd.n_layers + 1, -1);  // layer-tensor index -> plan tensor id
    map[0] = 0;
    int64_t poff = 0;
    int i = 0;
    while (i < sd.n_layers) {
      const cdp_layer_desc& L = sd.layers[i];
      const int src_lt = (L.src < 0) ? i : L.src;
      if (src_lt > i || map[src_lt] < 0) return err(s, i, "src refers to a tensor that is not materialised");
      const int in_id = map[src_lt];
      const TensorInfo tin = sp.tensors[in_id];
      Op op;
      op.in = in_id;
      TensorInfo tout;
      int j = i + 1;
      if (L.kind == CDP_LINEAR) {
        if (L.p[0] <= 0 || L.p[1] <= 0) return err(s, i, "bad linear dims");
        if (tin.per_sample() != L.p[0]) return err(s, i, "linear in_features does not match its input");
        op.kind = OPK_GEMM;
        op.Cin = L.p[0];
        op.Cout = L.p[1];
        op.w_off = poff;
        poff += (int64_t)L.p[0] * L.p[1];
        op.b_off = poff;
        poff += L.p[1];
        tout.C = L.p[1];
        if (j < sd.n_layers && sd.layers[j].kind == CDP_RELU && follows(sd.layers[j], j)) {
          op.relu = true;
          ++j;
        } else if (j < sd.n_layers && sd.layers[j].kind == CDP_CE_HEAD && follows(sd.layers[j], j)) {
          op.out_f32 = true;
          tout.f32 = true;
        }
      } else if (L.kind == CDP_CONV2D) {
        const int cin = L.p[0], cout = L.p[1], ks = L.p[2], st = L.p[3], pd = L.p[4];
        if (cin <= 0 || cout <= 0 || ks <= 0 || st <= 0 || pd < 0) return err(s, i, "bad conv2d parameters");
        if (tin.C != cin) return err(s, i, "conv2d cin does not match its input");
        if (tin.H + 2 * pd < ks || tin.W + 2 * pd < ks) return err(s, i, "conv2d kernel larger than padded input");
        op.kind = OPK_GEMM;
        op.is_conv = true;
        op.Cin = cin; op.Cout = cout; op.KH = ks; op.KW = ks; op.stride = st; op.pad = pd;
        op.Hin = tin.H; op.Win = tin.W;
        op.Hout = (tin.H + 2 * pd - ks) / st + 1;
        op.Wout = (tin.W + 2 * pd - ks) / st + 1;
        op.w_off = poff;
        poff += (int64_t)cout * ks * ks * cin;
        tout.H = op.Hout; tout.W = op.Wout; tout.C = cout;
        if (cin % (16 / out->elem_bytes) != 0) op.kpad = (int)align_up((int64_t)ks * ks * cin, out->elem_bytes == 2 ? 64 : 32);
        if (j < sd.n_layers && sd.layers[j].kind == CDP_AFFINE && follows(sd.layers[j], j)) {
          if (sd.layers[j].p[0] != cout) return err(s, j, "affine channels do not match the conv");
          op.has_gamma = true;
          op.g_off = poff;
          poff += cout;
          op.b_off = poff;
          poff += cout;
          ++j;
        }
        if (j < sd.n_layers && sd.layers[j].kind == CDP_TOKENS && follows(sd.layers[j], j)) {
          tout.W = tout.H * tout.W;  // the patch grid read as one row of tokens: same memory
          tout.H = 1;
          ++j;
        }
        if (j < sd.n_layers && sd.layers[j].kind == CDP_ADD && follows(sd.layers[j], j)) {
          const int s2 = sd.layers[j].p[0];
          if (s2 < 0 || s2 > j || map[s2] < 0) return err(s, j, "add src2 is not a materialised tensor");
          op.res = map[s2];
          const TensorInfo& tr = sp.tensors[op.res];
          if (tr.H != tout.H || tr.W != tout.W || tr.C != tout.C) return err(s, j, "add operand shapes differ");
          ++j;
        }
        if (j < sd.n_layers && sd.layers[j].kind == CDP_RELU && follows(sd.layers[j], j)) {
          op.relu = true;
          ++j;
        }
      } else if (L.kind == CDP_MAXPOOL) {
        op.kind = OPK_MAXPOOL;
        op.pk = L.p[0]; op.ps = L.p[1]; op.pp = L.p[2];
        if (op.pk <= 0 || op.ps <= 0 || op.pp < 0 || 2 * op.pp >= op.pk + op.ps) return err(s, i, "bad maxpool parameters");
        op.Hin = tin.H; op.Win = tin.W; op.Cin = op.Cout = tin.C;
        op.Hout = (tin.H + 2 * op.pp - op.pk) / op.ps + 1;
        op.Wout = (tin.W + 2 * op.pp - op.pk) / op.ps + 1;
        if (op.Hout <= 0 || op.Wout <= 0) return err(s, i, "maxpool output is empty");
        tout.H = op.Hout; tout.W = op.Wout; tout.C = tin.C;
        tout.relu = tin.relu;  // a max over non-negative values stays non-negative
      } else if (L.kind == CDP_GAP) {
        op.kind = OPK_GAP;
        op.Hin = tin.H; op.Win = tin.W; op.Cin = op.Cout = tin.C;
        tout.C = tin.C;
      } else if ((L.kind == CDP_LAYERNORM || L.kind == CDP_GELU || L.kind == CDP_ATTENTION) && tin.relu) {
        return err(s, i, "layernorm / gelu / attention directly on a ReLU output is not supported");
      } else if (L.kind == CDP_LAYERNORM) {
        if (L.p[0] != tin.C || tin.C > 1024) return err(s, i, "layernorm channels must match its input and be at most 1024");
        if (tin.f32) return err(s, i, "layernorm cannot read logits");
        op.kind = OPK_LN;
        op.Hin = op.Hout = tin.H; op.Win = op.Wout = tin.W; op.Cin = op.Cout = tin.C;
        op.g_off = poff;
        poff += tin.C;
        op.b_off = poff;
        poff += tin.C;
        tout.H = tin.H; tout.W = tin.W; tout.C = tin.C;
      } else if (L.kind == CDP_GELU) {
        if (tin.f32) return err(s, i, "gelu cannot read logits");
        op.kind = OPK_GELU;
        op.Hin = op.Hout = tin.H; op.Win = op.Wout = tin.W; op.Cin = op.Cout = tin.C;
        tout.H = tin.H; tout.W = tin.W; tout.C = tin.C;
      } else if (L.kind == CDP_ATTENTION) {
        const int heads = L.p[0];
        if (heads <= 0 || tin.H != 1 || tin.C % (3 * heads) != 0 || tin.W > 1024 || tin.f32)
          return err(s, i, "attention needs tokens [1, T <= 1024, 3*D] with D a multiple of heads");
        op.kind = OPK_ATTN;
        op.heads = heads;
        op.Hin = op.Hout = 1; op.Win = op.Wout = tin.W; op.Cin = tin.C; op.Cout = tin.C / 3;
        tout.H = 1; tout.W = tin.W; tout.C = tin.C / 3;
        // the attention probabilities [heads][T][T] are a saved tensor of their own
        TensorInfo tp;
        tp.H = heads; tp.W = tin.W; tp.C = tin.W;
        tp.consumed = true;
        tp.n_consumers = 1;
        tp.producer = (int)sp.ops.size();
        op.aux = (int)sp.tensors.size();
        sp.tensors.push_back(tp);
      } else if (L.kind == CDP_CE_HEAD) {
        if (s != n_stages - 1 || i != sd.n_layers - 1) return err(s, i, "ce_head must be the last layer of the last stage");
        if (!tin.f32 || tin.per_sample() != L.p[0]) return err(s, i, "ce_head must follow a linear layer with `classes` outputs");
        op.kind = OPK_CE;
        op.classes = L.p[0];
        tout = tin;
        tout.f32 = false;  // output slot holds dlogits in the compute type
        sp.has_head = true;
      } else {
        return err(s, i, "layer kind cannot start a fused group (RELU/AFFINE/ADD must follow LINEAR or CONV2D)");
      }
      if (op.kind == OPK_GEMM) tout.relu = op.relu;
      tout.producer = (int)sp.ops.size();
      op.out = (int)sp.tensors.size();
      sp.tensors[op.in].consumed = true;
      sp.tensors[op.in].n_consumers++;
      if (op.res >= 0) sp.tensors[op.res].is_residual = true;
      sp.tensors.push_back(tout);
      map[j] = op.out;
      sp.ops.push_back(op);
      i = j;
    }
    // structural checks the backward pass relies on
    for (size_t k = 0; k < sp.tensors.size(); ++k) {
      const TensorInfo& t = sp.tensors[k];
      const bool last = (k + 1 == sp.tensors.size());
      if (!last && !t.consumed && !t.is_residual) return err(s, (int)k, "tensor is never used");
      if (t.is_residual && !t.consumed && t.relu) return err(s, (int)k, "a ReLU output used only as residual is not supported");
      if (t.n_consumers > 1 || t.is_residual)
        for (const Op& o : sp.ops)
          if (o.in == (int)k && o.kind != OPK_GEMM && o.kind != OPK_LN)
            return err(s, (int)k, "a tensor read by a pooling, GELU or attention layer must have no other use");
    }
    if ((s == n_stages - 1) != sp.has_head) return err(s, 0, "the last stage, and only it, must end in ce_head");
    // ring slot layout
    int64_t off = 0;
    for (Op& o : sp.ops) {
      if (o.kind == OPK_LN) {  // fp32 copies of gamma and beta
        o.gamma_c = off; off = align_up(off + (int64_t)o.Cout * 4, 256);
        o.bias_c = off; off = align_up(off + (int64_t)o.Cout * 4, 256);
        sp.has_gamma = true;
        continue;
      }
      if (o.kind != OPK_GEMM) continue;
      o.wf = off; off = align_up(off + (o.kpad ? (int64_t)o.Cout * o.kpad : o.w_count()) * out->elem_bytes, 256);
      o.wt = off; off = align_up(off + o.w_count() * out->elem_bytes, 256);
      if (o.has_gamma) { o.wp = off; off = align_up(off + o.w_count() * out->elem_bytes, 256); sp.has_gamma = true; }
      if (o.b_off >= 0) { o.bias_c = off; off = align_up(off + (int64_t)o.Cout * 4, 256); }
      if (o.has_gamma) { o.gamma_c = off; off = align_up(off + (int64_t)o.Cout * 4, 256); }
    }
    sp.slot_bytes = off;
    sp.n_params = poff;
    cur = sp.tensors.back();
    out->stages.push_back(sp);
  }
  return "";
}

}  // namespace cdp
