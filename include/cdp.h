/* libcdp -- single-GPU hot path of Cyclic Data Parallelism (CDP) training on MI355X.
 *
 * The library executes the paper's execution timeline (Sec. 3.2 "Algorithmic
 * description", Fig. 1b/1c): N micro-batches run one uniform delay apart; in every
 * tick ("time step") each active micro-batch runs the forward or the backward of one
 * stage with the per-stage weight version chosen by the update rule (Eq. (CDP),
 * Eq. (CDP-v1), Eq. (CDP-v2), Eq. (DP)); backward passes add into a per-stage
 * gradient accumulator and a stage is updated by SGD as soon as it holds N gradients.
 * Placement is the single-GPU one of Sec. 4.1 "Cyclic implementation" (Fig. 2.a.ii).
 *
 * Conventions
 *   - every function returns CDP_OK (0) or a negative cdp_status; nothing throws;
 *     a call that fails before it changed anything leaves the context as it was; a tick that fails
 *     half-way (arena exhausted, a HIP error) leaves a context that refuses further ticks with
 *     CDP_ESTATE and can only be read and destroyed;
 *   - "dev" pointers are HIP device pointers, "host" pointers are ordinary host memory;
 *   - the caller owns every pointer it passes (inputs, labels, output buffers, the
 *     arena, the stream); the library owns only cdp_ctx and sub-allocates the arena;
 *   - all device work is enqueued on opts->hip_stream; calls return without waiting
 *     unless stated otherwise;
 *   - indices are 0-based: stage j in [0,S), micro-batch i in [0,N), step t >= 0,
 *     tick >= 0.  Micro-batch i of step t starts at tick 2*S*t + d*i, d = 2S/N.
 */
#ifndef CDP_H
#define CDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cdp_ctx cdp_ctx;

typedef enum {
  CDP_OK = 0,
  CDP_EINVAL = -1, /* bad argument, unsupported layer pattern, N does not divide 2S */
  CDP_ENOMEM = -2, /* arena too small (cdp_arena_bytes tells the need)               */
  CDP_ESTATE = -3, /* call not valid now (e.g. weight version no longer in the ring) */
  CDP_EHIP = -4    /* a HIP runtime call failed; see cdp_last_error                  */
} cdp_status;

/* Update rule u_{i,j} of Eq. (CDP).  DP runs the lock-step timeline of Fig. 1a. */
typedef enum {
  CDP_RULE_DP = 0, /* Eq. (DP):     every gradient of step t at theta_t               */
  CDP_RULE_V1 = 1, /* Eq. (CDP-v1): every gradient of step t at theta_{t-1}           */
  CDP_RULE_V2 = 2, /* Eq. (CDP-v2): freshest version in memory when the stage is read */
  CDP_RULE_MASK = 3 /* a rule in between (Sec. 3.2, "Update rules"): cdp_opts.fresh_mask says, per
                       (micro-batch, stage), v2's choice (1) or v1's (0)                  */
} cdp_rule;

/* Arithmetic of the contractions.  Accumulation, master weights, gradient
 * accumulators and the loss head are always fp32. */
typedef enum { CDP_F32 = 0, CDP_BF16 = 1 } cdp_dtype;

typedef enum {
  CDP_LINEAR = 1,  /* p = {in, out}                  params W[out][in], b[out]          */
  CDP_RELU = 2,    /* p = {}                                                           */
  CDP_CONV2D = 3,  /* p = {cin, cout, k, stride, pad} params W[cout][k][k][cin], NHWC   */
  CDP_AFFINE = 4,  /* p = {channels}                 params gamma[c], beta[c]           */
  CDP_ADD = 5,     /* p = {src2}  y = tensor[src] + tensor[src2]                       */
  CDP_MAXPOOL = 6, /* p = {k, stride, pad}                                             */
  CDP_GAP = 7,     /* p = {}      global average pool [B,H,W,C] -> [B,C]               */
  CDP_CE_HEAD = 8, /* p = {classes} mean softmax cross-entropy of the micro-batch      */
  /* ViT-shaped stages (the homogeneous stages of Sec. 5 "Memory"); tokens are kept as [B,1,T,D]: */
  CDP_LAYERNORM = 9,  /* p = {channels}  over the channel axis     params gamma[c], beta[c] */
  CDP_GELU = 10,      /* p = {}          x * Phi(x), exact form                             */
  CDP_ATTENTION = 11, /* p = {heads}     [B,1,T,3D] = (q|k|v) per token -> [B,1,T,D]:
                                         softmax(q k^T / sqrt(D/heads)) v per head          */
  CDP_TOKENS = 12     /* p = {}          [B,H,W,C] -> [B,1,H*W,C], no data movement; directly
                                         after CONV2D [AFFINE]                              */
} cdp_layer_kind;

/* One layer of a stage.  Tensors of a stage are numbered: 0 = stage input, k+1 =
 * output of layer k.  src = tensor read by the layer, -1 = output of the previous
 * layer.  Supported sequences (fused into one kernel each):
 *   LINEAR [RELU] | CONV2D [AFFINE] [TOKENS] [ADD] [RELU] | MAXPOOL | GAP | LINEAR CE_HEAD |
 *   LAYERNORM | GELU | ATTENTION.
 * CE_HEAD must be the last layer of the last stage and only there. */
typedef struct {
  int32_t kind;
  int32_t src;
  int32_t p[6];
} cdp_layer_desc;

typedef struct {
  const cdp_layer_desc* layers; /* host */
  int32_t n_layers;
} cdp_stage_desc;

typedef struct {
  int32_t dtype;       /* cdp_dtype                                                     */
  int32_t dry_run;     /* 1: host bookkeeping only (schedule, versions, pool); no HIP
                          call is made, arena and stream are ignored                    */
  int32_t in_rank;     /* 1: in_dims = {features}; 3: in_dims = {H, W, C}               */
  int32_t in_dims[3];  /* per-sample input shape                                        */
  void* hip_stream;    /* hipStream_t, may be NULL (default stream)                     */
  void* arena;         /* dev, 256-byte aligned, at least cdp_arena_bytes() long        */
  size_t arena_bytes;
  float momentum;      /* SGD momentum in [0,1); 0 = plain SGD of Eq. (CDP).  With momentum the
                          arena also holds one fp32 velocity per parameter                 */
  float weight_decay;  /* L2 coefficient added to the mean gradient (all parameters), >= 0   */
  int32_t dp_batched;  /* only with CDP_RULE_DP: 1 runs the lock-step timeline of Sec. 3.1 with the N
                          micro-batches of a step as ONE batch of N*micro_batch rows per stage pass
                          (every weight matrix is read once per pass instead of N times): the
                          throughput baseline the cyclic schedule is compared with.  Same update
                          (Eq. (DP)), same trace, live counts and per-micro-batch losses as the
                          pass-by-pass DP run; summation order inside a contraction differs.     */
  const uint8_t* fresh_mask; /* host, N*S bytes, [micro-batch][stage]; read at cdp_init; needed by (and only
                                by) CDP_RULE_MASK.  All ones is CDP_RULE_V2, all zeros CDP_RULE_V1.   */
  int32_t bwd_fresh;   /* 1: the backward of a stage reads the parameters that are freshest in memory at
                          its own tick instead of the version its forward read (the variant Sec. 3.2
                          alludes to: no second copy of the parameters needed).  The applied gradient is
                          then not the gradient of f_i at one point.  The trace records the version the
                          backward read.  Not combined with dp_batched.                              */
  int32_t dw_group;    /* 0 or 1: every backward pass adds its weight gradient to the stage accumulator (Eq. (CDP),
                          sum over i).  g = 2..4 (a divisor of N, cyclic rules): the Linear layers keep (dY, X) of g
                          consecutive micro-batches of a stage and take ONE pass over the accumulator per group -
                          the same sum in the same order i = 0..N-1, a g-th of the accumulator traffic, paid with
                          the activations of up to g-1 finished backward passes per stage staying in the pool (they
                          show in peak_activation_bytes and cdp_get_live_bytes).  Convolution layers are not grouped. */
} cdp_opts;

/* One executed (micro-batch, stage) pass. */
typedef struct {
  int32_t tick, mb, step, stage, dir /* 0 fwd, 1 bwd */, version;
} cdp_trace_rec;

typedef struct {
  int64_t ticks_run;
  int64_t steps_enqueued;
  int64_t peak_live_stage_inputs;   /* max over ticks of retained stage inputs (in-tick)  */
  int64_t last_live_stage_inputs;   /* value in the most recent tick                      */
  int64_t peak_activation_bytes;    /* high-water mark of retained activations + gradients
                                       in flight (the pool); per-tick workspace is separate */
  int64_t cur_activation_bytes;
  int64_t pool_span_bytes;          /* arena bytes the pool ever touched                  */
  int64_t dp_activation_bytes;      /* same stages under lock-step DP: N * sum_j bytes_j  */
  int64_t weight_bytes;             /* ring (2 versions) + fp32 master + fp32 accumulator */
  int64_t kernel_launches;
  int64_t scratch_bytes;            /* peak per-tick workspace (im2col buffers, partial sums) */
} cdp_stats;

/* Bytes of device arena the configuration needs (weights ring, master, accumulators,
 * activation pool found by a dry simulation of the schedule).  Host-only. */
int cdp_arena_bytes(const cdp_stage_desc* stages, int n_stages, int n_microbatches,
                    int micro_batch, int rule, const cdp_opts* opts, size_t* bytes_out);

/* Create a context.  stages/N/micro_batch/lr/rule are the quantities of Sec. 3
 * (theta = {theta^j}, N micro-batches of size B, learning rate gamma, rule u_{i,j}).
 * Requires N | 2S for the cyclic rules.  Weights start at zero until cdp_set_weights.
 * Update of a stage holding N gradients (Sec. 5 "Hyperparameters" optimiser when momentum or
 * weight decay are set): g = (1/N) sum_i grad f_i + wd*theta, v = momentum*v + g, theta -= lr*v. */
int cdp_init(cdp_ctx** out, const cdp_stage_desc* stages, int n_stages, int n_microbatches,
             int micro_batch, float lr, int rule, const cdp_opts* opts);

/* theta_0^j: host fp32, the stage's parameter tensors concatenated in layer order.
 * Both ring slots receive it (theta_{-1} := theta_0).  Only valid before the first tick. */
int cdp_set_weights(cdp_ctx* ctx, int stage, const float* host_f32, size_t n);

/* Number of fp32 parameters of a stage. */
int cdp_param_count(const cdp_ctx* ctx, int stage, size_t* n_out);

/* Advance one tick = one "time step" of Sec. 3.1 / Sec. 3.2 "Algorithmic description": every micro-batch in
 * flight runs the forward or the backward of the one stage the timeline of Fig. 1 assigns to it, with the
 * weight version u_{i,j} of Eq. (CDP) selects; stages that then hold N gradients are updated.  x_dev: fp32 [N*B, in_dims...] and y_dev: int32 [N*B] of the
 * mini-batch whose micro-batches may start in this tick (the step tick/(2S)); they are
 * read only in ticks where a micro-batch starts (x) -- labels are copied at that time.
 * May be NULL in ticks where no micro-batch starts (the drain). */
int cdp_tick(cdp_ctx* ctx, const float* x_dev, const int32_t* y_dev);

/* One training step t of Eq. (CDP) as the timeline executes it: enqueue mini-batch t (the next one) and run the 2S
 * ticks in which its N micro-batches start (the last of them finishes d*(N-1) ticks into the following steps, Fig. 1).  x_dev/y_dev as above;
 * they must stay valid until the enqueued work has run. */
int cdp_step(cdp_ctx* ctx, const float* x_dev, const int32_t* y_dev);

/* Run the remaining d*(N-1) ticks so that every stage reaches theta_T: the tail of the cyclic timeline of
 * Sec. 3.2 (micro-batch i starts d*i ticks after micro-batch 0) with no new mini-batch entering. */
int cdp_drain(cdp_ctx* ctx);

/* theta^j_t of Eq. (CDP): copy a stage's parameters to host fp32 (synchronises the stream).  The ring holds the two
 * versions Eq. (CDP) can ask for, theta_t and theta_{t-1}.  version = -1:
 * freshest (fp32 master values); version = freshest-1: the compute-precision copy
 * still held in the ring (its folded/rounded form is not inverted: CDP_ESTATE for
 * stages with AFFINE layers).  Any other version: CDP_ESTATE. */
int cdp_get_weights(cdp_ctx* ctx, int stage, int version, float* host_f32, size_t cap,
                    size_t* n_out);

/* Micro-batch objectives f_i of step t: host fp32 [N] (synchronises).  CDP_ESTATE if
 * the step's head passes have not all run yet or the step left the log (last 1024). */
int cdp_get_losses(cdp_ctx* ctx, int64_t step, float* host_f32, size_t cap);

/* Executed passes in order (tick, then micro-batch ascending). Host-only. */
int cdp_get_trace(const cdp_ctx* ctx, cdp_trace_rec* out, size_t cap, size_t* n_out);

/* In-tick count of retained stage inputs for every tick run so far. Host-only. */
int cdp_get_live_counts(const cdp_ctx* ctx, int32_t* out, size_t cap, size_t* n_out);

/* In-tick activation bytes for every tick run so far (Sec. 4.1: the memory the cyclic schedule keeps
 * nearly constant over the time steps; Table 1, rows "Single-GPU").  kind 0: bytes retained for a later
 * backward (stage inputs and the intermediates a backward reads; same counting as the live count: a
 * forward of the tick has stored, a backward of the tick has not released); kind 1: everything the
 * activation pool holds while the tick's kernels run (adds activations / gradients travelling between
 * stages).  Constant over steady-state ticks for homogeneous stages except for the head's extra
 * tensors, periodic with the delay d in general.  Host-only. */
int cdp_get_live_bytes(const cdp_ctx* ctx, int kind, int64_t* out, size_t cap, size_t* n_out);

int cdp_get_stats(const cdp_ctx* ctx, cdp_stats* out);

/* Timing of the grouped contraction launches, the dominant kernel of a tick (forward,
 * data-gradient and weight-gradient tiles of all active (micro-batch, stage) pairs).
 * While enabled, every such launch is bracketed by two HIP events on the work stream.
 * flops / bytes are the algorithmic work of the timed launches: 2 * multiply-adds of each
 * contraction; bytes with every operand read once and every result written once. */
typedef struct {
  int64_t launches;
  double total_ms;   /* sum of the event-to-event times of the launches */
  double flops;
  double bytes;
  double empty_pair_ms; /* what an event pair with nothing between reads on this stream (median of 32
                           pairs taken when recording was enabled): the bracket's own share of every
                           event-to-event time, to be subtracted per launch                          */
} cdp_gemm_profile;

/* enable != 0 starts a fresh measurement, 0 stops recording (synchronises). */
int cdp_profile_gemm(cdp_ctx* ctx, int enable);
/* Sums over the launches recorded since the last cdp_profile_gemm (synchronises). */
int cdp_get_gemm_profile(cdp_ctx* ctx, cdp_gemm_profile* out);

/* Text of the last error on this context (or of the last failed cdp_init /
 * cdp_arena_bytes when ctx is NULL).  Never NULL. */
const char* cdp_last_error(const cdp_ctx* ctx);

void cdp_destroy(cdp_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* CDP_H */
