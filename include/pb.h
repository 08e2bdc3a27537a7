/* pb.h -- C ABI of the batch-1 Pipelined Backpropagation (PB) tick engine for
 * AMD MI355X (gfx950).
 *
 * One context simulates an S-stage pipeline on one GPU.  One call of pb_tick
 * is one time step of the pipeline described in the paper's appendix
 * "Pipelined Backpropagation": every stage performs the forward pass of one
 * in-flight sample and the backward pass of another, then every stage that
 * produced a gradient is updated, without ever draining the pipeline
 * (Eq. sgdpb).  Stage s sees, on its forward pass, weights that are
 * D^s = 2(S-1-s) updates older than those its backward pass sees (Eq. wf).
 * The forward pass runs on Linear-Weight-Predicted weights
 * w_hat = w - lr*T*v, T = D^s (Eq. lwp_v_form); the update is the
 * Spike-Compensated momentum step  v <- m v + g ; w <- w - lr (a v + b g)
 * with a = m^D, b = (1-m^D)/(1-m) (Eqs. gscv, gscw, scd; combination in
 * Section "Combined Mitigation").
 *
 * All functions return 0 (or a non-negative count) on success and a negative
 * PB_E* code on failure; pb_last_error() then describes the failure.  No
 * function throws.  Unless said otherwise pointers are HOST pointers.  The
 * library is not thread-safe per context.
 */
#ifndef PB_H_
#define PB_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pb_ctx pb_ctx;

enum {
  PB_OK = 0,
  PB_E_INVALID = -1,      /* bad descriptor / argument                     */
  PB_E_UNSUPPORTED = -2,  /* valid request the GPU path does not implement  */
  PB_E_NOMEM = -3,        /* arena too small or device allocation failed    */
  PB_E_HIP = -4           /* a HIP runtime call failed                      */
};

/* Operations a pipeline stage is composed of.  A stage holds exactly one
 * weight layer (LINEAR or CONV2D) -- the paper assigns one layer per stage
 * and fuses its normalisation, activation and the residual sum into it
 * (Section "Experiments").  Accepted op order inside a stage:
 *   [GROUPNORM] [RELU] [GLOBAL_AVGPOOL] (CONV2D|LINEAR)
 *   [GROUPNORM RELU [MAXPOOL]] [ADD_SKIP] [SOFTMAX_CE]
 * with at most one GROUPNORM per stage; SOFTMAX_CE only as the last op of the
 * last stage, where it is mandatory. */
typedef enum {
  PB_OP_LINEAR = 0,         /* y = W x + b; x is the flattened (C,H,W) input; cin, cout, has_bias */
  PB_OP_CONV2D = 1,         /* square kernel k, stride, pad; weight [cout][cin][k][k]; has_bias   */
  PB_OP_GROUPNORM = 2,      /* groups; cin = cout = channels; biased variance, eps 1e-5, affine   */
  PB_OP_RELU = 3,           /* max(x,0); derivative 0 at 0                                        */
  PB_OP_MAXPOOL = 4,        /* window k, stride, pad; gradient to the first maximum (row-major)   */
  PB_OP_GLOBAL_AVGPOOL = 5, /* mean over H*W                                                      */
  PB_OP_ADD_SKIP = 6,       /* y += tensor that entered stage skip_from_stage (same sample);      *
                             * has_proj: through a 1x1 conv cin->cout with the given stride first, *
                             * whose weight [cout][cin] belongs to this stage                      */
  PB_OP_SOFTMAX_CE = 7      /* loss = -log softmax(x)[label]; dlogits = softmax - onehot           */
} pb_op_kind;

typedef struct {
  int32_t kind;             /* pb_op_kind */
  int32_t cin, cout;
  int32_t k, stride, pad;
  int32_t groups;
  int32_t has_bias;
  int32_t skip_from_stage;  /* ADD_SKIP only; must be < index of the stage holding the op */
  int32_t has_proj;         /* ADD_SKIP only */
} pb_op;

typedef struct {
  int32_t n_ops;
  const pb_op* ops;
} pb_stage;

/* Planner settings a caller may override (all zero = the library's own choices). */
typedef struct {
  int32_t tile_target;      /* latency-tiled networks: workgroups a forward GEMM step is split into at least   */
  int32_t tile_target_bwd;  /* ... and a backward GEMM step                                                     */
  float tile_budget_us;     /* > 0: tile for throughput with this budget for the longest tile (microseconds,
                               estimate); < 0: tile for latency whatever the network's size; 0: by size       */
  int32_t nt_stores;        /* kernel instantiation with non-temporal output stores: 1 on, -1 off, 0 by policy  */
  int32_t one_launch;       /* one kernel launch per tick -- the workgroups of a later phase wait inside the launch
                               for the stage's workgroups of the earlier phases --: 1 on, -1 off, 0 by policy
                               (on where a tick has no more workgroups than the GPU has compute units)             */
  int32_t tail_merge;       /* n > 0: the phases from phase n on share one launch in the same way (n = 0 with
                               one_launch = 1); 0 or -1: off (measured slower on every configuration); -2: the
                               longest run of last phases that hold steps of at most two stages                    */
  int32_t spin_limit;       /* bound of such a wait, in polls (0 = default, 65536: a fraction of a second); when it expires the
                               step is skipped and the next synchronising call returns PB_E_HIP                    */
  int32_t dense_1x1;        /* 1x1 layers in throughput-tiled networks as dense matrix products with register tiles:
                               -1 off, 0 or 1 on where the shapes allow, 2 also forward and backward weights of k x k
                               layers (their operands gathered tap by tap: measured slower, never chosen by policy)  */
  int32_t gemm_lds_kb;      /* LDS a GEMM tile may plan with, KB: 62 or 76 (two workgroups share a compute unit's 160 KB);
                               0: by policy (76 where a tick holds long reductions, 62 elsewhere)                  */
} pb_tuning;

typedef struct {
  int32_t n_stages;
  const pb_stage* stages;
  int32_t in_c, in_h, in_w;   /* one sample is in_c*in_h*in_w floats, CHW order */
  int32_t n_classes;
  int32_t mitigation;         /* 0 plain delayed SGDM, 1 SC_D, 2 LWP^v_D, 3 SC_D + LWP^v_D */
  int32_t bwd_weights;        /* 0 backward pass uses current weights (the paper's PB); 1 weight
                                 stashing: it uses the predicted weights its forward pass read,
                                 kept in a ring of delays[s] + 2 versions per stage            */
  int32_t act_dtype;          /* 0 fp32 activations; 1 bf16: tensors that cross a stage boundary are
                                 rounded to bf16 (nearest even) by the step that writes them      */
  int32_t loss_capacity;      /* losses kept (most recent); 0 = 1<<20                       */
  int32_t kernel_set;         /* 0 tiled MFMA kernels (default), 1 plain direct kernels     */
  void* device_arena;         /* DEVICE memory owned by the caller (>= pb_arena_bytes, 256-byte
                                 aligned) that must outlive the context, or NULL: the library
                                 allocates and frees its own */
  size_t arena_bytes;
  void* stream;               /* hipStream_t to launch on, NULL = the null stream */
  float sc_scale;             /* over-compensation: SC uses the coefficients of delay sc_scale * delays[s]  */
  float lwp_scale;            /* ... and LWP the horizon T = lwp_scale * delays[s]; 0 means 1 for both     */
  int32_t lwp_form;           /* 0 velocity form w_hat = w - lr T v (Eq. lwp_v_form); 1 weight-difference
                                 form w_hat = w + T (w - w_prev) (Eq. lwp_w_form)                          */
  int32_t update_size;        /* samples per update (Appendix "Small Batch Size Training"; the paper uses 1 = 0
                                 here).  N > 1: still one sample per stage and tick; a stage adds up the
                                 gradients of N consecutive samples and applies one update with their mean
                                 after the last one's backward pass; SC and LWP count the stage's delay in
                                 updates, delays[s] / N                                                     */
  const pb_tuning* tuning;    /* NULL = defaults */
} pb_net_desc;

/* Device bytes pb_init needs for this network (0 on an invalid descriptor). */
size_t pb_arena_bytes(const pb_net_desc* net, const int32_t* delays);

/* Build a context.  delays: n_stages entries or NULL for the pipeline's own
 * D^s = 2(S-1-s) (Eq. wf).  delays[s] > 2(S-1-s): the forward pass of stage s
 * uses predicted weights that many updates old, read from a ring of
 * delays[s] - 2(S-1-s) + 2 weight versions per stage (more device memory:
 * ask pb_arena_bytes with the same delays), and SC / LWP use delays[s] as the
 * stage's delay.  If any delays[s] < 2(S-1-s) -- which a pipeline that never
 * stalls cannot produce -- the context runs the sample-indexed form instead
 * (Eqs. wi, sgdpb, wf): one pb_tick pushes one sample through all stages in
 * dependency order, forward pass of stage s with the weights delays[s] updates
 * old, backward pass with the current ones, then the update; pb_loss_history
 * then has one entry per tick.  With all delays zero that is SGD with
 * momentum.  A verification mode (several launches per stage and tick), not
 * a performance path.  Negative delays are rejected.  Weights are initialised on
 * the host from `seed` (Kaiming normal, std sqrt(2/fan_in), biases 0,
 * GroupNorm scale 1 / shift 0) and uploaded; velocity starts at 0.
 * The descriptor is copied; the caller may free it afterwards. */
int pb_init(pb_ctx** out, const pb_net_desc* net, const int32_t* delays, float lr, float momentum,
            uint64_t seed);

/* pb_init for callers that cannot allocate device memory (code under HIP graph
 * capture set-up, tight serving loops, harnesses that forbid hipMalloc): the
 * same context, the same kernels, but the arena -- weights, velocities,
 * gradients, activation rings, partial sums, step tables -- lies in a device
 * array that is part of the library itself, pb_static_arena_bytes() = 64 MiB
 * per GPU, held by every GPU the library runs on until the process ends.
 * Calls no hipMalloc / hipFree and no allocating library routine; the array
 * is cleared by a kernel.  net->device_arena must be NULL.  A network whose
 * pb_arena_bytes exceeds the array is refused with PB_E_NOMEM (ResNet-20 at
 * 32x32 needs 55 MiB with the default loss_capacity; VGG-11 and larger do not
 * fit: use pb_init).  All contexts built by this call on one GPU would share
 * that GPU's array -- overlapping use would race --, so a second call on the
 * same GPU is refused with PB_E_UNSUPPORTED until pb_destroy has released the
 * first context.  The array keeps the previous context's contents until the
 * next call clears it.  Everything else is as for pb_init. */
int pb_init_static(pb_ctx** out, const pb_net_desc* net, const int32_t* delays, float lr, float momentum,
                   uint64_t seed);
size_t pb_static_arena_bytes(void);

/* One pipeline time step: feeds `sample` (host, in_c*in_h*in_w floats) with
 * its class label, runs every stage's forward and backward work and the fused
 * update.  The sample is copied before the call returns; GPU work is
 * asynchronous on the context's stream. */
int pb_tick(pb_ctx* ctx, const float* sample, int32_t label);

/* n_ticks time steps fed from a pool resident in DEVICE memory: tick j of
 * this call consumes item (first_index + j) mod n_pool of samples_dev
 * ([n_pool][in_c*in_h*in_w] floats) / labels_dev ([n_pool] int32).  Nothing
 * crosses the host-device boundary.  Asynchronous. */
int pb_run_resident(pb_ctx* ctx, const float* samples_dev, const int32_t* labels_dev,
                    int32_t n_pool, int64_t first_index, int64_t n_ticks);

/* Master weights w (not the predicted ones) in canonical order: stage-major;
 * within a stage: layer weight [cout][cin][kh][kw], bias, projection weight,
 * GroupNorm scale, shift.  Synchronises the stream.  dst == NULL returns the
 * number of floats; otherwise at most cap floats are written and the count
 * returned.  After K ticks stage s has received max(0, K - 2(S-1) + s)
 * updates. */
int64_t pb_read_weights(pb_ctx* ctx, float* dst, int64_t cap);

/* Same layout, the velocity v. */
int64_t pb_read_velocity(pb_ctx* ctx, float* dst, int64_t cap);

/* Loss of sample i at entry i (the sample fed by the i-th tick); after K
 * ticks max(0, K-S+1) losses exist.  Returns the most recent
 * min(count, loss_capacity, cap) of them in sample order.  dst == NULL
 * returns the number available.  Synchronises the stream. */
int64_t pb_loss_history(pb_ctx* ctx, float* dst, int64_t cap);

int64_t pb_num_params(const pb_ctx* ctx);
int64_t pb_num_ticks(const pb_ctx* ctx);

/* Launch policy: 0 = one launch per pipeline phase (default), 1 = one launch
 * per step of every stage, update steps included (profiling and debugging
 * aid; same records, same arithmetic, bit-identical results). */
int pb_set_launch_mode(pb_ctx* ctx, int32_t mode);

/* Kernel timing with HIP events on the context's stream.  pb_profile_begin
 * starts recording every launch of the following ticks (at most `max_events`
 * launches), pb_profile_end synchronises and returns, for kernel class
 * `which`, the number of launches recorded and their total milliseconds.
 * Classes: 0 = phase launches (launch mode 0) or forward / backward steps
 * (launch mode 1); 1 = update steps and 2 = ingest, both recorded separately
 * only in launch mode 1. */
int pb_profile_begin(pb_ctx* ctx, int32_t max_events);
int pb_profile_end(pb_ctx* ctx, int32_t which, int64_t* n_launches, double* total_ms);

/* Stand-alone launch of the fused update kernel over caller-provided DEVICE
 * arrays of n floats (n a multiple of 1024, every array 16-byte aligned:
 * PB_E_INVALID otherwise) with one set of coefficients:
 * v <- m v + g; w <- w - lr (a v + b g); w_hat <- w - lrT v (skipped when
 * w_hat == NULL).  Used to measure the kernel at sizes beyond the caches. */
int pb_update_standalone(float* w_dev, float* v_dev, const float* g_dev, float* what_dev, int64_t n,
                         float lr, float m, float a, float b, float lrT, void* stream);

/* Human-readable table of the steps one tick consists of (stage, phase, kernel
 * kind, tiles, GEMM tiling), one line per step.  Returns the bytes needed
 * including the terminator; writes at most cap bytes into buf (may be NULL). */
int64_t pb_plan_summary(const pb_net_desc* net, char* buf, int64_t cap);

/* Learning rate and momentum for update size n from the values in use at a
 * reference update size n_ref (Appendix "Small Batch Size Training",
 * Eq. hpscale): the momentum's decay per sample stays the same,
 * m = m_ref^(n/n_ref), and the effective learning rate lr/(1-m) grows
 * linearly with the update size, lr = lr_ref (1-m) n / ((1-m_ref) n_ref).
 * The paper trains at n = 1 with hyper-parameters published for n_ref = 128
 * or 32; the results are what pb_init takes as lr and momentum.  Host
 * arithmetic in double, results rounded once to float.  lr_out, momentum_out:
 * host pointers, written on success.  PB_E_INVALID if a pointer is NULL,
 * n or n_ref < 1, momentum_ref outside [0,1] or lr_ref < 0. */
int pb_scale_hyperparameters(float lr_ref, float momentum_ref, int32_t n_ref, int32_t n, float* lr_out,
                             float* momentum_out);

int pb_sync(pb_ctx* ctx);
void pb_destroy(pb_ctx* ctx);
const char* pb_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PB_H_ */
