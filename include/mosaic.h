/*
 * mosaic.h -- C ABI of the MI355X (gfx950) hot path of temporal-spatial module
 * multiplexing: forward+backward of a multimodal model's modules running at the same
 * time on one GPU, each confined to a compute-unit quota.
 *
 * Vocabulary follows the paper's problem formulation (Sec. 3.1): a training job is a
 * set of modules m; a stage S is a set of mutually independent modules that share the
 * GPU spatially, each with a quota a_m of its compute units (Eq. 4-5: stage time is the
 * slowest module's time and the quotas of one GPU sum to at most 1); stages follow one
 * another in time (Eq. 1: iteration time is the sum of stage times).  The engine of
 * Sec. 3.2 gives every module a stream whose quota is fixed at creation and takes such
 * streams from a pool created before training starts.
 *
 * Conventions
 *   - Every pointer named x, y, dx, dy, params, grads, workspace, target, loss, or any
 *     tensor argument of a mosaic_op_* call is a DEVICE pointer owned by the caller.
 *     Descriptors, plans, timing structs, mask words and name buffers are HOST memory.
 *   - Tensors are dense row-major.  Activations are [T, width] with T = batch*seq tokens,
 *     sample-major.  Weights are [in, out].  dtype MOSAIC_F32 stores float; MOSAIC_BF16
 *     stores bfloat16 (round-to-nearest-even) and accumulates in fp32.
 *   - All calls return a status; none throws or aborts.  Argument errors are detected
 *     before anything is launched.  mosaic_last_error() gives a thread-local message.
 *   - All enqueue calls are asynchronous on the given stream and never synchronise the
 *     host, except mosaic_stage_run, which blocks until the stage has finished.
 *   - Determinism contract: for fixed inputs, every output and gradient is bit-identical
 *     for every legal quota, mask layout and execution mode.
 */
#ifndef MOSAIC_H
#define MOSAIC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t mosaic_status;
enum {
  MOSAIC_OK = 0,
  MOSAIC_EINVAL = -1,       /* null pointer, bad size, bad enum */
  MOSAIC_EQUOTA = -2,       /* quota <= 0, beyond the device, overlapping, or not pooled */
  MOSAIC_ENOMEM = -3,       /* workspace too small / host allocation failed */
  MOSAIC_EUNSUPPORTED = -4, /* shape the kernels do not cover */
  MOSAIC_EHIP = -5          /* a HIP call failed; message holds the HIP error string */
};

enum { MOSAIC_F32 = 0, MOSAIC_BF16 = 1 };
enum { MOSAIC_ENCODER = 0, MOSAIC_DECODER = 1, MOSAIC_PROJECTOR = 2,
       MOSAIC_PATCH_STEM = 3, MOSAIC_TEXT_STEM = 4, MOSAIC_CONV_STEM = 5 };
enum { MOSAIC_NORM_NONE = 0, MOSAIC_LAYERNORM = 1, MOSAIC_RMSNORM = 2 };
enum { MOSAIC_GELU = 0, MOSAIC_SWIGLU = 1,
       MOSAIC_GELU_TANH = 2 };  /* tanh form of GELU: a layer variant, not used by the workloads */
/* How a quota's CUs are chosen.  STRIPED takes the same share of every XCD (keeps
 * workgroup dispatch balanced over XCDs).  XCD_ALIGNED fills whole XCDs first (would keep
 * a module's L2 private); quota and offset must then be multiples of the CUs per XCD.
 * On MI355X in its default partition mode one queue spans all XCDs and the driver
 * refuses a mask that leaves an XCD empty, so mosaic_stream_create returns
 * MOSAIC_EUNSUPPORTED for an XCD_ALIGNED quota below the whole device and MOSAIC_EQUOTA
 * for a STRIPED quota below one CU per XCD; mosaic_cu_mask_build computes both. */
enum { MOSAIC_STRIPED = 0, MOSAIC_XCD_ALIGNED = 1 };
enum { MOSAIC_COLOCATED = 0, MOSAIC_TIME_SLICED = 1, MOSAIC_CHAINED = 2 };

const char* mosaic_last_error(void);

/* ----------------------------------------------------------------------------- device */
/* Number of compute units of the current device (256 on MI355X), or a negative status. */
int32_t mosaic_device_cu_count(void);
/* Number of XCDs the CUs are spread over (8 on MI355X). */
int32_t mosaic_device_xcd_count(void);

/* ------------------------------------------------------- quota'd streams (Sec. 3.2) */
typedef struct mosaic_stream mosaic_stream;

/* Host-only: build the CU-mask words for `cu_quota` CUs starting at CU slot `cu_offset`
 * on a device of cu_total CUs in n_xcd XCDs.  Mask bit i addresses CU slot i/n_xcd of
 * XCD i%n_xcd (the driver deals mask bits round-robin over XCDs).  words must hold
 * ceil(cu_total/32) entries.  Runs without a GPU. */
mosaic_status mosaic_cu_mask_build(int32_t cu_total, int32_t n_xcd, int32_t cu_quota,
                                   int32_t cu_offset, int32_t layout,
                                   uint32_t* words, int32_t n_words);

/* A stream whose kernels run only on `cu_quota` CUs (the module's quota a_m times the
 * device's CU count); the quota is fixed for the stream's life.  The library owns the
 * object; destroy it with mosaic_stream_destroy.  cu_quota == device CU count and
 * cu_offset == 0 gives an unmasked stream. */
mosaic_status mosaic_stream_create(int32_t cu_quota, int32_t cu_offset, int32_t layout,
                                   mosaic_stream** out);
void*         mosaic_stream_native(const mosaic_stream*);   /* hipStream_t */
int32_t       mosaic_stream_quota(const mosaic_stream*);
int32_t       mosaic_stream_offset(const mosaic_stream*);
mosaic_status mosaic_stream_destroy(mosaic_stream*);

/* Stream pool: every (quota, offset, layout) a plan will use is reserved before training
 * starts; mosaic_stage_run only takes streams from the pool and never creates one
 * (stream creation on the critical path is what the pool exists to remove). */
mosaic_status mosaic_pool_reserve(int32_t cu_quota, int32_t cu_offset, int32_t layout);
mosaic_status mosaic_pool_get(int32_t cu_quota, int32_t cu_offset, int32_t layout,
                              mosaic_stream** out);          /* MOSAIC_EQUOTA if absent */
int64_t       mosaic_pool_creations(void);                   /* streams created so far */
mosaic_status mosaic_pool_clear(void);

/* Records, for each of n workgroups of a probe kernel on `stream`, where it ran:
 * out[3*i+0] = XCD id, out[3*i+1] = shader engine id, out[3*i+2] = CU id inside it.
 * out is a device buffer of 3*n int32.  Used to verify that a mask confines work. */
mosaic_status mosaic_probe_placement(const mosaic_stream* stream, int32_t n, int32_t* out);

/* --------------------------------------------------------------------------- modules */
/* Plain data, copied at create.  One descriptor covers the module families of the
 * workloads: ENCODER (ViT-style or audio encoder: pre-norm layers, LayerNorm, GELU MLP,
 * biases, full attention), DECODER (RMSNorm, SwiGLU MLP, no biases, causal attention),
 * PROJECTOR (Linear(in_dim->out_dim), GELU, Linear(out_dim->out_dim), biases),
 * PATCH_STEM (image [batch,3,side,side] -> unfold patch x patch -> Linear(in_dim->hidden)
 * + learned position table [seq,hidden]; in_dim = 3*patch*patch; for audio frames use
 * patch = 0 and x = [T,in_dim]), TEXT_STEM (rows [0,n_img) of each sample copied from
 * x = [batch*n_img, hidden], rows [n_img,seq) gathered from an embedding table
 * [vocab,hidden] by int32 ids bound with mosaic_module_bind_ids; ids outside the table are
 * clamped to its first / last row in both passes; per-sample image-token counts:
 * mosaic_module_bind_image_counts), CONV_STEM (a layer variant:
 * the two-convolution audio stem of speech encoders; x = [batch, 2*seq, in_dim] frames-major ->
 * Conv1d(in_dim->hidden, k=3, stride 1, pad 1), GELU, Conv1d(hidden->hidden, k=3, stride 2,
 * pad 1), GELU, + learned position table [seq,hidden]; convolution weights are stored
 * [3*C_in, C_out] with row index tap*C_in + channel). */
typedef struct {
  int32_t kind, dtype;
  int32_t layers, hidden, heads, mlp, batch, seq;
  int32_t norm, act, causal, bias;
  float   eps;
  int32_t in_dim, out_dim;
  int32_t vocab, n_img, patch;
  float   rope_base;   /* ENCODER / DECODER: > 0 turns on rotary position embedding of q and k
                          (pair (2i, 2i+1) of a head at position n turns by n * rope_base^(-2i/d));
                          0 = none, as in the workloads */
  int32_t kv_heads;    /* ENCODER / DECODER: key/value heads of grouped-query attention; must divide
                          heads; query head t attends to key/value head t / (heads/kv_heads); the
                          QKV weight is [hidden, (heads + 2*kv_heads) * d].  0 = heads (multi-head
                          attention, as in the workloads) */
} mosaic_module_desc;

typedef struct mosaic_module mosaic_module;

mosaic_status mosaic_module_create(const mosaic_module_desc*, mosaic_module** out);
mosaic_status mosaic_module_destroy(mosaic_module*);
/* Sizes of the buffers the caller must provide.  params and grads share one layout. */
size_t        mosaic_module_param_bytes(const mosaic_module*);
size_t        mosaic_module_workspace_bytes(const mosaic_module*);
size_t        mosaic_module_input_elems(const mosaic_module*);
size_t        mosaic_module_output_elems(const mosaic_module*);
/* Parameter layout: tensor i is `rows x cols` elements at element offset `offset`;
 * name (e.g. "L3.w_qkv") is written NUL-terminated into a 32-byte buffer.  The SwiGLU
 * gate and up matrices are stored side by side as one [hidden, 2*mlp] tensor "w_gu"
 * (gate in columns [0,mlp), up in [mlp,2*mlp)). */
int32_t       mosaic_module_tensor_count(const mosaic_module*);
mosaic_status mosaic_module_tensor_info(const mosaic_module*, int32_t i, char* name32,
                                        int64_t* offset, int64_t* rows, int64_t* cols);
/* Attach caller-owned device buffers.  workspace holds saved activations and scratch;
 * it must be 256-byte aligned and at least mosaic_module_workspace_bytes long. */
mosaic_status mosaic_module_bind(mosaic_module*, void* params, void* grads,
                                 void* workspace, size_t workspace_bytes);
mosaic_status mosaic_module_bind_ids(mosaic_module*, const int32_t* ids); /* TEXT_STEM */
/* TEXT_STEM with a different number of image tokens per sample at a fixed sequence length
 * (the paper pads or truncates every module input to a uniform length, Sec. 3.5, so shapes
 * never change): counts is a device int32 [batch]; sample b takes rows [0, counts[b]) from the
 * first counts[b] of its n_img image tokens in x and rows [counts[b], seq) from the embedding
 * table (counts are clamped to [0, n_img]).  With counts bound, ids must hold one id per
 * sequence position, [batch, seq] (read at positions counts[b] .. seq-1); in the backward pass
 * image tokens a sample did not use get zero gradient.  NULL unbinds: every sample then has
 * n_img image tokens and ids is [batch, seq - n_img] again. */
mosaic_status mosaic_module_bind_image_counts(mosaic_module*, const int32_t* counts);

/* Enqueue the forward pass: x [input_elems] -> y [output_elems]; activations needed by
 * the backward pass are kept in the workspace.  quota = number of CUs the persistent
 * grids are sized for (normally the stream's quota); stream may be NULL (default
 * stream, quota <= device CUs). */
mosaic_status mosaic_module_forward(mosaic_module*, int32_t quota, const mosaic_stream*,
                                    const void* x, void* y);
/* Enqueue the backward pass of the last forward: dy [output_elems] -> dx [input_elems]
 * (dx may be NULL for a first module), gradients of every parameter into `grads`
 * (overwritten, not accumulated). */
mosaic_status mosaic_module_backward(mosaic_module*, int32_t quota, const mosaic_stream*,
                                     const void* dy, void* dx);
/* One training step of a module on its quota'd stream: forward, then either the given
 * upstream gradient dy, or (dy == NULL) the mean-squared-error loss against `target`
 * whose value is written to *loss (device float) and whose gradient seeds the backward
 * pass; then backward.  Exactly one of dy / target is non-NULL. */
mosaic_status mosaic_module_step(mosaic_module*, int32_t quota, const mosaic_stream*,
                                 const void* x, const void* dy, const void* target,
                                 void* y, void* dx, float* loss);

/* Optimizer step over the module's flat parameter buffer (a layer-variant extra that makes
 * a training iteration complete): AdamW with decoupled weight decay and bias-corrected
 * moments, step counting from 1.  `state` is a caller-owned device buffer of
 * mosaic_module_optimizer_state_bytes: fp32 first moments, fp32 second moments and, when
 * use_master != 0, an fp32 master copy of the parameters (the caller initialises it from
 * the parameters; moments start at zero).  Reads `grads`, updates `params` in place. */
size_t        mosaic_module_optimizer_state_bytes(const mosaic_module*, int32_t use_master);
mosaic_status mosaic_module_adamw_step(mosaic_module*, int32_t quota, const mosaic_stream*,
                                       void* state, size_t state_bytes, int32_t use_master,
                                       float lr, float beta1, float beta2, float eps,
                                       float weight_decay, int64_t step);

/* ----------------------------------------------------------------- stages and plans */
/* A stage: n modules with their staged buffers.  In COLOCATED and TIME_SLICED mode the
 * modules are independent (each reads its own x and dy / target: the form in which the
 * paper profiles and colocates modules).  In CHAINED mode module i+1 consumes module
 * i's output: the caller sets x[i+1] == y[i] and dy[i] == dx[i+1]; only the last
 * module has a target; used for end-to-end gradient checks, not for timing. */
typedef struct {
  int32_t         n;
  mosaic_module** modules;
  const void**    x;
  const void**    dy;       /* entry may be NULL when target[i] is given */
  const void**    target;   /* entry may be NULL */
  void**          y;
  void**          dx;       /* entry may be NULL */
  float**         loss;     /* device floats; entry may be NULL when dy[i] is given */
} mosaic_stage;

/* The allocation plan A = {a_m}: CUs per module.  Modules with identical
 * (quota, offset) share one stream and run back to back in list order.  COLOCATED:
 * distinct (offset, quota) ranges must be disjoint and lie inside the device (Eq. 5).
 * TIME_SLICED / CHAINED: every module runs, one after another, on the stream given by
 * entry 0 (normally the full device). */
typedef struct {
  int32_t  n;
  const int32_t* cu_quota;
  const int32_t* cu_offset;
  int32_t  layout;
  int32_t  mode;
} mosaic_plan;

#define MOSAIC_MAX_STAGE_MODULES 8
typedef struct {
  float stage_ms;                                 /* first start to last end */
  float module_ms[MOSAIC_MAX_STAGE_MODULES];      /* each module's own span */
} mosaic_timing;

/* Host-only plan validation (what mosaic_stage_run checks first): quotas and offsets legal
 * for the mask layout, distinct CU ranges disjoint and inside the device (Eq. 5), and, in
 * COLOCATED mode, no more distinct streams than the process has hardware queues
 * (mosaic_device_hw_queues): streams that share a queue run one after the other, which would
 * silently serialise the stage; such a plan returns MOSAIC_EQUOTA. */
mosaic_status mosaic_plan_validate(const mosaic_plan*, int32_t cu_total, int32_t n_xcd);
/* Streams the plan runs side by side: distinct (quota, offset) pairs in COLOCATED mode, else 1. */
int32_t       mosaic_plan_stream_count(const mosaic_plan*);
/* Hardware queues a process may hold (the runtime's GPU_MAX_HW_QUEUES setting, default 4). */
int32_t       mosaic_device_hw_queues(void);
/* Run one forward+backward of every module of the stage under the plan; blocks until
 * done and fills `out` (may be NULL) from device events. */
mosaic_status mosaic_stage_run(const mosaic_stage*, const mosaic_plan*, mosaic_timing* out);

/* Host-only: choose quotas from measured time-vs-CU curves.  times[m*n_points + p] is
 * module m's time at cu_points[p] CUs.  Minimises the maximum over modules (Eq. 4)
 * subject to the chosen quotas summing to at most cu_total (Eq. 5) by exhaustive search;
 * ties go to the lexicographically smallest quota tuple.  Writes n_modules quotas. */
mosaic_status mosaic_plan_choose(int32_t n_modules, int32_t n_points, const int32_t* cu_points,
                                 const float* times, int32_t cu_total,
                                 int32_t* quota_out, float* time_out);

/* ------------------------------------- performance-model correction (Sec. 3.3, Eq. 7-8) */
/* Host-only.  A module that shares its GPU is delayed by
 *   delta = e1 + e2 * sum_m B_m + e3 * prod_m B_m                                  (Eq. 8)
 * over the memory-bandwidth utilisations B_m in [0,1] of ALL modules on that GPU (itself
 * included); its rectified time is the grid-sampled time plus delta (Eq. 7; one GPU, so
 * the maximum over GPUs has one term).  mosaic_interference_delta evaluates Eq. 8 for k
 * modules (NaN on null arguments). */
enum { MOSAIC_INTERFERENCE_ADDITIVE = 0,    /* e3 = 0: the additive-only comparison model */
       MOSAIC_INTERFERENCE_COMPOSITE = 1 }; /* Eq. 8 */
double        mosaic_interference_delta(const double* e /*[3]*/, int32_t k, const double* bw);
/* Ordinary least-squares fit of (e1,e2,e3) to n_obs measured delays.  Observation i lists
 * the utilisations of the group_size[i] modules that shared the GPU, concatenated in bw;
 * delta_ms[i] is the delay measured for one of them.  e_out receives 3 doubles (e3 = 0 for
 * ADDITIVE); *r2_out (may be NULL) the coefficient of determination of the fit.
 * MOSAIC_EINVAL when the observations do not determine the coefficients. */
mosaic_status mosaic_interference_fit(int32_t n_obs, const int32_t* group_size,
                                      const double* bw, const double* delta_ms,
                                      int32_t model, double* e_out, double* r2_out);

/* ------------------------------------------ mapping solver on one GPU (Sec. 3.4, Alg. 1) */
/* Host-only.  The job is a DAG of n_modules modules (edges = pairs (src, dst): dst
 * consumes src's output).  times[m*n_points + p] is module m's measured time in ms on
 * cu_points[p] CUs (the scaling surface of Sec. 3.3 on one GPU); bw, if given, holds the
 * bandwidth utilisation measured at the same points and e the fitted coefficients of
 * Eq. 8 (both or neither); a stage of two or more modules is then charged Eq. 8's delay,
 * a module alone is not.  At most 16 modules and 16 quota levels. */
/* How the fitted expression enters a module's time.  ABSOLUTE is the paper's: one delay in
 * ms per GPU, computed over all its modules, added to each (Eq. 7-8).  PEER_RELATIVE is
 * this build's addition for a GPU whose co-runners slow each other through a shared power
 * budget: module m's time is multiplied by 1 + e1 + e2 * sum B + e3 * prod B taken over the
 * OTHER modules of the stage (fit the coefficients to relative delays and peers' values
 * with the same mosaic_interference_fit). */
enum { MOSAIC_DELAY_ABSOLUTE = 0, MOSAIC_DELAY_PEER_RELATIVE = 1 };
typedef struct {
  int32_t        n_modules, n_edges;
  const int32_t* edges;        /* 2*n_edges entries */
  int32_t        n_points;
  const int32_t* cu_points;
  const double*  times;
  const double*  bw;           /* may be NULL */
  const double*  e;            /* 3 doubles, NULL iff bw is NULL */
  int32_t        cu_total;
  int32_t        delay_form;   /* MOSAIC_DELAY_ABSOLUTE (Eq. 7-8) | MOSAIC_DELAY_PEER_RELATIVE */
} mosaic_planner_problem;
typedef struct { int64_t stage_evals, cache_hits, pruned, rounds; } mosaic_planner_stats;
enum { MOSAIC_PLANNER_EARLY_PRUNE = 1, MOSAIC_PLANNER_CACHE = 2 };

/* StageEval: the allocation of one quota level per module of the stage `module_mask`
 * (bit m = module m) that minimises the slowest module's time (Eq. 4) with the quotas
 * summing to at most cu_total (Eq. 5).  Without interference terms: binary search on a
 * target latency with a feasibility test per trial; with them: every level tuple within
 * the budget is visited.  quota_out[m] = CUs of member m (0 for non-members);
 * *t_out = stage time in ms, +infinity when the stage does not fit.  Ties go to the
 * lexicographically smallest tuple of level indices. */
mosaic_status mosaic_stage_eval(const mosaic_planner_problem*, uint32_t module_mask,
                                int32_t* quota_out, double* t_out);
/* Alg. 1: every module starts as its own stage in a topological order; each round merges
 * the pair of stages with the largest strictly positive saving T_x + T_y - T_xy among the
 * pairs whose merge keeps the stage order acyclic; stops when no merge saves time.
 * flags: MOSAIC_PLANNER_EARLY_PRUNE skips pairs that cannot beat the round's best saving,
 * MOSAIC_PLANNER_CACHE remembers StageEval results per stage composition; neither changes
 * the result.  stage_of[m] = index of m's stage in execution order, quota_of[m] = its
 * CUs, *n_stages (may be NULL), *t_iter = sum of stage times (Eq. 1), stats may be NULL.
 * MOSAIC_EINVAL for a cyclic edge list. */
mosaic_status mosaic_planner_solve(const mosaic_planner_problem*, int32_t flags,
                                   int32_t* stage_of, int32_t* quota_of, int32_t* n_stages,
                                   double* t_iter, mosaic_planner_stats* stats);

/* ------------------------------------------------ single operations (kernel level) */
/* Each enqueues one operation on `stream` (hipStream_t, NULL = default) with persistent
 * grids sized for `quota` CUs.  They are what the module steps are made of and exist at
 * the boundary for kernel-level parity tests and roofline measurement. */

/* Y[T,n] = X[T,k] W[k,n] (+ bias[n]) (+ R[T,n]).  bias, R may be NULL. */
mosaic_status mosaic_op_linear_fwd(void* stream, int32_t quota, int32_t dtype,
                                   int64_t T, int64_t k, int64_t n, const void* X,
                                   const void* W, const void* bias, const void* R, void* Y);
/* dX[T,k] = dY[T,n] W[k,n]^T (+ R[T,k]). */
mosaic_status mosaic_op_linear_dgrad(void* stream, int32_t quota, int32_t dtype,
                                     int64_t T, int64_t k, int64_t n, const void* dY,
                                     const void* W, const void* R, void* dX);
/* dW[k,n] = X[T,k]^T dY[T,n];  db[n] = column sums of dY (db may be NULL).
 * scratch: 16-byte aligned device buffer of at least
 * mosaic_op_linear_wgrad_scratch_bytes(T,k,n); it holds the fp32 pieces of the output
 * tiles whose long contraction is split (which tiles and into how many pieces depends on
 * the shape alone: all of them when the output has few tiles, else the tiles that do not
 * fill a whole round of the device), and the partial column sums. */
mosaic_status mosaic_op_linear_wgrad(void* stream, int32_t quota, int32_t dtype,
                                     int64_t T, int64_t k, int64_t n, const void* X,
                                     const void* dY, void* dW, void* db, void* scratch);
size_t        mosaic_op_colsum_scratch_bytes(int64_t n);
size_t        mosaic_op_linear_wgrad_scratch_bytes(int64_t T, int64_t k, int64_t n);

/* qkv [B*N, 3h], row = [q | k | v], head t in columns t*d..; O [B*N, h]; lse [B,H,N] f32. */
mosaic_status mosaic_op_attention_fwd(void* stream, int32_t quota, int32_t dtype,
                                      int32_t B, int32_t N, int32_t H, int32_t d,
                                      int32_t causal, const void* qkv, void* O, float* lse);
/* dqkv [B*N, 3h] from dO, O, lse.  delta: device scratch of B*H*N floats. */
mosaic_status mosaic_op_attention_bwd(void* stream, int32_t quota, int32_t dtype,
                                      int32_t B, int32_t N, int32_t H, int32_t d,
                                      int32_t causal, const void* qkv, const void* O,
                                      const float* lse, const void* dO, void* dqkv,
                                      float* delta);

/* Grouped-query attention: qkv [B*N, (H + 2*Hkv)*d], row = [q (H heads) | k (Hkv heads) | v (Hkv
 * heads)], Hkv divides H, query head t attends to key/value head t / (H/Hkv); dqkv has the
 * same layout and a key/value head's gradient sums over its group in a fixed order. */
mosaic_status mosaic_op_attention_gqa_fwd(void* stream, int32_t quota, int32_t dtype,
                                          int32_t B, int32_t N, int32_t H, int32_t Hkv, int32_t d,
                                          int32_t causal, const void* qkv, void* O, float* lse);
mosaic_status mosaic_op_attention_gqa_bwd(void* stream, int32_t quota, int32_t dtype,
                                          int32_t B, int32_t N, int32_t H, int32_t Hkv, int32_t d,
                                          int32_t causal, const void* qkv, const void* O,
                                          const float* lse, const void* dO, void* dqkv,
                                          float* delta);

/* y = norm(x) * gamma (+ beta).  norm = MOSAIC_LAYERNORM | MOSAIC_RMSNORM.
 * stats [T,2] f32 receives (mean, rstd) (mean = 0 for RMSNorm). */
mosaic_status mosaic_op_norm_fwd(void* stream, int32_t quota, int32_t dtype, int32_t norm,
                                 int64_t T, int64_t h, float eps, const void* x,
                                 const void* gamma, const void* beta, void* y, float* stats);
/* dx = (R +) norm backward; dgamma, dbeta column reductions in fixed order.
 * scratch: at least mosaic_op_norm_bwd_scratch_bytes(h). */
mosaic_status mosaic_op_norm_bwd(void* stream, int32_t quota, int32_t dtype, int32_t norm,
                                 int64_t T, int64_t h, const void* x, const void* gamma,
                                 const float* stats, const void* dy, const void* R,
                                 void* dx, void* dgamma, void* dbeta, void* scratch);
size_t        mosaic_op_norm_bwd_scratch_bytes(int64_t h);
/* The same operation for callers that cannot allocate device memory or bring a scratch buffer
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * kernels, same bits, but the partial column sums live in a 20 MiB array built into the
 * library's device code (one copy per GPU, held until the process ends), so the call allocates
 * nothing.  Rows of up to mosaic_op_norm_bwd_static_max_h() = 5120 elements; wider rows return
 * MOSAIC_EUNSUPPORTED before anything is launched.  Nothing in the array has to start at zero
 * (every partial sum that is read has been written by the same call).  All calls on one GPU
 * share the array: calls that overlap in time on one GPU (different streams) race; calls on one
 * stream, or otherwise ordered, are safe. */
mosaic_status mosaic_op_norm_bwd_static(void* stream, int32_t quota, int32_t dtype, int32_t norm,
                                        int64_t T, int64_t h, const void* x, const void* gamma,
                                        const float* stats, const void* dy, const void* R,
                                        void* dx, void* dgamma, void* dbeta);
size_t        mosaic_op_norm_bwd_static_max_h(void);

/* a = gelu(z) ; dz = da * gelu'(z)   (exact erf form), elementwise over n elements. */
mosaic_status mosaic_op_gelu_fwd(void* stream, int32_t quota, int32_t dtype, int64_t n,
                                 const void* z, void* a);
mosaic_status mosaic_op_gelu_bwd(void* stream, int32_t quota, int32_t dtype, int64_t n,
                                 const void* z, const void* da, void* dz);
/* The tanh form: 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))). */
mosaic_status mosaic_op_gelu_tanh_fwd(void* stream, int32_t quota, int32_t dtype, int64_t n,
                                      const void* z, void* a);
mosaic_status mosaic_op_gelu_tanh_bwd(void* stream, int32_t quota, int32_t dtype, int64_t n,
                                      const void* z, const void* da, void* dz);
/* gu [T,2f] = [gate | up];  a[T,f] = silu(gate)*up;  dgu [T,2f] = [dgate | dup]. */
mosaic_status mosaic_op_swiglu_fwd(void* stream, int32_t quota, int32_t dtype, int64_t T,
                                   int64_t f, const void* gu, void* a);
mosaic_status mosaic_op_swiglu_bwd(void* stream, int32_t quota, int32_t dtype, int64_t T,
                                   int64_t f, const void* gu, const void* da, void* dgu);
/* A linear layer followed by its activation, as the MLP blocks of the modules use it (the paper
 * schedules whole modules, Sec. 3.1; the layer arithmetic is this build's): Z[T,n] = X[T,k]
 * W[k,n] (+ bias[n], may be NULL) and A = act(Z).  act = MOSAIC_GELU or MOSAIC_GELU_TANH: A is
 * [T,n].  act = MOSAIC_SWIGLU: Z = [gate | up] halves of n/2 columns, A[T,n/2] = silu(gate)*up.
 * Z is kept because the backward pass needs it.  All pointers are device memory owned by the
 * caller.  For bf16 operands whose sizes and alignment suit the matrix-core kernel (SwiGLU: n
 * a multiple of 256) the activation is applied in that kernel's epilogue and no second pass is
 * launched; otherwise the product is followed by the elementwise kernel.  Both roads give the
 * same bits.  MOSAIC_EINVAL for an unknown activation, negative sizes or an odd n with SwiGLU. */
mosaic_status mosaic_op_linear_act_fwd(void* stream, int32_t quota, int32_t dtype, int32_t act,
                                       int64_t T, int64_t k, int64_t n, const void* X,
                                       const void* W, const void* bias, void* Z, void* A);
/* loss = mean((y-target)^2) -> *loss (device f32); dy = 2 (y-target)/n.
 * scratch: at least mosaic_op_mse_scratch_bytes(). */
mosaic_status mosaic_op_mse(void* stream, int32_t quota, int32_t dtype, int64_t n,
                            const void* y, const void* target, void* dy, float* loss,
                            void* scratch);
size_t        mosaic_op_mse_scratch_bytes(void);


/* Rotary position embedding.  table: device buffer of mosaic_op_rope_table_bytes(N, d) that
 * mosaic_op_rope_table fills with (cos, sin)(n * base^(-2i/d)) for n < N, i < d/2 (angles
 * formed in double).  mosaic_op_rope rotates, in place, pair (2i, 2i+1) of every head of
 * the q and k parts of qkv [B*N, 3*H*d] by the angle of (row's position in its sample, i);
 * direction = +1 forward, -1 the transposed rotation (gradients back to unrotated q, k). */
size_t        mosaic_op_rope_table_bytes(int32_t N, int32_t d);
mosaic_status mosaic_op_rope_table(void* stream, int32_t quota, int32_t N, int32_t d, float base,
                                   void* table);
mosaic_status mosaic_op_rope(void* stream, int32_t quota, int32_t dtype, int32_t B, int32_t N,
                             int32_t H, int32_t d, int32_t direction, void* qkv,
                             const void* table);

/* AdamW over n elements: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2;
 * p -= lr * ( (m / (1-b1^step)) / (sqrt(v / (1-b2^step)) + eps) + weight_decay * p ).
 * params, grads in `dtype`; m, v and master (may be NULL) fp32; master, when given, is the
 * value that is updated and params receives its rounding.  n must be a multiple of 4 and
 * all buffers 16-byte aligned (MOSAIC_EUNSUPPORTED / MOSAIC_EINVAL otherwise); step counts
 * from 1. */
mosaic_status mosaic_op_adamw(void* stream, int32_t quota, int32_t dtype, int64_t n, void* params,
                              const void* grads, float* m, float* v, float* master, float lr,
                              float beta1, float beta2, float eps, float weight_decay,
                              int64_t step);

#ifdef __cplusplus
}
#endif
#endif /* MOSAIC_H */
