/*
 * karma.h -- C ABI of the MI355X out-of-core training-step library.
 *
 * The library runs one training step of a layer stack whose activations do not fit a
 * configured HBM budget, following KARMA (SC20): a CPU planner chooses per layer between
 * keeping, swapping to host and dropping-and-recomputing (Sec. III-E capacity-based
 * strategy, Sec. III-F interleaved recompute, Fig. 4 optimisation problems), a schedule
 * generator turns the choice into stages (Algorithm 1), and a three-stream executor
 * overlaps layer compute with swap-out and prefetch (Fig. 2(c)), updating fp32 master
 * weights on the host (Sec. III-G, pipeline stage 5).
 *
 * Conventions for every entry point
 *   - returns a karma_status (0 = ok, negative = error); never throws, never aborts;
 *     karma_last_error() gives a text for the last failure of a context.
 *   - pointers named *_host are host memory, *_dev are device (HBM) memory; output
 *     buffers are allocated and owned by the caller; inputs are only read during the call.
 *   - a layer record stands for one "block" of the paper (footnote in Sec. III-B).
 *   - all times are integer nanoseconds, all sizes integer bytes.
 *   - a context is not thread-safe; calls on one context must not overlap.
 */
#ifndef KARMA_H
#define KARMA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct karma_ctx karma_ctx;

typedef enum {
  KARMA_OK = 0,
  KARMA_E_INVAL = -1,   /* bad argument (null pointer, bad shape, invalid action vector) */
  KARMA_E_BUDGET = -2,  /* no assignment fits the budget (constraint 9.4 cannot be met) */
  KARMA_E_OOM = -3,     /* caller's buffer or arena too small */
  KARMA_E_HIP = -4,     /* a HIP runtime call failed */
  KARMA_E_STATE = -5,   /* call out of order (step before plan, ...) */
  KARMA_E_HOSTMEM = -6  /* pinned host allocation failed */
} karma_status;

/* Per-layer action.  x_i is the layer's input tensor, "internals" what backward needs
 * besides x_i.
 *   KEEP      both stay in HBM (the resident tail of Sec. III-E)
 *   SWAP      both copied to host right after F_i, copied back before B_i
 *   RC_KEEP   internals dropped after F_i and recomputed before B_i; x_i stays (checkpoint)
 *   RC_SWAP   as RC_KEEP, but the checkpoint x_i itself is swapped
 *   RC_CHAIN  x_i and internals dropped; recomputed by the chain that starts at the
 *             nearest preceding RC_KEEP / RC_SWAP (the set "Delta" of Eq. 10)
 * RC_CHAIN is valid only directly after RC_KEEP, RC_SWAP or RC_CHAIN, never at layer 0. */
typedef enum { KARMA_KEEP = 0, KARMA_SWAP = 1, KARMA_RC_KEEP = 2, KARMA_RC_SWAP = 3, KARMA_RC_CHAIN = 4 } karma_action;

/* Cost-model inputs (Sec. III-C compute cost, Sec. III-D memory per variable type). */
typedef struct {
  int64_t tf_ns, tb_ns, trc_ns; /* forward, backward time; trc: recomputing the layer's internals without its output
                                   (the last layer of a recomputed run: its output still exists as the next
                                   layer's input); a layer inside a run is re-run whole and costs tf */
  uint64_t sav_bytes;           /* internals needed by backward, excluding x_i */
  uint64_t out_bytes;           /* output = input of the next layer (x_0 is the step input
                                   and lives in the fixed region) */
  uint64_t ws_bytes;            /* transient workspace of any one op of the layer */
  uint64_t w_bytes;             /* weights streamed over the host link for this layer (Sec. III-G:
                                   a swapped block carries its weights); 0 = weights resident,
                                   their bytes are part of the fixed region */
  uint64_t g_bytes;             /* gradients of those weights (ignored when w_bytes is 0) */
  int64_t th_ns;                /* host optimiser time for the layer's parameters (Sec. III-G, stage 5: the
                                   weights are updated on the CPU); 0 = no host update is priced */
  uint64_t hg_bytes;            /* resident weights: gradients that leave for the host after B_i */
  uint64_t hw_bytes;            /* resident weights: new weights that come back after the update (a streamed
                                   layer's gradients are g_bytes, its new weights stay on the host) */
} karma_layer_cost;

typedef struct {
  uint64_t bw_h2d, bw_d2h; /* bytes per second, one measured figure per direction (Eq. 4) */
  int64_t lat_ns;          /* fixed cost per copy */
  uint64_t bw_h2d_loaded, bw_d2h_loaded; /* the same while the other direction copies and the host optimiser
                                            streams through host memory: the price of every copy issued after
                                            the forward pass of a step with host updates; 0 = as above */
} karma_link;

typedef struct {
  int64_t t_ns;      /* loss op (forward and gradient w.r.t. its input) */
  uint64_t ws_bytes; /* its workspace */
  int64_t th_ns;     /* host optimiser time, gradient and weight bytes of the parameters that belong */
  uint64_t hg_bytes; /* to the loss record (a final normalisation, a classifier), as for a layer */
  uint64_t hw_bytes;
} karma_loss_cost;

typedef struct {
  int64_t makespan_ns;  /* end of the last op on any queue */
  int64_t stall_ns;     /* idle time of the compute queue (Eq. 1 denominator minus busy) */
  int64_t busy_ns;      /* compute-queue busy time, recompute included */
  int64_t recompute_ns; /* part of busy_ns spent recomputing */
  uint64_t peak_bytes;  /* fixed + high-water mark of the arena */
  uint64_t bytes_d2h, bytes_h2d; /* what the plan moves: swapped activations, streamed weights and their gradients
                                    (gradients and weights of resident layers, the same under every plan, not counted) */
  int64_t host_busy_ns; /* host optimiser queue: sum of the updates, */
  int64_t host_end_ns;  /* and the end of the last one */
} karma_plan_summary;

/* One op of the simulated/executed timeline, in issue order.
 * kind: 'F' forward, 'B' backward, 'R' recompute, 'L' loss, 'O' swap-out, 'I' swap-in,
 *   'W' copy-in of a layer's streamed weights, 'G' copy-out of their gradients, 'H' (models with connections
 *   between non-consecutive layers only; no time passes) the buffer in which the readers of x_layer leave their
 *   gradient for it starts to exist: issued right before the first backward op that writes it.
 * off[]: arena offsets (relative to the end of the fixed region, -1 = none) of what the
 *   op allocates: F {x_{i+1}, internals, workspace}; R {internals, x_{i+1}, workspace};
 *   B {dx, workspace, gradients of streamed weights}; L {dx, workspace, -1};
 *   I {x_i, internals, -1}; W {weights, -1, -1}; H {that buffer, -1, -1}; O and G {-1,-1,-1}. */
typedef struct {
  uint8_t kind;
  uint32_t layer;
  int64_t start_ns, end_ns;
  int64_t off[3];
} karma_op;

/* ---- planner: pure CPU functions, no GPU needed -------------------------------- */

/* Timeline of one step under a given action vector (three in-order queues and a
 * two-ended first-fit arena of budget - fixed bytes; constraint 9.4 is checked at every
 * allocation).  weights_kept (host, n_layers bytes, may be NULL = all 0) says per layer
 * with streamed weights whether they stay in HBM from F_i to B_i (1) or are freed after
 * F_i and copied in again before R_i / B_i (0); weights are copied in one layer ahead of
 * the forward pass and queued with the swap-ins, in order of need, during backward;
 * gradients leave right after B_i (Sec. III-G, pipeline stage 3).  Host optimiser (stage 5), a fourth in-order
 * queue: a layer's update (th_ns) starts when its gradients have landed on the host and the updates before it,
 * in the order of the backward ops, are done; new weights of a resident layer go back on the host-to-device
 * queue behind every copy of the step's own program; the makespan ends with the last update and weight copy
 * (one step in isolation).  ops_out may be NULL;
 * otherwise *n_ops_inout holds its capacity on entry and the number of ops on return
 * (KARMA_E_OOM if too small: at most 8*n+2 are written).
 * Errors: KARMA_E_INVAL (invalid vector), KARMA_E_BUDGET (does not fit). */
int karma_simulate(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                   const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                   const uint8_t* actions, const uint8_t* weights_kept, karma_plan_summary* summary_out,
                   karma_op* ops_out, uint32_t* n_ops_inout);

/* The planner (Sec. III-E capacity rule, Eq. 10.1 recompute marking, makespan
 * refinement by local search over the simulator, which starts with a feasibility phase when
 * none of the start patterns fits: an assignment that does not fit is measured by how many
 * compute ops its timeline completes before an allocation fails; then, for layers with streamed weights,
 * the capacity rule applied to weights: going down from the last layer, a layer keeps
 * its weights between F_i and B_i while that fits and does not lengthen the step).
 * Writes n_layers actions and, when weights_kept_out is not NULL, n_layers bytes.
 * Errors: KARMA_E_BUDGET when nothing fits. */
int karma_plan_pure(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                    const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                    uint8_t* actions_out, uint8_t* weights_kept_out, karma_plan_summary* summary_out);

/* The planner with the block granularity chosen as well (Sec. III-E/F: the first tier of the optimisation groups
 * layers into blocks that are kept, swapped or recomputed as a whole).  For group sizes 1, 2, 3, 4, 6, 8 up to
 * max_group, consecutive layers are merged, the merged stack is planned, the block-level plan is expanded to
 * per-layer actions (a recomputed block checkpoints its first member's input and chains the rest) and priced by the
 * per-layer simulator; the cheapest wins (the smaller size on ties), so the result is never worse than
 * karma_plan_pure.  *group_out (may be NULL): the size chosen.  Outputs and errors as karma_plan_pure. */
int karma_plan_grouped_pure(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                            const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes, uint32_t max_group,
                            uint8_t* actions_out, uint8_t* weights_kept_out, karma_plan_summary* summary_out,
                            uint32_t* group_out);

/* ---- the same three calls for a model with connections between non-consecutive layers
 * (Sec. III-F.3: residual connections that cross blocks, connections from the contracting to
 * the expansive path of a fully convolutional network).  skips (host, n_skips entries, may be
 * NULL when n_skips is 0): the output of layer src, which is the input x_s of layer s = src + 1,
 * is read again by layer dst >= src + 2, in its forward and in its backward pass.  x_s follows
 * the action of layer s: kept, or kept as a recompute checkpoint, it is still there; swapped
 * out, it needs a premature swap-in on the host-to-device queue before F_dst (queued one layer
 * ahead of its first reader when memory allows, else at the reader, which waits) and then stays
 * until B_s, whose own swap-in brings only the internals; it cannot be KARMA_RC_CHAIN (a chained
 * layer drops its input).  B_dst leaves a gradient for x_s that is held, from the first such
 * backward, until B_s adds it to its own.  The planner searches two more neighbourhoods when
 * connections are present (four consecutive layers; one layer forced and the rest descending).
 * karma_simulate_graph writes at most 8*n_layers + 2 + 2*n_skips ops.
 * Errors as the plain calls; KARMA_E_INVAL also for a connection with dst < src + 2 or
 * dst >= n_layers, and for an action vector that chains a read-again input. */
typedef struct {
  uint32_t src, dst;
} karma_skip;
int karma_simulate_graph(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                         const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                         const karma_skip* skips, uint32_t n_skips, const uint8_t* actions,
                         const uint8_t* weights_kept, karma_plan_summary* summary_out, karma_op* ops_out,
                         uint32_t* n_ops_inout);
int karma_plan_graph(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                     const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                     const karma_skip* skips, uint32_t n_skips, uint8_t* actions_out, uint8_t* weights_kept_out,
                     karma_plan_summary* summary_out);
/* Block level: a connection is kept between blocks when its source is the last member of its block
 * and its reader sits at least two blocks on; every expansion is priced per layer with all of them. */
int karma_plan_grouped_graph(const karma_layer_cost* layers, uint32_t n_layers, const karma_link* link,
                             const karma_loss_cost* loss, uint64_t budget_bytes, uint64_t fixed_bytes,
                             const karma_skip* skips, uint32_t n_skips, uint32_t max_group, uint8_t* actions_out,
                             uint8_t* weights_kept_out, karma_plan_summary* summary_out, uint32_t* group_out);

/* Algorithm 1's output in the paper's notation ("F1 -> F2||S1^out -> ...", layers
 * 1-based, recompute printed as F; copies of streamed weights and of their gradients
 * print as W<i>^in and G<i>^out).  Writes a NUL-terminated string; KARMA_E_OOM if
 * buf_len is too small. */
int karma_stage_string(const karma_op* ops, uint32_t n_ops, char* buf, size_t buf_len);

/* ---- model and context ---------------------------------------------------------- */

/* KARMA_MODEL_WRN: a wide residual network (the WRN-28-10 row of Table III).  width = channels of the first
 * group (160 = 16 * 10), stage_blocks[0..2] = basic blocks per group (4, 4, 4; stage_blocks[3] must be 0), group k
 * has width << k channels and starts with stride 2 (group 0: 1); seq = image size (32, a multiple of 4); vocab =
 * classes, a multiple of 8 (10 classes are stored as 16: rows 10..15 of the fully connected weight zero and their
 * bias -30000, so that their probabilities and gradients are exactly zero).  Records: 0 = the 3x3 convolution to 16
 * channels (one tensor: its weight, 3 image channels stored as 8); 1.. = pre-activated basic blocks (tensors: BN1
 * gain, BN1 shift, first 3x3 weight, BN2 gain, BN2 shift, second 3x3 weight and, where the shape changes, the 1x1
 * shortcut weight, which convolves the activated input); loss record: batch norm, ReLU, global average pooling, fully
 * connected layer, mean cross entropy (tensors: gain, shift, weight, bias).  No dropout.  Inputs as for the CNN. */
/* KARMA_MODEL_UNET: a fully convolutional network (the U-Net row of Table III; Sec. III-F.3: connections from the
 * contracting to the expansive path).  n_layers = depth D (1..6), width = channels of level 0 (64), level l has
 * width << l channels at (seq >> l)^2 pixels; seq = image size, a multiple of 2^D; vocab = classes stored, 8 or 16
 * (two classes are stored as 8: rows 2..7 of the classifier weight zero and their bias -30000).  Records 0..D:
 * contracting levels (2x2 max pooling of the record above, except record 0; then twice: 3x3 convolution with padding
 * 1 and no bias, batch normalisation, ReLU; tensors: first weight [C][3][3][c_in], gain, shift, second weight, gain,
 * shift; the one image channel is stored as 8).  Records D+1..2D: expansive levels D-1..0 (2x2 stride-2
 * up-convolution [c_below][2][2][C] without bias, then the same two convolutions, the first of them over the
 * contracting record's output followed by the up-convolution's result; tensors: up-convolution weight, the first
 * weight's half for the contracting output [C][3][3][C], its half for the up-convolution's result [C][3][3][C],
 * gain, shift, second weight, gain, shift).  Record 2D - l reads the output of record l again (karma_model_skips).
 * Loss record: 1x1 classifier with bias and the mean cross entropy over all pixels (tensors: weight [classes][width],
 * bias).  Inputs: fp32 images [batch][seq][seq] (one channel), int32 labels [batch][seq][seq].  stream_weights
 * must be 0. */
typedef enum {
  KARMA_MODEL_MLP = 1, KARMA_MODEL_GPT = 2, KARMA_MODEL_CNN = 3, KARMA_MODEL_WRN = 4, KARMA_MODEL_UNET = 5
} karma_model_kind;
/* SGD with momentum: buf = beta1 * buf + g; w -= lr * buf (no dampening, no Nesterov) */
typedef enum { KARMA_OPT_SGD = 1, KARMA_OPT_ADAM = 2, KARMA_OPT_SGD_MOMENTUM = 3 } karma_opt_kind;

typedef struct {
  uint32_t kind;      /* karma_model_kind */
  uint32_t n_layers;  /* MLP: Linear+ReLU layers; GPT: transformer blocks; UNET: depth; CNN, WRN: ignored */
  uint32_t width;     /* MLP width / GPT hidden size / CNN: bottleneck width of the first stage (64) / WRN: channels of
                         the first group (160) */
  uint32_t batch;
  uint32_t seq;       /* GPT: sequence length; CNN: image height = width (multiple of 32); WRN: the same (multiple of 4) */
  uint32_t n_heads;   /* GPT only; width / n_heads must be 64, 128 or 152 */
  uint32_t ffn;       /* GPT only */
  uint32_t vocab;     /* GPT: vocabulary; CNN, WRN: number of classes (multiple of 8) */
  uint32_t stream_weights; /* 1: the weights of every MLP layer / transformer block live in
                              pinned host memory and are streamed through the arena around the
                              layer's ops, their gradients streamed out after its backward
                              (Sec. III-G); embeddings and the final LayerNorm stay resident.
                              2: the same, and a block's gradients land in the pinned buffer its
                              weights were copied from (the host update replaces each gradient by
                              the new weight): half the pinned memory.  The gradients then leave the
                              device only in steps run with KARMA_STEP_APPLY_OPTIMIZER, and
                              karma_get_grad on such a block returns KARMA_E_STATE.  Tensors whose
                              gradient is wider than the weight (fp32 gradients of bf16 vectors)
                              keep a small gradient buffer of their own */
  uint32_t stage_blocks[4]; /* CNN only: bottleneck blocks per stage (ResNet-200: 3, 24, 36, 3).
                               Stage k has bottleneck width `width << k` and 4x that many output
                               channels; its first block carries stride 2 (stage 0: 1) on the 3x3
                               convolution and a projection shortcut.  Stem: 7x7 stride-2
                               convolution to `width` channels, batch norm, ReLU, 3x3 stride-2 max
                               pooling; head: global average pooling, fully connected layer, mean
                               cross entropy.  Inputs: fp32 images [batch][seq][seq][3]; labels int32. */
  uint32_t split_blocks;    /* GPT only, 1: every transformer block is two plannable records, its attention half
                               (LayerNorm, QKV projection, attention, output projection, residual add) and
                               its feed-forward half (LayerNorm, FC1, GELU, FC2, residual add), so that the
                               planner chooses per half (Sec. III-E: a block is any run of consecutive
                               layers).  The same kernels run in the same order: results equal those of
                               whole blocks bit for bit */
} karma_model_desc;

typedef struct {
  uint32_t optimizer; /* karma_opt_kind */
  float lr, beta1, beta2, eps;
  uint32_t host_threads; /* worker threads of the host optimiser (0 = 1) */
  uint32_t device_update_first; /* n: the parameters of records 0 .. n-1 (those with resident weights) keep their fp32
                                   master copy and optimiser state in HBM, inside the fixed region (12 bytes per
                                   parameter, charged to the budget), and are updated there by a kernel right after the
                                   record's backward.  The first records are the last the backward pass completes and the
                                   first the next forward pass reads: on the host their update (gradients out, update,
                                   weights back) is a tail nothing can hide.  Every other record is updated on the host as
                                   Sec. III-G describes.  Same arithmetic as the host update */
} karma_config;

/* Number of plannable layer records of a model (MLP: n_layers; GPT: n_layers + 1, record
 * 0 being the embedding, or 2 n_layers + 1 with split_blocks: block k is then records 2k + 1
 * (attention half: tensors LN1 gain, LN1 shift, Wqkv, bqkv, Wo, bo) and 2k + 2 (feed-forward half:
 * LN2 gain, LN2 shift, W1, b1, W2, b2); CNN: 1 + sum of stage_blocks, record 0 being the stem; WRN: 1 + sum of
 * stage_blocks[0..2], record 0 being the first convolution) and
 * of parameter tensors of record `layer`. */
int karma_model_layers(const karma_model_desc* desc, uint32_t* n_out);

/* The model's connections between non-consecutive records (Sec. III-F.3), the ones karma_plan, karma_set_plan and
 * karma_step of a context of this model honour (premature swap-in of a swapped record input that a later record
 * reads again, the readers' gradient held until that record's backward adds it to its own).  skips_out (host, may
 * be NULL to ask for the count): *n_inout holds its capacity on entry and the number of connections on return
 * (KARMA_E_OOM if too small).  Only KARMA_MODEL_UNET has any. */
int karma_model_skips(const karma_model_desc* desc, karma_skip* skips_out, uint32_t* n_inout);

/* Creates a context.  arena_dev: device slab of arena_bytes owned by the caller (e.g. a
 * torch uint8 tensor), 256-byte aligned, must outlive the context.  The three streams are
 * hipStream_t values owned by the caller, all of default priority.  The library owns its
 * pinned host pool, events, host master weights and everything it places in the slab. */
int karma_create(const karma_model_desc* desc, const karma_config* cfg, void* arena_dev,
                 uint64_t arena_bytes, void* stream_compute, void* stream_h2d, void* stream_d2h,
                 karma_ctx** out);
void karma_destroy(karma_ctx* ctx);
const char* karma_last_error(const karma_ctx* ctx);

/* Parameter tensors.  Record/tensor numbering: see karma_param_count/karma_param_size.
 * set: copies n fp32 values into the host master copy and uploads the device copy
 * (rounded to bf16 by round-to-nearest-even for bf16 models; for streamed weights the
 * "device copy" is the pinned host buffer the next step streams from).  get_param reads
 * the master copy; get_grad copies the gradient of the last step (converted to fp32). */
int karma_param_count(const karma_ctx* ctx, uint32_t layer, uint32_t* n_tensors_out);
int karma_param_size(const karma_ctx* ctx, uint32_t layer, uint32_t tensor, uint64_t* n_elems_out);
int karma_set_param(karma_ctx* ctx, uint32_t layer, uint32_t tensor, const float* host_fp32, uint64_t n);
int karma_get_param(karma_ctx* ctx, uint32_t layer, uint32_t tensor, float* host_fp32_out, uint64_t n);
int karma_get_grad(karma_ctx* ctx, uint32_t layer, uint32_t tensor, float* host_fp32_out, uint64_t n);

/* One host-optimiser update of n parameters (Sec. III-G stage 5: the weights are updated on the CPU), through
 * the loops karma_step runs per record as its gradients land.  All pointers are host pointers.  master (fp32,
 * updated in place), m and v (fp32 moments, in place; m alone for SGD with momentum, none for SGD), grad (fp32 or,
 * with grad_is_bf16, bf16 bit patterns), out (the new weights in device format: bf16 when out_is_bf16, else fp32).
 * out may be the gradient buffer itself when both have one element type (each gradient is then replaced by its new
 * weight); no other overlap is allowed.
 * optimizer: karma_opt_kind; Adam is bias-corrected, step counts from 1.  narrow_vectors != 0 forces the AVX2
 * build of the loops (the AVX-512 build is used where the CPU has it; both give identical results).  Not
 * thread-safe.  Errors: KARMA_E_INVAL. */
int karma_host_update(uint32_t optimizer, float* master, float* m, float* v, const void* grad, uint32_t grad_is_bf16,
                      uint64_t n, float lr, float beta1, float beta2, float eps, uint64_t step, void* out,
                      uint32_t out_is_bf16, uint32_t narrow_vectors);

/* Analytic cost model (Sec. III-C: the number of arithmetic operations of a block's layers as the proxy of
 * its cost, projected on the device's throughput; memory from the shapes, Sec. III-D).  No GPU is used: with
 * these records karma_plan_pure / karma_simulate project a model at any batch size.  One multiply-add counts
 * as one operation, as in the paper.  matrix_ops_per_s: rate of the matrix operations (convolutions, fully
 * connected layers, attention products); other_ops_per_s: rate of everything else (normalisations,
 * activations, softmax, pooling, adds).  Times: t_fwd = ceil(matrix*1e9/rate) + ceil(other*1e9/rate),
 * t_bwd = 2 t_fwd, t_recompute = t_fwd; the loss op takes three times its forward count.
 * *n_inout: capacity of layers_out on entry (KARMA_E_OOM and the needed count if too small), count on
 * return.  loss_out, fixed_out may be NULL.  Errors: KARMA_E_INVAL. */
typedef struct {
  uint64_t matrix_ops_per_s;
  uint64_t other_ops_per_s;
} karma_device_rates;
int karma_model_costs(const karma_model_desc* desc, const karma_device_rates* rates, karma_layer_cost* layers_out,
                      uint32_t* n_inout, karma_loss_cost* loss_out, uint64_t* fixed_out);

/* Cost records of the model: bytes from shapes (exact, the library owns the allocator),
 * times from the last karma_measure (0 before).  layers_out has karma_model_layers
 * entries.  fixed_out: bytes resident for the whole step (weights, gradients, inputs). */
int karma_get_costs(karma_ctx* ctx, karma_layer_cost* layers_out, karma_loss_cost* loss_out,
                    uint64_t* fixed_out);
/* Measures per-layer forward/backward/recompute times (in-core, median of `reps`), the
 * pinned-copy bandwidth of both directions, alone and while the other direction copies and the host
 * optimiser runs, and the host optimiser's rate on a scratch tensor, from which every record's th_ns
 * (Sec. III-D: profiled once per model).  Needs arena_bytes large enough for one layer in-core. */
int karma_measure(karma_ctx* ctx, uint32_t reps, karma_link* link_out);
/* Replaces every record's th_ns by the time its host update actually took the last time it ran in a step
 * with KARMA_STEP_APPLY_OPTIMIZER (on the real master weights and moments, whose working set can be far
 * larger than the scratch tensor karma_measure times: 200 GB for the largest workload).  Records that have
 * not been updated yet keep their value.  KARMA_E_STATE if no update has run. */
int karma_refine_host_costs(karma_ctx* ctx);
/* Overrides measured figures (tests, reproducible plans). */
int karma_set_costs(karma_ctx* ctx, const karma_layer_cost* layers, const karma_loss_cost* loss,
                    const karma_link* link);

/* Plans for a budget (<= arena_bytes) with the current cost records and builds the
 * executable schedule.  actions_out and weights_kept_out (each may be NULL, n_layers
 * bytes) receive the chosen actions and, for streamed weights, which layers keep them
 * between forward and backward. */
int karma_plan(karma_ctx* ctx, uint64_t budget_bytes, uint8_t* actions_out, uint8_t* weights_kept_out,
               karma_plan_summary* summary_out);
/* karma_plan with the block granularity chosen as well (see karma_plan_grouped_pure): plans on the context's
 * cost records and installs the result.  *group_out (may be NULL): the group size chosen. */
int karma_plan_grouped(karma_ctx* ctx, uint64_t hbm_budget_bytes, uint32_t max_group, uint8_t* actions_out,
                       uint8_t* weights_kept_out, karma_plan_summary* summary_out, uint32_t* group_out);
/* Forces an action vector and weight choice (weights_kept may be NULL = no layer keeps
 * its streamed weights); validated against the budget by simulation. */
int karma_set_plan(karma_ctx* ctx, uint64_t budget_bytes, const uint8_t* actions, const uint8_t* weights_kept,
                   karma_plan_summary* summary_out);
/* Stage string of the current plan. */
int karma_plan_string(karma_ctx* ctx, char* buf, size_t buf_len);

#define KARMA_STEP_APPLY_OPTIMIZER 1u /* D2H gradients, host update of the master weights, H2D new weights */
#define KARMA_STEP_PROFILE 2u         /* events around every op; read with karma_get_op_times / karma_get_stats */
#define KARMA_STEP_KERNEL_TIMES 4u    /* events around one GEMM launch in eight (which ones rotates from step to step); read with karma_get_gemm_stats */
/* One training step.  MLP: inputs_host fp32 [batch, width], labels_host fp32 targets of
 * the same shape.  GPT: inputs_host int32 token ids [batch, seq], labels_host int32
 * [batch, seq].  Synchronous: on return the loss is valid, all streams are drained and
 * gradients can be read; with KARMA_STEP_APPLY_OPTIMIZER some records' host updates may still
 * be pending (karma_finish_updates).  CNN, WRN: inputs_host fp32 images [batch][seq][seq][3], labels_host int32.
 * inputs_host and labels_host both NULL: the batch of the previous karma_step, which is still resident in HBM
 * (and in the pinned staging buffers), is used again without being converted or copied (a training loop whose
 * data already lives on the device; KARMA_E_STATE when there is no such batch: before the first step, after
 * karma_measure).  One of them NULL: KARMA_E_INVAL. */
int karma_step(karma_ctx* ctx, const void* inputs_host, const void* labels_host, uint32_t flags, float* loss_out);

typedef struct {
  double step_ms;          /* wall time of the last step */
  double compute_busy_ms;  /* sum of compute-op durations from events */
  double d2h_ms, h2d_ms;   /* busy time of the copy streams */
  uint64_t bytes_d2h, bytes_h2d;
  uint64_t arena_peak_bytes;
  double host_opt_ms;      /* host optimiser wall time spent since this step began: updates the previous step left
                              pending and finished here count, updates this step leaves pending do not */
  uint64_t updates_deferred; /* records whose host update the step left pending (karma_finish_updates) */
} karma_step_stats;
int karma_get_stats(karma_ctx* ctx, karma_step_stats* out);
/* Host updates that the last karma_step put off (Sec. III-G: the update of stage 5 overlaps the
 * next iteration).  A step run with KARMA_STEP_APPLY_OPTIMIZER updates records on the host while
 * the GPU is still busy with that step; once the GPU has finished, the records not yet updated are
 * left pending and karma_step returns.  Each pending update is finished right before the first
 * operation that reads the record's weights in the next karma_step, and before karma_get_param,
 * karma_set_param, karma_plan / karma_set_plan and karma_measure touch anything.  This call
 * finishes all of them now and waits for the weight copies they start (host thread blocks).
 * A caller that times steps calls it before stopping the clock.  Steps run with
 * KARMA_STEP_PROFILE never leave updates pending.  Returns KARMA_OK or the first error. */
int karma_finish_updates(karma_ctx* ctx);
/* The sampled GEMM launches of the last step run with KARMA_STEP_KERNEL_TIMES: how many were
 * timed, the sum of their durations (HIP events on the compute stream) and of their 2*m*n*k
 * flop counts.  Eight consecutive steps sample every launch of a step once. */
int karma_get_gemm_stats(karma_ctx* ctx, uint64_t* launches_out, double* ms_out, double* flops_out);
/* The ops of the current plan (predicted times) and, for the last step run with
 * KARMA_STEP_PROFILE, their measured durations in ms.  *n_inout: capacity in, count out. */
int karma_get_op_times(karma_ctx* ctx, karma_op* ops_out, float* ms_out, uint32_t* n_inout);
/* When each op of the last step run with KARMA_STEP_PROFILE began on its stream, in ms from the begin of the
 * first op (same order and count as karma_get_op_times).  With the durations this gives the time the compute
 * stream stood idle before each op (the stall profile of Sec. V, Fig. 6).  *n_inout: capacity in, count out;
 * KARMA_E_OOM with the count when the capacity is too small. */
int karma_get_op_starts(karma_ctx* ctx, float* start_ms_out, uint32_t* n_inout);

/* ---- single kernels (device pointers, launched on `stream`, asynchronous) --------
 * Exposed so that each can be checked against the CPU oracle on its own.  Shapes are
 * row-major.  bf16 tensors are uint16_t bit patterns. */

/* fp32 fully connected layer with ReLU (Sec. III-C): z = x W^T + b, y = max(z, 0).
 * x [m,k], w [n,k], b [n], z and y [m,n]. */
int karma_k_linear_relu_fwd_f32(const float* x_dev, const float* w_dev, const float* b_dev, float* z_dev,
                                float* y_dev, uint32_t m, uint32_t n, uint32_t k, void* stream);
/* dz = dy * (z > 0); dx = dz W (skipped when dx_dev is NULL); dW = dz^T x; db = colsum dz. */
int karma_k_linear_relu_bwd_f32(const float* x_dev, const float* w_dev, const float* z_dev, const float* dy_dev,
                                float* dz_ws_dev, float* dx_dev, float* dw_dev, float* db_dev, uint32_t m,
                                uint32_t n, uint32_t k, void* stream);
/* loss = mean((y - t)^2) over n elements, dy = 2 (y - t) / n; partial_ws_dev: >= 1024 floats. */
int karma_k_mse_f32(const float* y_dev, const float* t_dev, float* dy_dev, float* loss_dev, float* partial_ws_dev,
                    uint64_t n, void* stream);

/* bf16 GEMM with fp32 accumulation on the matrix cores (the fully connected layer of
 * Sec. III-C and its two gradients): c[m,n] = sum_k A(m,k) B(n,k) + bias[n] + residual[m,n].
 * a_dev is [m][k] (k contiguous) or, with KARMA_GEMM_A_STRIDED, [k][m]; b_dev is [n][k] or,
 * with KARMA_GEMM_B_STRIDED, [k][n].  bias_dev (bf16 [n]) and residual_dev (bf16 [m][n]) may
 * be NULL.  Output bf16 [m][n], or fp32 with KARMA_GEMM_OUT_F32 (then KARMA_GEMM_ACCUMULATE
 * adds to what c_dev holds; no residual).  k must be a multiple of 8; a strided operand
 * needs its row count to be a multiple of 4.  ws_dev (may be NULL): workspace that lets the
 * kernel split a long reduction over more workgroups when m*n alone cannot fill the chip
 * (up to 16*m*n floats are used; partial sums are added in a fixed order).
 * Errors: KARMA_E_INVAL. */
#define KARMA_GEMM_A_STRIDED 1u
#define KARMA_GEMM_B_STRIDED 2u
#define KARMA_GEMM_OUT_F32 4u
#define KARMA_GEMM_ACCUMULATE 8u
int karma_k_gemm_bf16(const void* a_dev, const void* b_dev, void* c_dev, const void* bias_dev,
                      const void* residual_dev, uint32_t m, uint32_t n, uint32_t k, uint32_t flags, void* ws_dev,
                      uint64_t ws_bytes, void* stream);

/* karma_k_gemm_bf16 for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the split-reduction workspace is a fixed device array inside the
 * library (KARMA_GEMM_STATIC_WS_BYTES per GPU the library runs on, held until the process ends) instead of a
 * caller's buffer; the call allocates nothing.  Same arguments, result and errors as karma_k_gemm_bf16 called with
 * a workspace of that size; products whose result is too large for two partial results in the array (2 * m * n * 4
 * bytes > KARMA_GEMM_STATIC_WS_BYTES) are refused with KARMA_E_OOM.  All calls on one GPU share the array: calls
 * that overlap on one GPU (different streams or threads) race and must be serialised by the caller. */
#define KARMA_GEMM_STATIC_WS_BYTES (64u << 20)
int karma_k_gemm_bf16_static_ws(const void* a_dev, const void* b_dev, void* c_dev, const void* bias_dev,
                                const void* residual_dev, uint32_t m, uint32_t n, uint32_t k, uint32_t flags,
                                void* stream);

/* The same product with the GELU of the feed-forward layer (Sec. III-C, fully connected layer followed by its
 * activation) folded into the kernel's output stage, bf16 output only.
 * KARMA_GEMM_GELU_FWD: c_dev = a b^T + bias (the pre-activation, which backward needs) and aux_dev (bf16 [m][n],
 * written) = GELU(c_dev as stored).  KARMA_GEMM_GELU_BWD: c_dev = (a b^T) * GELU'(aux_dev), aux_dev (read)
 * holding the pre-activation; bias_dev must be NULL.  Layouts as the feed-forward layer has them: FWD takes both
 * operands k-contiguous (flags 0), BWD takes b_dev strided (flags KARMA_GEMM_B_STRIDED).  Errors: KARMA_E_INVAL. */
#define KARMA_GEMM_GELU_FWD 1u
#define KARMA_GEMM_GELU_BWD 2u
int karma_k_gemm_gelu_bf16(const void* a_dev, const void* b_dev, void* c_dev, const void* bias_dev, void* aux_dev,
                           uint32_t m, uint32_t n, uint32_t k, uint32_t flags, uint32_t mode, void* stream);

/* karma_k_attention_bwd_bf16 together with the column sums of dqkv over all batch * seq tokens, colsum_out_dev fp32
 * [3 * heads * d]: the gradient of the QKV projection's bias.  Head dimension 64 takes them inside the kernels (one
 * row of partial sums per 32 tokens, from the fp32 values), other head dimensions by a pass over dqkv.
 * ws_dev: batch * seq / 32 * 3 * heads * d floats (KARMA_E_OOM if smaller). */
int karma_k_attention_bwd_colsum_bf16(const void* qkv_dev, const void* ctx_dev, const void* dctx_dev, const float* lse_dev,
                                      float* delta_ws_dev, void* dqkv_dev, float* colsum_out_dev, float* ws_dev,
                                      uint64_t ws_bytes, uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d,
                                      void* stream);

/* KARMA_GEMM_GELU_BWD (b_dev strided) together with the column sums of its result, colsum_out_dev[j] = sum over i
 * of c[i][j], fp32 [n]: the gradient of the bias of the layer whose pre-activation aux_dev holds.  Whole 256-tiles
 * take the sums in the kernel's output stage (from the fp32 values, before they are rounded to bf16); other shapes
 * run the product and then sum the stored bf16 result.  ws_dev: ceil(m/64)*n floats (KARMA_E_OOM if smaller). */
int karma_k_gemm_gelu_bwd_colsum_bf16(const void* a_dev, const void* b_dev, void* c_dev, const void* aux_dev,
                                      float* colsum_out_dev, float* ws_dev, uint64_t ws_bytes, uint32_t m, uint32_t n,
                                      uint32_t k, void* stream);

/* LayerNorm over the last dimension (eps 1e-5, biased variance), bf16 in/out, fp32
 * statistics: stats_dev[2*row] = mean, [2*row+1] = 1/std.  h multiple of 8, <= 6144. */
int karma_k_layernorm_fwd_bf16(const void* x_dev, const void* gamma_dev, const void* beta_dev, void* y_dev,
                               float* stats_dev, uint32_t rows, uint32_t h, void* stream);
/* Its backward: dx (+ add_dev if not NULL, e.g. a residual gradient), dgamma/dbeta fp32 [h]
 * reduced in a fixed order.  ws_dev: ceil(rows/64)*3*h floats (KARMA_E_OOM if smaller). */
int karma_k_layernorm_bwd_bf16(const void* dy_dev, const void* x_dev, const float* stats_dev, const void* gamma_dev,
                               const void* add_dev, void* dx_dev, float* dgamma_dev, float* dbeta_dev, float* ws_dev,
                               uint64_t ws_bytes, uint32_t rows, uint32_t h, void* stream);
/* The same with add_dev required and its column sums delivered as well: add_colsum_dev[c] = sum over rows of
 * add[r][c], fp32 [h] (add is the gradient of the sum the LayerNorm's input went into; its column sums are that
 * sum's bias gradient, taken here without another pass over the tensor). */
int karma_k_layernorm_bwd_addsum_bf16(const void* dy_dev, const void* x_dev, const float* stats_dev, const void* gamma_dev,
                                      const void* add_dev, void* dx_dev, float* dgamma_dev, float* dbeta_dev,
                                      float* add_colsum_dev, float* ws_dev, uint64_t ws_bytes, uint32_t rows, uint32_t h,
                                      void* stream);
/* out[c] = sum over rows of x[r][c] (bias gradients), fixed order.  ws: ceil(rows/64)*cols floats. */
int karma_k_colsum_bf16(const void* x_dev, float* out_dev, float* ws_dev, uint64_t ws_bytes, uint32_t rows,
                        uint32_t cols, void* stream);
/* tanh-form GELU and its gradient dx = dy * gelu'(x); n multiple of 8. */
int karma_k_gelu_fwd_bf16(const void* x_dev, void* y_dev, uint64_t n, void* stream);
int karma_k_gelu_bwd_bf16(const void* x_dev, const void* dy_dev, void* dx_dev, uint64_t n, void* stream);
/* out[t] = wte[ids[t]] + wpe[t % seq]. */
int karma_k_embed_fwd_bf16(const int32_t* ids_dev, const void* wte_dev, const void* wpe_dev, void* out_dev,
                           uint32_t tokens, uint32_t seq, uint32_t h, void* stream);
/* Embedding gradients without atomics.  order_dev: token positions sorted by id (stable);
 * seg_start_dev[u..u+1] delimits the run of the u-th distinct id seg_id_dev[u] (n_seg runs,
 * n_seg+1 starts).  dwte_f32_dev [vocab][h] is added to; dwpe_dev bf16 [seq][h] is written. */
int karma_k_embed_bwd_bf16(const void* dx_dev, const int32_t* order_dev, const int32_t* seg_start_dev,
                           const int32_t* seg_id_dev, uint32_t n_seg, float* dwte_f32_dev, void* dwpe_dev,
                           uint32_t batch, uint32_t seq, uint32_t h, void* stream);
/* Softmax cross-entropy, forward and gradient in one pass (Sec. III-C softmax layer):
 * rowloss_dev[r] = logsumexp(z_r) - z_r[label_r]; logits_dev is overwritten with
 * (softmax(z_r) - onehot) * scale.  cols multiple of 8, cols*2 bytes <= 150 KiB. */
int karma_k_softmax_ce_bf16(void* logits_dev, const int32_t* labels_dev, float* rowloss_dev, uint32_t rows,
                            uint32_t cols, float scale, void* stream);
/* out = scale * sum(x[0..n)) in a fixed order; ws_dev >= 1024 floats. */
int karma_k_sum_f32(const float* x_dev, float* out_dev, float* ws_dev, uint64_t n, float scale, void* stream);

/* Fused causal self-attention, Attention(Q,K,V) = Softmax(QK^T/sqrt(d)) V per head
 * (Sec. III-C self-attention layer).  qkv_dev bf16 [batch][seq][3*heads*d] with q|k|v in
 * thirds and head j in columns j*d..; ctx_dev bf16 [batch][seq][heads*d]; lse_dev fp32
 * [batch][heads][seq] receives log2 of the row sums of 2^(score*log2(e)/sqrt(d)).
 * seq must be a multiple of 128, d 64, 128 or 152 (else KARMA_E_INVAL). */
int karma_k_attention_fwd_bf16(const void* qkv_dev, void* ctx_dev, float* lse_dev, uint32_t batch, uint32_t seq,
                               uint32_t heads, uint32_t d, void* stream);
/* Its backward: dqkv_dev (same layout as qkv) from dctx_dev, the forward's ctx and lse.
 * delta_ws_dev: batch*heads*seq floats of workspace.  No atomics: results are reproducible. */
int karma_k_attention_bwd_bf16(const void* qkv_dev, const void* ctx_dev, const void* dctx_dev, const float* lse_dev,
                               float* delta_ws_dev, void* dqkv_dev, uint32_t batch, uint32_t seq, uint32_t heads,
                               uint32_t d, void* stream);

/* ---- convolutional workload (Sec. III-C: convolution, batch normalisation, ReLU and
 * pooling layers).  Tensors are NHWC bf16, convolution weights [c_out][r][s][c_in]; c_in and
 * c_out must be multiples of 8 (an image with 3 channels is stored with 8, the rest zero).
 * Output size per dimension: (in + 2*pad - kernel)/stride + 1.  KARMA_E_INVAL on bad shapes. */
typedef struct {
  uint32_t n, h, w, c_in, c_out, r, s, stride, pad;
} karma_conv_shape;

/* y[n][ho][wo][c_out] = sum over the r x s taps and c_in channels, padding counting as
 * zero: the direct convolution of Sec. III-C computed as an implicit GEMM (no im2col). */
int karma_k_conv2d_fwd_bf16(const void* x_dev, const void* w_dev, void* y_dev, const karma_conv_shape* shape, void* stream);
/* The same with add_dev (y's shape, may be NULL) added to the result before it is rounded: the residual
 * sum of a pre-activated block, whose last layer is a convolution. */
int karma_k_conv2d_fwd_add_bf16(const void* x_dev, const void* w_dev, const void* add_dev, void* y_dev,
                                const karma_conv_shape* shape, void* stream);
/* dx_dev [n][h][w][c_in] (+ add_dev, same shape, may be NULL) from dy_dev [n][ho][wo][c_out].
 * wt_ws_dev: r*s*c_in*c_out bf16 elements of workspace (transposed weights); may be NULL
 * for a 1x1 stride-1 convolution. */
int karma_k_conv2d_dgrad_bf16(const void* dy_dev, const void* w_dev, void* wt_ws_dev, const void* add_dev, void* dx_dev,
                              const karma_conv_shape* shape, void* stream);
/* dw_dev [c_out][r][s][c_in] bf16.  ws_dev/ws_bytes: optional fp32 workspace that lets the
 * reduction over the pixels be split (up to 16 * c_out*r*s*c_in floats are used); results
 * are reproducible either way. */
int karma_k_conv2d_wgrad_bf16(const void* dy_dev, const void* x_dev, void* dw_dev, void* ws_dev, uint64_t ws_bytes,
                              const karma_conv_shape* shape, void* stream);

/* Training-mode batch normalisation of x_dev bf16 [rows][c] over its rows (rows = n*h*w):
 * mean and biased variance per channel, eps 1e-5; y = xhat*gamma + beta (+ add_dev, may be
 * NULL), then ReLU when relu != 0.  stats_dev fp32 [2][c] receives mean and 1/sqrt(var+eps);
 * ws_dev: karma_k_batchnorm_ws_bytes(rows, c) bytes (per-band channel sums).  c must be a
 * multiple of 8. */
uint64_t karma_k_batchnorm_ws_bytes(uint32_t rows, uint32_t c);
int karma_k_batchnorm_fwd_bf16(const void* x_dev, const void* gamma_dev, const void* beta_dev, const void* add_dev,
                               void* y_dev, void* stats_dev, void* ws_dev, uint32_t rows, uint32_t c, uint32_t relu,
                               void* stream);
/* Its backward from the forward's x and stats.  relu != 0: dy first passes the ReLU that
 * followed the normalisation (the mask is recomputed from xhat*gamma + beta > 0).
 * dgamma_dev, dbeta_dev fp32 [c]; ws_dev as above. */
int karma_k_batchnorm_bwd_bf16(const void* dy_dev, const void* x_dev, const void* stats_dev, const void* gamma_dev,
                               const void* beta_dev, uint32_t relu, void* dx_dev, void* dgamma_dev, void* dbeta_dev,
                               void* ws_dev, uint32_t rows, uint32_t c, void* stream);
/* The same with add_dev (x's shape, may be NULL, may be dy_dev) added to dx before it is rounded: the gradient
 * that reaches x through a shortcut around the normalisation. */
int karma_k_batchnorm_bwd_add_bf16(const void* dy_dev, const void* x_dev, const void* stats_dev, const void* gamma_dev,
                                   const void* beta_dev, uint32_t relu, const void* add_dev, void* dx_dev,
                                   void* dgamma_dev, void* dbeta_dev, void* ws_dev, uint32_t rows, uint32_t c,
                                   void* stream);
/* dz = dy where y > 0, else 0; n elements, multiple of 8. */
int karma_k_relu_mask_bwd_bf16(const void* dy_dev, const void* y_dev, void* dz_dev, uint64_t n, void* stream);
/* 3x3 max pooling, stride 2, padding 1 (Sec. III-C pooling layer); the backward gives the
 * gradient of a window to its first maximum in row-major window order, without atomics. */
int karma_k_maxpool_fwd_bf16(const void* x_dev, void* y_dev, uint32_t n, uint32_t h, uint32_t w, uint32_t c, void* stream);
int karma_k_maxpool_bwd_bf16(const void* x_dev, const void* dy_dev, void* dx_dev, uint32_t n, uint32_t h, uint32_t w,
                             uint32_t c, void* stream);
/* 2x2 max pooling with stride 2 (Sec. III-C pooling layer; the contracting path of the fully convolutional
 * network): x_dev [n][h][w][c] -> y_dev [n][h/2][w/2][c]; h and w even, c a multiple of 8.  The backward writes
 * all of dx_dev (x's shape): dy to the first maximum of each window in row-major window order, zero elsewhere. */
int karma_k_maxpool2_fwd_bf16(const void* x_dev, void* y_dev, uint32_t n, uint32_t h, uint32_t w, uint32_t c, void* stream);
int karma_k_maxpool2_bwd_bf16(const void* x_dev, const void* dy_dev, void* dx_dev, uint32_t n, uint32_t h, uint32_t w,
                              uint32_t c, void* stream);
/* y += a, n bf16 elements (a multiple of 8), one rounding: how the gradient that other readers of a tensor left
 * for it (Sec. III-F.3, connections between non-consecutive layers) joins the gradient of its direct consumer. */
int karma_k_add_inplace_bf16(void* y_dev, const void* a_dev, uint64_t n, void* stream);
/* Global average pooling over hw positions: x [n][hw][c] -> y [n][c], and its backward. */
int karma_k_avgpool_fwd_bf16(const void* x_dev, void* y_dev, uint32_t n, uint32_t hw, uint32_t c, void* stream);
int karma_k_avgpool_bwd_bf16(const void* dy_dev, void* dx_dev, uint32_t n, uint32_t hw, uint32_t c, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KARMA_H */
