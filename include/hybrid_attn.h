/*
 * hybrid_attn.h -- C ABI of the MI355X (gfx950) hybrid-attention forward.
 *
 * The operator is the hybrid attention of "Attention Surgery" (arXiv 2509.24899), Sec. 3.2,
 * Eq. "hybrid": per (batch, head) and query token i
 *
 *            sum_{j in T_S} exp(scale q_i.k_j - c_i) v_j  +  phi_q(q_i) . S
 *    y_i  =  ------------------------------------------------------------------ ,
 *            sum_{j in T_S} exp(scale q_i.k_j - c_i)      +  phi_q(q_i) . z
 *
 *    S = sum_{j in T_L} phi_k(k_j)^T v_j  (F x d),   z = sum_{j in T_L} phi_k(k_j)  (F),
 *
 * T_S = every R-th token starting with the first (the stride rule of Sec. 3.2, stated there on 1-indexed tokens),
 * T_L = the other tokens, c_i = max_{j in T_S} scale q_i.k_j (it stabilises the softmax terms
 * only, exactly as the equation is printed), and phi the polynomial feature map of Sec. 3.2
 * ("Characterization of phi"): per-head 2-layer MLP with ReLU, a positive output activation,
 * P equal channel slices, slice p raised to the power p.
 *
 * Everything is plain C: POD structs, raw pointers, sizes.  Unless a parameter says "host", a
 * data pointer is a DEVICE pointer (HIP global memory on the current device).  The library never
 * allocates or frees device memory, never synchronises, and launches all work on the stream the
 * caller passes; the caller owns every buffer.  No exception crosses the boundary: every entry
 * point that can fail returns an ha_status, and all argument checks run on the host before the
 * first HIP call (they work on a machine without a GPU).
 */
#ifndef HYBRID_ATTN_H
#define HYBRID_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HA_OK = 0,
  HA_ERR_NULL = 1,        /* a required pointer is NULL */
  HA_ERR_SHAPE = 2,       /* non-positive or inconsistent sizes / strides */
  HA_ERR_UNSUPPORTED = 3, /* a valid problem this build has no kernel for */
  HA_ERR_ALIGN = 4,       /* a device pointer or stride breaks the 16-byte rule */
  HA_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than hybrid_attn_workspace_bytes() */
  HA_ERR_DEVICE = 6,      /* a HIP call failed; see hybrid_attn_last_device_error() */
  HA_ERR_INFEASIBLE = 7   /* hybrid_attn_select_rates: no assignment fits the budget */
} ha_status;

typedef enum { HA_BF16 = 0, HA_F32 = 1 } ha_dtype;

/* Output activation that makes phi non-negative (Sec. 3.1 requires phi >= 0).  SOFTMAX runs over
 * all F output channels of one token and head, before the slice / power step. */
typedef enum { HA_ACT_SOFTMAX = 0, HA_ACT_EXP = 1, HA_ACT_RELU = 2 } ha_act;

/* One feature map (phi_q or phi_k): the per-head map of Sec. 3.2 ("Characterization of phi"), one set of weights
 * per head, shared over the batch.
 *   hidden = relu(W1 x + b1),  u = W2 hidden + b2,  t = act(u),
 *   phi(x)[c] = t[c] ^ (1 + c / (F / P))          (integer division: slice p gets power p).
 * Three-layer map (Tab. "phi", the P = 6 row): with w_mid != NULL, hidden2 = relu(W_mid hidden + b_mid) sits
 * between the two and W2 is [H, d_out, d_mid].  A caller that only knows the two-layer struct leaves the
 * trailing fields zero. */
typedef struct {
  const void  *w1;        /* device [H, d_hidden, d_head], io dtype, row-major, contiguous */
  const float *b1;        /* device [H, d_hidden] fp32, or NULL for zero bias */
  const void  *w2;        /* device [H, d_out, d_hidden], io dtype, row-major, contiguous */
  const float *b2;        /* device [H, d_out] fp32, or NULL for zero bias */
  int32_t d_hidden;       /* Hd: multiple of 32 */
  int32_t d_out;          /* F = P * D': multiple of 32 */
  int32_t poly_degree;    /* P in 1..8, must divide d_out */
  int32_t out_act;        /* ha_act */
  const void  *w_mid;     /* device [H, d_mid, d_hidden], io dtype, or NULL: two-layer map */
  const float *b_mid;     /* device [H, d_mid] fp32, or NULL for zero bias */
  int32_t d_mid;          /* width of the second hidden layer (ignored when w_mid is NULL) */
  int32_t reserved;       /* 0 */
} ha_feature_map;

/* One forward problem.  q, k, v and out are [B, H, N, d_head] views: element (b, h, n, c) lives at
 * base + b*stride_b + h*stride_h + n*stride_n + c (strides in ELEMENTS, the innermost d_head run is
 * contiguous), the same strides for all four tensors. */
typedef struct {
  int32_t B, H, N, d_head;
  int32_t dtype;          /* ha_dtype of q, k, v, out, w1, w2.  HA_F32 inputs are rounded to bf16
                             on load (the matrix cores run in bf16 with fp32 accumulation) and
                             the result is written as fp32. */
  int32_t block_size;     /* 64 or 128: tiling of the softmax loop.  128: workgroups of 256 queries
                             (8 waves x 32), keys staged through LDS 64 at a time; 64: workgroups
                             of 128 queries (4 waves x 32), keys staged 32 at a time.  A tiling knob
                             only: every query column sees the same keys in the same order, so the
                             result does not depend on it. */
  int32_t hybrid_rate;    /* R.  0: no softmax tokens (pure linear attention, r = 0);
                             1: every token is a softmax token (plain softmax attention, r = 1);
                             R >= 2: tokens 0, R, 2R, ... (0-indexed) are softmax tokens, r = 1/R.
                             Any R <= N is accepted; it is never rounded. */
  float   softmax_scale;  /* multiplies q.k; pass 1/sqrt(d_head) for the paper's operator */
  int64_t stride_b, stride_h, stride_n;
  int32_t split_granularity; /* 0 or 1: the split of Sec. 3.2, per token.  g >= 2 (a variant, not the paper's
                             method): whole groups of g consecutive tokens are softmax tokens, every R-th
                             group: token j is a softmax token when (j / g) mod R == 0.  Any g <= N
                             with R g <= 2^30. */
  int32_t causal_chunk;   /* 0: every query sees every token (the paper's operator).  C > 0 (a variant; the paper
                             leaves causal attention to future work and defines none): chunks of C consecutive
                             tokens, a query sees its own and all earlier chunks, so S and z are prefix sums over
                             chunks.  C must be a multiple of 2 * block_size.  hybrid_attn_forward only, with maps
                             the fused kernels take (d_hidden, d_out = d_head, or 256 at d_head = 128);
                             HA_ERR_UNSUPPORTED elsewhere. */
  int32_t local_window;   /* 0: off.  W > 0 (a variant: the local-window design that Sec. 3.2 sets the uniform
                             stride against, in a blocked form): with tiles of T = 2 * block_size tokens, the
                             softmax tokens of a query in tile t are the tokens of tiles t - W/T .. t + W/T, every
                             other token is a linear token; Eq. "hybrid" is evaluated with these per-tile sets.
                             W must be a multiple of T, hybrid_rate must be 0 (no strided softmax tokens),
                             split_granularity <= 1 and causal_chunk == 0.  hybrid_attn_forward only, fused maps
                             only, as for causal_chunk. */
  int32_t reserved;       /* must be 0 */
} ha_problem;

/* Host-only argument check (no HIP call).  phi_q and phi_k may be NULL iff the problem has no
 * linear tokens (hybrid_rate == 1); otherwise both are required and must agree in d_out.
 * Pointers inside the feature maps are checked for NULL and alignment but never dereferenced.
 * Supported here: d_head in {64, 128} with d_hidden == d_out == d_head, or d_head == 128 with
 * d_hidden == d_out == 256 (the paper's default widths, Tab. "phi"), both through kernels that keep a token's
 * activations in registers; at d_head == 128 also any d_hidden, d_mid, d_out that are multiples of 128 up to 768,
 * with two or three layers (the other rows of Tab. "phi"), layer by layer through HBM.  phi_q and phi_k must have
 * the same widths and depth. */
ha_status hybrid_attn_validate(const ha_problem *p, const ha_feature_map *phi_q,
                               const ha_feature_map *phi_k);

/* Bytes of device scratch hybrid_attn_forward needs for this problem (0 if the problem does not
 * validate).  Holds the compacted softmax keys / values, the MLP weights in matrix-core operand
 * order, the per-chunk partial states and the reduced state S, z.  Host only. */
size_t hybrid_attn_workspace_bytes(const ha_problem *p, const ha_feature_map *phi_q,
                                   const ha_feature_map *phi_k);

/* Enqueue one forward on `hip_stream` (a hipStream_t passed as void*, NULL = the default stream)
 * and return without waiting.  q, k, v: device, read-only.  out: device, written in full.
 * workspace: device, 256-byte aligned, at least hybrid_attn_workspace_bytes() bytes, contents
 * undefined before and after.  out and workspace must not overlap the inputs.  Two calls that
 * share a workspace must be ordered on one stream.  Returns HA_OK once everything is enqueued. */
ha_status hybrid_attn_forward(const ha_problem *p, const void *q, const void *k, const void *v,
                              const ha_feature_map *phi_q, const ha_feature_map *phi_k,
                              void *out, void *workspace, size_t workspace_bytes, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture with a foreign allocator, tight
 * serving loops, harnesses that forbid hipMalloc): hybrid_attn_forward with the scratch taken from a static device
 * array inside the library instead of a caller workspace.  The array is HA_STATIC_SCRATCH_MIB MiB; every GPU the
 * library runs on holds its own copy until the process ends, and its address on a GPU is looked up at the first
 * call on that GPU.  The call allocates nothing, frees nothing and does not synchronise; apart from the workspace
 * it takes the arguments of hybrid_attn_forward and returns the same result bit for bit.  A problem whose
 * hybrid_attn_workspace_bytes() exceeds hybrid_attn_static_scratch_bytes() is refused with HA_ERR_WORKSPACE before
 * any HIP call (at the 480p / 81-frame shape with 12 heads the workspace is about 75 MB, so that shape does not fit;
 * 12 heads of 16 K tokens at rate 4 do).  All calls on one GPU share the one array, whose contents are undefined
 * between calls (nothing in it has to start at zero): calls on one GPU must be ordered on one stream, or
 * otherwise not overlap; calls that overlap on one GPU race. */
#define HA_STATIC_SCRATCH_MIB 64
size_t hybrid_attn_static_scratch_bytes(void);
ha_status hybrid_attn_forward_static(const ha_problem *p, const void *q, const void *k, const void *v,
                                     const ha_feature_map *phi_q, const ha_feature_map *phi_k,
                                     void *out, void *hip_stream);

/* Debug / test taps into the same pipeline: run only the key-side passes (weight re-ordering,
 * softmax-key compaction, state pass) and copy the reduced state out in plain layout.
 * state_S: device fp32 [B, H, F, d_head]; state_z: device fp32 [B, H, F]. */
ha_status hybrid_attn_linear_state(const ha_problem *p, const void *k, const void *v,
                                   const ha_feature_map *phi_k, float *state_S, float *state_z,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* Per-stage timing tap for benchmarks.  hybrid_attn_profile_enable(n) (n >= 1) creates n sets of HIP
 * events on the current device; from then on every hybrid_attn_forward on this host thread records
 * one set on its stream around its stages (record i uses set i % n); n = 0 switches the tap off and
 * destroys the events.  hybrid_attn_profile_read waits for record `index` to finish and returns the
 * stage durations in milliseconds: ms[0] softmax-key compaction, ms[1] key-side feature map + state
 * pass + state reduction, ms[2] query-side weight re-ordering, ms[3] the fused query kernel (softmax
 * tile loop, phi_q, contraction with the state and merge), ms[4] the whole forward.  Stages that did
 * not run report 0.  HA_ERR_SHAPE for an index that was never recorded.  Host memory only.
 * A negative count, hybrid_attn_profile_enable(-n), creates n sets as well but records only the pair of events around
 * the fused query kernel (two event records per forward instead of five, each of which costs the stream a few
 * microseconds): ms[3] is measured, the other entries read 0. */
ha_status hybrid_attn_profile_enable(int n_records);
ha_status hybrid_attn_profile_read(int index, float ms[5]);
int hybrid_attn_profile_count(void);   /* forwards recorded since the last enable */

/* Measurement aid for benchmarks (no part of the method): enqueue `launches` launches of a kernel that
 * issues nothing but dense bf16 32x32x16 matrix instructions on register operands, one 512-thread
 * workgroup per compute unit of the current device, 16 * iters instructions per wave.  Timed by the
 * caller, it gives the matrix-core rate the device sustains next to its published peak; the rate
 * depends on the operand values through power and clock, hence random_operands: 0 = all-zero
 * operands, non-zero = pseudo-random values in [-1, 1).  sink: device, 16-byte aligned, at least
 * 2 KiB per compute unit (HA_ERR_WORKSPACE otherwise), overwritten.  *flops_per_launch (host)
 * receives the flop count of one launch.  Returns once everything is enqueued on `hip_stream`. */
ha_status hybrid_attn_mfma_probe(int random_operands, int iters, int launches, void *sink, size_t sink_bytes,
                                 double *flops_per_launch, void *hip_stream);

/* Value-distillation objective (Sec. 3.3, Eq. "vd_loss"; the loss line of Alg. 1 for one sample batch):
 * || y - y_hat ||_1, y the softmax attention of q, k, v (Eq. "softmax": the forward at rate 1, feature maps
 * unused) and y_hat the hybrid attention at p->hybrid_rate (Eq. "hybrid"), summed over every batch entry,
 * head, token and channel (Alg. 1 averages over samples: divide by B).  Enqueues the teacher forward
 * (skipped when teacher_is_cached != 0: y_teacher then already holds it, as Alg. 1 caches the teacher's
 * outputs for several student updates), the student forward and a two-stage reduction in a fixed order
 * (bitwise reproducible).  y_teacher, y_student: device, [B, H, N, d_head] with p's strides and dtype,
 * distinct buffers, both hold the two outputs afterwards.  loss: device double[1 + B * H]: loss[0] the
 * total, loss[1 + b * H + h] the share of (batch b, head h).  workspace: device, 256-byte aligned, at
 * least hybrid_attn_value_distill_workspace_bytes() bytes.  Other arguments and errors as for
 * hybrid_attn_forward. */
size_t hybrid_attn_value_distill_workspace_bytes(const ha_problem *p, const ha_feature_map *phi_q,
                                                 const ha_feature_map *phi_k);
ha_status hybrid_attn_value_distill_loss(const ha_problem *p, const void *q, const void *k, const void *v,
                                         const ha_feature_map *phi_q, const ha_feature_map *phi_k,
                                         int teacher_is_cached, void *y_teacher, void *y_student, double *loss,
                                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* Gradient of the value-distillation objective with respect to the two feature maps (Sec. 3.3: the update
 * line of Alg. 1, phi <- phi - eta grad_phi L, with L of Eq. "vd_loss"; everything but phi_q, phi_k is frozen in
 * that stage, so q, k, v are constants).  Buffers of one map's gradient, all device fp32, overwritten in full,
 * summed over the batch (the parameters are shared by it): w1 [H, d_hidden, d_head], b1 [H, d_hidden],
 * w2 [H, d_out, d_hidden], b2 [H, d_out].  All four are required, also for a map given without biases.  For a
 * three-layer map (w_mid given): w2 [H, d_out, d_mid], and w_mid [H, d_mid, d_hidden], b_mid [H, d_mid] are
 * required as well; for a two-layer map they are ignored. */
typedef struct ha_feature_map_grad {
  float *w1, *b1, *w2, *b2;
  float *w_mid, *b_mid;
} ha_feature_map_grad;

/* Enqueues: the teacher forward (unless teacher_is_cached), the student forward, which also leaves the
 * denominator l_i + phi_q(q_i).z of every row of Eq. "hybrid" in row_den (unless student_is_cached: y_student
 * and row_den are then inputs, e.g. kept from an earlier call with the same phi), the loss as in
 * hybrid_attn_value_distill_loss, and the backward pass: d loss / d y_hat = sign(y_hat - y) taken from the two
 * stored outputs (0 where they are equal), then the chain rule through Eq. "hybrid" and the feature maps
 * (Sec. 3.2) down to the eight parameter tensors.  The loss is the plain sum, so is the gradient; Alg. 1's
 * 1 / (m |T|) is the caller's.  row_den: device fp32 [B, H, N].  At hybrid_rate == 1 the gradients are zero.
 * Supported here: every feature-map shape the forward takes (both maps of one shape).  Matrix products
 * run in bf16 with fp32 accumulation; the sums over tokens are formed in a fixed order (bitwise reproducible).
 * workspace: device, 256-byte aligned, at least hybrid_attn_value_distill_grad_workspace_bytes() bytes.  Other
 * arguments and errors as for hybrid_attn_value_distill_loss. */
size_t hybrid_attn_value_distill_grad_workspace_bytes(const ha_problem *p, const ha_feature_map *phi_q,
                                                      const ha_feature_map *phi_k);
ha_status hybrid_attn_value_distill_grad(const ha_problem *p, const void *q, const void *k, const void *v,
                                         const ha_feature_map *phi_q, const ha_feature_map *phi_k,
                                         int teacher_is_cached, int student_is_cached, void *y_teacher,
                                         void *y_student, float *row_den, double *loss,
                                         const ha_feature_map_grad *grad_q, const ha_feature_map_grad *grad_k,
                                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* Parameter update of the distillation loop (Sec. 3.3, Alg. 1: phi <- phi - eta grad_phi L; the training details
 * name AdamW, learning rate 1e-3, for this stage).  HA_OPT_SGD is the line as printed: master -= lr * grad_scale *
 * grad.  HA_OPT_ADAMW is Adam with decoupled weight decay: master *= 1 - lr * weight_decay; m = beta1 m +
 * (1 - beta1) g; v = beta2 v + (1 - beta2) g^2; master -= lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) +
 * eps), g = grad_scale * grad, step counted from 1.  grad_scale carries Alg. 1's 1 / (m |T|) (the gradient entry
 * point returns the gradient of the plain sum). */
typedef enum ha_optimizer_kind { HA_OPT_SGD = 0, HA_OPT_ADAMW = 1 } ha_optimizer_kind;
typedef struct ha_optimizer {
  int32_t kind;           /* ha_optimizer_kind */
  int32_t step;           /* AdamW: number of this update, >= 1 */
  float lr, grad_scale;
  float beta1, beta2, eps, weight_decay;   /* AdamW only */
} ha_optimizer;

/* Enqueues one update of one parameter tensor of n elements.  master: device fp32, in/out, the full-precision copy
 * of the parameter; grad: device fp32 (e.g. a tensor of ha_feature_map_grad); m, v: device fp32, in/out, AdamW's
 * moments (zero before the first step; NULL for HA_OPT_SGD); param_io: device, n elements of io_dtype (ha_dtype),
 * out, or NULL: the updated parameter rounded to the dtype the forward reads (the weights; the biases are fp32 and
 * need no copy).  fp32 arithmetic.  Errors (nothing is enqueued): HA_ERR_NULL, HA_ERR_ALIGN (4-byte alignment, 2 for a
 * bf16 copy), HA_ERR_SHAPE (negative or non-finite rates, step < 1, beta outside [0, 1), param_io == master),
 * HA_ERR_UNSUPPORTED (unknown kind or dtype), HA_ERR_DEVICE. */
ha_status hybrid_attn_param_update(const ha_optimizer *opt, size_t n, float *master, const float *grad, float *m, float *v,
                                   void *param_io, int32_t io_dtype, void *hip_stream);

/* Block-rate selection (Sec. 3.3, "Heterogeneous Block-Rate Optimization"; host memory only, no GPU
 * involved).  A model has n_blocks attention blocks and n_rates candidate hybrid rates; cost[i * n_rates + r]
 * and error[i * n_rates + r] (both >= 0, finite) are the pre-computed cost c_ir (flops or measured
 * latency) and error e_ir of giving block i candidate r.  Writes to choice[i] the candidate of block i in
 * the assignment that minimises the summed error subject to summed cost <= budget (the multiple-choice
 * knapsack of that section, solved exactly), and its sums to *total_cost / *total_error, formed in
 * block order.  Among assignments of equal error the cheapest is returned, among those the
 * lexicographically smallest choice vector.  HA_ERR_INFEASIBLE when even the cheapest assignment exceeds
 * the budget; HA_ERR_SHAPE for sizes < 1 or negative / non-finite entries; HA_ERR_UNSUPPORTED when the
 * search would need more than 2^22 undominated (cost, error) states. */
ha_status hybrid_attn_select_rates(int n_blocks, int n_rates, const double *cost, const double *error,
                                   double budget, int *choice, double *total_cost, double *total_error);

/* Static, NUL-terminated description of a status code. */
const char *hybrid_attn_status_string(ha_status s);

/* hipError_t (as int) behind the most recent HA_ERR_DEVICE on the calling thread, 0 if none. */
int hybrid_attn_last_device_error(void);

/* Version of this ABI (bumped on any incompatible change). */
int hybrid_attn_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HYBRID_ATTN_H */
