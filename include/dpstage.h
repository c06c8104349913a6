/*
 * dpstage - forward+backward training step of one pipeline stage under a
 * per-tensor keep / recompute / swap plan, for AMD MI355X (gfx950).
 *
 * The paper models a stage x as a node set N_x whose time is the sum of the
 * nodes' forward and backward times (Section 4.1, Eq. 1), run within a device
 * memory capacity M (Algorithm 1, feasibility test of AdjacentPartition), under
 * a memory-optimisation result "mopt" that assigns swap or recomputation to
 * individual saved tensors (Section 4.3).  This library is the executor of that
 * statement for a stage made of transformer layers:
 *
 *   dp_stage_init    (layer config, weights)            -> stage handle
 *   dp_stage_step    (micro-batch, plan, memory budget) -> Y, dX, dTheta
 *   dp_plan_validate (config, plan, budget)             -> peak-memory report
 *
 * and, around that core:
 *   dp_stage_forward / dp_stage_backward   the step cut where a one-forward-one-backward
 *                                          schedule cuts it (micro-batch slots, gradient
 *                                          accumulation); dp_stage_set_weights (parameter
 *                                          versions); dp_stage_set_rng (dropout masks);
 *                                          dp_stage_set_cross / dp_stage_bind_memory (decoder
 *                                          stages with a cross-attention block)
 *   dp_stage_measure_cost_model, dp_plan_cost, dp_plan_generate
 *                                          Section 4.3's memory optimisation from measured costs
 *   dp_partition                           Section 4.2's partition search over a chain of layers
 *   dp_op_*, dp_stage_op_times, dp_probe_mfma   operators one at a time, and diagnostics
 *
 * Plain C ABI: POD structs, raw pointers, sizes.  "device pointer" means memory
 * of the current HIP device; "host pointer" ordinary process memory.  No call
 * throws; every call returns a dp_status and dp_last_error() gives the text.
 */
#ifndef DPSTAGE_H
#define DPSTAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dp_stage dp_stage; /* opaque, library-owned */

typedef enum {
  DP_OK = 0,
  DP_E_INVAL = -1,       /* null pointer, bad enum, bad length, bad shape        */
  DP_E_PLAN = -2,        /* plan asks for something impossible                    */
  DP_E_BUDGET = -3,      /* inflight x peak_bytes exceeds budget_bytes            */
  DP_E_DEVMEM = -4,      /* device allocation failed                              */
  DP_E_HOSTMEM = -5,     /* pinned host allocation failed                         */
  DP_E_HIP = -6,         /* a HIP runtime call or launch failed                   */
  DP_E_UNSUPPORTED = -7  /* shape outside what the kernels were written for       */
} dp_status;

/* Plan actions, one byte per saved tensor.  Section 4.3: the candidates of the
 * memory optimisation are the entries of every node's saved-tensor list, each
 * left alone, swapped or recomputed. */
typedef enum { DP_KEEP = 0, DP_RECOMPUTE = 1, DP_SWAP = 2 } dp_action;

typedef enum { DP_POST_LN = 0, DP_PRE_LN = 1 } dp_norm_style;
/* The feed-forward activation: GELU in its exact or tanh form, or ReLU (derivative 0 at 0). */
typedef enum { DP_GELU_ERF = 0, DP_GELU_TANH = 1, DP_ACT_RELU = 2 } dp_gelu_kind;
typedef enum { DP_F32 = 0, DP_BF16 = 1 } dp_dtype;
/* What the layers' normalisations compute: LayerNorm, or RMSNorm (T5's: no mean is subtracted,
 * y = gamma * x / sqrt(mean(x^2) + eps) + beta; a model without the additive term passes beta = 0
 * and ignores its gradient).  The *_STATS slots then hold 0 where the mean would be. */
typedef enum { DP_NORM_LAYER = 0, DP_NORM_RMS = 1 } dp_norm_kind;

/* Saved tensors ("slots") of one layer, in plan order.  T = micro_batch*seq.
 *   X_IN      [T,H]   layer input (stage input for layer 0; caller memory there)
 *   LN1_STATS [T,2]   fp32 (mean, 1/sqrt(var+eps)) of LayerNorm 1
 *   LN1_OUT   [T,H]
 *   QKV       [T,3H]  columns [Q | K | V], head h = columns h*dh..(h+1)*dh-1
 *   ATTN_LSE  [B,nh,S] fp32 log-sum-exp of the scaled logits
 *   ATTN_OUT  [T,H]
 *   RES1      [T,H]   X_IN + ATTN_OUT*Wo + bo
 *   LN2_STATS [T,2]
 *   LN2_OUT   [T,H]   pre-LN only (post-LN: it is the layer output; ignored)
 *   FC1_OUT   [T,F]
 *   GELU_OUT  [T,F]
 *   RES2      [T,H]   post-LN only (pre-LN: it is the layer output; ignored)
 */
enum {
  DP_SLOT_X_IN = 0, DP_SLOT_LN1_STATS, DP_SLOT_LN1_OUT, DP_SLOT_QKV, DP_SLOT_ATTN_LSE,
  DP_SLOT_ATTN_OUT, DP_SLOT_RES1, DP_SLOT_LN2_STATS, DP_SLOT_LN2_OUT, DP_SLOT_FC1_OUT,
  DP_SLOT_GELU_OUT, DP_SLOT_RES2, DP_SLOTS_PER_LAYER
};
/* A stage with a cross-attention block (mem_seq > 0) has seven more slots per layer, after
 * those above; its plans have DP_SLOTS_PER_LAYER_CROSS bytes a layer.  Tm = micro_batch*mem_seq.
 *   LNC_STATS  [T,2]    fp32 statistics of the block's LayerNorm
 *   LNC_OUT    [T,H]
 *   Q_C        [T,H]    queries
 *   KV_C       [Tm,2H]  columns [K | V] projected from the encoder memory (its producer reads
 *                       no slot: a RECOMPUTE of it repeats the projection of the memory)
 *   ATTN_C_LSE [B,nh,S] fp32
 *   ATTN_C_OUT [T,H]
 *   RES_C      [T,H]    RES1 + ATTN_C_OUT*Wo_c + bo_c */
enum {
  DP_SLOT_LNC_STATS = DP_SLOTS_PER_LAYER, DP_SLOT_LNC_OUT, DP_SLOT_Q_C, DP_SLOT_KV_C, DP_SLOT_ATTN_C_LSE,
  DP_SLOT_ATTN_C_OUT, DP_SLOT_RES_C, DP_SLOTS_PER_LAYER_CROSS
};

/* A stage = n_layers identical transformer layers on one micro-batch.
 *   pre-LN : a=LN1(x); m=x+Attn(a*Wqkv+b)*Wo+bo; c=LN2(m); y=m+GELU(c*W1+b1)*W2+b2
 *   post-LN: r1=x+Attn(x*Wqkv+b)*Wo+bo; m=LN1(r1); r2=m+GELU(m*W1+b1)*W2+b2; y=LN2(r2)
 * The paper names the workloads only (BERT, GPT-2; Section 5.1); the layer
 * mathematics is the textbook one.  No padding mask.  Dropout (off when both rates
 * are 0) acts where those models apply it: on the attention probabilities
 * (p_attn) and on the outputs of the attention projection and of FC2 before the
 * residual add (p_hidden).  Whether an element is kept is a pure function of
 * (seed, micro-batch counter, layer, site, position) -- see dp_stage_set_rng --
 * so a recomputed tensor and the backward pass see the mask the forward saw.
 * dtype DP_BF16: weights, slots, outputs and gradients are bf16, accumulation
 * and statistics fp32.  DP_F32: everything fp32 (debug mode).
 * mem_seq > 0 makes the stage a decoder stage of an encoder-decoder model (T5 is among the
 * workloads of Section 5.1): every layer gets a cross-attention block between its attention
 * and its feed-forward block, whose keys and values come from the encoder memory
 * mem [micro_batch*mem_seq, H], the same for all layers:
 *   pre-LN : r1 = x+Attn(..)*Wo+bo;  rc = r1 + CrossAttn(LNc(r1)*Wq+bq, mem*Wkv+bkv)*Wo_c+bo_c;
 *            y = rc+GELU(LN2(rc)*W1+b1)*W2+b2        (no mask in the cross-attention)
 * and the step also returns dMem, the sum over layers of the gradient reaching mem.  Dropout
 * acts in the block as in the rest of the layer: p_attn on its attention probabilities, p_hidden
 * on the output of its projection.  Such a stage needs norm_style DP_PRE_LN (DP_E_UNSUPPORTED
 * otherwise), its block's parameters from dp_stage_set_cross and its memory buffers from
 * dp_stage_bind_memory.  The validator, the plan generator, the cost model and the
 * partitioner (a chain of such layers, all reading the same memory) take it like any stage. */
typedef struct {
  int32_t n_layers, hidden, n_heads, ffn, seq, micro_batch;
  int32_t norm_style; /* dp_norm_style */
  int32_t causal;     /* 0: full attention, 1: causal mask */
  int32_t gelu_kind;  /* dp_gelu_kind */
  int32_t dtype;      /* dp_dtype */
  float ln_eps;
  float p_attn, p_hidden; /* dropout rates in [0, 1); 0 = none */
  int32_t mem_seq;        /* 0: no cross-attention block; > 0: length of the encoder memory */
  int32_t norm_kind;      /* dp_norm_kind */
} dp_stage_config;

/* Device pointers.  Linear weights are [in, out] row-major (y = x*W + b);
 * w_qkv is [H, 3H]; element type = config dtype.  Caller-owned. */
typedef struct {
  const void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  const void *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} dp_layer_weights;

/* Device pointers receiving the weight gradients: same shapes, layouts and
 * dtype as the weights.  dp_stage_step overwrites them; dp_stage_backward
 * overwrites or, with DP_GRAD_ACCUMULATE, adds to them.  Caller-owned. */
typedef struct {
  void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  void *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} dp_layer_grads;

/* Memory report of one plan.  peak_bytes follows the running-peak walk of
 * Algorithm 2 (add what a node allocates, take the max, subtract what it
 * releases), carried over forward, replay and backward:
 *   peak_bytes = fixed_bytes + arena_peak_bytes, where
 *   fixed_bytes      = library weight copies + caller's weights, gradients, x, dy, y, dx
 *   arena_peak_bytes = high-water mark of the library's activation arena under
 *                      the same offset allocator dp_stage_step uses
 *   live_peak_bytes  = fixed_bytes + max over time of the sum of live arena
 *                      blocks (the walk without fragmentation) */
typedef struct {
  uint64_t peak_bytes, live_peak_bytes, fixed_bytes, arena_peak_bytes;
  uint64_t weight_bytes, grad_bytes, kept_act_bytes;
  uint64_t swap_out_bytes, swap_in_bytes, host_pinned_bytes;
  double replay_flops, step_flops;
  int32_t n_replayed_ops, n_swapped_slots;
  int32_t first_bad_layer, first_bad_slot; /* -1 if none */
  /* launches of a bf16 stage that this shape sends to the vector-ALU kernels instead of the
   * matrix cores (a GEMM with a contraction that is no multiple of 8 or an unaligned operand,
   * attention with a head dimension other than 64 or 128): 20-50 times slower each; 0 for every
   * shape the kernels were written for */
  int32_t n_fallback_launches;
} dp_plan_report;

/* Statistics of one step (asking for them makes dp_stage_step wait for the step).  The times
 * come from HIP events: step/fwd/bwd on the caller's stream; d2h_busy_ms and h2d_busy_ms are
 * the summed durations of the plan's copies, each bracketed on the copy stream it ran on;
 * swap_wait_ms is the time the compute stream spent waiting for a swap-in it needed, or for a
 * block handed on behind a copy-out (what the swaps cost that did not overlap with
 * computation, Section 4.3); replay_ms the time of the recomputed forward nodes. */
typedef struct {
  float step_ms, fwd_ms, bwd_ms;
  uint64_t d2h_bytes, h2d_bytes, arena_high_water, peak_bytes;
  int32_t n_kernel_launches, n_replayed_ops;
  float replay_ms, d2h_busy_ms, h2d_busy_ms, swap_wait_ms;
  int32_t n_fallback_launches; /* as in dp_plan_report */
} dp_step_stats;

/* Kernel classes for dp_stage_op_times. */
enum {
  DP_OPC_GEMM_FWD = 0, DP_OPC_GEMM_DGRAD, DP_OPC_GEMM_WGRAD, DP_OPC_ATTN_FWD, DP_OPC_ATTN_BWD,
  DP_OPC_LN_FWD, DP_OPC_LN_BWD, DP_OPC_GELU_FWD, DP_OPC_GELU_BWD, DP_OPC_REDUCE, DP_OPC_DROPOUT, DP_OPC_COUNT
};

/* Number of plan bytes: n_layers * DP_SLOTS_PER_LAYER (DP_SLOTS_PER_LAYER_CROSS with
 * mem_seq > 0); 0 if cfg is invalid.  plan[l*slots_per_layer + slot] is a dp_action. */
size_t dp_plan_len(const dp_stage_config *cfg);

/* Pure host code: walks the step's schedule under `plan` and fills `report`
 * (nullable).  Feasible iff inflight * peak_bytes <= budget_bytes (Algorithm 1's
 * test (l-x+1)*M_x against M; a budget equal to the peak must run);
 * budget_bytes == 0 means "no limit"; inflight >= 1 is the number of
 * micro-batches whose activations the stage holds at once.
 * Errors: DP_E_INVAL (null cfg/plan, wrong plan_len, action > 2, bad config),
 * DP_E_PLAN (X_IN of layer 0 marked RECOMPUTE: it has no producer in the stage;
 * report->first_bad_* name it), DP_E_UNSUPPORTED (shape), DP_E_BUDGET.
 * Plan bytes of slots without storage (see the slot list) are ignored; SWAP on
 * X_IN of layer 0 is treated as KEEP because that buffer is the caller's.
 * Swap policy: with budget_bytes == 0 a swapped-out block returns to the
 * allocator as soon as its copy-out is queued (smallest peak; its next user
 * waits for the copy) and the swap-ins of a layer are issued one layer of
 * backward ahead of it.  With a budget, the headroom is spent on the swaps,
 * from the most generous policy down, and the first whose peak fits is taken:
 * swap-ins as many layers ahead as the stage is deep, then half as many, ...,
 * then one; for each distance, swapped-out blocks held back until the backward
 * has released them and the copy-outs of all but the bottom layers queued only
 * when the forward has been issued, in the order the backward asks for them;
 * then the same with every copy-out queued as its tensor is produced; then
 * blocks held until the forward is over, then for ever shorter spans, then not
 * at all.  Computation then waits for the host link as little
 * as the memory allows.  dp_stage_step makes the same choice, so its arena has
 * exactly the validated size. */
dp_status dp_plan_validate(const dp_stage_config *cfg, const uint8_t *plan, size_t plan_len,
                           uint64_t budget_bytes, uint32_t inflight, dp_plan_report *report);

/* ---- plan generator: the memory-optimisation step in front of the stage step -----------
 * Section 4.3: the candidates are the saved tensors; they are rated by FreeTime and by
 * memory saving per second, the two quantities of the cost model the section cites;
 * swapping is applied while the transfers still overlap with computation, after that every
 * step takes the cheaper of swapping and recomputation; the plan must fit the device
 * (Algorithm 1's test) and a stage is judged by T_x + T_x^moo (Section 4.2).
 *
 * Cost model of one layer (all layers of a stage are alike).  Node order, forward:
 *   pre-LN  LN1, QKV, ATTN, PROJ, LN2, FC1, GELU, FC2     post-LN  QKV, ATTN, PROJ, LN1, FC1, GELU, FC2, LN2
 * backward (execution order):
 *   pre-LN  FC2, GELU, FC1, LN2, PROJ, ATTN, QKV, LN1     post-LN  LN2, FC2, GELU, FC1, LN1, PROJ, ATTN, QKV
 * A backward node's time covers all its kernels (input and weight gradients, reductions).
 * A decoder layer (mem_seq > 0) has thirteen nodes; forward:
 *   LN1, QKV, ATTN, PROJ, LNC, QC, KVC, ATTNC, PROJC, LN2, FC1, GELU, FC2
 * backward:
 *   FC2, GELU, FC1, LN2, PROJC, ATTNC, KVC, QC, LNC, PROJ, ATTN, QKV, LN1
 * (LNC, QC, KVC, ATTNC, PROJC: the cross-attention block's LayerNorm, query projection,
 * key/value projection of the memory, attention and output projection); nodes 0..7 of these
 * orders are fwd_ns / bwd_ns, nodes 8..12 are fwd_more_ns / bwd_more_ns. */
typedef struct {
  int64_t fwd_ns[8], bwd_ns[8];                /* nanoseconds per node */
  uint64_t d2h_bytes_per_us, h2d_bytes_per_us; /* host link speed each way, one direction busy */
  /* The same with both directions busy at once (0 = not known, the figures above are used).
   * The planners take these for a stage that keeps two or more micro-batches in flight: in
   * the steady state of a one-forward-one-backward schedule the copy-outs of one micro-batch
   * and the copy-ins of another run side by side all the time. */
  uint64_t d2h_duplex_bytes_per_us, h2d_duplex_bytes_per_us;
  int64_t fwd_more_ns[5], bwd_more_ns[5];      /* decoder layers only: nodes 8..12 (else ignored) */
} dp_cost_model;

typedef struct {
  int64_t step_ns;      /* modelled step time */
  uint64_t peak_bytes;  /* fixed_bytes + running peak of the saved tensors (Algorithm 2's walk) */
  uint64_t d2h_bytes, h2d_bytes;
  int32_t n_replayed_ops;
} dp_plan_cost_report;

typedef struct {
  int32_t feasible;
  int64_t base_ns, moo_ns;        /* T_x of the unoptimised step and T_x^moo the plan adds (model) */
  uint64_t peak_bytes;            /* model peak of the plan */
  int32_t n_free_swaps, n_paid_swaps, n_recomputed;
  /* DP_MEMOPT_VALIDATE only: */
  uint64_t validated_peak_bytes;  /* dp_plan_validate's peak_bytes of the plan */
  int64_t exact_step_ns;          /* the model's clocks on the executor's own arena and hold policy */
  int32_t refine_rounds;
} dp_memopt_report;

enum { DP_MEMOPT_VALIDATE = 1 };

/* Pure host code.  Plays one step under `plan` on three clocks (compute, copy-out, copy-in)
 * with the executor's event rules: a swap-out starts when its tensor's last forward reader
 * is done and the copy-out stream is free; the swap-ins of layer l-1 are issued when the
 * backward of layer l starts, in the order the backward reads them, each behind its own
 * copy-out; a backward node waits for the
 * swap-ins it reads; recomputed tensors are regenerated on the compute clock before their
 * first backward reader.  Memory is the saved tensors only (no transient gradients, no
 * fragmentation); fixed_bytes is added to the peak.  Errors as dp_plan_validate, plus
 * DP_E_INVAL for a null or negative cost model or a zero link speed. */
dp_status dp_plan_cost(const dp_stage_config *cfg, const dp_cost_model *cm, const uint8_t *plan,
                       size_t plan_len, uint64_t fixed_bytes, dp_plan_cost_report *report);

/* Pure host code.  Writes a plan to plan_out[plan_len] (host) whose inflight * peak fits
 * budget_bytes (0 = no limit: the all-KEEP plan):
 *   1. candidates by decreasing FreeTime = (first backward use - copy-in time) - (last
 *      forward use + copy-out time) on the unoptimised timeline; each is swapped if that
 *      does not lengthen the modelled step; the first that does ends the phase;
 *   2. until it fits: over all remaining candidates and both actions, the one with the
 *      largest (peak reduction) / (added time), ties to the smaller added time, then SWAP.
 * flags = 0: peak = fixed_bytes + saved tensors, as dp_plan_cost (the planner of the model).
 * flags = DP_MEMOPT_VALIDATE: fixed_bytes is ignored; the plan is checked with
 * dp_plan_validate and the model's budget lowered by the difference until the true peak fits.
 * DP_E_BUDGET if nothing fits (plan_out then holds the last attempt, report->feasible = 0). */
dp_status dp_plan_generate(const dp_stage_config *cfg, const dp_cost_model *cm, uint64_t budget_bytes,
                           uint32_t inflight, uint64_t fixed_bytes, uint32_t flags, uint8_t *plan_out,
                           size_t plan_len, dp_memopt_report *report);

/* Creates a stage on the current HIP device.  `layers` is a host array of
 * n_layers structs of device pointers; the weights are copied (and re-laid
 * out) into library-owned device memory before the call returns, so the caller
 * may free theirs.  arena_bytes_hint: initial size of the activation arena
 * (0 = size it on first use; it grows when a plan needs more).  The library
 * owns the arena (hipMalloc), the pinned host pool (hipHostMalloc, sized by the
 * first plan that swaps), two copy streams and its events. */
dp_status dp_stage_init(const dp_stage_config *cfg, const dp_layer_weights *layers,
                        uint64_t arena_bytes_hint, dp_stage **out);

/* One forward+backward step of the stage on one micro-batch.
 *   x_in  [T,H] device, read     dy     [T,H] device, read (gradient of y_out)
 *   y_out [T,H] device, written  dx_out [T,H] device, written
 *   dw: host array of n_layers structs of device pointers, all written.
 * All four activations and all gradients have the config dtype, row-major,
 * token t = b*seq + s.  Buffers must not overlap each other.
 * The plan is validated first: any error (see dp_plan_validate; inflight = 1)
 * is returned before anything is enqueued.  Work is enqueued on `hip_stream`
 * (a hipStream_t; NULL = the default stream) and on the library's copy streams,
 * which are joined back into hip_stream before return; the call does not wait
 * for this step unless `stats` is non-NULL, but it first waits (on the host) for
 * the step issued two calls earlier on the same handle, so that at most two
 * steps are in flight; a plan that swaps waits for the previous step as well.  DP_E_HIP after a partial enqueue
 * leaves the outputs undefined.  One step at a time per handle.
 * The results are bit-identical for every plan. */
dp_status dp_stage_step(dp_stage *st, const void *x_in, const void *dy, const uint8_t *plan,
                        size_t plan_len, uint64_t budget_bytes, void *y_out, void *dx_out,
                        const dp_layer_grads *dw, void *hip_stream, dp_step_stats *stats);

/* The step split at the point where a one-forward-one-backward pipeline schedule
 * splits it (Sections 1 and 4.1, Algorithm 1: stage x of l holds l - x micro-batches
 * between their forward and their backward, and a partition is feasible when
 * inflight * peak fits the device).
 *
 * dp_stage_forward runs the forward pass of one micro-batch under `plan` and
 * leaves its saved tensors (kept on the device, or on their way to pinned host
 * memory) in the micro-batch slot `slot` (0 <= slot < inflight <= 64).  Every
 * slot owns an arena of the plan's validated size, a pinned pool and its events,
 * allocated on first use and grown when a later plan needs more, so the device
 * memory the slots hold is inflight * arena_peak_bytes; the plan is validated
 * with this `inflight` against `budget_bytes` before anything is enqueued.
 * dp_stage_backward runs the backward pass of the micro-batch in `slot` and
 * frees the slot.  flags = 0 overwrites the gradients; DP_GRAD_ACCUMULATE adds
 * this micro-batch's gradients to what `dw` holds (in fp32, rounded once to the
 * config dtype), which is what a schedule does for every micro-batch after the
 * first of an optimiser step.
 *
 * Buffers and layouts as dp_stage_step.  x_in may be reused once the forward's
 * work on `hip_stream` has run; dy, dx_out and dw belong to the backward call.
 * Errors: DP_E_INVAL for a slot that is out of range, still occupied (forward)
 * or empty (backward), unknown flags, null buffers; the validator's errors
 * from the forward.  Calls on one handle are made from one thread; a backward
 * given another stream than its forward is ordered after it by an event.
 * The forward is ordered (on the device) after the backward that last used the
 * slot, and first waits on the host for the backward issued two calls earlier
 * (under a plan that swaps: for the slot's last backward), which bounds how far
 * the host runs ahead.
 * y_out and dx_out are bit-identical to dp_stage_step's for every plan; so are
 * the gradients of a backward with flags = 0. */
enum { DP_GRAD_ACCUMULATE = 1 };
dp_status dp_stage_forward(dp_stage *st, uint32_t slot, uint32_t inflight, const void *x_in,
                           const uint8_t *plan, size_t plan_len, uint64_t budget_bytes, void *y_out,
                           void *hip_stream);
dp_status dp_stage_backward(dp_stage *st, uint32_t slot, const void *dy, void *dx_out,
                            const dp_layer_grads *dw, uint32_t flags, void *hip_stream);

/* New parameter values for the stage (an optimiser step happened).  The values
 * are copied, on `hip_stream`, into a parameter version of the library's own
 * (layout and pointers as dp_stage_init); every later dp_stage_step and
 * dp_stage_forward uses it.  A micro-batch that is between its forward and its
 * backward keeps the version its forward used, so that both passes see the same
 * parameters while an asynchronous schedule updates them in between (Section 1:
 * stage x of l keeps l - x parameter versions for that reason); a version's
 * memory is reused once no slot holds it.  With no micro-batch in flight the
 * current version is overwritten in place (ordered after its last reader).
 * dp_stage_weight_versions returns how many versions are alive (held by a slot,
 * or current): at most the micro-batches in flight plus one, each of
 * dp_plan_report.weight_bytes. */
dp_status dp_stage_set_weights(dp_stage *st, const dp_layer_weights *layers, void *hip_stream);
int32_t dp_stage_weight_versions(const dp_stage *st);

/* Diagnostics: copies one saved tensor of the micro-batch that dp_stage_forward left in
 * `slot` (its backward not yet issued) to dst (device, exactly the tensor's size in bytes:
 * the slot list gives the shape, the stage's dtype the element size), ordered on hip_stream
 * behind that forward.  For tests that need a decision the stage took on a stored value
 * (the sign ReLU's derivative reads, R32-style comparisons) rather than a recomputed one.
 * Errors: DP_E_INVAL (no micro-batch in the slot, layer or tensor out of range, a tensor
 * without storage of its own, wrong dst_bytes), DP_E_PLAN (the plan did not KEEP the tensor:
 * it is not on the device). */
dp_status dp_stage_read_saved(dp_stage *st, uint32_t slot, uint32_t layer, uint32_t tensor, void *dst,
                              size_t dst_bytes, void *hip_stream);

/* Dropout state (only matters when the configuration has a non-zero rate).  A mask is a
 * pure function of (seed, micro-batch number, layer, site, position): every dp_stage_step and
 * dp_stage_forward takes the current micro-batch number and increments it, so successive
 * micro-batches draw different masks, and a caller that sets (seed, counter) again gets the
 * same masks again.  The generator (a keyed 32-bit integer mixer over the element index; an
 * element is kept when its 32 bits are >= floor(p * 2^32), kept values are scaled by
 * 1/(1-p)) is stated in full in csrc/common.h.  Defaults: seed 0, counter 0. */
dp_status dp_stage_set_rng(dp_stage *st, uint64_t seed, uint64_t counter);

/* Decoder stages (mem_seq > 0).  Parameters of the cross-attention block of each layer, device
 * pointers in the stage's dtype, caller-owned, copied by dp_stage_set_cross on `hip_stream` into
 * the current parameter version (required once after dp_stage_init).  They are versioned with
 * the rest: a version made by dp_stage_set_weights starts with the block of the version before
 * it, and a dp_stage_set_cross after it gives the new version its own; a version that a
 * micro-batch in flight still uses cannot be overwritten (DP_E_INVAL):
 *   ln_g, ln_b [H];  w_q [H,H], b_q [H];  w_kv [H,2H] = [Wk | Wv], b_kv [2H];  w_o [H,H], b_o [H]
 * (matrices [in, out] row-major, as dp_layer_weights).  dp_cross_grads: where their gradients
 * go, same shapes; written as dp_layer_grads is: overwritten, or added to with
 * DP_GRAD_ACCUMULATE. */
typedef struct {
  const void *ln_g, *ln_b, *w_q, *b_q, *w_kv, *b_kv, *w_o, *b_o;
} dp_cross_weights;
typedef struct {
  void *ln_g, *ln_b, *w_q, *b_q, *w_kv, *b_kv, *w_o, *b_o;
} dp_cross_grads;
dp_status dp_stage_set_cross(dp_stage *st, const dp_cross_weights *layers, void *hip_stream);
/* The buffers the following calls use: mem [micro_batch*mem_seq, H] (read by dp_stage_step and
 * dp_stage_forward; a micro-batch between forward and backward keeps the pointer its forward
 * saw, and the caller keeps that memory unchanged until its backward has run, since a
 * recomputed KV_C reads it again), d_mem (same shape; overwritten by dp_stage_step and by every
 * dp_stage_backward with the sum over layers, each layer's share added in bf16 or fp32 as the
 * dtype says) and dw_cross[n_layers] (copied here).  All device memory, caller-owned; d_mem
 * and dw_cross may be NULL for a caller that only runs dp_stage_forward. */
dp_status dp_stage_bind_memory(dp_stage *st, const void *mem, void *d_mem, const dp_cross_grads *dw_cross);

/* Per-kernel-class timing of later steps: when enabled, every kernel launch is
 * bracketed by HIP events on the stream it runs on.  dp_stage_op_times waits
 * for the device, then returns (and clears) the summed milliseconds and launch
 * counts per class since the last call; arrays of DP_OPC_COUNT entries. */
dp_status dp_stage_set_profiling(dp_stage *st, int32_t enabled);
dp_status dp_stage_op_times(dp_stage *st, float *ms_by_class, uint64_t *launches_by_class);
/* Algorithmic work of the GEMM launches bracketed since the last call, 2*M*N*K each, summed per
 * class (DP_OPC_GEMM_FWD counts replayed forward GEMMs as well; the other classes stay 0), so
 * that a rate can be formed from exactly the launches that were timed.  Clears the sums. */
dp_status dp_stage_op_flops(dp_stage *st, double *flops_by_class);

/* The pipeline partition search (Section 4.2, Algorithm 1: AdjacentPartition and BiPar; the
 * compute- and memory-balanced positions of Appendix B.1, Algorithm 2; dp_plan_generate's
 * planner as MemOpt) for a chain of chain_cfg->n_layers identical layers cut into n_stages
 * stages between layers.  Host only.
 *   A layer costs the sum of the cost model's node times plus extra_ns[l] (nullable: work tied
 *   to layer l that memory optimisation cannot touch, e.g. an embedding or an output head) and
 *   holds fixed_per_layer + extra_bytes[l] (nullable) bytes of parameters, gradients and
 *   optimiser state besides its saved tensors; a stage holds fixed_per_stage more.  Stage x of
 *   l keeps l - x + 1 micro-batches and parameter versions (Appendix B.1) and fits when
 *   (l - x + 1) * peak <= budget_bytes (0 = no limit).
 *   Both traversals run from the compute-balanced to the memory-balanced cut and stop where
 *   no memory optimisation was needed; if no position of that interval fits, they go on past
 *   the memory-balanced cut to the first one that does (beyond the paper, whose theorem
 *   assumes that memory can be optimised away evenly).
 * flags = DP_MEMOPT_VALIDATE: a stage's memory is what dp_plan_validate reports for its plan
 *   (library weight copies, gradients, buffers, arena with its transients and fragmentation)
 *   plus its extra_bytes, and MemOpt runs as dp_plan_generate does under that flag (a stage's
 *   time is then the report's exact_step_ns), so every stage of the result is executable
 *   within the budget; fixed_per_layer and fixed_per_stage
 *   still steer the memory-balanced walk.  The balance walks and the traversal are unchanged.
 * Outputs: cuts_out[n_stages-1] (first layer of stages 2..l), plan_out (the stages' plans one
 * after the other, n_layers * DP_SLOTS_PER_LAYER bytes; each stage's first X_IN is KEEP),
 * stages_out[n_stages], report (nullable).  The objective is time_ns = max over stages of
 * T_x + T_x^moo.  Returns DP_E_BUDGET, with the outputs of the last position tried, if nothing
 * fits; DP_E_INVAL for n_stages outside 1..min(32, n_layers), null outputs, negative extras. */
typedef struct {
  int32_t first_layer, n_layers, inflight, used_memopt;
  int64_t time_ns, base_ns, moo_ns;  /* time = base (Eq. 1 plus extras) + moo; INT64_MAX: does not fit */
  uint64_t peak_bytes;               /* model peak of one micro-batch */
} dp_partition_stage;
typedef struct {
  int32_t feasible, any_memopt;
  int64_t time_ns;
  int32_t rho_cb, rho_mb;            /* outermost level: cut after stage n_stages/2 */
  int32_t n_memopt, n_positions;     /* MemOpt runs and positions visited */
} dp_partition_report;
dp_status dp_partition(const dp_stage_config *chain_cfg, const dp_cost_model *cm, int32_t n_stages,
                       uint64_t budget_bytes, uint64_t fixed_per_layer, uint64_t fixed_per_stage,
                       const int64_t *extra_ns, const uint64_t *extra_bytes, uint32_t flags,
                       int32_t *cuts_out, uint8_t *plan_out, size_t plan_len,
                       dp_partition_stage *stages_out, dp_partition_report *report);

/* Fills a cost model from this stage on this machine: `steps` all-KEEP steps with every
 * launch bracketed (node times averaged over layers and steps), then a block of FC1_OUT's
 * size copied four times each way through pinned host memory on the library's copy
 * streams, first one direction at a time, then both at once (the two-way figures).  Buffers as dp_stage_step (they are overwritten).  Waits for the device. */
dp_status dp_stage_measure_cost_model(dp_stage *st, const void *x_in, const void *dy, void *y_out,
                                      void *dx_out, const dp_layer_grads *dw, void *hip_stream,
                                      int32_t steps, dp_cost_model *out);

/* Debug switches, all default 0: bit 0 = serialise (copies on the compute
 * stream, no overlap); bit 1 = poison arena blocks with NaN patterns when they
 * are released (catches use-after-release and late swap-in); bit 2 = produce the
 * forward GELU in the FC1 GEMM epilogue instead of as its own kernel (results must
 * be the same bits either way); bit 3 = dp_stage_forward under a plan that swaps
 * does not wait for the slot's last backward (timing experiments). */
dp_status dp_stage_set_debug(dp_stage *st, uint32_t flags);

void dp_stage_destroy(dp_stage *st);

/* Text of the calling thread's last error ("" if none); static storage. */
const char *dp_last_error(void);

/* Standalone operator entry points (device pointers, row-major, enqueue on
 * `hip_stream`, no host wait).  They run the same kernels dp_stage_step uses
 * and exist for operator-level parity tests and microbenchmarks.
 * `ws` is a device workspace of at least dp_op_workspace_bytes(...) bytes
 * (needed by the ops that reduce over rows; may be NULL otherwise).
 * Empty inputs are valid: with a zero extent nothing is read (the corresponding
 * pointers may be NULL), sums over no rows are written as zeros, and a GEMM with
 * K = 0 writes bias + res. */
size_t dp_op_workspace_bytes(int32_t rows, int32_t cols);

/* y = LayerNorm(x)*gamma+beta per row of [rows, cols]; stats [rows,2] fp32
 * (mean, rstd); y or stats may be NULL (not written). */
dp_status dp_op_layernorm_fwd(int32_t dtype, int32_t rows, int32_t cols, float eps, const void *x,
                              const void *gamma, const void *beta, void *y, float *stats, void *hip_stream);
/* dx = [dres +] LayerNorm-backward(dy); dgamma, dbeta over all rows; dx_colsum
 * (nullable, [cols]) receives the column sums of dx as stored.  dy may be dx. */
dp_status dp_op_layernorm_bwd(int32_t dtype, int32_t rows, int32_t cols, const void *dy, const void *x,
                              const float *stats, const void *gamma, const void *dres /*nullable*/,
                              void *dx, void *dgamma, void *dbeta, void *dx_colsum /*nullable*/, void *ws,
                              void *hip_stream);
/* The same two with RMSNorm (DP_NORM_RMS): y = gamma * x / sqrt(mean(x^2) + eps) + beta, no mean
 * subtracted; stats holds (0, 1/sqrt(mean(x^2) + eps)). */
dp_status dp_op_rmsnorm_fwd(int32_t dtype, int32_t rows, int32_t cols, float eps, const void *x,
                            const void *gamma, const void *beta, void *y, float *stats, void *hip_stream);
dp_status dp_op_rmsnorm_bwd(int32_t dtype, int32_t rows, int32_t cols, const void *dy, const void *x,
                            const float *stats, const void *gamma, const void *dres /*nullable*/,
                            void *dx, void *dgamma, void *dbeta, void *dx_colsum /*nullable*/, void *ws,
                            void *hip_stream);
dp_status dp_op_gelu_fwd(int32_t dtype, int32_t gelu_kind, size_t n, const void *x, void *y, void *hip_stream);
/* dx = dy * gelu'(x) over [rows, cols], and dbias [cols] = the column sums of dx as stored (the
 * bias gradient of the linear layer in front of the activation): the one kernel the stage's
 * backward runs for this node.  dy may be dx.  ws: dp_op_workspace_bytes(rows, cols). */
dp_status dp_op_gelu_bwd(int32_t dtype, int32_t gelu_kind, int32_t rows, int32_t cols, const void *dy,
                         const void *x, void *dx, void *dbias, void *ws, void *hip_stream);
/* C[M,N] = op(A)*op(B) (+bias[N]) (+res[M,N]).  mode 0 ("NT"): A [M,K], B [N,K]
 * (both contraction-contiguous: forward with the transposed weight copy, and
 * dX = dY*W^T with W as stored); mode 1 ("TN"): A [K,M], B [K,N] (contraction
 * over the leading dimension of both: dW = X^T*dY).  res may be C itself
 * (C += op(A)*op(B), how gradients are accumulated); no other overlap. */
dp_status dp_op_gemm(int32_t dtype, int32_t mode, int32_t M, int32_t N, int32_t K, const void *A, const void *B,
                     const void *bias, const void *res, void *C, void *hip_stream);
/* out[cols] = sum over rows of x[rows, cols] */
dp_status dp_op_colsum(int32_t dtype, int32_t rows, int32_t cols, const void *x, void *out, void *ws,
                       void *hip_stream);
/* dp_op_colsum for callers that cannot allocate device memory and have no workspace to hand in
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * partial sums of the two-pass reduction go to a device array inside the library, 8 MiB on every
 * GPU the library runs on, held until the process ends.  Same kernels and same bits as
 * dp_op_colsum.  Calls neither hipMalloc nor hipFree nor any allocating routine.  Limit: the
 * partials, (number of row blocks, at most 512) x cols x 4 bytes, must fit the array, e.g.
 * cols <= 4096 at any row count; larger shapes are refused with DP_E_UNSUPPORTED and a message.
 * All calls on one GPU share the array: calls that overlap on one GPU (different streams or
 * threads) race; calls on one stream are ordered. */
dp_status dp_op_colsum_static(int32_t dtype, int32_t rows, int32_t cols, const void *x, void *out,
                              void *hip_stream);
/* o [T,H], lse [B,nh,S] from qkv [T,3H]; o or lse may be NULL.  (All attention entry points: in
 * bf16 with a head dimension of 64 or 128 the matrix-core kernels run; they move 16 bytes a lane,
 * so every tensor pointer handed in must then be 16-byte aligned, as allocations are; a pointer
 * that is not is refused with DP_E_HIP "invalid argument" before anything is launched.) */
dp_status dp_op_attention_fwd(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t dh, int32_t causal,
                              const void *qkv, void *o, float *lse, void *hip_stream);
/* dqkv [T,3H] from qkv, o, lse, d_o; ws: device workspace of
 * dp_op_workspace_bytes(T, nh) bytes. */
dp_status dp_op_attention_bwd(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t dh, int32_t causal,
                              const void *qkv, const void *o, const float *lse, const void *d_o, void *dqkv,
                              void *ws, void *hip_stream);

/* The same operations with dropout, as the stage applies it.  `drop` names the mask: rate,
 * seed, micro-batch number and layer (see dp_stage_set_rng); p = 0 gives the plain operation.
 * dp_op_dropout: y = (res ? res : 0) + mask * x / (1-p) over n elements (n a multiple of 8,
 * below 2^32; x and res may be y), site 1 = after the attention projection, 2 = after FC2,
 * 4 = after the projection of a decoder layer's cross-attention block; the
 * backward of a site is the same call on the gradient with res = NULL.
 * Attention: the probabilities are masked and scaled after the softmax (lse is that of the
 * plain softmax); the backward masks the same positions. */
typedef struct {
  float p;
  uint64_t seed, micro_batch;
  int32_t layer;
} dp_dropout;
dp_status dp_op_dropout(int32_t dtype, size_t n, const void *x, const void *res, void *y,
                        const dp_dropout *drop, int32_t site, void *hip_stream);
dp_status dp_op_attention_dropout_fwd(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t dh,
                                      int32_t causal, const void *qkv, void *o, float *lse,
                                      const dp_dropout *drop, void *hip_stream);
dp_status dp_op_attention_dropout_bwd(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t dh,
                                      int32_t causal, const void *qkv, const void *o, const float *lse,
                                      const void *d_o, void *dqkv, void *ws, const dp_dropout *drop,
                                      void *hip_stream);

/* Cross-attention, the decoder-side block of an encoder-decoder model (Section 5.1 lists T5
 * among the workloads; the paper does not define the layer mathematics): queries q [B*Sq, H]
 * attend, without a mask, to the keys and values of kv [B*Sk, 2H] = [K | V], per sample and per
 * head (head h = columns h*dh .. of each H-wide block):
 *   o [B*Sq, H] = softmax(Q K^T / sqrt(dh)) V,   lse [B, nh, Sq] (fp32) = log of the row sums.
 * o or lse may be NULL.  The backward writes dq [B*Sq, H] and dkv [B*Sk, 2H] from q, kv, o, lse
 * and d_o [B*Sq, H]; ws: device workspace of dp_op_workspace_bytes(B*Sq, nh) bytes.  drop: NULL,
 * or dropout of the probabilities as in dp_op_attention_dropout_* with positions
 * query*Sk + key at a site of its own (needs Sq*Sk < 2^32).  Empty inputs: no queries writes
 * nothing forward and dkv = 0 backward; queries without keys are DP_E_INVAL.  The same kernels
 * as self-attention, which is the case q, K, V = the three blocks of one tensor and Sq = Sk. */
dp_status dp_op_cross_attention_fwd(int32_t dtype, int32_t B, int32_t Sq, int32_t Sk, int32_t nh, int32_t dh,
                                    const void *q, const void *kv, void *o, float *lse, const dp_dropout *drop,
                                    void *hip_stream);
dp_status dp_op_cross_attention_bwd(int32_t dtype, int32_t B, int32_t Sq, int32_t Sk, int32_t nh, int32_t dh,
                                    const void *q, const void *kv, const void *o, const float *lse,
                                    const void *d_o, void *dq, void *dkv, void *ws, const dp_dropout *drop,
                                    void *hip_stream);

/* Diagnostic for reading the roofline: the rate at which the matrix cores issue
 * v_mfma_f32_32x32x16_bf16 when nothing else limits them (operands in registers, 16
 * independent accumulators a wave, one workgroup a CU, `iters` rounds), with the operand bits
 * taken from `data_bf16` (device, n_elems a multiple of 8), and the shader clock held over the
 * loop.  The clock, and with it the attainable rate, depends on the data: all-zero operands
 * run at the nominal clock, operands with random mantissas draw more power and run slower.
 * Allocates a small device buffer and waits for completion. */
dp_status dp_probe_mfma(const void *data_bf16, size_t n_elems, int32_t iters, float *tflops,
                        float *shader_mhz, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DPSTAGE_H */
