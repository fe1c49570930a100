/*
 * lynx.h - C ABI of the per-layer recompute-and-backward library for one
 * tensor-parallel shard of a GPT transformer block on one MI355X (gfx950).
 *
 * The paper (Lynx, arXiv 2406.08756) schedules which operator outputs of a
 * layer stay resident after the forward pass and where the discarded ones are
 * regenerated (Sec. 4.2 "Problem definition": Boolean S_i per operator,
 * recompute phases 1..5).  This library is the GPU-side mechanism under that
 * policy: a forward that keeps or drops each named activation, a recompute
 * call that regenerates a set of operators (one phase's segment), and a
 * backward that regenerates on demand whatever is still missing (phase 5,
 * the critical path) and then differentiates the layer.
 *
 * The layer is a chain of 13 operators; A_i is OP_i's output:
 *   A0 X (input)     A1 Y1=LN1(X)       A2 QKV=Y1 Wqkv^T+bqkv   A3 S=Q K^T
 *   A4 P=softmax     A5 Pd=dropout(P)   A6 C=Pd V               A7 O=C Wo^T
 *   A8 X2=X+drop(O+bo)  A9 Y2=LN2(X2)   A10 U=Y2 W1^T+b1        A11 G=gelu(U)
 *   A12 V2=G W2^T    A13 OUT=X2+drop(V2+b2)
 * Bit i of a retain mask is S_i; bit i of a segment mask means "run OP_i".
 *
 * General rules
 *  - Every pointer named "device" is device memory on the current HIP device,
 *    16-byte aligned; everything else is host memory.
 *  - The library never allocates or frees device memory and never
 *    synchronises: all work is enqueued on the caller's stream (a hipStream_t
 *    passed as void*; NULL is the default stream).
 *  - All argument checking happens on the host before anything is launched;
 *    a call that returns an error other than LYNX_ERR_HIP has launched nothing
 *    and changed no state.  After LYNX_ERR_HIP call lynx_layer_reset.
 *  - Tensors are row-major.  Tokens are batch-major (t = bi*seq + i).  QKV
 *    columns are ordered [q|k|v][head][head_dim].  Weights are [out, in].
 *    S, P, Pd are [micro_batch, local_heads, seq, seq]; only j <= i is defined
 *    for causal layers.
 *  - A handle is not thread-safe; distinct handles are independent.
 */
#ifndef LYNX_H
#define LYNX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lynx_layer_s* lynx_layer_t; /* opaque, library-owned (host) */

typedef enum {
  LYNX_OK = 0,
  LYNX_ERR_INVALID_ARG = 1, /* null/misaligned pointer, bad enum, bad mask */
  LYNX_ERR_SHAPE = 2,       /* dimension not supported (see lynx_layer_config) */
  LYNX_ERR_STATE = 3,       /* call order violated */
  LYNX_ERR_DEPENDENCY = 4,  /* segment names an operator whose input is absent */
  LYNX_ERR_OOM = 5,         /* workspace too small */
  LYNX_ERR_HIP = 6          /* a HIP call or kernel launch failed */
} lynx_status;

typedef enum { LYNX_F32 = 0, LYNX_BF16 = 1 } lynx_dtype;

/* Shape and constants of one shard.  Constraints (else LYNX_ERR_SHAPE):
 * hidden, head_dim, local_ffn, seq multiples of 8; all sizes > 0;
 * 0 <= dropout_p < 1; 0 <= tp_rank < tp_size; layer_id < 2^30; causal == 1. */
typedef struct {
  int32_t dtype;       /* lynx_dtype: storage type of activations, params, grads */
  int32_t hidden;      /* h */
  int32_t local_heads; /* a: attention heads on this rank */
  int32_t head_dim;    /* d */
  int32_t local_ffn;   /* f: FFN columns on this rank */
  int32_t seq;         /* s */
  int32_t micro_batch; /* b */
  int32_t tp_size;     /* tensor-parallel group size (only indexes dropout) */
  int32_t tp_rank;
  int32_t causal;
  float dropout_p;     /* same p at all three dropout sites */
  float ln_eps;
  uint64_t seed;       /* Philox key */
  uint32_t layer_id;   /* enters the Philox counter */
  uint32_t flags;      /* LYNX_FLAG_*; other bits must be 0 */
} lynx_layer_config;

/* Attention without the seq x seq tensors.  Under a retain mask that keeps none of S, P
 * and Pd (the tensors Selective Recomputation drops, Sec. 2.2) and for shapes the kernels
 * take (bf16, head_dim 128, seq a multiple of 128), operators 3-5 never run: operator 6
 * forms C from QKV in one launch and leaves two fp32 row statistics per (batch element,
 * head, row) behind C; backward rebuilds P and Pd from them tile by tile.  Then naming
 * operators 3-5 in a segment is a no-op, operator 6 depends on QKV alone, backward reads
 * QKV and C instead of P and Pd, and no seq x seq activation is ever allocated (one
 * seq x seq gradient, dS, remains as a transient of backward).  Every result is
 * bit-identical to the unfused kernels'.  It trades arithmetic for memory: the dropout
 * generator and the exponentials run once more per kernel that needs P, which on this chip
 * costs more time than the seq x seq traffic it saves; the peak workspace of a
 * full-recompute layer drops by about three seq x seq tensors.  Off by default. */
#define LYNX_FLAG_FUSED_ATTENTION 1u

/* Device pointers to the parameters, borrowed until the next set_params or
 * destroy.  Shapes: wqkv [3*a*d, h], bqkv [3*a*d], wo [h, a*d], bo [h],
 * w1 [f, h], b1 [f], w2 [h, f], b2 [h], LayerNorm g1, be1, g2, be2 [h]. */
typedef struct {
  const void *wqkv, *bqkv, *wo, *bo, *w1, *b1, *w2, *b2, *g1, *be1, *g2, *be2;
} lynx_params;

/* Device pointers to caller-owned gradient buffers of the same shapes and
 * dtype as the parameters; each is overwritten (not accumulated into). */
typedef struct {
  void *wqkv, *bqkv, *wo, *bo, *w1, *b1, *w2, *b2, *g1, *be1, *g2, *be2;
} lynx_grads;

/* Retain-mask presets (Sec. 2.2 of the paper: Full Recomputation keeps only
 * the layer input; Selective Recomputation drops the attention operators'
 * seq x seq tensors).  Bits 0 and 13 are always treated as set. */
#define LYNX_RETAIN_STORE_ALL 0x3FFFu
#define LYNX_RETAIN_FULL_RECOMPUTE 0x2001u
#define LYNX_RETAIN_ATTENTION_ONLY (0x3FFFu & ~0x0038u)   /* drop S, P, Pd */
#define LYNX_RETAIN_ELEMENTWISE_ONLY (0x3FFFu & ~0x0830u) /* drop P, Pd, G */
/* Segment meaning "whatever backward still needs, with its missing ancestors" */
#define LYNX_SEG_ALL_MISSING 0xFFFFFFFFu

#define LYNX_NUM_ACTIVATIONS 14

/* M_i of the paper's memory constraint (Eq. 8): bytes of activation act_id
 * (0..13) for this shape.  LayerNorm outputs (A1, A9) include their two fp32
 * per-token statistics, the context A6 two fp32 attention row statistics per
 * (batch element, head, row).  Returns 0 for a bad argument. */
size_t lynx_activation_bytes(const lynx_layer_config* cfg, int act_id);

/* Workspace (device bytes) that lynx_layer_create needs so that
 * forward(retain_mask) -> [recompute(ALL_MISSING)] -> backward fits, including
 * all transient buffers.  Found by replaying that call sequence against the
 * library's own (deterministic, first-fit) allocator without launching
 * anything, so it is exact for that sequence.  Explicit segments issued in
 * another order place buffers differently and can need more; a planner can
 * rehearse any sequence with lynx_layer_set_dry_run and read
 * lynx_layer_peak_bytes.  0 on a bad config. */
size_t lynx_workspace_bytes(const lynx_layer_config* cfg, uint32_t retain_mask);

/* The same for a schedule with explicit regeneration phases (Sec. 4.2: the
 * memory constraints, Eq. cons15-cons17, count what phases 1 and 2 bring back
 * on top of what the forward pass retained): the sequence rehearsed is
 * forward(retain_mask) -> recompute(phase_masks[0]) .. recompute(phase_masks[3])
 * (zero entries skipped) -> backward.  phase_masks (host, 4 entries) may be NULL,
 * which gives lynx_workspace_bytes.  Exact for that sequence; 0 on a bad config
 * or when a phase names an operator whose input is absent at that point. */
size_t lynx_workspace_bytes_for_schedule(const lynx_layer_config* cfg, uint32_t retain_mask,
                                         const uint32_t* phase_masks);

/* Create a layer over a caller-owned device workspace (borrowed until
 * destroy).  Errors: INVALID_ARG (null/misaligned), SHAPE. */
lynx_status lynx_layer_create(const lynx_layer_config* cfg, void* workspace_device,
                              size_t workspace_bytes, lynx_layer_t* out_layer);
lynx_status lynx_layer_destroy(lynx_layer_t layer);

/* lynx_layer_create for callers that cannot allocate device memory (code under
 * HIP graph capture, serving loops, harnesses that forbid hipMalloc): the
 * layer's workspace is a block of LYNX_STATIC_WORKSPACE_BYTES that is part of
 * the library's code object, so neither this call nor any later call on the
 * handle calls an allocation routine.  Each GPU has its own copy of the block,
 * held until the process ends; the layer uses the copy of the device that is
 * current at this call.  Everything else is lynx_layer_create: same kernels,
 * same bits.  The block keeps whatever the previous layer left in it (no
 * kernel reads workspace memory it has not written), and one layer at a time
 * may live in it per GPU: two would overwrite each other, so a second create on
 * the same device before the first is destroyed fails with STATE.  Errors:
 * INVALID_ARG, SHAPE, OOM when even the leanest schedule of this shape
 * (lynx_workspace_bytes(cfg, LYNX_RETAIN_FULL_RECOMPUTE)) exceeds the block -
 * later calls return OOM as usual when a richer retain mask does not fit -,
 * HIP when the block's address cannot be obtained. */
#define LYNX_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
lynx_status lynx_layer_create_static(const lynx_layer_config* cfg, lynx_layer_t* out_layer);

lynx_status lynx_layer_set_params(lynx_layer_t layer, const lynx_params* params);

/* Forward pass (operators 1..13) under a retain policy: after an operator's
 * last forward consumer has run, its output is released unless its retain bit
 * is set.  x_device [T, h] is borrowed and must stay valid and unchanged
 * until backward returns (it is the layer's checkpoint); out_device [T, h] is
 * written.  `step` selects the dropout masks (the Philox counter).
 * Errors: STATE (forward already pending), INVALID_ARG, OOM. */
lynx_status lynx_layer_forward(lynx_layer_t layer, const void* x_device, void* out_device,
                               uint32_t retain_mask, uint64_t step, void* hip_stream);

/* Regenerate a segment: the operators named in segment_mask run in index
 * order with the forward's kernels and launch geometry, so their outputs are
 * bit-identical to the forward's.  An operator whose output is resident is
 * skipped.  An operator with an absent input that no earlier operator of the
 * segment produces fails the whole call with DEPENDENCY (Eq. 4: a parent must
 * be stored or already regenerated).  Regenerated S, O or V2 (which backward
 * never reads) are released again as soon as their consumers are resident.
 * Errors: STATE (no forward pending), DEPENDENCY, OOM. */
lynx_status lynx_recompute(lynx_layer_t layer, uint32_t segment_mask, void* hip_stream);

/* Backward pass.  First regenerates everything still missing (phase 5), then
 * computes d_x_device [T, h] and all twelve parameter gradients from
 * d_out_device [T, h] (borrowed, read-only), releasing activations as it goes.
 * Afterwards the layer is idle again and holds nothing.
 * Errors: STATE, INVALID_ARG, OOM. */
lynx_status lynx_layer_backward(lynx_layer_t layer, const void* d_out_device, void* d_x_device,
                                const lynx_grads* grads, void* hip_stream);

/* Drop all resident activations and return to idle without a backward
 * (inference-style use, or abandoning a micro-batch). */
lynx_status lynx_layer_reset(lynx_layer_t layer);

/* Bookkeeping queries (host only, no GPU work).  live mask: bit i set iff A_i
 * is resident (bits 0 and 13 refer to the caller's buffers).  live bytes:
 * sum of M_i over resident A_1..A_12, i.e. sum_i S_i*M_i right after forward.
 * peak bytes: high-water mark of the workspace since create. */
lynx_status lynx_layer_live_mask(lynx_layer_t layer, uint32_t* live);
/* The operators LYNX_SEG_ALL_MISSING stands for right now (bit i = OP_i): those
 * whose outputs backward reads and that are not resident, plus, transitively,
 * their absent inputs - what phase 5 would run (Sec. 4.2).  STATE when no
 * forward is pending. */
lynx_status lynx_layer_missing_mask(lynx_layer_t layer, uint32_t* missing);
lynx_status lynx_layer_live_bytes(lynx_layer_t layer, size_t* bytes);
lynx_status lynx_layer_peak_bytes(lynx_layer_t layer, size_t* bytes);

/* Device address and size of a resident activation (for parity checks); the
 * pointer is NULL when the activation is not resident.  For A1 / A9 the
 * statistics follow the [T, h] tensor directly: mean[T] then rstd[T], fp32. */
lynx_status lynx_layer_activation(lynx_layer_t layer, int act_id, const void** device_ptr,
                                  size_t* bytes);

/* Parity aid for the backward pass (Sec. 4.2 places no requirement on it: the
 * method must leave every gradient unchanged, and this is how a test looks at
 * the ones that never reach the caller).  While device_dst is set for act_id,
 * every lynx_layer_backward also copies the gradient with respect to activation
 * A_act_id, as its kernels formed it, to device_dst on the call's stream:
 *   12 dV2 [T, h]   10 dU [T, f]   9 dY2 [T, h]   8 dX2 [T, h]   7 dO [T, h]
 *   6 dC [T, a*d]   3 dS [b, a, s, s] (j <= i defined)   2 dQKV [T, 3*a*d]
 *   1 dY1 [T, h]
 * in the storage dtype; device_dst holds that many elements (dS: the whole
 * dense [b, a, s, s] block is copied).  NULL clears the tap.
 * Other act_id (gradients no kernel materialises) -> INVALID_ARG. */
lynx_status lynx_layer_set_gradient_tap(lynx_layer_t layer, int act_id, void* device_dst);

/* Write the keep-mask of one dropout site as bytes (1 = keep) for parity
 * checks: site 0 -> [b, a, s, s] (all j, also above the diagonal), sites 1, 2
 * -> [T, h].  Masks are a pure function of (seed, step, layer_id, site,
 * element index) and are never stored by the library. */
lynx_status lynx_dropout_mask(const lynx_layer_config* cfg, uint64_t step, int site,
                              uint8_t* out_device, void* hip_stream);

/* When on, calls do all host bookkeeping (allocation, residency, errors) but
 * launch no kernel; pointers are then only checked for alignment.  Used by
 * lynx_workspace_bytes and by planners that want a policy's memory curve. */
lynx_status lynx_layer_set_dry_run(lynx_layer_t layer, int on);

/* Per-kernel timing, the hook for the paper's Model Profiler (Sec. 3: it
 * records each operator's execution time C_i).  While on, every kernel group
 * the layer enqueues is bracketed by a HIP event pair on the call's stream
 * (this adds a few microseconds per kernel, so leave it off when timing whole
 * calls).  lynx_layer_profile_ms blocks until the recorded events complete
 * and writes, per slot, the milliseconds of its most recent run since the
 * previous query, or -1 if it did not run.  Slots 1..13 are the forward
 * operators; an operator that ran inside the launch of the one before it has
 * no time of its own (-1) and is covered by that slot: OP5 by slot 4, and,
 * where the matrix-core kernels apply, OP8 by slot 7 and OP13 by slot 12.  The
 * rest are the backward kernels (likewise the GeLU backward may run inside
 * the FC2 gradient launch, and dPd with the softmax backward as one launch);
 * lynx_profile_slot_name names them ("" when unused). */
#define LYNX_PROFILE_SLOTS 40
lynx_status lynx_layer_set_profiling(lynx_layer_t layer, int on);
lynx_status lynx_layer_profile_ms(lynx_layer_t layer, float* ms_out /* [LYNX_PROFILE_SLOTS], host */);
const char* lynx_profile_slot_name(int slot);

/* ---- Single-layer recomputation policy (Sec. 4.2, "Lynx-HEU") ------------
 * Host only; no GPU is touched.  A layer of n_ops operators OP_1..OP_n; all
 * masks use bit i for OP_i (bit 0 is the layer input and is ignored on input).
 * The program solved is the paper's: minimise the regeneration time left on
 * the critical path, sum_i (1 - S_i) R_{5,i} C_i (Eq. objective2), subject to
 *   - each regenerated operator runs in exactly one phase (Eq. cons11);
 *   - OP_i may run in phase t only if each input OP_j is retained or was
 *     regenerated in a phase <= t, for every edge j -> i (Eq. cons12);
 *   - the time placed in phase t <= 4 fits the communication it overlaps,
 *     CTime_t (Eq. cons13); operators in comm_mask only run in phase 5 (cons14);
 *   - m_static + n_layer n_batch sum_i S_i M_i
 *       + n_layer sum_i (1 - S_i)(R_{1,i} + R_{2,i}) M_i <= m_budget
 *     (Eq. cons15-17), with S_n = 1;
 *   - last_stage != 0: phases 1 and 2 do not exist and the third memory term
 *     is dropped ("Optimizations").
 * Where the text sums Eq. cons11 over every operator, an operator is
 * regenerated here only when required: needed_mask names the operators whose
 * outputs backward reads; a discarded one must be regenerated, and so must
 * every discarded input of a regenerated operator.  needed_mask = all ones
 * gives the model exactly as printed.
 * Exact search, exponential in n_ops (n_ops <= 24; a GPT layer has 13).
 * Among equal critical-path times the least total regenerated time wins, then
 * the lower peak.  Returns LYNX_ERR_OOM when no policy fits the budget,
 * LYNX_ERR_INVALID_ARG for null arrays, negative numbers, n_ops out of range
 * or an input that is not an earlier operator. */
typedef struct {
  int32_t n_ops;
  const double* cost;      /* C_i, any time unit, n_ops entries (host) */
  const double* bytes;     /* M_i, n_ops entries (host) */
  const uint32_t* parents; /* n_ops masks: bit j of parents[i-1] = OP_j feeds OP_i, j < i (host) */
  uint32_t comm_mask;
  uint32_t needed_mask;
  double ctime[4];         /* CTime_1..4, same unit as cost */
  double m_budget, m_static;
  int32_t n_layer, n_batch;
  int32_t last_stage;
} lynx_policy_problem;

typedef struct {
  uint32_t retain_mask;    /* S_i; bit 0 always set; usable as a forward retain mask */
  uint32_t phase_mask[5];  /* operators regenerated in phase 1..5; 1..4 usable as recompute segments */
  double critical_cost;    /* the objective */
  double recompute_cost;   /* time regenerated over all five phases */
  double peak_bytes;       /* left side of Eq. cons15 */
} lynx_policy;

lynx_status lynx_policy_solve(const lynx_policy_problem* problem, lynx_policy* policy_out);

/* ---- Recomputation-aware model partitioning (Sec. 5) -----------------------
 * Host only.  n_total_layers identical layers are dealt to n_stages pipeline
 * stages by the section's greedy search: (1) equal shares (the remainder one
 * each to the first stages); (2) every stage's policy from lynx_policy_solve;
 * (3) every stage's time; (4) one layer moves from the slowest stage to the
 * fastest; the move is kept if every stage still fits its memory and the
 * slowest stage became faster; (5) otherwise the current scheme is the answer.
 * The section prints no formula for its training cost model; the one used: a
 * stage's time per micro-batch = its layers x (t_fwd + t_bwd + the policy's
 * critical_cost), stage s holds n_stages - s forward passes before its first
 * backward (one-forward-one-backward), the last stage uses the last-stage
 * variant, and a stage's static bytes are static_per_layer x its layers.  Of
 * `layer`, the fields n_layer, n_batch, last_stage, m_static and m_budget are
 * ignored (set per stage).  layers_out[n_stages], time_out[n_stages] and, if
 * not NULL, policies_out[n_stages] are caller arrays.  Errors: INVALID_ARG
 * (also n_stages > 64 or fewer layers than stages), OOM when the equal-share
 * scheme does not fit. */
typedef struct {
  const lynx_policy_problem* layer;
  int32_t n_total_layers, n_stages;
  double t_fwd, t_bwd;       /* per layer and micro-batch, same unit as layer->cost */
  double static_per_layer;   /* bytes of weights, gradients and optimizer state per layer */
  double m_budget;           /* bytes per GPU */
} lynx_partition_problem;

lynx_status lynx_partition_solve(const lynx_partition_problem* problem, int32_t* layers_out,
                                 double* time_out, lynx_policy* policies_out);

/* Fills the layer-shaped parts of a problem for this library's 13-operator
 * block: n_ops = 13, parents, needed_mask (what lynx_layer_backward reads),
 * comm_mask = 0 (a shard has no communication operator) and bytes = M_i of
 * `cfg` (lynx_activation_bytes).  parents_out[13] and bytes_out[13] are caller
 * arrays the problem will point into; cost, ctime, budget and counts stay the
 * caller's to set.  Errors: INVALID_ARG, SHAPE. */
lynx_status lynx_policy_layer_problem(const lynx_layer_config* cfg, lynx_policy_problem* problem_out,
                                      uint32_t* parents_out, double* bytes_out);

/* Measurement aid, not part of the method: a device copy of `bytes` (multiple of
 * 16; both pointers device, 16-byte aligned, not overlapping) done by a fixed
 * number of workgroups (1..4096), enqueued on `hip_stream`.  It stands in for the
 * tensor-parallel all-reduce that the paper overlaps regeneration with (Sec. 4,
 * phases 1-4) when that overlap is measured on one GPU: a bounded number of
 * compute units and a bounded share of memory bandwidth, busy for a while.
 * Errors: INVALID_ARG, HIP. */
lynx_status lynx_comm_standin(void* dst_device, const void* src_device, size_t bytes, int workgroups,
                              void* hip_stream);

const char* lynx_status_string(lynx_status status);

#ifdef __cplusplus
}
#endif
#endif /* LYNX_H */
