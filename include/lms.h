/*
 * lms.h -- C ABI of the MI355X large-model-support library.
 *
 * The library takes a user-defined computational graph of a CNN training step,
 * rewrites it with swap-out / swap-in operations so that it runs inside a
 * device-memory budget, and executes the rewritten graph on one GPU
 * (paper: Figure "TFLMS module", Section 5: user model -> graph rewriting -> session).
 *
 * Conventions
 *  - every call returns an lms_status (0 = OK, negative = error); after an error
 *    lms_last_error() gives a thread-local message.  Nothing throws or aborts.
 *  - handles (lms_graph*, lms_exec*) are owned by the library until *_destroy.
 *  - a vertex ("node") has exactly one output tensor; a tensor is named by the id
 *    of the node producing it.  Ids are dense, in creation order.
 *  - activations are channels-last: (N, H, W, C) or (N, D, H, W, C); convolution
 *    filters are (R, S, C, K) or (T, R, S, C, K); bf16 storage, fp32 accumulation;
 *    weight gradients, affine/bias parameters and their gradients are fp32.
 *  - "device" pointers are HIP device memory, "host" pointers ordinary or pinned host
 *    memory, as stated per argument.  The library never allocates device memory:
 *    the caller hands it an arena whose size IS the memory budget.
 */
#ifndef LMS_H
#define LMS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lms_graph lms_graph;
typedef struct lms_exec lms_exec;

typedef enum {
  LMS_OK = 0,
  LMS_EINVAL = -1,      /* bad argument, shape mismatch, unknown id */
  LMS_ECYCLE = -2,      /* the graph (with its control edges) has a cycle */
  LMS_EBUDGET = -3,     /* no rewrite fits the budget (smaller than the largest single-op working set) */
  LMS_EOOM_DEVICE = -4, /* arena too small for the graph as it is (caller did not rewrite / plan) */
  LMS_EOOM_HOST = -5,   /* pinned host pool too small for the swapped tensors */
  LMS_EHIP = -6         /* a HIP runtime call failed */
} lms_status;

typedef enum { LMS_BF16 = 0, LMS_F32 = 1, LMS_I32 = 2 } lms_dtype;
typedef enum { LMS_VAR_PARAM = 0, LMS_VAR_INPUT = 1, LMS_VAR_TARGET = 2, LMS_VAR_CONST = 3 } lms_var_kind;
/* Section 3.3: forward / backward / update phases; LMS_SWAP tags inserted swap operations. */
typedef enum { LMS_FWD = 0, LMS_BWD = 1, LMS_UPD = 2, LMS_SWAP = 3 } lms_phase;
/* Definition 1: the action an edge carries. */
typedef enum { LMS_READ = 0, LMS_UPDATE = 1, LMS_CONTROL = 2 } lms_action;
/* Section 3.4: device placement; swap operations are the identity placed on the host. */
typedef enum { LMS_DEVICE = 0, LMS_HOST = 1 } lms_placement;

typedef enum {
  LMS_OP_VARIABLE = 0,
  LMS_OP_CONV = 1,          /* in: x, w, [scale, shift | shift], [res] ; y = act(scale*conv(x,w)+shift+res) */
  LMS_OP_CONV_DGRAD = 2,    /* in: dy, w, [scale], [addend], [mask] ; dx = (convT(dy, w*scale) + addend) * [mask>0] */
  LMS_OP_CONV_WGRAD = 3,    /* in: x, dy ; dw (fp32) */
  LMS_OP_TCONV = 4,         /* in: x, w ; window 2 stride 2 transposed convolution */
  LMS_OP_TCONV_DGRAD = 5,   /* in: dy, w, [addend], [mask] */
  LMS_OP_TCONV_WGRAD = 6,   /* in: x, dy */
  LMS_OP_MAXPOOL = 7,       /* in: x */
  LMS_OP_MAXPOOL_BWD = 8,   /* in: dy, x ; gradient to the first maximum of each window; [mask] means x>0 */
  LMS_OP_GAP = 9,           /* in: x ; mean over spatial positions */
  LMS_OP_GAP_BWD = 10,      /* in: dy, [mask] */
  LMS_OP_CONCAT = 11,       /* in: a, b ; channel concatenation */
  LMS_OP_SLICE_C = 12,      /* in: x, [mask] ; channels [c_begin, c_begin + c_count) */
  LMS_OP_MSE = 13,          /* in: y, t ; scalar fp32 loss = mean over all elements of (y-t)^2 */
  LMS_OP_MSE_GRAD = 14,     /* in: y, t, [mask] */
  LMS_OP_SOFTMAX_CE = 15,   /* in: z, labels(i32) ; scalar fp32 mean over rows of -log softmax(z)[label] */
  LMS_OP_SOFTMAX_CE_GRAD = 16, /* in: z, labels, [mask] */
  LMS_OP_GRAD_SUM = 17,     /* in: g1..gn (n<=4), [mask] ; (g1+..+gn) * [mask>0] */
  LMS_OP_COLSUM = 18,       /* in: dy ; fp32 per-channel sum over all positions (bias / shift gradient).  If its output is
                             * bound to caller memory (lms_node_set_external) and the CONV_WGRAD node of the same dy lies at most 8
                             * ids before it, the executor takes the sums from that node's pass over dy */
  LMS_OP_SCALE_COLS = 19,   /* in: dw_raw(fp32), scale ; dw = dw_raw * scale_k */
  LMS_OP_DOT_COLS = 20,     /* in: dw_raw(fp32), w ; dscale_k = sum_j w[j,k] * dw_raw[j,k] */
  LMS_OP_SWAP_OUT = 21,     /* in: t ; identity placed on the host (Eq. 2) */
  LMS_OP_SWAP_IN = 22,      /* in: swap-out ; identity bringing the tensor back (Eq. 5) */
  LMS_OP_SGD = 23,          /* in: p, dp(fp32) ; p - attr.lr * dp in p's type: the update of Section 3.3 (phase LMS_UPD) */
  LMS_OP_MOMENTUM = 24      /* in: v(fp32), dp(fp32) ; attr.lr * v + dp (fp32): the velocity of classical momentum (phase LMS_UPD) */
} lms_op;

/* flags of lms_attr.flags */
#define LMS_F_RELU   0x01u  /* ReLU after everything else (forward ops) */
#define LMS_F_AFFINE 0x02u  /* per-output-channel scale and shift inputs present */
#define LMS_F_BIAS   0x04u  /* per-output-channel shift input only */
#define LMS_F_RES    0x08u  /* residual input added before the ReLU */
#define LMS_F_ADDEND 0x10u  /* backward ops: an already computed gradient is added to the result */
#define LMS_F_MASK   0x20u  /* backward ops: result is zeroed where the mask tensor is <= 0 (ReLU backward) */

typedef struct {
  int32_t filt[3];     /* filter / window extent per spatial axis (unused axes 1) */
  int32_t stride;      /* same in every spatial axis */
  int32_t pad;         /* zero padding on both sides of every spatial axis */
  uint32_t flags;      /* LMS_F_* */
  int32_t cout;        /* output channels (conv, tconv) */
  int32_t c_begin;     /* SLICE_C */
  int32_t c_count;     /* SLICE_C */
  int32_t ndim_out;    /* ops whose output shape cannot be inferred (CONV_DGRAD, GAP_BWD): the shape */
  int64_t out_dims[5];
  float lr;            /* SGD: learning rate */
} lms_attr;

/* ------------------------------------------------------------------ errors */
const char* lms_last_error(void);
const char* lms_version(void);

/* ------------------------------------------------------------------ graph (Definition 1) */
lms_status lms_graph_create(lms_graph** out);
lms_status lms_graph_destroy(lms_graph* g);
lms_status lms_graph_clone(const lms_graph* g, lms_graph** out);

/* A parameterised vertex (variable or constant): order 0, lives outside the arena in caller memory
 * bound later with lms_exec_bind.  `name` is copied.  dims: ndim <= 5 extents.
 * Storage types: activations, filters and regression targets are bf16 on the product path (bf16 MFMA kernels).
 * fp32 check mode: if the input batch, the filters and the regression target are declared LMS_F32, every
 * activation of the graph is fp32 and the executor runs the whole step (forward, loss, backward, swaps) with plain
 * fp32 kernels; it exists to compare with an fp64 reference at 1e-4 and is not tuned.  Affine / bias parameters,
 * weight gradients and the loss are fp32 in both modes; a convolution's x and w must have the same type. */
lms_status lms_add_variable(lms_graph* g, const char* name, lms_dtype dtype, int32_t ndim,
                            const int64_t* dims, lms_var_kind kind, int32_t* node_out);
/* A normal operation reading `n_in` tensors (read edges in slot order).  The output shape and type
 * are inferred and checked; attr may be NULL for ops without attributes. */
lms_status lms_add_op(lms_graph* g, const char* name, lms_op op, const lms_attr* attr, int32_t n_in,
                      const int32_t* inputs, lms_phase phase, int32_t* node_out);
/* update edge: `from` writes into variable `var` (Table 1). */
lms_status lms_add_update_edge(lms_graph* g, int32_t from, int32_t var);
/* control edge: `to` may not run before `from` has finished; never into a variable (Section 3.2). */
lms_status lms_add_control_edge(lms_graph* g, int32_t from, int32_t to);
/* Appends the backward phase (Section 3.3): for every forward operation between the learnable
 * parameters and `loss_node`, gradient operations tagged LMS_BWD that read the forward tensors
 * they need.  Parameter gradients are the nodes named "grad/<parameter name>". */
lms_status lms_build_backward(lms_graph* g, int32_t loss_node);
/* Update phase (Section 3.3): for every learnable parameter p that lms_build_backward gave a gradient grad/p, appends
 * the operation update/p = p - lr * grad/p (LMS_OP_SGD, phase LMS_UPD) and an update edge from it to p.  With
 * momentum > 0 each such parameter also gets a variable velocity/p (fp32, kind LMS_VAR_CONST, same shape; the caller
 * binds zero-initialised memory), the operation update/velocity/p = momentum * velocity/p + grad/p (LMS_OP_MOMENTUM)
 * with an update edge to velocity/p, and update/p = p - lr * update/velocity/p.  The executor writes an update
 * wherever the caller binds it; bound to the variable's own memory the step trains in place.  Operations execute in
 * creation order, so an update runs after every earlier reader of its variable, and an operation created after it
 * reads the updated value (Section 3.2: an operation always uses the latest value of a variable).  bf16 parameters
 * are rounded to nearest even after the subtraction.  n_updates (may be NULL): parameters updated. */
lms_status lms_build_update(lms_graph* g, float lr, float momentum, int32_t* n_updates);

/* Declares that the output of operation `node` (a parameter gradient "grad/...", an update) will live in caller
 * memory bound with lms_exec_bind, not in the arena: lms_memory_need, lms_rewrite and lms_exec_create then plan no
 * arena block for it, so the budget is not charged for memory the step never uses (Section 5.1 leaves variables
 * and what is written into them outside the rewriting; the budget covers activations and workspaces).
 * lms_exec_step fails with LMS_EINVAL if such a node is not bound.  external: 1 to set, 0 to clear. */
lms_status lms_node_set_external(lms_graph* g, int32_t node, int32_t external);

/* ------------------------------------------------------------------ rewriting (Sections 4, 5.1; Table 2) */
typedef enum { LMS_CHAIN_RULE = 0, LMS_DIRECT_ORDER = 1, LMS_OWN = 2 } lms_strategy;

typedef struct {
  int32_t n_tensors;        /* tensors to swap, breadth-first from the inputs; -1 = all (Table 2) */
  int32_t lb, ub;           /* lower / upper bound of the control-operation search (Section 4.3) */
  int32_t ctrld_strategy;   /* lms_strategy; LMS_OWN hoists each swap-in as early as the budget allows */
  int32_t fuse_swapins;     /* one swap-in for consumers within fuse_distance orders (Section 4.2.3) */
  int32_t fuse_distance;    /* < 0 = unlimited */
  int32_t swap_branches;    /* also rewrite forward->forward edges longer than branch_threshold */
  int32_t branch_threshold;
  uint64_t budget_bytes;    /* 0 = none.  Otherwise n_tensors is ignored and the smallest number of
                               tensors (in the same breadth-first order) whose rewrite fits is used */
  /* Table 2's list-valued fields.  A list of names is one string with the entries separated by commas (names hold
   * no comma); NULL or "" = empty list.  Lists of operation types are bit masks: bit (1u << lms_op). */
  const char* starting_op_names; /* NULL = start the walk at the input variables, else at the operations so named */
  const char* excl_scopes;  /* name prefixes whose operations' outputs are never swapped */
  const char* incl_scopes;  /* name prefixes: if given, only these operations' outputs are swapped */
  uint32_t excl_types;      /* operation types whose outputs are never swapped (0 = none) */
  uint32_t incl_types;      /* if non-zero, only outputs of these operation types are swapped */
  /* Recomputation (the future work named in Section 7; the paper gives no rule, these are this library's):
   * 0 off.
   * 1: a tensor the selection would swap whose producer is a cheap operation (max pooling, concatenation, global
   *    average pooling) is not swapped; each group of late consumers reads a copy of the producer instead, inserted
   *    with a control edge exactly like a swap-in.  Applies to every such tensor whatever n_tensors says.
   * 2: chained recomputation.  A selected tensor whose producer is a convolution, transposed convolution, pooling
   *    or concatenation gets ONE late copy of the producer, read by all its late consumers; a copy reads the copies
   *    of those inputs that are recomputed too, so up to recompute_depth recomputed tensors follow one another
   *    before a stored tensor is needed (walking the selected tensors in creation order, a tensor is recomputed
   *    if that keeps its chain within the depth).  A copy is triggered by the control operation the strategy picks
   *    for its earliest late consumer; a copy feeding another copy is triggered no later than that one.
   *    With a budget and recompute_depth <= 0 the library plans per tensor between recomputing, swapping and
   *    keeping: starting from the plan with swaps alone, it moves one tensor at a time between "recomputed" and
   *    "stored" (a forward tensor that only a recomputed producer reads, such as a shortcut branch, included) and
   *    keeps a change if the plan still fits and its estimated step is shorter.  The estimate plays the step
   *    through on three streams with the figures below: operations one after the other, copies at the link rate, a
   *    block of the memory plan handed on only when the copy out of it is over (lms_rewrite_stats.estimated_ms).
   * In both modes the swap pass then runs on the graph with the copies. */
  int32_t recompute;
  int32_t recompute_depth;  /* mode 2: longest chain of recomputed tensors; <= 0: chosen by the planner (2 without a budget) */
  /* Machine figures for the planner's estimate, 0 = default: arithmetic rate of convolutions (default 800 TFLOP/s),
   * device memory rate (5000 GB/s), host link rate per direction as the swap copies see it (50 GB/s). */
  float device_tflops, hbm_gbs, link_gbs;
  int32_t encoded_swaps;    /* 1: the executor will run with LMS_X_ENCODE_SWAPS; the estimate then counts the bytes
                               a swapped tensor is expected to put on the link: half of a ReLU output's bytes (every
                               second element is zero and the rest take 11 to 13 bits), 0.7 of any other 16-bit
                               tensor's */
} lms_params;

typedef struct {
  int32_t tensors_swapped, swap_outs, swap_ins, control_edges, unrewritten;
  uint64_t peak_live_before, peak_live_after;  /* largest sum of live arena tensor bytes, sequential run */
  uint64_t arena_needed_before, arena_needed_after; /* bytes the offset planner needs (>= peak_live) */
  uint64_t swapped_bytes_out, swapped_bytes_in;
  int32_t recomputed;       /* recomputation copies inserted (each also counts in control_edges) */
  float estimated_ms;       /* the planner's estimate of the rewritten step (see lms_params.device_tflops), with a budget */
} lms_rewrite_stats;

/* Table 2 defaults: n_tensors -1, lb 1, ub 10000, chain_rule, no fusing, no branches, threshold 0. */
lms_status lms_params_default(lms_params* p);
/* Rewrites g in place (the paper's run(graph)).  p and stats are caller-owned; stats may be NULL.
 * LMS_EBUDGET if budget_bytes > 0 and even swapping every tensor does not fit; then stats (if given)
 * report the best attempt and g is left unchanged. */
lms_status lms_rewrite(lms_graph* g, const lms_params* p, lms_rewrite_stats* stats);
/* Memory need of g as it is, without rewriting: peak live bytes and planned arena bytes. */
lms_status lms_memory_need(const lms_graph* g, uint64_t* peak_live, uint64_t* arena_bytes);

/* ------------------------------------------------------------------ inspection (read-only) */
typedef struct {
  int32_t id, op, phase, placement, is_variable, var_kind, dtype, ndim;
  int64_t dims[5];
  int32_t gamma;            /* order: 0 for variables; for inserted swap ops the label of Figure 3 */
  int32_t n_inputs, n_control_inputs;
  uint32_t flags;
  uint64_t bytes;
  uint64_t workspace_bytes; /* transient arena scratch the operation needs while it runs */
  char name[96];
} lms_node_info;
typedef struct { int32_t src, dst, action, slot; uint64_t bytes; } lms_edge_info;

lms_status lms_node_count(const lms_graph* g, int32_t* n);
lms_status lms_node_info_get(const lms_graph* g, int32_t id, lms_node_info* out);
lms_status lms_node_find(const lms_graph* g, const char* name, int32_t* id_out); /* LMS_EINVAL if absent */
/* Attributes of a node as the library holds them (filter extents filled in from the filter shape). */
lms_status lms_node_attr_get(const lms_graph* g, int32_t id, lms_attr* out);
lms_status lms_edge_count(const lms_graph* g, int32_t* n);
lms_status lms_edge_info_get(const lms_graph* g, int32_t index, lms_edge_info* out);
/* gamma[i] for every node: the topological ordering of Definition 2 recomputed on g as it is now
 * (minimal levels; control edges count, update edges do not).  gamma: host array of node_count. */
lms_status lms_topo_order(const lms_graph* g, int32_t* gamma);
/* Execution order the executor and the memory simulation use; order: host array of node_count. */
lms_status lms_schedule(const lms_graph* g, int32_t* order);

/* ------------------------------------------------------------------ executor */
#define LMS_X_POISON     0x1u  /* fill every arena block with bf16 NaN when it is released */
#define LMS_X_NO_OVERLAP 0x2u  /* run copies on the compute stream (no side streams) */
#define LMS_X_KEEP_ALL   0x4u  /* never reuse arena memory: every tensor stays readable after the step */
#define LMS_X_DMA_COPY   0x8u  /* swap with hipMemcpyAsync (copy engines) instead of the library's copy kernels */
#define LMS_X_ENCODE_SWAPS 0x10u /* swap-out / swap-in are an encoding / decoding pair instead of two identities
                                  * (Section 4.2.1, remark after Eq. 4): bf16 tensors whose element count is a multiple
                                  * of 8 cross the host link as bitmap + non-zero elements (lossless, see
                                  * lms_swap_encode); other tensors are copied as they are.  The pinned pool must hold
                                  * lms_swap_encoded_bytes per such tensor.  Ignored together with LMS_X_DMA_COPY.
                                  * lms_step_stats then counts the bytes really moved: for a synchronised step
                                  * (loss_out non-NULL) those of that step; an unsynchronised step cannot know the sizes
                                  * of copies still running and reports those of the latest synchronised step of the
                                  * same executor (0 before the first). */
#define LMS_X_STAGED_SWAPS 0x40u /* with LMS_X_ENCODE_SWAPS: the encoded bytes cross the link through the copy engines
                                  * instead of being written / read by the encoding kernels themselves, which slow the
                                  * convolutions running beside them down once they saturate the link.  The last
                                  * lms_swap_staging_bytes() of the arena become four staging buffers (two per
                                  * direction) and are not available to the plan: rewrite for budget - staging.  A
                                  * tensor goes chunk by chunk: the encoder writes the first w bytes of every slot of
                                  * the chunk into the staging buffer and a pitched hipMemcpy2DAsync of w-byte rows
                                  * carries them into the host buffer (the reverse for a swap-in); what a slot has
                                  * beyond w the kernels move directly as before, so the host buffer holds the same
                                  * encoding whatever w is.  w is chosen per tensor after every synchronised step from
                                  * the slot sizes just seen (95 % of the slots fit); before the first one it is 0 and
                                  * the transfer is the direct one.  lms_step_stats counts the bytes that crossed the
                                  * link (w per slot plus the tails). */
#define LMS_X_TIMING     0x20u /* time the waits between streams and the copies with events created in lms_exec_create
                                * (two per waiting operation and per copy): fills the *_ms fields of lms_step_stats
                                * for synchronised steps.  Costs a few microseconds per event; leave it off to time
                                * the step itself. */

/* Bytes at the end of the arena that LMS_X_STAGED_SWAPS takes for its staging buffers (two per direction). */
uint64_t lms_swap_staging_bytes(void);

/* Plans the run of g inside [arena, arena+arena_bytes) (device memory, 256-byte aligned, caller-owned)
 * with swapped tensors parked in [pinned, pinned+pinned_bytes) (pinned host memory that is mapped into
 * the device address space at the same address, as hipHostMalloc returns it; caller-owned, 256-byte aligned).
 * compute / d2h / h2d are hipStream_t handles passed as void* (d2h, h2d may equal compute).
 * Fails with LMS_EOOM_DEVICE / LMS_EOOM_HOST if the plan does not fit.  No HIP allocation happens
 * here or in lms_exec_step except HIP events created once here. */
lms_status lms_exec_create(const lms_graph* g, void* arena, uint64_t arena_bytes, void* pinned,
                           uint64_t pinned_bytes, void* compute_stream, void* d2h_stream,
                           void* h2d_stream, uint32_t flags, lms_exec** out);
lms_status lms_exec_destroy(lms_exec* e);
/* A pinned host pool of exactly `bytes` bytes for lms_exec_create (hipHostMalloc: page-locked, mapped into the device
 * address space at the same address, 4 KiB aligned), for callers whose own pinned allocator rounds sizes up (a
 * power-of-two rounding pins 64 GB for a 33 GB pool, and 128 GB, which a machine may refuse, for 70 GB).  The two
 * calls that allocate in this library; nothing else does.  *host_out: host pointer, owned by the caller until
 * lms_pinned_free, which waits for all work of the current device first (an executor may still be copying) and
 * accepts NULL.  LMS_EOOM_HOST if the system cannot pin that much, LMS_EINVAL for bytes == 0 or a NULL argument. */
lms_status lms_pinned_alloc(uint64_t bytes, void** host_out);
lms_status lms_pinned_free(void* host);
/* Binds device memory (caller-owned, must outlive the steps) to a variable, or to the output of an
 * operation that should be written outside the arena (e.g. a "grad/..." node).  Size must be
 * at least the node's bytes.  All variables must be bound before lms_exec_step. */
lms_status lms_exec_bind(lms_exec* e, int32_t node, void* device_ptr);

typedef struct {
  float ms;                 /* wall time of the step, only if it was synchronous */
  uint64_t bytes_d2h, bytes_h2d;
  uint64_t arena_bytes_used, pinned_bytes_used;
  int32_t n_kernels, n_copies;
  /* With LMS_X_TIMING, synchronous steps only (else 0).  Section 4.3 trades exactly these against memory: a swap-in
   * triggered too late makes its consumer wait, one triggered too early holds memory. */
  float stall_h2d_ms;       /* time the compute stream stood waiting for swap-ins (data not back yet) */
  float stall_d2h_ms;       /* time it stood waiting for swap-outs only (a block it needs is still being copied out) */
  float busy_d2h_ms, busy_h2d_ms; /* time the swap-out / swap-in streams spent inside copies */
  float device_ms;          /* first to last operation of the step on the compute stream */
} lms_step_stats;

/* Work-groups of the kernels that encode (swap-out) and decode (swap-in) a tensor with LMS_X_ENCODE_SWAPS, 1 to 4096
 * each, 0 = leave as it is.  Defaults 512 / 160.  A kernel that saturates the host link slows the convolutions that
 * run beside it (the encoder from about 112 work-groups on): where a step is as long as its swap-outs the full rate
 * (512) is right, where it is not fewer work-groups (128) can give a shorter step; callers may try both.  Takes
 * effect from the next lms_exec_step; LMS_EINVAL outside the range. */
lms_status lms_exec_set_swap_grid(lms_exec* e, int32_t encode_workgroups, int32_t decode_workgroups);
/* One pass over the graph: forward, loss, backward and, where lms_build_update added them, the updates (those that
 * read and write caller memory only are held back and leave in launches of up to 64 tensors, at the end of the step
 * or before the first operation that reads an updated variable; the arithmetic per element is the same).
 * Asynchronous on the three streams unless loss_out (host pointer) is non-NULL: then the call waits for the step
 * and stores the loss.  stats may be NULL. */
lms_status lms_exec_step(lms_exec* e, float* loss_out, lms_step_stats* stats);
/* Device address of a node's output inside the arena in the current plan (valid to read after a
 * synchronised step only if the block was not reused, i.e. with LMS_X_KEEP_ALL). */
lms_status lms_exec_tensor_ptr(lms_exec* e, int32_t node, void** device_ptr);

/* ------------------------------------------------------------------ stand-alone kernels
 * Same kernels the executor launches, callable on raw device pointers for parity tests and
 * profiling.  All pointers are device memory; `stream` is a hipStream_t passed as void*.
 * workspace: device scratch of at least lms_conv_workspace_bytes(desc, which) bytes. */
typedef struct {
  int32_t ndim_sp;          /* 2 or 3 */
  int64_t n;                /* batch */
  int64_t in_sp[3];         /* input spatial extents (unused axes 1), order (D,) H, W */
  int32_t c, k;             /* input / output channels */
  int32_t filt[3];
  int32_t stride, pad;
  uint32_t flags;           /* LMS_F_* */
} lms_conv_desc;

typedef enum { LMS_CONV_FWD = 0, LMS_CONV_DGRAD_K = 1, LMS_CONV_WGRAD_K = 2, LMS_CONV_WGRAD_BIAS_K = 3 } lms_conv_which;
lms_status lms_conv_workspace_bytes(const lms_conv_desc* d, int32_t which, uint64_t* bytes);
/* y = act(scale*conv(x,w)+shift+res); scale/shift/res may be NULL according to d->flags. */
lms_status lms_conv_fwd(const lms_conv_desc* d, const void* x, const void* w, const float* scale,
                        const float* shift, const void* res, void* y, void* workspace, void* stream);
/* dx = (convT(dy, w*scale) + addend) * [mask>0]; scale/addend/mask may be NULL. */
lms_status lms_conv_dgrad(const lms_conv_desc* d, const void* dy, const void* w, const float* scale,
                          const void* addend, const void* mask, void* dx, void* workspace, void* stream);
/* dw (fp32, filter layout) = sum over batch and positions of x (x) dy; deterministic reduction. */
lms_status lms_conv_wgrad(const lms_conv_desc* d, const void* x, const void* dy, float* dw,
                          void* workspace, void* stream);
/* The two parameter gradients of a convolution layer that the chain rule takes from dy (Section 2.1: every
 * backward operation of a layer reads the layer's output gradient): dw as lms_conv_wgrad, and dbias[k] (fp32,
 * d->k values) = sum of dy over batch and positions, the gradient of a per-channel bias or shift.  Where the
 * weight-gradient kernel stages dy through registers (1x1 filters, 2-D 3x3 filters with at least 48 channels on both
 * sides) the sums come out of the same pass over dy; otherwise a separate pass follows.  Deterministic.
 * workspace: lms_conv_workspace_bytes(d, LMS_CONV_WGRAD_BIAS_K) bytes.  All pointers device memory, caller-owned. */
lms_status lms_conv_wgrad_bias(const lms_conv_desc* d, const void* x, const void* dy, float* dw, float* dbias,
                               void* workspace, void* stream);

/* For callers that cannot allocate device memory (code under stream capture, tight serving loops, harnesses that
 * forbid hipMalloc): lms_conv_wgrad with its workspace inside the library.  The split partial sums go to a fixed
 * array of lms_static_scratch_bytes() = 64 MiB that every device the library runs on holds until the process ends;
 * its device address is looked up once per device on the first call there (the device current at the call).
 * A geometry whose lms_conv_workspace_bytes(d, LMS_CONV_WGRAD_K) exceeds that size is refused with LMS_EINVAL and
 * nothing is launched.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine); results
 * are bit-identical to lms_conv_wgrad.  All calls on one device share the one array: calls that overlap on
 * different streams of the same device race; calls on one stream are ordered.  Nothing in it has to start at
 * zero (every partial sum is written before it is read).  x, dy, dw: device memory, caller-owned. */
uint64_t lms_static_scratch_bytes(void);
lms_status lms_conv_wgrad_static(const lms_conv_desc* d, const void* x, const void* dy, float* dw, void* stream);

/* Plain device-to-device copy of `bytes` (multiple of 16, both pointers 16-byte aligned) with the
 * library's copy kernel: the known-size reference that profiler traffic counters are calibrated on. */
lms_status lms_device_copy(void* dst, const void* src, uint64_t bytes, void* stream);

/* Matrix-pipe probe, a measurement aid like lms_device_copy: launches 512 work-groups whose waves each issue
 * iters x 16 v_mfma_f32_32x32x16_bf16 with one conflict-free 16-byte LDS read per product (the instruction mix of the
 * patch-tiled convolution kernels) on operands of zeros (random_operands = 0) or of random bfloat16 values, without
 * global memory traffic.  *flops (may be NULL) receives the floating-point operations of the launch; the caller times
 * it with events on `stream`.  The device lowers clock and issue rate with the switching activity of the operands, so
 * the rate on random operands is the ceiling a convolution on N(0,1) data can approach on this device.  iters in
 * 1 .. 2^22, else LMS_EINVAL. */
lms_status lms_mfma_probe(uint32_t iters, int32_t random_operands, uint64_t* flops, void* stream);

/* Lossless encoding of a swapped tensor (the f / f^-1 pair that Section 4.2.1 of the paper allows in place of the
 * two identities of Eq. 5).  A tensor of `numel` 16-bit elements (numel % 8 == 0, else LMS_EINVAL) is cut into slots
 * of 2048 elements (bfloat16 bit patterns); slot s occupies bytes [s*4368, (s+1)*4368) of the host buffer: a 256-byte
 * bitmap (bit i%8 of byte i/8 set iff element i differs from 0x0000), a 16-byte header (byte 0: mode, byte 1: the
 * largest exponent field emax of the non-zero elements unless the mode is 0, bytes 2-3: the slot's value bytes as
 * little-endian u16, the rest unspecified), then the non-zero elements in order.  Mode 0, raw: little-endian u16 each.
 * Otherwise bit 0 of the mode is set (packed), bit 1 says wide, bit 2 signed, bit 3 split.  Not split: each element is
 * a code of B = 7 + (wide ? 5 : 4) + (signed ? 1 : 0) bits, sign << (B-1) | (emax - exponent) << 7 | mantissa (the sign
 * only if signed), in a little-endian bit stream (code j in bits [B j, B j + B), unused bits of the last byte zero).
 * Split (mode = packed | split), with d = emax - exponent: one byte (d & 1) << 7 | mantissa per element, unspecified
 * bytes up to the next multiple of 4, then a little-endian bit stream in which element j adds d >> 1 zero bits and a
 * one bit (a Rice code: the differences crowd near zero).  A slot is packed iff it has a non-zero element and all
 * their exponent fields lie within 31 of the largest, wide iff not within 15, signed iff one of them has its sign bit
 * set, and split instead iff it is packed without signs and the split form has fewer value bytes; so every bit
 * pattern survives (-0.0, NaNs, infinities and denormals included).  The remaining bytes of a slot are unspecified.
 * After the last slot: one u32 per slot with its count of non-zero elements in bits 0-11, the flags packed / wide /
 * signed / split in bits 15 / 14 / 13 / 12 and its value bytes in bits 16-31 (region padded to 16 bytes), then a
 * 16-byte trailer holding, as u64, the slot bytes a copy moves (per slot 272 + the value bytes rounded up to 16).
 *   lms_swap_encoded_bytes  size of the host buffer (out: host pointer).
 *   lms_swap_encode         src: device memory, 16-byte aligned; dst_host: pinned host memory mapped into the device
 *                           address space (hipHostMalloc), 16-byte aligned, lms_swap_encoded_bytes large.
 *   lms_swap_decode         the inverse: src_host -> dst (device, numel elements); reads bitmaps, headers and values only.
 *   lms_swap_moved_bytes    after the encode has finished: the trailer's value; host: the encoded buffer (host
 *                           pointer), out: host pointer.
 * Asynchronous on `stream`; buffers are caller-owned. */
lms_status lms_swap_encoded_bytes(uint64_t numel, uint64_t* bytes);
lms_status lms_swap_encode(void* dst_host, const void* src, uint64_t numel, void* stream);
lms_status lms_swap_decode(void* dst, const void* src_host, uint64_t numel, void* stream);
lms_status lms_swap_moved_bytes(const void* host, uint64_t numel, uint64_t* bytes);
/* The same pair on the slots [slot_begin, slot_end) of the tensor (a slot is 2048 elements and 4368 bytes of the host
 * buffer), with the first w bytes of every slot (w a multiple of 16, at most 4368) written to / read from device
 * memory at stage + (slot - slot_begin) * 4368 instead of the host buffer: what LMS_X_STAGED_SWAPS launches around its
 * pitched copies.  stage NULL or w 0: everything goes to / comes from the host buffer.  The encoder also writes the
 * slots' counts (host buffer), no trailer.  Whatever w is, host buffer and staging buffer together hold the encoding
 * lms_swap_encode writes.  Pointers 16-byte aligned; stage: device memory of (slot_end - slot_begin) * 4368 bytes. */
lms_status lms_swap_encode_staged(void* dst_host, const void* src, uint64_t numel, int64_t slot_begin, int64_t slot_end,
                                  void* stage, int32_t w, void* stream);
lms_status lms_swap_decode_staged(void* dst, const void* src_host, uint64_t numel, int64_t slot_begin, int64_t slot_end,
                                  const void* stage, int32_t w, void* stream);


#ifdef __cplusplus
}
#endif
#endif /* LMS_H */
