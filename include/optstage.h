/*
 * optstage — one pipeline stage of LLM training on one MI355X, driven by a per-stage schedule.
 *
 * The calls follow the paper's problem statement (Sec. 3 and the appendix with the mathematical
 * model): a stage i processes micro-batches j with three compute ops c in {F, B, W} (forward,
 * backward for activations, backward for weights; Sec. 2.2), may Offload (O) an activation to host
 * memory and Reload (R) it before its consumer, and must keep activation memory within the per-device
 * limit M_limit_i (Eq. 7).  A schedule for the stage is one ordered event list; list order plays the
 * role of the paper's precedence binaries (P, K, L, H, M, N).
 *
 * General rules
 *  - Plain C ABI.  Every pointer argument says whether it is HOST or DEVICE memory.
 *  - Every call returns an optstage_status; nothing throws or aborts.  optstage_last_error() gives a
 *    thread-local, library-owned message for the last failing call on the calling thread.
 *  - The library never allocates device or pinned memory: the activation arena, the workspace and the
 *    pinned host pool are caller-owned blocks handed over in optstage_desc and must outlive the handle.
 *  - Weights, gradient accumulators, stage inputs x[j], output gradients dy[j], stage outputs y[j] and
 *    input gradients dx[j] are caller-owned DEVICE buffers that must stay valid until
 *    optstage_synchronize() returns.
 *  - Compute ops are enqueued on desc.compute_stream, transfers on desc.copy_stream (reloads on
 *    desc.reload_stream when one is given); all hipStream_t passed as void*.  Calls return after
 *    enqueueing; only optstage_synchronize() blocks.
 *  - The library orders its own streams against each other and nothing else: work the caller has
 *    queued on OTHER streams that produces a buffer the library will read (a weight, x[j], dy[j]) must
 *    have completed, or been made a dependency of the library's streams, before the call that reads it.
 *  - A call that fails on its arguments, on the ordering rules or on the budget changes no accounting state and
 *    enqueues nothing (the whole list is validated on a copy of the state before anything is committed).  The one
 *    exception: if a HIP runtime call fails while a validated list is being enqueued (OPTSTAGE_E_HIP), the
 *    accounting is ahead of what reached the streams; the handle then refuses every further event with
 *    OPTSTAGE_E_STATE until optstage_synchronize() and optstage_reset() have been called.
 *  - A handle is not thread-safe; use one host thread per handle.
 */
#ifndef OPTSTAGE_H
#define OPTSTAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct optstage optstage_t;

typedef enum {
  OPTSTAGE_OK = 0,
  OPTSTAGE_E_ARG = -1,      /* null pointer, bad enum, unsupported shape, buffer too small            */
  OPTSTAGE_E_ORDER = -2,    /* event violates the ordering rules (Eq. 6, fixed micro-batch order, O/R)  */
  OPTSTAGE_E_BUDGET = -3,   /* an allocation would push live activation bytes above hbm_budget_bytes    */
  OPTSTAGE_E_HOSTPOOL = -4, /* pinned host pool exhausted                                               */
  OPTSTAGE_E_HIP = -5,      /* a HIP runtime call failed                                                */
  OPTSTAGE_E_STATE = -6,    /* call not valid in the handle's state (unbound io, missing weight, ...)   */
  OPTSTAGE_E_ARENA = -7     /* the physical arena block is too small or too fragmented                  */
} optstage_status;

/* op types: the paper's c in {F, B, W} and transfers O, R; OWAIT is the list position from which an
 * offload counts as completed (its memory is credited, Eq. 12). */
typedef enum { OPTSTAGE_F = 0, OPTSTAGE_B = 1, OPTSTAGE_W = 2, OPTSTAGE_O = 3, OPTSTAGE_OWAIT = 4, OPTSTAGE_R = 5 } optstage_op;

typedef enum { OPTSTAGE_GPT = 0 /* LayerNorm, GELU, no rotary */, OPTSTAGE_LLAMA = 1 /* RMSNorm, rotary, SwiGLU */ } optstage_family;
typedef enum { OPTSTAGE_FP32 = 0, OPTSTAGE_BF16 = 1 } optstage_dtype;

/* activation kinds of one layer of one micro-batch (store-all inventory).  Kinds 0..9 are produced by
 * F and may be offloaded; DY and DX_MID are produced by B and kept for W. */
typedef enum {
  OPTSTAGE_K_X_IN = 0, OPTSTAGE_K_N1 = 1, OPTSTAGE_K_QKV = 2, OPTSTAGE_K_O = 3, OPTSTAGE_K_LSE = 4,
  OPTSTAGE_K_X_MID = 5, OPTSTAGE_K_N2 = 6, OPTSTAGE_K_GU = 7, OPTSTAGE_K_A = 8, OPTSTAGE_K_STATS = 9,
  OPTSTAGE_K_DY = 10, OPTSTAGE_K_DX_MID = 11, OPTSTAGE_N_KINDS = 12
} optstage_kind;
#define OPTSTAGE_N_F_KINDS 10

/* per-layer parameters.  Linear weights are [out_features, in_features] row-major in the stage dtype
 * (z = W x, Sec. 2.2); norm gains/biases are [hidden] in the stage dtype.  B1/B2 exist only for GPT.
 * QKV rows are packed [q heads | k heads | v heads]; for LLAMA, GU rows are packed [gate | up]. */
typedef enum {
  OPTSTAGE_W_G1 = 0, OPTSTAGE_W_B1 = 1, OPTSTAGE_W_QKV = 2, OPTSTAGE_W_O = 3,
  OPTSTAGE_W_G2 = 4, OPTSTAGE_W_B2 = 5, OPTSTAGE_W_GU = 6, OPTSTAGE_W_D = 7, OPTSTAGE_N_WEIGHTS = 8
} optstage_weight;

typedef struct {
  uint32_t struct_size;                 /* sizeof(optstage_desc), for versioning */
  uint32_t family;                      /* optstage_family */
  uint32_t dtype;                       /* optstage_dtype: storage type of activations and weights */
  uint32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, seq, micro_batch;
  uint32_t stage_index, n_stages, n_microbatches;   /* i, p, m */
  float norm_eps, rope_base;
  uint32_t recompute;                   /* memory-table variant.  0: F keeps every kind it produces.  1: F keeps no
                                           N1, N2, A (norm outputs and MLP activation output live in transients);
                                           B rebuilds them from X_IN, X_MID, GU, bit for bit, and holds them for W.
                                           Delta_F shrinks and Delta_B grows by their bytes; they cannot be
                                           offloaded */
  uint32_t n_chunks;                    /* model chunks held by this stage (interleaved and V-shaped schedules
                                           of the comparison methods in Sec. 5 place more than one on a stage);
                                           0 or 1 = one.  n_layers counts all of them and must divide evenly:
                                           chunk c is layers c * n_layers / n_chunks onwards.  Every chunk has its
                                           own F / B / W per micro-batch and its own boundary tensors; arena,
                                           budget and transfer channel are shared */
  uint32_t no_fusion;                   /* 0: where the shapes allow it (bf16 LLAMA, head_dim 128, ffn % 128 == 0, products
                                           large enough for the direct GEMM kernel) the rotary embedding runs in the
                                           epilogue of the QKV projection and the MLP activation in the epilogue of the
                                           gate / up projection, each from the fp32 accumulators (one rounding to the
                                           storage type less than the separate kernels; the stored kinds and their
                                           bytes are the same).  1: always the separate kernels */
  uint32_t reserved;                    /* 0 */
  uint64_t hbm_budget_bytes;            /* M_limit_i for activations (Eq. 7); 0 = unlimited */
  void* arena; uint64_t arena_bytes;          /* DEVICE block for activations, 256-byte aligned */
  void* workspace; uint64_t workspace_bytes;  /* DEVICE block for transients, >= optstage_query_sizes' figure */
  void* host_pool; uint64_t host_pool_bytes;  /* pinned HOST block for offloaded activations (may be null if no O) */
  void* compute_stream; void* copy_stream;    /* hipStream_t; at default priority */
  void* reload_stream;                        /* hipStream_t for R events, or null: R shares copy_stream with O, the
                                                 single serial transfer channel of the paper's model (Eq. 8-11).  A
                                                 stream of its own lets reloads run while offloads are in flight (the
                                                 host link is full duplex); ordering of an item's R after its O, of R
                                                 after the compute ops listed before it and of B after its reloads is
                                                 kept by events either way */
} optstage_desc;

typedef struct {
  uint32_t op;          /* optstage_op */
  uint32_t microbatch;  /* j */
  uint32_t layer;       /* O / OWAIT / R: layer index on the stage (over all chunks).  F / B / W: model chunk
                           (0 on a stage with one chunk) */
  uint32_t kind_mask;   /* O / OWAIT / R only: bit k set = activation kind k (k < OPTSTAGE_N_F_KINDS) */
} optstage_event;

typedef enum {
  OPTSTAGE_KC_GEMM_NT_STORE = 0 /* the four dX products of B (C = A B^T, plain store) */,
  OPTSTAGE_KC_GEMM_NT_RESID = 1 /* output and down projection, residual added */, OPTSTAGE_KC_GEMM_TN_ACCUM = 2,
  OPTSTAGE_KC_ATTN_FWD = 3, OPTSTAGE_KC_ATTN_BWD = 4, OPTSTAGE_KC_NORM_FWD = 5, OPTSTAGE_KC_NORM_BWD = 6,
  OPTSTAGE_KC_ACT_FWD = 7, OPTSTAGE_KC_ACT_BWD = 8, OPTSTAGE_KC_ROPE = 9,
  OPTSTAGE_KC_GEMM_NT_QKV = 10 /* QKV projection (rotary in its epilogue when fused) */,
  OPTSTAGE_KC_GEMM_NT_GU = 11 /* gate / up projection (activation in its epilogue when fused) */,
  OPTSTAGE_N_KERNEL_CLASSES = 12
} optstage_kernel_class;

typedef struct {
  uint64_t live_bytes, peak_bytes;              /* logical (list-order) activation accounting */
  uint64_t bytes_offloaded, bytes_reloaded;
  uint64_t n_ops[6];                            /* count per optstage_op */
  double ms_ops[6];                             /* summed device time per optstage_op (F, B, W on the compute
                                                   stream; O, R on the copy stream); valid after synchronize */
  uint64_t arena_high_water;                    /* highest physical arena offset ever used */
  /* per kernel class, filled only while kernel timing is on (optstage_set_kernel_timing): launches,
   * summed device time, and summed algorithmic work (flops for the GEMM / attention classes 0-4, 10, 11: 2*M*N*K, causal
   * attention 2*s^2*n_q*d forward and 5*s^2*n_q*d backward; bytes for the elementwise classes: norm
   * forward 2e per element, norm backward 4e, activation forward 3e per output element, backward 5e,
   * rotary 2e over the q and k heads; e = element size) */
  uint64_t kernel_launches[OPTSTAGE_N_KERNEL_CLASSES];
  double kernel_ms[OPTSTAGE_N_KERNEL_CLASSES];
  double kernel_work[OPTSTAGE_N_KERNEL_CLASSES];
  /* list-order accounting over the executed events since the last reset: the lowest live byte count after any
   * event while a micro-batch was in flight (F done, W not done), and the mean of the live bytes after every event */
  uint64_t min_live_bytes;
  double avg_live_bytes;
  /* time the compute stream spent waiting for transfers (valid after synchronize): [0] at OWAIT events, for an
   * offload to end before the bytes it frees are reused (Eq. 12); [1] ahead of B ops, for the reloads of their
   * micro-batch to end */
  double stall_ms[2];
  uint64_t n_trace;                             /* entries optstage_get_trace() holds */
} optstage_stats;

/* One executed event: what was enqueued, the live activation bytes after it (list-order accounting), and, once
 * optstage_synchronize() has returned, its device times in ms since the first event after the last reset: F, B, W
 * on the compute stream, O and R on their transfer stream; -1 for OWAIT, which takes no time of its own.
 * stall_ms: how long the compute stream waited at this event (OWAIT: for the offload; B: for the reloads). */
typedef struct {
  uint32_t op, microbatch, layer, kind_mask;    /* as in optstage_event */
  uint64_t live_bytes;
  double start_ms, end_ms, stall_ms;
} optstage_trace_entry;

/* The memory table (the parameters Delta and Gamma of Eq. 7): bytes of each activation kind for one
 * layer of one micro-batch (each rounded up to 256), written to bytes_per_kind[OPTSTAGE_N_KINDS] (HOST);
 * *act_bytes_per_mb = Delta_F = sum over all layers of the kinds F keeps (desc.recompute decides which);
 * *min_workspace = required workspace_bytes.  Only the shape fields and recompute are read.  Any out pointer may be null. */
optstage_status optstage_query_sizes(const optstage_desc* desc, uint64_t* min_workspace,
                                     uint64_t* act_bytes_per_mb, uint64_t* bytes_per_kind);

/* Creates a handle (HOST object).  Builds the rotary table in the workspace on compute_stream. */
optstage_status optstage_create(const optstage_desc* desc, optstage_t** out);
void optstage_destroy(optstage_t* st);

/* Registers layer `layer`'s parameter `which` (DEVICE, stage dtype) and its gradient accumulator
 * (DEVICE, fp32, same shape; B and W add into it, so the caller zeroes it, unless
 * optstage_set_grad_overwrite is on).  For the four linear weights the
 * library also keeps a transposed copy in the workspace (enqueued on compute_stream) so that B's
 * dX = dY W runs with both operands contiguous along the contraction; call again after the weight
 * changes. */
optstage_status optstage_set_weight(optstage_t* st, uint32_t layer, uint32_t which, const void* weight_dev,
                                    float* grad_fp32_dev);

/* Binds micro-batch mb's boundary tensors (all DEVICE, [seq*micro_batch, hidden], stage dtype):
 * x_in (read by F), dy_out (read by B), y_out (written by F), dx_in (written by B). */
optstage_status optstage_bind_io(optstage_t* st, uint32_t mb, const void* x_in, const void* dy_out,
                                 void* y_out, void* dx_in);
/* The same for model chunk `chunk` of a stage that holds several (optstage_bind_io is chunk 0): the fixed
 * micro-batch order and Eq. 6 apply per chunk, each chunk's first layer reads its own x_in and its last
 * layer its own dy_out. */
optstage_status optstage_bind_io_chunk(optstage_t* st, uint32_t chunk, uint32_t mb, const void* x_in,
                                       const void* dy_out, void* y_out, void* dx_in);

/* Checks a whole list against the ordering rules and the budget without running anything, starting
 * from an empty stage.  events is HOST memory.  On failure *first_bad (may be null) is the index of the
 * first offending event (n if something is missing at the end). */
optstage_status optstage_validate(const optstage_t* st, const optstage_event* events, size_t n, size_t* first_bad);

/* Validates (as above, but from the handle's current state) and enqueues the whole list. */
optstage_status optstage_run(optstage_t* st, const optstage_event* events, size_t n);

/* Step-wise equivalents: same semantics as one-event lists.  The three compute calls act on model chunk 0; a
 * stage that holds several chunks reaches the others through event lists (the event's layer field). */
optstage_status optstage_forward(optstage_t* st, uint32_t mb);
optstage_status optstage_backward_input(optstage_t* st, uint32_t mb);
optstage_status optstage_backward_weight(optstage_t* st, uint32_t mb);
optstage_status optstage_offload(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t kind_mask);
optstage_status optstage_offload_wait(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t kind_mask);
optstage_status optstage_reload(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t kind_mask);

/* Blocks until both streams have drained, then resolves timing events into the stats. */
optstage_status optstage_synchronize(optstage_t* st);
/* Forgets all per-iteration state (every micro-batch back to "not started", accounting to zero, stats
 * cleared).  Requires that nothing is in flight (call after optstage_synchronize). */
optstage_status optstage_reset(optstage_t* st);
optstage_status optstage_get_stats(optstage_t* st, optstage_stats* out /* HOST */);
/* The executed trace since the last reset, in enqueue order: copies min(capacity, total) entries to out (HOST,
 * may be null when capacity is 0) and writes the total to *n_total (may be null). */
optstage_status optstage_get_trace(optstage_t* st, optstage_trace_entry* out /* HOST */, size_t capacity,
                                   size_t* n_total);
/* on != 0: the first B and the first W of every model chunk after a reset (micro-batch 0: the fixed micro-batch
 * order makes it the first) STORE their parameter gradients (dW = dY^T X of Sec. 2.2, norm gains and biases)
 * instead of adding them to what the accumulators hold, so nobody has to clear the accumulators between
 * iterations and the first W op reads none of them; later ops add as usual.  The stored values are bit for bit
 * what adding to zeroed accumulators gives.  Off by default (gradients accumulate across iterations). */
optstage_status optstage_set_grad_overwrite(optstage_t* st, uint32_t on);
/* on != 0: bracket every kernel launch of the op graphs with timing events on the compute stream (the
 * measurement mode the benchmark uses for per-kernel roofline figures); off by default. */
optstage_status optstage_set_kernel_timing(optstage_t* st, uint32_t on);

/* Test support: two 64-bit checksums of a live or offloaded activation buffer, written to out (HOST, TWO words):
 * out[0] = sum of the buffer's 64-bit words mod 2^64, out[1] = their xor.  where: 0 = the device copy, 1 = the
 * pinned host copy.  Blocks (drains all of the handle's streams first). */
optstage_status optstage_debug_checksum(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t kind,
                                        uint32_t where, uint64_t out[2] /* HOST */);
/* Test support: copies a live activation buffer to dst (HOST, at least the kind's byte size).  Blocks (waits for
 * the transfer streams first, so a reload into the buffer has landed). */
optstage_status optstage_debug_read(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t kind,
                                    void* dst_host, uint64_t dst_bytes);

const char* optstage_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
