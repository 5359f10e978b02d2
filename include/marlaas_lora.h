/*
 * marlaas_lora.h -- C ABI of the MI355X (gfx950) mixed-tenant multi-LoRA linear layer.
 *
 * One frozen base weight W is shared by every tenant; token i of a batch
 * belongs to task t(i) and gets that task's LoRA adapter (A_t, B_t) added
 * (shared base + per-task adapters: paper Sec. 1 principle (1), Sec. 4.2 and
 * Sec. 4.5; LoRA itself is the cited low-rank update of Sec. 2.3):
 *
 *     y_i = x_i W + s_t (x_i A_t) B_t          t = t(i);  t = -1: y_i = x_i W
 *
 * The same layer runs in rollout decode and prefill (forward only, Sec. 4.4
 * "Rollout") and in the policy update (forward + backward, Sec. 4.4
 * "Training"), where only the LoRA parameters are trained (Sec. 4.2), so the
 * backward produces dX and per-adapter dA_t, dB_t and never dW.
 *
 * Conventions common to all entry points
 *  - Every tensor pointer is a DEVICE pointer owned by the caller unless it is
 *    marked HOST.  The library never frees caller memory.  Outputs must not
 *    alias inputs.
 *  - All tensors are row-major.  Device pointers must be 16-byte aligned,
 *    leading dimensions are in elements and must keep rows 16-byte aligned;
 *    d_in and d_out must be multiples of 8.  Otherwise MARLAAS_EALIGN.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    The passes (marlaas_lora_fwd, marlaas_lora_bwd, marlaas_lora_bwd_adamw, marlaas_lora_fwd_multi,
 *    marlaas_adapter_table_update) only enqueue kernels on it and return: they
 *    allocate nothing, copy nothing from host memory, wait for nothing, and may
 *    be recorded into a HIP graph by stream capture, first call included.
 *    Device memory is only ever allocated by the *_create / *_build calls.
 *    marlaas_segmap_update enqueues, then waits for its own kernels.
 *  - Argument errors are reported synchronously as negative status codes with a
 *    message retrievable by marlaas_last_error(); HIP failures map to
 *    MARLAAS_EHIP.  No C++ exception crosses this boundary.
 *  - A ctx may be used by one host thread at a time.
 *  - Two environment variables are read when a ctx is created; both only select between ways of
 *    computing the same result for small batches with a packed weight (see marlaas_pack_weight):
 *    MARLAAS_DECODE_FINISH = 0 | 1 | 2 | 3: who adds up the contraction splits and applies the
 *    expand after the decode kernel: the generic finish kernel, the decode kernel itself, a
 *    second launch of the decode kernel's own finish, or (default, 3) the second for an unsplit
 *    contraction and the third otherwise.  MARLAAS_SPIN_LIMIT = n: polls of the one bounded wait
 *    of the in-kernel finish before a workgroup stops waiting and the work is finished without it
 *    (0 exercises that path; default 2^20).
 */
#ifndef MARLAAS_LORA_H
#define MARLAAS_LORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct marlaas_ctx marlaas_ctx;       /* device id, workspace, last error text */
typedef struct marlaas_segmap marlaas_segmap; /* token grouping by adapter (device + host copies) */
typedef struct marlaas_adapter_table marlaas_adapter_table; /* registered adapters, versioned (device + host mirror) */

typedef enum {
  MARLAAS_OK = 0,
  MARLAAS_EINVAL = -1,       /* null pointer, negative size, bad enum, bad token id */
  MARLAAS_ESHAPE = -2,       /* sizes inconsistent with each other or with the segmap */
  MARLAAS_EALIGN = -3,       /* pointer / leading dimension / feature size alignment */
  MARLAAS_ENOMEM = -4,       /* workspace missing or too small, or allocation failed */
  MARLAAS_EHIP = -5,         /* a HIP runtime call failed */
  MARLAAS_EUNSUPPORTED = -6  /* valid request this build does not implement */
} marlaas_status;

typedef enum { MARLAAS_BF16 = 0, MARLAAS_F32 = 1 } marlaas_dtype;

/* Storage orientation of the weights.
 *   MARLAAS_LAYOUT_MATH  : W[d_in,d_out], A_t[d_in,r_t], B_t[r_t,d_out]
 *   MARLAAS_LAYOUT_TORCH : W[d_out,d_in], A_t[r_t,d_in], B_t[d_out,r_t]  (nn.Linear / PEFT)
 * Gradients dA_t, dB_t are written in the same orientation as A_t, B_t. */
typedef enum { MARLAAS_LAYOUT_MATH = 0, MARLAAS_LAYOUT_TORCH = 1 } marlaas_layout;

#define MARLAAS_MAX_RANK 128
#define MARLAAS_MAX_ADAPTERS 4096

typedef struct {
  int64_t T;             /* tokens (rows of x); 0 is a legal no-op */
  int64_t d_in;          /* K */
  int64_t d_out;         /* N */
  int32_t n_adapters;    /* 0 .. MARLAAS_MAX_ADAPTERS */
  int32_t in_dtype;      /* marlaas_dtype of x, W, A_t, B_t, dY */
  int32_t out_dtype;     /* marlaas_dtype of y, dX (dA_t, dB_t are always fp32) */
  int32_t layout;        /* marlaas_layout */
  const void* x;         /* [T, d_in], leading dimension ldx */
  int64_t ldx;
  const void* W;         /* math: [d_in, d_out]; torch: [d_out, d_in]; leading dimension ldw <= 4194304 */
  int64_t ldw;
  const void* const* A;  /* HOST array of n_adapters device pointers, each dense (no padding) */
  const void* const* B;  /* HOST array of n_adapters device pointers, each dense */
  const int32_t* ranks;  /* HOST int32[n_adapters], 1 .. MARLAAS_MAX_RANK */
  const float* scales;   /* HOST float[n_adapters], s_t (= alpha / r_t) */
  const marlaas_segmap* map; /* grouping of the T tokens by adapter, see marlaas_segmap_build */
  /* Optional: the adapters come from a table object instead of the four host arrays above (which
   * are then ignored and may be NULL); n_adapters must equal the table's.  `proj` selects the
   * projection inside the table (0 for a table of one projection). */
  const marlaas_adapter_table* table;
  int32_t proj;
  int32_t reserved;      /* set to 0 */
  /* Optional (bf16 only): packed copies of W written once by marlaas_pack_weight, for the forward
   * product (direction 0) and for the backward product dY W^T (direction 1).  Small batches
   * (decode) then read the packed copy and not W.  NULL means not available. */
  const void* W_packed_fwd;
  const void* W_packed_bwd;
  /* Optional (bf16 only): dense transposed copy of W written once by marlaas_transpose_weight
   * (math: [d_out, d_in]; torch: [d_in, d_out]).  W is frozen for the life of the model (paper
   * Sec. 1 principle (1)), so the large-batch product whose contraction runs along W's strided
   * dimension (math: the forward, torch: the backward) reads this copy instead of transposing W into the
   * workspace on every call.  NULL means not available. */
  const void* W_t;
} marlaas_lora_desc;

/* Create a context bound to HIP device `device`.  *out is NULL on failure. */
int marlaas_create(marlaas_ctx** out, int device);
void marlaas_destroy(marlaas_ctx* ctx);

/* Static text for a status code; per-context detail of the last failure. */
const char* marlaas_strerror(int status);
const char* marlaas_last_error(const marlaas_ctx* ctx);

/*
 * Group tokens by adapter (the token->adapter map of a mixed-tenant batch,
 * Sec. 4.5).  token_adapter is a device int32[T]; -1 means "base weight only".
 * Builds, by a stable counting sort on the GPU: counts[n+1] (slot n = tokens
 * with id -1), seg_off[n+2] (exclusive prefix sums) and perm[T] (token indices,
 * grouped by adapter, original order kept inside each group, id -1 last).
 * Ids outside [-1, n_adapters) give MARLAAS_EINVAL and *out = NULL.  The call
 * waits for its kernels (it reads the counts back to plan launches); build the
 * map once per batch and reuse it for every layer and for forward + backward.
 * The map owns its device memory (hipMalloc) until marlaas_segmap_destroy.
 */
int marlaas_segmap_build(marlaas_ctx* ctx, const int32_t* token_adapter, int64_t T,
                         int32_t n_adapters, void* stream, marlaas_segmap** out);
void marlaas_segmap_destroy(marlaas_segmap* map);
/*
 * The same in two steps, for a serving or training loop that regroups a new
 * batch every step: marlaas_segmap_create allocates a map object able to hold
 * any batch of up to T_max tokens over up to n_adapters_max adapters (device
 * buffers and one pinned host buffer, holding no map yet); marlaas_segmap_update
 * regroups a batch into it without allocating: five small kernels, one
 * device-to-host copy of the n_adapters + 2 offsets and one wait on `stream` (the
 * host plans launch grids from the segment sizes).  Sizes beyond the capacity
 * give MARLAAS_ESHAPE, ids outside [-1, n_adapters) MARLAAS_EINVAL (the object
 * then holds no map until the next successful update), a capturing stream
 * MARLAAS_EUNSUPPORTED.  marlaas_segmap_build = create(T, n_adapters) + update.
 */
int marlaas_segmap_create(marlaas_ctx* ctx, int64_t T_max, int32_t n_adapters_max, marlaas_segmap** out);
int marlaas_segmap_update(marlaas_ctx* ctx, marlaas_segmap* map, const int32_t* token_adapter, int64_t T,
                          int32_t n_adapters, void* stream);
/* Copy the map to HOST buffers (either may be NULL): perm int32[T],
 * seg_off int32[n_adapters + 2].  Waits for the copy. */
int marlaas_segmap_export(const marlaas_segmap* map, int32_t* perm, int32_t* seg_off);

/*
 * Adapter table: the per-task LoRA parameters as the manager holds them, one
 * entry per task, replaced by a new version after every policy update of that
 * task (paper Sec. 4.2 "theta_t^(v)", Alg. 1 commit step) while rollouts of the
 * other tasks keep running.  The table lives in device memory; an entry is
 * (A_t, B_t, rank, scale, and optionally the fp32 gradient buffers dA_t, dB_t
 * shaped like A_t, B_t).  A table of n_proj > 1 projections holds the adapters
 * of the projections of one block that share their input (q / k / v, gate / up);
 * entry (proj, t) belongs to projection proj.  max_rank bounds the ranks the
 * table will accept.
 *
 * marlaas_adapter_table_update registers or replaces entry (proj, t) by
 * enqueueing tiny kernels on `stream` (the values travel in the kernel
 * arguments): it allocates nothing, waits for nothing and may be captured.
 * Passes enqueued later on the same stream see the new entry, passes enqueued
 * earlier the old one; a HIP graph that was captured with a descriptor referring
 * to this table reads the table when it is replayed, so a new adapter version
 * needs no new capture as long as no rank changed.  An update that changes a
 * rank also changes how the host plans launches (scratch layout, whether the
 * shrink is fused): it bumps marlaas_adapter_table_plan_version, and graphs
 * captured under an older plan version must be captured again.  Caller keeps
 * the pointed-to tensors alive while passes that may read them are in flight.
 * marlaas_adapter_table_version(table, proj, t) = number of updates of that
 * entry (0: never registered), with t < 0 the number of updates of the table;
 * -1 on bad arguments.  An adapter that no token of a batch uses may stay
 * unregistered.  One host thread at a time per table.
 */
int marlaas_adapter_table_create(marlaas_ctx* ctx, int32_t n_adapters, int32_t n_proj, int32_t max_rank,
                                 marlaas_adapter_table** out);
void marlaas_adapter_table_destroy(marlaas_adapter_table* table);
int marlaas_adapter_table_update(marlaas_ctx* ctx, marlaas_adapter_table* table, int32_t proj, int32_t t,
                                 const void* A, const void* B, int32_t rank, float scale,
                                 void* dA, void* dB, void* stream);
int64_t marlaas_adapter_table_version(const marlaas_adapter_table* table, int32_t proj, int32_t t);
int64_t marlaas_adapter_table_plan_version(const marlaas_adapter_table* table);

/*
 * Packed weight.  The base weight is frozen and shared by every tenant (paper
 * Sec. 1 principle (1)), so it can be laid out once for the kernel that streams
 * it on every decode step: marlaas_pack_weight writes W (bf16, either layout)
 * into `packed`, a caller-owned device buffer of marlaas_packed_weight_bytes
 * bytes, in the order in which the small-batch kernel's matrix-core fragments
 * consume it (blocks of 16 output columns x 32 contraction values, 1 KB each,
 * zero beyond the matrix), for direction 0 = forward (x W) or 1 = backward
 * (dY W^T).  Only enqueues one kernel on `stream`; allocates nothing.  Pass the
 * buffer in marlaas_lora_desc::W_packed_fwd / W_packed_bwd together with W
 * itself (large batches keep reading W); the results are those of the unpacked
 * path up to summation order.  With adapters, the packed path is taken when the
 * factors that multiply the layer input are stored contraction-contiguous
 * (forward: torch layout; backward: math layout); otherwise the call runs as
 * without a packed copy.
 */
size_t marlaas_packed_weight_bytes(int64_t d_in, int64_t d_out, int32_t direction);
int marlaas_pack_weight(marlaas_ctx* ctx, const void* W, int64_t ldw, int64_t d_in, int64_t d_out,
                        int32_t layout, int32_t direction, void* packed, void* stream);

/*
 * Dense transposed copy of a frozen bf16 weight for the descriptor's W_t: `out` is a caller-owned
 * device buffer of 2 * d_in * d_out bytes, written by one kernel on `stream`; it stays valid until
 * W changes.
 */
int marlaas_transpose_weight(marlaas_ctx* ctx, const void* W, int64_t ldw, int64_t d_in, int64_t d_out,
                             int32_t layout, void* out, void* stream);

/*
 * Scratch memory.  The caller hands over one device buffer (e.g. a torch
 * tensor) that must stay alive and unused by others while calls on this ctx
 * are in flight.  It holds the intermediates u, v, partial sums, a transposed
 * weight copy for some large batches and, for descriptors without an adapter
 * table, a per-call copy of their pointer tables (written by a small kernel at
 * the start of the pass).  marlaas_workspace_bytes returns the size needed by
 * marlaas_lora_fwd (want_bwd = 0) or by fwd and bwd (want_bwd = 1) for this
 * descriptor (only sizes, ranks, dtypes, table and map are read), or 0 if the
 * descriptor is invalid.
 */
size_t marlaas_workspace_bytes(const marlaas_lora_desc* desc, int want_bwd);
int marlaas_set_workspace(marlaas_ctx* ctx, void* dev_ptr, size_t bytes);

/*
 * Forward: y[T, d_out] (out_dtype, leading dimension ldy) = x W + s_t (x A_t) B_t.
 * bf16 inputs are multiplied on the matrix cores with fp32 accumulation; the
 * intermediate u = x A_t is kept in fp32 and enters the second product as a
 * two-term bf16 split, so no intermediate is rounded to bf16.  fp32 inputs use
 * fp32 arithmetic throughout.
 * u_save (nullable): device fp32 [T, marlaas_u_stride(desc)]; receives
 * s_t (x A_t) per token in the grouped order of the map, for reuse by
 * marlaas_lora_bwd (its content is otherwise opaque).
 * Results do not depend on timing: every sum that is split over workgroups is
 * added up in a fixed order.
 */
int marlaas_lora_fwd(marlaas_ctx* ctx, const marlaas_lora_desc* desc, void* y, int64_t ldy,
                     void* u_save, void* stream);

/*
 * marlaas_lora_fwd for callers that cannot allocate device memory or hand over
 * a workspace: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and same
 * results as marlaas_lora_fwd, but every intermediate (u, split-contraction
 * partial sums, the per-call copy of pointer tables) lives in one static array
 * of MARLAAS_STATIC_SCRATCH_BYTES in the library's device code: each GPU the
 * library runs on holds its own copy until the process ends, and the call
 * allocates nothing and ignores marlaas_set_workspace.  A descriptor whose
 * forward needs more scratch than that (marlaas_workspace_bytes(desc, 0)) gives
 * MARLAAS_ENOMEM with a message and enqueues nothing.  All calls on one GPU
 * share the array: calls that may overlap in time (different streams, different
 * contexts or threads) race on it; calls on one stream are ordered and safe.
 * Nothing in the array has to be cleared between calls.
 */
#define MARLAAS_STATIC_SCRATCH_BYTES (32u << 20)
int marlaas_lora_fwd_static(marlaas_ctx* ctx, const marlaas_lora_desc* desc, void* y, int64_t ldy,
                            void* u_save, void* stream);

/*
 * Forward of several projections of the same input in one call (a transformer
 * block's q / k / v, or gate / up: what a rollout engine with multi-LoRA
 * batching, paper Sec. 1, launches per layer for every decode step):
 *   y_p[T, d_out_p] = x W_p + s_{t,p} (x A_{t,p}) B_{t,p},   p = 0 .. n_proj - 1.
 * descs: HOST array of n_proj descriptors that agree in T, d_in, x, ldx, both
 * dtypes, layout, n_adapters and map; W, d_out, A, B, ranks and scales are per
 * projection.  y, ldy: HOST arrays of n_proj device pointers / leading
 * dimensions.  The result is that of n_proj calls of marlaas_lora_fwd (up to
 * summation order).  Small bf16 batches whose summed ranks fit the GEMM's
 * extended columns run as ONE GEMM launch over the concatenated columns plus one
 * finish launch; every other case runs the projections one after the other.
 * Scratch: marlaas_workspace_bytes_multi(descs, n_proj) bytes set with
 * marlaas_set_workspace (0 if the descriptors are invalid or disagree).
 */
#define MARLAAS_MAX_PROJ 8
size_t marlaas_workspace_bytes_multi(const marlaas_lora_desc* descs, int32_t n_proj);
int marlaas_lora_fwd_multi(marlaas_ctx* ctx, const marlaas_lora_desc* descs, int32_t n_proj,
                           void* const* y, const int64_t* ldy, void* stream);

/*
 * Backward for a loss with dL/dy = dY[T, d_out] (in_dtype, leading dimension lddy):
 *   dX[T, d_in] (out_dtype, lddx) = dY W^T + v A_t^T,   v = s_t dY B_t^T
 *   dA_t = sum_{i in seg(t)} x_i^T v_i,   dB_t = s_t sum_{i in seg(t)} (x_i A_t)^T dY_i
 * dA, dB: HOST arrays of n_adapters device fp32 pointers, each shaped like
 * A_t / B_t (dense).  accumulate = 0 overwrites them (an adapter without tokens
 * gets zeros), accumulate = 1 adds to their contents.  dX may be NULL (skip),
 * and dA and dB may both be NULL (skip).  With a descriptor that refers to an
 * adapter table the gradient buffers are the ones registered in the table: pass
 * MARLAAS_GRADS_IN_TABLE for both dA and dB.  u_saved: what marlaas_lora_fwd wrote
 * to u_save for the same descriptor, or NULL to recompute it.
 */
#define MARLAAS_GRADS_IN_TABLE ((void* const*)(uintptr_t)1)
int marlaas_lora_bwd(marlaas_ctx* ctx, const marlaas_lora_desc* desc, const void* dY, int64_t lddy,
                     const void* u_saved, void* dX, int64_t lddx, void* const* dA,
                     void* const* dB, int accumulate, void* stream);

/*
 * Backward with the policy update attached: the training engine's step for
 * the task(s) being trained (paper Sec. 4.2, Alg. 1: (theta_t, phi_t) of
 * version v becomes version v + 1; Sec. 4.5: one task is trained per update).
 * dX as in marlaas_lora_bwd; dA_t and dB_t are not written anywhere: each
 * gradient element is consumed where its reduction completes, by one AdamW
 * step (Adam with decoupled weight decay; the paper names no optimizer)
 *   p <- p - lr wd p;  m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;
 *   p <- p - lr (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + eps)
 * in fp32 on the task's optimizer state phi_t.
 * states: HOST array of n_adapters entries (1 <= n_adapters <= 8, bf16 inputs;
 * else MARLAAS_EUNSUPPORTED).  Per adapter, device pointers: fp32 master copies
 * of A_t and B_t, first and second moments of each (all shaped like A_t / B_t,
 * dense, same layout), and A_next / B_next: bf16 buffers that receive the
 * factors of the next version (the master values rounded to nearest even).
 * They may be the current A_t / B_t (update in place: every kernel that reads a
 * factor has been enqueued before the one that overwrites it) or separate
 * buffers to be committed with marlaas_adapter_table_update while the old
 * version is still being served.  An adapter without tokens in the batch is
 * left untouched (no decay, no step).  hp->step is the number of this update,
 * 1 for the first; it and the other hyper-parameters travel in the kernel
 * arguments, so a captured graph replays the step count it was captured with.
 */
typedef struct { float lr, beta1, beta2, eps, weight_decay; int32_t step; } marlaas_adamw;
typedef struct {
  float* master_A; float* master_B;
  float* m_A; float* v_A; float* m_B; float* v_B;
  void* A_next; void* B_next;
} marlaas_adapter_state;
int marlaas_lora_bwd_adamw(marlaas_ctx* ctx, const marlaas_lora_desc* desc, const void* dY, int64_t lddy,
                           const void* u_saved, void* dX, int64_t lddx,
                           const marlaas_adapter_state* states, const marlaas_adamw* hp, void* stream);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel launch of
 * marlaas_lora_fwd / marlaas_lora_bwd on this ctx is bracketed by a pair of HIP
 * events on the caller's stream (this allocates events: not for production
 * loops).  marlaas_profile_read waits for the recorded events of one kernel
 * family and returns their summed duration and count; enabling or disabling
 * clears the record.
 */
typedef enum {
  MARLAAS_KERNEL_SHRINK = 1,  /* u = s_t x A_t  /  v = s_t dY B_t^T */
  MARLAAS_KERNEL_GEMM = 2,    /* base product with the fused expand (small batches: also the shrink,
                                 the split-K finish kernel and no separate SHRINK span) */
  MARLAAS_KERNEL_REDUCE = 3   /* dA_t / dB_t reductions */
} marlaas_kernel;
int marlaas_profile_enable(marlaas_ctx* ctx, int on);
int marlaas_profile_read(marlaas_ctx* ctx, int kernel, double* total_ms, int64_t* launches);

/* Row stride (in floats) of u_save: the largest rank rounded up to 16; 0 if invalid. */
int64_t marlaas_u_stride(const marlaas_lora_desc* desc);

#ifdef __cplusplus
}
#endif
#endif /* MARLAAS_LORA_H */
