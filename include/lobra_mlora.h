/*
 * lobra_mlora.h - C ABI of the MI355X (gfx950) multi-adapter LoRA linear layer.
 *
 * The operation (paper section 2.1, "Fine-tuning based on LoRA", and the batch
 * fusion of section 1 / Figure 1): one frozen weight W shared by all tasks, one
 * low-rank adapter per task, the tokens of several tasks packed into one batch
 * (section 2.1, "Processing Variable-length Data": sequences concatenated
 * without padding).  For a token i that belongs to task t
 *
 *     y_i  = x_i W + s_t (A_t x_i) B_t                          forward
 *     dx_i = dy_i W^T + s_t (B_t dy_i) A_t                      backward, input
 *     dA_t = s_t sum_{i in t} (B_t dy_i)^T x_i                  backward, down factor
 *     dB_t = s_t sum_{i in t} (A_t x_i)^T dy_i                  backward, up factor
 *
 * and a token without adapter (task -1) takes only the W terms.  W is never
 * updated, so there is no dW.  The paper names the factors the other way round
 * and has no scale (s_t = 1); the names here are the usual ones: A_t = down
 * projection, B_t = up projection.
 *
 * Layouts (all row-major, all tensors DEVICE pointers owned by the caller):
 *     x  [T, d_in]      W  [d_in, d_out]     y, dy [T, d_out]     dx [T, d_in]
 *     A  [R_tot, d_in]  rows rank_off[t] .. rank_off[t+1]-1 are A_t (r_t x d_in)
 *     B  [R_tot, d_out] rows rank_off[t] .. rank_off[t+1]-1 are B_t (r_t x d_out)
 *     s  [n_tasks] fp32;   dA [R_tot, d_in] fp32;   dB [R_tot, d_out] fp32
 * x, W, A, B, y, dy, dx have the element type desc.dtype (fp32, or bf16 with
 * fp32 accumulation and one rounding to bf16 at the store).
 *
 * The packed batch is described by a segment table on the HOST: segment k holds
 * tokens seg_off[k] .. seg_off[k+1]-1, all of task seg_task[k].  A task may own
 * any number of segments, segments may be empty, seg_task = -1 marks tokens
 * that take the base product only.
 *
 * Every function returns a lobra_status; nothing throws.  All argument checks
 * run on the host before anything is launched, and on error nothing is
 * written.
 *
 * Two ways to call the layer:
 *   one-shot   lobra_mlora_workspace_bytes, lobra_mlora_fwd, lobra_mlora_bwd, lobra_token_task_map take the
 *              descriptor itself.  The library allocates no device memory and never synchronises: the
 *              tables derived from the descriptor are placed at the start of the caller's workspace by an
 *              asynchronous copy on the caller's stream.  Every call pays for building them on the host
 *              (about 0.1 ms for 16384 tokens).
 *   with plan  a packed batch goes through every LoRA linear of every layer with the same segment table,
 *              so lobra_mlora_plan_init (device image in caller memory, asynchronous upload) or
 *              lobra_mlora_plan_create (the one call that allocates device memory and blocks) builds the
 *              tables once and lobra_mlora_plan_fwd / _bwd / ... reuse them; these calls do no host
 *              work beyond the launches and can be captured in a HIP graph.
 */
#ifndef LOBRA_MLORA_H
#define LOBRA_MLORA_H

#include <stddef.h>
#include <stdint.h>

/* The library is built with hidden visibility; only the entry points below are exported. */
#define LOBRA_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOBRA_OK = 0,
    LOBRA_ERR_NULL = -1,      /* a required pointer is NULL */
    LOBRA_ERR_SHAPE = -2,     /* T, d_in, d_out, n_tasks or S out of range (see lobra_mlora_desc) */
    LOBRA_ERR_DTYPE = -3,     /* dtype is neither LOBRA_F32 nor LOBRA_BF16 */
    LOBRA_ERR_SEGMENTS = -4,  /* seg_off[0] != 0, decreasing, or seg_off[S] != T */
    LOBRA_ERR_TASK_ID = -5,   /* a seg_task outside [-1, n_tasks) */
    LOBRA_ERR_RANK = -6,      /* rank_off[0] != 0 or a rank outside [1, LOBRA_MAX_RANK] */
    LOBRA_ERR_WORKSPACE = -7, /* workspace NULL or smaller than lobra_mlora_workspace_bytes / _plan_sizes say */
    LOBRA_ERR_ALIGN = -8,     /* a pointer not 16-byte aligned, or bf16 d_in/d_out not a multiple of 8 */
    LOBRA_ERR_HIP = -9,       /* a HIP runtime call failed (no device, launch error, ...) */
    LOBRA_ERR_PLAN = -10,     /* plan is NULL, host-only, or was built for another device */
    LOBRA_ERR_NOMEM = -11     /* host or device allocation for the plan failed */
} lobra_status;

typedef enum { LOBRA_F32 = 0, LOBRA_BF16 = 1 } lobra_dtype;

enum { LOBRA_MAX_RANK = 128,
       LOBRA_MAX_WIDTH = 1 << 20 };  /* d_in, d_out: the kernels' launch grids and 32-bit tile offsets end here */

/* flags of lobra_mlora_bwd */
enum {
    LOBRA_FLAG_ACCUMULATE_GRADS = 1, /* dA += ..., dB += ... (gradient accumulation over the
                                        chunks of a step, section 2.1) instead of overwriting */
    LOBRA_FLAG_NO_DX = 2             /* skip dx (first layer of a model) */
};

/* flags of lobra_mlora_plan_create */
enum {
    LOBRA_PLAN_HOST_ONLY = 1, /* build and keep the plan on the host only: no HIP call is made,
                                 the plan can be inspected with lobra_mlora_plan_query but not run */
    LOBRA_PLAN_PLAIN_KERNELS = 2 /* bf16 only: run the plain fp32-FMA kernels of the fp32 path on
                                    bf16 storage instead of the MFMA kernels (slow; a cross-check) */
};

/* Problem descriptor.  Plain data; the three tables are HOST pointers that are read
 * during lobra_mlora_validate / lobra_mlora_plan_create only (the plan keeps copies). */
typedef struct {
    int32_t dtype;           /* lobra_dtype of x, W, A, B, y, dy, dx */
    int32_t d_in, d_out;     /* 1 .. LOBRA_MAX_WIDTH; multiples of 8 for LOBRA_BF16 */
    int64_t T;               /* packed tokens, 0 <= T < 2^31 (fp32 and LOBRA_PLAN_PLAIN_KERNELS: T <= 4194240);
                                ceil(T / 256) * ceil(max(d_in, d_out) / 256) < 2^31, and with adapters
                                ceil(T / 2048) * (d_in + d_out) / 64 < 2^31 roughly (exactly: reduction chunks x
                                64-column tiles; plan creation and the one-shot calls report LOBRA_ERR_SHAPE) */
    int32_t n_tasks;         /* >= 0; 0 = base product only */
    int32_t S;               /* segments, >= 0 (S = 0 requires T = 0) */
    const int32_t *rank_off; /* [n_tasks+1], rank_off[0] = 0, r_t = rank_off[t+1]-rank_off[t] */
    const int32_t *seg_off;  /* [S+1], seg_off[0] = 0, non-decreasing, seg_off[S] = T */
    const int32_t *seg_task; /* [S], each in [-1, n_tasks) */
    int32_t n_proj;          /* 0 or 1: one layer.  P > 1: P layers that read the same x, fused
                                into one call (see "Shared-input projections" below) */
} lobra_mlora_desc;

/* Shared-input projections (n_proj = P > 1).  The q/k/v projections of an attention block, or the
 * gate/up projections of an MLP, are P LoRA linears that read the same x.  Fused into one call they
 * share the pass over x (down projections), the pass over x of the dA reduction, and the sum of
 * their P contributions to dx (one product over the concatenated dy).  Layouts, with
 * dg = d_out / P and r_t = (rank_off[t+1] - rank_off[t]) / P the rank of task t in every projection:
 *     W  [d_in, d_out]   projection j in columns j dg .. (j+1) dg - 1;  y, dy [T, d_out] likewise
 *     A  [R_tot, d_in]   task t owns rows rank_off[t] ..; of those, rows j r_t .. (j+1) r_t - 1
 *                        are the down projection of task t in projection j;  dA alike
 *     B  [R_tot, dg]     row (t, j, rho) is row rho of the up projection of task t in projection j
 *                        (it only ever meets columns of projection j);  dB alike
 * so that  y[:, j] = x W[:, j] + s_t (A_t^j x) B_t^j  and  dx = sum_j dy[:, j] W[:, j]^T + s_t (B_t^j dy[:, j]) A_t^j.
 * Requires d_out a multiple of 8 P (else LOBRA_ERR_ALIGN) and every stacked rank a multiple of 8 P
 * (else LOBRA_ERR_RANK); 1 <= P <= 16. */

/* Opaque per-batch plan (section 1 / Figure 1: the fused batch of task-tagged sequences, turned into what the
 * kernels iterate over): the validated table plus the device-resident work lists (token
 * blocks, per-tile segment ranges, reduction chunks).  One packed batch passes through every
 * LoRA linear of every layer with the same table, so a plan is built once per batch and
 * shared by all those calls.  Immutable after creation; concurrent calls may share it. */
typedef struct lobra_mlora_plan lobra_mlora_plan;

/* Host-only argument check of a descriptor (the checks plan_create performs). */
LOBRA_API lobra_status lobra_mlora_validate(const lobra_mlora_desc *desc);

/* Build a plan on the current HIP device.  Allocates one small device buffer
 * (a few bytes per 32 tokens) with hipMalloc and fills it with a blocking copy.
 * *out is set only on success. */
LOBRA_API lobra_status lobra_mlora_plan_create(const lobra_mlora_desc *desc, uint32_t plan_flags,
                                     lobra_mlora_plan **out);

/* The same without any allocation of device memory and without blocking: the plan's device image
 * (*bytes of lobra_mlora_plan_device_bytes for the same desc and flags) goes into device_mem, device memory of the
 * caller (16-byte aligned, device_bytes long), by an asynchronous copy on hip_stream; work that uses the plan
 * must be ordered after that copy (same stream, or an event).  device_mem belongs to the plan until
 * lobra_mlora_plan_destroy, which does not free it.  LOBRA_ERR_WORKSPACE when device_bytes is too small,
 * LOBRA_ERR_PLAN with LOBRA_PLAN_HOST_ONLY. */
LOBRA_API lobra_status lobra_mlora_plan_device_bytes(const lobra_mlora_desc *desc, uint32_t plan_flags, size_t *bytes);
LOBRA_API lobra_status lobra_mlora_plan_init(const lobra_mlora_desc *desc, uint32_t plan_flags, void *device_mem,
                                   size_t device_bytes, void *hip_stream, lobra_mlora_plan **out);

/* Frees the plan (and the device buffer of lobra_mlora_plan_create).  The caller makes sure that no launched
 * work, and no upload of lobra_mlora_plan_init, still uses it.  NULL is accepted. */
LOBRA_API lobra_status lobra_mlora_plan_destroy(lobra_mlora_plan *plan);

/* Buffer sizes in bytes (each may be 0): h_save = the saved down-projected activations that
 * fwd can hand to bwd; fwd_ws / bwd_ws = scratch for one call.  Any out pointer may be NULL. */
LOBRA_API lobra_status lobra_mlora_plan_sizes(const lobra_mlora_plan *plan, size_t *h_save_bytes,
                                    size_t *fwd_ws_bytes, size_t *bwd_ws_bytes);

/* Introspection of the host side of a plan (tests, debugging).  Copies up to `capacity`
 * int32 values of list `what` into out (out may be NULL) and stores the list's full
 * length in *count.
 *   LOBRA_Q_SEGMENTS     compacted table (empty segments dropped, equal-task neighbours merged):
 *                        n x {row0, row_end, task}
 *   LOBRA_Q_ROWBLOCK_SEG per 32-row block: index of the compacted segment holding its first row
 *   LOBRA_Q_TOKEN_BLOCKS n x {row0, nrows, task, rank_row0}: runs of <= 32 tokens of one adapter
 *                        segment, grouped by task; rank_row0 = rank_off[task]
 *   LOBRA_Q_GRAD_CHUNKS  n x {block_begin, block_end, task, partial_row0}: reduction work items
 *   LOBRA_Q_TASK_CHUNKS  [n_tasks+1]: prefix of chunks per task
 *   LOBRA_Q_BLOCK_RUNS   [n_runs+1]: token blocks run[k] .. run[k+1]-1 (all of one task) are
 *                        projected by one workgroup
 *   LOBRA_Q_BLOCK_ORDER  order in which the token blocks are handed to the down-projection's
 *   LOBRA_Q_RUN_ORDER    workgroups, and the same for the runs: a permutation by descending rank
 *                        (stable), or empty when that is the stored order (e.g. equal ranks)
 *   LOBRA_Q_SLICED       {slices_in, slices_out, fused_db, fused_rows, workgroups}: long batches of ranks up
 *                        to 16 are projected by a fixed grid of `workgroups` workgroups that walk (token block,
 *                        512-column slice) items (slices_* = number of slices of d_in / d_out, 0 = the
 *                        one-block-per-workgroup kernels are used for that direction); fused_db = 1: the backward
 *                        projection of dy accumulates dB in the same pass, its sums in fused_rows rows
 *   LOBRA_Q_FUSED_WG_RUNS  [workgroups + 1]: the runs of items of one (task, slice) that workgroup g meets are
 *                        number wg_runs[g] .. wg_runs[g + 1] - 1 (all four lists are empty unless fused_db)
 *   LOBRA_Q_FUSED_RUN_ROW  per run: first of its 16 rows in the array of dB sums
 *   LOBRA_Q_FUSED_COUNT  [n_tasks * slices_out]: runs of (task t, slice c) over all workgroups; its k-th run sits
 *   LOBRA_Q_FUSED_TASK_ROW  at row task_row[t] + 16 k
 *   LOBRA_Q_GEMM_TILE_ROWS  n x 8, one record per 256-token tile row of the base product (tile row i starts at token
 *                        max(0, min(256 i, T - 256))): {segment, first token, last token + 1, task or -1, the task's
 *                        first rank row, its stacked rank, 0, 0} of the compacted segment that holds that token */
enum { LOBRA_Q_SEGMENTS = 0, LOBRA_Q_ROWBLOCK_SEG = 1, LOBRA_Q_TOKEN_BLOCKS = 2,
       LOBRA_Q_GRAD_CHUNKS = 3, LOBRA_Q_TASK_CHUNKS = 4, LOBRA_Q_BLOCK_RUNS = 5,
       LOBRA_Q_BLOCK_ORDER = 6, LOBRA_Q_RUN_ORDER = 7, LOBRA_Q_SLICED = 8, LOBRA_Q_FUSED_WG_RUNS = 9,
       LOBRA_Q_FUSED_RUN_ROW = 10, LOBRA_Q_FUSED_COUNT = 11, LOBRA_Q_FUSED_TASK_ROW = 12,
       LOBRA_Q_GEMM_TILE_ROWS = 13 };
LOBRA_API lobra_status lobra_mlora_plan_query(const lobra_mlora_plan *plan, int32_t what, int32_t *out,
                                    size_t capacity, size_t *count);

/* Forward: y = x W + s_t (A_t x) B_t for every token (section 2.1; fused batch, section 1).
 *   x, W, A, B, y : device, element type desc.dtype, 16-byte aligned; A, B, s may be NULL
 *                   when n_tasks = 0 or no segment carries a task
 *   s             : device fp32 [n_tasks]
 *   h_save        : device, h_save_bytes, or NULL.  When given, bwd can reuse the
 *                   down-projected activations instead of recomputing them
 *   ws, ws_bytes  : device scratch of at least fwd_ws_bytes.  With h_save given only its first
 *                   fwd_ws_bytes - h_save_bytes bytes are used and checked: the partial sums of the
 *                   K-sliced down projection that long batches of ranks up to 16 take (0 bytes for all
 *                   other batches, for which ws may then be NULL)
 *   hip_stream    : hipStream_t (NULL = default stream); work is enqueued, not awaited
 * x, W, A, B, s are read only; y and h_save are overwritten. */
LOBRA_API lobra_status lobra_mlora_plan_fwd(const lobra_mlora_plan *plan, const void *x, const void *W,
                                  const void *A, const void *B, const float *s, void *y,
                                  void *h_save, void *ws, size_t ws_bytes, void *hip_stream);

/* lobra_mlora_plan_fwd for callers that cannot allocate device memory or have none to spare for scratch
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the forward
 * pass with h_save = NULL whose scratch is a fixed array of LOBRA_STATIC_WS_BYTES inside the library's
 * own device image instead of a caller buffer.  Arguments as for lobra_mlora_plan_fwd.  Makes no allocation
 * of any kind and does not synchronise.  LOBRA_ERR_WORKSPACE when the projected activations (h_save_bytes)
 * exceed LOBRA_STATIC_WS_BYTES (nothing is launched); a plan whose fwd_ws_bytes exceed the array only because of
 * the K-sliced projection's partial sums runs the one-block-per-workgroup projection here (same result up to the
 * order of the sums).  Each GPU has ONE such array, which keeps the last
 * call's contents: two calls of this function (or of lobra_token_task_map, which parks its tables there)
 * that overlap in time on the same GPU (different streams, or different threads) race on it and must be
 * ordered by the caller; the saved activations are not available to bwd (pass h_saved = NULL there). */
enum { LOBRA_STATIC_WS_BYTES = 16 * 1024 * 1024 };
LOBRA_API lobra_status lobra_mlora_fwd_static_ws(const lobra_mlora_plan *plan, const void *x, const void *W,
                                       const void *A, const void *B, const float *s, void *y,
                                       void *hip_stream);

/* Backward: dx, dA, dB as defined at the top (derivatives of the section 2.1 layer; W is
 * frozen, so no dW).
 *   dy      : device [T, d_out], element type desc.dtype
 *   h_saved : what the matching fwd call wrote into h_save, or NULL to recompute from x
 *   dx      : device [T, d_in], overwritten (ignored, may be NULL, with LOBRA_FLAG_NO_DX)
 *   dA, dB  : device fp32 [R_tot, d_in] / [R_tot, d_out / n_proj]; overwritten (rows of a task without
 *             tokens become 0), or added to with LOBRA_FLAG_ACCUMULATE_GRADS
 *   ws      : device scratch of at least bwd_ws_bytes
 * The reductions run in a fixed order: results are bit-identical from run to run. */
LOBRA_API lobra_status lobra_mlora_plan_bwd(const lobra_mlora_plan *plan, const void *x, const void *W,
                                  const void *A, const void *B, const float *s, const void *dy,
                                  const void *h_saved, void *dx, float *dA, float *dB,
                                  uint32_t flags, void *ws, size_t ws_bytes, void *hip_stream);

/* Index probe (section 1 / Figure 1: a fused batch is a sequence of task-tagged token runs): writes the task of
 * every token (device int32 [T], -1 = none) and the number of tokens per task (device int64 [n_tasks]) with
 * the same device-side table walk the kernels use.  Either output may be NULL. */
LOBRA_API lobra_status lobra_mlora_plan_token_task_map(const lobra_mlora_plan *plan, int32_t *out_task,
                                             int64_t *out_count, void *hip_stream);

/* ---- one-shot forms: the same operations on the descriptor itself (section 1 / Figure 1: the fused batch is
 * given as its task-tagged token runs; section 2.1: the layer).  Each call validates the descriptor, builds the
 * tables on the host, copies them asynchronously (on hip_stream) to the start of ws and runs the kernels behind
 * that copy.  No device memory is allocated or freed and nothing synchronises; the host image of the tables is
 * released by a host callback on the stream (which is why these forms cannot be captured in a HIP graph: use a
 * plan there).
 *   lobra_mlora_workspace_bytes : bytes of ws that lobra_mlora_fwd (with h_save = NULL) and lobra_mlora_bwd
 *                                 need for this descriptor; host only, no HIP call; either out pointer may be NULL
 *   lobra_mlora_fwd / _bwd      : arguments as for the plan forms; ws (16-byte aligned, device) must hold
 *                                 *fwd_bytes / *bwd_bytes (LOBRA_ERR_WORKSPACE otherwise, before any launch)
 *   lobra_token_task_map        : has no workspace argument: its tables go into the library's static device
 *                                 array (see lobra_mlora_fwd_static_ws for the sharing rule; LOBRA_ERR_WORKSPACE
 *                                 beyond LOBRA_STATIC_WS_BYTES, about 30 million tokens) */
LOBRA_API lobra_status lobra_mlora_workspace_bytes(const lobra_mlora_desc *desc, size_t *fwd_bytes, size_t *bwd_bytes);
LOBRA_API lobra_status lobra_mlora_fwd(const lobra_mlora_desc *desc, const void *x, const void *W, const void *A,
                             const void *B, const float *s, void *y, void *h_save, void *ws, size_t ws_bytes,
                             void *hip_stream);
LOBRA_API lobra_status lobra_mlora_bwd(const lobra_mlora_desc *desc, const void *x, const void *W, const void *A,
                             const void *B, const float *s, const void *dy, const void *h_saved, void *dx,
                             float *dA, float *dB, uint32_t flags, void *ws, size_t ws_bytes, void *hip_stream);
LOBRA_API lobra_status lobra_token_task_map(const lobra_mlora_desc *desc, int32_t *out_task, int64_t *out_count,
                                  void *hip_stream);

/* Fused multi-adapter Adam step: the update that follows the backward pass, for the adapters of
 * all tasks in one launch (the paper trains every task with Adam and cites its decoupled
 * weight-decay form next to it: section 5.1).  Per element of task t, in fp32:
 *     g = grad_scale[t] * grad;  m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2
 *     theta -= lr[t] * ( (m / (1-beta1^k)) / (sqrt(v / (1-beta2^k)) + eps) + weight_decay * theta )
 * with k = step[t], the 1-based count of the step being taken by task t (tasks join a running
 * batch at different times, so every task carries its own count, rate and gradient scale).
 *   plan                 : any plan of this task set (supplies dtype, ranks, d_in, d_out)
 *   lr, grad_scale       : device fp32 [n_tasks]; grad_scale may be NULL (= 1)
 *   step                 : device int32 [n_tasks], every entry >= 1
 *   dA, dB               : device fp32 gradients [R_tot, d_in] / [R_tot, d_out] (read only)
 *   master_A, m_A, v_A   : device fp32 [R_tot, d_in], updated in place; likewise *_B with d_out
 *   A, B                 : device, element type of the plan, or NULL: receive the updated parameters
 *                          rounded once (to nearest even) for the next forward pass
 * Rows of a task whose step entry is <= 0 are left untouched. */
typedef struct {
    float beta1, beta2, eps, weight_decay;
} lobra_adam_config;
LOBRA_API lobra_status lobra_mlora_adam_step(const lobra_mlora_plan *plan, const lobra_adam_config *cfg,
                                   const float *lr, const int32_t *step, const float *grad_scale,
                                   const float *dA, const float *dB, float *master_A,
                                   float *master_B, float *m_A, float *v_A, float *m_B, float *v_B,
                                   void *A, void *B, void *hip_stream);

/* Host-side dynamic bucketing (paper section 4.3, "Dynamic Bucketing"): the caller's step right before
 * the layer when chunks are padded.  Given the lengths of a batch and U candidate boundaries
 * u_1 < ... < u_U, choose at most R of them so that padding every sequence to the closest chosen
 * boundary at or above its length costs the fewest pad tokens (the paper's dynamic programme over
 * State_{i,j}; O(n_seq + R U^2) with prefix sums, empty intervals cost nothing).  Pure host code: all
 * pointers are HOST pointers, no HIP call is made.
 *   seq_len [n_seq]   : every length in [1, bounds[U-1]]
 *   bounds  [U]       : strictly increasing, positive
 *   out_bounds [R]    : the chosen boundaries, ascending, *out_n of them (the rest set to 0); the
 *                       largest one is the smallest candidate that covers the longest sequence
 *   out_padding       : total pad tokens of the batch under the chosen boundaries (may be NULL)
 * LOBRA_ERR_SHAPE for U < 1, R < 1, a non-increasing table or a length outside the table. */
LOBRA_API lobra_status lobra_dynamic_buckets(const int32_t *seq_len, int64_t n_seq, const int32_t *bounds,
                                   int32_t U, int32_t R, int32_t *out_bounds, int32_t *out_n,
                                   int64_t *out_padding);

/* The paper's default chunk layout as input of this operator (section 2.1, "Processing Variable-length Data": the
 * sequences of a chunk are padded to a common length, [b, s_j] tokens): writes the segment table that makes the
 * packed operator treat such a chunk correctly.  Sequence i occupies padded_len[i] consecutive token rows
 * (padded_len = NULL: every sequence occupies uniform_len rows, the [b, s_j] case with b = n_seq, s_j = uniform_len);
 * its first valid_len[i] rows become a segment of task[i], the remaining rows a segment of task -1 (pad tokens:
 * base product only, no contribution to dA and dB).  Pure host code, all pointers are HOST pointers.
 *   seg_off [2 n_seq + 1], seg_task [2 n_seq] : the table (a segment may be empty); *T_out = seg_off[2 n_seq] =
 *                                               the token rows of the chunk (T of the descriptor); may be NULL
 * LOBRA_ERR_SEGMENTS for a valid_len outside [0, padded length], LOBRA_ERR_TASK_ID for a task outside
 * [-1, n_tasks), LOBRA_ERR_SHAPE when the chunk has 2^31 rows or more; on error nothing is written. */
LOBRA_API lobra_status lobra_padded_segments(int64_t n_seq, const int32_t *padded_len, int32_t uniform_len,
                                   const int32_t *valid_len, const int32_t *task, int32_t n_tasks,
                                   int32_t *seg_off, int32_t *seg_task, int64_t *T_out);

/* Profiling aid (bench, tests).  While a trace is attached, every kernel that fwd / bwd /
 * token_task_map launch through this plan is bracketed by hipEventRecord on the call's stream:
 * the i-th launch since the trace was attached records events[2i] before and events[2i+1]
 * after it and stores which kernel it was in kernel_ids[i] (LOBRA_K_*); launches beyond
 * n_pairs are not bracketed.  events are hipEvent_t created by the caller with timing
 * enabled; events and kernel_ids are HOST arrays that must outlive the trace.  *n_launched
 * (host, may be NULL) counts the launches seen.  n_pairs = 0 or events = NULL detaches.
 * A plan with a trace attached must not be used from two threads at once. */
enum { LOBRA_K_SHRINK = 1, LOBRA_K_GEMM = 2, LOBRA_K_GRAD_STAGE1 = 3, LOBRA_K_GRAD_STAGE2 = 4,
       LOBRA_K_TOKEN_TASK = 5, LOBRA_K_ADAM = 6 };
LOBRA_API lobra_status lobra_mlora_plan_set_trace(lobra_mlora_plan *plan, void *const *events,
                                        int32_t n_pairs, int32_t *kernel_ids,
                                        int32_t *n_launched);

/* Static, never NULL. */
LOBRA_API const char *lobra_status_string(lobra_status st);

/* major * 10000 + minor * 100 + patch */
LOBRA_API int lobra_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LOBRA_MLORA_H */
