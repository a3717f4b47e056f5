/*
 * shardupdate: the per-replica hot path of cross-replica weight-update sharding
 * (Xu et al., "Automatic Cross-Replica Sharding of Weight Update in Data-Parallel
 * Training"), hand-written for AMD MI355X (gfx950).
 *
 * One replica out of N owns 1/N of every variable.  The library
 *   (1) formats full tensors into that replica's packed shard        (shard_format),
 *   (2) runs the fused optimizer update on the shard                 (shard_update_*),
 *   (3) restores full tensors from the N gathered shards             (unshard_format).
 * The three calls mirror the paper's sharding program / main program / unsharding
 * program (Section 4.2, "Out-of-loop all-gather placement").  The cross-replica
 * reduce-scatter, all-gather and scalar all-reduce are NOT part of this library: the
 * shard gradient is an input, the gathered [N][S] buffer is an input, and LAMB's
 * per-variable sums of squares are exported / imported as plain device arrays.
 *
 * Layout (Section 4.1, "Data formatting"; Section 5.2, "Batched communication operators").
 * Variable i has n_i elements, taken in row-major order (flattening moves no data).
 *     L_i   = roundup(ceil(n_i / N), align)         piece length, equal on all replicas
 *     off_i = L_0 + ... + L_{i-1},   S = sum L_i    one piece of every variable per shard
 *     shard_r[off_i + k] = (r*L_i + k < n_i) ? var_i[r*L_i + k] : +0.0     0 <= k < L_i
 *     gathered[r][..]    = shard_r                                          shape [N][S] (rows may be strided)
 * Gradient, weight and every auxiliary variable use the same plan (Section 4.1: all
 * inputs of the update must be sharded the same way).
 *
 * Conventions.
 *  - Every function returns an int status: SHARD_OK (0) or a negative SHARD_E* code.
 *    Nothing throws, aborts or prints.
 *  - "device" pointers are HIP device memory on the current device; "host" pointers are
 *    ordinary process memory.  The library allocates no device memory: every device
 *    buffer, including the plan's tables (shard_plan_bind), is the caller's.
 *  - Device buffers of packed shards (w, g, m, v, shard_out, gathered, bf16 outputs,
 *    sums) must be 16-byte aligned, else SHARD_EALIGN.  Full tensors may have any
 *    alignment; each 16-byte aligned one (with align_elems a multiple of 8) is moved with
 *    128-bit accesses, the others element by element, with the same results.
 *  - Kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL = the default
 *    stream) and are asynchronous; errors reported are argument and launch errors.
 *  - A plan is not thread-safe, and calls that use one plan must be ordered on one
 *    stream (or otherwise synchronised by the caller): they share the plan's workspace.
 *  - HIP graphs: the formatting and update calls only launch kernels (no allocation, no
 *    synchronisation, no memset, no events), so a step can be recorded with stream capture.  Scalars passed by
 *    value (replica id, step, hyper-parameters) are frozen into the graph.  The device tables of
 *    full-tensor pointers are cached in the plan's workspace (the 4 most recently used lists), and a
 *    recorded graph reads, at every replay, the tables its calls used while they were captured.  Those
 *    tables are therefore pinned: they keep their pointers, other lists share the remaining slots, and a
 *    call that brings a new list when all 4 are pinned returns SHARD_ESTATE instead of overwriting one.
 *    shard_plan_release_captured_tables unpins them once the graphs that used the plan are gone;
 *    shard_plan_bind to another workspace does too (graphs recorded on the old one are void).
 *    A list that a captured call brings for the first time is uploaded by a kernel recorded into that graph
 *    (no eager warm-up call is needed); until an eager call has brought the same list, eager calls do not
 *    use that table but upload one of their own into another slot.  shard_profile_* timing skips launches on
 *    a capturing stream; do not enable it while another stream of the same thread is being captured in
 *    the global capture mode (event calls are not allowed then).
 */
#ifndef SHARDUPDATE_H
#define SHARDUPDATE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct shard_plan_s shard_plan_t;   /* opaque host object */
typedef void* shard_stream_t;             /* hipStream_t */

enum {
  SHARD_OK = 0,
  SHARD_EINVAL = -1,   /* bad argument (null pointer, r outside [0,N), step < 1, eps <= 0, ...) */
  SHARD_ENOMEM = -2,   /* host allocation failed, or workspace too small */
  SHARD_EALIGN = -3,   /* a packed-shard device pointer is not 16-byte aligned */
  SHARD_EHIP = -4,     /* the HIP runtime reported an error (no device, launch failure) */
  SHARD_ESTATE = -5,   /* the plan has no bound workspace but the call needs one, the workspace holds the
                          intermediate results of another call (shard_update_adafactor_apply), or every
                          pointer-table slot is reserved for recorded graphs and the call brings a new list */
  SHARD_ELIMIT = -6    /* shard_update_lamb_noalloc: the plan exceeds SHARD_NOALLOC_MAX_CHUNKS or _MAX_VARS */
};

enum { SHARD_F32 = 0, SHARD_BF16 = 1 };   /* element types of formatted buffers */

/* Per-variable flags (LAMB and LARS only). */
enum {
  SHARD_VAR_NO_DECAY = 1u,   /* weight decay is not applied to this variable */
  SHARD_VAR_NO_ADAPT = 2u    /* the trust ratio of this variable is fixed at 1 */
};

/* Order of the work items of the whole-model copies (shard_plan_set_copy_walk) and which copy is meant
 * (shard_plan_copy_walk). */
enum { SHARD_WALK_AUTO = 0, SHARD_WALK_BY_REPLICA = 1, SHARD_WALK_BY_VARIABLE = 2 };
enum { SHARD_COPY_UNSHARD = 0, SHARD_COPY_FORMAT_ALL = 1 };

/* Kernel ids for shard_profile_read. */
enum {
  SHARD_K_FORMAT = 0, SHARD_K_UNSHARD = 1, SHARD_K_ADAM = 2, SHARD_K_MOMENTUM = 3,
  SHARD_K_LAMB_P1 = 4, SHARD_K_NORM_REDUCE = 5, SHARD_K_LAMB_P2 = 6, SHARD_K_PTR_TABLE = 7,
  SHARD_K_LARS_P1 = 8, SHARD_K_LARS_P2 = 9, SHARD_K_ROWCOL_P1 = 10, SHARD_K_ROWCOL_P2 = 11,
  SHARD_K_ADAFACTOR_STATE = 12, SHARD_K_ADAFACTOR_USQ = 13, SHARD_K_ADAFACTOR_APPLY = 14,
  SHARD_K_PLAIN_COPY = 15, SHARD_K_ITEM_TOTAL = 16, SHARD_K_ADAM_SHAPE = 17,
  SHARD_K_COUNT = 18
};

const char* shard_strerror(int status);
const char* shard_kernel_name(int kernel_id);   /* NULL if out of range */

/* ------------------------------------------------------------------------------------------
 * shard_plan: the sharding representation (Section 4.1: formatting steps followed by a slice
 * whose offset is a function of the replica id).  Host only, integer arithmetic.
 *   V            number of variables (>= 0)
 *   numel        host array [V], n_i >= 0 (0 is legal and gives L_i = 0)
 *   N            replica count (>= 1)
 *   align_elems  power of two >= 1; the piece granule in elements (8 keeps fp32 and bf16
 *                pieces 16-byte aligned; 1 is the paper's bare ceil(n/N))
 *   var_flags    host array [V] of SHARD_VAR_* bits, or NULL for all zero
 *   chunk_elems  work-item size of the table-driven kernels; 0 picks the tuned default,
 *                otherwise a multiple of 1024 in [1024, 16384]
 *   out          receives the plan; free with shard_plan_free
 * Errors: SHARD_EINVAL, SHARD_ENOMEM.
 */
int shard_plan(int V, const int64_t* numel, int N, int align_elems, const uint32_t* var_flags,
               int chunk_elems, shard_plan_t** out);

/* shard_plan_rows: the paper's own format (Section 4.1): variable i is a row-major rows_i x cols_i
 * matrix (leading dimensions combined into rows, trailing ones into cols; e.g. [3,3,256,256] as
 * 9 x 65536); the row dimension is padded to a multiple of N and replica r owns the whole rows
 * [r*Lr_i, (r+1)*Lr_i), Lr_i = ceil(rows_i / N).  No reshape merges a row with a column, so
 * reductions along either survive sharding (Section 4.1, "Non-elementwise operators").
 *     L_i = roundup(Lr_i * cols_i, align);  shard_r[off_i + k] = (k < Lr_i*cols_i and
 *     r*Lr_i*cols_i + k < rows_i*cols_i) ? var_i[r*Lr_i*cols_i + k] : +0.0
 * Everything else (formatting, updates, unshard) works on such a plan unchanged.  Pieces whose
 * start in the full tensor is not 16-byte aligned are moved element by element.
 * rows, cols: host arrays [V], >= 0.  Other arguments and errors as shard_plan. */
int shard_plan_rows(int V, const int64_t* rows, const int64_t* cols, int N, int align_elems,
                    const uint32_t* var_flags, int chunk_elems, shard_plan_t** out);

/* Sizes of a plan.  Any out pointer may be NULL.
 *   S                packed shard length in elements
 *   total            sum of n_i
 *   n_chunks         entries of the chunk table (a chunk never crosses a variable boundary)
 *   chunk_elems      the chunk size in use
 *   workspace_bytes  device bytes shard_plan_bind needs
 */
int shard_plan_info(const shard_plan_t* plan, int64_t* S, int64_t* total, int64_t* n_chunks,
                    int* chunk_elems, size_t* workspace_bytes);

/* Copies off_i and L_i into host arrays [V] (either may be NULL). */
int shard_plan_segments(const shard_plan_t* plan, int64_t* seg_off, int64_t* seg_len);

/* Host array real[V]: how many of replica r's L_i slots hold real (unpadded) elements. */
int shard_plan_real_count(const shard_plan_t* plan, int r, int64_t* real);

/* Uploads the plan's tables into caller-owned device memory of at least workspace_bytes
 * (256-byte aligned) and remembers it.  The memory must stay valid, and must not be written
 * by the caller, until the plan is freed or bound elsewhere.  The copy is enqueued on
 * `stream`; later calls on the same stream see it. */
int shard_plan_bind(shard_plan_t* plan, void* device_workspace, size_t bytes, shard_stream_t stream);

void shard_plan_free(shard_plan_t* plan);

/* Pointer tables that calls on a capturing stream have used stay reserved for the recorded graphs (see "HIP
 * graphs" above).  Call this when those graphs have been destroyed, to let other lists of tensors use the slots
 * again.  Replaying a graph recorded before this call is then undefined.  Errors: SHARD_EINVAL. */
int shard_plan_release_captured_tables(shard_plan_t* plan);

/* ------------------------------------------------------------------------------------------
 * shard_format: replica r's zero-padded piece of every variable, packed (Section 4.1: the pad
 * is fused into the slice, so only about S elements of the inputs are read).
 *   full_ptrs  HOST array [V] of DEVICE pointers to the full variables (n_i elements of
 *              src_dtype each; entries of empty variables may be NULL)
 *   shard_out  device [S] of dst_dtype
 * dtype pairs: f32->f32 and bf16->bf16 move bits unchanged (NaN payloads, -0.0 survive);
 * f32->bf16 rounds to nearest even (NaN stays NaN, sign kept); bf16->f32 widens exactly.
 * Needs a bound plan.
 */
int shard_format(shard_plan_t* plan, int r, const void* const* full_ptrs, int src_dtype,
                 void* shard_out, int dst_dtype, shard_stream_t stream);

/* shard_format_all: all N pieces in one pass, row r of `out` = shard_r, rows row_stride elements
 * apart (>= S; 0 means S): the buffer a reduce-scatter over N equal contiguous rows consumes
 * (Section 5.1: the piece boundaries of the collective equal the sharding format and the padding
 * is written in place while the pieces are prepared).  Reads every input element once. */
int shard_format_all(shard_plan_t* plan, const void* const* full_ptrs, int src_dtype, void* out,
                     int64_t row_stride, int dst_dtype, shard_stream_t stream);

/* unshard_format: the reverse formatting after the all-gather (Section 4.2).  Reads the gathered
 * shards (device, src_dtype), row r = shard_r starting at element r * row_stride, and writes every
 * full variable (device pointers in the HOST array full_ptrs[V], dst_dtype), dropping the padding.
 *   row_stride  distance between rows in elements, >= S; 0 means S (rows back to back).  Rows that
 *               start on 128-byte boundaries (row_stride a multiple of 32 float32 / 64 bfloat16
 *               elements) copy fastest; the slots between S and row_stride are never touched.
 * Same dtype pairs as shard_format (f32->bf16 is the reduced-precision weight the forward pass
 * needs, Section 4.2). */
int unshard_format(shard_plan_t* plan, const void* gathered, int64_t row_stride, int src_dtype,
                   void* const* full_ptrs, int dst_dtype, shard_stream_t stream);

/* The order in which shard_format_all and unshard_format, which move the whole model, take their work
 * items: replica by replica (each row of the gathered buffer from end to end) or variable by variable (each
 * full tensor from end to end).  The bytes written are the same; the time is not.  Small pieces (many
 * replicas) go by variable, which shard_plan decides.  With large pieces going by replica is the faster by
 * 2 to 6 %, unless the caller's full tensors lie where the pieces that are in flight together collide
 * in memory: equal-sized tensors an exact power of two apart (a framework's allocator places a layer stack's
 * 4 MiB matrices like that) cost that order a quarter of its rate on MI355X, by variable nothing.  Addresses
 * alone do not tell, and the library measures nothing behind the caller's back: which kernel a call launches
 * never depends on timing, and the two copies record and query no events.
 *   SHARD_WALK_AUTO         (default) small pieces go by variable; large pieces (a flat plan, N > 1) go by replica
 *                           unless shard_plan_tune_copy_walk has measured this list of tensors and found by
 *                           variable faster.
 *   SHARD_WALK_BY_REPLICA, SHARD_WALK_BY_VARIABLE   always that order (row plans and N = 1 know only the first).
 * shard_plan_tune_copy_walk: measures both orders of `copy` (SHARD_COPY_UNSHARD: reads `gathered`, writes the full
 *   tensors; SHARD_COPY_FORMAT_ALL: reads the full tensors, writes `gathered`) on the caller's real buffers, and
 *   fixes the order for later calls with the same list of full tensors, element types and row_stride, while that
 *   list stays among the plan's 4 cached ones.  It RUNS the copy 8 times (the destination is overwritten with what
 *   the copy writes), one untimed and three timed launches back to back in each order, and WAITS for them
 *   (hipEventSynchronize): a set-up call, not for the training loop, and refused on a capturing stream
 *   (SHARD_ESTATE).  By variable is taken if it is at least 5 % faster per launch, else by replica.  Where the
 *   order is already fixed (small pieces, a row plan, N = 1, shard_plan_set_copy_walk) nothing is launched.
 *   walk_out (may be NULL) receives the order, best_ms_out (host, 2 floats, may be NULL) the milliseconds per
 *   launch by replica and by variable.  Arguments and errors otherwise as the copy itself.
 * shard_plan_copy_walk reports, for `copy` (SHARD_COPY_*) and a host list of full-tensor pointers (may be NULL),
 *   the order the next such call takes (never SHARD_WALK_AUTO); best_ms_out (host, 2 floats, may be NULL) receives
 *   what shard_plan_tune_copy_walk measured for that list, 0 if it has not been called.  Errors: SHARD_EINVAL. */
int shard_plan_set_copy_walk(shard_plan_t* plan, int walk);
int shard_plan_copy_walk(const shard_plan_t* plan, int copy, const void* const* full_ptrs, int* walk_out,
                         float* best_ms_out);
int shard_plan_tune_copy_walk(shard_plan_t* plan, int copy, void* gathered, int64_t row_stride, int gathered_dtype,
                              void* const* full_ptrs, int full_dtype, shard_stream_t stream, int* walk_out,
                              float* best_ms_out);

/* ------------------------------------------------------------------------------------------
 * Fused optimizer updates on one packed shard (Section 2.2: read gradient, weight and
 * auxiliaries, write weight and auxiliaries; all float32).  w, m, v are updated in place;
 * g is only read.  w_bf16_out, if not NULL, receives bf16(w') [S] (Section 4.2, Figure
 * "all-gather in bfloat16").  Padded slots hold +0.0 and stay +0.0.
 *
 * Adam:     g' = g + wd*w;  m = b1*m + (1-b1)*g';  v = b2*v + (1-b2)*g'^2
 *           w -= lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)           t = step >= 1
 * Momentum: g' = g + wd*w;  m = mu*m + g';  w -= lr*m
 * Requirements: 0 <= beta < 1, eps > 0, step >= 1, else SHARD_EINVAL.
 */
typedef struct { float lr, beta1, beta2, eps, weight_decay; } shard_adam_hp;
typedef struct { float lr, mu, weight_decay; } shard_momentum_hp;
typedef struct { float lr, beta1, beta2, eps, weight_decay; } shard_lamb_hp;
typedef struct { float lr, mu, weight_decay, trust_coeff, eps; } shard_lars_hp;

int shard_update_adam(shard_plan_t* plan, int r, float* w, const float* g, float* m, float* v,
                      void* w_bf16_out, const shard_adam_hp* hp, int64_t step, shard_stream_t stream);

int shard_update_momentum(shard_plan_t* plan, int r, float* w, const float* g, float* m,
                          void* w_bf16_out, const shard_momentum_hp* hp, shard_stream_t stream);

/* LAMB, a non-elementwise optimizer on a shard (Section 4.1, "Non-elementwise operators":
 * mask the padding by position, reduce locally, all-reduce the scalars, then apply).
 *   m, v as Adam (no decay folded in);  u = m_hat/(sqrt(v_hat)+eps) + wd_i*w
 *   per variable i, over ALL replicas:  ratio_i = ||w_i|| / ||u_i||  (1 unless both norms are positive
 *   numbers, i.e. also when one is 0 or NaN, and 1 if the variable has SHARD_VAR_NO_ADAPT);  w -= lr * ratio_i * u
 * Sums of squares are exchanged as float32 tables [V][2] = {sum w^2, sum u^2} in device memory.
 *
 * shard_update_lamb_partials: phase 1.  Updates m and v, leaves w untouched, and writes this
 *   replica's sums over its real elements into local_sumsq_out (padding is masked by
 *   position, whatever the padded slots hold).
 * shard_update_lamb_apply: phase 2.  global_sumsq is the element-wise sum of all replicas'
 *   tables (the scalar all-reduce the caller performs).  Must see the m, v that phase 1 wrote
 *   and the w phase 1 read.
 * shard_update_lamb: both phases in one call; other_replicas_sumsq (may be NULL = zeros) is
 *   added to the local table in place of the all-reduce, and local_sumsq_out (may be NULL)
 *   receives the local table.
 * All need a bound plan.  The reduction order is fixed: results are run-to-run identical.
 */
int shard_update_lamb_partials(shard_plan_t* plan, int r, const float* w, const float* g, float* m, float* v,
                               const shard_lamb_hp* hp, int64_t step, float* local_sumsq_out,
                               shard_stream_t stream);

int shard_update_lamb_apply(shard_plan_t* plan, int r, float* w, const float* m, const float* v,
                            void* w_bf16_out, const shard_lamb_hp* hp, int64_t step,
                            const float* global_sumsq, shard_stream_t stream);

int shard_update_lamb(shard_plan_t* plan, int r, float* w, const float* g, float* m, float* v,
                      void* w_bf16_out, const shard_lamb_hp* hp, int64_t step,
                      const float* other_replicas_sumsq, float* local_sumsq_out, shard_stream_t stream);

/* shard_update_lamb_noalloc: shard_update_lamb for callers that may not allocate device memory and have none to
 * spare for intermediate sums: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels, same results bit for bit; the only difference is where the
 * intermediate sums live: the per-chunk sums of phase 1 and the per-variable sums that phase 2 reads are kept in
 * a fixed array inside the library's code object (2.25 MiB per GPU, held from the library's load to the
 * process's end) instead of the plan's workspace.  The call allocates nothing and frees nothing; the array's
 * address is looked up once per device, at the first call with that device current (make that call outside a
 * stream capture).
 *   Limits: the plan's n_chunks (shard_plan_info) <= SHARD_NOALLOC_MAX_CHUNKS and V <= SHARD_NOALLOC_MAX_VARS,
 *   else SHARD_ELIMIT and nothing is launched.  The plan must still be bound (its tables are read).
 *   Every call on one GPU uses that GPU's one array, whatever the plan or stream: calls that overlap in
 *   time on one GPU race on it and must be ordered by the caller (one stream, or events).  Nothing in the
 *   array has to be cleared between calls: each call writes every entry it later reads.
 * Other errors as shard_update_lamb. */
#define SHARD_NOALLOC_MAX_CHUNKS 262144
#define SHARD_NOALLOC_MAX_VARS 32768
int shard_update_lamb_noalloc(shard_plan_t* plan, int r, float* w, const float* g, float* m, float* v,
                              void* w_bf16_out, const shard_lamb_hp* hp, int64_t step,
                              const float* other_replicas_sumsq, float* local_sumsq_out, shard_stream_t stream);

/* LARS, the optimizer of the paper's ResNet-50 runs (Section 6, Table 1) and its example of a
 * reduce inside the weight update (Section 4.1); same two-phase shape as LAMB.
 *   per variable i over ALL replicas:
 *     local_lr_i = trust_coeff * ||w_i|| / (||g_i|| + wd_i*||w_i|| + eps)
 *     (1 unless both norms are positive numbers, or if the variable has SHARD_VAR_NO_ADAPT; wd_i = 0 with
 *     SHARD_VAR_NO_DECAY)
 *   m = mu*m + lr*local_lr_i*(g + wd_i*w);   w -= m
 * Tables are float32 [V][2] = {sum w^2, sum g^2} in device memory.
 * shard_update_lars_partials reads w and g only; shard_update_lars_apply updates w and m in place
 * from the all-reduced table; shard_update_lars does both, adding other_replicas_sumsq (may be
 * NULL) in place of the all-reduce.  trust_coeff, lr, mu, weight_decay, eps must be finite,
 * eps >= 0.  All need a bound plan.
 */
int shard_update_lars_partials(shard_plan_t* plan, int r, const float* w, const float* g,
                               float* local_sumsq_out, shard_stream_t stream);

int shard_update_lars_apply(shard_plan_t* plan, int r, float* w, const float* g, float* m,
                            void* w_bf16_out, const shard_lars_hp* hp, const float* global_sumsq,
                            shard_stream_t stream);

int shard_update_lars(shard_plan_t* plan, int r, float* w, const float* g, float* m,
                      void* w_bf16_out, const shard_lars_hp* hp, const float* other_replicas_sumsq,
                      float* local_sumsq_out, shard_stream_t stream);

/* The updates with the formatting of the gradient fused into them (Section 5.1: the formatting steps
 * are fused into the operators around them, so that no replica reads and writes the full data just
 * to pad and slice it).  full_g: host array [V] of device pointers to the FULL gradient tensors, the
 * argument shard_format takes (g_dtype SHARD_F32 or SHARD_BF16; any alignment: 16-byte aligned
 * float32 and 8-byte aligned bfloat16 pieces are read with vector loads, the others element by
 * element).  Every kernel that needs the gradient reads replica r's piece of each tensor in place,
 * with +0.0 for the padded slots, so the result is bit for bit that of
 *     shard_format(full_g -> g, float32) followed by the function of the same name without
 *     _full_grads on g,
 * without the 8 bytes per slot of writing g and reading it back.  The pointer list is cached like
 * shard_format's.  All of them need a bound plan (Adam and momentum too: reading in place needs the
 * chunk table).  Other arguments, state and errors as in the plain functions; the second phase of
 * LAMB does not read the gradient and is shard_update_lamb_apply.
 */
int shard_update_adam_full_grads(shard_plan_t* plan, int r, float* w, const void* const* full_g,
                                 int g_dtype, float* m, float* v, void* w_bf16_out,
                                 const shard_adam_hp* hp, int64_t step, shard_stream_t stream);

int shard_update_momentum_full_grads(shard_plan_t* plan, int r, float* w, const void* const* full_g,
                                     int g_dtype, float* m, void* w_bf16_out,
                                     const shard_momentum_hp* hp, shard_stream_t stream);

int shard_update_lamb_partials_full_grads(shard_plan_t* plan, int r, const float* w,
                                          const void* const* full_g, int g_dtype, float* m, float* v,
                                          const shard_lamb_hp* hp, int64_t step, float* local_sumsq_out,
                                          shard_stream_t stream);

int shard_update_lamb_full_grads(shard_plan_t* plan, int r, float* w, const void* const* full_g,
                                 int g_dtype, float* m, float* v, void* w_bf16_out,
                                 const shard_lamb_hp* hp, int64_t step, const float* other_replicas_sumsq,
                                 float* local_sumsq_out, shard_stream_t stream);

int shard_update_lars_partials_full_grads(shard_plan_t* plan, int r, const float* w,
                                          const void* const* full_g, int g_dtype, float* local_sumsq_out,
                                          shard_stream_t stream);

int shard_update_lars_apply_full_grads(shard_plan_t* plan, int r, float* w, const void* const* full_g,
                                       int g_dtype, float* m, void* w_bf16_out, const shard_lars_hp* hp,
                                       const float* global_sumsq, shard_stream_t stream);

int shard_update_lars_full_grads(shard_plan_t* plan, int r, float* w, const void* const* full_g,
                                 int g_dtype, float* m, void* w_bf16_out, const shard_lars_hp* hp,
                                 const float* other_replicas_sumsq, float* local_sumsq_out,
                                 shard_stream_t stream);

/* Reductions that keep a dimension, on a row plan (Section 4.1, "Non-elementwise operators": the
 * format may not merge a collapsed dimension with a passed-through one; with rows sharded, a reduce
 * over columns is complete on the owning replica and a reduce over rows gives per-replica partial
 * results for an all-reduce; padded rows contribute the identity).  These are the two reductions
 * factored second-moment optimizers (Adafactor) take of the gradient.
 *
 * shard_plan_rowcol_layout: host arrays row_off[V], col_off[V] (either may be NULL) and totals:
 *   variable i's Lr_i row sums start at row_off[i] in row_out, its cols_i column sums at
 *   col_off[i] in col_out; total_rows = sum Lr_i, total_cols = sum cols_i.  SHARD_EINVAL on a
 *   flat plan.
 * shard_reduce_sq_rows_cols: x is replica r's packed shard [S] (device, float32).
 *   row_out[row_off[i] + k] = sum over columns of x^2 in row k of the piece (0 for padded rows)
 *   col_out[col_off[i] + c] = sum over the replica's REAL rows of x^2 in column c
 *   Both are device float32 arrays, 16-byte aligned.  Padding is masked by position.  The
 *   summation order is fixed.  Needs a bound row plan.
 */
int shard_plan_rowcol_layout(const shard_plan_t* plan, int64_t* row_off, int64_t* col_off,
                             int64_t* total_rows, int64_t* total_cols);

int shard_reduce_sq_rows_cols(shard_plan_t* plan, int r, const float* x, float* row_out, float* col_out,
                              shard_stream_t stream);

/* ------------------------------------------------------------------------------------------
 * Adafactor on a row plan: an optimizer whose update reduces along rows and along columns (named in
 * Section 3, "Non-elementwise optimizers"; sharded as Section 4.1, "Non-elementwise operators",
 * prescribes: local reduces with the padding masked by position, an all-reduce of the partial
 * results, then element-wise work).  Variable i is a rows_i x cols_i matrix with Lr_i rows on this
 * replica; step t >= 1:
 *     beta2 = 1 - t^(-decay_exponent),  rho = min(max_rho, 1/sqrt(t))
 *     R_k = beta2 R_k + (1-beta2) sum_j (g_kj^2 + eps1)          row state, this replica's rows
 *     C_j = beta2 C_j + (1-beta2) sum_k (g_kj^2 + eps1)          column state, sums over ALL rows, same on all replicas
 *     Vhat_kj = R_k C_j / sum_k R_k;   U = G / sqrt(Vhat);   Uhat = U / max(1, RMS(U) / clip_threshold)
 *     X -= max(eps2, RMS(X)) * rho * Uhat                        RMS over the whole variable
 *   A variable with cols_i == 1 is a vector: R holds the unfactored second moment, Vhat = R, and its
 *   slot of C is never touched.  No momentum, no weight decay; variable flags are ignored.
 * State (device, float32): R [total_rows] laid out by row_off, C [total_cols] laid out by col_off
 * (shard_plan_rowcol_layout); both start at zero.  Padded rows keep R = 0; padded slots of w are not
 * touched.  Two all-reduces separate three local phases:
 *   shard_update_adafactor_partials: reads w, g, R.  row_sq_out [total_rows]: sum over columns of g^2
 *     per row of the piece (0 for padded rows), stays local.  col_sq_out [total_cols]: sum over this
 *     replica's real rows of g^2 per column.  table_out [V][2]: {sum of w^2 over real elements, sum of
 *     R over real rows}.  The caller all-reduces (adds over replicas) col_sq_out and table_out.
 *   shard_update_adafactor_moments: updates R and C in place from row_sq (local) and the all-reduced
 *     col_sq_global and table_global, keeps the factors of 1/sqrt(Vhat) in the plan's workspace and
 *     writes u_sumsq_out [V] = this replica's sum of U^2 over real elements.  The caller all-reduces it.
 *   shard_update_adafactor_apply: updates w (and writes bf16(w') to w_bf16_out, if not NULL) from the
 *     factors phase 2 left in the workspace; must follow the moments call of the same replica and step
 *     on the same plan, with the same hp (SHARD_ESTATE if the last moments call on this plan was for
 *     another replica or step: one plan holds one replica's factors at a time).
 *   shard_update_adafactor: all three; other_col_sq [total_cols], other_table [V][2], other_u_sumsq [V]
 *     (each may be NULL = zeros) are added to the local results in place of the all-reduces.
 * Requirements: a bound row plan; eps1 > 0, eps2 >= 0, clip_threshold > 0, decay_exponent > 0,
 * max_rho > 0, step >= 1 (SHARD_EINVAL otherwise); w and g 16-byte aligned.  Summation orders are fixed.
 */
typedef struct { float eps1, eps2, clip_threshold, decay_exponent, max_rho; } shard_adafactor_hp;

int shard_update_adafactor_partials(shard_plan_t* plan, int r, const float* w, const float* g, const float* R,
                                    float* row_sq_out, float* col_sq_out, float* table_out, shard_stream_t stream);

int shard_update_adafactor_moments(shard_plan_t* plan, int r, const float* g, float* R, float* C, const float* row_sq,
                                   const float* col_sq_global, const float* table_global,
                                   const shard_adafactor_hp* hp, int64_t step, float* u_sumsq_out,
                                   shard_stream_t stream);

int shard_update_adafactor_apply(shard_plan_t* plan, int r, float* w, const float* g, const float* table_global,
                                 const float* u_sumsq_global, void* w_bf16_out, const shard_adafactor_hp* hp,
                                 int64_t step, shard_stream_t stream);

int shard_update_adafactor(shard_plan_t* plan, int r, float* w, const float* g, float* R, float* C, void* w_bf16_out,
                           const shard_adafactor_hp* hp, int64_t step, const float* other_col_sq,
                           const float* other_table, const float* other_u_sumsq, shard_stream_t stream);

/* ------------------------------------------------------------------------------------------
 * Replica arrays (host only, integer arithmetic; the collectives themselves are the caller's).
 * Replica ids are row-major over a rows x cols array: replica = row * cols + column.
 *
 * shard_partial_sharding (Section 5.2, "Partial sharding"): the rows of the array are independent
 *   sharding groups and the columns all-reduce the groups' partial results.  For `replica`:
 *   *group = its row; *shard_id = its column, i.e. the r to pass to shard_plan(.., N = cols, ..)'s
 *   formatting and update calls; shard_group[cols] = the replicas of its row (its reduce-scatter and
 *   all-gather partners, in shard-id order); reduce_group[rows] = the replicas of its column (all
 *   hold the same shard id).  Any out pointer may be NULL.
 * shard_two_phase_shard_id (Section 5.1): full sharding rows*cols ways by a reduce-scatter inside
 *   every row, then inside every column; the final piece of replica (i, j), counted by position in
 *   the data, is j * rows + i.
 * shard_concat_partition (Section 5.2, "Batched communication operators"): a combined all-reduce
 *   concatenates its inputs and cuts the concatenation into `parts` internal pieces of
 *   ceil(total / parts) elements (the last ones shorter or empty), ignoring tensor boundaries.
 * shard_peak_memory (Section 4.2, "Memory saving"): W weights, V auxiliary variables, P peak of
 *   live activations and gradients, in any one unit: *replicated = W + V + P,
 *   *sharded = max(W + V/N + P, W + V).
 * shard_plan_peak_bytes: the same model on a plan, in bytes: W = total * weight_bytes,
 *   V = total * aux_bytes (aux_bytes = bytes of all auxiliary variables per weight element, 8 for
 *   Adam's two float32 moments, weight_bytes + aux_bytes <= 16), and V/N becomes S * aux_bytes,
 *   padding included.
 * Errors: SHARD_EINVAL (dimension < 1, rows * cols >= 2^31, replica or part out of range, negative
 * size, NULL where a result is required).
 */
int shard_partial_sharding(int rows, int cols, int replica, int* group, int* shard_id, int* shard_group,
                           int* reduce_group);
int shard_two_phase_shard_id(int rows, int cols, int replica, int* shard_id);
int shard_concat_partition(int64_t total, int parts, int part, int64_t* start, int64_t* length);
int shard_peak_memory(double W, double V, double P, int N, double* replicated, double* sharded);
int shard_plan_peak_bytes(const shard_plan_t* plan, int weight_bytes, int aux_bytes, int64_t P,
                          int64_t* replicated, int64_t* sharded);

/* ------------------------------------------------------------------------------------------
 * Per-kernel timing with HIP events recorded on the launch stream, for benchmarks.
 * shard_profile_enable(plan, 1) makes every later launch through this plan record an event
 * pair; shard_profile_read synchronises with the recorded events and returns, for one kernel
 * id, the number of launches and their summed duration in milliseconds since the last
 * shard_profile_reset.  Off by default; costs nothing when off.
 */
int shard_profile_enable(shard_plan_t* plan, int on);
int shard_profile_read(shard_plan_t* plan, int kernel_id, int64_t* launches, double* total_ms);
int shard_profile_reset(shard_plan_t* plan);

/* A measurement aid, not part of the path: the plainest device copy there is (one 128-bit access per thread,
 * non-temporal, no table, no padding), launched and timed through the same event mechanism under the kernel
 * id SHARD_K_PLAIN_COPY.  What it reaches on a GPU is the practical ceiling the formatting kernels, which move
 * the same bytes through a chunk table, can be compared with in the same run.
 * dst, src: device pointers, 16-byte aligned, not overlapping; bytes: a positive multiple of 16.
 * Errors: SHARD_EINVAL, SHARD_EALIGN, SHARD_EHIP. */
int shard_profile_plain_copy(shard_plan_t* plan, void* dst, const void* src, size_t bytes, shard_stream_t stream);

/* A second measurement aid: shard_update_adam (without the bf16 output) in a launch shape the caller names instead
 * of the one the library chooses by shard size, timed under the kernel id SHARD_K_ADAM_SHAPE.  It exists so that
 * the measurement behind the library's choice can be repeated: how fast an update of 4 streams read and 3 written
 * runs depends on how many bytes a CU keeps in flight, i.e. on threads per workgroup and on how many workgroups stay
 * resident (capped by reserving LDS the kernel never touches).  The same kernels run, so the state ends up
 * bit for bit as after shard_update_adam.
 *   block_threads      128 or 256
 *   workgroups_per_cu  0 = no cap (what the hardware fits), else 3 .. 16
 * Other arguments and errors as shard_update_adam; SHARD_EINVAL for a shape outside the above. */
int shard_profile_adam_shape(shard_plan_t* plan, float* w, const float* g, float* m, float* v, const shard_adam_hp* hp,
                             int64_t step, int block_threads, int workgroups_per_cu, shard_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* SHARDUPDATE_H */
