// Internal declarations shared by the host-side plan, the C-ABI layer and the HIP launchers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <vector>

#include "shardupdate.h"

namespace su {

// ---- device-visible tables (uploaded by shard_plan_bind) ------------------------------------

// One variable of the plan.  Section 4.1: the piece of replica r starts at r*stride in the flat
// variable; a slot is padding if it lies past the piece's `stride` real slots or if its flat
// index reaches n.
struct VarDesc {
  int64_t n;            // elements of the full variable
  int64_t L;            // slots per replica in the packed shard
  int64_t off;          // offset of the piece in a packed shard
  int64_t stride;       // flat plan: L; row plan: rows per replica * cols (<= L)
  int32_t first_chunk;  // this variable's chunks are [first_chunk, first_chunk + n_chunks)
  int32_t n_chunks;
  uint32_t flags;       // SHARD_VAR_*
  uint32_t reserved;
};
static_assert(sizeof(VarDesc) == 48, "VarDesc layout");

// One work item of the table-driven kernels: `len` consecutive slots of one variable's piece,
// starting k0 slots into the piece.  Never crosses a variable boundary.
struct ChunkDesc {
  int64_t k0;
  int32_t var;
  int32_t len;
};
static_assert(sizeof(ChunkDesc) == 16, "ChunkDesc layout");

// Flat plans only: one work item of the whole-model copies (unshard_format, shard_format_all).
// With stride == L, replica r's piece of variable i is the slots [r*L_i, (r+1)*L_i) of the variable
// padded to N*L_i slots, so the gathered buffer is an [N][L_i] view of that padded variable.  An item
// is `len` consecutive slots of it starting at p0; items are listed variable by variable, so the
// number of workgroups depends on the model size and not on how many (and how small) the pieces are.
// Used when pieces are small (plan_build decides, shard_plan_s::flat_copies); with few large pieces
// the replica-by-replica walk over ChunkDesc items measures 7 % faster.
struct FullChunk {
  int64_t p0;       // first padded slot (= flat index in the full tensor)
  int32_t var;
  int32_t len;
};
static_assert(sizeof(FullChunk) == 16, "FullChunk layout");

// Row plans only: one variable seen as a row-major rows x cols matrix whose rows are sharded, and the
// work items of the kernels that keep rows and columns apart.
struct RowColVar {
  int64_t off;        // piece offset in the packed shard
  int64_t rows;       // rows of the full matrix
  int64_t Lr;         // rows per replica
  int64_t cols;
  int64_t row_off;    // this variable's place in per-row arrays    (sum of Lr of earlier variables)
  int64_t col_off;    // and in per-column arrays                    (sum of cols of earlier variables)
  int64_t cp_off;     // column partials [n_rb][cols] in the workspace
  int64_t rp_off;     // row partials [n_ct][Lr] in the workspace
  int64_t L;          // slots of the piece in the packed shard (>= Lr * cols: alignment tail)
  int32_t n_rb;       // row blocks: kRowBlock rows (tall tiles) or kRowBlock/4 rows (flat tiles)
  int32_t n_ct;       // column tiles: one wavefront's span of columns (tall) or four of them (flat)
  int32_t shape;      // kRcVec: rows start on 16-byte boundaries, threads own 4 adjacent columns;
                      // kRcFlat: at most kRowBlock/4 rows per replica, the four wavefronts sit side by side
  int32_t first_item; // this variable's tile items are [first_item, first_item + n_rb * n_ct)
  int32_t first_col_item, n_col_items;   // its column items (col_span(n_rb) columns each)
};
static_assert(sizeof(RowColVar) == 96, "RowColVar layout");
// One tile.  Tall (the usual case): kRowBlock rows x one wavefront's span of columns; wavefront w of
// the workgroup takes rows 8w .. 8w+7, lane l the columns l*4 .. l*4+3 (or column l) of the tile.
// Flat (pieces of at most 8 rows, e.g. a [3,3,Cin,Cout] kernel's 9 rows over 8 replicas): 8 rows x
// four spans; wavefront w takes the w-th span, so no wavefront idles on rows that do not exist.
constexpr int kRcVec = 1, kRcFlat = 2;
struct RowColItem {
  int32_t var, rb, ct, reserved;
};
// col_span consecutive columns of one variable (per-column work: adding partials, state update).
// A variable with many row blocks gets 64-column items whose four wavefronts share the row blocks;
// one with few gets 256-column items with a thread per column.
struct ColItem {
  int32_t var, tile;
};
constexpr int kDeepRowBlocks = 8;
inline __host__ __device__ int col_span(int n_rb) { return n_rb > kDeepRowBlocks ? 64 : 256; }
// Per-row work.  wide == 0: kBlock consecutive rows starting at first_row, one thread per row;
// wide == 1: the single row first_row, the whole workgroup adds across its many column tiles.
struct RowItem {
  int32_t var, wide;
  int64_t first_row;
};
constexpr int kRowBlock = 32;        // rows per tile
constexpr int kWideTiles = 32;       // a variable with more column tiles than this gets one workgroup per row

constexpr int kBlock = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int kPtrSlots = 4;         // cached device pointer tables per plan
constexpr int kPtrBatch = 256;       // pointers carried by one table-writing launch

struct PtrBatch {
  const void* p[kPtrBatch];
};

// ---- optimizer constants, precomputed on the host in double and rounded once -----------------

struct AdamK {
  float b1, omb1, b2, omb2, rbc1, rbc2, eps, lr, wd;
};
struct MomentumK {
  float mu, lr, wd;
};
struct LarsK {
  float mu, lr, wd, trust, eps;
};
// Adafactor, step t: beta2 = 1 - t^-decay_exponent, omb2 = t^-decay_exponent, rho = min(max_rho, 1/sqrt(t))
struct AdafactorK {
  float beta2, omb2, rho, eps1, eps2, inv_clip;
};

// ---- the plan --------------------------------------------------------------------------------

struct Workspace {
  char* base = nullptr;
  size_t bytes = 0;
  // byte offsets inside base
  size_t vars = 0, chunks = 0, ptrs = 0, chunk_sums = 0, var_sums = 0;
  size_t full_chunks = 0;                                             // flat plans only
  size_t major_chunks = 0, small_full_chunks = 0;                     // flat plans with flat_copies only
  size_t rc_vars = 0, rc_items = 0, rc_colpart = 0, rc_rowpart = 0;   // row plans only
  size_t rc_col_items = 0, rc_row_items = 0, rc_colitem_part = 0;
  // Adafactor (row plans only): per-item partial sums, per-variable scalars, the factors of 1/sqrt(Vhat),
  // and the tables the fused call keeps between its phases
  size_t af_wpart = 0, af_upart = 0, af_inv_r = 0, af_inv_c = 0;
  size_t af_rowsq = 0, af_colsq = 0, af_table = 0, af_usq = 0;
};

struct ProfRecord {
  hipEvent_t start, stop;
  int kernel;
};

// Which of the two orders a whole-model copy takes for one cached pointer table, once shard_plan_tune_copy_walk
// has measured both.  One per (pointer slot, operation); void when the slot gets other pointers, and only valid
// for the element types and row stride it was measured with.
constexpr int kWalkTuneLaunches = 3;  // timed launches per order
struct WalkTrial {
  int src_dtype = -1, dst_dtype = -1;
  int64_t row_stride = -1;
  float best_ms[2] = {0.0f, 0.0f};    // per launch: by replica, by variable
  int chosen = SHARD_WALK_AUTO;       // SHARD_WALK_AUTO: not measured
  void restart() {
    src_dtype = dst_dtype = -1;
    row_stride = -1;
    best_ms[0] = best_ms[1] = 0.0f;
    chosen = SHARD_WALK_AUTO;
  }
};

}  // namespace su

struct shard_plan_s {
  int V = 0, N = 1, align = 1, chunk = 0;
  int64_t S = 0, total = 0;
  std::vector<int64_t> n, L, off, stride;
  std::vector<uint32_t> flags;
  std::vector<su::VarDesc> vars;
  std::vector<su::ChunkDesc> chunks;
  std::vector<su::FullChunk> full_chunks;  // flat plans only
  bool flat_copies = false;                // pieces are small: whole-model copies go variable by variable
  int copy_walk = SHARD_WALK_AUTO;         // shard_plan_set_copy_walk
  su::WalkTrial walk_trial[su::kPtrSlots][2];   // [slot][SHARD_COPY_UNSHARD or SHARD_COPY_FORMAT_ALL]
  // With flat_copies, shard_format_all splits the variables: those whose pieces hold at least one whole chunk go
  // replica by replica (their chunks, copied here), the others variable by variable (their items of full_chunks).
  std::vector<su::ChunkDesc> major_chunks;
  std::vector<su::FullChunk> small_full_chunks;
  bool row_plan = false;
  std::vector<su::RowColVar> rc_vars;      // row plans only
  std::vector<su::RowColItem> rc_items;
  std::vector<su::ColItem> rc_col_items;
  std::vector<su::RowItem> rc_row_items;
  int64_t rc_total_rows = 0, rc_total_cols = 0, rc_colpart_elems = 0, rc_rowpart_elems = 0;

  su::Workspace ws;
  size_t ws_need = 0;

  // cache of uploaded pointer tables: slot -> the V pointers it holds, and an age for LRU
  std::vector<const void*> slot_ptrs[su::kPtrSlots];
  uint64_t slot_age[su::kPtrSlots] = {0, 0, 0, 0};
  bool slot_valid[su::kPtrSlots] = {false, false, false, false};
  // a slot whose table a stream capture has read: a recorded graph reads it at every replay, so it keeps its
  // pointers until shard_plan_release_captured_tables (or the plan's end)
  bool slot_pinned[su::kPtrSlots] = {false, false, false, false};
  // false: the slot's only upload was recorded by a stream capture, so the device may not hold the table yet
  bool slot_on_device[su::kPtrSlots] = {false, false, false, false};
  uint64_t clock = 0;

  // Adafactor: which (replica, step) the factors in the workspace belong to; -1 = none yet
  int af_r = -1;
  int64_t af_step = -1;

  bool prof = false;
  std::vector<su::ProfRecord> prof_live;   // recorded, not yet read
  std::vector<su::ProfRecord> prof_free;   // event pairs ready for reuse
  int64_t prof_count[SHARD_K_COUNT] = {};
  double prof_ms[SHARD_K_COUNT] = {};
};

namespace su {

// plan.cpp (host only)
// cols == nullptr: flat plan over numel[i] elements; otherwise numel[i] is the row count of a rows x cols matrix
int plan_build(shard_plan_t* p, int V, const int64_t* numel, const int64_t* cols, int N, int align,
               const uint32_t* flags, int chunk);
size_t workspace_layout(const shard_plan_t* p, Workspace* ws);

// copies.hip, updates.hip, rowplan.hip: every launcher enqueues on `stream`, returns a hipError_t and never
// synchronises.
hipError_t launch_ptr_table(shard_plan_t* p, const void* const* host_ptrs, const void** dev_table, hipStream_t stream);

hipError_t launch_format(shard_plan_t* p, int r, const void* const* dev_ptr_table, int src_dtype, void* out,
                         int dst_dtype, bool vec, hipStream_t stream);
// by_variable: the work items are chunks of the padded variables (flat plans only), else (replica, chunk)
hipError_t launch_unshard(shard_plan_t* p, const void* gathered, int64_t row_stride, int src_dtype,
                          void* const* dev_ptr_table, int dst_dtype, bool vec, bool by_variable,
                          hipStream_t stream);

hipError_t launch_adam(shard_plan_t* p, float* w, const float* g, float* m, float* v, void* w16, const AdamK& k,
                       hipStream_t stream);
hipError_t launch_momentum(shard_plan_t* p, float* w, const float* g, float* m, void* w16, const MomentumK& k,
                           hipStream_t stream);
// block: 128 or 256 threads; workgroups_per_cu: 0 = no cap, else 3..16 resident workgroups per CU
hipError_t launch_adam_shape(shard_plan_t* p, float* w, const float* g, float* m, float* v, const AdamK& k, int block,
                             int workgroups_per_cu, hipStream_t stream);

// g_source 0: g is the packed shard gradient; 1 / 2: g_full is the device table of full float32 /
// bfloat16 gradient tensors and g is unused.
// chunk_sums (both launchers): where the per-chunk sums go and come from; nullptr = the plan's workspace.
hipError_t launch_lamb_p1(shard_plan_t* p, int r, const float* w, const float* g, int g_source,
                          const void* const* g_full, float* m, float* v, const AdamK& k, hipStream_t stream,
                          float* chunk_sums = nullptr);
// Sums each variable's chunk partials in a fixed order, adds `other` (nullable), writes the totals to
// `sums_out` (nullable) and `local_out` (nullable, without `other`).
hipError_t launch_norm_reduce(shard_plan_t* p, const float* other, float* sums_out, float* local_out,
                              hipStream_t stream, const float* chunk_sums = nullptr);
// The current device's copy of the library's static scratch array (updates.hip): room for the chunk sums of
// SHARD_NOALLOC_MAX_CHUNKS chunks and the sums of SHARD_NOALLOC_MAX_VARS variables.  Resolved once per device.
hipError_t static_lamb_scratch(float** chunk_sums, float** var_sums);
hipError_t launch_lamb_p2(shard_plan_t* p, int r, float* w, const float* m, const float* v, void* w16, const AdamK& k,
                          const float* sums, hipStream_t stream);

hipError_t launch_plain_copy(shard_plan_t* p, void* dst, const void* src, size_t units16, hipStream_t stream);
hipError_t launch_format_all(shard_plan_t* p, const void* const* dev_ptr_table, int src_dtype, void* out,
                             int64_t row_stride, int dst_dtype, bool vec, bool by_variable, hipStream_t stream);
hipError_t launch_lars_p1(shard_plan_t* p, int r, const float* w, const float* g, int g_source,
                          const void* const* g_full, hipStream_t stream);
hipError_t launch_lars_p2(shard_plan_t* p, int r, float* w, const float* g, int g_source, const void* const* g_full,
                          float* m, void* w16, const LarsK& k, const float* sums, hipStream_t stream);
// Chunk-table versions of the Adam and momentum updates that read the gradient from full tensors
// (g_source 1: float32, 2: bfloat16).
hipError_t launch_adam_full_grads(shard_plan_t* p, int r, float* w, int g_source, const void* const* g_full, float* m,
                                  float* v, void* w16, const AdamK& k, hipStream_t stream);
hipError_t launch_momentum_full_grads(shard_plan_t* p, int r, float* w, int g_source, const void* const* g_full,
                                      float* m, void* w16, const MomentumK& k, hipStream_t stream);

// Row/column sums of squares on a row plan: phase 1 writes per-item partials, phase 2 adds them in
// a fixed order into row_out [sum Lr] and col_out [sum cols].
hipError_t launch_rowcol_sumsq(shard_plan_t* p, int r, const float* x, float* row_out, float* col_out,
                               hipStream_t stream);

// Adafactor on a row plan (rowplan.hip).  Phase 1: row sums and column sums of g^2, and per variable
// {sum w^2, sum of the old row state}; other_* (nullable) are added (all-reduce stand-ins).
hipError_t launch_adafactor_partials(shard_plan_t* p, int r, const float* w, const float* g, const float* R,
                                     const float* other_col, const float* other_table, float* row_sq, float* col_sq,
                                     float* table, bool keep_column_item_sums, hipStream_t stream);
// Phase 2: new row/column state, the factors of 1/sqrt(Vhat) (kept in the workspace), per-variable sum of U^2.
hipError_t launch_adafactor_moments(shard_plan_t* p, int r, const float* g, float* R, float* C, const float* row_sq,
                                    const float* col_sq_global, const float* table_global, const AdafactorK& k,
                                    bool have_column_item_sums, const float* other_usq, float* usq_local,
                                    float* usq_total, hipStream_t stream);
// Phase 3: the weight update, from the factors phase 2 left in the workspace.
hipError_t launch_adafactor_apply(shard_plan_t* p, int r, float* w, const float* g, const float* table_global,
                                  const float* usq_global, void* w16, const AdafactorK& k, hipStream_t stream);

// Whether work enqueued on `stream` is being recorded into a graph rather than run (profile.cpp).
bool stream_is_capturing(hipStream_t stream);

// RAII helper: records an event pair around a launch when profiling is on and the stream is not capturing.
struct ProfScope {
  shard_plan_t* p;
  hipStream_t stream;
  ProfRecord rec;
  bool on;
  ProfScope(shard_plan_t* plan, int kernel, hipStream_t s);
  ~ProfScope();
};

}  // namespace su
