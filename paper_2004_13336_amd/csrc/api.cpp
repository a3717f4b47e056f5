// The C-ABI layer: argument checks, host-side constant folding, pointer-table caching.
// Every kernel launch lives in the .hip files; nothing here computes on tensor data.
#include <cmath>
#include <cstring>
#include <new>

#include "internal.hpp"

using namespace su;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline hipStream_t as_stream(shard_stream_t s) { return reinterpret_cast<hipStream_t>(s); }
inline int hip_status(hipError_t e) { return e == hipSuccess ? SHARD_OK : SHARD_EHIP; }
inline bool dtype_ok(int d) { return d == SHARD_F32 || d == SHARD_BF16; }

// Folds the hyper-parameters of an Adam-shaped step into float constants.  Powers and
// reciprocals are taken in double and rounded once.
int fold_adam(float lr, float beta1, float beta2, float eps, float wd, int64_t step, AdamK* k) {
  if (step < 1) return SHARD_EINVAL;
  if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f)) return SHARD_EINVAL;
  if (!(eps > 0.0f) || !std::isfinite(lr) || !std::isfinite(wd)) return SHARD_EINVAL;
  const double b1 = beta1, b2 = beta2;
  k->b1 = beta1;
  k->b2 = beta2;
  k->omb1 = (float)(1.0 - b1);
  k->omb2 = (float)(1.0 - b2);
  k->rbc1 = (float)(1.0 / (1.0 - std::pow(b1, (double)step)));
  k->rbc2 = (float)(1.0 / (1.0 - std::pow(b2, (double)step)));
  k->eps = eps;
  k->lr = lr;
  k->wd = wd;
  return SHARD_OK;
}

int check_shard_ptr(const void* p) {
  if (p == nullptr) return SHARD_EINVAL;
  return aligned16(p) ? SHARD_OK : SHARD_EALIGN;
}

int check_plan_r(const shard_plan_t* p, int r, bool need_ws) {
  if (p == nullptr || r < 0 || r >= p->N) return SHARD_EINVAL;
  if (need_ws && p->ws.base == nullptr) return SHARD_ESTATE;
  return SHARD_OK;
}

// Returns the device address of a pointer table holding `ptrs`, uploading it into the least
// recently used slot unless an identical table is already resident.  A table that a capturing stream uses is
// pinned: the recorded graph will read that slot at every replay, so no other list may take it (SHARD_ESTATE
// once every slot is pinned and yet another list arrives).
// A launch on a capturing stream is recorded, not run: a table whose only upload was recorded is not on the
// device until the graph's first replay (slot_on_device stays false).  Eager calls never use such a slot, they
// upload the list into another one; captured calls that meet it record the upload again, so that every graph
// carries the uploads it depends on.
int resident_ptr_table(shard_plan_t* p, const void* const* ptrs, hipStream_t stream, const void*** table,
                       int* slot_out = nullptr) {
  const size_t bytes = (size_t)p->V * sizeof(void*);
  const bool capturing = stream_is_capturing(stream);
  int slot = -1;
  for (int s = 0; s < kPtrSlots; ++s) {
    if (!p->slot_valid[s] || (bytes != 0 && std::memcmp(p->slot_ptrs[s].data(), ptrs, bytes) != 0)) continue;
    if (!p->slot_on_device[s] && !capturing) continue;                 // only a recorded upload: not for eager use
    if (slot < 0 || (p->slot_on_device[s] && !p->slot_on_device[slot])) slot = s;
  }
  const void** base = reinterpret_cast<const void**>(p->ws.base + p->ws.ptrs);
  const bool fresh = slot < 0;
  if (fresh) {
    for (int s = 0; s < kPtrSlots && slot < 0; ++s)
      if (!p->slot_valid[s] && !p->slot_pinned[s]) slot = s;  // a free slot first
    if (slot < 0) {
      for (int s = 0; s < kPtrSlots; ++s)                    // else the least recently used that no graph reads
        if (!p->slot_pinned[s] && (slot < 0 || p->slot_age[s] < p->slot_age[slot])) slot = s;
      if (slot < 0) return SHARD_ESTATE;
    }
  }
  if (fresh || !p->slot_on_device[slot]) {
    const void** dev = base + (size_t)slot * p->V;
    if (p->V > 0) {
      if (launch_ptr_table(p, ptrs, dev, stream) != hipSuccess) {
        if (fresh) p->slot_valid[slot] = false;
        return SHARD_EHIP;
      }
      if (fresh) std::memcpy(p->slot_ptrs[slot].data(), ptrs, bytes);
    }
    if (fresh) {
      p->slot_valid[slot] = true;
      p->slot_on_device[slot] = !capturing;
      for (WalkTrial& t : p->walk_trial[slot]) t.restart();  // other tensors: what was measured no longer holds
    }
  }
  if (capturing) p->slot_pinned[slot] = true;
  p->slot_age[slot] = ++p->clock;
  *table = base + (size_t)slot * p->V;
  if (slot_out) *slot_out = slot;
  return SHARD_OK;
}

// ---- the order of a whole-model copy -----------------------------------------------------------
// Both orders move the same bytes to the same places.  Which is faster depends on the piece size (small
// pieces: by variable, decided when the plan is built) and, for large pieces, on how the caller's full tensors
// lie in memory: equal-sized tensors a power of two apart make the pieces that are in flight together by
// replica fall on the same memory channels and banks, and that order then loses a quarter of its rate
// while the other keeps it.  The library cannot tell from the addresses and measures nothing behind the
// caller's back: large pieces go by replica unless the caller fixes the order (shard_plan_set_copy_walk) or has
// it measured for a list of tensors (shard_plan_tune_copy_walk), so the kernel a call launches never depends on
// timing, and the copies themselves record and query no events.

// Static answer, or SHARD_WALK_AUTO where the order belongs to the list of tensors (tuned, else by replica).
int static_walk(const shard_plan_t* p) {
  if (p->row_plan || p->full_chunks.empty() || p->N == 1) return SHARD_WALK_BY_REPLICA;
  if (p->copy_walk != SHARD_WALK_AUTO) return p->copy_walk;
  if (p->flat_copies) return SHARD_WALK_BY_VARIABLE;
  return SHARD_WALK_AUTO;
}

bool go_by_variable(const shard_plan_t* p, int slot, int op, int src_dtype, int dst_dtype, int64_t row_stride) {
  const int fixed = static_walk(p);
  if (fixed != SHARD_WALK_AUTO) return fixed == SHARD_WALK_BY_VARIABLE;
  const WalkTrial& t = p->walk_trial[slot][op];
  return t.chosen == SHARD_WALK_BY_VARIABLE && t.src_dtype == src_dtype && t.dst_dtype == dst_dtype &&
         t.row_stride == row_stride;
}

// 128-bit path: pieces start on 16-byte boundaries for both element sizes.  (Whether each full
// tensor does too is checked per variable inside the kernels.)
bool pieces_vectorisable(const shard_plan_t* p) { return p->align % 8 == 0; }

int check_full_ptrs(const shard_plan_t* p, const void* const* ptrs) {
  if (p->V > 0 && ptrs == nullptr) return SHARD_EINVAL;
  for (int i = 0; i < p->V; ++i)
    if (p->n[i] > 0 && ptrs[i] == nullptr) return SHARD_EINVAL;
  return SHARD_OK;
}

const char* const kKernelNames[SHARD_K_COUNT] = {
    "format_kernel", "unshard_kernel", "adam_kernel", "momentum_kernel",
    "lamb_p1_kernel", "norm_reduce_kernel", "lamb_p2_kernel", "ptr_table_kernel",
    "lars_p1_kernel", "lars_p2_kernel", "rowcol_p1_kernel", "rowcol_p2_kernel",
    "adafactor_state_kernel", "adafactor_usq_kernel", "adafactor_apply_kernel", "plain_copy_kernel",
    "item_total_kernel", "adam_kernel (named shape)",
};

// Step-dependent constants of Adafactor, taken in double and rounded once.
int fold_adafactor(const shard_adafactor_hp* hp, int64_t step, AdafactorK* k) {
  if (hp == nullptr || step < 1) return SHARD_EINVAL;
  if (!(hp->eps1 > 0.0f) || !(hp->eps2 >= 0.0f) || !(hp->clip_threshold > 0.0f) || !(hp->decay_exponent > 0.0f) ||
      !(hp->max_rho > 0.0f) || !std::isfinite(hp->eps1) || !std::isfinite(hp->eps2) ||
      !std::isfinite(hp->clip_threshold) || !std::isfinite(hp->decay_exponent) || !std::isfinite(hp->max_rho))
    return SHARD_EINVAL;
  const double t = (double)step;
  const double one_minus = std::pow(t, -(double)hp->decay_exponent);       // 1 - beta2
  const double inv_sqrt_t = 1.0 / std::sqrt(t);
  k->beta2 = (float)(1.0 - one_minus);
  k->omb2 = (float)one_minus;
  k->rho = (float)((double)hp->max_rho < inv_sqrt_t ? (double)hp->max_rho : inv_sqrt_t);
  k->eps1 = hp->eps1;
  k->eps2 = hp->eps2;
  k->inv_clip = (float)(1.0 / (double)hp->clip_threshold);
  return SHARD_OK;
}

int check_row_plan(const shard_plan_t* p, int r) {
  const int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  return p->row_plan ? SHARD_OK : SHARD_EINVAL;
}

int fold_lars(const shard_lars_hp* hp, LarsK* k) {
  if (hp == nullptr) return SHARD_EINVAL;
  if (!std::isfinite(hp->lr) || !std::isfinite(hp->mu) || !std::isfinite(hp->weight_decay) ||
      !std::isfinite(hp->trust_coeff) || !std::isfinite(hp->eps) || hp->eps < 0.0f)
    return SHARD_EINVAL;
  k->mu = hp->mu;
  k->lr = hp->lr;
  k->wd = hp->weight_decay;
  k->trust = hp->trust_coeff;
  k->eps = hp->eps;
  return SHARD_OK;
}

// The gradient argument of an update: a packed shard, or the list of full tensors the shard would have
// been formatted from (the *_full_grads entry points).
struct GradArg {
  const float* shard;
  const void* const* full;
  int dtype;
  bool from_full;
};
inline GradArg shard_grad(const float* g) { return GradArg{g, nullptr, SHARD_F32, false}; }
inline GradArg full_grads(const void* const* ptrs, int dtype) { return GradArg{nullptr, ptrs, dtype, true}; }

int check_grad(const shard_plan_t* p, const GradArg& g) {
  if (!g.from_full) return p->S > 0 ? check_shard_ptr(g.shard) : SHARD_OK;
  if (!dtype_ok(g.dtype)) return SHARD_EINVAL;
  return check_full_ptrs(p, g.full);
}

// g_source of the launchers (0 shard, 1 full float32, 2 full bfloat16) and, for full tensors, the device
// table of their pointers.
int resolve_grad(shard_plan_t* p, const GradArg& g, hipStream_t s, int* source, const void*** table) {
  *source = 0;
  *table = nullptr;
  if (!g.from_full) return SHARD_OK;
  *source = g.dtype == SHARD_F32 ? 1 : 2;
  return resident_ptr_table(p, g.full, s, table);
}

int lamb_partials_any(shard_plan_t* p, int r, const float* w, const GradArg& g, float* m, float* v,
                      const shard_lamb_hp* hp, int64_t step, float* local_sumsq_out, shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  if (hp == nullptr) return SHARD_EINVAL;
  AdamK k;
  if ((rc = fold_adam(hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, step, &k)) != SHARD_OK) return rc;
  if (g.from_full && (rc = check_grad(p, g)) != SHARD_OK) return rc;
  if (p->V == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(local_sumsq_out)) != SHARD_OK) return rc;
  if (p->S > 0 && ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_grad(p, g)) != SHARD_OK ||
                   (rc = check_shard_ptr(m)) != SHARD_OK || (rc = check_shard_ptr(v)) != SHARD_OK))
    return rc;
  hipStream_t s = as_stream(stream);
  int source;
  const void** table;
  if ((rc = resolve_grad(p, g, s, &source, &table)) != SHARD_OK) return rc;
  hipError_t e = launch_lamb_p1(p, r, w, g.shard, source, table, m, v, k, s);
  if (e == hipSuccess) e = launch_norm_reduce(p, nullptr, nullptr, local_sumsq_out, s);
  return hip_status(e);
}

int lamb_any(shard_plan_t* p, int r, float* w, const GradArg& g, float* m, float* v, void* w_bf16_out,
             const shard_lamb_hp* hp, int64_t step, const float* other_replicas_sumsq, float* local_sumsq_out,
             shard_stream_t stream, bool static_scratch = false) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  if (hp == nullptr) return SHARD_EINVAL;
  if (static_scratch && (p->chunks.size() > (size_t)SHARD_NOALLOC_MAX_CHUNKS || p->V > SHARD_NOALLOC_MAX_VARS))
    return SHARD_ELIMIT;
  AdamK k;
  if ((rc = fold_adam(hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, step, &k)) != SHARD_OK) return rc;
  if (g.from_full && (rc = check_grad(p, g)) != SHARD_OK) return rc;
  if (p->V == 0) return SHARD_OK;
  if ((other_replicas_sumsq && !aligned16(other_replicas_sumsq)) || (local_sumsq_out && !aligned16(local_sumsq_out)))
    return SHARD_EALIGN;
  if (p->S > 0 && ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_grad(p, g)) != SHARD_OK ||
                   (rc = check_shard_ptr(m)) != SHARD_OK || (rc = check_shard_ptr(v)) != SHARD_OK))
    return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  hipStream_t s = as_stream(stream);
  int source;
  const void** table;
  if ((rc = resolve_grad(p, g, s, &source, &table)) != SHARD_OK) return rc;
  float* sums = reinterpret_cast<float*>(p->ws.base + p->ws.var_sums);
  float* chunk_sums = nullptr;                                 // the workspace's
  // Every chunk's pair and every variable's pair is written before it is read, so the static array
  // needs no clearing between calls.
  if (static_scratch && static_lamb_scratch(&chunk_sums, &sums) != hipSuccess) return SHARD_EHIP;
  hipError_t e = launch_lamb_p1(p, r, w, g.shard, source, table, m, v, k, s, chunk_sums);
  if (e == hipSuccess) e = launch_norm_reduce(p, other_replicas_sumsq, sums, local_sumsq_out, s, chunk_sums);
  if (e == hipSuccess) e = launch_lamb_p2(p, r, w, m, v, w_bf16_out, k, sums, s);
  return hip_status(e);
}

int lars_partials_any(shard_plan_t* p, int r, const float* w, const GradArg& g, float* local_sumsq_out,
                      shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  if (g.from_full && (rc = check_grad(p, g)) != SHARD_OK) return rc;
  if (p->V == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(local_sumsq_out)) != SHARD_OK) return rc;
  if (p->S > 0 && ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_grad(p, g)) != SHARD_OK)) return rc;
  hipStream_t s = as_stream(stream);
  int source;
  const void** table;
  if ((rc = resolve_grad(p, g, s, &source, &table)) != SHARD_OK) return rc;
  hipError_t e = launch_lars_p1(p, r, w, g.shard, source, table, s);
  if (e == hipSuccess) e = launch_norm_reduce(p, nullptr, nullptr, local_sumsq_out, s);
  return hip_status(e);
}

int lars_apply_any(shard_plan_t* p, int r, float* w, const GradArg& g, float* m, void* w_bf16_out,
                   const shard_lars_hp* hp, const float* global_sumsq, shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  LarsK k;
  if ((rc = fold_lars(hp, &k)) != SHARD_OK) return rc;
  if (g.from_full && (rc = check_grad(p, g)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(global_sumsq)) != SHARD_OK || (rc = check_shard_ptr(w)) != SHARD_OK ||
      (rc = check_grad(p, g)) != SHARD_OK || (rc = check_shard_ptr(m)) != SHARD_OK)
    return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  hipStream_t s = as_stream(stream);
  int source;
  const void** table;
  if ((rc = resolve_grad(p, g, s, &source, &table)) != SHARD_OK) return rc;
  return hip_status(launch_lars_p2(p, r, w, g.shard, source, table, m, w_bf16_out, k, global_sumsq, s));
}

int lars_any(shard_plan_t* p, int r, float* w, const GradArg& g, float* m, void* w_bf16_out, const shard_lars_hp* hp,
             const float* other_replicas_sumsq, float* local_sumsq_out, shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  LarsK k;
  if ((rc = fold_lars(hp, &k)) != SHARD_OK) return rc;
  if (g.from_full && (rc = check_grad(p, g)) != SHARD_OK) return rc;
  if (p->V == 0) return SHARD_OK;
  if ((other_replicas_sumsq && !aligned16(other_replicas_sumsq)) || (local_sumsq_out && !aligned16(local_sumsq_out)))
    return SHARD_EALIGN;
  if (p->S > 0 && ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_grad(p, g)) != SHARD_OK ||
                   (rc = check_shard_ptr(m)) != SHARD_OK))
    return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  hipStream_t s = as_stream(stream);
  int source;
  const void** table;
  if ((rc = resolve_grad(p, g, s, &source, &table)) != SHARD_OK) return rc;
  float* sums = reinterpret_cast<float*>(p->ws.base + p->ws.var_sums);
  hipError_t e = launch_lars_p1(p, r, w, g.shard, source, table, s);
  if (e == hipSuccess) e = launch_norm_reduce(p, other_replicas_sumsq, sums, local_sumsq_out, s);
  if (e == hipSuccess) e = launch_lars_p2(p, r, w, g.shard, source, table, m, w_bf16_out, k, sums, s);
  return hip_status(e);
}

}  // namespace

extern "C" {

const char* shard_strerror(int status) {
  switch (status) {
    case SHARD_OK: return "ok";
    case SHARD_EINVAL: return "invalid argument";
    case SHARD_ENOMEM: return "out of memory or workspace too small";
    case SHARD_EALIGN: return "packed-shard pointer not 16-byte aligned";
    case SHARD_EHIP: return "HIP runtime error";
    case SHARD_ESTATE: return "plan has no bound workspace, or its workspace holds another call's intermediate results";
    case SHARD_ELIMIT: return "the plan has more chunks or variables than the library's static scratch array holds";
    default: return "unknown status";
  }
}

const char* shard_kernel_name(int kernel_id) {
  return (kernel_id >= 0 && kernel_id < SHARD_K_COUNT) ? kKernelNames[kernel_id] : nullptr;
}

int shard_plan(int V, const int64_t* numel, int N, int align_elems, const uint32_t* var_flags, int chunk_elems,
               shard_plan_t** out) {
  if (out == nullptr) return SHARD_EINVAL;
  *out = nullptr;
  shard_plan_t* p = new (std::nothrow) shard_plan_s();
  if (p == nullptr) return SHARD_ENOMEM;
  const int rc = plan_build(p, V, numel, nullptr, N, align_elems, var_flags, chunk_elems);
  if (rc != SHARD_OK) {
    delete p;
    return rc;
  }
  *out = p;
  return SHARD_OK;
}

int shard_plan_rows(int V, const int64_t* rows, const int64_t* cols, int N, int align_elems, const uint32_t* var_flags,
                    int chunk_elems, shard_plan_t** out) {
  if (out == nullptr) return SHARD_EINVAL;
  *out = nullptr;
  if (V > 0 && cols == nullptr) return SHARD_EINVAL;
  static const int64_t none = 0;
  shard_plan_s* p = new (std::nothrow) shard_plan_s();
  if (p == nullptr) return SHARD_ENOMEM;
  const int rc = plan_build(p, V, rows, V > 0 ? cols : &none, N, align_elems, var_flags, chunk_elems);
  if (rc != SHARD_OK) {
    delete p;
    return rc;
  }
  *out = p;
  return SHARD_OK;
}

int shard_plan_info(const shard_plan_t* p, int64_t* S, int64_t* total, int64_t* n_chunks, int* chunk_elems,
                    size_t* workspace_bytes) {
  if (p == nullptr) return SHARD_EINVAL;
  if (S) *S = p->S;
  if (total) *total = p->total;
  if (n_chunks) *n_chunks = (int64_t)p->chunks.size();
  if (chunk_elems) *chunk_elems = p->chunk;
  if (workspace_bytes) *workspace_bytes = p->ws_need;
  return SHARD_OK;
}

int shard_plan_segments(const shard_plan_t* p, int64_t* seg_off, int64_t* seg_len) {
  if (p == nullptr) return SHARD_EINVAL;
  for (int i = 0; i < p->V; ++i) {
    if (seg_off) seg_off[i] = p->off[i];
    if (seg_len) seg_len[i] = p->L[i];
  }
  return SHARD_OK;
}

int shard_plan_real_count(const shard_plan_t* p, int r, int64_t* real) {
  if (p == nullptr || real == nullptr || r < 0 || r >= p->N) return SHARD_EINVAL;
  for (int i = 0; i < p->V; ++i) {
    const int64_t rem = p->n[i] - (int64_t)r * p->stride[i];
    real[i] = rem <= 0 ? 0 : (rem < p->stride[i] ? rem : p->stride[i]);
  }
  return SHARD_OK;
}

int shard_plan_bind(shard_plan_t* p, void* device_workspace, size_t bytes, shard_stream_t stream) {
  if (p == nullptr || device_workspace == nullptr) return SHARD_EINVAL;
  if ((reinterpret_cast<uintptr_t>(device_workspace) & 255u) != 0) return SHARD_EALIGN;
  if (bytes < p->ws_need) return SHARD_ENOMEM;
  Workspace ws;
  workspace_layout(p, &ws);
  ws.base = static_cast<char*>(device_workspace);
  ws.bytes = bytes;
  hipStream_t s = as_stream(stream);
  if (!p->vars.empty() &&
      hipMemcpyAsync(ws.base + ws.vars, p->vars.data(), p->vars.size() * sizeof(VarDesc), hipMemcpyHostToDevice, s) !=
          hipSuccess)
    return SHARD_EHIP;
  if (!p->chunks.empty() && hipMemcpyAsync(ws.base + ws.chunks, p->chunks.data(), p->chunks.size() * sizeof(ChunkDesc),
                                           hipMemcpyHostToDevice, s) != hipSuccess)
    return SHARD_EHIP;
  if (!p->full_chunks.empty() && hipMemcpyAsync(ws.base + ws.full_chunks, p->full_chunks.data(),
                                                p->full_chunks.size() * sizeof(FullChunk), hipMemcpyHostToDevice,
                                                s) != hipSuccess)
    return SHARD_EHIP;
  if (!p->major_chunks.empty() && hipMemcpyAsync(ws.base + ws.major_chunks, p->major_chunks.data(),
                                                 p->major_chunks.size() * sizeof(ChunkDesc), hipMemcpyHostToDevice,
                                                 s) != hipSuccess)
    return SHARD_EHIP;
  if (!p->small_full_chunks.empty() && hipMemcpyAsync(ws.base + ws.small_full_chunks, p->small_full_chunks.data(),
                                                      p->small_full_chunks.size() * sizeof(FullChunk),
                                                      hipMemcpyHostToDevice, s) != hipSuccess)
    return SHARD_EHIP;
  if (p->row_plan) {
    if (!p->rc_vars.empty() && hipMemcpyAsync(ws.base + ws.rc_vars, p->rc_vars.data(), p->rc_vars.size() * sizeof(RowColVar),
                                              hipMemcpyHostToDevice, s) != hipSuccess)
      return SHARD_EHIP;
    if (!p->rc_items.empty() && hipMemcpyAsync(ws.base + ws.rc_items, p->rc_items.data(),
                                               p->rc_items.size() * sizeof(RowColItem), hipMemcpyHostToDevice,
                                               s) != hipSuccess)
      return SHARD_EHIP;
    if (!p->rc_col_items.empty() && hipMemcpyAsync(ws.base + ws.rc_col_items, p->rc_col_items.data(),
                                                   p->rc_col_items.size() * sizeof(ColItem), hipMemcpyHostToDevice,
                                                   s) != hipSuccess)
      return SHARD_EHIP;
    if (!p->rc_row_items.empty() && hipMemcpyAsync(ws.base + ws.rc_row_items, p->rc_row_items.data(),
                                                   p->rc_row_items.size() * sizeof(RowItem), hipMemcpyHostToDevice,
                                                   s) != hipSuccess)
      return SHARD_EHIP;
  }
  p->ws = ws;
  for (int i = 0; i < kPtrSlots; ++i) p->slot_valid[i] = p->slot_pinned[i] = p->slot_on_device[i] = false;   // graphs recorded on the old workspace are void
  return SHARD_OK;
}

void shard_plan_free(shard_plan_t* p) {
  if (p == nullptr) return;
  for (auto& rec : p->prof_live) {
    (void)hipEventDestroy(rec.start);
    (void)hipEventDestroy(rec.stop);
  }
  for (auto& rec : p->prof_free) {
    (void)hipEventDestroy(rec.start);
    (void)hipEventDestroy(rec.stop);
  }
  delete p;
}

int shard_format(shard_plan_t* p, int r, const void* const* full_ptrs, int src_dtype, void* shard_out, int dst_dtype,
                 shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  if (!dtype_ok(src_dtype) || !dtype_ok(dst_dtype)) return SHARD_EINVAL;
  if ((rc = check_full_ptrs(p, full_ptrs)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(shard_out)) != SHARD_OK) return rc;
  const void** table = nullptr;
  if ((rc = resident_ptr_table(p, full_ptrs, as_stream(stream), &table)) != SHARD_OK) return rc;
  return hip_status(launch_format(p, r, table, src_dtype, shard_out, dst_dtype,
                                  pieces_vectorisable(p), as_stream(stream)));
}

int shard_format_all(shard_plan_t* p, const void* const* full_ptrs, int src_dtype, void* out, int64_t row_stride,
                     int dst_dtype, shard_stream_t stream) {
  int rc = check_plan_r(p, 0, true);
  if (rc != SHARD_OK) return rc;
  if (!dtype_ok(src_dtype) || !dtype_ok(dst_dtype)) return SHARD_EINVAL;
  if (row_stride == 0) row_stride = p->S;
  if (row_stride < p->S) return SHARD_EINVAL;
  if ((rc = check_full_ptrs(p, full_ptrs)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(out)) != SHARD_OK) return rc;
  const void** table = nullptr;
  int slot = 0;
  if ((rc = resident_ptr_table(p, full_ptrs, as_stream(stream), &table, &slot)) != SHARD_OK) return rc;
  const bool vec = pieces_vectorisable(p) && row_stride % 8 == 0;
  const bool by_variable = go_by_variable(p, slot, SHARD_COPY_FORMAT_ALL, src_dtype, dst_dtype, row_stride);
  return hip_status(launch_format_all(p, table, src_dtype, out, row_stride, dst_dtype, vec, by_variable,
                                      as_stream(stream)));
}

int unshard_format(shard_plan_t* p, const void* gathered, int64_t row_stride, int src_dtype, void* const* full_ptrs,
                   int dst_dtype, shard_stream_t stream) {
  int rc = check_plan_r(p, 0, true);
  if (rc != SHARD_OK) return rc;
  if (!dtype_ok(src_dtype) || !dtype_ok(dst_dtype)) return SHARD_EINVAL;
  if (row_stride == 0) row_stride = p->S;
  if (row_stride < p->S) return SHARD_EINVAL;
  if ((rc = check_full_ptrs(p, full_ptrs)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(gathered)) != SHARD_OK) return rc;
  const void** table = nullptr;
  int slot = 0;
  if ((rc = resident_ptr_table(p, full_ptrs, as_stream(stream), &table, &slot)) != SHARD_OK) return rc;
  const bool vec = pieces_vectorisable(p) && row_stride % 8 == 0;   // rows stay 16-byte aligned
  const bool by_variable = go_by_variable(p, slot, SHARD_COPY_UNSHARD, src_dtype, dst_dtype, row_stride);
  return hip_status(launch_unshard(p, gathered, row_stride, src_dtype,
                                   reinterpret_cast<void* const*>(const_cast<void**>(table)), dst_dtype, vec,
                                   by_variable, as_stream(stream)));
}

int shard_plan_release_captured_tables(shard_plan_t* p) {
  if (p == nullptr) return SHARD_EINVAL;
  for (int s = 0; s < kPtrSlots; ++s) {
    p->slot_pinned[s] = false;
    if (!p->slot_on_device[s]) p->slot_valid[s] = false;     // its upload was only ever recorded
  }
  return SHARD_OK;
}

int shard_plan_set_copy_walk(shard_plan_t* p, int walk) {
  if (p == nullptr || (walk != SHARD_WALK_AUTO && walk != SHARD_WALK_BY_REPLICA && walk != SHARD_WALK_BY_VARIABLE))
    return SHARD_EINVAL;
  p->copy_walk = walk;
  return SHARD_OK;
}

int shard_plan_copy_walk(const shard_plan_t* p, int copy, const void* const* full_ptrs, int* walk_out,
                         float* best_ms_out) {
  if (p == nullptr || walk_out == nullptr || (copy != SHARD_COPY_UNSHARD && copy != SHARD_COPY_FORMAT_ALL))
    return SHARD_EINVAL;
  if (best_ms_out) best_ms_out[0] = best_ms_out[1] = 0.0f;
  *walk_out = static_walk(p);
  if (*walk_out != SHARD_WALK_AUTO) return SHARD_OK;
  *walk_out = SHARD_WALK_BY_REPLICA;                       // large pieces, nothing fixed, nothing tuned
  if (full_ptrs == nullptr) return SHARD_OK;
  const size_t bytes = (size_t)p->V * sizeof(void*);
  for (int s = 0; s < kPtrSlots; ++s)
    if (p->slot_valid[s] && p->slot_on_device[s] && std::memcmp(p->slot_ptrs[s].data(), full_ptrs, bytes) == 0) {
      const WalkTrial& t = p->walk_trial[s][copy];
      if (t.chosen == SHARD_WALK_AUTO) continue;
      *walk_out = t.chosen;
      if (best_ms_out) {
        best_ms_out[0] = t.best_ms[0];
        best_ms_out[1] = t.best_ms[1];
      }
    }
  return SHARD_OK;
}

int shard_plan_tune_copy_walk(shard_plan_t* p, int copy, void* gathered, int64_t row_stride, int gathered_dtype,
                              void* const* full_ptrs, int full_dtype, shard_stream_t stream, int* walk_out,
                              float* best_ms_out) {
  int rc = check_plan_r(p, 0, true);
  if (rc != SHARD_OK) return rc;
  if (copy != SHARD_COPY_UNSHARD && copy != SHARD_COPY_FORMAT_ALL) return SHARD_EINVAL;
  if (!dtype_ok(gathered_dtype) || !dtype_ok(full_dtype)) return SHARD_EINVAL;
  if (row_stride == 0) row_stride = p->S;
  if (row_stride < p->S) return SHARD_EINVAL;
  const void* const* cptrs = const_cast<const void* const*>(full_ptrs);
  if ((rc = check_full_ptrs(p, cptrs)) != SHARD_OK) return rc;
  if (best_ms_out) best_ms_out[0] = best_ms_out[1] = 0.0f;
  hipStream_t s = as_stream(stream);
  if (stream_is_capturing(s)) return SHARD_ESTATE;          // it waits for its own launches
  const int src_dtype = copy == SHARD_COPY_UNSHARD ? gathered_dtype : full_dtype;
  const int dst_dtype = copy == SHARD_COPY_UNSHARD ? full_dtype : gathered_dtype;
  const int fixed = static_walk(p);
  if (fixed != SHARD_WALK_AUTO || p->S == 0) {              // nothing for a measurement to decide
    if (walk_out) *walk_out = fixed == SHARD_WALK_AUTO ? SHARD_WALK_BY_REPLICA : fixed;
    return SHARD_OK;
  }
  if ((rc = check_shard_ptr(gathered)) != SHARD_OK) return rc;
  const void** table = nullptr;
  int slot = 0;
  if ((rc = resident_ptr_table(p, cptrs, s, &table, &slot)) != SHARD_OK) return rc;
  const bool vec = pieces_vectorisable(p) && row_stride % 8 == 0;
  hipEvent_t ev[2] = {nullptr, nullptr};
  if (hipEventCreate(&ev[0]) != hipSuccess || hipEventCreate(&ev[1]) != hipSuccess) {
    if (ev[0]) (void)hipEventDestroy(ev[0]);
    return SHARD_EHIP;
  }
  // Each order: one untimed launch, then kWalkTuneLaunches back to back inside one event pair, so that each
  // launch also pays for what its predecessor left in the caches, as in a training loop.
  float ms[2] = {0.0f, 0.0f};
  hipError_t e = hipSuccess;
  for (int order = 0; order < 2 && e == hipSuccess; ++order) {
    const bool by_variable = order == 1;
    for (int k = 0; k <= kWalkTuneLaunches && e == hipSuccess; ++k) {
      if (k == 1) e = hipEventRecord(ev[0], s);
      if (e != hipSuccess) break;
      e = copy == SHARD_COPY_UNSHARD
              ? launch_unshard(p, gathered, row_stride, src_dtype, reinterpret_cast<void* const*>(const_cast<void**>(table)),
                               dst_dtype, vec, by_variable, s)
              : launch_format_all(p, table, src_dtype, gathered, row_stride, dst_dtype, vec, by_variable, s);
    }
    if (e == hipSuccess) e = hipEventRecord(ev[1], s);
    if (e == hipSuccess) e = hipEventSynchronize(ev[1]);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms[order], ev[0], ev[1]);
    ms[order] /= (float)kWalkTuneLaunches;
  }
  (void)hipEventDestroy(ev[0]);
  (void)hipEventDestroy(ev[1]);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return SHARD_EHIP;
  }
  WalkTrial& t = p->walk_trial[slot][copy];
  t.src_dtype = src_dtype;
  t.dst_dtype = dst_dtype;
  t.row_stride = row_stride;
  t.best_ms[0] = ms[0];
  t.best_ms[1] = ms[1];
  // Well-placed tensors go 2 to 6 % faster by replica inside a training step; colliding ones 8 to 25 % faster by
  // variable.  Launches of the same copy back to back flatter going by variable by up to 4 % (part of what the
  // copy reads is still in the memory-side cache, which other kernels of a real step would have displaced), so only
  // a lead beyond that changes the order.
  t.chosen = ms[1] < 0.95f * ms[0] ? SHARD_WALK_BY_VARIABLE : SHARD_WALK_BY_REPLICA;
  if (walk_out) *walk_out = t.chosen;
  if (best_ms_out) {
    best_ms_out[0] = ms[0];
    best_ms_out[1] = ms[1];
  }
  return SHARD_OK;
}

int shard_update_adam(shard_plan_t* p, int r, float* w, const float* g, float* m, float* v, void* w_bf16_out,
                      const shard_adam_hp* hp, int64_t step, shard_stream_t stream) {
  int rc = check_plan_r(p, r, false);
  if (rc != SHARD_OK) return rc;
  if (hp == nullptr) return SHARD_EINVAL;
  AdamK k;
  if ((rc = fold_adam(hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, step, &k)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_shard_ptr(g)) != SHARD_OK ||
      (rc = check_shard_ptr(m)) != SHARD_OK || (rc = check_shard_ptr(v)) != SHARD_OK)
    return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  return hip_status(launch_adam(p, w, g, m, v, w_bf16_out, k, as_stream(stream)));
}

int shard_update_momentum(shard_plan_t* p, int r, float* w, const float* g, float* m, void* w_bf16_out,
                          const shard_momentum_hp* hp, shard_stream_t stream) {
  int rc = check_plan_r(p, r, false);
  if (rc != SHARD_OK) return rc;
  if (hp == nullptr || !std::isfinite(hp->lr) || !std::isfinite(hp->mu) || !std::isfinite(hp->weight_decay))
    return SHARD_EINVAL;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_shard_ptr(g)) != SHARD_OK ||
      (rc = check_shard_ptr(m)) != SHARD_OK)
    return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  MomentumK k{hp->mu, hp->lr, hp->weight_decay};
  return hip_status(launch_momentum(p, w, g, m, w_bf16_out, k, as_stream(stream)));
}

int shard_update_adam_full_grads(shard_plan_t* p, int r, float* w, const void* const* full_g, int g_dtype, float* m,
                                 float* v, void* w_bf16_out, const shard_adam_hp* hp, int64_t step,
                                 shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  if (hp == nullptr) return SHARD_EINVAL;
  AdamK k;
  if ((rc = fold_adam(hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, step, &k)) != SHARD_OK) return rc;
  const GradArg g = full_grads(full_g, g_dtype);
  if ((rc = check_grad(p, g)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_shard_ptr(m)) != SHARD_OK ||
      (rc = check_shard_ptr(v)) != SHARD_OK)
    return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  hipStream_t s = as_stream(stream);
  int source;
  const void** table;
  if ((rc = resolve_grad(p, g, s, &source, &table)) != SHARD_OK) return rc;
  return hip_status(launch_adam_full_grads(p, r, w, source, table, m, v, w_bf16_out, k, s));
}

int shard_update_momentum_full_grads(shard_plan_t* p, int r, float* w, const void* const* full_g, int g_dtype,
                                     float* m, void* w_bf16_out, const shard_momentum_hp* hp, shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  if (hp == nullptr || !std::isfinite(hp->lr) || !std::isfinite(hp->mu) || !std::isfinite(hp->weight_decay))
    return SHARD_EINVAL;
  const GradArg g = full_grads(full_g, g_dtype);
  if ((rc = check_grad(p, g)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_shard_ptr(m)) != SHARD_OK) return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  hipStream_t s = as_stream(stream);
  int source;
  const void** table;
  if ((rc = resolve_grad(p, g, s, &source, &table)) != SHARD_OK) return rc;
  MomentumK k{hp->mu, hp->lr, hp->weight_decay};
  return hip_status(launch_momentum_full_grads(p, r, w, source, table, m, w_bf16_out, k, s));
}

int shard_update_lamb_partials(shard_plan_t* p, int r, const float* w, const float* g, float* m, float* v,
                               const shard_lamb_hp* hp, int64_t step, float* local_sumsq_out, shard_stream_t stream) {
  return lamb_partials_any(p, r, w, shard_grad(g), m, v, hp, step, local_sumsq_out, stream);
}

int shard_update_lamb_partials_full_grads(shard_plan_t* p, int r, const float* w, const void* const* full_g,
                                          int g_dtype, float* m, float* v, const shard_lamb_hp* hp, int64_t step,
                                          float* local_sumsq_out, shard_stream_t stream) {
  return lamb_partials_any(p, r, w, full_grads(full_g, g_dtype), m, v, hp, step, local_sumsq_out, stream);
}

int shard_update_lamb_apply(shard_plan_t* p, int r, float* w, const float* m, const float* v, void* w_bf16_out,
                            const shard_lamb_hp* hp, int64_t step, const float* global_sumsq, shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  if (hp == nullptr) return SHARD_EINVAL;
  AdamK k;
  if ((rc = fold_adam(hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, step, &k)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(global_sumsq)) != SHARD_OK || (rc = check_shard_ptr(w)) != SHARD_OK ||
      (rc = check_shard_ptr(m)) != SHARD_OK || (rc = check_shard_ptr(v)) != SHARD_OK)
    return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  return hip_status(launch_lamb_p2(p, r, w, m, v, w_bf16_out, k, global_sumsq, as_stream(stream)));
}

int shard_update_lamb(shard_plan_t* p, int r, float* w, const float* g, float* m, float* v, void* w_bf16_out,
                      const shard_lamb_hp* hp, int64_t step, const float* other_replicas_sumsq,
                      float* local_sumsq_out, shard_stream_t stream) {
  return lamb_any(p, r, w, shard_grad(g), m, v, w_bf16_out, hp, step, other_replicas_sumsq, local_sumsq_out, stream);
}

int shard_update_lamb_noalloc(shard_plan_t* p, int r, float* w, const float* g, float* m, float* v, void* w_bf16_out,
                              const shard_lamb_hp* hp, int64_t step, const float* other_replicas_sumsq,
                              float* local_sumsq_out, shard_stream_t stream) {
  return lamb_any(p, r, w, shard_grad(g), m, v, w_bf16_out, hp, step, other_replicas_sumsq, local_sumsq_out, stream,
                  true);
}

int shard_update_lamb_full_grads(shard_plan_t* p, int r, float* w, const void* const* full_g, int g_dtype, float* m,
                                 float* v, void* w_bf16_out, const shard_lamb_hp* hp, int64_t step,
                                 const float* other_replicas_sumsq, float* local_sumsq_out, shard_stream_t stream) {
  return lamb_any(p, r, w, full_grads(full_g, g_dtype), m, v, w_bf16_out, hp, step, other_replicas_sumsq,
                  local_sumsq_out, stream);
}

int shard_update_lars_partials(shard_plan_t* p, int r, const float* w, const float* g, float* local_sumsq_out,
                               shard_stream_t stream) {
  return lars_partials_any(p, r, w, shard_grad(g), local_sumsq_out, stream);
}

int shard_update_lars_partials_full_grads(shard_plan_t* p, int r, const float* w, const void* const* full_g,
                                          int g_dtype, float* local_sumsq_out, shard_stream_t stream) {
  return lars_partials_any(p, r, w, full_grads(full_g, g_dtype), local_sumsq_out, stream);
}

int shard_update_lars_apply(shard_plan_t* p, int r, float* w, const float* g, float* m, void* w_bf16_out,
                            const shard_lars_hp* hp, const float* global_sumsq, shard_stream_t stream) {
  return lars_apply_any(p, r, w, shard_grad(g), m, w_bf16_out, hp, global_sumsq, stream);
}

int shard_update_lars_apply_full_grads(shard_plan_t* p, int r, float* w, const void* const* full_g, int g_dtype,
                                       float* m, void* w_bf16_out, const shard_lars_hp* hp, const float* global_sumsq,
                                       shard_stream_t stream) {
  return lars_apply_any(p, r, w, full_grads(full_g, g_dtype), m, w_bf16_out, hp, global_sumsq, stream);
}

int shard_update_lars(shard_plan_t* p, int r, float* w, const float* g, float* m, void* w_bf16_out,
                      const shard_lars_hp* hp, const float* other_replicas_sumsq, float* local_sumsq_out,
                      shard_stream_t stream) {
  return lars_any(p, r, w, shard_grad(g), m, w_bf16_out, hp, other_replicas_sumsq, local_sumsq_out, stream);
}

int shard_update_lars_full_grads(shard_plan_t* p, int r, float* w, const void* const* full_g, int g_dtype, float* m,
                                 void* w_bf16_out, const shard_lars_hp* hp, const float* other_replicas_sumsq,
                                 float* local_sumsq_out, shard_stream_t stream) {
  return lars_any(p, r, w, full_grads(full_g, g_dtype), m, w_bf16_out, hp, other_replicas_sumsq, local_sumsq_out,
                  stream);
}

int shard_plan_rowcol_layout(const shard_plan_t* p, int64_t* row_off, int64_t* col_off, int64_t* total_rows,
                             int64_t* total_cols) {
  if (p == nullptr || !p->row_plan) return SHARD_EINVAL;
  for (int i = 0; i < p->V; ++i) {
    if (row_off) row_off[i] = p->rc_vars[i].row_off;
    if (col_off) col_off[i] = p->rc_vars[i].col_off;
  }
  if (total_rows) *total_rows = p->rc_total_rows;
  if (total_cols) *total_cols = p->rc_total_cols;
  return SHARD_OK;
}

int shard_reduce_sq_rows_cols(shard_plan_t* p, int r, const float* x, float* row_out, float* col_out,
                              shard_stream_t stream) {
  int rc = check_plan_r(p, r, true);
  if (rc != SHARD_OK) return rc;
  if (!p->row_plan) return SHARD_EINVAL;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(x)) != SHARD_OK) return rc;
  if (p->rc_total_rows > 0 && (rc = check_shard_ptr(row_out)) != SHARD_OK) return rc;
  if (p->rc_total_cols > 0 && (rc = check_shard_ptr(col_out)) != SHARD_OK) return rc;
  return hip_status(launch_rowcol_sumsq(p, r, x, row_out, col_out, as_stream(stream)));
}

int shard_update_adafactor_partials(shard_plan_t* p, int r, const float* w, const float* g, const float* R,
                                    float* row_sq_out, float* col_sq_out, float* table_out, shard_stream_t stream) {
  int rc = check_row_plan(p, r);
  if (rc != SHARD_OK) return rc;
  if (p->V == 0) return SHARD_OK;
  if (table_out == nullptr) return SHARD_EINVAL;
  if ((p->rc_total_rows > 0 && (R == nullptr || row_sq_out == nullptr)) || (p->rc_total_cols > 0 && col_sq_out == nullptr))
    return SHARD_EINVAL;
  if (p->S > 0 && ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_shard_ptr(g)) != SHARD_OK)) return rc;
  return hip_status(launch_adafactor_partials(p, r, w, g, R, nullptr, nullptr, row_sq_out, col_sq_out, table_out,
                                              false, as_stream(stream)));
}

int shard_update_adafactor_moments(shard_plan_t* p, int r, const float* g, float* R, float* C, const float* row_sq,
                                   const float* col_sq_global, const float* table_global,
                                   const shard_adafactor_hp* hp, int64_t step, float* u_sumsq_out,
                                   shard_stream_t stream) {
  int rc = check_row_plan(p, r);
  if (rc != SHARD_OK) return rc;
  AdafactorK k;
  if ((rc = fold_adafactor(hp, step, &k)) != SHARD_OK) return rc;
  if (p->V == 0) return SHARD_OK;
  if (table_global == nullptr || u_sumsq_out == nullptr) return SHARD_EINVAL;
  if ((p->rc_total_rows > 0 && (R == nullptr || row_sq == nullptr)) ||
      (p->rc_total_cols > 0 && (C == nullptr || col_sq_global == nullptr)))
    return SHARD_EINVAL;
  if (p->S > 0 && (rc = check_shard_ptr(g)) != SHARD_OK) return rc;
  p->af_r = r;
  p->af_step = step;
  return hip_status(launch_adafactor_moments(p, r, g, R, C, row_sq, col_sq_global, table_global, k, false, nullptr,
                                             u_sumsq_out, nullptr, as_stream(stream)));
}

int shard_update_adafactor_apply(shard_plan_t* p, int r, float* w, const float* g, const float* table_global,
                                 const float* u_sumsq_global, void* w_bf16_out, const shard_adafactor_hp* hp,
                                 int64_t step, shard_stream_t stream) {
  int rc = check_row_plan(p, r);
  if (rc != SHARD_OK) return rc;
  AdafactorK k;
  if ((rc = fold_adafactor(hp, step, &k)) != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if (table_global == nullptr || u_sumsq_global == nullptr) return SHARD_EINVAL;
  if ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_shard_ptr(g)) != SHARD_OK) return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  if (p->af_r != r || p->af_step != step) return SHARD_ESTATE;   // the workspace holds another call's factors
  return hip_status(launch_adafactor_apply(p, r, w, g, table_global, u_sumsq_global, w_bf16_out, k, as_stream(stream)));
}

int shard_update_adafactor(shard_plan_t* p, int r, float* w, const float* g, float* R, float* C, void* w_bf16_out,
                           const shard_adafactor_hp* hp, int64_t step, const float* other_col_sq,
                           const float* other_table, const float* other_u_sumsq, shard_stream_t stream) {
  int rc = check_row_plan(p, r);
  if (rc != SHARD_OK) return rc;
  AdafactorK k;
  if ((rc = fold_adafactor(hp, step, &k)) != SHARD_OK) return rc;
  if (p->V == 0) return SHARD_OK;
  if ((p->rc_total_rows > 0 && R == nullptr) || (p->rc_total_cols > 0 && C == nullptr)) return SHARD_EINVAL;
  if (p->S > 0 && ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_shard_ptr(g)) != SHARD_OK)) return rc;
  if (w_bf16_out && !aligned16(w_bf16_out)) return SHARD_EALIGN;
  hipStream_t s = as_stream(stream);
  float* row_sq = reinterpret_cast<float*>(p->ws.base + p->ws.af_rowsq);
  float* col_sq = reinterpret_cast<float*>(p->ws.base + p->ws.af_colsq);
  float* table = reinterpret_cast<float*>(p->ws.base + p->ws.af_table);
  float* usq = reinterpret_cast<float*>(p->ws.base + p->ws.af_usq);
  p->af_r = -1;                                                  // the fused call leaves nothing for a later apply
  hipError_t e = launch_adafactor_partials(p, r, w, g, R, other_col_sq, other_table, row_sq, col_sq, table, true, s);
  if (e == hipSuccess) e = launch_adafactor_moments(p, r, g, R, C, row_sq, col_sq, table, k, true, other_u_sumsq, nullptr, usq, s);
  if (e == hipSuccess) e = launch_adafactor_apply(p, r, w, g, table, usq, w_bf16_out, k, s);
  return hip_status(e);
}

int shard_profile_enable(shard_plan_t* p, int on) {
  if (p == nullptr) return SHARD_EINVAL;
  p->prof = on != 0;
  return SHARD_OK;
}

int shard_profile_read(shard_plan_t* p, int kernel_id, int64_t* launches, double* total_ms) {
  if (p == nullptr || kernel_id < 0 || kernel_id >= SHARD_K_COUNT) return SHARD_EINVAL;
  int rc = SHARD_OK;
  for (auto& rec : p->prof_live) {
    float ms = 0.0f;
    if (hipEventSynchronize(rec.stop) != hipSuccess || hipEventElapsedTime(&ms, rec.start, rec.stop) != hipSuccess) {
      rc = SHARD_EHIP;
    } else {
      p->prof_count[rec.kernel] += 1;
      p->prof_ms[rec.kernel] += (double)ms;
    }
    p->prof_free.push_back(rec);
  }
  p->prof_live.clear();
  if (launches) *launches = p->prof_count[kernel_id];
  if (total_ms) *total_ms = p->prof_ms[kernel_id];
  return rc;
}

int shard_profile_reset(shard_plan_t* p) {
  if (p == nullptr) return SHARD_EINVAL;
  int64_t n;
  (void)shard_profile_read(p, 0, &n, nullptr);   // drain pending records
  for (int i = 0; i < SHARD_K_COUNT; ++i) {
    p->prof_count[i] = 0;
    p->prof_ms[i] = 0.0;
  }
  return SHARD_OK;
}

int shard_profile_adam_shape(shard_plan_t* p, float* w, const float* g, float* m, float* v, const shard_adam_hp* hp,
                             int64_t step, int block_threads, int workgroups_per_cu, shard_stream_t stream) {
  if (p == nullptr || hp == nullptr) return SHARD_EINVAL;
  if (block_threads != 128 && block_threads != 256) return SHARD_EINVAL;
  if (workgroups_per_cu != 0 && (workgroups_per_cu < 3 || workgroups_per_cu > 16)) return SHARD_EINVAL;
  AdamK k;
  int rc = fold_adam(hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, step, &k);
  if (rc != SHARD_OK) return rc;
  if (p->S == 0) return SHARD_OK;
  if ((rc = check_shard_ptr(w)) != SHARD_OK || (rc = check_shard_ptr(g)) != SHARD_OK ||
      (rc = check_shard_ptr(m)) != SHARD_OK || (rc = check_shard_ptr(v)) != SHARD_OK)
    return rc;
  return hip_status(launch_adam_shape(p, w, g, m, v, k, block_threads, workgroups_per_cu, as_stream(stream)));
}

int shard_profile_plain_copy(shard_plan_t* p, void* dst, const void* src, size_t bytes, shard_stream_t stream) {
  if (p == nullptr || dst == nullptr || src == nullptr || bytes == 0 || bytes % 16 != 0) return SHARD_EINVAL;
  if (!aligned16(dst) || !aligned16(src)) return SHARD_EALIGN;
  if (bytes / 16 > (size_t)0x7FFFFFFF * 256) return SHARD_EINVAL;          // more workgroups than a launch can hold
  return hip_status(launch_plain_copy(p, dst, src, bytes / 16, as_stream(stream)));
}

}  // extern "C"
