// Host-side arithmetic of replica arrays: partial sharding, multi-phase shard ids, the internal
// partition of a combined all-reduce, and the peak-memory model.  Integer bookkeeping only; the
// collectives themselves are outside this library.
//
// Section 5.1: on an N x M device array a reduce-scatter runs inside each row, then inside each
// column, and the shard id follows the topology of all phases.  Section 5.2: the rows of an N x M
// array of replicas are independent sharding groups, the columns all-reduce the partial results;
// a combined all-reduce partitions the concatenation of its inputs.  Section 4.2 ("Memory
// saving"): W + V + P becomes max(W + V/N + P, W + V).
#include <limits>

#include "internal.hpp"

namespace {
inline bool array_ok(int rows, int cols, int replica) {
  if (rows < 1 || cols < 1) return false;
  if ((int64_t)rows * cols > (int64_t)std::numeric_limits<int32_t>::max()) return false;
  return replica >= 0 && (int64_t)replica < (int64_t)rows * cols;
}
}  // namespace

extern "C" {

int shard_partial_sharding(int rows, int cols, int replica, int* group, int* shard_id, int* shard_group,
                           int* reduce_group) {
  if (!array_ok(rows, cols, replica)) return SHARD_EINVAL;
  const int row = replica / cols, col = replica % cols;     // replica ids are row-major over the array
  if (group) *group = row;
  if (shard_id) *shard_id = col;
  if (shard_group)
    for (int j = 0; j < cols; ++j) shard_group[j] = row * cols + j;
  if (reduce_group)
    for (int i = 0; i < rows; ++i) reduce_group[i] = i * cols + col;
  return SHARD_OK;
}

int shard_two_phase_shard_id(int rows, int cols, int replica, int* shard_id) {
  if (!array_ok(rows, cols, replica) || shard_id == nullptr) return SHARD_EINVAL;
  const int row = replica / cols, col = replica % cols;
  // the row phase hands out `cols` pieces by column, the column phase cuts each into `rows` by row
  *shard_id = col * rows + row;
  return SHARD_OK;
}

int shard_concat_partition(int64_t total, int parts, int part, int64_t* start, int64_t* length) {
  if (total < 0 || parts < 1 || part < 0 || part >= parts) return SHARD_EINVAL;
  const int64_t piece = total / parts + (total % parts != 0 ? 1 : 0);
  // part * piece can exceed total only when piece >= 1, and then by less than parts * piece <= total + parts
  int64_t s = (piece == 0) ? 0 : ((int64_t)part <= total / piece ? (int64_t)part * piece : total);
  if (s > total) s = total;
  if (start) *start = s;
  if (length) *length = (total - s < piece) ? (total - s) : piece;
  return SHARD_OK;
}

int shard_peak_memory(double W, double V, double P, int N, double* replicated, double* sharded) {
  if (N < 1 || !(W >= 0.0) || !(V >= 0.0) || !(P >= 0.0)) return SHARD_EINVAL;
  if (replicated) *replicated = W + V + P;
  if (sharded) {
    const double in_loop = W + V / (double)N + P, out_of_loop = W + V;
    *sharded = in_loop > out_of_loop ? in_loop : out_of_loop;
  }
  return SHARD_OK;
}

int shard_plan_peak_bytes(const shard_plan_t* plan, int weight_bytes, int aux_bytes, int64_t P, int64_t* replicated,
                          int64_t* sharded) {
  if (plan == nullptr || weight_bytes < 1 || aux_bytes < 0 || P < 0) return SHARD_EINVAL;
  const int64_t kMax = std::numeric_limits<int64_t>::max();
  const int64_t per_elem = (int64_t)weight_bytes + aux_bytes;
  // plan_build keeps total and N*S below 2^63 / 16; refuse element sizes that could still overflow
  if (per_elem > 16 || P > kMax / 4) return SHARD_EINVAL;
  const int64_t W = plan->total * weight_bytes, V = plan->total * aux_bytes;
  if (replicated) *replicated = W + V + P;
  if (sharded) {
    const int64_t in_loop = W + plan->S * aux_bytes + P, out_of_loop = W + V;
    *sharded = in_loop > out_of_loop ? in_loop : out_of_loop;
  }
  return SHARD_OK;
}

}  // extern "C"
