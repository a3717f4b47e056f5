// The chunk table as the table-driven kernels see it: one ChunkDesc per work item, resolved against its
// variable and the replica id.  Shared by the formatting kernels and the update kernels.
#pragma once

#include "device_common.hpp"

namespace su {
namespace {

struct ChunkView {
  int var;
  int len;          // slots in this chunk
  int valid;        // leading slots that hold real elements on replica r (Section 4.1: position
                    // in the full variable = replica offset + index, compared with its length)
  int64_t shard0;   // offset of the chunk inside a packed shard
  int64_t flat0;    // offset of the chunk inside the flat variable
  uint32_t flags;
};

__device__ __forceinline__ ChunkView chunk_view(const VarDesc* __restrict__ vars, const ChunkDesc* __restrict__ chunks,
                                                int c, int r) {
  const ChunkDesc cd = chunks[c];
  const VarDesc vd = vars[cd.var];
  ChunkView cv;
  cv.var = cd.var;
  cv.len = cd.len;
  cv.flat0 = (int64_t)r * vd.stride + cd.k0;
  int64_t rem = vd.n - cv.flat0;                            // up to the end of the variable ...
  if (vd.stride - cd.k0 < rem) rem = vd.stride - cd.k0;     // ... and of the piece's real slots
  cv.valid = rem <= 0 ? 0 : (rem < (int64_t)cd.len ? (int)rem : cd.len);
  cv.shard0 = vd.off + cd.k0;
  cv.flags = vd.flags;
  return cv;
}

}  // namespace
}  // namespace su
