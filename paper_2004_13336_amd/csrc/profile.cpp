// Per-kernel timing with HIP event pairs on the launch stream (shard_profile_*).
#include "internal.hpp"

namespace su {

bool stream_is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &status) != hipSuccess) {
    (void)hipGetLastError();      // e.g. the legacy default stream while another stream captures: nothing is recorded here
    return false;
  }
  return status != hipStreamCaptureStatusNone;
}

// Launches that are being recorded into a graph are not timed: an event pair inside a graph would be recorded
// as nodes and never hold a time that shard_profile_read could fetch.
ProfScope::ProfScope(shard_plan_t* plan, int kernel, hipStream_t s) : p(plan), stream(s), on(plan->prof) {
  if (!on) return;
  if (stream_is_capturing(s)) {
    on = false;
    return;
  }
  if (!p->prof_free.empty()) {
    rec = p->prof_free.back();
    p->prof_free.pop_back();
  } else if (hipEventCreate(&rec.start) != hipSuccess || hipEventCreate(&rec.stop) != hipSuccess) {
    on = false;
    return;
  }
  rec.kernel = kernel;
  (void)hipEventRecord(rec.start, stream);
}

ProfScope::~ProfScope() {
  if (!on) return;
  (void)hipEventRecord(rec.stop, stream);
  p->prof_live.push_back(rec);
}

}  // namespace su
