// Per-kernel timing with HIP event pairs on the launch stream (shard_profile_*).
#include "internal.hpp"

namespace su {

ProfScope::ProfScope(shard_plan_t* plan, int kernel, hipStream_t s) : p(plan), stream(s), on(plan->prof) {
  if (!on) return;
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
