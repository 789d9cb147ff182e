// Optional per-kernel timing: when enabled on a handle, every kernel launch is bracketed by two HIP events
// on the caller's stream; dw_profile_read turns them into launch counts and total milliseconds per class.
#include "dw_internal.h"

namespace dw {

thread_local Profiler* tl_profiler = nullptr;

KernelScope::KernelScope(int kclass, hipStream_t stream) : p(tl_profiler), slot(-1), s(stream) {
  if (!p) return;
  if (p->used >= Profiler::kMaxLaunches) { p->dropped += 1; return; }
  if (p->used >= p->created) {
    if (hipEventCreate(&p->start[p->created]) != hipSuccess) { p->dropped += 1; return; }
    if (hipEventCreate(&p->stop[p->created]) != hipSuccess) {
      (void)hipEventDestroy(p->start[p->created]);
      p->dropped += 1;
      return;
    }
    p->created += 1;
  }
  slot = p->used++;
  p->cls[slot] = kclass;
  (void)hipEventRecord(p->start[slot], s);
}

KernelScope::~KernelScope() {
  if (p && slot >= 0) (void)hipEventRecord(p->stop[slot], s);
}

}  // namespace dw
