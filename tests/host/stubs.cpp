// Stand-ins for the kernel launchers of kernels.hip, for the sanitized host-only build: a host-only context
// never launches a kernel, so every one of them aborts if it is reached.
#include <stdio.h>
#include <stdlib.h>

#include "kernels.h"

namespace recover {
[[noreturn]] static void reached(const char *what) {
  fprintf(stderr, "host-only context reached the kernel launcher %s\n", what);
  abort();
}
Tuning &tuning() {
  static Tuning t;
  return t;
}
hipError_t launch_compare(const float *, const float *, size_t, CompareResult *, hipStream_t) { reached("compare"); }
hipError_t launch_accumulate_many(const AccumulateManyArgs &, int, bool, size_t, size_t, hipStream_t) { reached("accumulate_many"); }
hipError_t launch_accumulate(float *, float *, const void *, bool, bool, size_t, size_t, hipStream_t) { reached("accumulate"); }
hipError_t launch_copy(float *, const float *, size_t, size_t, bool, hipStream_t) { reached("copy"); }
hipError_t launch_copy_many(const CopyManyArgs &, int, size_t, size_t, bool, hipStream_t) { reached("copy_many"); }
hipError_t launch_reduce(const ReduceArgs &, size_t, size_t, hipStream_t) { reached("reduce"); }
hipError_t static_step_state(int, StepState **) { reached("static_step_state"); }
hipError_t launch_clear_step_state(StepState *, hipStream_t) { reached("clear_step_state"); }
hipError_t launch_adam_prologue(StepState *, float, float, float, float, float, hipStream_t) { reached("adam_prologue"); }
hipError_t launch_adamw(float *, float *, float *, const float *, uint16_t *, size_t, size_t, const AdamArgs &, const AdamArgs *,
                        hipStream_t) { reached("adamw"); }
hipError_t launch_reduce_adamw(const ReduceArgs &, float *, float *, float *, uint16_t *, bool, size_t, size_t, const AdamArgs &,
                               const AdamArgs *, hipStream_t) { reached("reduce_adamw"); }
}  // namespace recover
