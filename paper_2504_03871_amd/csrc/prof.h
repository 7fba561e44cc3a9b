// Benchmark aid: optional HIP-event brackets around individual kernel launches (see moe_profile_kernel).
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/moe.h"

namespace moe {

struct ProfSlot {
  void** start = nullptr;
  void** stop = nullptr;
  int n = 0;
  long long count = 0;
};
ProfSlot& prof_slot(int which);   // per host thread

// Records the armed events of kernel `which` on `s` at construction and destruction.
struct ProfScope {
  ProfSlot& slot;
  hipStream_t s;
  int i = -1;
  ProfScope(int which, hipStream_t stream) : slot(prof_slot(which)), s(stream) {
    if (slot.n > 0) {
      i = (int)(slot.count++ % slot.n);
      (void)hipEventRecord((hipEvent_t)slot.start[i], s);
    }
  }
  ~ProfScope() {
    if (i >= 0) (void)hipEventRecord((hipEvent_t)slot.stop[i], s);
  }
};

}  // namespace moe
