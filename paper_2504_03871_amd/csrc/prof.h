// Benchmark aid: optional HIP-event brackets around individual kernel launches, driven by the caller-owned
// moe_prof that a moe_cfg may point at (moe.h).  The library itself holds no profiling state.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/moe.h"

namespace moe {

// Records the armed events of kernel `which` on `s` at construction and destruction.
struct ProfScope {
  moe_prof* p;
  hipStream_t s;
  int which;
  int i = -1;
  ProfScope(const moe_cfg* c, int which_, hipStream_t stream) : p(c->prof), s(stream), which(which_) {
    if (p != nullptr && p->n[which] > 0) {
      i = (int)(p->count[which]++ % p->n[which]);
      (void)hipEventRecord((hipEvent_t)p->start[which][i], s);
    }
  }
  ~ProfScope() {
    if (i >= 0) (void)hipEventRecord((hipEvent_t)p->stop[which][i], s);
  }
};

}  // namespace moe
