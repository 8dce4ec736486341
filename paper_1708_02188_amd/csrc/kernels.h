// Launch interface between the C ABI (api.cpp) and the gfx950 kernels (kernels.hip).
#pragma once

#include <hip/hip_runtime_api.h>

#include "plan.h"

namespace ddl {

// Learner base pointers travel in the kernel-argument segment when they fit, so a call
// needs no host-to-device copy and a plan can serve several streams at once.
constexpr int kKernargLearners = 256;
struct PtrTable {
    void* p[kKernargLearners];
};

// Enqueue the kernel of one step.  d_ops points at that step's P operations in device
// memory.  Learner pointers come from `table` (P <= kKernargLearners) or, if d_ptrs is not
// NULL, from that device array.  A step that moves nothing enqueues nothing.
hipError_t launch_step(const ddl_plan& plan, const Step& step, const Op* d_ops,
                       const PtrTable& table, void* const* d_ptrs, hipStream_t stream);

}  // namespace ddl
