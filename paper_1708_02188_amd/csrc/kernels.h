// Launch interface between the C ABI (api.cpp) and the gfx950 kernels (kernels.hip).
#pragma once

#include <hip/hip_runtime_api.h>

#include "plan.h"

namespace ddl {

// Learner base pointers travel in the kernel-argument segment when they fit, so a call
// needs no host-to-device copy of its own.
constexpr int kKernargLearners = 256;
struct PtrTable {
    void* p[kKernargLearners];
};

// Enqueue the kernel that fills d_rops (one ResolvedOp per entry of the plan's operation
// table d_ops) for the learner pointers in `table` (P <= kKernargLearners) or, if d_ptrs is
// not NULL, in that device array.
hipError_t launch_resolve(const ddl_plan& plan, const Op* d_ops, ResolvedOp* d_rops,
                          const PtrTable& table, void* const* d_ptrs, hipStream_t stream);

// Enqueue the kernel of one step.  d_rops points at that step's resolved operations in
// device memory; d_descs at the plan's work list (several-tensor plans, else unused).
// A step that moves nothing enqueues nothing.
hipError_t launch_step(const ddl_plan& plan, const Step& step, const ResolvedOp* d_rops,
                       const BlockDesc* d_descs, hipStream_t stream);

// Plain copy of n elements with the all-gather phase's streaming shape.
hipError_t launch_assign(ddl_dtype_t dtype, void* dst, const void* src, uint64_t n, hipStream_t stream);

// Step-fused allreduce.  launch_fused_resolve binds the summation-order table to the
// caller's buffers: d_ptrs_out[c * padded + i] = address of finest chunk c in learner
// seq[c][i].  launch_fused runs the single pass over all chunks.
hipError_t launch_fused_resolve(const ddl_plan& plan, const DeviceTables& t, int padded,
                                const uint64_t* d_own_off, const PtrTable& table,
                                void* const* d_ptrs, hipStream_t stream);
// mode: 0 = fold and store to all learners, 1 = fold and store to the chunk's owner,
// 2 = copy the owner's chunk to all other learners.
hipError_t launch_fused(const ddl_plan& plan, const DeviceTables& t, int padded, int levels,
                        uint64_t max_chunk, int mode, hipStream_t stream);

}  // namespace ddl
