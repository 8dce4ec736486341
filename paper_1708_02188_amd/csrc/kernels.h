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

// The box as kernel arguments, for the resolver that needs no uploaded operation table.
struct BoxArgs {
    int32_t m;
    int32_t dims[DDL_MAX_DIMS];
    uint32_t P;
    uint32_t elem_size;
    uint32_t steps;
    uint64_t count;
};

#if defined(__HIPCC__)
#define DDL_HOST_DEVICE __host__ __device__
#else
#define DDL_HOST_DEVICE
#endif

// Part k of d of [lo, hi), cut on granules of G elements (the planner's chunking rule).
DDL_HOST_DEVICE inline void box_split(uint64_t lo, uint64_t hi, uint64_t d, uint64_t k, uint64_t G,
                                      uint64_t* a, uint64_t* b) {
    const uint64_t n = hi - lo;
    const uint64_t granules = (n + G - 1) / G;
    const uint64_t first = (k * granules / d) * G;
    const uint64_t last = ((k + 1) * granules / d) * G;
    *a = lo + (first < n ? first : n);
    *b = lo + (last < n ? last : n);
}

// Transfer i = phase * P + sender of the whole schedule, derived from the box alone
// (Sec. 4.3: reduce-scatter rings of dimension 1..m, then all-gather rings of dimension
// m..1, d-1 phases each): elements [*off, *off + *n) go from learner *src to learner *dst.
// Requires i < box.steps * box.P with box.steps = 2 * sum (d_t - 1).
DDL_HOST_DEVICE inline void box_op(const BoxArgs& box, unsigned i, uint64_t* off, uint64_t* n, int* src,
                                   int* dst) {
    int s = int(i / box.P);
    const int r = int(i % box.P);
    int half = 0;
    for (int t = 0; t < box.m; ++t) half += box.dims[t] - 1;
    const bool reduce = s < half;
    if (!reduce) s -= half;
    // which dimension's rings run in this phase, and which of their d-1 phases it is
    int t = reduce ? 0 : box.m - 1;
    while (s >= box.dims[t] - 1) {
        s -= box.dims[t] - 1;
        t += reduce ? 1 : -1;
    }
    const uint64_t G = 16u / box.elem_size;
    uint64_t lo = 0, hi = box.count;
    int stride = 1;
    for (int u = 0; u < t; ++u) {
        box_split(lo, hi, uint64_t(box.dims[u]), uint64_t((r / stride) % box.dims[u]), G, &lo, &hi);
        stride *= box.dims[u];
    }
    const int d = box.dims[t];
    const int pos = (r / stride) % d;
    const int back = reduce ? s + 1 : s;  // reduce passes on part c-s-1, gather part c-s
    const int part = ((pos - back) % d + d) % d;
    uint64_t a, b;
    box_split(lo, hi, uint64_t(d), uint64_t(part), G, &a, &b);
    *off = a;
    *n = b - a;
    *src = r;
    *dst = r + ((pos + 1) % d - pos) * stride;
}

// Operation records the allocation-free entry point keeps in a static device array.
constexpr size_t kStaticOps = DDL_NOALLOC_MAX_OPS;
constexpr size_t kStaticScratchBytes = kStaticOps * sizeof(ResolvedOp);

// Device address of that array on the current device (looked up once per device).
hipError_t static_scratch(ResolvedOp** out);

// Enqueue the kernel that writes every phase's records for the learner pointers in `table`
// into d_rops, computing the transfers from the plan's box on the device.
hipError_t launch_resolve_from_box(const ddl_plan& plan, const PtrTable& table, ResolvedOp* d_rops,
                                   hipStream_t stream);

// Enqueue the kernel that fills d_rops (one ResolvedOp per entry of the plan's operation
// table d_ops) for the learner pointers in `table` (P <= kKernargLearners) or, if d_ptrs is
// not NULL, in that device array.
hipError_t launch_resolve(const ddl_plan& plan, const Op* d_ops, ResolvedOp* d_rops,
                          const PtrTable& table, void* const* d_ptrs, hipStream_t stream);

// Enqueue the kernel of one step (`step` must be an element of plan.steps).  d_rops points at
// the plan's whole table of resolved operations in device memory; d_items / d_ragged at the
// bound whole items and the ragged work list (several-tensor plans, else unused).
// A step that moves nothing enqueues nothing.
hipError_t launch_step(const ddl_plan& plan, const Step& step, const ResolvedOp* d_rops, const ItemRec* d_items,
                       const BlockDesc* d_ragged, hipStream_t stream);

// Several-tensor plans: bind the whole work items (d_whole, plan.whole.size() of them) to
// the buffers d_rops was resolved for.  Enqueue after launch_resolve on the same stream.
hipError_t launch_resolve_items(const ddl_plan& plan, const ResolvedOp* d_rops, const BlockDesc* d_whole,
                                ItemRec* d_items, hipStream_t stream);

// Plain copy of n elements with the all-gather phase's streaming shape.
hipError_t launch_assign(ddl_dtype_t dtype, void* dst, const void* src, uint64_t n, hipStream_t stream);

// Ring walk (all d-1 phases of a box dimension in one launch).  launch_resolve_walk binds the
// plan's walk rows (d_walk_plan, learner indices) to the caller's buffers in d_rows;
// launch_walk runs one dimension over bound rows: mode 0 = its all-gather, 1 = its
// reduce-scatter, 2 = both at once (the sum stored to all d positions: the last dimension of a
// whole allreduce, whose gather overwrites its own partial sums).  d_items: the plan's tiles
// (several-tensor plans, else unused).
hipError_t launch_resolve_walk(const ddl_plan& plan, const uint64_t* d_walk_plan, uint64_t* d_rows,
                               const PtrTable& table, void* const* d_ptrs, hipStream_t stream);
hipError_t launch_walk(const ddl_plan& plan, const WalkLevel& level, const uint64_t* d_rows,
                       const BlockDesc* d_items, int mode, hipStream_t stream);

// Copy the P learner pointers of the host array `bufs` into the device array d_ptrs, through
// kernel arguments (kKernargLearners per launch); `bufs` is not referenced after return.
hipError_t launch_store_pointers(void* const* bufs, int P, void** d_ptrs, hipStream_t stream);

// Step-fused allreduce.  launch_fused_resolve binds the summation-order table to the
// caller's buffers: fused_ptrs[c * padded + i] = address of finest chunk c in learner
// seq[c][i].  launch_fused runs one pass over all chunks.
hipError_t launch_fused_resolve(const ddl_plan& plan, const DeviceTables& t, uint64_t* fused_ptrs,
                                const PtrTable& table, void* const* d_ptrs, hipStream_t stream);
// mode: 0 = fold and store to all learners, 1 = fold and store to the chunk's owner,
// 2 = copy the owner's chunk to all other learners.
hipError_t launch_fused(const ddl_plan& plan, const DeviceTables& t, const uint64_t* fused_ptrs,
                        uint64_t max_chunk, int mode, hipStream_t stream);

}  // namespace ddl
