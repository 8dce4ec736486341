// C ABI of libddlsim (declared in include/ddlsim.h): argument checks, device tables,
// and the per-step launches.  No element arithmetic happens on the host.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "kernels.h"
#include "plan.h"

// Learners from which the step-fused allreduce runs as two passes (see run_fused).
#ifndef DDL_FUSED_TWO_PASS_FROM
#define DDL_FUSED_TWO_PASS_FROM 16
#endif

namespace {

using ddl::DeviceTables;
using ddl::Op;
using ddl::PtrTable;

void set_status(ddl_status_t* status, ddl_status_t value) {
    if (status) *status = value;
}

template <typename T>
void release(T** d) {
    if (*d) (void)hipFree(*d);
    *d = nullptr;
}

void release_binding(ddl::Binding* b) {
    release(&b->rops);
    release(&b->items);
    release(&b->d_ptrs);
    release(&b->fused_ptrs);
    release(&b->walk);
    delete b;
}

void release_tables(DeviceTables* t) {
    for (ddl::Binding* b : t->bindings) release_binding(b);
    t->bindings.clear();
    release(&t->ops);
    release(&t->walk_plan);
    release(&t->walk_items);
    release(&t->whole);
    release(&t->ragged);
    release(&t->fused_seq);
    release(&t->fused_ctl);
    release(&t->fused_n);
    release(&t->fused_off);
}

template <typename T>
bool reserve(T** d, size_t count) {
    return hipMalloc(reinterpret_cast<void**>(d), count * sizeof(T)) == hipSuccess;
}

template <typename T>
bool upload(T** d, const std::vector<T>& h) {
    return reserve(d, h.size()) &&
           hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) == hipSuccess;
}

// The plan's tables on the current device, created on first use.  Caller holds plan->mu.
ddl_status_t device_tables_locked(const ddl_plan* plan, DeviceTables** out) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return DDL_ERR_HIP;
    for (DeviceTables* t : plan->tables)
        if (t->device == device) {
            *out = t;
            return DDL_OK;
        }
    DeviceTables* t = new (std::nothrow) DeviceTables;
    if (t == nullptr) return DDL_ERR_NOMEM;
    t->device = device;
    bool ok = true;
    if (!plan->ops.empty()) ok = upload(&t->ops, plan->ops);
    if (ok && !plan->walk_plan.empty()) ok = upload(&t->walk_plan, plan->walk_plan);
    if (ok && !plan->walk_items.empty()) ok = upload(&t->walk_items, plan->walk_items);
    if (ok && !plan->whole.empty()) ok = upload(&t->whole, plan->whole);
    if (ok && !plan->ragged.empty()) ok = upload(&t->ragged, plan->ragged);
    if (!ok) {
        release_tables(t);
        delete t;
        return DDL_ERR_NOMEM;
    }
    plan->tables.push_back(t);
    *out = t;
    return DDL_OK;
}

// Adds the tables of the step-fused path.  Caller holds plan->mu.
ddl_status_t fused_tables_locked(const ddl_plan* plan, DeviceTables* t) {
    if (t->fused_seq != nullptr) return DDL_OK;
    std::vector<uint32_t> seq, ctl;
    int padded = 0;
    t->fused_levels = ddl::build_fused_order(*plan, &seq, &ctl, &padded);
    t->fused_padded = padded;
    const bool ok = upload(&t->fused_seq, seq) && upload(&t->fused_ctl, ctl) &&
                    upload(&t->fused_n, plan->own_n) && upload(&t->fused_off, plan->own_off);
    if (!ok) {
        release(&t->fused_seq);
        release(&t->fused_ctl);
        release(&t->fused_n);
        release(&t->fused_off);
        return DDL_ERR_NOMEM;
    }
    return DDL_OK;
}

bool stream_is_capturing(hipStream_t stream) {
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &status) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return status != hipStreamCaptureStatusNone;
}

// Device memory of one binding slot (nothing bound yet).  Caller holds plan->mu.
ddl::Binding* new_binding(const ddl_plan* plan, const DeviceTables* t, bool fused) {
    ddl::Binding* b = new (std::nothrow) ddl::Binding;
    if (b == nullptr) return nullptr;
    bool ok = plan->ops.empty() || reserve(&b->rops, plan->ops.size());
    if (ok && !plan->whole.empty()) ok = reserve(&b->items, plan->whole.size());
    if (ok && plan->walk_words) ok = reserve(&b->walk, plan->walk_words);
    if (ok && plan->P > ddl::kKernargLearners) ok = reserve(&b->d_ptrs, size_t(plan->P));
    if (ok && fused) ok = reserve(&b->fused_ptrs, size_t(plan->P) * size_t(t->fused_padded));
    if (!ok) {
        release_binding(b);
        return nullptr;
    }
    return b;
}

// The slot that holds this call's binding.  An eager call whose buffers are those of an
// existing slot finds its tables bound; otherwise a slot is bound to `bufs` here: a free
// one, a new one (never while the stream is being captured: nothing may allocate then),
// or the least recently used.  The kernels that fill the slot's tables are enqueued on
// `stream` before this returns.  A call under capture always records them into the graph
// (a replay must not depend on what later eager calls did to the slot) and pins the slot.
ddl_status_t acquire_binding(void** bufs, int P, const ddl_plan* plan, hipStream_t stream, bool fused,
                             DeviceTables** tables_out, ddl::Binding** out, bool* was_bound) {
    std::lock_guard<std::mutex> lock(plan->mu);
    const bool capturing = stream_is_capturing(stream);
    DeviceTables* t = nullptr;
    if (capturing) {
        // nothing may allocate or copy now: the tables must exist (ddl_plan_prepare)
        int device = -1;
        if (hipGetDevice(&device) != hipSuccess) return DDL_ERR_HIP;
        for (DeviceTables* have : plan->tables)
            if (have->device == device) t = have;
        if (t == nullptr) return DDL_ERR_UNSUPPORTED;
    }
    ddl_status_t st = t ? DDL_OK : device_tables_locked(plan, &t);
    if (st != DDL_OK) return st;
    if (fused && t->fused_seq == nullptr) {
        if (capturing) return DDL_ERR_UNSUPPORTED;  // ddl_plan_prepare was not called
        st = fused_tables_locked(plan, t);
        if (st != DDL_OK) return st;
    }
    ddl::Binding* slot = nullptr;
    for (ddl::Binding* b : t->bindings)
        if (b->key.size() == size_t(P) && std::memcmp(b->key.data(), bufs, size_t(P) * sizeof(void*)) == 0) {
            slot = b;
            break;
        }
    if (slot == nullptr) {
        for (ddl::Binding* b : t->bindings)
            if (b->key.empty()) {
                slot = b;
                break;
            }
        if (slot == nullptr && !capturing && t->bindings.size() < size_t(DDL_PLAN_MAX_BINDINGS)) {
            slot = new_binding(plan, t, fused);
            if (slot == nullptr) return DDL_ERR_NOMEM;
            t->bindings.push_back(slot);
        }
        if (slot == nullptr) {
            for (ddl::Binding* b : t->bindings)
                if (!b->pinned && (slot == nullptr || b->last_use < slot->last_use)) slot = b;
            if (slot == nullptr) return capturing ? DDL_ERR_UNSUPPORTED : DDL_ERR_NOMEM;
        }
        slot->key.assign(bufs, bufs + P);
        slot->rops_valid = slot->fused_valid = false;
    }
    if (fused && slot->fused_ptrs == nullptr) {
        if (capturing) return DDL_ERR_UNSUPPORTED;
        if (!reserve(&slot->fused_ptrs, size_t(P) * size_t(t->fused_padded))) return DDL_ERR_NOMEM;
    }
    slot->last_use = ++t->clock;
    const bool valid = fused ? slot->fused_valid : slot->rops_valid;
    *was_bound = valid && !capturing;
    if (!*was_bound) {
        PtrTable table;
        std::memset(&table, 0, sizeof(table));
        void* const* d_ptrs = nullptr;
        if (P <= ddl::kKernargLearners) {
            std::memcpy(table.p, bufs, size_t(P) * sizeof(void*));
        } else {
            if (ddl::launch_store_pointers(bufs, P, slot->d_ptrs, stream) != hipSuccess) return DDL_ERR_HIP;
            d_ptrs = slot->d_ptrs;
        }
        hipError_t err = fused ? ddl::launch_fused_resolve(*plan, *t, slot->fused_ptrs, table, d_ptrs, stream)
                               : ddl::launch_resolve(*plan, t->ops, slot->rops, table, d_ptrs, stream);
        if (err == hipSuccess && !fused)
            err = ddl::launch_resolve_items(*plan, slot->rops, t->whole, slot->items, stream);
        if (err == hipSuccess && !fused && slot->walk)
            err = ddl::launch_resolve_walk(*plan, t->walk_plan, slot->walk, table, d_ptrs, stream);
        if (err != hipSuccess) return DDL_ERR_HIP;
        if (capturing) slot->pinned = true;
        else if (fused) slot->fused_valid = true;
        else slot->rops_valid = true;
    }
    *tables_out = t;
    *out = slot;
    return DDL_OK;
}

ddl_status_t check_call(void** bufs, int P, const ddl_plan* plan, size_t count, ddl_dtype_t dtype) {
    if (plan == nullptr || bufs == nullptr || P < 1) return DDL_ERR_ARG;
    if (ddl::dtype_size(dtype) == 0) return DDL_ERR_DTYPE;
    if (P != plan->P || count != plan->count || dtype != plan->dtype) return DDL_ERR_PLAN_MISMATCH;
    if (count == 0) return DDL_OK;  // nothing will be touched: empty buffers may be NULL
    for (int j = 0; j < P; ++j) {
        if (bufs[j] == nullptr) return DDL_ERR_ARG;
        if (reinterpret_cast<uintptr_t>(bufs[j]) % 16 != 0) return DDL_ERR_ALIGN;
    }
    // learners must not share memory: sorted by address, each buffer must end before the next
    // (on the stack while the learners fit the kernel-argument table: no heap use then)
    uintptr_t few[ddl::kKernargLearners];
    std::vector<uintptr_t> many;
    uintptr_t* sorted = few;
    if (P > ddl::kKernargLearners) {
        many.resize(P);
        sorted = many.data();
    }
    for (int j = 0; j < P; ++j) sorted[j] = reinterpret_cast<uintptr_t>(bufs[j]);
    std::sort(sorted, sorted + P);
    const uintptr_t bytes = uintptr_t(count) * uintptr_t(plan->elem_size);
    for (int j = 0; j + 1 < P; ++j) {
        if (sorted[j] == sorted[j + 1]) return DDL_ERR_ARG;
        if (sorted[j] + bytes > sorted[j + 1]) return DDL_ERR_ARG;
    }
    return DDL_OK;
}

// Enqueue the kernels of steps [first, last) for the slot's buffers.
ddl_status_t launch_steps(const ddl_plan* plan, const DeviceTables* t, const ddl::Binding* slot, int first,
                          int last, hipStream_t stream, hipEvent_t* events) {
    for (int s = first; s < last; ++s) {
        if (ddl::launch_step(*plan, plan->steps[s], slot->rops, slot->items, t->ragged, stream) != hipSuccess)
            return DDL_ERR_HIP;
        if (events && hipEventRecord(events[s - first + 1], stream) != hipSuccess) return DDL_ERR_HIP;
    }
    return DDL_OK;
}

// Phases shorter than this on average are launch-bound (a phase boundary costs the GPU
// about as long as moving this many bytes): such plans walk their rings by default.
constexpr uint64_t kWalkPhaseBytes = uint64_t(16) << 20;

bool wants_walk(const ddl_plan* plan) {
    if (plan->walk_levels.empty() || plan->walk_mode == DDL_WALK_OFF) return false;
    if (plan->walk_mode == DDL_WALK_ON) return true;
    return plan->bytes_total / plan->steps.size() < kWalkPhaseBytes;
}

// The reduce-scatter and / or the all-gather as ring walks: one launch per box dimension.
ddl_status_t launch_walks(const ddl_plan* plan, const DeviceTables* t, const ddl::Binding* slot, bool reduce,
                          bool gather, hipStream_t stream) {
    const int levels = static_cast<int>(plan->walk_levels.size());
    // a whole allreduce takes the last dimension's reduce-scatter and all-gather in one launch
    const int both = reduce && gather ? levels - 1 : -1;
    if (reduce)
        for (int l = 0; l < levels; ++l)
            if (ddl::launch_walk(*plan, plan->walk_levels[l], slot->walk, t->walk_items, l == both ? 2 : 1, stream) != hipSuccess)
                return DDL_ERR_HIP;
    if (gather)
        for (int l = levels - 1; l >= 0; --l)
            if (l != both && ddl::launch_walk(*plan, plan->walk_levels[l], slot->walk, t->walk_items, 0, stream) != hipSuccess)
                return DDL_ERR_HIP;
    return DDL_OK;
}

// Run steps [first, last) of the plan.  events: NULL, or last-first+1 created events that
// are recorded round every launch.  Ranges that are the whole reduce-scatter, the whole
// all-gather or both may run as ring walks (see ddl_plan_set_walk); the buffers end up the same.
ddl_status_t run_steps(void** bufs, int P, const ddl_plan* plan, size_t count, ddl_dtype_t dtype,
                       void* stream_v, int first, int last, hipEvent_t* events) {
    ddl_status_t st = check_call(bufs, P, plan, count, dtype);
    if (st != DDL_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    if (count == 0 || plan->steps.empty()) return DDL_OK;

    DeviceTables* t = nullptr;
    ddl::Binding* slot = nullptr;
    bool was_bound = false;
    st = acquire_binding(bufs, P, plan, stream, false, &t, &slot, &was_bound);
    if (st != DDL_OK) return st;
    if (events && hipEventRecord(events[0], stream) != hipSuccess) return DDL_ERR_HIP;
    const int steps = static_cast<int>(plan->steps.size());
    const bool reduce = first == 0 && last >= plan->first_gather;
    const bool gather = last == steps && first <= plan->first_gather;
    const bool halves = (first == 0 || first == plan->first_gather) && (last == steps || last == plan->first_gather);
    bool walk;
    {
        std::lock_guard<std::mutex> lock(plan->mu);
        walk = events == nullptr && halves && first < last && slot->walk != nullptr && wants_walk(plan);
    }
    if (walk) return launch_walks(plan, t, slot, reduce, gather, stream);
    return launch_steps(plan, t, slot, first, last, stream, events);
}

ddl_plan_t* make_plan(const int* dims, int m, int P, const size_t* seg_off, const size_t* seg_count,
                      int S, size_t count, ddl_dtype_t dtype, ddl_status_t* status) {
    const int elem = ddl::dtype_size(dtype);
    if (elem == 0) {
        set_status(status, DDL_ERR_DTYPE);
        return nullptr;
    }
    ddl_status_t st = ddl::validate_dims(dims, m, P);
    if (st == DDL_OK && count > (uint64_t(1) << 56)) st = DDL_ERR_ARG;
    if (st == DDL_OK && (S < 1 || S > DDL_MAX_TENSORS || seg_off == nullptr || seg_count == nullptr))
        st = DDL_ERR_ARG;
    const uint64_t G = 16 / uint64_t(elem);
    uint64_t end = 0;  // tensors ascending, disjoint, inside the buffer, starts on 16-byte granules
    for (int s = 0; st == DDL_OK && s < S; ++s) {
        if (seg_off[s] % G != 0) st = DDL_ERR_ALIGN;
        else if (seg_off[s] < end || seg_count[s] > count || seg_off[s] > count - seg_count[s]) st = DDL_ERR_ARG;
        end = seg_off[s] + seg_count[s];
    }
    if (st == DDL_OK) {
        // the schedule is held as explicit tables: phases x tensors x learners operations
        uint64_t phases = 0;
        for (int t = 0; t < m; ++t) phases += 2 * uint64_t(dims[t] - 1);
        if (phases * uint64_t(S) > DDL_MAX_PLAN_OPS / uint64_t(P)) st = DDL_ERR_NOMEM;
        // several tensors: one work item per 16 KiB a learner sends, over both halves
        if (S > 1 && P > 1 &&
            count > DDL_MAX_LIST_ITEMS * uint64_t(8192) / (uint64_t(elem) * uint64_t(P - 1)))
            st = DDL_ERR_NOMEM;
    }
    if (st != DDL_OK) {
        set_status(status, st);
        return nullptr;
    }
    ddl_plan* plan = nullptr;
    try {
        plan = new ddl_plan;
        plan->dims.assign(dims, dims + m);
        plan->P = P;
        plan->count = count;
        plan->dtype = dtype;
        plan->elem_size = elem;
        plan->seg_off.assign(seg_off, seg_off + S);
        plan->seg_count.assign(seg_count, seg_count + S);
        ddl::build_schedule(plan);
        ddl::build_walk(plan);
    } catch (const std::bad_alloc&) {
        delete plan;
        set_status(status, DDL_ERR_NOMEM);
        return nullptr;
    }
    set_status(status, DDL_OK);
    return plan;
}

}  // namespace

extern "C" {

ddl_plan_t* ddl_ring_plan(const int* dims, int m, int P, size_t count, ddl_dtype_t dtype,
                          ddl_status_t* status) {
    const size_t off = 0;
    return make_plan(dims, m, P, &off, &count, 1, count, dtype, status);
}

ddl_plan_t* ddl_ring_plan_tensors(const int* dims, int m, int P, const size_t* tensor_off,
                                  const size_t* tensor_count, int num_tensors, size_t count,
                                  ddl_dtype_t dtype, ddl_status_t* status) {
    return make_plan(dims, m, P, tensor_off, tensor_count, num_tensors, count, dtype, status);
}

void ddl_plan_free(ddl_plan_t* plan) {
    if (plan == nullptr) return;
    for (DeviceTables* t : plan->tables) {
        release_tables(t);
        delete t;
    }
    delete plan;
}

namespace {

// Whether ddl_allreduce_fused_sim serves this plan.
bool fused_supported(const ddl_plan* plan) {
    int levels = 0;
    for (int d : plan->dims) levels += d > 1;
    return plan->P <= DDL_FUSED_MAX_LEARNERS && levels <= DDL_FUSED_MAX_LEVELS && plan->seg_off.size() == 1;
}

// Tables on the current device plus at least `slots` binding slots.
ddl_status_t prepare(const ddl_plan* plan, int slots) {
    if (plan == nullptr || slots < 0 || slots > DDL_PLAN_MAX_BINDINGS) return DDL_ERR_ARG;
    {
        std::lock_guard<std::mutex> lock(plan->mu);
        DeviceTables* t = nullptr;
        ddl_status_t st = device_tables_locked(plan, &t);
        if (st != DDL_OK) return st;
        const bool fused = plan->P > 1 && plan->count > 0 && fused_supported(plan);
        if (fused) {
            st = fused_tables_locked(plan, t);
            if (st != DDL_OK) return st;
        }
        for (ddl::Binding* b : t->bindings)
            if (fused && b->fused_ptrs == nullptr &&
                !reserve(&b->fused_ptrs, size_t(plan->P) * size_t(t->fused_padded)))
                return DDL_ERR_NOMEM;
        while (t->bindings.size() < size_t(slots)) {
            ddl::Binding* b = new_binding(plan, t, fused);
            if (b == nullptr) return DDL_ERR_NOMEM;
            t->bindings.push_back(b);
        }
    }
    // set-up of the allocation-free entry point: its static array's address on this device
    ddl::ResolvedOp* records = nullptr;
    return ddl::static_scratch(&records) == hipSuccess ? DDL_OK : DDL_ERR_HIP;
}

}  // namespace

ddl_status_t ddl_plan_prepare(const ddl_plan_t* plan) { return prepare(plan, 2); }

ddl_status_t ddl_plan_reserve_bindings(const ddl_plan_t* plan, int slots) { return prepare(plan, slots); }

ddl_status_t ddl_plan_set_walk(const ddl_plan_t* plan, int mode) {
    if (plan == nullptr || mode < DDL_WALK_AUTO || mode > DDL_WALK_ON) return DDL_ERR_ARG;
    if (mode == DDL_WALK_ON && plan->walk_levels.empty() && !plan->steps.empty()) return DDL_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(plan->mu);
    plan->walk_mode = mode;
    return DDL_OK;
}

ddl_status_t ddl_allreduce_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                               ddl_dtype_t dtype, void* stream) {
    const int steps = plan ? static_cast<int>(plan->steps.size()) : 0;
    return run_steps(bufs, P, plan, count, dtype, stream, 0, steps, nullptr);
}

ddl_status_t ddl_allreduce_sim_noalloc(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                       ddl_dtype_t dtype, void* stream_v) {
    // more learners than the kernel-argument table holds are refused before the argument
    // check, which would need heap memory to sort that many pointers
    if (plan != nullptr && bufs != nullptr && P > ddl::kKernargLearners) return DDL_ERR_UNSUPPORTED;
    ddl_status_t st = check_call(bufs, P, plan, count, dtype);
    if (st != DDL_OK) return st;
    const size_t steps = plan->steps.size();
    if (P > ddl::kKernargLearners || plan->seg_off.size() != 1 || steps * size_t(P) > DDL_NOALLOC_MAX_OPS)
        return DDL_ERR_UNSUPPORTED;
    if (count == 0 || steps == 0) return DDL_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    ddl::ResolvedOp* records = nullptr;
    if (ddl::static_scratch(&records) != hipSuccess) return DDL_ERR_HIP;
    PtrTable table;
    std::memset(&table, 0, sizeof(table));
    std::memcpy(table.p, bufs, size_t(P) * sizeof(void*));
    if (ddl::launch_resolve_from_box(*plan, table, records, stream) != hipSuccess) return DDL_ERR_HIP;
    for (size_t s = 0; s < steps; ++s)
        if (ddl::launch_step(*plan, plan->steps[s], records, nullptr, nullptr, stream) != hipSuccess)
            return DDL_ERR_HIP;
    return DDL_OK;
}

ddl_status_t ddl_reduce_scatter_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                    ddl_dtype_t dtype, void* stream) {
    const int split = plan ? plan->first_gather : 0;
    return run_steps(bufs, P, plan, count, dtype, stream, 0, split, nullptr);
}

ddl_status_t ddl_allgather_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                               ddl_dtype_t dtype, void* stream) {
    const int split = plan ? plan->first_gather : 0;
    const int steps = plan ? static_cast<int>(plan->steps.size()) : 0;
    return run_steps(bufs, P, plan, count, dtype, stream, split, steps, nullptr);
}

namespace {

// which: 0 = whole allreduce, 1 = reducing pass only, 2 = distributing pass only
ddl_status_t run_fused(void** bufs, int P, const ddl_plan* plan, size_t count, ddl_dtype_t dtype,
                       void* stream_v, int which) {
    ddl_status_t st = check_call(bufs, P, plan, count, dtype);
    if (st != DDL_OK) return st;
    if (!fused_supported(plan)) return DDL_ERR_UNSUPPORTED;
    if (count == 0 || P == 1) return DDL_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    DeviceTables* t = nullptr;
    ddl::Binding* slot = nullptr;
    bool was_bound = false;
    st = acquire_binding(bufs, P, plan, stream, true, &t, &slot, &was_bound);
    if (st != DDL_OK) return st;
    uint64_t max_chunk = 0;
    for (uint64_t n : plan->own_n) max_chunk = n > max_chunk ? n : max_chunk;
    auto pass = [&](int mode) {
        return ddl::launch_fused(*plan, *t, slot->fused_ptrs, max_chunk, mode, stream) == hipSuccess;
    };
    // Measured on MI355X: from 16 learners on, two passes (all reads of the reduction first,
    // then all writes of the distribution) sustain more bandwidth than one pass that mixes P
    // read and P write streams, at the price of writing and re-reading the result once (1/P
    // more traffic): 0.59 instead of 0.63 ms for 16 learners of 25.6 M elements.
    bool ok;
    if (which == 1) ok = pass(1);
    else if (which == 2) ok = pass(2);
    else if (P >= DDL_FUSED_TWO_PASS_FROM) ok = pass(1) && pass(2);
    else ok = pass(0);
    return ok ? DDL_OK : DDL_ERR_HIP;
}

}  // namespace

ddl_status_t ddl_assign_sim(void* dst, const void* src, size_t count, ddl_dtype_t dtype, void* stream) {
    const int elem = ddl::dtype_size(dtype);
    if (elem == 0) return DDL_ERR_DTYPE;
    if (count == 0) return DDL_OK;
    if (dst == nullptr || src == nullptr) return DDL_ERR_ARG;
    const uintptr_t d = reinterpret_cast<uintptr_t>(dst), s = reinterpret_cast<uintptr_t>(src);
    if (d % 16 != 0 || s % 16 != 0) return DDL_ERR_ALIGN;
    const uintptr_t bytes = uintptr_t(count) * uintptr_t(elem);
    if ((d <= s && s < d + bytes) || (s <= d && d < s + bytes)) return DDL_ERR_ARG;
    return ddl::launch_assign(dtype, dst, src, count, static_cast<hipStream_t>(stream)) == hipSuccess
               ? DDL_OK : DDL_ERR_HIP;
}

ddl_status_t ddl_allreduce_fused_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                     ddl_dtype_t dtype, void* stream) {
    return run_fused(bufs, P, plan, count, dtype, stream, 0);
}

ddl_status_t ddl_reduce_scatter_fused_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                          ddl_dtype_t dtype, void* stream) {
    return run_fused(bufs, P, plan, count, dtype, stream, 1);
}

ddl_status_t ddl_allgather_fused_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                     ddl_dtype_t dtype, void* stream) {
    return run_fused(bufs, P, plan, count, dtype, stream, 2);
}

ddl_status_t ddl_allreduce_sim_profile(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                       ddl_dtype_t dtype, void* stream, float* step_ms) {
    if (step_ms == nullptr) return DDL_ERR_ARG;
    ddl_status_t st = check_call(bufs, P, plan, count, dtype);
    if (st != DDL_OK) return st;
    const int steps = static_cast<int>(plan->steps.size());
    for (int s = 0; s < steps; ++s) step_ms[s] = 0.0f;
    if (steps == 0 || count == 0) return DDL_OK;
    std::vector<hipEvent_t> events(steps + 1, nullptr);
    st = DDL_OK;
    for (int i = 0; i <= steps && st == DDL_OK; ++i)
        if (hipEventCreate(&events[i]) != hipSuccess) st = DDL_ERR_HIP;
    if (st == DDL_OK) st = run_steps(bufs, P, plan, count, dtype, stream, 0, steps, events.data());
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess && st == DDL_OK)
        st = DDL_ERR_HIP;
    if (st == DDL_OK)
        for (int s = 0; s < steps; ++s)
            if (plan->steps[s].max_n != 0 &&
                hipEventElapsedTime(&step_ms[s], events[s], events[s + 1]) != hipSuccess)
                st = DDL_ERR_HIP;
    for (hipEvent_t e : events)
        if (e) (void)hipEventDestroy(e);
    return st;
}

ddl_status_t ddl_allreduce_sim_timed(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                     ddl_dtype_t dtype, void* stream, float* reduce_ms,
                                     float* gather_ms) {
    ddl_status_t st = check_call(bufs, P, plan, count, dtype);
    if (st != DDL_OK) return st;
    if (reduce_ms) *reduce_ms = 0.0f;
    if (gather_ms) *gather_ms = 0.0f;
    const int steps = static_cast<int>(plan->steps.size());
    if (steps == 0 || count == 0) return DDL_OK;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    for (int i = 0; i < 3 && st == DDL_OK; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) st = DDL_ERR_HIP;
    // bind first (untimed: an empty range of steps), then the two halves between events
    if (st == DDL_OK) st = run_steps(bufs, P, plan, count, dtype, stream, 0, 0, nullptr);
    if (st == DDL_OK && hipEventRecord(ev[0], hs) != hipSuccess) st = DDL_ERR_HIP;
    if (st == DDL_OK) st = run_steps(bufs, P, plan, count, dtype, stream, 0, plan->first_gather, nullptr);
    if (st == DDL_OK && hipEventRecord(ev[1], hs) != hipSuccess) st = DDL_ERR_HIP;
    if (st == DDL_OK) st = run_steps(bufs, P, plan, count, dtype, stream, plan->first_gather, steps, nullptr);
    if (st == DDL_OK && hipEventRecord(ev[2], hs) != hipSuccess) st = DDL_ERR_HIP;
    if (hipStreamSynchronize(hs) != hipSuccess && st == DDL_OK) st = DDL_ERR_HIP;
    float ms = 0.0f;
    if (st == DDL_OK && reduce_ms) {
        if (hipEventElapsedTime(&ms, ev[0], ev[1]) == hipSuccess) *reduce_ms = ms; else st = DDL_ERR_HIP;
    }
    if (st == DDL_OK && gather_ms) {
        if (hipEventElapsedTime(&ms, ev[1], ev[2]) == hipSuccess) *gather_ms = ms; else st = DDL_ERR_HIP;
    }
    for (hipEvent_t e : ev)
        if (e) (void)hipEventDestroy(e);
    return st;
}

ddl_status_t ddl_plan_verify(const ddl_plan_t* plan) {
    return plan ? ddl::verify_plan(*plan) : DDL_ERR_ARG;
}

int ddl_plan_num_steps(const ddl_plan_t* plan) {
    return plan ? static_cast<int>(plan->steps.size()) : -1;
}

int ddl_plan_num_learners(const ddl_plan_t* plan) { return plan ? plan->P : 0; }

size_t ddl_plan_bytes_moved(const ddl_plan_t* plan) { return plan ? plan->bytes_total : 0; }

size_t ddl_plan_fused_bytes(const ddl_plan_t* plan) {
    if (plan == nullptr) return 0;
    // one pass: P reads + P writes per element; two passes: one more write and read
    const size_t per_elem = plan->P >= DDL_FUSED_TWO_PASS_FROM ? size_t(2) * plan->P + 2 : size_t(2) * plan->P;
    return per_elem * plan->elem_size * plan->count;
}

size_t ddl_plan_walk_bytes(const ddl_plan_t* plan) { return plan ? plan->walk_bytes : 0; }

size_t ddl_plan_step_bytes(const ddl_plan_t* plan, int step) {
    if (plan == nullptr || step < 0 || step >= static_cast<int>(plan->steps.size())) return 0;
    return plan->steps[step].bytes;
}

ddl_status_t ddl_plan_get_step(const ddl_plan_t* plan, int step, int* kind, int* dim, int* src,
                               int* dst, size_t* off, size_t* n) {
    if (plan == nullptr || step < 0 || step >= static_cast<int>(plan->steps.size()))
        return DDL_ERR_ARG;
    const ddl::Step& st = plan->steps[step];
    if (kind) *kind = st.kind;
    if (dim) *dim = st.dim;
    const size_t per_step = size_t(plan->P) * plan->seg_off.size();
    const Op* ops = plan->ops.data() + size_t(step) * per_step;
    for (size_t i = 0; i < per_step; ++i) {
        if (src) src[i] = ops[i].src;
        if (dst) dst[i] = ops[i].dst;
        if (off) off[i] = ops[i].off;
        if (n) n[i] = ops[i].n;
    }
    return DDL_OK;
}

int ddl_plan_num_tensors(const ddl_plan_t* plan) {
    return plan ? static_cast<int>(plan->seg_off.size()) : 0;
}

ddl_status_t ddl_plan_owned_chunk_tensor(const ddl_plan_t* plan, int tensor, int learner, size_t* off,
                                         size_t* n) {
    if (plan == nullptr || learner < 0 || learner >= plan->P || tensor < 0 ||
        tensor >= static_cast<int>(plan->seg_off.size()))
        return DDL_ERR_ARG;
    if (off) *off = plan->own_off[size_t(tensor) * plan->P + learner];
    if (n) *n = plan->own_n[size_t(tensor) * plan->P + learner];
    return DDL_OK;
}

ddl_status_t ddl_plan_owned_chunk(const ddl_plan_t* plan, int learner, size_t* off, size_t* n) {
    return ddl_plan_owned_chunk_tensor(plan, 0, learner, off, n);
}

double ddl_plan_model_time(const ddl_plan_t* plan, const double* bw, const double* lat) {
    if (plan == nullptr || bw == nullptr || lat == nullptr) return -1.0;
    const int m = static_cast<int>(plan->dims.size());
    for (int t = 0; t < m; ++t)
        if (!(bw[t] > 0.0) || lat[t] < 0.0) return -1.0;
    return ddl::model_time(plan->dims.data(), m, double(plan->count) * plan->elem_size, bw, lat);
}

ddl_status_t ddl_choose_dims(int P, size_t bytes, int m, const double* bw, const double* lat,
                             const int* max_dim, int* dims_out, double* time_out) {
    return ddl::choose_dims(P, double(bytes), m, bw, lat, max_dim, dims_out, time_out);
}

ddl_status_t ddl_device_memory_info(int* clock_khz, int* bus_bits) {
    int device = -1, clock = 0, bus = 0;
    if (hipGetDevice(&device) != hipSuccess ||
        hipDeviceGetAttribute(&clock, hipDeviceAttributeMemoryClockRate, device) != hipSuccess ||
        hipDeviceGetAttribute(&bus, hipDeviceAttributeMemoryBusWidth, device) != hipSuccess)
        return DDL_ERR_HIP;
    if (clock_khz) *clock_khz = clock;
    if (bus_bits) *bus_bits = bus;
    return DDL_OK;
}

const char* ddl_status_string(ddl_status_t status) {
    switch (status) {
        case DDL_OK: return "ok";
        case DDL_ERR_ARG: return "invalid argument";
        case DDL_ERR_DIMS: return "box dimensions do not describe the learners";
        case DDL_ERR_DTYPE: return "unknown element type";
        case DDL_ERR_ALIGN: return "learner buffer is not 16-byte aligned";
        case DDL_ERR_PLAN_MISMATCH: return "arguments differ from the plan's";
        case DDL_ERR_NOMEM: return "out of memory";
        case DDL_ERR_HIP: return "HIP runtime error";
        case DDL_ERR_UNSUPPORTED: return "not supported by this entry point";
    }
    return "unknown status";
}

}  // extern "C"
