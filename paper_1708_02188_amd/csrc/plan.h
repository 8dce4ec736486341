// Host-side schedule planner of libddlsim: box dimensions -> per-step operation tables.
// Pure integer code, no HIP; see include/ddlsim.h for the vocabulary.
#pragma once

#include <cstddef>
#include <cstdint>
#include <mutex>
#include <vector>

#include "../../include/ddlsim.h"

namespace ddl {

// One transfer of a phase: elements [off, off+n) of learner src go to learner dst.
// Layout is shared with the kernels (read from device memory as-is).
struct Op {
    uint64_t off;
    uint64_t n;
    int32_t src;
    int32_t dst;
};
static_assert(sizeof(Op) == 24, "Op is read by the kernels with this layout");

// An operation bound to one call's buffers: absolute device addresses, length in elements.
struct ResolvedOp {
    uint64_t src;
    uint64_t dst;
    uint64_t n;
    uint64_t reserved;
};
static_assert(sizeof(ResolvedOp) == 32, "one 32-byte scalar load per workgroup");

// Work items of a phase of a several-tensor plan.  A row is 64 lanes x 16 bytes of the
// kernels' tiling, which is laid on absolute 1 KiB boundaries of the destination at run time
// (row r of an operation of nv whole vectors covers its vectors [64 r - shift, 64 r + 64 -
// shift), 0 <= shift < 64).  Rows kListHeadRows .. and on, as long as kListRows of them end
// at or before vector nv, lie inside the operation whatever the shift: they form "whole"
// items of kListRows rows, whose addresses are bound per call (ItemRec) so that a workgroup
// finds its row with one 16-byte load.  The rows before and after them form "ragged" items
// of up to kListTailRows rows that one workgroup walks with bounds checks.
// `op` indexes the plan's whole operation table (phase-major).
constexpr int kListRows = 16;
constexpr int kListTailRows = 4;
constexpr int kListHeadRows = 4;
struct BlockDesc {
    uint32_t op;
    uint32_t row;
};
// A whole item bound to one call's buffers: addresses of its first row in source and destination.
struct ItemRec {
    uint64_t src;
    uint64_t dst;
};
static_assert(sizeof(ItemRec) == 16, "one 16-byte scalar load per workgroup");

struct Step {
    int kind;           // DDL_STEP_REDUCE / DDL_STEP_GATHER
    int dim;            // 0-based box dimension whose rings run in this phase
    uint64_t max_n;     // longest operation of the phase (sizes the launch)
    uint64_t bytes;     // memory traffic of the phase
    size_t whole_first, whole_count;    // several-tensor plans: this phase's slices of the
    size_t ragged_first, ragged_count;  // whole and ragged work lists
};

// Tables of the step-fused allreduce.  Finest chunk c (owned by learner c) is summed over
// the learners in the order seq[c][0..P-1]; ctl[i] says which ring levels item i opens
// (bits 0-7) and closes (bits 8-15); bit 31 marks a real item (rows are padded to a
// multiple of kFusedBatch).
#ifndef DDL_FUSED_BATCH
#define DDL_FUSED_BATCH 8
#endif
constexpr int kFusedBatch = DDL_FUSED_BATCH;
constexpr uint32_t kFusedValid = 0x80000000u;

// A plan's operations bound to one set of learner buffers on one device.  The phase kernels
// read absolute addresses from `rops`; a call whose buffers equal `key` finds them there
// and binds nothing.  Slots are bound by the calls themselves (least recently used first
// once DDL_PLAN_MAX_BINDINGS exist).
struct Binding {
    std::vector<void*> key;           // the P learner pointers (empty: never bound)
    ResolvedOp* rops = nullptr;       // the plan's operations for these buffers, step-major
    ItemRec* items = nullptr;         // several-tensor plans: the whole work items for these buffers
    void** d_ptrs = nullptr;          // the pointers on the device, when P exceeds the kernarg table
    uint64_t* fused_ptrs = nullptr;   // step-fused path: P * padded absolute addresses (on demand)
    bool rops_valid = false;          // an eager call has enqueued the kernel that fills rops for `key`
    bool fused_valid = false;         // the same for fused_ptrs
    uint64_t* walk = nullptr;         // ring-walk rows bound to these buffers (plans that have them)
    bool pinned = false;              // a captured graph refers to this slot: it is never rebound
    uint64_t last_use = 0;
};

// One box dimension of size d > 1 walked in a single launch (see build_walk): `reduce` /
// `gather` index the first of S * P rows (tensor-major, then the learner a chunk sets out
// from) in the plan's walk table and in a binding's resolved copy.  Several-tensor plans
// also list the tiles of kWalkListRows rows their rows consist of (BlockDesc{row, tile}),
// since their rows differ in length by orders of magnitude.
constexpr int kWalkListRows = 4;
struct WalkLevel {
    int dim;              // 0-based box dimension
    int d;                // ring size
    uint64_t max_n;       // longest chunk (sizes the launch of a single-tensor plan)
    size_t reduce_plan, gather_plan;   // rows of d + 2 words: element offset, length, the d ring members in order
    size_t reduce_rows, gather_rows;   // rows of d + 1 words: length, then the chunk's d addresses in ring order
    size_t reduce_items, gather_items; // several-tensor plans: first tile of each half in walk_items,
    size_t reduce_count, gather_count; // and how many
};

struct DeviceTables {
    int device = -1;
    Op* ops = nullptr;           // num_steps * P operations, step-major
    uint64_t* walk_plan = nullptr;   // ring-walk rows (learner indices), see WalkLevel
    BlockDesc* walk_items = nullptr; // ring-walk tiles of a several-tensor plan
    BlockDesc* whole = nullptr;   // work lists of a several-tensor plan
    BlockDesc* ragged = nullptr;
    // step-fused path, created at its first use
    uint32_t* fused_seq = nullptr;    // P * padded learner ranks
    uint32_t* fused_ctl = nullptr;    // padded control words
    uint64_t* fused_n = nullptr;      // elements of each finest chunk
    uint64_t* fused_off = nullptr;    // element offset of each finest chunk
    int fused_levels = 0;             // box dimensions of size > 1
    int fused_padded = 0;             // row length of fused_seq / fused_ptrs
    std::vector<Binding*> bindings;
    uint64_t clock = 0;               // orders the bindings' last uses
};

}  // namespace ddl

struct ddl_plan {
    std::vector<int> dims;
    int P = 0;
    uint64_t count = 0;
    ddl_dtype_t dtype = DDL_F32;
    int elem_size = 4;
    int first_gather = 0;                 // index of the first all-gather step
    std::vector<ddl::Step> steps;
    std::vector<uint64_t> seg_off, seg_count;  // the tensors inside every learner's buffer (S >= 1)
    std::vector<ddl::Op> ops;             // steps.size() * S * P, step-major, then tensor, then sender
    std::vector<ddl::BlockDesc> whole, ragged;  // work lists, only when S > 1
    std::vector<uint64_t> own_off, own_n; // finest chunk per (tensor, learner)
    uint64_t bytes_total = 0;
    std::vector<ddl::WalkLevel> walk_levels;   // empty: the plan has no ring-walk form
    std::vector<uint64_t> walk_plan;           // rows of all levels (learner indices)
    std::vector<ddl::BlockDesc> walk_items;    // tiles of all levels, only when S > 1
    size_t walk_words = 0;                     // size of a binding's resolved copy
    uint64_t walk_bytes = 0;                   // memory traffic of the ring-walk form

    mutable std::mutex mu;                       // guards `tables` and everything below them
    mutable std::vector<ddl::DeviceTables*> tables;  // one entry per device the plan ran on
    mutable int walk_mode = 0;                   // DDL_WALK_AUTO / _OFF / _ON
};

namespace ddl {

int dtype_size(ddl_dtype_t dtype);  // 0 for an unknown type

// Part k of d of [lo, hi), cut on granules of G elements.
void split_range(uint64_t lo, uint64_t hi, uint64_t d, uint64_t k, uint64_t G,
                 uint64_t* a, uint64_t* b);

// Fills `plan` (dims, P, count, dtype already validated by the caller).
void build_schedule(ddl_plan* plan);

// Ring-walk form of a plan, derived from its phases (call after build_schedule):
// the d-1 phases of a dimension's reduce-scatter pass every chunk once round its ring, so one
// launch can carry each chunk's partial sum from the position after its owner to the owner,
// storing it at every position on the way exactly as the phases do; likewise the d-1 gather
// phases copy every completed chunk from its owner to the other d-1 positions.  Leaves the
// plan without the form if its tables would exceed kWalkMaxWords.
constexpr size_t kWalkMaxWords = size_t(1) << 24;
void build_walk(ddl_plan* plan);

ddl_status_t validate_dims(const int* dims, int m, int P);

// Self-check of a built plan (the schedule's race-freedom and coverage, independent of how
// build_schedule derived it): every operation inside its tensor and on 16-byte granules; in
// every phase each learner sends exactly one and receives exactly one operation per tensor,
// along its ring of the phase's dimension; the range a learner receives is disjoint from the
// range it sends in the same phase (so the P transfers of a phase can run in any order or
// at once); each learner's finest chunks tile every tensor; the ring-walk rows list each
// chunk's ring in order.  Returns DDL_OK or DDL_ERR_ARG.
ddl_status_t verify_plan(const ddl_plan& plan);

// Summation order of the step-fused allreduce; returns the number of box dimensions of
// size > 1 ("levels") and the padded row length.  seq: P * padded, ctl: padded.
int build_fused_order(const ddl_plan& plan, std::vector<uint32_t>* seq, std::vector<uint32_t>* ctl,
                      int* padded);

// Estimated cluster time of reduction + distribution for a box (Sec. 4.3 ring estimate per
// dimension, on the bytes left at that level).
double model_time(const int* dims, int m, double bytes, const double* bw, const double* lat);

// Exhaustive search over boxes; see ddl_choose_dims.
ddl_status_t choose_dims(int P, double bytes, int m, const double* bw, const double* lat,
                         const int* max_dim, int* dims_out, double* time_out);

}  // namespace ddl
