// gfx950 kernels of the simulated multi-ring allreduce: one launch executes all P transfers
// of one phase (Sec. 4.3: a phase is N concurrent transfers of an N-th of the data each).
//
//   reduce_add_step : dst[off .. off+n) <- dst[..] + src[..]   (Sec. 4.1 ReduceScatter phase)
//   copy_step       : dst[off .. off+n) <- src[..]             (Sec. 4.1 AllGather phase,
//                                                               i.e. the paper's assignment)
//   resolve_ops     : per call, turns the plan's (learner, offset) operations into absolute
//                     (src address, dst address, length) records for the caller's buffers
//   step_kernel_list: the same two phase operations for plans over several tensors
//   fused_kernel, fused_gather_kernel: the step-fused allreduce (further down)
//
// The two phase kernels stream through HBM once: 12 resp. 8 bytes of traffic per fp32
// element and one add, so the bound is memory bandwidth.  No LDS (every element is touched
// by exactly one lane), no MFMA (nothing is contracted).  Each lane moves 16-byte vectors
// (global_load/store_dwordx4, non-temporal), so one wave instruction covers 1 KiB.
//
// Shape, from measurement on MI355X: the highest sustained bandwidth comes from very many
// small workgroups (one wave, one 1 KiB vector row per operand) dispatched in address
// order, not from persistent or deeply unrolled loops: the set of rows in flight then
// stays a narrow window that slides through memory.  A workgroup that small lives only a
// few memory latencies, so its prologue must be short: the operation record is one
// 32-byte scalar load from a table of absolute addresses (written by resolve_ops).
//
// Grid: blockIdx.y = operation (sending learner), blockIdx.x strides over that
// operation's tiles.  Consecutive workgroups are handed to the 8 XCDs round-robin, so
// neighbouring tiles of one chunk stream through different L2s/channels in parallel; there
// is no reuse to keep local to one XCD.
//
// The sum is formed in the element type with one rounding per add; the build disables
// packed-fp32 instructions and floating-point contraction.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <utility>
#include <vector>

#include "kernels.h"

#ifndef DDL_THREADS
#define DDL_THREADS 64
#endif
#ifndef DDL_UNROLL
#define DDL_UNROLL 1
#endif
#ifndef DDL_NT_LOAD
#define DDL_NT_LOAD 1
#endif
#ifndef DDL_NT_STORE
#define DDL_NT_STORE 1
#endif
// A launch stays below this many threads; the kernels stride over what is left.  (A build
// with a small value makes small inputs take the striding paths: that is how they are tested.)
#ifndef DDL_MAX_GRID_THREADS
#define DDL_MAX_GRID_THREADS (uint64_t(1) << 32)
#endif

namespace ddl {
namespace {

// Element traits: the scalar S as stored, the 16-byte vector V a lane moves, and the sum of
// two of either (X = S or V), formed in the element type with one rounding per element.
template <typename T> struct Elem;
template <> struct Elem<float> {
    typedef float S;
    typedef float V __attribute__((ext_vector_type(4)));
    template <typename X> static __device__ __forceinline__ X sum(X a, X b) { return a + b; }
};
template <> struct Elem<double> {
    typedef double S;
    typedef double V __attribute__((ext_vector_type(2)));
    template <typename X> static __device__ __forceinline__ X sum(X a, X b) { return a + b; }
};
// 32-bit integers are summed as unsigned: wrap-around, the same bits as two's complement
template <> struct Elem<unsigned> {
    typedef unsigned S;
    typedef unsigned V __attribute__((ext_vector_type(4)));
    template <typename X> static __device__ __forceinline__ X sum(X a, X b) { return a + b; }
};
template <> struct Elem<_Float16> {
    typedef _Float16 S;
    typedef _Float16 V __attribute__((ext_vector_type(8)));
    template <typename X> static __device__ __forceinline__ X sum(X a, X b) { return a + b; }
};
// bfloat16 travels as its 16 raw bits; widened to binary32 (exact), added there, and
// rounded back to the nearest bfloat16, ties to even.
struct bf16_bits {};
template <> struct Elem<bf16_bits> {
    typedef unsigned short S;
    typedef unsigned short V __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ S sum(S a, S b) {
        const float f = __uint_as_float(unsigned(a) << 16) + __uint_as_float(unsigned(b) << 16);
        const unsigned w = __float_as_uint(f);
        if ((w & 0x7FFFFFFFu) > 0x7F800000u) return S((w >> 16) | 0x0040u);  // NaN stays NaN
        return S((w + 0x7FFFu + ((w >> 16) & 1u)) >> 16);
    }
    static __device__ __forceinline__ V sum(V a, V b) {
        V r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = sum(S(a[i]), S(b[i]));
        return r;
    }
};

// Pointers are tagged as global memory so the loads and stores are global_* rather than
// flat_* instructions (no aperture check, no LDS counter involvement).
#define DDL_GLOBAL __attribute__((address_space(1)))

template <typename V> __device__ __forceinline__ V stream_load(const DDL_GLOBAL V* p) {
#if DDL_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename V> __device__ __forceinline__ void stream_store(DDL_GLOBAL V* p, V v) {
#if DDL_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// Learner pointers beyond what one kernel-argument table holds reach the device in slices
// of that table, so that no call ever reads the caller's host array asynchronously.
__global__ __launch_bounds__(256) void store_pointers(const PtrTable slice, void** __restrict__ d_ptrs,
                                                      unsigned first, unsigned P) {
    const unsigned j = first + threadIdx.x;
    if (threadIdx.x < unsigned(kKernargLearners) && j < P) d_ptrs[j] = slice.p[threadIdx.x];
}

// One thread per (step, sender): absolute addresses for this call's buffers.
__global__ __launch_bounds__(256) void resolve_ops(const PtrTable table, void* const* __restrict__ d_ptrs,
                                                   const Op* __restrict__ ops, ResolvedOp* __restrict__ out,
                                                   unsigned total, unsigned elem_size) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= total) return;
    const Op op = ops[i];
    const uint64_t byte_off = op.off * elem_size;
    const uint64_t src = reinterpret_cast<uint64_t>(d_ptrs ? d_ptrs[op.src] : table.p[op.src]);
    const uint64_t dst = reinterpret_cast<uint64_t>(d_ptrs ? d_ptrs[op.dst] : table.p[op.dst]);
    ResolvedOp r;
    r.src = src + byte_off;
    r.dst = dst + byte_off;
    r.n = op.n;
    r.reserved = 0;
    out[i] = r;
}

// The allocation-free entry point has no uploaded operation table: one thread per
// (phase, sender) derives its transfer from the box itself and writes the record for this
// call's buffers.
__global__ __launch_bounds__(256) void resolve_from_box(const PtrTable table, const BoxArgs box,
                                                        ResolvedOp* __restrict__ out) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= box.steps * box.P) return;
    uint64_t off, n;
    int src, dst;
    box_op(box, i, &off, &n, &src, &dst);
    ResolvedOp rec;
    rec.src = reinterpret_cast<uint64_t>(table.p[src]) + off * box.elem_size;
    rec.dst = reinterpret_cast<uint64_t>(table.p[dst]) + off * box.elem_size;
    rec.n = n;
    rec.reserved = 0;
    out[i] = rec;
}

// Operation records of the allocation-free entry point.  Every GPU the library runs on
// holds its own copy of this array at its own address; host code uses the address that
// hipGetSymbolAddress returns for the current device, never the array's name.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

typedef uint64_t u64x4 __attribute__((ext_vector_type(4)));

// Rows of one wave (64 lanes x 16 bytes) are laid on absolute 1 KiB boundaries of the
// destination, whatever the chunk offset: a row that straddles cache lines would be fetched
// and partially written by two different XCDs.
constexpr uint64_t kRowBytes = 1024;
constexpr uint64_t kRowVecs = kRowBytes / 16;

// One tile of one operation: DDL_THREADS * DDL_UNROLL vectors starting at vector index
// `first` of the row-aligned tiling (first may be negative or reach past the end at the
// edges of the operation).
template <typename T, bool REDUCE>
__device__ __forceinline__ void step_tile(const DDL_GLOBAL typename Elem<T>::V* src,
                                          DDL_GLOBAL typename Elem<T>::V* dst, int64_t n, int64_t nv,
                                          int64_t first, int64_t tid) {
    typedef typename Elem<T>::V V;
    typedef typename Elem<T>::S S;
    constexpr int64_t VL = 16 / sizeof(S);
    constexpr int64_t TILE = int64_t(DDL_THREADS) * DDL_UNROLL;
    if (first >= 0 && first + TILE <= nv) {
        const DDL_GLOBAL V* s = src + first + tid;
        DDL_GLOBAL V* d = dst + first + tid;
        V a[DDL_UNROLL];
        V b[DDL_UNROLL];
#pragma unroll
        for (int u = 0; u < DDL_UNROLL; ++u) a[u] = stream_load(s + u * DDL_THREADS);
        if (REDUCE) {
#pragma unroll
            for (int u = 0; u < DDL_UNROLL; ++u) b[u] = stream_load(d + u * DDL_THREADS);
#pragma unroll
            for (int u = 0; u < DDL_UNROLL; ++u) a[u] = Elem<T>::sum(b[u], a[u]);
        }
#pragma unroll
        for (int u = 0; u < DDL_UNROLL; ++u) stream_store(d + u * DDL_THREADS, a[u]);
    } else {
        // first or last tile of the operation: per-lane bounds
#pragma unroll
        for (int u = 0; u < DDL_UNROLL; ++u) {
            const int64_t v = first + u * DDL_THREADS + tid;
            if (v >= 0 && v < nv) {
                V a = src[v];
                if (REDUCE) a = Elem<T>::sum(dst[v], a);
                dst[v] = a;
            } else if (v == nv) {
                // the buffer's last, short vector: element by element
                const DDL_GLOBAL S* se = (const DDL_GLOBAL S*)(src + nv);
                DDL_GLOBAL S* de = (DDL_GLOBAL S*)(dst + nv);
                for (int64_t e = 0; e < n - nv * VL; ++e) {
                    S a = se[e];
                    if (REDUCE) a = Elem<T>::sum(de[e], a);
                    de[e] = a;
                }
            }
        }
    }
}

template <typename T, bool REDUCE>
__global__ __launch_bounds__(DDL_THREADS) void step_kernel(const ResolvedOp* __restrict__ rops,
                                                           unsigned tile_stride) {
    typedef typename Elem<T>::V V;
    constexpr int64_t VL = 16 / sizeof(typename Elem<T>::S);        // elements per vector
    constexpr int64_t TILE = int64_t(DDL_THREADS) * DDL_UNROLL;     // vectors per tile

    // the whole record in one scalar load: {src address, dst address, n, -}
    const u64x4 rec = *reinterpret_cast<const u64x4*>(rops + blockIdx.y);
    const DDL_GLOBAL V* src = (const DDL_GLOBAL V*)rec.x;
    DDL_GLOBAL V* dst = (DDL_GLOBAL V*)rec.y;
    const int64_t n = int64_t(rec.z);
    const int64_t nv = n / VL;                                      // whole vectors
    const int64_t shift = int64_t((rec.y % kRowBytes) / 16);        // vectors past a row boundary

    // vector index v of the operation <-> slot v + shift of the row-aligned tiling
    for (int64_t first = int64_t(blockIdx.x) * TILE - shift; first <= nv; first += int64_t(tile_stride) * TILE)
        step_tile<T, REDUCE>(src, dst, n, nv, first, threadIdx.x);
}

// Assignment of one buffer to another: the copy phase for a single operation whose record
// arrives as kernel arguments.
template <typename T>
__global__ __launch_bounds__(DDL_THREADS) void assign_kernel(uint64_t src_addr, uint64_t dst_addr, uint64_t n_,
                                                             unsigned tile_stride) {
    typedef typename Elem<T>::V V;
    constexpr int64_t VL = 16 / sizeof(typename Elem<T>::S);
    constexpr int64_t TILE = int64_t(DDL_THREADS) * DDL_UNROLL;
    const int64_t n = int64_t(n_);
    const int64_t nv = n / VL;
    const int64_t shift = int64_t((dst_addr % kRowBytes) / 16);
    for (int64_t first = int64_t(blockIdx.x) * TILE - shift; first <= nv; first += int64_t(tile_stride) * TILE)
        step_tile<T, false>((const DDL_GLOBAL V*)src_addr, (DDL_GLOBAL V*)dst_addr, n, nv, first, threadIdx.x);
}

template <typename T>
hipError_t launch_assign_typed(void* dst, const void* src, uint64_t n, hipStream_t stream) {
    constexpr uint64_t VL = 16 / sizeof(typename Elem<T>::S);
    constexpr uint64_t TILE = uint64_t(DDL_THREADS) * DDL_UNROLL;
    uint64_t tiles = (n / VL + 1 + (kRowVecs - 1) + TILE - 1) / TILE;
    uint64_t max_x = DDL_MAX_GRID_THREADS / DDL_THREADS - 1;
    if (max_x == 0) max_x = 1;
    if (tiles > max_x) tiles = max_x;
    hipLaunchKernelGGL((assign_kernel<T>), dim3(static_cast<unsigned>(tiles)), dim3(DDL_THREADS), 0, stream,
                       reinterpret_cast<uint64_t>(src), reinterpret_cast<uint64_t>(dst), n,
                       static_cast<unsigned>(tiles));
    return hipGetLastError();
}

// Several-tensor plans: the phase's transfers differ in length by orders of magnitude, so
// the launch is a flat list of work items.  Whole items (kListRows interior rows of one
// operation) come first and get one single-wave workgroup per row, like the single-tensor
// kernel; their addresses were bound to the call's buffers beforehand (resolve_items), so
// the workgroup's prologue is one 16-byte scalar load and needs no bounds.  The ragged items
// that hold the first and last rows of each operation (all there is of a tiny tensor's
// chunk) get one workgroup each, which walks their rows with bounds checks.
__global__ __launch_bounds__(256) void resolve_items(const ResolvedOp* __restrict__ rops,
                                                     const BlockDesc* __restrict__ whole,
                                                     ItemRec* __restrict__ out, unsigned total) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= total) return;
    const BlockDesc item = whole[i];
    const ResolvedOp rec = rops[item.op];
    const uint64_t shift = (rec.dst % kRowBytes) / 16;
    const uint64_t byte_off = (uint64_t(item.row) * 64 - shift) * 16;   // row >= 1: never negative
    ItemRec r;
    r.src = rec.src + byte_off;
    r.dst = rec.dst + byte_off;
    out[i] = r;
}

typedef uint64_t u64x2 __attribute__((ext_vector_type(2)));

template <typename T, bool REDUCE>
__global__ __launch_bounds__(64) void step_kernel_list(const ResolvedOp* __restrict__ rops,
                                                       const ItemRec* __restrict__ items,
                                                       const BlockDesc* __restrict__ ragged,
                                                       unsigned whole_blocks, unsigned ragged_count,
                                                       unsigned period, unsigned block_offset) {
    static_assert(DDL_THREADS * DDL_UNROLL == 64, "a row is one wave's worth of vectors");
    typedef typename Elem<T>::V V;
    typedef typename Elem<T>::S S;
    constexpr int64_t VL = 16 / sizeof(S);
    // Ragged items are latency-bound (a chain of two table loads, then rows with bounds):
    // they are spread evenly through the launch, the last workgroup of every `period`,
    // so that the streaming rows around them hide them.
    const unsigned b = blockIdx.x + block_offset;
    unsigned q, w;
    bool whole;
    if (period == 0) {   // all ragged items after the whole rows
        whole = b < whole_blocks;
        w = b;
        q = b - whole_blocks;
    } else {
        q = b / period;
        whole = b % period != period - 1 || q >= ragged_count;
        w = b - (q < ragged_count ? q : ragged_count);   // index among the whole rows
    }
    if (whole) {
        const u64x2 rec = *reinterpret_cast<const u64x2*>(items + w / kListRows);
        const uint64_t row_off = uint64_t(w % kListRows) * kRowBytes;
        const DDL_GLOBAL V* s = (const DDL_GLOBAL V*)(rec.x + row_off) + threadIdx.x;
        DDL_GLOBAL V* d = (DDL_GLOBAL V*)(rec.y + row_off) + threadIdx.x;
        V a = stream_load(s);
        if (REDUCE) a = Elem<T>::sum(stream_load((const DDL_GLOBAL V*)d), a);
        stream_store(d, a);
        return;
    }
    const BlockDesc item = ragged[q];
    const u64x4 rec = *reinterpret_cast<const u64x4*>(rops + item.op);
    const DDL_GLOBAL V* src = (const DDL_GLOBAL V*)rec.x;
    DDL_GLOBAL V* dst = (DDL_GLOBAL V*)rec.y;
    const int64_t n = int64_t(rec.z);
    const int64_t nv = n / VL;
    const int64_t shift = int64_t((rec.y % kRowBytes) / 16);
    // all rows of the item at once: loads first, then the stores
    const int64_t v0 = int64_t(item.row) * 64 - shift + threadIdx.x;
    V a[kListTailRows], c[kListTailRows];
#pragma unroll
    for (int k = 0; k < kListTailRows; ++k) {
        const int64_t v = v0 + k * 64;
        if (v >= 0 && v < nv) {
            a[k] = src[v];
            if (REDUCE) c[k] = dst[v];
        }
    }
#pragma unroll
    for (int k = 0; k < kListTailRows; ++k) {
        const int64_t v = v0 + k * 64;
        if (v >= 0 && v < nv) {
            dst[v] = REDUCE ? Elem<T>::sum(c[k], a[k]) : a[k];
        } else if (v == nv) {
            // the buffer's last, short vector: element by element
            const DDL_GLOBAL S* se = (const DDL_GLOBAL S*)(src + nv);
            DDL_GLOBAL S* de = (DDL_GLOBAL S*)(dst + nv);
            for (int64_t e = 0; e < n - nv * VL; ++e) {
                S x = se[e];
                if (REDUCE) x = Elem<T>::sum(de[e], x);
                de[e] = x;
            }
        }
    }
}

// Workgroups one launch of the list kernel holds at most (64 threads each: below 2^32 threads).
#ifndef DDL_LIST_PER_LAUNCH
#define DDL_LIST_PER_LAUNCH ((uint64_t(1) << 26) - 1)
#endif

template <typename T>
hipError_t launch_list_typed(const Step& step, int learners, const ResolvedOp* d_rops, const ItemRec* d_items,
                             const BlockDesc* d_ragged, hipStream_t stream) {
    static_assert(kListHeadRows == kListTailRows, "the head of an operation is one ragged item");
    const uint64_t whole_blocks = uint64_t(step.whole_count) * kListRows;
    const uint64_t blocks = whole_blocks + uint64_t(step.ragged_count);
    if (blocks == 0) return hipSuccess;
    if (blocks > 0xFFFFFFFFull) return hipErrorInvalidValue;
    const uint64_t per_launch = DDL_LIST_PER_LAUNCH;
    // Measured on MI355X with ResNet-sized tensor lists: spreading the ragged items through
    // the launch gains 2-3 % with 16 and 64 learners and loses 15 % with 256, where the
    // ragged items of one phase touch small ranges of some five hundred different buffers
    // (which presumably evicts the address translations the streaming rows use); then they
    // go last.
#ifndef DDL_LIST_INTERLEAVE_MAX_LEARNERS
#define DDL_LIST_INTERLEAVE_MAX_LEARNERS 64
#endif
    const unsigned period = learners <= DDL_LIST_INTERLEAVE_MAX_LEARNERS && step.ragged_count
                                ? static_cast<unsigned>(blocks / step.ragged_count) : 0u;
    for (uint64_t start = 0; start < blocks; start += per_launch) {
        const uint64_t now = blocks - start < per_launch ? blocks - start : per_launch;
        const dim3 grid(static_cast<unsigned>(now), 1, 1);
        if (step.kind == DDL_STEP_REDUCE)
            hipLaunchKernelGGL((step_kernel_list<T, true>), grid, dim3(64), 0, stream, d_rops,
                               d_items + step.whole_first, d_ragged + step.ragged_first, unsigned(whole_blocks),
                               unsigned(step.ragged_count), period, unsigned(start));
        else
            hipLaunchKernelGGL((step_kernel_list<T, false>), grid, dim3(64), 0, stream, d_rops,
                               d_items + step.whole_first, d_ragged + step.ragged_first, unsigned(whole_blocks),
                               unsigned(step.ragged_count), period, unsigned(start));
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

template <typename T>
hipError_t launch_typed(const ddl_plan& plan, const Step& step, const ResolvedOp* d_rops,
                        hipStream_t stream) {
    constexpr uint64_t VL = 16 / sizeof(typename Elem<T>::S);
    constexpr uint64_t TILE = uint64_t(DDL_THREADS) * DDL_UNROLL;  // vectors
    // slots to cover: the whole vectors, one for a short last vector, and the row shift
    uint64_t tiles = (step.max_n / VL + 1 + (kRowVecs - 1) + TILE - 1) / TILE;
    // keep gridDim.x * gridDim.y * blockDim.x below 2^32; the kernel strides over the rest
    const uint64_t max_x = (DDL_MAX_GRID_THREADS / DDL_THREADS - 1) / uint64_t(plan.P);
    if (tiles > max_x) tiles = max_x;
    if (tiles == 0) tiles = 1;
    const dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(plan.P), 1);
    const dim3 block(DDL_THREADS, 1, 1);
    if (step.kind == DDL_STEP_REDUCE)
        hipLaunchKernelGGL((step_kernel<T, true>), grid, block, 0, stream, d_rops, grid.x);
    else
        hipLaunchKernelGGL((step_kernel<T, false>), grid, block, 0, stream, d_rops, grid.x);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Step-fused allreduce
// ---------------------------------------------------------------------------------------
// Tables are read through the constant address space so that every access is a scalar
// load even after the kernel has started storing to the learners' buffers.
#define DDL_CONST __attribute__((address_space(4)))

__global__ __launch_bounds__(256) void fused_resolve(const PtrTable table, void* const* __restrict__ d_ptrs,
                                                     const uint32_t* __restrict__ seq,
                                                     const uint64_t* __restrict__ own_off,
                                                     uint64_t* __restrict__ out, unsigned P, unsigned padded,
                                                     unsigned elem_size) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= P * padded) return;
    const unsigned c = i / padded;
    const unsigned r = seq[i];
    const uint64_t base = reinterpret_cast<uint64_t>(d_ptrs ? d_ptrs[r] : table.p[r]);
    out[i] = base + own_off[c] * elem_size;
}

// One item enters the nest of ring folds: level 0 takes the learner's value; a level that
// this item completes hands its sum on to the next level (Sec. 4.3: the box is reduced
// one dimension after the other, each ring adding its partial results in ring order).
// `word` is uniform across the wave, so every branch here is a scalar branch.
template <typename T, typename X>
__device__ __forceinline__ void fused_feed(X (&acc)[DDL_FUSED_MAX_LEVELS], X v, uint32_t word, int levels) {
    if (word & 1u) acc[0] = v;
    else acc[0] = Elem<T>::sum(acc[0], v);
    if (!(word & 0x100u)) return;  // the ring of level 0 is not complete yet
    v = acc[0];
#pragma unroll
    for (int t = 1; t < DDL_FUSED_MAX_LEVELS; ++t) {
        if (t >= levels) return;
        if ((word >> t) & 1u) acc[t] = v;
        else acc[t] = Elem<T>::sum(acc[t], v);
        if (!((word >> (8 + t)) & 1u)) return;
        v = acc[t];
    }
}

// Stores of one value to many learners (single-pass form, distribution pass).
#ifndef DDL_GATHER_NT
#define DDL_GATHER_NT 0
#endif
template <typename V> __device__ __forceinline__ void gather_store(DDL_GLOBAL V* p, V v) {
#if DDL_GATHER_NT
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}
// What one pass of the fused kernel stores at every place of a finest chunk.
enum { FUSED_ALL = 0,      // the result to all learners (single-pass form)
       FUSED_REDUCE = 1 }; // the result to the chunk's owner only (first pass of two)

// All P learners' values at one place (a 16-byte vector X = V, or one element X = S): fold
// them in schedule order and store the result.  The chunk's owner is the last learner of
// the summation order (the partial sum travels once round every ring and ends at the
// owner's position).
template <typename T, typename X, int MODE>
__device__ __forceinline__ void fused_place(const DDL_CONST uint64_t* row, const DDL_CONST uint32_t* ctl,
                                            int P, int padded, int levels, uint64_t byte_off) {
    X acc[DDL_FUSED_MAX_LEVELS];
    for (int i0 = 0; i0 < padded; i0 += kFusedBatch) {
        X x[kFusedBatch];
#pragma unroll
        for (int j = 0; j < kFusedBatch; ++j)
            x[j] = stream_load((const DDL_GLOBAL X*)(row[i0 + j] + byte_off));
#pragma unroll
        for (int j = 0; j < kFusedBatch; ++j) {
            const uint32_t word = ctl[i0 + j];
            if (word & kFusedValid) fused_feed<T, X>(acc, x[j], word, levels);
        }
    }
    const X result = acc[levels - 1];
    if (MODE == FUSED_REDUCE) {
        stream_store((DDL_GLOBAL X*)(row[P - 1] + byte_off), result);
        return;
    }
    for (int i0 = 0; i0 < P; i0 += kFusedBatch) {
#pragma unroll
        for (int j = 0; j < kFusedBatch; ++j)
            if (i0 + j < P) gather_store((DDL_GLOBAL X*)(row[i0 + j] + byte_off), result);
    }
}

template <typename T, int MODE>
__global__ __launch_bounds__(64) void fused_kernel(const uint64_t* ptrs_, const uint32_t* ctl_,
                                                   const uint64_t* chunk_n_, int P, int padded,
                                                   int levels, unsigned tile_stride) {
    typedef typename Elem<T>::V V;
    typedef typename Elem<T>::S S;
    constexpr int64_t VL = 16 / sizeof(S);
    const DDL_CONST uint64_t* row = (const DDL_CONST uint64_t*)ptrs_ + size_t(blockIdx.y) * padded;
    const DDL_CONST uint32_t* ctl = (const DDL_CONST uint32_t*)ctl_;
    const int64_t n = int64_t(((const DDL_CONST uint64_t*)chunk_n_)[blockIdx.y]);
    const int64_t nv = n / VL;
    const int64_t shift = int64_t((row[P - 1] % kRowBytes) / 16);
    const int64_t tid = threadIdx.x;

    for (int64_t first = int64_t(blockIdx.x) * 64 - shift; first <= nv; first += int64_t(tile_stride) * 64) {
        const int64_t v = first + tid;
        if (v >= 0 && v < nv) {
            fused_place<T, V, MODE>(row, ctl, P, padded, levels, uint64_t(v) * 16);
        } else if (v == nv) {
            // the buffer's last, short vector: element by element
            for (int64_t e = nv * VL; e < n; ++e)
                fused_place<T, S, MODE>(row, ctl, P, padded, levels, uint64_t(e) * sizeof(S));
        }
    }
}

// Distribution pass of the two-pass form: every wave reads DDL_GATHER_ROWS consecutive rows of
// a chunk from its owner, keeps them in registers and stores them to all other learners.
// Measured on MI355X (one chunk to 15 / 63 / 255 destinations): the shape of the workgroup
// hardly matters; plain stores beat non-temporal ones by 3-10 % here, and four waves of
// four rows are the best of the shapes tried.  Splitting the destinations over several
// workgroups that re-read the rows from cache is never better.
#ifndef DDL_GATHER_ROWS
#define DDL_GATHER_ROWS 4
#endif
#ifndef DDL_GATHER_WAVES
#define DDL_GATHER_WAVES 4
#endif
template <typename T>
__global__ __launch_bounds__(64 * DDL_GATHER_WAVES) void fused_gather_kernel(const uint64_t* ptrs_,
                                                                             const uint64_t* chunk_n_, int P,
                                                                             int padded, unsigned tile_stride) {
    typedef typename Elem<T>::V V;
    typedef typename Elem<T>::S S;
    constexpr int64_t VL = 16 / sizeof(S);
    constexpr int R = DDL_GATHER_ROWS;
    constexpr int64_t kWaveVecs = int64_t(R) * 64;                      // vectors per wave
    constexpr int64_t kTileVecs = kWaveVecs * DDL_GATHER_WAVES;         // vectors per workgroup
    const DDL_CONST uint64_t* row = (const DDL_CONST uint64_t*)ptrs_ + size_t(blockIdx.y) * padded;
    const int64_t n = int64_t(((const DDL_CONST uint64_t*)chunk_n_)[blockIdx.y]);
    const int64_t nv = n / VL;
    const uint64_t src_addr = row[P - 1];
    const int64_t shift = int64_t((src_addr % kRowBytes) / 16);
    const int64_t lane = threadIdx.x % 64;
    const int64_t wave = threadIdx.x / 64;
    for (int64_t tile = int64_t(blockIdx.x) * kTileVecs - shift; tile <= nv; tile += int64_t(tile_stride) * kTileVecs) {
        const int64_t first = tile + wave * kWaveVecs;   // this wave's R rows: vectors [first, first + R * 64)
        if (first >= 0 && first + kWaveVecs <= nv) {
            V x[R];
#pragma unroll
            for (int r = 0; r < R; ++r) x[r] = stream_load((const DDL_GLOBAL V*)src_addr + first + r * 64 + lane);
            for (int j = 0; j < P - 1; ++j) {
                DDL_GLOBAL V* d = (DDL_GLOBAL V*)row[j] + first + lane;
#pragma unroll
                for (int r = 0; r < R; ++r) gather_store(d + r * 64, x[r]);
            }
        } else {
            // first or last rows of the chunk: per-lane bounds
            for (int r = 0; r < R; ++r) {
                const int64_t v = first + r * 64 + lane;
                if (v >= 0 && v < nv) {
                    const V x = ((const DDL_GLOBAL V*)src_addr)[v];
                    for (int j = 0; j < P - 1; ++j) ((DDL_GLOBAL V*)row[j])[v] = x;
                } else if (v == nv) {
                    // the buffer's last, short vector: element by element
                    for (int64_t e = nv * VL; e < n; ++e) {
                        const S x = ((const DDL_GLOBAL S*)src_addr)[e];
                        for (int j = 0; j < P - 1; ++j) ((DDL_GLOBAL S*)row[j])[e] = x;
                    }
                }
            }
        }
    }
}

template <typename T>
hipError_t launch_fused_typed(const ddl_plan& plan, const DeviceTables& t, const uint64_t* fused_ptrs,
                              int padded, int levels, uint64_t max_chunk, int mode, hipStream_t stream) {
    constexpr uint64_t VL = 16 / sizeof(typename Elem<T>::S);
    uint64_t tiles = (max_chunk / VL + 1 + (kRowVecs - 1) + 63) / 64;
    const uint64_t max_x = (DDL_MAX_GRID_THREADS / 64 - 1) / uint64_t(plan.P);
    if (tiles > max_x) tiles = max_x;
    if (tiles == 0) tiles = 1;
    const dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(plan.P), 1);
    if (mode == FUSED_ALL)
        hipLaunchKernelGGL((fused_kernel<T, FUSED_ALL>), grid, dim3(64), 0, stream, fused_ptrs,
                           t.fused_ctl, t.fused_n, plan.P, padded, levels, grid.x);
    else if (mode == FUSED_REDUCE)
        hipLaunchKernelGGL((fused_kernel<T, FUSED_REDUCE>), grid, dim3(64), 0, stream, fused_ptrs,
                           t.fused_ctl, t.fused_n, plan.P, padded, levels, grid.x);
    else {
        constexpr uint64_t kTileVecs = uint64_t(DDL_GATHER_ROWS) * 64 * DDL_GATHER_WAVES;
        constexpr uint64_t kThreads = 64 * DDL_GATHER_WAVES;
        uint64_t wide = (max_chunk / VL + 1 + (kRowVecs - 1) + kTileVecs - 1) / kTileVecs;
        const uint64_t max_w = (DDL_MAX_GRID_THREADS / kThreads - 1) / uint64_t(plan.P);
        if (wide > max_w) wide = max_w;
        const dim3 grid2(static_cast<unsigned>(wide ? wide : 1), static_cast<unsigned>(plan.P), 1);
        hipLaunchKernelGGL((fused_gather_kernel<T>), grid2, dim3(kThreads), 0, stream, fused_ptrs, t.fused_n,
                           plan.P, padded, grid2.x);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Ring walk: all d-1 phases of one box dimension in one launch
// ---------------------------------------------------------------------------------------
// During the d-1 reduce-scatter phases of a dimension every chunk travels once round its
// ring: it sets out from the position after its owner and each next position adds its own
// copy and stores the sum (Sec. 4.3: d-1 phases of d concurrent transfers).  One wave can
// carry a row of the chunk along that whole path: it loads the row from all d positions,
// adds them in ring order and stores every partial sum where the phases would have left
// it.  The memory state after the launch is the phases' state bit for bit, but the partial
// sum is never read back: (2d-1) accesses per element instead of 3(d-1).  The gather is the
// same walk with one load and d-1 stores (d accesses instead of 2(d-1)).
// Rows of the table: length n, then the chunk's address at the d positions in ring order.
__global__ __launch_bounds__(256) void resolve_walk(const PtrTable table, void* const* __restrict__ d_ptrs,
                                                    const uint64_t* __restrict__ plan_rows,
                                                    uint64_t* __restrict__ out, unsigned rows, unsigned d,
                                                    unsigned elem_size) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= rows) return;
    const uint64_t* in = plan_rows + size_t(i) * (d + 2);
    uint64_t* o = out + size_t(i) * (d + 1);
    const uint64_t byte_off = in[0] * elem_size;
    o[0] = in[1];
    for (unsigned k = 0; k < d; ++k) {
        const uint64_t r = in[2 + k];
        o[1 + k] = reinterpret_cast<uint64_t>(d_ptrs ? d_ptrs[r] : table.p[r]) + byte_off;
    }
}

#ifndef DDL_WALK_ROWS
#define DDL_WALK_ROWS 4
#endif
#ifndef DDL_WALK_GATHER_ROWS
#define DDL_WALK_GATHER_ROWS 1
#endif
#ifndef DDL_WALK_GATHER_NT
#define DDL_WALK_GATHER_NT 0
#endif
template <typename V> __device__ __forceinline__ void walk_gather_store(DDL_GLOBAL V* p, V v) {
#if DDL_WALK_GATHER_NT
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}
constexpr int kWalkBatch = 8;   // ring positions whose rows a wave loads before it adds and stores

// What a walk does at every place of a chunk.  WALK_BOTH serves the last dimension of a whole
// allreduce: its gather overwrites the partial sums of its own reduce-scatter at once, so the
// sum is formed in ring order and stored to all d positions (2d accesses per element).
enum { WALK_GATHER = 0, WALK_REDUCE = 1, WALK_BOTH = 2 };

template <typename T, typename X, int MODE>
__device__ __forceinline__ void walk_place(const DDL_CONST uint64_t* addr, int d, uint64_t byte_off) {
    X acc = *(const DDL_GLOBAL X*)(addr[0] + byte_off);
    for (int i = 1; i < d; ++i) {
        DDL_GLOBAL X* p = (DDL_GLOBAL X*)(addr[i] + byte_off);
        if (MODE != WALK_GATHER) acc = Elem<T>::sum(*p, acc);
        if (MODE != WALK_BOTH) *p = acc;
    }
    if (MODE == WALK_BOTH)
        for (int i = 0; i < d; ++i) *(DDL_GLOBAL X*)(addr[i] + byte_off) = acc;
}

// One tile (R rows of 64 lanes x 16 bytes, starting at vector index `tile` of the chunk's
// row-aligned tiling, which may begin before the chunk or reach past its end).
template <typename T, int MODE, int R>
__device__ __forceinline__ void walk_tile(const DDL_CONST uint64_t* addr, int d, int64_t n, int64_t nv,
                                          int64_t tile, int64_t lane) {
    typedef typename Elem<T>::V V;
    typedef typename Elem<T>::S S;
    constexpr int64_t VL = 16 / sizeof(S);
    constexpr int64_t kTileVecs = int64_t(R) * 64;
    if (tile >= 0 && tile + kTileVecs <= nv) {
        const uint64_t byte_off = uint64_t(tile + lane) * 16;
        V acc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r] = stream_load((const DDL_GLOBAL V*)(addr[0] + byte_off) + r * 64);
        if (MODE != WALK_GATHER) {
            for (int i0 = 1; i0 < d; i0 += kWalkBatch) {
                V x[kWalkBatch][R];
#pragma unroll
                for (int j = 0; j < kWalkBatch; ++j)
                    if (i0 + j < d) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
                            x[j][r] = stream_load((const DDL_GLOBAL V*)(addr[i0 + j] + byte_off) + r * 64);
                    }
#pragma unroll
                for (int j = 0; j < kWalkBatch; ++j)
                    if (i0 + j < d) {
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            acc[r] = Elem<T>::sum(x[j][r], acc[r]);
                            if (MODE == WALK_REDUCE)
                                stream_store((DDL_GLOBAL V*)(addr[i0 + j] + byte_off) + r * 64, acc[r]);
                        }
                    }
            }
        }
        if (MODE != WALK_REDUCE) {
            for (int i = MODE == WALK_BOTH ? 0 : 1; i < d; ++i) {
#pragma unroll
                for (int r = 0; r < R; ++r) walk_gather_store((DDL_GLOBAL V*)(addr[i] + byte_off) + r * 64, acc[r]);
            }
        }
    } else {
        // first or last rows of the chunk: per-lane bounds
        for (int r = 0; r < R; ++r) {
            const int64_t v = tile + r * 64 + lane;
            if (v >= 0 && v < nv) {
                walk_place<T, V, MODE>(addr, d, uint64_t(v) * 16);
            } else if (v == nv) {
                // the buffer's last, short vector: element by element
                for (int64_t e = nv * VL; e < n; ++e) walk_place<T, S, MODE>(addr, d, uint64_t(e) * sizeof(S));
            }
        }
    }
}

// Single-tensor plans: blockIdx.y = the chunk (the learner it sets out from), blockIdx.x
// strides over its tiles.
template <typename T, int MODE>
__global__ __launch_bounds__(64) void walk_kernel(const uint64_t* table_, int d, unsigned tile_stride) {
    constexpr int64_t VL = 16 / sizeof(typename Elem<T>::S);
    constexpr int R = MODE == WALK_GATHER ? DDL_WALK_GATHER_ROWS : DDL_WALK_ROWS;
    constexpr int64_t kTileVecs = int64_t(R) * 64;
    const DDL_CONST uint64_t* row = (const DDL_CONST uint64_t*)table_ + size_t(blockIdx.y) * (d + 1);
    const int64_t n = int64_t(row[0]);
    const DDL_CONST uint64_t* addr = row + 1;
    const int64_t nv = n / VL;
    // rows on absolute 1 KiB boundaries of the chunk at its last position (the owner of a
    // reduced chunk; every learner's copy has the same offset within its buffer)
    const int64_t shift = int64_t((addr[d - 1] % kRowBytes) / 16);
    for (int64_t tile = int64_t(blockIdx.x) * kTileVecs - shift; tile <= nv; tile += int64_t(tile_stride) * kTileVecs)
        walk_tile<T, MODE, R>(addr, d, n, nv, tile, threadIdx.x);
}

// Several-tensor plans: one workgroup per listed tile (chunk, tile index) of kWalkListRows rows.
template <typename T, int MODE>
__global__ __launch_bounds__(64) void walk_kernel_list(const uint64_t* table_, const BlockDesc* __restrict__ items,
                                                       int d, unsigned block_offset) {
    constexpr int64_t VL = 16 / sizeof(typename Elem<T>::S);
    const BlockDesc item = items[blockIdx.x + block_offset];
    const DDL_CONST uint64_t* row = (const DDL_CONST uint64_t*)table_ + size_t(item.op) * (d + 1);
    const int64_t n = int64_t(row[0]);
    const DDL_CONST uint64_t* addr = row + 1;
    const int64_t nv = n / VL;
    const int64_t shift = int64_t((addr[d - 1] % kRowBytes) / 16);
    walk_tile<T, MODE, kWalkListRows>(addr, d, n, nv, int64_t(item.row) * kWalkListRows * 64 - shift, threadIdx.x);
}

template <typename T, int MODE>
hipError_t launch_walk_mode(const ddl_plan& plan, const WalkLevel& level, const uint64_t* d_rows,
                            const BlockDesc* d_items, hipStream_t stream) {
    constexpr uint64_t VL = 16 / sizeof(typename Elem<T>::S);
    // the reduce rows list each chunk's positions from the one after its owner to the owner
    const uint64_t* rows = d_rows + (MODE == WALK_GATHER ? level.gather_rows : level.reduce_rows);
    if (plan.seg_off.size() > 1) {
        const uint64_t blocks = MODE == WALK_GATHER ? level.gather_count : level.reduce_count;
        const BlockDesc* items = d_items + (MODE == WALK_GATHER ? level.gather_items : level.reduce_items);
        if (blocks > 0xFFFFFFFFull) return hipErrorInvalidValue;
        const uint64_t per_launch = DDL_LIST_PER_LAUNCH;
        for (uint64_t start = 0; start < blocks; start += per_launch) {
            const uint64_t now = blocks - start < per_launch ? blocks - start : per_launch;
            hipLaunchKernelGGL((walk_kernel_list<T, MODE>), dim3(static_cast<unsigned>(now)), dim3(64), 0, stream,
                               rows, items, level.d, unsigned(start));
            const hipError_t err = hipGetLastError();
            if (err != hipSuccess) return err;
        }
        return hipSuccess;
    }
    const uint64_t tile_vecs = uint64_t(MODE == WALK_GATHER ? DDL_WALK_GATHER_ROWS : DDL_WALK_ROWS) * 64;
    uint64_t tiles = (level.max_n / VL + 1 + (kRowVecs - 1) + tile_vecs - 1) / tile_vecs;
    const uint64_t max_x = (DDL_MAX_GRID_THREADS / 64 - 1) / uint64_t(plan.P);
    if (tiles > max_x) tiles = max_x;
    if (tiles == 0) tiles = 1;
    const dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(plan.P), 1);
    hipLaunchKernelGGL((walk_kernel<T, MODE>), grid, dim3(64), 0, stream, rows, level.d, grid.x);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_walk_typed(const ddl_plan& plan, const WalkLevel& level, const uint64_t* d_rows,
                             const BlockDesc* d_items, int mode, hipStream_t stream) {
    if (mode == WALK_REDUCE) return launch_walk_mode<T, WALK_REDUCE>(plan, level, d_rows, d_items, stream);
    if (mode == WALK_BOTH) return launch_walk_mode<T, WALK_BOTH>(plan, level, d_rows, d_items, stream);
    return launch_walk_mode<T, WALK_GATHER>(plan, level, d_rows, d_items, stream);
}

}  // namespace

hipError_t launch_resolve_walk(const ddl_plan& plan, const uint64_t* d_walk_plan, uint64_t* d_rows,
                               const PtrTable& table, void* const* d_ptrs, hipStream_t stream) {
    for (const WalkLevel& level : plan.walk_levels)
        for (int half = 0; half < 2; ++half) {
            const unsigned rows = static_cast<unsigned>(size_t(plan.P) * plan.seg_off.size());
            hipLaunchKernelGGL(resolve_walk, dim3((rows + 255) / 256), dim3(256), 0, stream, table, d_ptrs,
                               d_walk_plan + (half == 0 ? level.reduce_plan : level.gather_plan),
                               d_rows + (half == 0 ? level.reduce_rows : level.gather_rows), rows,
                               unsigned(level.d), unsigned(plan.elem_size));
            const hipError_t err = hipGetLastError();
            if (err != hipSuccess) return err;
        }
    return hipSuccess;
}

hipError_t launch_walk(const ddl_plan& plan, const WalkLevel& level, const uint64_t* d_rows,
                       const BlockDesc* d_items, int mode, hipStream_t stream) {
    if (level.max_n == 0) return hipSuccess;
    switch (plan.dtype) {
        case DDL_F32: return launch_walk_typed<float>(plan, level, d_rows, d_items, mode, stream);
        case DDL_F64: return launch_walk_typed<double>(plan, level, d_rows, d_items, mode, stream);
        case DDL_I32: return launch_walk_typed<unsigned>(plan, level, d_rows, d_items, mode, stream);
        case DDL_F16: return launch_walk_typed<_Float16>(plan, level, d_rows, d_items, mode, stream);
        case DDL_BF16: return launch_walk_typed<bf16_bits>(plan, level, d_rows, d_items, mode, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_store_pointers(void* const* bufs, int P, void** d_ptrs, hipStream_t stream) {
    for (int first = 0; first < P; first += kKernargLearners) {
        PtrTable slice;
        std::memset(&slice, 0, sizeof(slice));
        const int now = P - first < kKernargLearners ? P - first : kKernargLearners;
        std::memcpy(slice.p, bufs + first, size_t(now) * sizeof(void*));
        hipLaunchKernelGGL(store_pointers, dim3(1), dim3(256), 0, stream, slice, d_ptrs, unsigned(first),
                           unsigned(P));
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

hipError_t launch_resolve(const ddl_plan& plan, const Op* d_ops, ResolvedOp* d_rops,
                          const PtrTable& table, void* const* d_ptrs, hipStream_t stream) {
    const unsigned total = static_cast<unsigned>(plan.ops.size());
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(resolve_ops, dim3((total + 255) / 256), dim3(256), 0, stream, table, d_ptrs,
                       d_ops, d_rops, total, static_cast<unsigned>(plan.elem_size));
    return hipGetLastError();
}

hipError_t static_scratch(ResolvedOp** out) {
    // the array's device address, looked up once per device with that device current
    static std::mutex mu;
    static std::vector<std::pair<int, void*>> known;
    int device = -1;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess) return err;
    std::lock_guard<std::mutex> lock(mu);
    for (const auto& k : known)
        if (k.first == device) {
            *out = static_cast<ResolvedOp*>(k.second);
            return hipSuccess;
        }
    void* ptr = nullptr;
    err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (err != hipSuccess) return err;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    known.emplace_back(device, ptr);
    *out = static_cast<ResolvedOp*>(ptr);
    return hipSuccess;
}

hipError_t launch_resolve_from_box(const ddl_plan& plan, const PtrTable& table, ResolvedOp* d_rops,
                                   hipStream_t stream) {
    BoxArgs box;
    std::memset(&box, 0, sizeof(box));
    box.m = static_cast<int32_t>(plan.dims.size());
    for (int t = 0; t < box.m; ++t) box.dims[t] = plan.dims[t];
    box.P = static_cast<uint32_t>(plan.P);
    box.elem_size = static_cast<uint32_t>(plan.elem_size);
    box.steps = static_cast<uint32_t>(plan.steps.size());
    box.count = plan.count;
    const unsigned total = box.steps * box.P;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(resolve_from_box, dim3((total + 255) / 256), dim3(256), 0, stream, table, box, d_rops);
    return hipGetLastError();
}

hipError_t launch_resolve_items(const ddl_plan& plan, const ResolvedOp* d_rops, const BlockDesc* d_whole,
                                ItemRec* d_items, hipStream_t stream) {
    const unsigned total = static_cast<unsigned>(plan.whole.size());
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(resolve_items, dim3((total + 255) / 256), dim3(256), 0, stream, d_rops, d_whole, d_items,
                       total);
    return hipGetLastError();
}

hipError_t launch_step(const ddl_plan& plan, const Step& step, const ResolvedOp* d_rops, const ItemRec* d_items,
                       const BlockDesc* d_ragged, hipStream_t stream) {
    if (step.max_n == 0) return hipSuccess;
    if (plan.seg_off.size() > 1) {
        // the lists index the plan's whole table: d_rops is the first step's
        switch (plan.dtype) {
            case DDL_F32: return launch_list_typed<float>(step, plan.P, d_rops, d_items, d_ragged, stream);
            case DDL_F64: return launch_list_typed<double>(step, plan.P, d_rops, d_items, d_ragged, stream);
            case DDL_I32: return launch_list_typed<unsigned>(step, plan.P, d_rops, d_items, d_ragged, stream);
            case DDL_F16: return launch_list_typed<_Float16>(step, plan.P, d_rops, d_items, d_ragged, stream);
            case DDL_BF16: return launch_list_typed<bf16_bits>(step, plan.P, d_rops, d_items, d_ragged, stream);
        }
        return hipErrorInvalidValue;
    }
    d_rops += size_t(&step - plan.steps.data()) * size_t(plan.P);
    switch (plan.dtype) {
        case DDL_F32: return launch_typed<float>(plan, step, d_rops, stream);
        case DDL_F64: return launch_typed<double>(plan, step, d_rops, stream);
        case DDL_I32: return launch_typed<unsigned>(plan, step, d_rops, stream);
        case DDL_F16: return launch_typed<_Float16>(plan, step, d_rops, stream);
        case DDL_BF16: return launch_typed<bf16_bits>(plan, step, d_rops, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_assign(ddl_dtype_t dtype, void* dst, const void* src, uint64_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    switch (dtype) {
        case DDL_F32: return launch_assign_typed<float>(dst, src, n, stream);
        case DDL_F64: return launch_assign_typed<double>(dst, src, n, stream);
        case DDL_I32: return launch_assign_typed<unsigned>(dst, src, n, stream);
        case DDL_F16: return launch_assign_typed<_Float16>(dst, src, n, stream);
        case DDL_BF16: return launch_assign_typed<bf16_bits>(dst, src, n, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_fused_resolve(const ddl_plan& plan, const DeviceTables& t, uint64_t* fused_ptrs,
                                const PtrTable& table, void* const* d_ptrs, hipStream_t stream) {
    const int padded = t.fused_padded;
    const unsigned total = unsigned(plan.P) * unsigned(padded);
    hipLaunchKernelGGL(fused_resolve, dim3((total + 255) / 256), dim3(256), 0, stream, table, d_ptrs,
                       t.fused_seq, t.fused_off, fused_ptrs, unsigned(plan.P), unsigned(padded),
                       unsigned(plan.elem_size));
    return hipGetLastError();
}

hipError_t launch_fused(const ddl_plan& plan, const DeviceTables& t, const uint64_t* fused_ptrs,
                        uint64_t max_chunk, int mode, hipStream_t stream) {
    const int padded = t.fused_padded, levels = t.fused_levels;
    switch (plan.dtype) {
        case DDL_F32: return launch_fused_typed<float>(plan, t, fused_ptrs, padded, levels, max_chunk, mode, stream);
        case DDL_F64: return launch_fused_typed<double>(plan, t, fused_ptrs, padded, levels, max_chunk, mode, stream);
        case DDL_I32: return launch_fused_typed<unsigned>(plan, t, fused_ptrs, padded, levels, max_chunk, mode, stream);
        case DDL_F16: return launch_fused_typed<_Float16>(plan, t, fused_ptrs, padded, levels, max_chunk, mode, stream);
        case DDL_BF16: return launch_fused_typed<bf16_bits>(plan, t, fused_ptrs, padded, levels, max_chunk, mode, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace ddl
