// gfx950 kernels of the simulated multi-ring allreduce: one launch executes all P transfers
// of one phase (Sec. 4.3: a phase is N concurrent transfers of 1/N of the data).
//
//   reduce_add_step : dst[off .. off+n) <- dst[..] + src[..]   (Sec. 4.1 ReduceScatter phase)
//   copy_step       : dst[off .. off+n) <- src[..]             (Sec. 4.1 AllGather phase,
//                                                               i.e. the paper's assignment)
//
// Both stream through HBM once: 12 resp. 8 bytes of traffic per fp32 element and one add,
// so the bound is memory bandwidth.  No LDS (every element is touched by exactly one
// lane), no MFMA (nothing is contracted).  Each lane moves 16-byte vectors
// (global_load/store_dwordx4); a wave covers 1 KiB per instruction, and every lane keeps
// DDL_UNROLL such loads per operand in flight before the first use.  The sum is formed in
// the element type with one rounding per add; the build disables packed-fp32 instructions.
//
// Grid: blockIdx.y = operation (sending learner), blockIdx.x strides over that
// operation's tiles.  Consecutive workgroups are handed to the 8 XCDs round-robin, so
// neighbouring tiles of one chunk stream through different L2s/channels in parallel; there
// is no reuse to keep local to one XCD.
#include <hip/hip_runtime.h>

#include "kernels.h"

#ifndef DDL_THREADS
#define DDL_THREADS 256
#endif
#ifndef DDL_UNROLL
#define DDL_UNROLL 4
#endif
#ifndef DDL_NT_LOAD
#define DDL_NT_LOAD 1
#endif
#ifndef DDL_NT_STORE
#define DDL_NT_STORE 0
#endif

namespace ddl {
namespace {

template <typename T> struct Vec16;
template <> struct Vec16<float>  { typedef float  type __attribute__((ext_vector_type(4))); };
template <> struct Vec16<double> { typedef double type __attribute__((ext_vector_type(2))); };
// 32-bit integers are summed as unsigned: wrap-around, the same bits as two's complement
template <> struct Vec16<unsigned> { typedef unsigned type __attribute__((ext_vector_type(4))); };

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

template <typename T, bool REDUCE>
__global__ __launch_bounds__(DDL_THREADS) void step_kernel(const PtrTable table,
                                                           void* const* __restrict__ d_ptrs,
                                                           const Op* __restrict__ ops) {
    typedef typename Vec16<T>::type V;
    constexpr uint64_t VL = 16 / sizeof(T);                             // elements per vector
    constexpr uint64_t TILE = uint64_t(DDL_THREADS) * DDL_UNROLL * VL;  // elements per tile

    const Op* op = ops + blockIdx.y;
    const uint64_t n = op->n;
    const uint64_t off = op->off;
    const int si = __builtin_amdgcn_readfirstlane(op->src);
    const int di = __builtin_amdgcn_readfirstlane(op->dst);
    const DDL_GLOBAL T* src_base =
        (const DDL_GLOBAL T*)(static_cast<const T*>(d_ptrs ? d_ptrs[si] : table.p[si])) + off;
    DDL_GLOBAL T* dst_base = (DDL_GLOBAL T*)(static_cast<T*>(d_ptrs ? d_ptrs[di] : table.p[di])) + off;
    const unsigned tid = threadIdx.x;

    for (uint64_t base = uint64_t(blockIdx.x) * TILE; base < n; base += uint64_t(gridDim.x) * TILE) {
        const DDL_GLOBAL T* src = src_base + base;
        DDL_GLOBAL T* dst = dst_base + base;
        const uint64_t rem = n - base;
        if (rem >= TILE) {
            const DDL_GLOBAL V* s = (const DDL_GLOBAL V*)src + tid;
            DDL_GLOBAL V* d = (DDL_GLOBAL V*)dst + tid;
            V a[DDL_UNROLL];
            V b[DDL_UNROLL];
#pragma unroll
            for (int u = 0; u < DDL_UNROLL; ++u) a[u] = stream_load(s + u * DDL_THREADS);
            if (REDUCE) {
#pragma unroll
                for (int u = 0; u < DDL_UNROLL; ++u) b[u] = stream_load(d + u * DDL_THREADS);
#pragma unroll
                for (int u = 0; u < DDL_UNROLL; ++u) a[u] = b[u] + a[u];
            }
#pragma unroll
            for (int u = 0; u < DDL_UNROLL; ++u) stream_store(d + u * DDL_THREADS, a[u]);
        } else {
            // ragged end of an operation: whole vectors first, then single elements
            const uint64_t nvec = rem / VL;
            const DDL_GLOBAL V* s = (const DDL_GLOBAL V*)src;
            DDL_GLOBAL V* d = (DDL_GLOBAL V*)dst;
            for (uint64_t i = tid; i < nvec; i += DDL_THREADS) {
                V a = s[i];
                if (REDUCE) a = d[i] + a;
                d[i] = a;
            }
            for (uint64_t i = nvec * VL + tid; i < rem; i += DDL_THREADS) {
                T a = src[i];
                if (REDUCE) a = dst[i] + a;
                dst[i] = a;
            }
        }
    }
}

template <typename T>
hipError_t launch_typed(const ddl_plan& plan, const Step& step, const Op* d_ops,
                        const PtrTable& table, void* const* d_ptrs, hipStream_t stream) {
    constexpr uint64_t TILE = uint64_t(DDL_THREADS) * DDL_UNROLL * (16 / sizeof(T));
    uint64_t tiles = (step.max_n + TILE - 1) / TILE;
    // keep gridDim.x * gridDim.y * blockDim.x below 2^32; the kernel strides over the rest
    const uint64_t max_x = ((uint64_t(1) << 32) / DDL_THREADS - 1) / uint64_t(plan.P);
    if (tiles > max_x) tiles = max_x;
    if (tiles == 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(plan.P), 1);
    const dim3 block(DDL_THREADS, 1, 1);
    if (step.kind == DDL_STEP_REDUCE)
        hipLaunchKernelGGL((step_kernel<T, true>), grid, block, 0, stream, table, d_ptrs, d_ops);
    else
        hipLaunchKernelGGL((step_kernel<T, false>), grid, block, 0, stream, table, d_ptrs, d_ops);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_step(const ddl_plan& plan, const Step& step, const Op* d_ops,
                       const PtrTable& table, void* const* d_ptrs, hipStream_t stream) {
    if (step.max_n == 0) return hipSuccess;
    switch (plan.dtype) {
        case DDL_F32: return launch_typed<float>(plan, step, d_ops, table, d_ptrs, stream);
        case DDL_F64: return launch_typed<double>(plan, step, d_ops, table, d_ptrs, stream);
        case DDL_I32: return launch_typed<unsigned>(plan, step, d_ops, table, d_ptrs, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace ddl
