/*
 * libddlsim -- the multi-dimensional ring ("multi-ring") allreduce of gradient buffers,
 * run as a simulated collective inside ONE gfx950 GPU: P virtual learners' buffers sit in
 * that GPU's HBM and every phase of the schedule is executed by a HIP kernel.
 *
 * Plain C ABI: pointers and sizes only.  Where a pointer is a DEVICE pointer it says so;
 * everything else is host memory.  `stream` arguments are a hipStream_t passed as void*
 * (NULL = the default stream).
 *
 * Vocabulary (Sec. 4.3, "Topology aware communication"): N = P learners are placed in an
 * m-dimensional box, P = d_1 * d_2 * ... * d_m; learner rank r has coordinates (c_1..c_m)
 * with c_1 varying fastest (dimension 1 = fastest links).  A ring of d nodes reduces in
 * d-1 phases; in each phase every node passes 1/d of the data to its +1 neighbour.  The
 * reduce-scatter (Sec. 4.1 ReduceScatter) runs the rings of dimension 1, then 2, ... m,
 * each on the part left over by the previous one; the all-gather (Sec. 4.1 AllGather)
 * runs back through the dimensions m ... 1 and copies completed parts (Sec. 4.1
 * assignment).  Afterwards every learner holds R = sum_j V_j (Sec. 4.3).
 *
 * A "step" is one phase: P independent operations, one per sending learner, each a
 * contiguous element range [off, off+n) read from learner `src` and added into
 * (reduce-scatter) or stored over (all-gather) the same range of learner `dst`.
 *
 * Chunk boundaries: a range of n elements is cut into ceil(n/G) granules of G = 16 /
 * sizeof(element) elements; part k of d holds granules floor(k*ng/d) .. floor((k+1)*ng/d)-1.
 * Every non-empty part therefore starts on a 16-byte boundary, only the part that ends
 * the buffer can have a short granule, and parts may be empty for tiny buffers.
 */
#ifndef DDLSIM_H
#define DDLSIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Opaque schedule; created by ddl_ring_plan, owned by the library, freed by ddl_plan_free. */
typedef struct ddl_plan ddl_plan_t;

/* Element types.  Sums are formed in the element type itself, one rounding per addition,
 * round-to-nearest-even (Sec. 4.3 sizes the gradient vector at 4 bytes per element: 90 M
 * entries = 350 MB).  For the 16-bit types that is the correctly rounded 16-bit sum (bf16
 * is widened to binary32, added there and rounded once, which gives the same value). */
typedef enum {
    DDL_F32 = 0,
    DDL_F64 = 1,
    DDL_I32 = 2,  /* two's complement, wraps */
    DDL_F16 = 3,  /* IEEE binary16 */
    DDL_BF16 = 4  /* bfloat16: the upper 16 bits of a binary32 */
} ddl_dtype_t;

typedef enum {
    DDL_OK = 0,
    DDL_ERR_ARG = -1,           /* NULL pointer, P < 1, duplicate buffers, bad step index   */
    DDL_ERR_DIMS = -2,          /* m < 1, a dimension < 1, or product of dims != P          */
    DDL_ERR_DTYPE = -3,         /* unknown element type                                     */
    DDL_ERR_ALIGN = -4,         /* a buffer or a tensor's start is not 16-byte aligned      */
    DDL_ERR_PLAN_MISMATCH = -5, /* P / count / dtype differ from what the plan was made for */
    DDL_ERR_NOMEM = -6,         /* host or device allocation failed                         */
    DDL_ERR_HIP = -7,           /* a HIP runtime call failed (no device, launch error, ...) */
    DDL_ERR_UNSUPPORTED = -8    /* valid arguments this entry point does not serve          */
} ddl_status_t;

enum { DDL_STEP_REDUCE = 0, DDL_STEP_GATHER = 1 };

/* Largest supported numbers of learners, box dimensions and tensors per buffer. */
#define DDL_MAX_LEARNERS 65535
#define DDL_MAX_DIMS 16
#define DDL_MAX_TENSORS 65536
/* A plan stores phases x tensors x learners operations (56 bytes each, host + device);
 * plans beyond this many are refused with DDL_ERR_NOMEM. */
#define DDL_MAX_PLAN_OPS (1ull << 26)
/* A several-tensor plan also stores one work item per 16 KiB that the learners send (8 bytes
 * on the host, 24 on the device per buffer set); plans of more than about this many items
 * (count * sizeof(element) * (P - 1) / 8192) are refused with DDL_ERR_NOMEM. */
#define DDL_MAX_LIST_ITEMS (1ull << 28)

/*
 * Build the schedule for a box dims[0..m-1] (Sec. 4.3: N = d_1*...*d_m) over P learners
 * and `count` elements of `dtype` per learner.  Host-only: needs no GPU.  Dimensions of
 * size 1 are allowed and contribute no steps; count == 0 is allowed.
 * Returns NULL on error; *status (if not NULL) receives the code either way.
 */
ddl_plan_t* ddl_ring_plan(const int* dims, int m, int P, size_t count, ddl_dtype_t dtype,
                          ddl_status_t* status);

/*
 * The same for a buffer that holds several tensors, each reduced on its own (a network's
 * gradients are a list of per-layer tensors; Sec. 4.1: the objects the library works on are
 * such tensors plus metadata).  Tensor s occupies elements [tensor_off[s], tensor_off[s] + tensor_count[s])
 * of every learner's buffer of `count` elements; tensors must be given in ascending order,
 * must not overlap, and must start on 16-byte granules (DDL_ERR_ALIGN otherwise).  Every
 * tensor is chunked by itself (tiny tensors give empty chunks), but all transfers of one
 * phase, over all tensors, are batched into one kernel launch.  Elements outside every
 * tensor are never touched.  The plan is used with the same ddl_*_sim entry points;
 * ddl_allreduce_fused_sim does not serve it (DDL_ERR_UNSUPPORTED).
 */
ddl_plan_t* ddl_ring_plan_tensors(const int* dims, int m, int P, const size_t* tensor_off,
                                  const size_t* tensor_count, int num_tensors, size_t count,
                                  ddl_dtype_t dtype, ddl_status_t* status);

/* Free a plan and its device tables.  NULL is a no-op.  The caller must make sure no
 * enqueued work still uses the plan (synchronise the streams first). */
void ddl_plan_free(ddl_plan_t* plan);

/*
 * Create the plan's device tables on the current device now (those of the step-fused path
 * included, where it serves the plan) together with two free binding slots (see
 * ddl_allreduce_sim), instead of at the first ddl_*_sim calls that need them, which
 * otherwise allocate.  Call it before capturing ddl_*_sim calls into a HIP graph: under
 * capture nothing may allocate.  A capture that uses the plan with more than two buffer
 * sets reserves its slots with ddl_plan_reserve_bindings first.
 */
ddl_status_t ddl_plan_prepare(const ddl_plan_t* plan);

/* ddl_plan_prepare with at least `slots` binding slots (0 .. DDL_PLAN_MAX_BINDINGS). */
#define DDL_PLAN_MAX_BINDINGS 64
ddl_status_t ddl_plan_reserve_bindings(const ddl_plan_t* plan, int slots);

/*
 * Ring walk: how ddl_allreduce_sim, ddl_reduce_scatter_sim and ddl_allgather_sim execute the
 * d-1 phases of one box dimension.  Phase by phase (one kernel launch per phase, the
 * schedule as Sec. 4.3 states it), or as one launch per dimension in which every wave
 * carries a piece of a chunk once round its ring: it loads the piece from all d positions,
 * adds them in ring order and stores each partial sum where the phases would have left it
 * (the gather loads once and stores d-1 times).  Every byte of every buffer ends up exactly
 * as after the phases -- partial sums in the other learners' chunks included -- but the
 * travelling partial sum is never read back from memory: (2d-1) + d memory accesses per
 * element of a dimension's segment instead of 3(d-1) + 2(d-1), and 2 launches per dimension
 * instead of 2(d-1).  A whole allreduce takes its last dimension's two halves in one launch
 * (the sum goes straight to all d positions, 2d accesses: that dimension's gather would
 * overwrite its own partial sums at once).  ddl_plan_walk_bytes gives the traffic of this form.
 *   DDL_WALK_AUTO (default)  walk when the plan's phases average under 16 MiB of traffic
 *                            (launch-bound: the saved phase boundaries dominate), else phases
 *   DDL_WALK_OFF             always phase by phase
 *   DDL_WALK_ON              always walk (DDL_ERR_UNSUPPORTED for a plan without the form:
 *                            one whose walk tables, 2 * tensors * P * (d + 2) words summed over
 *                            the dimensions, would exceed 2^24 words)
 * Several-tensor plans walk too (every tensor's chunks round their rings, all of a
 * dimension in one launch over a list of 4 KiB tiles).
 * The measurement entry points with an event per step always run phase by phase.
 */
enum { DDL_WALK_AUTO = 0, DDL_WALK_OFF = 1, DDL_WALK_ON = 2 };
ddl_status_t ddl_plan_set_walk(const ddl_plan_t* plan, int mode);

/*
 * In-place allreduce (Sec. 4.3: reduction R = sum_j V_j and its distribution to all
 * learners) over the plan's schedule.
 *   bufs   HOST array of P DEVICE pointers; bufs[j] is learner j's buffer of at least
 *          `count` elements, 16-byte aligned, pairwise distinct and non-overlapping,
 *          owned by the caller.  The array itself may be reused as soon as the call returns.
 *          With count == 0 the pointers are not examined (empty buffers may be NULL).
 *   P, count, dtype must equal the plan's.
 * Enqueues one kernel per step (or per dimension, see ddl_plan_set_walk) on `stream` and
 * returns without synchronising; when the stream has drained, every bufs[j] holds the sum,
 * bit-identical across learners, formed in the order the schedule fixes: within the ring of dimension t the partial sum of part k
 * starts at ring position k+1 and is extended by positions k+2, ..., k+d_t (= k).
 * Bindings: the kernels read absolute addresses from a per-plan table bound to one buffer
 * set ("binding slot").  A call whose P pointers equal those of an existing slot uses it as
 * it is; any other call binds a slot first with one more small kernel on `stream` (a free
 * slot, else a new one, else -- with DDL_PLAN_MAX_BINDINGS slots in existence -- the least
 * recently used).  The plan's own tables are read-only, so one plan serves any number of
 * streams and host threads at once as long as concurrent calls use different buffer sets
 * (they must anyway: the operation is in place) and no more than DDL_PLAN_MAX_BINDINGS
 * sets are in flight; beyond that number a slot may be rebound while enqueued work of
 * another stream still reads it, which the caller must then order.  Slots allocate device
 * memory when they are created; see ddl_plan_prepare for callers that must avoid that.
 * A call under stream capture records its own binding kernel into the caller's graph and
 * keeps its slot for the plan's lifetime (replays of that graph stay valid whatever runs in
 * between); if the plan's tables do not exist yet (ddl_plan_prepare), or no slot is free and
 * none can be created, it returns DDL_ERR_UNSUPPORTED.
 * Errors are reported before anything is enqueued, except DDL_ERR_HIP for a failed launch.
 */
ddl_status_t ddl_allreduce_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                               ddl_dtype_t dtype, void* stream);

/*
 * ddl_allreduce_sim for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result
 * (bit for bit) and errors as ddl_allreduce_sim, but nothing is allocated, freed or copied
 * from the host, not even at the plan's first use: the per-call operation records are
 * computed on the device from the box and kept in a static device array of
 * DDL_NOALLOC_MAX_OPS records (32 bytes each, 512 KiB, held by every GPU the library has
 * run on until the process ends) instead of the plan's device tables.  The only set-up is
 * the lookup of that array's address at the first call on a device (ddl_plan_prepare does
 * it too, so call that before a capture).  Always runs phase by phase.
 * Limits, beyond which it returns DDL_ERR_UNSUPPORTED and enqueues nothing: P <= 256,
 * phases * P <= DDL_NOALLOC_MAX_OPS, plans of ddl_ring_plan only (one tensor).
 * All calls on one GPU share the array (each call rewrites the records it uses, nothing
 * needs clearing): calls whose execution may overlap on one GPU -- different streams, or
 * another thread -- race; order them.  ddl_allreduce_sim has no such restriction.
 */
#define DDL_NOALLOC_MAX_OPS 16384
ddl_status_t ddl_allreduce_sim_noalloc(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                       ddl_dtype_t dtype, void* stream);

/*
 * The two halves as operations of their own (Sec. 4.1 ReduceScatter, AllGather); same
 * arguments and rules as ddl_allreduce_sim.
 * After ddl_reduce_scatter_sim learner r holds the completed sum on its own finest chunk
 * (ddl_plan_owned_chunk) and partial sums elsewhere.  ddl_allgather_sim copies every
 * learner's finest chunk into all learners and leaves the rest of the phases' ranges
 * overwritten the same way.
 */
ddl_status_t ddl_reduce_scatter_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                    ddl_dtype_t dtype, void* stream);
ddl_status_t ddl_allgather_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                               ddl_dtype_t dtype, void* stream);

/*
 * ddl_allreduce_sim with a HIP event recorded on `stream` before and after every step's
 * kernel.  SYNCHRONISES the stream before returning.  step_ms (host, ddl_plan_num_steps
 * floats) receives each step's elapsed milliseconds (0 for a step that moves nothing).
 * Meant for measurement; the events add a little time between kernels.
 */
ddl_status_t ddl_allreduce_sim_profile(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                       ddl_dtype_t dtype, void* stream, float* step_ms);

/*
 * ddl_allreduce_sim with only three HIP events on `stream`: before the first reduce-scatter
 * step, between the halves, after the last all-gather step.  SYNCHRONISES the stream.
 * *reduce_ms / *gather_ms (host, either may be NULL) receive the elapsed milliseconds of
 * each half, kernel-to-kernel gaps included; dividing by the number of steps of that kind
 * gives the average launch duration of the reduce-add resp. copy kernel.
 */
ddl_status_t ddl_allreduce_sim_timed(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                     ddl_dtype_t dtype, void* stream, float* reduce_ms,
                                     float* gather_ms);

/*
 * Assignment (Sec. 4.1: the elementary operation of the library, one object receives a copy of another):
 * dst[0 .. count) <- src[0 .. count), both DEVICE pointers, 16-byte aligned, not
 * overlapping, with the copy kernel of the all-gather phases.  Needs no plan.  Enqueued on
 * `stream`, does not synchronise.  DDL_ERR_ARG for NULL or overlapping ranges (count > 0),
 * DDL_ERR_ALIGN, DDL_ERR_DTYPE, DDL_ERR_HIP.
 */
ddl_status_t ddl_assign_sim(void* dst, const void* src, size_t count, ddl_dtype_t dtype, void* stream);

/*
 * Step-fused allreduce: the same final state as ddl_allreduce_sim (every learner holds the
 * sum, bit for bit the value the schedule's summation order gives) produced in ONE pass
 * that reads every learner's element once, folds the ring orders of all dimensions in
 * registers and writes the result to every learner, instead of executing the phases one
 * by one.  The partial sums the phases would have left in the buffers on the way are never
 * materialised.  Memory traffic is 2 * sizeof(element) * count * P bytes instead of
 * ddl_plan_bytes_moved; from 16 learners on the work is split into a reducing pass (result
 * to the chunk's owner) and a distributing pass, which adds one write and one read of the
 * result (ddl_plan_fused_bytes gives the exact figure).
 * Same arguments, rules and errors as ddl_allreduce_sim; additionally
 * DDL_ERR_UNSUPPORTED if P > DDL_FUSED_MAX_LEARNERS or the box has more than
 * DDL_FUSED_MAX_LEVELS dimensions of size > 1 (use ddl_allreduce_sim then).
 */
#define DDL_FUSED_MAX_LEARNERS 1024
#define DDL_FUSED_MAX_LEVELS 4
ddl_status_t ddl_allreduce_fused_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                     ddl_dtype_t dtype, void* stream);

/*
 * The two passes of the step-fused form as operations of their own (Sec. 4.1 ReduceScatter
 * and AllGather, each in one kernel pass); same arguments, limits and errors as
 * ddl_allreduce_fused_sim.
 * ddl_reduce_scatter_fused_sim: learner r's finest chunk (ddl_plan_owned_chunk) receives the
 * sum over all learners in the schedule's summation order; nothing else is written (unlike
 * ddl_reduce_scatter_sim, which leaves the phases' partial sums in the other chunks).
 * ddl_allgather_fused_sim: every learner's finest chunk is copied into all other learners.
 * One after the other they give exactly ddl_allreduce_sim's final state.
 */
ddl_status_t ddl_reduce_scatter_fused_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                          ddl_dtype_t dtype, void* stream);
ddl_status_t ddl_allgather_fused_sim(void** bufs, int P, const ddl_plan_t* plan, size_t count,
                                     ddl_dtype_t dtype, void* stream);

/* ---- plan introspection (host only) ------------------------------------------------ */

/*
 * Self-check of a plan's schedule on the host (no GPU): every operation lies inside its
 * tensor on 16-byte granules; in every phase each learner sends one operation and receives
 * one, from its ring neighbour of that phase's dimension (Sec. 4.3: N concurrent transfers
 * per phase); the range a learner receives never overlaps the range it sends in the same
 * phase, so the transfers of a phase are free of races whatever their order; the learners'
 * finest chunks tile every tensor; ring-walk rows follow their rings.  DDL_OK, or
 * DDL_ERR_ARG for a NULL or inconsistent plan.  Cost: O(phases x tensors x P).
 */
ddl_status_t ddl_plan_verify(const ddl_plan_t* plan);

/* 2 * sum_t (d_t - 1): Sec. 4.3, d-1 phases per ring, once reducing and once gathering.
 * Returns -1 for a NULL plan. */
int ddl_plan_num_steps(const ddl_plan_t* plan);

/* Learners P of the plan (0 for NULL). */
int ddl_plan_num_learners(const ddl_plan_t* plan);

/* Bytes the whole schedule moves through memory: 3 accesses per element of a reduce
 * operation (read src, read dst, write dst), 2 per element of a gather operation.
 * Equals 5 * sizeof(element) * count * (P - 1) when count is a multiple of G * P. */
size_t ddl_plan_bytes_moved(const ddl_plan_t* plan);

/* Bytes ddl_allreduce_fused_sim moves: every element of every learner read once and
 * written once, plus one write and read of the result when it runs as two passes. */
size_t ddl_plan_fused_bytes(const ddl_plan_t* plan);

/* Bytes the ring-walk form of the whole allreduce moves (see ddl_plan_set_walk): per dimension
 * of ring size d and element of its segment 2d-1 accesses reducing and d gathering, 2d in all
 * for the last dimension.  0 for a plan without it. */
size_t ddl_plan_walk_bytes(const ddl_plan_t* plan);

/* ddl_plan_bytes_moved for one step; 0 for a bad index. */
size_t ddl_plan_step_bytes(const ddl_plan_t* plan, int step);

/*
 * Describe step `step` (0-based).  *kind = DDL_STEP_REDUCE / DDL_STEP_GATHER, *dim = the
 * 0-based box dimension whose rings run; src/dst/off/n are caller arrays of
 * P * ddl_plan_num_tensors entries (any may be NULL), filled tensor by tensor and, within a
 * tensor, in order of the sending learner: operation i reads [off[i], off[i]+n[i]) of
 * learner src[i] = i mod P and targets the same range of dst[i].
 */
ddl_status_t ddl_plan_get_step(const ddl_plan_t* plan, int step, int* kind, int* dim,
                               int* src, int* dst, size_t* off, size_t* n);

/* The finest chunk learner `learner` owns after the reduce-scatter: [*off, *off + *n)
 * (of tensor 0 for a several-tensor plan). */
ddl_status_t ddl_plan_owned_chunk(const ddl_plan_t* plan, int learner, size_t* off, size_t* n);

/* Tensors of the plan: 1 for ddl_ring_plan, num_tensors for ddl_ring_plan_tensors, 0 for NULL. */
int ddl_plan_num_tensors(const ddl_plan_t* plan);

/* The finest chunk of tensor `tensor` that `learner` owns, offset relative to the buffer. */
ddl_status_t ddl_plan_owned_chunk_tensor(const ddl_plan_t* plan, int tensor, int learner, size_t* off,
                                         size_t* n);

/*
 * Estimated time on a cluster, seconds (Sec. 4.3: T ~ sum_{j=1}^{d-1} (S/(d*B) + L) per
 * ring): dimension t runs a ring of d_t nodes over the bytes left at its level with
 * bandwidth bw[t] (bytes/s) and per-phase latency lat[t] (s); charged once for the
 * reduction and once for the distribution.  bw, lat: host arrays of m doubles.
 * Returns a negative value on bad arguments.
 */
double ddl_plan_model_time(const ddl_plan_t* plan, const double* bw, const double* lat);

/*
 * Choose the box for P learners with `bytes` per learner over m levels of links
 * (Sec. 4.3: the dimensions are adjusted to the bandwidth and latency of the links so that
 * the fastest links carry the most and the slowest link does not dominate).
 *   bw[t], lat[t]  bandwidth (bytes/s) and per-phase latency (s) of dimension t
 *   max_dim        NULL, or m caps on d_t (0 = no cap), e.g. the GPUs of one node for t = 0
 * Every tuple (d_1..d_m) with d_t >= 1, product P and d_t <= max_dim[t] is scored with the
 * estimate of ddl_plan_model_time; the smallest wins, exact ties go to the tuple that is
 * smallest in lexicographic order.  dims_out: m ints; *time_out (may be NULL) the estimate.
 * Host only.  DDL_ERR_DIMS if no tuple fits the caps, DDL_ERR_ARG for bad arguments.
 */
ddl_status_t ddl_choose_dims(int P, size_t bytes, int m, const double* bw, const double* lat,
                             const int* max_dim, int* dims_out, double* time_out);

/* Memory clock (kHz) and bus width (bits) of the current device as the HIP runtime reports
 * them, for stating the bandwidth peak next to a measurement.  DDL_ERR_HIP without a device. */
ddl_status_t ddl_device_memory_info(int* clock_khz, int* bus_bits);

/* Static, human-readable name of a status code. */
const char* ddl_status_string(ddl_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* DDLSIM_H */
