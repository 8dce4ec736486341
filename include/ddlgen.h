/*
 * libddlgen -- seeded, counter-based generator of synthetic gradient buffers.
 *
 * Serves both sides of the parity tests: the same (seed, learner, element index) gives the
 * same fp32 bits from the host routine and from the device kernel, so neither the CPU
 * oracle nor the HIP library ever has to ship a buffer to the other.  It contains none of
 * the allreduce's arithmetic.
 *
 * Value of element e of learner j:  two 64-bit words
 *     h0 = mix(key + 2e), h1 = mix(key + 2e + 1),  key = mix(seed + PHI * (j + 1)),
 * where mix(x) is the SplitMix64 output function applied to x + PHI (PHI = 0x9E3779B97F4A7C15),
 * are turned into an integer q, and the value is float(q) * scale with a single fp32
 * multiply (exact for the first two distributions):
 *   DDLGEN_INT8     q = (h0 >> 32) mod 17 - 8,                scale = 1      -> integers in [-8, 8]
 *   DDLGEN_UNIFORM  q = (h0 >> 40) - 2^23,                    scale = 2^-23  -> uniform on [-1, 1)
 *   DDLGEN_NORMAL   q = (sum of the eight 16-bit fields of h0, h1) - 262140,
 *                   scale = float(0.01 / sqrt(8 * (2^32 - 1) / 12))          -> approx. N(0, 0.01^2)
 */
#ifndef DDLGEN_H
#define DDLGEN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DDLGEN_INT8 = 0, DDLGEN_UNIFORM = 1, DDLGEN_NORMAL = 2 } ddlgen_dist_t;

/*
 * Write elements first .. first+n-1 of learner `learner` to out[0 .. n-1] (HOST memory,
 * caller-owned).  Returns 0, or -1 for a NULL pointer with n > 0 or an unknown dist.
 */
int ddlgen_fill_host(float* out, size_t n, uint64_t seed, uint32_t learner, size_t first, int dist);

/*
 * The same into DEVICE memory d_out (4-byte aligned, caller-owned), enqueued on the
 * hipStream_t `stream` (NULL = default stream); does not synchronise.  Returns 0, -1 for
 * bad arguments, -2 if the launch failed.
 */
int ddlgen_fill_device(void* d_out, size_t n, uint64_t seed, uint32_t learner, size_t first,
                       int dist, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DDLGEN_H */
