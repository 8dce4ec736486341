// Counter-based input generator (declared in include/ddlgen.h): one definition of the
// value function, compiled for the host loop and for the device kernel.
#include <hip/hip_runtime.h>

#include <cmath>

#include "../../include/ddlgen.h"

namespace {

constexpr uint64_t kPhi = 0x9E3779B97F4A7C15ull;

// SplitMix64 output function (Steele, Lea, Flood 2014; constants of Vigna's reference)
__host__ __device__ inline uint64_t mix(uint64_t x) {
    uint64_t z = x + kPhi;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__host__ __device__ inline uint64_t learner_key(uint64_t seed, uint32_t learner) {
    return mix(seed + kPhi * (uint64_t(learner) + 1));
}

__host__ __device__ inline int32_t draw(uint64_t key, uint64_t e, int dist) {
    const uint64_t h0 = mix(key + 2 * e);
    if (dist == DDLGEN_INT8) return int32_t((h0 >> 32) % 17) - 8;
    if (dist == DDLGEN_UNIFORM) return int32_t(h0 >> 40) - (1 << 23);
    const uint64_t h1 = mix(key + 2 * e + 1);
    int32_t s = 0;
    for (int i = 0; i < 4; ++i) {
        s += int32_t((h0 >> (16 * i)) & 0xFFFF);
        s += int32_t((h1 >> (16 * i)) & 0xFFFF);
    }
    return s - 262140;  // 8 * 65535 / 2
}

float scale_of(int dist) {
    if (dist == DDLGEN_INT8) return 1.0f;
    if (dist == DDLGEN_UNIFORM) return 1.0f / 8388608.0f;
    return float(0.01 / std::sqrt(8.0 * (4294967296.0 - 1.0) / 12.0));
}

__global__ __launch_bounds__(256) void fill_kernel(float* __restrict__ out, uint64_t n,
                                                   uint64_t key, uint64_t first, int dist,
                                                   float scale) {
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
        out[i] = __fmul_rn(float(draw(key, first + i, dist)), scale);
}

bool known(int dist) { return dist == DDLGEN_INT8 || dist == DDLGEN_UNIFORM || dist == DDLGEN_NORMAL; }

}  // namespace

extern "C" {

int ddlgen_fill_host(float* out, size_t n, uint64_t seed, uint32_t learner, size_t first, int dist) {
    if (!known(dist) || (out == nullptr && n > 0)) return -1;
    const uint64_t key = learner_key(seed, learner);
    const float scale = scale_of(dist);
    for (size_t i = 0; i < n; ++i) {
        const float q = float(draw(key, first + i, dist));
        out[i] = q * scale;
    }
    return 0;
}

int ddlgen_fill_device(void* d_out, size_t n, uint64_t seed, uint32_t learner, size_t first,
                       int dist, void* stream) {
    if (!known(dist) || (d_out == nullptr && n > 0)) return -1;
    if (n == 0) return 0;
    const uint64_t key = learner_key(seed, learner);
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_kernel, dim3(unsigned(blocks)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<float*>(d_out), uint64_t(n),
                       key, uint64_t(first), dist, scale_of(dist));
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"
