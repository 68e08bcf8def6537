// Device side of the seeded synthetic-input generator: fills model-state buffers with the
// same bits the host generator (synth.py) produces, so 100 GB of state never crosses PCIe.
// Input production only; no arithmetic of the training step lives here.
//
// Element i of a stream with key K:  z = K + i * GOLDEN;  h = SplitMix64 output function of z;
// value = table[h >> 48] * sigma (fp32), optionally fabs; bf16 streams keep the high 16 bits
// of that fp32 pattern.  `table` is the 65,536-entry fp32 normal-quantile table, uploaded by
// the caller.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ float draw(uint64_t key, uint64_t index, const float *table, float sigma) {
    uint64_t h = mix64(key + index * 0x9E3779B97F4A7C15ull);
    return table[h >> 48] * sigma;
}

__global__ void fill_f32_kernel(float *out, uint64_t n, uint64_t key, uint64_t index0, const float *table,
                                float sigma, int absolute) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float x = draw(key, index0 + i, table, sigma);
        out[i] = absolute ? fabsf(x) : x;
    }
}

__global__ void fill_bf16_kernel(uint16_t *out, uint64_t n, uint64_t key, uint64_t index0, const float *table,
                                 float sigma) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        out[i] = (uint16_t)(__float_as_uint(draw(key, index0 + i, table, sigma)) >> 16);
}

int grid_for(uint64_t n) {
    uint64_t b = (n + 255) / 256;
    return (int)(b < 1 ? 1 : (b > 8192 ? 8192 : b));
}

}  // namespace

extern "C" {

// out: device fp32[n]; table: device fp32[65536]; returns 0 or -1 (HIP launch error).
int amsp_synth_fill_f32(float *out, uint64_t n, uint64_t key, uint64_t index0, const float *table, float sigma,
                        int absolute, void *stream) {
    if (n == 0) return 0;
    if (!out || !table) return -1;
    hipLaunchKernelGGL(fill_f32_kernel, dim3(grid_for(n)), dim3(256), 0, (hipStream_t)stream, out, n, key, index0,
                       table, sigma, absolute);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// out: device bf16[n] as uint16 patterns.
int amsp_synth_fill_bf16(uint16_t *out, uint64_t n, uint64_t key, uint64_t index0, const float *table, float sigma,
                         void *stream) {
    if (n == 0) return 0;
    if (!out || !table) return -1;
    hipLaunchKernelGGL(fill_bf16_kernel, dim3(grid_for(n)), dim3(256), 0, (hipStream_t)stream, out, n, key, index0,
                       table, sigma);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
