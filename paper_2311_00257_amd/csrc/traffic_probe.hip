// Traffic-only kernels in the fused step's exact access shape, for the benchmark's "ceilings": what the
// memory system gives that shape with the arithmetic taken out.  Not part of libamsp.so and not on
// the product path: bench.py times them next to the product kernel, in the same process.
//
// Shape (that of adamw_kernel on its vector path): one-wave workgroups, one launch covering the range
// once in address order, lane L of block b owning elements 256 b + 4 L .. + 3 of every stream: 8-byte
// loads of the k bf16 partials, 16-byte loads of the three fp32 state streams, all issued before
// anything waits; 16-byte stores of the three fp32 streams and an 8-byte store of the bf16 output; the
// non-temporal hint on every access; at most `waves_per_cu` waves resident per CU (an unused slice of
// LDS per workgroup imposes the cap).
//   mode 0  reads only   (2k + 12 bytes per element)
//   mode 1  writes only  (14 bytes per element)
//   mode 2  both         (2k + 26 bytes per element); the fp32 streams are written back unchanged
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kMaxK = 32;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct Streams {
    const uint16_t *g[kMaxK];
    float *p, *m, *v;
    uint16_t *out;
    uint32_t never;   // always 0: keeps the loads of mode 0 alive without a store ever happening
};

template <typename T>
__device__ __forceinline__ T ldnt(const T *p) { return __builtin_nontemporal_load(p); }
template <typename T>
__device__ __forceinline__ void stnt(T *p, T v) { __builtin_nontemporal_store(v, p); }

template <int K, int MODE>
__global__ void __launch_bounds__(64) traffic_kernel(Streams a) {
    const uint64_t e = ((uint64_t)blockIdx.x * 64 + threadIdx.x) * 4;   // the grid covers exactly n / 256 blocks
    f32x4 p = {1.f, 2.f, 3.f, 4.f}, m = p, v = p;
    uint32_t acc = threadIdx.x;
    if constexpr (MODE != 1) {
        p = ldnt(reinterpret_cast<const f32x4 *>(a.p + e));
        m = ldnt(reinterpret_cast<const f32x4 *>(a.m + e));
        v = ldnt(reinterpret_cast<const f32x4 *>(a.v + e));
        u32x2 w[K];
#pragma unroll
        for (int j = 0; j < K; ++j) w[j] = ldnt(reinterpret_cast<const u32x2 *>(a.g[j] + e));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);   // every load in flight before the first wait
#pragma unroll
        for (int j = 0; j < K; ++j) acc ^= w[j].x ^ w[j].y;
    }
    if constexpr (MODE != 0) {
        stnt(reinterpret_cast<f32x4 *>(a.p + e), p);
        stnt(reinterpret_cast<f32x4 *>(a.m + e), m);
        stnt(reinterpret_cast<f32x4 *>(a.v + e), v);
        const u32x2 o = {acc, acc};
        stnt(reinterpret_cast<u32x2 *>(a.out + e), o);
    } else {
        const uint32_t all = acc ^ __float_as_uint(p.x + p.y + p.z + p.w) ^ __float_as_uint(m.x + m.y + m.z + m.w) ^
                             __float_as_uint(v.x + v.y + v.z + v.w);
        if (a.never != 0 && all == 0x12345678u) a.out[e] = (uint16_t)all;
    }
}

template <int K>
int launch_k(int mode, const Streams &a, unsigned blocks, unsigned lds, hipStream_t hs) {
    switch (mode) {
        case 0: hipLaunchKernelGGL((traffic_kernel<K, 0>), dim3(blocks), dim3(64), lds, hs, a); break;
        case 1: hipLaunchKernelGGL((traffic_kernel<K, 1>), dim3(blocks), dim3(64), lds, hs, a); break;
        case 2: hipLaunchKernelGGL((traffic_kernel<K, 2>), dim3(blocks), dim3(64), lds, hs, a); break;
        default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // namespace

extern "C" {

// partials: host array of k device pointers (bf16[n]); p, m, v: device fp32[n]; out: device bf16[n];
// every device pointer 1 KiB-aligned; n a multiple of 256 and below 2^31 * 256; k in 1..16;
// waves_per_cu in 3..32.  Returns 0, -1 (bad argument) or -2 (launch error).  Modes 1 and 2 overwrite
// `out`; mode 1 also overwrites p, m and v.
int amsp_probe_traffic(int mode, const uint16_t *const *partials, uint32_t k, float *p, float *m, float *v,
                       uint16_t *out, uint64_t n, int waves_per_cu, void *stream) {
    if (k < 1 || k > 16 || partials == nullptr || p == nullptr || m == nullptr || v == nullptr || out == nullptr) return -1;
    if (n == 0 || (n & 255) != 0 || (n >> 8) >= (1ull << 31) || waves_per_cu < 3 || waves_per_cu > 32) return -1;
    Streams a{};
    uintptr_t bits = (uintptr_t)p | (uintptr_t)m | (uintptr_t)v | (uintptr_t)out;
    for (uint32_t j = 0; j < k; ++j) {
        if (partials[j] == nullptr) return -1;
        a.g[j] = partials[j];
        bits |= (uintptr_t)partials[j];
    }
    if ((bits & 1023) != 0) return -1;
    a.p = p; a.m = m; a.v = v; a.out = out; a.never = 0;
    const unsigned blocks = (unsigned)(n >> 8);
    const unsigned lds = waves_per_cu >= 32 ? 0u : (unsigned)((160 * 1024 / waves_per_cu) & ~255);
    hipStream_t hs = (hipStream_t)stream;
    (void)hipGetLastError();
    switch (k) {
#define AMSP_PROBE_CASE(KV) case KV: return launch_k<KV>(mode, a, blocks, lds, hs);
        AMSP_PROBE_CASE(1) AMSP_PROBE_CASE(2) AMSP_PROBE_CASE(3) AMSP_PROBE_CASE(4) AMSP_PROBE_CASE(5) AMSP_PROBE_CASE(6)
        AMSP_PROBE_CASE(7) AMSP_PROBE_CASE(8) AMSP_PROBE_CASE(9) AMSP_PROBE_CASE(10) AMSP_PROBE_CASE(11)
        AMSP_PROBE_CASE(12) AMSP_PROBE_CASE(13) AMSP_PROBE_CASE(14) AMSP_PROBE_CASE(15) AMSP_PROBE_CASE(16)
#undef AMSP_PROBE_CASE
        default: return -1;
    }
}

}  // extern "C"
