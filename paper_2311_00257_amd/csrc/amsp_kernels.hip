// HIP kernels (gfx950) and C ABI of the per-GPU model-state step: k-way bf16 gradient
// reduction, squared gradient norm, fused AdamW on fp32 master/m/v, bf16 parameter cast.
//
// Everything here is an HBM stream with a handful of fp32 operations per element, so the
// design is about memory traffic only: every lane moves 8 consecutive elements per stream
// per iteration (one 128-bit access per bf16 stream, two per fp32 stream), a wave covers
// 1 KiB (bf16) / 2 KiB (fp32) of contiguous memory per access, blocks walk the range with a
// grid stride, and nothing is staged through LDS except the block-level sum of the norm.
// No matrix cores: there is no contraction on this path.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include "amsp.h"

#ifndef AMSP_NT_LOAD
#define AMSP_NT_LOAD 1   // non-temporal hint on loads of streams that are read once
#endif
#ifndef AMSP_NT_STORE
#define AMSP_NT_STORE 1  // non-temporal hint on stores
#endif

namespace {

constexpr int kThreads = 256;          // 4 waves of 64
constexpr int kVec = 8;                // elements per lane per iteration
constexpr int kMaxBlocks = 4096;       // upper bound on any grid here; sizes the norm workspace
constexpr int kEdgeMax = 2 * (kVec - 1);

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct PartialPtrs {
    const uint16_t *p[AMSP_MAX_K];
};

// ---------------------------------------------------------------- memory access helpers
template <typename T>
__device__ __forceinline__ T ld_stream(const T *p) {
#if AMSP_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename T>
__device__ __forceinline__ void st_stream(T *p, T v) {
#if AMSP_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

__device__ __forceinline__ void ld8_f32(const float *base, uint64_t e, float (&x)[kVec]) {
    const f32x4 *q = reinterpret_cast<const f32x4 *>(base + e);
    f32x4 a = ld_stream(q), b = ld_stream(q + 1);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ __forceinline__ void st8_f32(float *base, uint64_t e, const float (&x)[kVec]) {
    f32x4 *q = reinterpret_cast<f32x4 *>(base + e);
    f32x4 a = {x[0], x[1], x[2], x[3]}, b = {x[4], x[5], x[6], x[7]};
    st_stream(q, a);
    st_stream(q + 1, b);
}

// bf16 -> fp32 is a 16-bit shift of the pattern (exact).
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_one(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even on the pattern; NaN -> 0x7FC0 | sign.
__device__ __forceinline__ uint32_t f32_to_bf16(float x) {
    uint32_t u = __float_as_uint(x);
    uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    uint32_t qnan = ((u >> 16) & 0x8000u) | 0x7FC0u;
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? qnan : rounded;
}
__device__ __forceinline__ void st8_bf16(uint16_t *base, uint64_t e, const float (&x)[kVec]) {
    u32x4 w;
    w.x = f32_to_bf16(x[0]) | (f32_to_bf16(x[1]) << 16);
    w.y = f32_to_bf16(x[2]) | (f32_to_bf16(x[3]) << 16);
    w.z = f32_to_bf16(x[4]) | (f32_to_bf16(x[5]) << 16);
    w.w = f32_to_bf16(x[6]) | (f32_to_bf16(x[7]) << 16);
    st_stream(reinterpret_cast<u32x4 *>(base + e), w);
}

// ---------------------------------------------------------------- the reduced gradient
// K > 0: k == K known at compile time (all loads issued up front); K == -1: run-time k;
// K == 0: the gradient is already reduced, read it as fp32.
// The sum runs j = 0..k-1 in fp32 in every kernel, so all of them see the same bits.
template <int K>
__device__ __forceinline__ void grad8(const PartialPtrs &pp, int k, const float *gf32, uint64_t e,
                                      float (&g)[kVec]) {
    if constexpr (K == 0) {
        ld8_f32(gf32, e, g);
    } else if constexpr (K > 0) {
        u32x4 w[K];
#pragma unroll
        for (int j = 0; j < K; ++j) w[j] = ld_stream(reinterpret_cast<const u32x4 *>(pp.p[j] + e));
        g[0] = bf16_lo(w[0].x); g[1] = bf16_hi(w[0].x); g[2] = bf16_lo(w[0].y); g[3] = bf16_hi(w[0].y);
        g[4] = bf16_lo(w[0].z); g[5] = bf16_hi(w[0].z); g[6] = bf16_lo(w[0].w); g[7] = bf16_hi(w[0].w);
#pragma unroll
        for (int j = 1; j < K; ++j) {
            g[0] += bf16_lo(w[j].x); g[1] += bf16_hi(w[j].x); g[2] += bf16_lo(w[j].y); g[3] += bf16_hi(w[j].y);
            g[4] += bf16_lo(w[j].z); g[5] += bf16_hi(w[j].z); g[6] += bf16_lo(w[j].w); g[7] += bf16_hi(w[j].w);
        }
    } else {
        u32x4 w = ld_stream(reinterpret_cast<const u32x4 *>(pp.p[0] + e));
        g[0] = bf16_lo(w.x); g[1] = bf16_hi(w.x); g[2] = bf16_lo(w.y); g[3] = bf16_hi(w.y);
        g[4] = bf16_lo(w.z); g[5] = bf16_hi(w.z); g[6] = bf16_lo(w.w); g[7] = bf16_hi(w.w);
#pragma unroll 4
        for (int j = 1; j < k; ++j) {
            w = ld_stream(reinterpret_cast<const u32x4 *>(pp.p[j] + e));
            g[0] += bf16_lo(w.x); g[1] += bf16_hi(w.x); g[2] += bf16_lo(w.y); g[3] += bf16_hi(w.y);
            g[4] += bf16_lo(w.z); g[5] += bf16_hi(w.z); g[6] += bf16_lo(w.w); g[7] += bf16_hi(w.w);
        }
    }
}

// One element, any alignment: the same sum in the same order.
template <int K>
__device__ __forceinline__ float grad1(const PartialPtrs &pp, int k, const float *gf32, uint64_t i) {
    if constexpr (K == 0) {
        return gf32[i];
    } else {
        float g = bf16_one(pp.p[0][i]);
        const int kk = K > 0 ? K : k;
        for (int j = 1; j < kk; ++j) g += bf16_one(pp.p[j][i]);
        return g;
    }
}

// A launch covers n elements: `head` leading ones (0..7) up to the common 16-byte phase of
// all streams, nvec groups of 8 taken with 128-bit accesses, and a tail of < 8.  Head and
// tail (at most 14 elements) are the "edge", done element-wise by block 0.  When the
// streams have no common phase the host sets nvec = 0 and vectorised = 0 and every element
// goes through the element-wise loop.
struct Span {
    uint64_t n;
    uint64_t nvec;
    uint32_t head;
    uint32_t vectorised;
};

__device__ __forceinline__ bool edge_index(const Span &s, uint32_t t, uint64_t &i) {
    // t-th edge element -> element index
    if (t < s.head) { i = t; return true; }
    uint64_t j = (uint64_t)s.head + s.nvec * kVec + (t - s.head);
    if (j < s.n) { i = j; return true; }
    return false;
}

// ---------------------------------------------------------------- step 4: cast
__global__ void __launch_bounds__(kThreads) cast_kernel(const float *__restrict__ master,
                                                        uint16_t *__restrict__ out, Span s) {
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    if (s.vectorised) {
        for (uint64_t v = (uint64_t)blockIdx.x * kThreads + threadIdx.x; v < s.nvec; v += stride) {
            const uint64_t e = s.head + v * kVec;
            float x[kVec];
            ld8_f32(master, e, x);
            st8_bf16(out, e, x);
        }
        uint64_t i;
        if (blockIdx.x == 0 && threadIdx.x < kEdgeMax && edge_index(s, threadIdx.x, i))
            out[i] = (uint16_t)f32_to_bf16(master[i]);
    } else {
        for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < s.n; i += stride)
            out[i] = (uint16_t)f32_to_bf16(master[i]);
    }
}

// ---------------------------------------------------------------- step 1: reduce
template <int K>
__global__ void __launch_bounds__(kThreads) reduce_kernel(PartialPtrs pp, int k, float *__restrict__ out,
                                                          int accumulate, Span s) {
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    if (s.vectorised) {
        for (uint64_t v = (uint64_t)blockIdx.x * kThreads + threadIdx.x; v < s.nvec; v += stride) {
            const uint64_t e = s.head + v * kVec;
            float g[kVec];
            grad8<K>(pp, k, nullptr, e, g);
            if (accumulate) {
                float o[kVec];
                ld8_f32(out, e, o);
#pragma unroll
                for (int c = 0; c < kVec; ++c) g[c] = o[c] + g[c];
            }
            st8_f32(out, e, g);
        }
        uint64_t i;
        if (blockIdx.x == 0 && threadIdx.x < kEdgeMax && edge_index(s, threadIdx.x, i)) {
            float g = grad1<K>(pp, k, nullptr, i);
            out[i] = accumulate ? out[i] + g : g;
        }
    } else {
        for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < s.n; i += stride) {
            float g = grad1<K>(pp, k, nullptr, i);
            out[i] = accumulate ? out[i] + g : g;
        }
    }
}

// ---------------------------------------------------------------- step 2: squared norm
// Every lane accumulates g^2 in fp64 over a fixed set of elements, lanes are summed by a
// shuffle tree, waves through LDS, and each block stores one double.  A second one-block
// kernel adds the block sums in index order.  No atomics, so the result depends only on
// (n, alignment, grid size), never on timing.
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    return x;
}

template <int K>
__global__ void __launch_bounds__(kThreads) sqnorm_kernel(PartialPtrs pp, int k, const float *__restrict__ gf32,
                                                          double *__restrict__ block_sums, Span s) {
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    double acc = 0.0;
    if (s.vectorised) {
        for (uint64_t v = (uint64_t)blockIdx.x * kThreads + threadIdx.x; v < s.nvec; v += stride) {
            float g[kVec];
            grad8<K>(pp, k, gf32, s.head + v * kVec, g);
#pragma unroll
            for (int c = 0; c < kVec; ++c) acc = fma((double)g[c], (double)g[c], acc);
        }
        uint64_t i;
        if (blockIdx.x == 0 && threadIdx.x < kEdgeMax && edge_index(s, threadIdx.x, i)) {
            double g = (double)grad1<K>(pp, k, gf32, i);
            acc = fma(g, g, acc);
        }
    } else {
        for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < s.n; i += stride) {
            double g = (double)grad1<K>(pp, k, gf32, i);
            acc = fma(g, g, acc);
        }
    }
    __shared__ double wave_part[kThreads / 64];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = wave_part[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) t += wave_part[w];
        block_sums[blockIdx.x] = t;
    }
}

__global__ void __launch_bounds__(kThreads) sqnorm_finish_kernel(const double *__restrict__ block_sums, int nblocks,
                                                                 double *__restrict__ out, int accumulate) {
    __shared__ double part[kThreads];
    double t = 0.0;
    for (int b = threadIdx.x; b < nblocks; b += kThreads) t += block_sums[b];
    part[threadIdx.x] = t;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = accumulate ? *out + part[0] : part[0];
}

// ---------------------------------------------------------------- step 3 (+1, +4): AdamW
struct AdamConsts {
    float lr, beta1, beta2, eps, wd;
    float one_minus_beta1, one_minus_beta2;   // rounded from double
    float rbc1, rbc2;                         // 1/(1-beta^t), computed in double on the host
    float max_norm, clip_eps, grad_scale;
    const double *d_total_sqnorm;
};

__device__ __forceinline__ float clip_scale(const AdamConsts &c) {
    double s = (double)c.grad_scale;
    if (c.d_total_sqnorm != nullptr && c.max_norm > 0.0f) {
        double clip = (double)c.max_norm / (sqrt(*c.d_total_sqnorm) + (double)c.clip_eps);
        s *= clip < 1.0 ? clip : 1.0;
    }
    return (float)s;
}

// fp32 throughout, fused multiply-adds spelled out so that every kernel rounds alike.
__device__ __forceinline__ void adamw1(const AdamConsts &c, float scale, float g, float &p, float &m, float &v) {
    const float gs = scale * g;
    m = fmaf(c.beta1, m, c.one_minus_beta1 * gs);
    v = fmaf(c.beta2, v, (c.one_minus_beta2 * gs) * gs);
    const float denom = sqrtf(v * c.rbc2) + c.eps;
    const float u = (m * c.rbc1) / denom;
    p = fmaf(-c.lr, fmaf(c.wd, p, u), p);
}

template <int K, bool WRITE_BF16>
__global__ void __launch_bounds__(kThreads) adamw_kernel(PartialPtrs pp, int k, const float *__restrict__ gf32,
                                                         float *__restrict__ master, float *__restrict__ exp_avg,
                                                         float *__restrict__ exp_avg_sq, uint16_t *__restrict__ out,
                                                         AdamConsts c, Span s) {
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    const float scale = clip_scale(c);
    if (s.vectorised) {
        for (uint64_t vi = (uint64_t)blockIdx.x * kThreads + threadIdx.x; vi < s.nvec; vi += stride) {
            const uint64_t e = s.head + vi * kVec;
            float g[kVec], p[kVec], m[kVec], v[kVec];
            grad8<K>(pp, k, gf32, e, g);
            ld8_f32(master, e, p);
            ld8_f32(exp_avg, e, m);
            ld8_f32(exp_avg_sq, e, v);
#pragma unroll
            for (int q = 0; q < kVec; ++q) adamw1(c, scale, g[q], p[q], m[q], v[q]);
            st8_f32(master, e, p);
            st8_f32(exp_avg, e, m);
            st8_f32(exp_avg_sq, e, v);
            if constexpr (WRITE_BF16) st8_bf16(out, e, p);
        }
    }
    const bool edge = s.vectorised != 0;
    if (edge && blockIdx.x != 0) return;
    const uint64_t first = edge ? threadIdx.x : (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    const uint64_t count = edge ? kEdgeMax : s.n;
    for (uint64_t t = first; t < count; t += edge ? (uint64_t)kThreads : stride) {
        uint64_t i = t;
        if (edge && !edge_index(s, (uint32_t)t, i)) continue;
        float p = master[i], m = exp_avg[i], v = exp_avg_sq[i];
        adamw1(c, scale, grad1<K>(pp, k, gf32, i), p, m, v);
        master[i] = p;
        exp_avg[i] = m;
        exp_avg_sq[i] = v;
        if constexpr (WRITE_BF16) out[i] = (uint16_t)f32_to_bf16(p);
    }
}

// ---------------------------------------------------------------- host side
struct Stream16 {
    const void *ptr;
    uint32_t elem;   // bytes per element: 2 or 4
};

// Smallest head in 0..7 at which every stream is 16-byte aligned, or -1.
int common_head(const Stream16 *st, int ns) {
    for (int h = 0; h < kVec; ++h) {
        bool ok = true;
        for (int i = 0; i < ns && ok; ++i) ok = ((reinterpret_cast<uintptr_t>(st[i].ptr) + (uintptr_t)h * st[i].elem) & 15u) == 0;
        if (ok) return h;
    }
    return -1;
}

Span make_span(uint64_t n, const Stream16 *st, int ns) {
    Span s{n, 0, 0, 0};
    int h = common_head(st, ns);
    if (h >= 0 && n >= (uint64_t)h + kVec) {
        s.head = (uint32_t)h;
        s.nvec = (n - (uint64_t)h) / kVec;
        s.vectorised = 1;
    }
    return s;
}

int blocks_per_cu() {
    static int v = [] {
        const char *e = getenv("AMSP_BLOCKS_PER_CU");
        int x = e ? atoi(e) : 0;
        return (x >= 1 && x <= 16) ? x : 8;
    }();
    return v;
}

int cu_count() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

int grid_for(const Span &s) {
    uint64_t work = s.vectorised ? s.nvec : s.n;
    uint64_t blocks = (work + kThreads - 1) / kThreads;
    uint64_t cap = (uint64_t)cu_count() * blocks_per_cu();
    if (cap > kMaxBlocks) cap = kMaxBlocks;
    if (blocks > cap) blocks = cap;
    return blocks == 0 ? 1 : (int)blocks;
}

bool misaligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_partials(const uint16_t *const *partials, uint32_t k, PartialPtrs &pp) {
    if (k == 0 || k > AMSP_MAX_K) return AMSP_EINVAL;
    if (partials == nullptr) return AMSP_ENULL;
    for (uint32_t j = 0; j < k; ++j) {
        if (partials[j] == nullptr) return AMSP_ENULL;
        if (misaligned(partials[j], 2)) return AMSP_EALIGN;
        pp.p[j] = partials[j];
    }
    for (uint32_t j = k; j < AMSP_MAX_K; ++j) pp.p[j] = nullptr;
    return AMSP_OK;
}

inline int launched() { return hipGetLastError() == hipSuccess ? AMSP_OK : AMSP_EDEVICE; }

// Calls f(offset, length) for each bucket of [0,n).
template <typename F>
int for_buckets(uint64_t n, uint64_t bucket_elems, F f) {
    if (bucket_elems == 0 || bucket_elems >= n) return f((uint64_t)0, n);
    for (uint64_t off = 0; off < n; off += bucket_elems) {
        uint64_t len = n - off < bucket_elems ? n - off : bucket_elems;
        int rc = f(off, len);
        if (rc != AMSP_OK) return rc;
    }
    return AMSP_OK;
}

PartialPtrs offset_partials(const PartialPtrs &pp, uint32_t k, uint64_t off) {
    PartialPtrs q = pp;
    for (uint32_t j = 0; j < k; ++j) q.p[j] = pp.p[j] + off;
    return q;
}

int add_partial_streams(Stream16 *st, int ns, const PartialPtrs &pp, uint32_t k) {
    for (uint32_t j = 0; j < k; ++j) st[ns++] = Stream16{pp.p[j], 2};
    return ns;
}

#define AMSP_DISPATCH_K(k, CALL)                 \
    switch (k) {                                 \
        case 1: { constexpr int KK = 1; CALL; } break;   \
        case 2: { constexpr int KK = 2; CALL; } break;   \
        case 4: { constexpr int KK = 4; CALL; } break;   \
        case 8: { constexpr int KK = 8; CALL; } break;   \
        case 16: { constexpr int KK = 16; CALL; } break; \
        default: { constexpr int KK = -1; CALL; } break; \
    }

}  // namespace

// ================================================================ C ABI
extern "C" {

const char *amsp_status_string(int status) {
    switch (status) {
        case AMSP_OK: return "ok";
        case AMSP_EINVAL: return "invalid argument (k, shard factor, rank or hyper-parameter)";
        case AMSP_ENULL: return "required pointer is NULL";
        case AMSP_EALIGN: return "pointer not aligned to its element size";
        case AMSP_EWORKSPACE: return "workspace too small";
        case AMSP_EDEVICE: return "HIP call failed";
        default: return "unknown status";
    }
}

size_t amsp_workspace_bytes(void) { return (size_t)kMaxBlocks * sizeof(double); }

int amsp_shard_range(uint64_t total_elems, uint32_t shard_factor, uint32_t rank, uint64_t *begin, uint64_t *end) {
    if (begin == nullptr || end == nullptr) return AMSP_ENULL;
    if (shard_factor == 0 || rank >= shard_factor) return AMSP_EINVAL;
    const uint64_t q = total_elems / shard_factor, r = total_elems % shard_factor;
    const uint64_t b = q * rank + (rank < r ? rank : r);
    *begin = b;
    *end = b + q + (rank < r ? 1 : 0);
    return AMSP_OK;
}

int amsp_cast_param_shard(const float *master, uint16_t *param_bf16_out, uint64_t n, void *stream) {
    if (n == 0) return AMSP_OK;
    if (master == nullptr || param_bf16_out == nullptr) return AMSP_ENULL;
    if (misaligned(master, 4) || misaligned(param_bf16_out, 2)) return AMSP_EALIGN;
    Stream16 st[2] = {{master, 4}, {param_bf16_out, 2}};
    Span s = make_span(n, st, 2);
    hipLaunchKernelGGL(cast_kernel, dim3(grid_for(s)), dim3(kThreads), 0, (hipStream_t)stream, master, param_bf16_out, s);
    return launched();
}

int amsp_reduce_grad_shard(const uint16_t *const *partials, uint32_t k, uint64_t n, uint64_t bucket_elems,
                           float *grad_out, int accumulate, void *stream) {
    PartialPtrs pp;
    int rc = check_partials(partials, k, pp);
    if (rc != AMSP_OK) return rc;
    if (n == 0) return AMSP_OK;
    if (grad_out == nullptr) return AMSP_ENULL;
    if (misaligned(grad_out, 4)) return AMSP_EALIGN;
    return for_buckets(n, bucket_elems, [&](uint64_t off, uint64_t len) {
        PartialPtrs q = offset_partials(pp, k, off);
        Stream16 st[AMSP_MAX_K + 1];
        int ns = add_partial_streams(st, 0, q, k);
        st[ns++] = Stream16{grad_out + off, 4};
        Span s = make_span(len, st, ns);
        AMSP_DISPATCH_K(k, hipLaunchKernelGGL(reduce_kernel<KK>, dim3(grid_for(s)), dim3(kThreads), 0,
                                              (hipStream_t)stream, q, (int)k, grad_out + off, accumulate, s));
        return launched();
    });
}

int amsp_grad_sqnorm(const uint16_t *const *partials, uint32_t k, const float *grad_f32, uint64_t n,
                     uint64_t bucket_elems, double *d_sqnorm, int accumulate, void *workspace,
                     size_t workspace_bytes, void *stream) {
    PartialPtrs pp{};
    if (k > 0) {
        int rc = check_partials(partials, k, pp);
        if (rc != AMSP_OK) return rc;
    } else if (n > 0) {
        if (grad_f32 == nullptr) return AMSP_ENULL;
        if (misaligned(grad_f32, 4)) return AMSP_EALIGN;
    }
    if (d_sqnorm == nullptr || workspace == nullptr) return AMSP_ENULL;
    if (misaligned(d_sqnorm, 8) || misaligned(workspace, 8)) return AMSP_EALIGN;
    if (workspace_bytes < amsp_workspace_bytes()) return AMSP_EWORKSPACE;
    double *block_sums = static_cast<double *>(workspace);
    hipStream_t hs = (hipStream_t)stream;
    if (n == 0) {
        if (!accumulate) {
            hipLaunchKernelGGL(sqnorm_finish_kernel, dim3(1), dim3(kThreads), 0, hs, block_sums, 0, d_sqnorm, 0);
            return launched();
        }
        return AMSP_OK;
    }
    bool first = true;
    return for_buckets(n, bucket_elems, [&](uint64_t off, uint64_t len) {
        PartialPtrs q = offset_partials(pp, k, off);
        Stream16 st[AMSP_MAX_K + 1];
        int ns = add_partial_streams(st, 0, q, k);
        const float *gf = nullptr;
        if (k == 0) {
            gf = grad_f32 + off;
            st[ns++] = Stream16{gf, 4};
        }
        Span s = make_span(len, st, ns);
        const int grid = grid_for(s);
        if (k == 0) {
            hipLaunchKernelGGL(sqnorm_kernel<0>, dim3(grid), dim3(kThreads), 0, hs, q, 0, gf, block_sums, s);
        } else {
            AMSP_DISPATCH_K(k, hipLaunchKernelGGL(sqnorm_kernel<KK>, dim3(grid), dim3(kThreads), 0, hs, q, (int)k,
                                                  gf, block_sums, s));
        }
        if (launched() != AMSP_OK) return (int)AMSP_EDEVICE;
        const int acc = (accumulate || !first) ? 1 : 0;
        first = false;
        hipLaunchKernelGGL(sqnorm_finish_kernel, dim3(1), dim3(kThreads), 0, hs, block_sums, grid, d_sqnorm, acc);
        return launched();
    });
}

int amsp_adamw_step_shard(const uint16_t *const *partials, uint32_t k, const float *grad_f32, uint64_t n,
                          uint64_t bucket_elems, float *master, float *exp_avg, float *exp_avg_sq,
                          uint16_t *param_bf16_out, const amsp_adamw_hparams *hp, void *stream) {
    if (hp == nullptr) return AMSP_ENULL;
    PartialPtrs pp{};
    if (k > 0) {
        int rc = check_partials(partials, k, pp);
        if (rc != AMSP_OK) return rc;
    }
    const bool finite = isfinite(hp->lr) && isfinite(hp->beta1) && isfinite(hp->beta2) && isfinite(hp->eps) &&
                        isfinite(hp->weight_decay) && isfinite(hp->grad_scale) && isfinite(hp->clip_eps) &&
                        !isnan(hp->max_norm);
    if (!finite || hp->step == 0 || !(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) ||
        !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f) || hp->eps < 0.0f)
        return AMSP_EINVAL;
    if (n == 0) return AMSP_OK;
    if (master == nullptr || exp_avg == nullptr || exp_avg_sq == nullptr) return AMSP_ENULL;
    if (k == 0 && grad_f32 == nullptr) return AMSP_ENULL;
    if (misaligned(master, 4) || misaligned(exp_avg, 4) || misaligned(exp_avg_sq, 4) ||
        (k == 0 && misaligned(grad_f32, 4)) || (param_bf16_out && misaligned(param_bf16_out, 2)) ||
        (hp->d_total_sqnorm && misaligned(hp->d_total_sqnorm, 8)))
        return AMSP_EALIGN;

    AdamConsts c;
    c.lr = hp->lr; c.beta1 = hp->beta1; c.beta2 = hp->beta2; c.eps = hp->eps; c.wd = hp->weight_decay;
    c.one_minus_beta1 = (float)(1.0 - (double)hp->beta1);
    c.one_minus_beta2 = (float)(1.0 - (double)hp->beta2);
    c.rbc1 = (float)(1.0 / (1.0 - pow((double)hp->beta1, (double)hp->step)));
    c.rbc2 = (float)(1.0 / (1.0 - pow((double)hp->beta2, (double)hp->step)));
    c.max_norm = hp->max_norm; c.clip_eps = hp->clip_eps; c.grad_scale = hp->grad_scale;
    c.d_total_sqnorm = hp->d_total_sqnorm;
    hipStream_t hs = (hipStream_t)stream;

    return for_buckets(n, bucket_elems, [&](uint64_t off, uint64_t len) {
        PartialPtrs q = offset_partials(pp, k, off);
        Stream16 st[AMSP_MAX_K + 5];
        int ns = add_partial_streams(st, 0, q, k);
        const float *gf = nullptr;
        if (k == 0) {
            gf = grad_f32 + off;
            st[ns++] = Stream16{gf, 4};
        }
        st[ns++] = Stream16{master + off, 4};
        st[ns++] = Stream16{exp_avg + off, 4};
        st[ns++] = Stream16{exp_avg_sq + off, 4};
        uint16_t *out = param_bf16_out ? param_bf16_out + off : nullptr;
        if (out) st[ns++] = Stream16{out, 2};
        Span s = make_span(len, st, ns);
        const dim3 grid(grid_for(s)), block(kThreads);
#define AMSP_LAUNCH_ADAMW(KV)                                                                              \
        if (out) hipLaunchKernelGGL((adamw_kernel<KV, true>), grid, block, 0, hs, q, (int)k, gf, master + off, \
                                    exp_avg + off, exp_avg_sq + off, out, c, s);                            \
        else hipLaunchKernelGGL((adamw_kernel<KV, false>), grid, block, 0, hs, q, (int)k, gf, master + off,  \
                                exp_avg + off, exp_avg_sq + off, out, c, s)
        if (k == 0) {
            AMSP_LAUNCH_ADAMW(0);
        } else {
            AMSP_DISPATCH_K(k, AMSP_LAUNCH_ADAMW(KK));
        }
#undef AMSP_LAUNCH_ADAMW
        return launched();
    });
}

}  // extern "C"
