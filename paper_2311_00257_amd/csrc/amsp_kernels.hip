// HIP kernels (gfx950) and C ABI of the per-GPU model-state step: k-way bf16 gradient
// reduction, squared gradient norm, fused AdamW on fp32 master/m/v, bf16 parameter cast.
//
// Everything here is an HBM stream with a handful of fp32 operations per element, so the
// design is about memory traffic only.  What measurement on MI355X settled:
//   - Every access of a wave is one fully contiguous piece: in the kernels that write, a lane
//     owns 4 consecutive elements per stream (8-byte bf16 and 16-byte fp32 accesses, so a wave
//     instruction covers 512 B or 1 KiB without gaps).  Letting a lane own 8 elements makes
//     its fp32 accesses two 16-byte pieces 32 bytes apart and costs 10-20 % of bandwidth.
//   - Kernels that read AND write are straight-line code, one vector per lane, on a grid that
//     covers the whole range once: the hardware dispatcher hands out the range in address order
//     and balances the CUs.  The same body as a persistent grid-stride loop reaches ~4.5 TB/s
//     instead of ~5.8 TB/s on the k = 8 fused step.
//   - Those kernels run one-wave (64-thread) workgroups under an occupancy cap: only as many
//     waves per CU as keep ~40 KiB of loads in flight, at least 8 (8 for k = 8, where the hardware
//     would take 32); the reduction 64 KiB and at least 12.  That brings the k = 8 fused step from
//     ~5.8 to 6.4-6.5 TB/s.  The cap is an unused slice of LDS per workgroup.  With so few waves,
//     nothing may stand between a wave's start and its loads: no blockDim/gridDim (a
//     dispatch-packet fetch), the clip scale worked out after the loads are in flight, and a
//     scheduling barrier that keeps all k + 3 loads ahead of the first wait.
//   - The head peeled off a misaligned range brings every stream to a multiple of what a wave
//     takes from it per access (512 B of bf16, 1 KiB of fp32): a wave's piece aligned to its own
//     size.  Pieces that are only line-aligned cost 4-5 %, pieces that straddle lines ~20 %.
//   - The read-only norm pass is the opposite case: a persistent grid of exactly the resident
//     size (two 1024-thread blocks per CU) with a grid-stride loop and 16-byte loads reads at
//     6.6-6.9 TB/s, more than any full-grid or 256-thread variant, and its per-block sums fit a
//     small fixed workspace, summed in a fixed order.
//   - Launches are shared: the buckets of a call, and the short segments of an inter-tensor shard
//     (32 to a launch, the table in the kernel arguments), so that neither many buckets nor many
//     small tensors make the step launch-bound.
//   - Non-temporal hints on all loads and stores: nothing is reused.
// Nothing is staged through LDS except the block-level sum of the norm.  No matrix cores:
// there is no contraction on this path.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <atomic>

#include "amsp.h"
#include "amsp_geometry.h"

#ifndef AMSP_NT_LOAD
#define AMSP_NT_LOAD 1   // non-temporal hint on loads
#endif
#ifndef AMSP_NT_STORE
#define AMSP_NT_STORE 1  // non-temporal hint on stores
#endif

namespace {

constexpr int kThreads = 256;          // helper kernels (finishing sums, fills): 4 waves of 64
constexpr int kRwThreads = 64;         // the kernels that read and write run one-wave workgroups
constexpr int kVecRW = 4;              // elements per lane per stream in the kernels that write
constexpr int kVecNorm = 8;            // elements per lane per stream in the norm pass
constexpr int kNormThreads = 1024;     // the norm pass runs 16-wave blocks, two per CU
constexpr int kNormBlocks = 2048;      // upper bound of the norm pass's grid; sizes its workspace
constexpr uint64_t kMaxGrid = (1ull << 31) - 1;

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
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

// VEC consecutive fp32 values as VEC/4 16-byte accesses.
template <int VEC>
__device__ __forceinline__ void ld_f32(const float *base, uint64_t e, float (&x)[VEC]) {
    const f32x4 *q = reinterpret_cast<const f32x4 *>(base + e);
#pragma unroll
    for (int h = 0; h < VEC / 4; ++h) {
        f32x4 a = ld_stream(q + h);
        x[4 * h] = a.x; x[4 * h + 1] = a.y; x[4 * h + 2] = a.z; x[4 * h + 3] = a.w;
    }
}
template <int VEC>
__device__ __forceinline__ void st_f32(float *base, uint64_t e, const float (&x)[VEC]) {
    f32x4 *q = reinterpret_cast<f32x4 *>(base + e);
#pragma unroll
    for (int h = 0; h < VEC / 4; ++h) {
        f32x4 a = {x[4 * h], x[4 * h + 1], x[4 * h + 2], x[4 * h + 3]};
        st_stream(q + h, a);
    }
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

// VEC consecutive bf16 values as one 8- or 16-byte access: VEC/2 packed words.
template <int VEC> struct Bf16Words;
template <> struct Bf16Words<4> { typedef u32x2 type; };
template <> struct Bf16Words<8> { typedef u32x4 type; };

template <int VEC>
__device__ __forceinline__ void st_bf16(uint16_t *base, uint64_t e, const float (&x)[VEC]) {
    typename Bf16Words<VEC>::type w;
#pragma unroll
    for (int c = 0; c < VEC / 2; ++c) w[c] = f32_to_bf16(x[2 * c]) | (f32_to_bf16(x[2 * c + 1]) << 16);
    st_stream(reinterpret_cast<typename Bf16Words<VEC>::type *>(base + e), w);
}

// ---------------------------------------------------------------- the reduced gradient
// K > 0: k == K known at compile time (all loads issued up front); K == -1: run-time k;
// K == 0: the gradient is already reduced, read it as fp32.
// The sum runs j = 0..k-1 in fp32 in every kernel, so all of them see the same bits.
template <int VEC, typename W>
__device__ __forceinline__ void widen_first(const W &w, float (&g)[VEC]) {
#pragma unroll
    for (int c = 0; c < VEC / 2; ++c) { g[2 * c] = bf16_lo(w[c]); g[2 * c + 1] = bf16_hi(w[c]); }
}
template <int VEC, typename W>
__device__ __forceinline__ void widen_add(const W &w, float (&g)[VEC]) {
#pragma unroll
    for (int c = 0; c < VEC / 2; ++c) { g[2 * c] += bf16_lo(w[c]); g[2 * c + 1] += bf16_hi(w[c]); }
}

// Keeps the compiler from sinking loads below this point: everything loaded so far is in flight
// before any arithmetic that waits on part of it.
__device__ __forceinline__ void loads_issued() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);   // nothing may be scheduled across: arithmetic stays below the loads
}

template <int K, int VEC>
__device__ __forceinline__ void grad_vec(const PartialPtrs &pp, int k, const float *gf32, uint64_t e,
                                         float (&g)[VEC]) {
    typedef typename Bf16Words<VEC>::type W;
    if constexpr (K == 0) {
        ld_f32<VEC>(gf32, e, g);
        loads_issued();
    } else if constexpr (K > 0) {
        W w[K];
#pragma unroll
        for (int j = 0; j < K; ++j) w[j] = ld_stream(reinterpret_cast<const W *>(pp.p[j] + e));
        loads_issued();
        widen_first<VEC>(w[0], g);
#pragma unroll
        for (int j = 1; j < K; ++j) widen_add<VEC>(w[j], g);
    } else {
        W w = ld_stream(reinterpret_cast<const W *>(pp.p[0] + e));
        loads_issued();
        widen_first<VEC>(w, g);
#pragma unroll 4
        for (int j = 1; j < k; ++j) {
            w = ld_stream(reinterpret_cast<const W *>(pp.p[j] + e));
            widen_add<VEC>(w, g);
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

using amsp_geom::Span;
using amsp_geom::Buckets;
static_assert(kRwThreads == amsp_geom::kWaveLanes, "the geometry assumes one-wave workgroups on the vector path");

// Element index of the t-th edge element, t < head + tail.
template <int VEC>
__device__ __forceinline__ uint64_t edge_elem(const Span &s, uint32_t t) {
    return amsp_geom::edge_elem(s, t, VEC);
}

// The range this block works on (a launch per 25 M-element bucket would also do, but buckets of one
// call share launches; see the geometry header).
template <int VEC>
__device__ __forceinline__ void block_range(const Buckets &bk, Span &s, uint64_t &off, uint32_t &local_block) {
    amsp_geom::block_range(bk, blockIdx.x, VEC, s, off, local_block);
}

// The read+write kernels are straight-line code: the grid covers the range exactly once, with
// one-wave workgroups (one vector per lane) on the vector path and 256-thread workgroups (one
// element per lane) on the element-wise path.  Nothing in them asks for blockDim or gridDim: those
// live in the dispatch packet, and fetching them would put one more memory round trip in front of
// the wave's loads.
__device__ __forceinline__ uint64_t vector_index() { return (uint64_t)blockIdx.x * kRwThreads + threadIdx.x; }
__device__ __forceinline__ uint64_t element_index() { return (uint64_t)blockIdx.x * kThreads + threadIdx.x; }

// ---------------------------------------------------------------- step 4: cast
__global__ void __launch_bounds__(kThreads) cast_kernel(const float *__restrict__ master,
                                                        uint16_t *__restrict__ out, Span s) {
    constexpr int VEC = kVecRW;
    if (s.vectorised) {
        const uint64_t v = vector_index();
        if (v < s.nvec) {
            const uint64_t e = s.head + v * VEC;
            float x[VEC];
            ld_f32<VEC>(master, e, x);
            st_bf16<VEC>(out, e, x);
        }
        if (blockIdx.x == 0)
            for (uint32_t t = threadIdx.x; t < s.head + s.tail; t += kRwThreads) {
                const uint64_t i = edge_elem<VEC>(s, t);
                out[i] = (uint16_t)f32_to_bf16(master[i]);
            }
    } else {
        const uint64_t i = element_index();
        if (i < s.n) out[i] = (uint16_t)f32_to_bf16(master[i]);
    }
}

// ---------------------------------------------------------------- block-level fp64 sums
// Lanes are summed by a shuffle tree, waves through LDS, in a fixed order; thread 0 gets the sum.
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    return x;
}

template <int THREADS>
__device__ __forceinline__ double block_sum(double acc) {
    __shared__ double wave_part[THREADS / 64];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0) {
        t = wave_part[0];
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) t += wave_part[w];   // THREADS bounds blockDim.x
    }
    return t;
}

// ---------------------------------------------------------------- step 1: reduce
// NORM: also sum the squares of the values written, one double per block into block_sums
// (step 2 fused into step 1 for callers that keep the fp32 gradient): one per 256 elements on the
// vector path (a one-wave block), a capped number on the element-wise path.
template <int K, bool NORM>
__global__ void __launch_bounds__(kThreads) reduce_kernel(PartialPtrs pp, int k, float *__restrict__ out,
                                                          int accumulate, double *__restrict__ block_sums, Span s,
                                                          Buckets bk) {
    constexpr int VEC = kVecRW;
    double acc = 0.0;
    if (s.vectorised) {
        uint64_t off;
        uint32_t lb;
        block_range<VEC>(bk, s, off, lb);
        const uint64_t v = (uint64_t)lb * kRwThreads + threadIdx.x;
        if (v < s.nvec) {
            const uint64_t e = off + s.head + v * VEC;
            float g[VEC], o[VEC];
            if (accumulate) ld_f32<VEC>(out, e, o);   // issued ahead of the partial loads
            grad_vec<K, VEC>(pp, k, nullptr, e, g);
            if (accumulate) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) g[c] = o[c] + g[c];
            }
            st_f32<VEC>(out, e, g);
            if constexpr (NORM) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc = fma((double)g[c], (double)g[c], acc);
            }
        }
        if (lb == 0)
            for (uint32_t t = threadIdx.x; t < s.head + s.tail; t += kRwThreads) {
                const uint64_t i = off + edge_elem<VEC>(s, t);
                float g1 = grad1<K>(pp, k, nullptr, i);
                if (accumulate) g1 = out[i] + g1;
                out[i] = g1;
                if constexpr (NORM) acc = fma((double)g1, (double)g1, acc);
            }
        if constexpr (NORM) {
            acc = wave_sum(acc);   // the block is one wave
            if (threadIdx.x == 0) block_sums[blockIdx.x] = acc;
        }
    } else {
        // element-wise path: with the norm the grid is capped (a fixed number of block sums), so loop
        const uint64_t stride = NORM ? (uint64_t)gridDim.x * kThreads : ~0ull;
        for (uint64_t i = element_index(); i < s.n; i += stride) {
            float g1 = grad1<K>(pp, k, nullptr, i);
            if (accumulate) g1 = out[i] + g1;
            out[i] = g1;
            if constexpr (NORM) acc = fma((double)g1, (double)g1, acc);
            if constexpr (!NORM) break;
        }
        if constexpr (NORM) {
            const double t = block_sum<kThreads>(acc);
            if (threadIdx.x == 0) block_sums[blockIdx.x] = t;
        }
    }
}

// ---------------------------------------------------------------- step 2: squared norm
// Every lane accumulates g^2 in fp64 over a fixed set of elements, lanes are summed by a
// shuffle tree, waves through LDS, and each block stores one double.  A second one-block
// kernel adds the block sums in index order.  No atomics, so the result depends only on
// (n, alignment, grid size), never on timing.
// One launch covers up to kMaxNormSegs ranges (buckets of a flat range, or the segments of an
// inter-tensor shard), each with its own head and tail: a read-only pass gains nothing from a launch per
// range, and short launches lose 10-30 % to their start and end.
constexpr int kMaxNormSegs = 32;
struct NormSeg {
    uint64_t base;   // first element of the range, relative to the stream pointers
    Span s;
};
struct NormSegTable {
    int count;
    NormSeg seg[kMaxNormSegs];
};

// acc += sum of g^2 over one range: this lane's share of the vectors, a grid stride apart.
template <int K, int VEC>
__device__ __forceinline__ double sqnorm_span(const PartialPtrs &pp, int k, const float *__restrict__ gf32,
                                              const uint64_t base, const Span &s, const uint64_t first,
                                              const uint64_t stride, double acc) {
    if (s.vectorised) {
        uint64_t v = first;
        // With one or two streams a single vector per lane leaves too little in flight: take U vectors,
        // a grid stride apart, per trip, all their loads issued before the first is used.
        constexpr int U = (K == 0 || K == 1) ? 4 : (K == 2 ? 2 : 1);
        if constexpr (U > 1) {
            constexpr int KS = K == 0 ? 1 : K;
            typedef typename Bf16Words<VEC == 8 ? 8 : 4>::type W;
            for (; v + (U - 1) * stride < s.nvec; v += U * stride) {
                f32x4 a[U];
                W w[U][KS];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint64_t e = base + s.head + (v + u * stride) * VEC;
                    if constexpr (K == 0) {
                        a[u] = ld_stream(reinterpret_cast<const f32x4 *>(gf32 + e));
                    } else {
#pragma unroll
                        for (int j = 0; j < KS; ++j) w[u][j] = ld_stream(reinterpret_cast<const W *>(pp.p[j] + e));
                    }
                }
                loads_issued();
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float g[VEC];
                    if constexpr (K == 0) {
                        g[0] = a[u].x; g[1] = a[u].y; g[2] = a[u].z; g[3] = a[u].w;
                    } else {
                        widen_first<VEC>(w[u][0], g);
#pragma unroll
                        for (int j = 1; j < KS; ++j) widen_add<VEC>(w[u][j], g);
                    }
#pragma unroll
                    for (int c = 0; c < VEC; ++c) acc = fma((double)g[c], (double)g[c], acc);
                }
            }
        }
        for (; v < s.nvec; v += stride) {
            float g[VEC];
            grad_vec<K, VEC>(pp, k, gf32, base + s.head + v * VEC, g);
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc = fma((double)g[c], (double)g[c], acc);
        }
        if (blockIdx.x == 0)
            for (uint32_t t = threadIdx.x; t < s.head + s.tail; t += kNormThreads) {
                const double g = (double)grad1<K>(pp, k, gf32, base + edge_elem<VEC>(s, t));
                acc = fma(g, g, acc);
            }
    } else {
        for (uint64_t i = first; i < s.n; i += stride) {
            double g = (double)grad1<K>(pp, k, gf32, base + i);
            acc = fma(g, g, acc);
        }
    }
    return acc;
}

template <int K, int VEC>
__global__ void __launch_bounds__(kNormThreads) sqnorm_kernel(PartialPtrs pp, int k, const float *__restrict__ gf32,
                                                              double *__restrict__ block_sums, NormSegTable t) {
    const uint64_t first = (uint64_t)blockIdx.x * kNormThreads + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * kNormThreads;
    double acc = 0.0;
    for (int i = 0; i < t.count; ++i) acc = sqnorm_span<K, VEC>(pp, k, gf32, t.seg[i].base, t.seg[i].s, first, stride, acc);
    const double total = block_sum<kNormThreads>(acc);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// Short ranges (norm gains, biases, small buckets): in the kernel above every block walks every
// range, so a range shorter than the grid leaves most blocks idle while the few that have work go
// through the ranges one memory round trip after the other.  Here each range gets blocks of its own,
// one vector per lane (a grid-stride loop on the element-wise path), and a block finds its range with
// 31 scalar compares against the table in the kernel arguments.  Run-time k: short ranges hold a
// sliver of the bytes.
struct ShortNormTable {
    uint32_t first_block[kMaxNormSegs];   // unused entries: 0xFFFFFFFF
    uint32_t blocks[kMaxNormSegs];
    NormSeg seg[kMaxNormSegs];
};

template <int K, int VEC>
__global__ void __launch_bounds__(kNormThreads) sqnorm_short_kernel(PartialPtrs pp, int k,
                                                                    const float *__restrict__ gf32,
                                                                    double *__restrict__ block_sums,
                                                                    ShortNormTable t) {
    uint32_t r = 0;
#pragma unroll
    for (int i = 1; i < kMaxNormSegs; ++i) r += blockIdx.x >= t.first_block[i] ? 1u : 0u;
    const uint32_t lb = blockIdx.x - t.first_block[r];
    const Span s = t.seg[r].s;
    const uint64_t base = t.seg[r].base;
    double acc = 0.0;
    if (s.vectorised) {
        const uint64_t v = (uint64_t)lb * kNormThreads + threadIdx.x;
        if (v < s.nvec) {
            float g[VEC];
            grad_vec<K, VEC>(pp, k, gf32, base + s.head + v * VEC, g);
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc = fma((double)g[c], (double)g[c], acc);
        }
        if (lb == 0)
            for (uint32_t e = threadIdx.x; e < s.head + s.tail; e += kNormThreads) {
                const double g = (double)grad1<K>(pp, k, gf32, base + edge_elem<VEC>(s, e));
                acc = fma(g, g, acc);
            }
    } else {
        const uint64_t stride = (uint64_t)t.blocks[r] * kNormThreads;
        for (uint64_t i = (uint64_t)lb * kNormThreads + threadIdx.x; i < s.n; i += stride) {
            const double g = (double)grad1<K>(pp, k, gf32, base + i);
            acc = fma(g, g, acc);
        }
    }
    const double total = block_sum<kNormThreads>(acc);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// Adds nblocks block sums in a fixed order (lane-strided, then a tree) and stores or adds the total.
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

// First stage for long lists of block sums: block f adds the slice [f*slice, (f+1)*slice).
__global__ void __launch_bounds__(kThreads) sum_slices_kernel(const double *__restrict__ block_sums, uint64_t count,
                                                              uint64_t slice, double *__restrict__ slice_sums) {
    const uint64_t lo = blockIdx.x * slice;
    const uint64_t hi = lo + slice < count ? lo + slice : count;
    double t = 0.0;
    for (uint64_t b = lo + threadIdx.x; b < hi; b += kThreads) t += block_sums[b];
    t = block_sum<kThreads>(t);
    if (threadIdx.x == 0) slice_sums[blockIdx.x] = t;
}

// ---------------------------------------------------------------- step 3 (+1, +4): AdamW
struct AdamConsts {
    float lr, beta1, beta2, eps, wd;
    float one_minus_beta1, one_minus_beta2;   // rounded from double
    float rbc1, rbc2;                         // 1/(1-beta^t), computed in double on the host
    float max_norm, clip_eps, grad_scale;
    const double *d_total_sqnorm;
};

// The squared norm is fetched first (an ordinary cached load of one address, which overlaps everything
// after it); the scale is worked out from it later, in double, once the wave's vector loads are in
// flight.  (Fetched with a device-coherent load instead, it costs 1-3 %: it misses the caches, and the
// in-order return of vector loads puts its latency in front of the first partial.)
__device__ __forceinline__ double load_sqnorm(const AdamConsts &c) {
    return (c.d_total_sqnorm != nullptr && c.max_norm > 0.0f) ? *c.d_total_sqnorm : -1.0;
}
__device__ __forceinline__ float clip_scale(const AdamConsts &c, double sqnorm) {
    double s = (double)c.grad_scale;
    if (sqnorm >= 0.0) {
        double clip = (double)c.max_norm / (sqrt(sqnorm) + (double)c.clip_eps);
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

// |x| as an ordered integer: for non-negative floats the bit patterns order like the values, with
// Inf above every finite value and NaN patterns above Inf, so an integer max is exact,
// order-independent and lets a NaN win.
__device__ __forceinline__ uint32_t abs_bits(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

// Per-segment maxima of |p'| taken inside the update.  An atomic on one word costs ~11 ns and is
// serialised in its memory channel, so the waves of a launch spread over kAmaxSubSlots words that lie
// kAmaxStrideWords apart (different channels), and a wave sends an atomic only when it beats what its
// word held when the wave started: the word only grows, so that early read (device-coherent: an
// ordinary cached read returns stale values and half of the waves would still send) filters out all
// but the record holders.  It is issued with the wave's first loads, so its latency is hidden.
constexpr int kAmaxSubSlots = 64;
constexpr int kAmaxStrideWords = 64;   // 256 bytes
constexpr size_t kAmaxWordsPerSegment = (size_t)kAmaxSubSlots * kAmaxStrideWords;

__device__ __forceinline__ uint32_t *amax_word(uint32_t *segment_words) {
    return segment_words + (blockIdx.x & (kAmaxSubSlots - 1)) * kAmaxStrideWords;
}
__device__ __forceinline__ uint32_t amax_seen(uint32_t *segment_words) {
    return __hip_atomic_load(amax_word(segment_words), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wave_amax_into(uint32_t m, uint32_t seen, uint32_t *segment_words) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_down((int)m, off, 64));
    if ((threadIdx.x & 63) == 0 && m > seen) atomicMax(amax_word(segment_words), m);
}

// d_amax[i] = the largest of segment i's words, as a float.
__global__ void __launch_bounds__(kAmaxSubSlots) amax_fold_kernel(const uint32_t *__restrict__ words,
                                                                 uint32_t *__restrict__ d_amax) {
    uint32_t m = words[(size_t)blockIdx.x * kAmaxWordsPerSegment + threadIdx.x * kAmaxStrideWords];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_down((int)m, off, 64));
    if (threadIdx.x == 0) d_amax[blockIdx.x] = m;
}

template <int K, bool WRITE_BF16, bool AMAX>
__global__ void __launch_bounds__(kThreads) adamw_kernel(PartialPtrs pp, int k, const float *__restrict__ gf32,
                                                         float *__restrict__ master, float *__restrict__ exp_avg,
                                                         float *__restrict__ exp_avg_sq, uint16_t *__restrict__ out,
                                                         uint32_t *__restrict__ amax, AdamConsts c, Span s,
                                                         Buckets bk) {
    constexpr int VEC = kVecRW;
    // Every kernel argument the common path needs is fetched before the squared norm is: scalar loads
    // return out of order, so a later wait for an argument would also wait for that value.
    const uint64_t bucket_elems = bk.bucket_elems;
    asm volatile("" ::"s"(bucket_elems), "s"(s.nvec), "s"(s.head));
    const double sqnorm = load_sqnorm(c);
    uint32_t seen = 0;
    if constexpr (AMAX) seen = amax_seen(amax);
    uint32_t biggest = 0;   // of |p'| over this lane's elements, with AMAX
    if (s.vectorised) {
        uint64_t off;
        uint32_t lb;
        block_range<VEC>(bk, s, off, lb);
        const uint64_t vi = (uint64_t)lb * kRwThreads + threadIdx.x;
        if (vi < s.nvec) {
            const uint64_t e = off + s.head + vi * VEC;
            float g[VEC], p[VEC], m[VEC], v[VEC];
            // every load of the vector is in flight before anything waits: one memory round trip
            ld_f32<VEC>(master, e, p);
            ld_f32<VEC>(exp_avg, e, m);
            ld_f32<VEC>(exp_avg_sq, e, v);
            grad_vec<K, VEC>(pp, k, gf32, e, g);
            const float scale = clip_scale(c, sqnorm);
#pragma unroll
            for (int q = 0; q < VEC; ++q) adamw1(c, scale, g[q], p[q], m[q], v[q]);
            st_f32<VEC>(master, e, p);
            st_f32<VEC>(exp_avg, e, m);
            st_f32<VEC>(exp_avg_sq, e, v);
            if constexpr (WRITE_BF16) st_bf16<VEC>(out, e, p);
            if constexpr (AMAX) {
#pragma unroll
                for (int q = 0; q < VEC; ++q) biggest = max(biggest, abs_bits(p[q]));
            }
        }
        if (lb == 0) {
            const float scale = clip_scale(c, sqnorm);
            for (uint32_t t = threadIdx.x; t < s.head + s.tail; t += kRwThreads) {
                const uint64_t i = off + edge_elem<VEC>(s, t);
                float p = master[i], m = exp_avg[i], v = exp_avg_sq[i];
                adamw1(c, scale, grad1<K>(pp, k, gf32, i), p, m, v);
                master[i] = p;
                exp_avg[i] = m;
                exp_avg_sq[i] = v;
                if constexpr (WRITE_BF16) out[i] = (uint16_t)f32_to_bf16(p);
                biggest = max(biggest, abs_bits(p));
            }
        }
    } else {
        const uint64_t i = element_index();
        if (i < s.n) {
            float p = master[i], m = exp_avg[i], v = exp_avg_sq[i];
            const float g = grad1<K>(pp, k, gf32, i);
            adamw1(c, clip_scale(c, sqnorm), g, p, m, v);
            master[i] = p;
            exp_avg[i] = m;
            exp_avg_sq[i] = v;
            if constexpr (WRITE_BF16) out[i] = (uint16_t)f32_to_bf16(p);
            biggest = max(biggest, abs_bits(p));
        }
    }
    if constexpr (AMAX) wave_amax_into(biggest, seen, amax);
}

// Many short ranges in one launch: the segments of an inter-tensor shard that are too short to be
// worth a launch each (norm gains, biases).  Range r owns the blocks [first_block[r], first_block[r+1])
// and has its own head; its gradient and bf16 output sit at flat_off[r] of the flat buffers, its
// optimizer states at local_off[r] of the compact ones.  The table travels in the kernel arguments, so a
// block finds its range with 31 scalar compares and no memory access of its own.  Run-time k only:
// these ranges hold a sliver of the model's bytes.
constexpr int kMaxTableRanges = 32;
constexpr uint64_t kShortSegment = 1ull << 20;   // elements: ~5 us of traffic, about what a launch costs
struct RangeTable {
    uint32_t first_block[kMaxTableRanges];   // unused entries: 0xFFFFFFFF
    uint32_t head[kMaxTableRanges];          // elements before the first aligned vector; == len: no vector at all
    uint32_t segment[kMaxTableRanges];       // index in the caller's segment list (for the maxima words)
    uint64_t flat_off[kMaxTableRanges];
    uint64_t local_off[kMaxTableRanges];
    uint64_t len[kMaxTableRanges];
};

template <int K, bool WRITE_BF16, bool AMAX>
__global__ void __launch_bounds__(kRwThreads) adamw_table_kernel(PartialPtrs pp, int k,
                                                                 const float *__restrict__ gf32_local,
                                                                 float *__restrict__ master,
                                                                 float *__restrict__ exp_avg,
                                                                 float *__restrict__ exp_avg_sq,
                                                                 uint16_t *__restrict__ out,
                                                                 uint32_t *__restrict__ amax_words, AdamConsts c,
                                                                 RangeTable t) {
    constexpr int VEC = kVecRW;
    const double sqnorm = load_sqnorm(c);
    uint32_t r = 0;
#pragma unroll
    for (int i = 1; i < kMaxTableRanges; ++i) r += blockIdx.x >= t.first_block[i] ? 1u : 0u;
    const uint32_t lb = blockIdx.x - t.first_block[r];
    const uint64_t len = t.len[r], flat = t.flat_off[r], local = t.local_off[r];
    const uint32_t head = t.head[r];
    uint32_t *words = nullptr;
    uint32_t seen = 0;
    if constexpr (AMAX) {
        words = amax_words + (size_t)t.segment[r] * kAmaxWordsPerSegment;
        seen = amax_seen(words);
    }
    const uint64_t nvec = (len - head) / VEC;
    const uint32_t tail = (uint32_t)(len - head - nvec * VEC);
    uint32_t biggest = 0;
    const uint64_t vi = (uint64_t)lb * kRwThreads + threadIdx.x;
    if (vi < nvec) {
        const uint64_t i = head + vi * VEC;
        float g[VEC], p[VEC], m[VEC], v[VEC];
        ld_f32<VEC>(master, local + i, p);
        ld_f32<VEC>(exp_avg, local + i, m);
        ld_f32<VEC>(exp_avg_sq, local + i, v);
        // K == 0: the gradient is the rank's compact fp32 buffer, indexed like its optimizer states
        grad_vec<K, VEC>(pp, k, gf32_local, (K == 0 ? local : flat) + i, g);
        const float scale = clip_scale(c, sqnorm);
#pragma unroll
        for (int q = 0; q < VEC; ++q) adamw1(c, scale, g[q], p[q], m[q], v[q]);
        st_f32<VEC>(master, local + i, p);
        st_f32<VEC>(exp_avg, local + i, m);
        st_f32<VEC>(exp_avg_sq, local + i, v);
        if constexpr (WRITE_BF16) st_bf16<VEC>(out, flat + i, p);
        if constexpr (AMAX) {
#pragma unroll
            for (int q = 0; q < VEC; ++q) biggest = max(biggest, abs_bits(p[q]));
        }
    }
    if (lb == 0) {
        const float scale = clip_scale(c, sqnorm);
        for (uint32_t e = threadIdx.x; e < head + tail; e += kRwThreads) {
            const uint64_t i = e < head ? (uint64_t)e : (uint64_t)head + nvec * VEC + (e - head);
            float p = master[local + i], m = exp_avg[local + i], v = exp_avg_sq[local + i];
            adamw1(c, scale, grad1<K>(pp, k, gf32_local, (K == 0 ? local : flat) + i), p, m, v);
            master[local + i] = p;
            exp_avg[local + i] = m;
            exp_avg_sq[local + i] = v;
            if constexpr (WRITE_BF16) out[flat + i] = (uint16_t)f32_to_bf16(p);
            biggest = max(biggest, abs_bits(p));
        }
    }
    if constexpr (AMAX) wave_amax_into(biggest, seen, words);
}

// ---------------------------------------------------------------- FP8 (E4M3) payload
// fp32 -> OCP E4M3 on the bit pattern: round to nearest even, saturate at +-448, NaN -> S.1111.111.
__device__ __forceinline__ uint32_t f32_to_e4m3(float x) {
    const uint32_t u = __float_as_uint(x);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7FFFFFFFu;
    uint32_t code;
    if (a > 0x7F800000u) {
        code = 0x7Fu;                                   // NaN
    } else if (a >= 0x43E80000u) {
        code = 0x7Eu;                                   // |x| >= 464 (midpoint above 448, tie to even) and Inf: 448
    } else if (a < 0x3C800000u) {
        // below 2^-6: multiples of 2^-9; |x| * 512 is exact in fp32 and rintf rounds ties to even
        code = (uint32_t)rintf(__uint_as_float(a) * 512.0f);   // 0..8, where 8 is the smallest normal
    } else {
        const uint32_t r = a + 0x7FFFFu + ((a >> 20) & 1u);    // round to 3 mantissa bits, ties to even
        code = (r >> 20) - (120u << 3);                        // re-bias the exponent from 127 to 7
    }
    return sign | code;
}

__global__ void __launch_bounds__(kThreads) fill_u32_kernel(uint32_t *p, uint32_t count, uint32_t value) {
    for (uint32_t i = blockIdx.x * kThreads + threadIdx.x; i < count; i += gridDim.x * kThreads) p[i] = value;
}

// Largest |x| of a range into *slot (integer atomic max: deterministic).  Persistent read-only
// grid like the norm pass.
__global__ void __launch_bounds__(kNormThreads) absmax_kernel(const float *__restrict__ x, Span s,
                                                              uint32_t *__restrict__ slot) {
    constexpr int VEC = 4;
    const uint64_t first = (uint64_t)blockIdx.x * kNormThreads + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * kNormThreads;
    uint32_t m = 0;
    if (s.vectorised) {
        for (uint64_t v = first; v < s.nvec; v += stride) {
            float t[VEC];
            ld_f32<VEC>(x, s.head + v * VEC, t);
#pragma unroll
            for (int c = 0; c < VEC; ++c) m = max(m, abs_bits(t[c]));
        }
        if (blockIdx.x == 0)
            for (uint32_t t = threadIdx.x; t < s.head + s.tail; t += kNormThreads) m = max(m, abs_bits(x[edge_elem<VEC>(s, t)]));
    } else {
        for (uint64_t i = first; i < s.n; i += stride) m = max(m, abs_bits(x[i]));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_down((int)m, off, 64));
    __shared__ uint32_t wave_max[kNormThreads / 64];
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kNormThreads / 64; ++w) m = max(m, wave_max[w]);
        atomicMax(slot, m);
    }
}

// scale[i] = 448 / amax[i] in fp32 (correctly rounded division); 1 when amax is 0, Inf or NaN.
__global__ void __launch_bounds__(kThreads) fp8_scale_kernel(const float *__restrict__ amax, float *__restrict__ scale,
                                                             uint32_t count) {
    for (uint32_t i = blockIdx.x * kThreads + threadIdx.x; i < count; i += gridDim.x * kThreads) {
        const float a = amax[i];
        scale[i] = (a > 0.0f && a < __uint_as_float(0x7F800000u)) ? 448.0f / a : 1.0f;
    }
}

__global__ void __launch_bounds__(kThreads) cast_fp8_kernel(const float *__restrict__ master,
                                                            const float *__restrict__ d_scale,
                                                            uint8_t *__restrict__ out, Span s) {
    constexpr int VEC = 4;
    const float scale = *d_scale;
    if (s.vectorised) {
        const uint64_t v = vector_index();
        if (v < s.nvec) {
            const uint64_t e = s.head + v * VEC;
            float x[VEC];
            ld_f32<VEC>(master, e, x);
            uint32_t w = 0;
#pragma unroll
            for (int c = 0; c < VEC; ++c) w |= f32_to_e4m3(x[c] * scale) << (8 * c);
            st_stream(reinterpret_cast<uint32_t *>(out + e), w);
        }
        if (blockIdx.x == 0)
            for (uint32_t t = threadIdx.x; t < s.head + s.tail; t += kRwThreads) {
                const uint64_t i = edge_elem<VEC>(s, t);
                out[i] = (uint8_t)f32_to_e4m3(master[i] * scale);
            }
    } else {
        const uint64_t i = element_index();
        if (i < s.n) out[i] = (uint8_t)f32_to_e4m3(master[i] * scale);
    }
}

// Step 1 for short segments, 32 to a launch: out_local[local + i] (=|+=) sum_j partials[j][flat + i].
__global__ void __launch_bounds__(kRwThreads) reduce_table_kernel(PartialPtrs pp, int k, float *__restrict__ out,
                                                                  int accumulate, RangeTable t) {
    constexpr int VEC = kVecRW;
    uint32_t r = 0;
#pragma unroll
    for (int i = 1; i < kMaxTableRanges; ++i) r += blockIdx.x >= t.first_block[i] ? 1u : 0u;
    const uint32_t lb = blockIdx.x - t.first_block[r];
    const uint64_t len = t.len[r], flat = t.flat_off[r], local = t.local_off[r];
    const uint32_t head = t.head[r];
    const uint64_t nvec = (len - head) / VEC;
    const uint32_t tail = (uint32_t)(len - head - nvec * VEC);
    const uint64_t vi = (uint64_t)lb * kRwThreads + threadIdx.x;
    if (vi < nvec) {
        const uint64_t i = head + vi * VEC;
        float g[VEC], o[VEC];
        if (accumulate) ld_f32<VEC>(out, local + i, o);
        grad_vec<-1, VEC>(pp, k, nullptr, flat + i, g);
        if (accumulate) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) g[c] = o[c] + g[c];
        }
        st_f32<VEC>(out, local + i, g);
    }
    if (lb == 0)
        for (uint32_t e = threadIdx.x; e < head + tail; e += kRwThreads) {
            const uint64_t i = e < head ? (uint64_t)e : (uint64_t)head + nvec * VEC + (e - head);
            float g1 = grad1<-1>(pp, k, nullptr, flat + i);
            if (accumulate) g1 = out[local + i] + g1;
            out[local + i] = g1;
        }
}

// The FP8 payload of short segments, 32 to a launch like the update above.  CAST = false: the largest
// |x| of each range into slots[segment] (integer atomic max, sent only when it beats the word's current
// value); CAST = true: codes = e4m3(x * d_scale[segment]) at the range's flat position.
template <bool CAST>
__global__ void __launch_bounds__(kRwThreads) fp8_table_kernel(const float *__restrict__ master,
                                                               const float *__restrict__ d_scale,
                                                               uint8_t *__restrict__ out, uint32_t *__restrict__ slots,
                                                               RangeTable t) {
    constexpr int VEC = 4;
    uint32_t r = 0;
#pragma unroll
    for (int i = 1; i < kMaxTableRanges; ++i) r += blockIdx.x >= t.first_block[i] ? 1u : 0u;
    const uint32_t lb = blockIdx.x - t.first_block[r];
    const uint64_t len = t.len[r], flat = t.flat_off[r], local = t.local_off[r];
    const uint32_t head = t.head[r], seg = t.segment[r];
    const uint64_t nvec = (len - head) / VEC;
    const uint32_t tail = (uint32_t)(len - head - nvec * VEC);
    const uint64_t vi = (uint64_t)lb * kRwThreads + threadIdx.x;
    if constexpr (CAST) {
        const float scale = d_scale[seg];
        if (vi < nvec) {
            const uint64_t i = head + vi * VEC;
            float x[VEC];
            ld_f32<VEC>(master, local + i, x);
            uint32_t w = 0;
#pragma unroll
            for (int c = 0; c < VEC; ++c) w |= f32_to_e4m3(x[c] * scale) << (8 * c);
            st_stream(reinterpret_cast<uint32_t *>(out + flat + i), w);
        }
        if (lb == 0)
            for (uint32_t e = threadIdx.x; e < head + tail; e += kRwThreads) {
                const uint64_t i = e < head ? (uint64_t)e : (uint64_t)head + nvec * VEC + (e - head);
                out[flat + i] = (uint8_t)f32_to_e4m3(master[local + i] * scale);
            }
    } else {
        uint32_t m = 0;
        if (vi < nvec) {
            float x[VEC];
            ld_f32<VEC>(master, local + head + vi * VEC, x);
#pragma unroll
            for (int c = 0; c < VEC; ++c) m = max(m, abs_bits(x[c]));
        }
        if (lb == 0)
            for (uint32_t e = threadIdx.x; e < head + tail; e += kRwThreads) {
                const uint64_t i = e < head ? (uint64_t)e : (uint64_t)head + nvec * VEC + (e - head);
                m = max(m, abs_bits(master[local + i]));
            }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_down((int)m, off, 64));
        if (threadIdx.x == 0 && m > __hip_atomic_load(slots + seg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(slots + seg, m);
    }
}

// ---------------------------------------------------------------- host side
typedef amsp_geom::Stream Stream16;
using amsp_geom::make_span;
using amsp_geom::make_buckets;

// Calls f(off, len, U).  U == 0: one launch over the single range [off, off + len).  U > 0: one launch
// over the buckets of U elements of [off, off + len): as many buckets as the grid limit allows.
template <typename F>
int for_bucket_launches(uint64_t n, uint64_t bucket_elems, F f) {
    if (bucket_elems == 0 || bucket_elems >= n) return f((uint64_t)0, n, (uint64_t)0);
    const uint64_t blocks_per_bucket = bucket_elems / ((uint64_t)kRwThreads * kVecRW) + 1;
    uint64_t per_launch = kMaxGrid / blocks_per_bucket;
    if (per_launch == 0) per_launch = 1;
    const uint64_t step = per_launch > (~0ull) / bucket_elems ? n : per_launch * bucket_elems;
    for (uint64_t off = 0; off < n; off += step) {
        const uint64_t len = n - off < step ? n - off : step;
        const int rc = f(off, len, bucket_elems);
        if (rc != AMSP_OK) return rc;
    }
    return AMSP_OK;
}

// Occupancy cap of the read+write kernels.  With one-wave workgroups and only as many waves resident
// per CU as it takes to keep a target amount of loads in flight, the same kernels move 5-12 % more
// bytes per second than at full occupancy (32 waves): fewer waves in flight keep the window of
// addresses being read and written at any moment small, and reads and writes disturb each other
// less.  The cap is imposed by giving every workgroup an unused slice of the CU's 160 KiB of LDS.
// `load_bytes_per_lane` is what one lane has in flight before it waits.
struct RwKnobs {
    int inflight_kib, min_waves, reduce_inflight_kib, reduce_min_waves;
};
RwKnobs read_rw_knobs() {   // developer knobs for sweeps; read once (thread-safe static below)
    auto knob = [](const char *name, int lo, int hi, int dflt) {
        const char *v = getenv(name);
        const int x = v ? atoi(v) : 0;
        return (x >= lo && x <= hi) ? x : dflt;
    };
    return RwKnobs{knob("AMSP_INFLIGHT_KIB", 8, 1024, 40), knob("AMSP_MIN_WAVES", 4, 32, 8),
                   knob("AMSP_REDUCE_INFLIGHT_KIB", 8, 1024, 64), knob("AMSP_REDUCE_MIN_WAVES", 4, 32, 12)};
}
const RwKnobs &rw_knobs() {
    static const RwKnobs knobs = read_rw_knobs();
    return knobs;
}

// What a kernel family wants in flight per CU, and the fewest waves it is given.
struct RwTarget {
    int inflight_kib, min_waves;
};
// AdamW kernels: 40 KiB, at least 8 waves (10 waves for an fp32 gradient, 12 for k = 1, 8 from k = 4 on),
// 7 once a wave loads more than 8 KiB (fused step from k = 9 on: k = 16 reads 6,330 GB/s at 7 waves
// against 6,010-6,270 at 8, while k = 8 is best at 8).
RwTarget adamw_target(unsigned load_bytes_per_lane) {
    const int floor = 64u * load_bytes_per_lane > 8192u ? rw_knobs().min_waves - 1 : rw_knobs().min_waves;
    return RwTarget{rw_knobs().inflight_kib, floor};
}
// Reduction (its writes are a small share of the traffic): 64 KiB, at least 12 waves (k = 8: 16 waves,
// 13 with accumulate; k = 16: 12; no cap below k = 8).
RwTarget reduce_target() { return RwTarget{rw_knobs().reduce_inflight_kib, rw_knobs().reduce_min_waves}; }

int rw_waves_per_cu(unsigned load_bytes_per_lane, RwTarget t) {
    const unsigned per_wave = 64u * load_bytes_per_lane;
    int waves = (int)(((unsigned)t.inflight_kib * 1024u + per_wave - 1) / per_wave);
    if (waves < t.min_waves) waves = t.min_waves;
    return waves > 32 ? 32 : waves;
}

// Bytes of dynamic LDS per one-wave workgroup so that at most that many of them fit a CU.
unsigned occupancy_lds(unsigned load_bytes_per_lane, RwTarget t) {
    const int waves = rw_waves_per_cu(load_bytes_per_lane, t);
    if (waves >= 32) return 0;
    return (unsigned)((160 * 1024 / waves) & ~255);
}

// One lane per vector in one-wave workgroups under the occupancy cap, or, on the element-wise path,
// one lane per element in 256-thread workgroups; the whole range in one grid either way.
struct RwLaunch {
    dim3 grid, block;
    unsigned lds;
};

RwLaunch rw_launch(const Span &s, unsigned load_bytes_per_lane, RwTarget t) {
    const uint64_t work = s.vectorised ? s.nvec : s.n;
    const unsigned threads = s.vectorised ? kRwThreads : kThreads;
    uint64_t blocks = (work + threads - 1) / threads;   // <= kMaxGrid: the entry points refuse larger launches
    if (blocks == 0) blocks = 1;
    return RwLaunch{dim3((unsigned)blocks), dim3(threads),
                    s.vectorised ? occupancy_lds(load_bytes_per_lane, t) : 0u};
}

// Reduce with the norm fused in: every block leaves one double.  One-wave blocks of one vector per
// lane on the vector path (a sum per 256 elements), a capped grid-stride grid on the element-wise path.
constexpr int kSliceBlocks = 256;

uint64_t reduce_norm_grid(const Span &s) {
    uint64_t blocks;
    if (s.vectorised) {
        blocks = (s.nvec + kRwThreads - 1) / kRwThreads;
    } else {
        blocks = (s.n + kThreads - 1) / kThreads;
        if (blocks > (uint64_t)kNormBlocks) blocks = kNormBlocks;
    }
    return blocks == 0 ? 1 : blocks;
}

// Upper bound of reduce_norm_grid over every alignment of a launch of `len` elements.
uint64_t reduce_norm_blocks_max(uint64_t len) { return len / ((uint64_t)kRwThreads * kVecRW) + 2; }

// Block sums of every bucket of a call lie side by side and are added once, after the last bucket.
uint64_t reduce_norm_slots(uint64_t n, uint64_t bucket_elems) {
    if (bucket_elems == 0 || bucket_elems >= n) return reduce_norm_blocks_max(n);
    const uint64_t buckets = (n + bucket_elems - 1) / bucket_elems;   // a short last bucket gets a full one's blocks
    return buckets * reduce_norm_blocks_max(bucket_elems);
}

int cu_count() {
    static std::atomic<int> cached[64];   // per device; zero until first asked (any thread may fill it: same value)
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// The norm pass: two 1024-thread blocks per CU (what a CU holds), at most kNormBlocks; `work` = lanes' worth
// of vectors (or elements on the element-wise path).
int norm_grid(uint64_t work) {
    uint64_t blocks = (work + kNormThreads - 1) / kNormThreads;
    uint64_t cap = 2 * (uint64_t)cu_count();
    if (cap > kNormBlocks) cap = kNormBlocks;
    if (blocks > cap) blocks = cap;
    return blocks == 0 ? 1 : (int)blocks;
}
int norm_grid(const Span &s) { return norm_grid(s.vectorised ? s.nvec : s.n); }

// One launch covers at most this many elements (one wave per 256 of them in a grid of < 2^31 blocks):
// about 5.5e11, beyond any buffer that fits the device.
constexpr uint64_t kMaxLaunchElems = kMaxGrid * (uint64_t)kRwThreads;
bool too_long(uint64_t n, uint64_t bucket_elems) {
    return ((bucket_elems != 0 && bucket_elems < n) ? bucket_elems : n) > kMaxLaunchElems;
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

// The HIP error state is per thread and shared with every other user of the runtime in the
// process, so anything left there by someone else is dropped before a launch and only the
// launch's own status is reported.
inline void clear_stale_error() { (void)hipGetLastError(); }
inline int launched() {
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) return AMSP_OK;
    fprintf(stderr, "amsp: kernel launch failed: %s\n", hipGetErrorString(e));
    return AMSP_EDEVICE;
}

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

// Block sums of consecutive norm launches (buckets, segments) go side by side into the workspace
// and are added once, in launch order, by a finishing pass: one finish per ~100 launches instead
// of one per launch.  Layout: [0, kNormSlots) block sums, then kSliceBlocks stage sums.
constexpr size_t kNormSlots = 64 * 1024;

int finish_sums(hipStream_t hs, double *sums, uint64_t count, double *stage, double *out, int accumulate);

struct NormBatch {
    hipStream_t hs;
    double *sums;
    double *out;
    size_t used;
    bool add;     // whether the next finish adds to *out

    int flush() {
        if (used == 0) return AMSP_OK;
        int rc = finish_sums(hs, sums, used, sums + kNormSlots, out, add ? 1 : 0);
        used = 0;
        add = true;
        return rc;
    }
    // Room for `blocks` more sums; returns where they go, flushing first when the workspace is full.
    int reserve(int blocks, double **where) {
        if (used + (size_t)blocks > kNormSlots) {
            int rc = flush();
            if (rc != AMSP_OK) return rc;
        }
        *where = sums + used;
        used += (size_t)blocks;
        return AMSP_OK;
    }
};

// Every k up to 16 has its own instantiation (all k loads of a vector in flight at once); larger k
// take the run-time loop.
#define AMSP_DISPATCH_K(k, CALL)                 \
    switch (k) {                                 \
        case 1: { constexpr int KK = 1; CALL; } break;   \
        case 2: { constexpr int KK = 2; CALL; } break;   \
        case 3: { constexpr int KK = 3; CALL; } break;   \
        case 4: { constexpr int KK = 4; CALL; } break;   \
        case 5: { constexpr int KK = 5; CALL; } break;   \
        case 6: { constexpr int KK = 6; CALL; } break;   \
        case 7: { constexpr int KK = 7; CALL; } break;   \
        case 8: { constexpr int KK = 8; CALL; } break;   \
        case 9: { constexpr int KK = 9; CALL; } break;   \
        case 10: { constexpr int KK = 10; CALL; } break;   \
        case 11: { constexpr int KK = 11; CALL; } break;   \
        case 12: { constexpr int KK = 12; CALL; } break;   \
        case 13: { constexpr int KK = 13; CALL; } break;   \
        case 14: { constexpr int KK = 14; CALL; } break;   \
        case 15: { constexpr int KK = 15; CALL; } break;   \
        case 16: { constexpr int KK = 16; CALL; } break;   \
        default: { constexpr int KK = -1; CALL; } break; \
    }

// Adds `count` block sums in index order into *out: one block when they are few, otherwise
// kSliceBlocks blocks each add a contiguous slice into `stage` and one block adds those.
int finish_sums(hipStream_t hs, double *sums, uint64_t count, double *stage, double *out, int accumulate) {
    const double *src = sums;
    int n = (int)count;
    if (count > (uint64_t)kNormBlocks) {
        const uint64_t slice = (count + kSliceBlocks - 1) / kSliceBlocks;
        n = (int)((count + slice - 1) / slice);
        hipLaunchKernelGGL(sum_slices_kernel, dim3(n), dim3(kThreads), 0, hs, sums, count, slice, stage);
        if (launched() != AMSP_OK) return AMSP_EDEVICE;
        src = stage;
    }
    hipLaunchKernelGGL(sqnorm_finish_kernel, dim3(1), dim3(kThreads), 0, hs, src, n, out, accumulate);
    return launched();
}

// One norm launch over up to kMaxNormSegs ranges [base[i], base[i] + len[i]) of the streams, its block sums
// appended to the batch.  The streams are the k partials (k >= 1) or the fp32 gradient (k == 0).
int norm_launch(NormBatch &batch, const PartialPtrs &pp, uint32_t k, const float *gf, const uint64_t *base,
                const uint64_t *len, int count) {
    // 16-byte accesses in every case: 8 bf16 elements per lane, or 4 of the fp32 gradient
    const int vec = k == 0 ? 4 : kVecNorm;
    NormSegTable t;
    t.count = count;
    uint64_t work = 0;
    for (int i = 0; i < count; ++i) {
        Stream16 st[AMSP_MAX_K + 1];
        int ns = add_partial_streams(st, 0, offset_partials(pp, k, base[i]), k);
        if (k == 0) st[ns++] = Stream16{gf + base[i], 4};
        t.seg[i].base = base[i];
        t.seg[i].s = make_span(len[i], st, ns, vec);
        work += t.seg[i].s.vectorised ? t.seg[i].s.nvec : t.seg[i].s.n;
    }
    const int grid = norm_grid(work);
    double *block_sums = nullptr;
    int rc = batch.reserve(grid, &block_sums);
    if (rc != AMSP_OK) return rc;
    hipStream_t hs = batch.hs;
#define AMSP_LAUNCH_SQNORM(KV, V)                                                                     \
    hipLaunchKernelGGL((sqnorm_kernel<KV, V>), dim3(grid), dim3(kNormThreads), 0, hs, pp, (int)k, gf, block_sums, t)
    if (k == 0) {
        AMSP_LAUNCH_SQNORM(0, 4);
    } else {
        AMSP_DISPATCH_K(k, AMSP_LAUNCH_SQNORM(KK, kVecNorm));
    }
#undef AMSP_LAUNCH_SQNORM
    return launched();
}

// One launch of the short-range kernel over up to kMaxNormSegs ranges.
int norm_launch_short(NormBatch &batch, const PartialPtrs &pp, uint32_t k, const float *gf, const uint64_t *base,
                      const uint64_t *len, int count) {
    const int vec = k == 0 ? 4 : kVecNorm;
    ShortNormTable t;
    uint32_t blocks_total = 0;
    for (int i = 0; i < kMaxNormSegs; ++i) {
        if (i >= count) {
            t.first_block[i] = 0xFFFFFFFFu;
            t.blocks[i] = 0;
            t.seg[i] = NormSeg{0, Span{0, 0, 0, 0, 0}};
            continue;
        }
        Stream16 st[AMSP_MAX_K + 1];
        int ns = add_partial_streams(st, 0, offset_partials(pp, k, base[i]), k);
        if (k == 0) st[ns++] = Stream16{gf + base[i], 4};
        t.seg[i].base = base[i];
        t.seg[i].s = make_span(len[i], st, ns, vec);
        uint64_t blocks = t.seg[i].s.vectorised ? (t.seg[i].s.nvec + kNormThreads - 1) / kNormThreads
                                                : (len[i] + kNormThreads - 1) / kNormThreads;
        if (!t.seg[i].s.vectorised && blocks > 64) blocks = 64;
        if (blocks == 0) blocks = 1;
        t.first_block[i] = blocks_total;
        t.blocks[i] = (uint32_t)blocks;
        blocks_total += (uint32_t)blocks;
    }
    double *block_sums = nullptr;
    int rc = batch.reserve((int)blocks_total, &block_sums);
    if (rc != AMSP_OK) return rc;
    hipStream_t hs = batch.hs;
    if (k == 0)
        hipLaunchKernelGGL((sqnorm_short_kernel<0, 4>), dim3(blocks_total), dim3(kNormThreads), 0, hs, pp, (int)k, gf,
                           block_sums, t);
    else
        hipLaunchKernelGGL((sqnorm_short_kernel<-1, kVecNorm>), dim3(blocks_total), dim3(kNormThreads), 0, hs, pp,
                           (int)k, gf, block_sums, t);
    return launched();
}

// Norm launches over a list of ranges, kMaxNormSegs per launch: ranges long enough to keep the whole
// persistent grid busy (a few vectors per lane) go to the grid-stride kernel, the others to the
// short-range kernel.
constexpr uint64_t kShortNormRange = 4ull << 20;   // elements; 4 Mi elements = one 16-byte vector per resident lane
struct NormRanges {
    NormBatch &batch;
    const PartialPtrs &pp;
    uint32_t k;
    const float *gf;
    uint64_t base[kMaxNormSegs], len[kMaxNormSegs];
    uint64_t short_base[kMaxNormSegs], short_len[kMaxNormSegs];
    int count = 0, short_count = 0;

    int flush_long() {
        if (count == 0) return AMSP_OK;
        const int rc = norm_launch(batch, pp, k, gf, base, len, count);
        count = 0;
        return rc;
    }
    int flush_short() {
        if (short_count == 0) return AMSP_OK;
        const int rc = norm_launch_short(batch, pp, k, gf, short_base, short_len, short_count);
        short_count = 0;
        return rc;
    }
    int flush() {
        const int rc = flush_long();
        return rc != AMSP_OK ? rc : flush_short();
    }
    int add(uint64_t b, uint64_t l) {
        if (l < kShortNormRange) {
            short_base[short_count] = b;
            short_len[short_count] = l;
            return ++short_count == kMaxNormSegs ? flush_short() : AMSP_OK;
        }
        base[count] = b;
        len[count] = l;
        return ++count == kMaxNormSegs ? flush_long() : AMSP_OK;
    }
};

// Collects short segments for one table launch.  A segment qualifies when it is shorter than
// kShortSegment and either has a common vector phase or is so short that the edge loop of one wave
// takes all of it; everything else gets a launch of its own.
struct TableBuilder {
    RangeTable table;
    uint32_t count = 0, blocks = 0;

    static bool takes(const amsp_segment &g, const Span &sp) {
        return g.length < kShortSegment && (sp.vectorised || g.length <= 16 * (uint64_t)kRwThreads);
    }
    // Adds segment `index`; true when the table is now full and must be launched.
    bool add(uint32_t index, const amsp_segment &g, const Span &sp) {
        table.first_block[count] = blocks;
        table.head[count] = sp.vectorised ? sp.head : (uint32_t)g.length;
        table.segment[count] = index;
        table.flat_off[count] = g.flat_offset;
        table.local_off[count] = g.local_offset;
        table.len[count] = g.length;
        const uint64_t b = sp.vectorised ? (sp.nvec + kRwThreads - 1) / kRwThreads : 0;
        blocks += (uint32_t)(b ? b : 1);
        return ++count == (uint32_t)kMaxTableRanges;
    }
    // Marks the unused entries; call before a launch, reset() after it.
    void pad() {
        for (uint32_t j = count; j < (uint32_t)kMaxTableRanges; ++j) {
            table.first_block[j] = 0xFFFFFFFFu;
            table.head[j] = 0; table.segment[j] = 0; table.flat_off[j] = 0; table.local_off[j] = 0; table.len[j] = 0;
        }
    }
    void reset() { count = 0; blocks = 0; }
};

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
        case AMSP_ENOPLAN: return "no sharding plan is feasible";
        default: return "unknown status";
    }
}

size_t amsp_workspace_bytes(void) { return (kNormSlots + kSliceBlocks) * sizeof(double); }

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
    if (too_long(n, 0)) return AMSP_EINVAL;
    if (master == nullptr || param_bf16_out == nullptr) return AMSP_ENULL;
    if (misaligned(master, 4) || misaligned(param_bf16_out, 2)) return AMSP_EALIGN;
    Stream16 st[2] = {{master, 4}, {param_bf16_out, 2}};
    Span s = make_span(n, st, 2, kVecRW);
    clear_stale_error();
    const RwLaunch L = rw_launch(s, 16, adamw_target(16));
    hipLaunchKernelGGL(cast_kernel, L.grid, L.block, L.lds, (hipStream_t)stream, master, param_bf16_out, s);
    return launched();
}

size_t amsp_reduce_workspace_bytes(uint64_t n, uint64_t bucket_elems) {
    return (size_t)(reduce_norm_slots(n, bucket_elems) + kSliceBlocks) * sizeof(double);
}

int amsp_reduce_grad_shard(const uint16_t *const *partials, uint32_t k, uint64_t n, uint64_t bucket_elems,
                           float *grad_out, int accumulate, double *d_sqnorm, int sqnorm_accumulate,
                           void *workspace, size_t workspace_bytes, void *stream) {
    PartialPtrs pp;
    int rc = check_partials(partials, k, pp);
    if (rc != AMSP_OK) return rc;
    const bool norm = d_sqnorm != nullptr;
    if (norm) {
        if (workspace == nullptr) return AMSP_ENULL;
        if (misaligned(d_sqnorm, 8) || misaligned(workspace, 8)) return AMSP_EALIGN;
        if (workspace_bytes < amsp_reduce_workspace_bytes(n, bucket_elems)) return AMSP_EWORKSPACE;
    }
    hipStream_t hs = (hipStream_t)stream;
    double *block_sums = static_cast<double *>(workspace);
    if (n == 0) {
        if (norm && !sqnorm_accumulate) {
            clear_stale_error();
            hipLaunchKernelGGL(sqnorm_finish_kernel, dim3(1), dim3(kThreads), 0, hs, block_sums, 0, d_sqnorm, 0);
            return launched();
        }
        return AMSP_OK;
    }
    if (too_long(n, bucket_elems)) return AMSP_EINVAL;
    if (grad_out == nullptr) return AMSP_ENULL;
    if (misaligned(grad_out, 4)) return AMSP_EALIGN;
    uint64_t used = 0;   // block sums written so far, bucket after bucket
    const unsigned lane_bytes = 8 * k + (accumulate ? 16 : 0);
    auto single = [&](uint64_t off, uint64_t len) -> int {
        PartialPtrs q = offset_partials(pp, k, off);
        Stream16 st[AMSP_MAX_K + 1];
        int ns = add_partial_streams(st, 0, q, k);
        st[ns++] = Stream16{grad_out + off, 4};
        Span s = make_span(len, st, ns, kVecRW);
        const Buckets none{};
        clear_stale_error();
        const RwLaunch L = rw_launch(s, lane_bytes, reduce_target());
        if (!norm) {
            AMSP_DISPATCH_K(k, hipLaunchKernelGGL((reduce_kernel<KK, false>), L.grid, L.block, L.lds, hs, q, (int)k,
                                                  grad_out + off, accumulate, block_sums, s, none));
            return launched();
        }
        const uint64_t blocks = reduce_norm_grid(s);   // == L.grid.x on the vector path, capped on the other
        AMSP_DISPATCH_K(k, hipLaunchKernelGGL((reduce_kernel<KK, true>), dim3((unsigned)blocks), L.block, L.lds, hs, q,
                                              (int)k, grad_out + off, accumulate, block_sums + used, s, none));
        used += blocks;
        return launched();
    };
    rc = for_bucket_launches(n, bucket_elems, [&](uint64_t off, uint64_t len, uint64_t U) -> int {
        if (U == 0) return single(off, len);
        PartialPtrs q = offset_partials(pp, k, off);
        Stream16 st[AMSP_MAX_K + 1];
        int ns = add_partial_streams(st, 0, q, k);
        st[ns++] = Stream16{grad_out + off, 4};
        Buckets bk;
        if (!make_buckets(len, U, st, ns, kVecRW, bk))
            return for_buckets(len, U, [&](uint64_t o, uint64_t l) { return single(off + o, l); });
        const dim3 grid((unsigned)(((len + U - 1) / U) * bk.blocks_per_bucket)), block(kRwThreads);
        const unsigned lds = occupancy_lds(lane_bytes, reduce_target());
        const Span s{len, 0, 0, 0, 1};
        clear_stale_error();
        if (!norm) {
            AMSP_DISPATCH_K(k, hipLaunchKernelGGL((reduce_kernel<KK, false>), grid, block, lds, hs, q, (int)k,
                                                  grad_out + off, accumulate, block_sums, s, bk));
            return launched();
        }
        AMSP_DISPATCH_K(k, hipLaunchKernelGGL((reduce_kernel<KK, true>), grid, block, lds, hs, q, (int)k,
                                              grad_out + off, accumulate, block_sums + used, s, bk));
        used += grid.x;
        return launched();
    });
    if (rc != AMSP_OK || !norm) return rc;
    // one finishing pass per call: the sums of all buckets in bucket order
    return finish_sums(hs, block_sums, used, block_sums + used, d_sqnorm, sqnorm_accumulate ? 1 : 0);
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
    NormBatch batch{(hipStream_t)stream, static_cast<double *>(workspace), d_sqnorm, 0, accumulate != 0};
    clear_stale_error();
    if (n == 0) {
        if (!accumulate) return finish_sums(batch.hs, batch.sums, 0, batch.sums + kNormSlots, d_sqnorm, 0);
        return AMSP_OK;
    }
    NormRanges ranges{batch, pp, k, grad_f32};
    int rc = for_buckets(n, bucket_elems, [&](uint64_t off, uint64_t len) { return ranges.add(off, len); });
    if (rc == AMSP_OK) rc = ranges.flush();
    if (rc != AMSP_OK) return rc;
    return batch.flush();
}

// Hyper-parameters checked and turned into the constants the kernels use (bias corrections in double).
static int adam_consts(const amsp_adamw_hparams *hp, AdamConsts &c) {
    if (hp == nullptr) return AMSP_ENULL;
    const bool finite = isfinite(hp->lr) && isfinite(hp->beta1) && isfinite(hp->beta2) && isfinite(hp->eps) &&
                        isfinite(hp->weight_decay) && isfinite(hp->grad_scale) && isfinite(hp->clip_eps) &&
                        !isnan(hp->max_norm);
    if (!finite || hp->step == 0 || !(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) ||
        !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f) || hp->eps < 0.0f)
        return AMSP_EINVAL;
    if (hp->d_total_sqnorm && misaligned(hp->d_total_sqnorm, 8)) return AMSP_EALIGN;
    c.lr = hp->lr; c.beta1 = hp->beta1; c.beta2 = hp->beta2; c.eps = hp->eps; c.wd = hp->weight_decay;
    c.one_minus_beta1 = (float)(1.0 - (double)hp->beta1);
    c.one_minus_beta2 = (float)(1.0 - (double)hp->beta2);
    c.rbc1 = (float)(1.0 / (1.0 - pow((double)hp->beta1, (double)hp->step)));
    c.rbc2 = (float)(1.0 / (1.0 - pow((double)hp->beta2, (double)hp->step)));
    c.max_norm = hp->max_norm; c.clip_eps = hp->clip_eps; c.grad_scale = hp->grad_scale;
    c.d_total_sqnorm = hp->d_total_sqnorm;
    return AMSP_OK;
}

// amax_slot: the range's kAmaxWordsPerSegment device words that collect the largest |p'| bit pattern, or NULL.
static int adamw_step_range(const uint16_t *const *partials, uint32_t k, const float *grad_f32, uint64_t n,
                            uint64_t bucket_elems, float *master, float *exp_avg, float *exp_avg_sq,
                            uint16_t *param_bf16_out, uint32_t *amax_slot, const amsp_adamw_hparams *hp,
                            void *stream) {
    if (hp == nullptr) return AMSP_ENULL;
    PartialPtrs pp{};
    if (k > 0) {
        int rc = check_partials(partials, k, pp);
        if (rc != AMSP_OK) return rc;
    }
    AdamConsts c;
    {
        const int rc = adam_consts(hp, c);
        if (rc != AMSP_OK) return rc;
    }
    if (n == 0) return AMSP_OK;
    if (too_long(n, bucket_elems)) return AMSP_EINVAL;
    if (master == nullptr || exp_avg == nullptr || exp_avg_sq == nullptr) return AMSP_ENULL;
    if (k == 0 && grad_f32 == nullptr) return AMSP_ENULL;
    if (misaligned(master, 4) || misaligned(exp_avg, 4) || misaligned(exp_avg_sq, 4) ||
        (k == 0 && misaligned(grad_f32, 4)) || (param_bf16_out && misaligned(param_bf16_out, 2)) ||
        (hp->d_total_sqnorm && misaligned(hp->d_total_sqnorm, 8)))
        return AMSP_EALIGN;

    hipStream_t hs = (hipStream_t)stream;

    const unsigned lane_bytes = (k != 0 ? 8 * k : 16) + 48;
    // one launch: a single range (U == 0, its Span worked out here) or the buckets of U elements of a range
    auto launch = [&](uint64_t off, uint64_t len, uint64_t U) -> int {
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
        Span s{len, 0, 0, 0, 1};
        Buckets bk{};
        dim3 grid, block(kRwThreads);
        unsigned lds = occupancy_lds(lane_bytes, adamw_target(lane_bytes));
        if (U == 0) {
            s = make_span(len, st, ns, kVecRW);
            const RwLaunch L = rw_launch(s, lane_bytes, adamw_target(lane_bytes));
            grid = L.grid; block = L.block; lds = L.lds;
        } else {
            if (!make_buckets(len, U, st, ns, kVecRW, bk)) return (int)AMSP_EALIGN;   // the caller falls back
            grid = dim3((unsigned)(((len + U - 1) / U) * bk.blocks_per_bucket));
        }
        clear_stale_error();
#define AMSP_LAUNCH_ADAMW_ONE(KV, B16, AM)                                                                  \
        hipLaunchKernelGGL((adamw_kernel<KV, B16, AM>), grid, block, lds, hs, q, (int)k, gf, master + off,       \
                           exp_avg + off, exp_avg_sq + off, out, amax_slot, c, s, bk)
#define AMSP_LAUNCH_ADAMW_AS(KV, b16, am)                                                                   \
        if (b16) { if (am) AMSP_LAUNCH_ADAMW_ONE(KV, true, true); else AMSP_LAUNCH_ADAMW_ONE(KV, true, false); } \
        else { if (am) AMSP_LAUNCH_ADAMW_ONE(KV, false, true); else AMSP_LAUNCH_ADAMW_ONE(KV, false, false); }
#define AMSP_LAUNCH_ADAMW(KV)                                                                              \
        AMSP_LAUNCH_ADAMW_AS(KV, (out != nullptr), (amax_slot != nullptr))
        if (k == 0) {
            AMSP_LAUNCH_ADAMW(0);
        } else {
            AMSP_DISPATCH_K(k, AMSP_LAUNCH_ADAMW(KK));
        }
#undef AMSP_LAUNCH_ADAMW
#undef AMSP_LAUNCH_ADAMW_AS
#undef AMSP_LAUNCH_ADAMW_ONE
        return launched();
    };
    return for_bucket_launches(n, bucket_elems, [&](uint64_t off, uint64_t len, uint64_t U) -> int {
        if (U == 0) return launch(off, len, 0);
        const int rc = launch(off, len, U);
        if (rc != AMSP_EALIGN) return rc;
        // streams without a common phase: a launch per bucket through the element-wise path
        return for_buckets(len, U, [&](uint64_t o, uint64_t l) { return launch(off + o, l, 0); });
    });
}

int amsp_adamw_step_shard(const uint16_t *const *partials, uint32_t k, const float *grad_f32, uint64_t n,
                          uint64_t bucket_elems, float *master, float *exp_avg, float *exp_avg_sq,
                          uint16_t *param_bf16_out, const amsp_adamw_hparams *hp, void *stream) {
    return adamw_step_range(partials, k, grad_f32, n, bucket_elems, master, exp_avg, exp_avg_sq, param_bf16_out,
                            nullptr, hp, stream);
}

// ---------------------------------------------------------------- inter-tensor shards
int amsp_partition_tensors(const uint64_t *tensor_elems, uint32_t num_tensors, uint32_t shard_factor,
                           uint32_t *owner) {
    if (shard_factor == 0) return AMSP_EINVAL;
    if (num_tensors == 0) return AMSP_OK;
    if (tensor_elems == nullptr || owner == nullptr) return AMSP_ENULL;
    uint64_t *load = static_cast<uint64_t *>(calloc(shard_factor, sizeof(uint64_t)));
    if (load == nullptr) return AMSP_EINVAL;
    for (uint32_t t = 0; t < num_tensors; ++t) {
        uint32_t best = 0;
        for (uint32_t r = 1; r < shard_factor; ++r)
            if (load[r] < load[best]) best = r;   // strict: the lowest rank wins a tie
        owner[t] = best;
        load[best] += tensor_elems[t];
    }
    free(load);
    return AMSP_OK;
}

int amsp_owned_segments(const uint64_t *tensor_elems, const uint32_t *owner, uint32_t num_tensors, uint32_t rank,
                        amsp_segment *segments, uint32_t capacity, uint32_t *num_segments, uint64_t *local_elems) {
    if (num_segments == nullptr || local_elems == nullptr) return AMSP_ENULL;
    if (num_tensors > 0 && (tensor_elems == nullptr || owner == nullptr)) return AMSP_ENULL;
    uint32_t count = 0;
    uint64_t flat = 0, local = 0, last_end = 0;
    for (uint32_t t = 0; t < num_tensors; ++t) {
        const uint64_t sz = tensor_elems[t];
        if (owner[t] == rank && sz > 0) {
            if (count > 0 && last_end == flat) {
                if (segments != nullptr && count <= capacity) segments[count - 1].length += sz;
            } else {
                if (segments != nullptr && count < capacity) segments[count] = amsp_segment{flat, local, sz};
                ++count;
            }
            local += sz;
            last_end = flat + sz;
        }
        flat += sz;
    }
    *num_segments = count;
    *local_elems = local;
    return (segments != nullptr && count > capacity) ? AMSP_EINVAL : AMSP_OK;
}

static int check_segments(const amsp_segment *segments, uint32_t num_segments, uint64_t flat_elems,
                          uint64_t local_elems) {
    if (num_segments > 0 && segments == nullptr) return AMSP_ENULL;
    for (uint32_t i = 0; i < num_segments; ++i) {
        const amsp_segment &g = segments[i];
        if (g.length > flat_elems || g.flat_offset > flat_elems - g.length) return AMSP_EINVAL;
        if (g.length > local_elems || g.local_offset > local_elems - g.length) return AMSP_EINVAL;
    }
    return AMSP_OK;
}

int amsp_grad_sqnorm_segments(const uint16_t *const *partials_flat, uint32_t k, uint64_t flat_elems,
                              const amsp_segment *segments, uint32_t num_segments, double *d_sqnorm, int accumulate,
                              void *workspace, size_t workspace_bytes, void *stream) {
    PartialPtrs pp;
    int rc = check_partials(partials_flat, k, pp);
    if (rc != AMSP_OK) return rc;
    rc = check_segments(segments, num_segments, flat_elems, UINT64_MAX);
    if (rc != AMSP_OK) return rc;
    if (d_sqnorm == nullptr || workspace == nullptr) return AMSP_ENULL;
    if (misaligned(d_sqnorm, 8) || misaligned(workspace, 8)) return AMSP_EALIGN;
    if (workspace_bytes < amsp_workspace_bytes()) return AMSP_EWORKSPACE;
    NormBatch batch{(hipStream_t)stream, static_cast<double *>(workspace), d_sqnorm, 0, accumulate != 0};
    clear_stale_error();
    bool any = false;
    NormRanges ranges{batch, pp, k, nullptr};
    for (uint32_t i = 0; i < num_segments; ++i) {
        if (segments[i].length == 0) continue;
        rc = ranges.add(segments[i].flat_offset, segments[i].length);
        if (rc != AMSP_OK) return rc;
        any = true;
    }
    rc = ranges.flush();
    if (rc != AMSP_OK) return rc;
    if (!any) {   // nothing owned: same contract as n == 0
        if (!accumulate) return finish_sums(batch.hs, batch.sums, 0, batch.sums + kNormSlots, d_sqnorm, 0);
        return AMSP_OK;
    }
    return batch.flush();
}

int amsp_reduce_grad_segments(const uint16_t *const *partials_flat, uint32_t k, uint64_t flat_elems,
                              const amsp_segment *segments, uint32_t num_segments, uint64_t local_elems,
                              float *grad_f32_local, int accumulate, void *stream) {
    PartialPtrs pp;
    int rc = check_partials(partials_flat, k, pp);
    if (rc != AMSP_OK) return rc;
    rc = check_segments(segments, num_segments, flat_elems, local_elems);
    if (rc != AMSP_OK) return rc;
    for (uint32_t i = 0; i < num_segments; ++i) {
        if (segments[i].length == 0) continue;
        if (grad_f32_local == nullptr) return AMSP_ENULL;
        if (too_long(segments[i].length, 0)) return AMSP_EINVAL;
    }
    if (misaligned(grad_f32_local, 4)) return AMSP_EALIGN;
    hipStream_t hs = (hipStream_t)stream;
    TableBuilder tb;
    auto flush_table = [&]() -> int {
        if (tb.count == 0) return AMSP_OK;
        tb.pad();
        const unsigned lds = occupancy_lds(8 * k + (accumulate ? 16 : 0), reduce_target());
        clear_stale_error();
        hipLaunchKernelGGL(reduce_table_kernel, dim3(tb.blocks), dim3(kRwThreads), lds, hs, pp, (int)k,
                           grad_f32_local, accumulate, tb.table);
        tb.reset();
        return launched();
    };
    for (uint32_t i = 0; i < num_segments; ++i) {
        const amsp_segment &g = segments[i];
        if (g.length == 0) continue;
        PartialPtrs q = offset_partials(pp, k, g.flat_offset);
        if (g.length < kShortSegment) {
            Stream16 st[AMSP_MAX_K + 1];
            int ns = add_partial_streams(st, 0, q, k);
            st[ns++] = Stream16{grad_f32_local + g.local_offset, 4};
            const Span sp = make_span(g.length, st, ns, kVecRW);
            if (TableBuilder::takes(g, sp)) {
                if (tb.add(i, g, sp)) {
                    rc = flush_table();
                    if (rc != AMSP_OK) return rc;
                }
                continue;
            }
        }
        rc = amsp_reduce_grad_shard(q.p, k, g.length, 0, grad_f32_local + g.local_offset, accumulate, nullptr, 0,
                                    nullptr, 0, stream);
        if (rc != AMSP_OK) return rc;
    }
    return flush_table();
}

size_t amsp_amax_workspace_bytes(uint32_t num_segments) {
    return (size_t)num_segments * kAmaxWordsPerSegment * sizeof(uint32_t);
}

int amsp_adamw_step_segments(const uint16_t *const *partials_flat, uint32_t k, const float *grad_f32_local,
                             uint64_t flat_elems, const amsp_segment *segments, uint32_t num_segments,
                             uint64_t local_elems, float *master_local, float *exp_avg_local,
                             float *exp_avg_sq_local, uint16_t *param_bf16_flat, float *d_amax,
                             void *amax_workspace, size_t amax_workspace_bytes, const amsp_adamw_hparams *hp,
                             void *stream) {
    PartialPtrs pp{};
    int rc = AMSP_OK;
    if (k > 0) {
        rc = check_partials(partials_flat, k, pp);
        if (rc != AMSP_OK) return rc;
    }
    rc = check_segments(segments, num_segments, flat_elems, local_elems);
    if (rc != AMSP_OK) return rc;
    AdamConsts c;
    rc = adam_consts(hp, c);
    if (rc != AMSP_OK) return rc;
    uint32_t *words = nullptr;
    if (d_amax != nullptr && num_segments > 0) {
        if (amax_workspace == nullptr) return AMSP_ENULL;
        if (misaligned(d_amax, 4) || misaligned(amax_workspace, 4)) return AMSP_EALIGN;
        if (amax_workspace_bytes < amsp_amax_workspace_bytes(num_segments)) return AMSP_EWORKSPACE;
        if ((size_t)num_segments * kAmaxWordsPerSegment > 0xFFFFFFFFull) return AMSP_EINVAL;
        words = static_cast<uint32_t *>(amax_workspace);
    }
    for (uint32_t i = 0; i < num_segments; ++i) {
        if (segments[i].length == 0) continue;
        if (master_local == nullptr || exp_avg_local == nullptr || exp_avg_sq_local == nullptr ||
            (k == 0 && grad_f32_local == nullptr))
            return AMSP_ENULL;
        if (too_long(segments[i].length, 0)) return AMSP_EINVAL;
    }
    if (misaligned(master_local, 4) || misaligned(exp_avg_local, 4) || misaligned(exp_avg_sq_local, 4) ||
        (k == 0 && misaligned(grad_f32_local, 4)) || (param_bf16_flat && misaligned(param_bf16_flat, 2)))
        return AMSP_EALIGN;
    // everything checked: from here on work is enqueued
    hipStream_t hs = (hipStream_t)stream;
    if (words != nullptr) {   // the maxima start from +0, the smallest |x| pattern
        const size_t count = (size_t)num_segments * kAmaxWordsPerSegment;
        clear_stale_error();
        const unsigned blocks = (unsigned)((count + kThreads - 1) / kThreads);
        hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks > 1024 ? 1024 : blocks), dim3(kThreads), 0, hs, words,
                           (uint32_t)count, 0u);
        if (launched() != AMSP_OK) return AMSP_EDEVICE;
    }
    // Segments shorter than kShortSegment share launches, up to kMaxTableRanges each (a launch costs more
    // than such a segment's traffic); the others get a launch of their own with every k loaded at once.
    TableBuilder tb;
    auto flush_table = [&]() -> int {
        if (tb.count == 0) return AMSP_OK;
        tb.pad();
        const unsigned lane_bytes = (k != 0 ? 8 * k : 16) + 48;
        const unsigned lds = occupancy_lds(lane_bytes, adamw_target(lane_bytes));
        const dim3 grid(tb.blocks), block(kRwThreads);
        clear_stale_error();
#define AMSP_LAUNCH_TABLE(KV, B16, AM)                                                                          \
        hipLaunchKernelGGL((adamw_table_kernel<KV, B16, AM>), grid, block, lds, hs, pp, (int)k, grad_f32_local, \
                           master_local, exp_avg_local, exp_avg_sq_local, param_bf16_flat, words, c, tb.table)
#define AMSP_LAUNCH_TABLE_K(KV)                                                                                  \
        if (param_bf16_flat) { if (words) AMSP_LAUNCH_TABLE(KV, true, true); else AMSP_LAUNCH_TABLE(KV, true, false); } \
        else { if (words) AMSP_LAUNCH_TABLE(KV, false, true); else AMSP_LAUNCH_TABLE(KV, false, false); }
        if (k == 0) { AMSP_LAUNCH_TABLE_K(0) } else { AMSP_LAUNCH_TABLE_K(-1) }
#undef AMSP_LAUNCH_TABLE_K
#undef AMSP_LAUNCH_TABLE
        tb.reset();
        return launched();
    };
    for (uint32_t i = 0; i < num_segments; ++i) {
        const amsp_segment &g = segments[i];
        if (g.length == 0) continue;
        PartialPtrs q = offset_partials(pp, k, g.flat_offset);
        const float *gf = k == 0 ? grad_f32_local + g.local_offset : nullptr;
        if (g.length < kShortSegment) {
            Stream16 st[AMSP_MAX_K + 5];
            int ns = add_partial_streams(st, 0, q, k);
            if (k == 0) st[ns++] = Stream16{gf, 4};
            st[ns++] = Stream16{master_local + g.local_offset, 4};
            st[ns++] = Stream16{exp_avg_local + g.local_offset, 4};
            st[ns++] = Stream16{exp_avg_sq_local + g.local_offset, 4};
            if (param_bf16_flat) st[ns++] = Stream16{param_bf16_flat + g.flat_offset, 2};
            const Span sp = make_span(g.length, st, ns, kVecRW);
            if (TableBuilder::takes(g, sp)) {
                if (tb.add(i, g, sp)) {
                    rc = flush_table();
                    if (rc != AMSP_OK) return rc;
                }
                continue;
            }
        }
        rc = adamw_step_range(q.p, k, gf, g.length, 0, master_local + g.local_offset,
                              exp_avg_local + g.local_offset, exp_avg_sq_local + g.local_offset,
                              param_bf16_flat ? param_bf16_flat + g.flat_offset : nullptr,
                              words ? words + (size_t)i * kAmaxWordsPerSegment : nullptr, hp, stream);
        if (rc != AMSP_OK) return rc;
    }
    rc = flush_table();
    if (rc != AMSP_OK) return rc;
    if (words != nullptr) {
        clear_stale_error();
        hipLaunchKernelGGL(amax_fold_kernel, dim3(num_segments), dim3(kAmaxSubSlots), 0, hs, words,
                           reinterpret_cast<uint32_t *>(d_amax));
        return launched();
    }
    return AMSP_OK;
}

// ---------------------------------------------------------------- FP8 payload entry points
int amsp_cast_param_fp8_shard(const float *master, uint64_t n, const float *d_scale, uint8_t *param_fp8_out,
                              void *stream) {
    if (n == 0) return AMSP_OK;
    if (too_long(n, 0)) return AMSP_EINVAL;
    if (master == nullptr || d_scale == nullptr || param_fp8_out == nullptr) return AMSP_ENULL;
    if (misaligned(master, 4) || misaligned(d_scale, 4)) return AMSP_EALIGN;
    Stream16 st[2] = {{master, 4}, {param_fp8_out, 1}};
    Span s = make_span(n, st, 2, 4);
    clear_stale_error();
    const RwLaunch L = rw_launch(s, 16, adamw_target(16));
    hipLaunchKernelGGL(cast_fp8_kernel, L.grid, L.block, L.lds, (hipStream_t)stream, master, d_scale, param_fp8_out, s);
    return launched();
}

int amsp_fp8_payload_segments(const float *master_local, uint64_t local_elems, const amsp_segment *segments,
                              uint32_t num_segments, uint64_t flat_elems, uint8_t *param_fp8_flat, float *d_amax,
                              int amax_ready, float *d_scale, void *stream) {
    int rc = check_segments(segments, num_segments, flat_elems, local_elems);
    if (rc != AMSP_OK) return rc;
    if (num_segments == 0) return AMSP_OK;
    if (master_local == nullptr || param_fp8_flat == nullptr || d_amax == nullptr || d_scale == nullptr) return AMSP_ENULL;
    if (misaligned(master_local, 4) || misaligned(d_amax, 4) || misaligned(d_scale, 4)) return AMSP_EALIGN;
    hipStream_t hs = (hipStream_t)stream;
    uint32_t *slots = reinterpret_cast<uint32_t *>(d_amax);
    clear_stale_error();
    // short segments share launches (tables of kMaxTableRanges); `cast` selects the pass
    TableBuilder tb;
    auto flush_table = [&](bool cast) -> int {
        if (tb.count == 0) return AMSP_OK;
        tb.pad();
        if (cast)
            hipLaunchKernelGGL((fp8_table_kernel<true>), dim3(tb.blocks), dim3(kRwThreads), 0, hs, master_local,
                               d_scale, param_fp8_flat, slots, tb.table);
        else
            hipLaunchKernelGGL((fp8_table_kernel<false>), dim3(tb.blocks), dim3(kRwThreads), 0, hs, master_local,
                               d_scale, param_fp8_flat, slots, tb.table);
        tb.reset();
        return launched();
    };
    // true when segment i went into the table
    auto tabled = [&](uint32_t i, bool cast, int *rc_out) -> bool {
        const amsp_segment &g = segments[i];
        if (g.length >= kShortSegment) return false;
        Stream16 st[2] = {{master_local + g.local_offset, 4}, {param_fp8_flat + g.flat_offset, 1}};
        const Span sp = make_span(g.length, st, cast ? 2 : 1, 4);
        if (!TableBuilder::takes(g, sp)) return false;
        *rc_out = tb.add(i, g, sp) ? flush_table(cast) : (int)AMSP_OK;
        return true;
    };
    if (!amax_ready) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(kThreads), 0, hs, slots, num_segments, 0u);
        if (launched() != AMSP_OK) return AMSP_EDEVICE;
        for (uint32_t i = 0; i < num_segments; ++i) {
            if (segments[i].length == 0) continue;
            if (tabled(i, false, &rc)) {
                if (rc != AMSP_OK) return rc;
                continue;
            }
            const float *x = master_local + segments[i].local_offset;
            Stream16 st[1] = {{x, 4}};
            Span s = make_span(segments[i].length, st, 1, 4);
            hipLaunchKernelGGL(absmax_kernel, dim3(norm_grid(s)), dim3(kNormThreads), 0, hs, x, s, slots + i);
            if (launched() != AMSP_OK) return AMSP_EDEVICE;
        }
        rc = flush_table(false);
        if (rc != AMSP_OK) return rc;
    }
    hipLaunchKernelGGL(fp8_scale_kernel, dim3(1), dim3(kThreads), 0, hs, d_amax, d_scale, num_segments);
    if (launched() != AMSP_OK) return AMSP_EDEVICE;
    for (uint32_t i = 0; i < num_segments; ++i) {
        if (segments[i].length == 0) continue;
        if (tabled(i, true, &rc)) {
            if (rc != AMSP_OK) return rc;
            continue;
        }
        rc = amsp_cast_param_fp8_shard(master_local + segments[i].local_offset, segments[i].length, d_scale + i,
                                       param_fp8_flat + segments[i].flat_offset, stream);
        if (rc != AMSP_OK) return rc;
    }
    return flush_table(true);
}

}  // extern "C"
