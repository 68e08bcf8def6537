// Device side of the model-state step: memory-access helpers, the reduced gradient, and the kernels
// (cast, reduce, squared norm, AdamW, their table-driven forms for short ranges, the FP8 payload).
// Included once, by amsp_kernels.hip, which holds the launch logic and the C ABI; everything here
// lives in that file's anonymous namespace.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

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
constexpr int kNormThreads = 64;       // the norm pass runs one-wave blocks, a few per CU (norm_waves_per_cu)
constexpr int kWideThreads = 1024;     // 16-wave blocks: the short-range norm kernel
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
// K > 0: k == K known at compile time (all loads issued up front); K < 0: run-time k (unrolled to a bound
// with uniform guards, see grad_vec); K == 0: the gradient is already reduced, read it as fp32.
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
        // run-time k, unrolled to a bound with wave-uniform guards, so that here too every load is in flight
        // before the first wait (a loop that loads and adds in turn reads 3.6-4.3 TB/s in the fused step at
        // k = 17..32).  K == -1: any k, every load guarded (the table kernels, where k is usually small);
        // K == -20, -24, -28, -32: k in (|K| - 4, |K|], only the last four loads guarded.
        constexpr int BOUND = K == -1 ? (int)AMSP_MAX_K : -K;
        constexpr int SURE = K == -1 ? 0 : BOUND - 4;   // partials known to exist
        static_assert(BOUND >= 4 && BOUND <= (int)AMSP_MAX_K, "unroll bound of the run-time k path");
        W w[BOUND];
#pragma unroll
        for (int j = 0; j < BOUND; ++j)
            if (j < SURE || j < k) w[j] = ld_stream(reinterpret_cast<const W *>(pp.p[j] + e));
        loads_issued();
        widen_first<VEC>(w[0], g);
#pragma unroll
        for (int j = 1; j < BOUND; ++j)
            if (j < SURE || j < k) widen_add<VEC>(w[j], g);
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
static_assert(kRwThreads == amsp_geom::kWaveLanes && kNormThreads == amsp_geom::kWaveLanes, "the geometry assumes one-wave workgroups on the vector path");

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
// Vectors per lane and block: with few partials one vector per lane leaves too little in flight even at 32
// waves per CU (k = 1, 6.7 G elements: 5,180 GB/s; two per lane 6,400, four 6,470-6,490 at 24-28 waves).
constexpr int reduce_rows(int k) { return k == 1 ? 4 : (k == 2 || k == 3) ? 2 : 1; }

template <int K, bool NORM>
__global__ void __launch_bounds__(kThreads) reduce_kernel(PartialPtrs pp, int k, float *__restrict__ out,
                                                          int accumulate, double *__restrict__ block_sums, Span s,
                                                          Buckets bk) {
    constexpr int VEC = kVecRW;
    constexpr int R = reduce_rows(K);
    double acc = 0.0;
    if (s.vectorised) {
        uint64_t off;
        uint32_t lb;
        block_range<VEC>(bk, s, off, lb);
        if constexpr (R > 1) {
            // R consecutive wave pieces per block, every load of every row issued before the first is used
            typedef typename Bf16Words<VEC>::type W;
            const uint64_t v0 = (uint64_t)lb * (kRwThreads * R) + threadIdx.x;
            float o[R][VEC];
            W w[R][K];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint64_t v = v0 + (uint64_t)r * kRwThreads;
                if (v < s.nvec) {
                    const uint64_t e = off + s.head + v * VEC;
                    if (accumulate) ld_f32<VEC>(out, e, o[r]);
#pragma unroll
                    for (int j = 0; j < K; ++j) w[r][j] = ld_stream(reinterpret_cast<const W *>(pp.p[j] + e));
                }
            }
            loads_issued();
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint64_t v = v0 + (uint64_t)r * kRwThreads;
                if (v < s.nvec) {
                    float g[VEC];
                    widen_first<VEC>(w[r][0], g);
#pragma unroll
                    for (int j = 1; j < K; ++j) widen_add<VEC>(w[r][j], g);
                    if (accumulate) {
#pragma unroll
                        for (int c = 0; c < VEC; ++c) g[c] = o[r][c] + g[c];
                    }
                    st_f32<VEC>(out, off + s.head + v * VEC, g);
                    if constexpr (NORM) {
#pragma unroll
                        for (int c = 0; c < VEC; ++c) acc = fma((double)g[c], (double)g[c], acc);
                    }
                }
            }
        }
        const uint64_t v = (uint64_t)lb * kRwThreads + threadIdx.x;
        if (R == 1 && v < s.nvec) {
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

// Shape of the read-only pass, per k (measured on MI355X, GB/s of the pass): a persistent grid of
// one-wave blocks, norm_waves_per_cu of them per CU (one per SIMD: 4), each taking per trip
// norm_unroll consecutive wave pieces (64 lanes x 16 bytes) of every stream, all loads issued before the
// first is used.  k = 1: 7,410 at 8 pieces per trip against 5,440 at 4; k = 2: 7,330 at 4, 6,820 at 8;
// k = 3..8: 6,950-7,090 at 8, 1 % less at 4; k = 10..16: 7,090-7,150 at 4.  The earlier shape (two
// 1024-thread blocks per CU, one vector per lane and trip) read 6,100-6,830.  More waves per CU lose:
// k = 8 reads 7,060 at 4 waves, 7,000 at 6-8; pieces a grid stride apart instead of consecutive lose up
// to 15 % at strides that are multiples of 2 MiB.
template <int K>
constexpr int norm_unroll() {
    return K < 0 ? 1 : (K == 2 || K > 8) ? 4 : 8;
}
constexpr int norm_waves_per_cu(int K) { return K < 0 ? 8 : 4; }   // run-time k (> 16): a sequential loop over j, so more waves

// acc += sum of g^2 over one range, its vectors visited as amsp_geom::norm_walk lays down.
// The range's head and tail (element by element, a few trips of one wave) go to block `edge_block`:
// a different block for every range of a launch, so that no block collects the edges of all of them.
template <int K, int VEC>
__device__ __forceinline__ double sqnorm_span(const PartialPtrs &pp, int k, const float *__restrict__ gf32,
                                              const uint64_t base, const Span &s, const uint32_t edge_block,
                                              double acc) {
    constexpr int U = norm_unroll<K>();
    if (s.vectorised) {
        constexpr int KS = K <= 0 ? 1 : K;
        typedef typename Bf16Words<VEC == 8 ? 8 : 4>::type W;
        const uint64_t first = base + s.head;
        // one trip: U vectors (with `guarded`, those of them that exist), every load in flight before the first is used
        auto trip = [&](uint64_t v, auto guarded) {
            constexpr bool G = decltype(guarded)::value;
            if constexpr (K < 0) {   // run-time k: U == 1
                float g[VEC];
                grad_vec<K, VEC>(pp, k, gf32, first + v * VEC, g);
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc = fma((double)g[c], (double)g[c], acc);
            } else {
                f32x4 a[U];
                W w[U][KS];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint64_t x = v + (uint64_t)u * kNormThreads;
                    if (G && x >= s.nvec) continue;
                    const uint64_t e = first + x * VEC;
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
                    if (G && v + (uint64_t)u * kNormThreads >= s.nvec) continue;
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
        };
        amsp_geom::norm_walk<U>(
            s.nvec, gridDim.x, blockIdx.x, threadIdx.x, [&](uint64_t v) { trip(v, std::false_type{}); },
            [&](uint64_t v) { trip(v, std::true_type{}); });
        if (blockIdx.x == edge_block)
            for (uint32_t t = threadIdx.x; t < s.head + s.tail; t += kNormThreads) {
                const double g = (double)grad1<K>(pp, k, gf32, base + edge_elem<VEC>(s, t));
                acc = fma(g, g, acc);
            }
    } else {
        // streams without a common vector phase: an element per lane, eight grid rows per trip so that a
        // lane has eight elements' loads in flight (one per trip reads 1.9 TB/s at k = 8)
        constexpr int E = 8;
        const uint64_t row = (uint64_t)gridDim.x * kNormThreads;
        uint64_t i = (uint64_t)blockIdx.x * kNormThreads + threadIdx.x;
        for (; i + (E - 1) * row < s.n; i += E * row) {
            float g[E];
#pragma unroll
            for (int u = 0; u < E; ++u) g[u] = grad1<K>(pp, k, gf32, base + i + u * row);
#pragma unroll
            for (int u = 0; u < E; ++u) acc = fma((double)g[u], (double)g[u], acc);
        }
        for (; i < s.n; i += row) {
            const double g = (double)grad1<K>(pp, k, gf32, base + i);
            acc = fma(g, g, acc);
        }
    }
    return acc;
}

template <int K, int VEC>
__global__ void __launch_bounds__(kNormThreads) sqnorm_kernel(PartialPtrs pp, int k, const float *__restrict__ gf32,
                                                              double *__restrict__ block_sums, NormSegTable t) {
    double acc = 0.0;
    for (int i = 0; i < t.count; ++i)
        acc = sqnorm_span<K, VEC>(pp, k, gf32, t.seg[i].base, t.seg[i].s, (uint32_t)i % gridDim.x, acc);
    acc = wave_sum(acc);   // the block is one wave
    if (threadIdx.x == 0) block_sums[blockIdx.x] = acc;
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
__global__ void __launch_bounds__(kWideThreads) sqnorm_short_kernel(PartialPtrs pp, int k,
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
        const uint64_t v = (uint64_t)lb * kWideThreads + threadIdx.x;
        if (v < s.nvec) {
            float g[VEC];
            grad_vec<K, VEC>(pp, k, gf32, base + s.head + v * VEC, g);
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc = fma((double)g[c], (double)g[c], acc);
        }
        if (lb == 0)
            for (uint32_t e = threadIdx.x; e < s.head + s.tail; e += kWideThreads) {
                const double g = (double)grad1<K>(pp, k, gf32, base + edge_elem<VEC>(s, e));
                acc = fma(g, g, acc);
            }
    } else {
        const uint64_t stride = (uint64_t)t.blocks[r] * kWideThreads;
        for (uint64_t i = (uint64_t)lb * kWideThreads + threadIdx.x; i < s.n; i += stride) {
            const double g = (double)grad1<K>(pp, k, gf32, base + i);
            acc = fma(g, g, acc);
        }
    }
    const double total = block_sum<kWideThreads>(acc);
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

__global__ void __launch_bounds__(kThreads) fill_u32_kernel(uint32_t *p, uint64_t count, uint32_t value) {
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;   // 64-bit index: no wrap-around however long the list
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += stride) p[i] = value;
}

// Largest |x| of up to kMaxNormSegs ranges, each into its own slot (integer atomic max: exact and order-free),
// in one launch (a launch per tensor reads a third slower: tensors of 17-130 M elements are 10-80 us of
// traffic each).  The shape of the norm pass: resident one-wave blocks, 8 consecutive wave pieces per trip with
// every load in flight before the first is used.  Every range has blocks of its own, in proportion to its
// length, which walk it like a grid of that size: one atomic per block.  (All blocks walking all ranges in
// turn send 32 times as many; the slots share a memory channel, where each atomic takes ~11 ns, and the
// pass then reads 5.4 TB/s instead of 7.)
struct AbsmaxTable {
    uint32_t first_block[kMaxNormSegs];   // unused entries: 0xFFFFFFFF
    uint32_t blocks[kMaxNormSegs];
    uint32_t slot[kMaxNormSegs];
    NormSeg seg[kMaxNormSegs];
};

__global__ void __launch_bounds__(kNormThreads) absmax_kernel(const float *__restrict__ x,
                                                              uint32_t *__restrict__ slots, AbsmaxTable t) {
    constexpr int VEC = 4, U = 8;
    uint32_t r = 0;
#pragma unroll
    for (int i = 1; i < kMaxNormSegs; ++i) r += blockIdx.x >= t.first_block[i] ? 1u : 0u;
    const uint32_t lb = blockIdx.x - t.first_block[r], grid = t.blocks[r];
    const Span s = t.seg[r].s;
    const uint64_t base = t.seg[r].base;
    uint32_t m = 0;
    if (s.vectorised) {
        const uint64_t first = base + s.head;
        auto trip = [&](uint64_t v, auto guarded) {
            constexpr bool G = decltype(guarded)::value;
            f32x4 a[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint64_t y = v + (uint64_t)u * kNormThreads;
                if (G && y >= s.nvec) continue;
                a[u] = ld_stream(reinterpret_cast<const f32x4 *>(x + first + y * VEC));
            }
            loads_issued();
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (G && v + (uint64_t)u * kNormThreads >= s.nvec) continue;
                m = max(max(m, max(abs_bits(a[u].x), abs_bits(a[u].y))), max(abs_bits(a[u].z), abs_bits(a[u].w)));
            }
        };
        amsp_geom::norm_walk<U>(
            s.nvec, grid, lb, threadIdx.x, [&](uint64_t v) { trip(v, std::false_type{}); },
            [&](uint64_t v) { trip(v, std::true_type{}); });
        if (lb == 0)
            for (uint32_t e = threadIdx.x; e < s.head + s.tail; e += kNormThreads)
                m = max(m, abs_bits(x[base + edge_elem<VEC>(s, e)]));
    } else {
        const uint64_t row = (uint64_t)grid * kNormThreads;
        for (uint64_t e = (uint64_t)lb * kNormThreads + threadIdx.x; e < s.n; e += row)
            m = max(m, abs_bits(x[base + e]));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_down((int)m, off, 64));
    if (threadIdx.x == 0 && m != 0) atomicMax(slots + t.slot[r], m);   // slots start at 0
}

// scale[i] = 448 / amax[i] in fp32 (correctly rounded division); 1 when amax is 0, Inf or NaN.
__global__ void __launch_bounds__(kThreads) fp8_scale_kernel(const float *__restrict__ amax, float *__restrict__ scale,
                                                             uint32_t count) {
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += stride) {
        const float a = amax[i];
        scale[i] = (a > 0.0f && a < __uint_as_float(0x7F800000u)) ? 448.0f / a : 1.0f;
    }
}

// E4M3 codes of up to kMaxNormSegs ranges in one launch (a launch per tensor loses a fifth of the rate to the
// starts and ends of 10-30 us kernels).  One-wave blocks of 1024 elements, each belonging to one range, found
// with 31 scalar compares against the table in the kernel arguments.  On the vector path: four 16-byte loads
// per lane (four gap-free 1 KiB rows per wave), and, when the output allows 16-byte accesses (`wide`), the
// four code words of a lane's rows are exchanged through 1 KiB of LDS so that every lane stores 16
// consecutive codes: one gap-free 1 KiB store per wave instead of four 256-byte ones.
constexpr int kFp8Rows = 4;   // a multiple of 4
constexpr uint32_t kFp8BlockElems = kFp8Rows * kRwThreads * 4;
struct Fp8CastTable {
    uint32_t first_block[kMaxNormSegs];   // unused entries: 0xFFFFFFFF
    uint32_t scale[kMaxNormSegs];         // index into d_scale
    uint32_t wide;                        // bit i: range i's vector path may store 16 bytes at a time
    uint64_t master_off[kMaxNormSegs], out_off[kMaxNormSegs];
    Span s[kMaxNormSegs];
};

__global__ void __launch_bounds__(kRwThreads) cast_fp8_kernel(const float *__restrict__ master_all,
                                                              const float *__restrict__ d_scale,
                                                              uint8_t *__restrict__ out_all, Fp8CastTable t) {
    constexpr int VEC = 4;
    uint32_t r = 0;
#pragma unroll
    for (int i = 1; i < kMaxNormSegs; ++i) r += blockIdx.x >= t.first_block[i] ? 1u : 0u;
    const uint32_t lb = blockIdx.x - t.first_block[r];
    const Span s = t.s[r];
    const float *__restrict__ master = master_all + t.master_off[r];
    uint8_t *__restrict__ out = out_all + t.out_off[r];
    const float scale = d_scale[t.scale[r]];
    if (s.vectorised) {
        __shared__ uint32_t tile[kFp8Rows * kRwThreads];
        const uint64_t v0 = (uint64_t)lb * (kFp8Rows * kRwThreads);
        float x[kFp8Rows][VEC];
#pragma unroll
        for (int row = 0; row < kFp8Rows; ++row) {
            const uint64_t v = v0 + row * kRwThreads + threadIdx.x;
            if (v < s.nvec) ld_f32<VEC>(master, s.head + v * VEC, x[row]);
        }
        loads_issued();
        uint32_t w[kFp8Rows];
#pragma unroll
        for (int row = 0; row < kFp8Rows; ++row) {
            w[row] = 0;
            if (v0 + row * kRwThreads + threadIdx.x < s.nvec) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) w[row] |= f32_to_e4m3(x[row][c] * scale) << (8 * c);
            }
        }
        if ((t.wide >> r) & 1u) {
#pragma unroll
            for (int row = 0; row < kFp8Rows; ++row) tile[row * kRwThreads + threadIdx.x] = w[row];
            __syncthreads();   // one wave: orders the LDS writes before the reads below
#pragma unroll
            for (int j = 0; j < kFp8Rows / 4; ++j) {
                const u32x4 q = reinterpret_cast<const u32x4 *>(tile)[j * kRwThreads + threadIdx.x];
                // the lane's four vectors of this store: 16 consecutive codes, 1 KiB gap-free per wave
                const uint64_t first = v0 + (uint64_t)(j * kRwThreads + threadIdx.x) * 4;
                uint8_t *dst = out + s.head + first * VEC;
                if (first + 4 <= s.nvec) {
                    st_stream(reinterpret_cast<u32x4 *>(dst), q);
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (first + c < s.nvec) st_stream(reinterpret_cast<uint32_t *>(dst + 4 * c), q[c]);
                }
            }
        } else {
#pragma unroll
            for (int row = 0; row < kFp8Rows; ++row) {
                const uint64_t v = v0 + row * kRwThreads + threadIdx.x;
                if (v < s.nvec) st_stream(reinterpret_cast<uint32_t *>(out + s.head + v * VEC), w[row]);
            }
        }
        if (lb == 0)
            for (uint32_t e = threadIdx.x; e < s.head + s.tail; e += kRwThreads) {
                const uint64_t i = edge_elem<VEC>(s, e);
                out[i] = (uint8_t)f32_to_e4m3(master[i] * scale);
            }
    } else {   // no common 4-element phase of input and output: a code per lane, 1024 per block
        const uint64_t i0 = (uint64_t)lb * kFp8BlockElems + threadIdx.x;
#pragma unroll 4
        for (uint32_t c = 0; c < kFp8BlockElems / kRwThreads; ++c) {
            const uint64_t i = i0 + (uint64_t)c * kRwThreads;
            if (i < s.n) out[i] = (uint8_t)f32_to_e4m3(master[i] * scale);
        }
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

}  // namespace
