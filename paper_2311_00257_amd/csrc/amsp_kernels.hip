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
#include "amsp_device.h"

namespace {

// ---------------------------------------------------------------- host side
typedef amsp_geom::Stream Stream16;
using amsp_geom::make_span;
using amsp_geom::make_buckets;

using amsp_geom::for_pieces;
using amsp_geom::kMaxLaunchBlocks;
using amsp_geom::kMaxLaunchElems;

// Calls f(off, len, U), one call per launch.  U == 0: a launch over the single range [off, off + len),
// len <= kMaxLaunchElems (a flat range, or a bucket, longer than that is cut into pieces).  U > 0: a launch
// over the buckets of U elements of [off, off + len): as many buckets as kMaxLaunchBlocks workgroups allow.
template <typename F>
int for_bucket_launches(uint64_t n, uint64_t bucket_elems, F f) {
    auto piece = [&](uint64_t off, uint64_t len) { return f(off, len, (uint64_t)0); };
    if (bucket_elems == 0 || bucket_elems >= n) return for_pieces(0, n, kMaxLaunchElems, piece);
    if (bucket_elems >= kMaxLaunchElems) {   // every bucket needs several launches of its own
        for (uint64_t off = 0; off < n; off += bucket_elems) {
            const int rc = for_pieces(off, n - off < bucket_elems ? n - off : bucket_elems, kMaxLaunchElems, piece);
            if (rc != AMSP_OK) return rc;
        }
        return AMSP_OK;
    }
    const uint64_t blocks_per_bucket = bucket_elems / ((uint64_t)kRwThreads * kVecRW) + 1;   // <= kMaxLaunchBlocks
    const uint64_t per_launch = kMaxLaunchBlocks / blocks_per_bucket;                          // >= 1
    const uint64_t step = per_launch * bucket_elems;                                           // < 2^34: no overflow
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
    int inflight_kib, min_waves;
};
constexpr RwKnobs kRwKnobs{40, 8};   // the AdamW kernels: what the sweeps on MI355X settled on
#ifdef AMSP_TUNING
// Sweep builds only (never the shipped library): the two numbers, or the wave count itself, can be
// overridden from the environment, read at every call so that one process can alternate settings.
// They change launch shapes, never results.
int env_knob(const char *name, int lo, int hi, int dflt) {
    const char *v = getenv(name);
    const int x = v ? atoi(v) : 0;
    return (x >= lo && x <= hi) ? x : dflt;
}
RwKnobs rw_knobs() {
    return RwKnobs{env_knob("AMSP_INFLIGHT_KIB", 8, 1024, kRwKnobs.inflight_kib),
                   env_knob("AMSP_MIN_WAVES", 4, 32, kRwKnobs.min_waves)};
}
int forced_waves() { return env_knob("AMSP_FORCE_WAVES", 3, 32, 0); }
#else
constexpr const RwKnobs &rw_knobs() { return kRwKnobs; }
constexpr int forced_waves() { return 0; }
#endif

// What a kernel family wants in flight per CU and the fewest waves it is given, or (waves > 0) the number of
// waves itself.
struct RwTarget {
    int inflight_kib, min_waves, waves;
};
// AdamW kernels: 40 KiB, at least 8 waves (10 waves for an fp32 gradient, 12 for k = 1, 8 for k = 4..8); 7 once
// a wave loads more than 7 KiB (fused step with k = 9..13) and 6 from 10 KiB on (k >= 14).  GB/s of the
// fused step at 6 / 7 / 8 / 9 waves, alternated in one process (streams placed 4 KiB apart modulo 8 KiB):
// k = 8: 6,040 / 6,590 / 6,600 / 6,610; k = 9: 6,190 / 6,630 / 6,570 / 6,580; k = 12: 6,510 / 6,590 / 6,490 /
// 6,480; k = 14: 6,550 / 6,500 / 6,430 / 6,400; k = 16: 6,480 / 6,430 / 6,340 / 6,360.
RwTarget adamw_target(unsigned load_bytes_per_lane) {
    const unsigned per_wave = 64u * load_bytes_per_lane;
    const int floor = rw_knobs().min_waves - (per_wave > 7168u ? 1 : 0) - (per_wave >= 10240u ? 1 : 0);
    return RwTarget{rw_knobs().inflight_kib, floor, 0};
}
// Reduction (its writes are a small share of the traffic): as many waves as keep 60 KiB of the partials in
// flight per CU, between 9 and 24; two more when the fp32 buffer is read too.  k = 1..3, where a block takes
// reduce_rows(k) vectors per lane: 20-22 (k = 1: 6,400 at 20-24, 6,120 at 32, 5,400 at 12; k = 2: 6,260 at
// 20, 6,370-6,415 at 24-28; k = 3: 6,495 at 20, 6,110 at 32), 16 with accumulate (6,360 / 6,270 / 6,520
// against 6,050 / 5,870 / 5,710 at 32).  GB/s of the
// reduce+norm pass by waves per CU (streams placed 4 KiB apart modulo 8 KiB): k = 4: 5,570 at 16, 6,740 at 24,
// 6,560 at 32; k = 8: 5,830 at 10, 6,610 at 13, 6,630 at 14-16, 6,440 at 20; k = 12: 5,900 at 8, 6,395 at 10,
// 6,300 at 13; k = 16: 5,935 at 7, 6,315 at 9, 6,145 at 12; with accumulate k = 8: 6,140 at 13, 6,460 at 16;
// k = 16: 6,060 at 9, 6,270 at 10-12.
RwTarget reduce_target(uint32_t k, bool accumulate) {
    if (k <= 3) return RwTarget{0, 0, accumulate ? 16 : (k == 3 ? 20 : 22)};
    int waves = (int)((120u + k - 1) / k);   // ceil(60 KiB / (64 lanes x 8 k bytes))
    waves = waves < 9 ? 9 : (waves > 24 ? 24 : waves);
    if (accumulate && waves < 23) waves += 2;
    return RwTarget{0, 0, waves};
}

int rw_waves_per_cu(unsigned load_bytes_per_lane, RwTarget t) {
    const unsigned per_wave = 64u * load_bytes_per_lane;
    int waves = t.waves;
    if (waves <= 0) {
        waves = (int)(((unsigned)t.inflight_kib * 1024u + per_wave - 1) / per_wave);
        if (waves < t.min_waves) waves = t.min_waves;
    }
    if (forced_waves() > 0) waves = forced_waves();
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
    uint64_t blocks = (work + threads - 1) / threads;   // <= kMaxLaunchBlocks: longer ranges come in pieces
    if (blocks == 0) blocks = 1;
    return RwLaunch{dim3((unsigned)blocks), dim3(threads),
                    s.vectorised ? occupancy_lds(load_bytes_per_lane, t) : 0u};
}

// Reduce with the norm fused in: every block leaves one double.  One-wave blocks of one vector per
// lane on the vector path (a sum per 256 elements), a capped grid-stride grid on the element-wise path.
constexpr int kSliceBlocks = 256;

uint64_t reduce_norm_grid(const Span &s, uint32_t k) {
    uint64_t blocks;
    if (s.vectorised) {
        const uint64_t per_block = (uint64_t)kRwThreads * reduce_rows((int)k);
        blocks = (s.nvec + per_block - 1) / per_block;
    } else {
        blocks = (s.n + kThreads - 1) / kThreads;
        if (blocks > (uint64_t)kNormBlocks) blocks = kNormBlocks;
    }
    return blocks == 0 ? 1 : blocks;
}

// Upper bound of the block sums one range of `len` elements leaves, over every alignment: one per 256
// elements and two more (a ragged head and tail) for each launch the range is cut into.
uint64_t reduce_norm_blocks_max(uint64_t len) {
    return len / ((uint64_t)kRwThreads * kVecRW) + 2 * (len / kMaxLaunchElems + 1);
}

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

// The norm pass: norm_waves_per_cu one-wave blocks per CU, at most kNormBlocks; `work` = lanes' worth of
// vectors (or elements on the element-wise path).  kk = the kernel's K (-1: run-time k).
int norm_grid(uint64_t work, int kk) {
    uint64_t blocks = (work + kNormThreads - 1) / kNormThreads;
    uint64_t cap = (uint64_t)norm_waves_per_cu(kk) * (uint64_t)cu_count();
    if (cap > kNormBlocks) cap = kNormBlocks;
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
// share four, unrolled to 20, 24, 28 and 32 partials with the last four loads guarded.
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
        default:                                                          \
            if (k <= 20) { constexpr int KK = -20; CALL; }                \
            else if (k <= 24) { constexpr int KK = -24; CALL; }           \
            else if (k <= 28) { constexpr int KK = -28; CALL; }           \
            else { constexpr int KK = -32; CALL; }                        \
            break;                                                        \
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
    const int grid = norm_grid(work, k > 16 ? -1 : (int)k);
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
        uint64_t blocks = t.seg[i].s.vectorised ? (t.seg[i].s.nvec + kWideThreads - 1) / kWideThreads
                                                : (len[i] + kWideThreads - 1) / kWideThreads;
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
        hipLaunchKernelGGL((sqnorm_short_kernel<0, 4>), dim3(blocks_total), dim3(kWideThreads), 0, hs, pp, (int)k, gf,
                           block_sums, t);
    else
        hipLaunchKernelGGL((sqnorm_short_kernel<-1, kVecNorm>), dim3(blocks_total), dim3(kWideThreads), 0, hs, pp,
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
// takes all of it; everything else gets a launch of its own (the update and the reduction) or shares the
// launches of the long segments (the FP8 maxima and codes).
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

// Collects ranges for cast_fp8_kernel: kMaxNormSegs to a launch, a range longer than one launch cut first.
struct Fp8CastBatch {
    const float *master;
    const float *d_scale;
    uint8_t *out;
    hipStream_t hs;
    Fp8CastTable table;
    uint32_t count = 0;
    uint64_t blocks = 0;

    Fp8CastBatch(const float *m, const float *sc, uint8_t *o, hipStream_t s) : master(m), d_scale(sc), out(o), hs(s) {
        table.wide = 0;
    }
    int flush() {
        if (count == 0) return AMSP_OK;
        for (uint32_t j = count; j < (uint32_t)kMaxNormSegs; ++j) {
            table.first_block[j] = 0xFFFFFFFFu;
            table.scale[j] = 0; table.master_off[j] = 0; table.out_off[j] = 0;
            table.s[j] = Span{0, 0, 0, 0, 0};
        }
        // 24 waves per CU: 6,600 GB/s on 843 M elements against 6,040 at 16 and 6,300 at 32 (8 rows per lane:
        // 6,510 at 16 waves, less above); the kernel's own tile counts towards the cap
        const unsigned lds = occupancy_lds(16 * kFp8Rows, RwTarget{0, 0, 24}) - kFp8Rows * kRwThreads * 4;
        hipLaunchKernelGGL(cast_fp8_kernel, dim3((unsigned)blocks), dim3(kRwThreads), lds, hs, master, d_scale, out, table);
        count = 0;
        blocks = 0;
        table.wide = 0;
        return launched();
    }
    // Range [master_off, +len) of the input to [out_off, +len) of the output, scaled by d_scale[scale_index].
    int add(uint64_t master_off, uint64_t out_off, uint64_t len, uint32_t scale_index) {
        return for_pieces(0, len, kMaxLaunchElems, [&](uint64_t off, uint64_t n) -> int {
            Stream16 st[2] = {{master + master_off + off, 4}, {out + out_off + off, 1}};
            Span s = make_span(n, st, 2, 4);
            if (s.vectorised && s.nvec > 4) {
                // a head up to three vectors longer puts the first stored vector on a 16-byte boundary
                const uint32_t more = (uint32_t)(-(reinterpret_cast<uintptr_t>(out + out_off + off) + s.head) & 15);
                s.head += more;   // a multiple of 4: the loads stay on 16-byte boundaries
                s.nvec = (n - s.head) / 4;
                s.tail = (uint32_t)(n - s.head - s.nvec * 4);
            }
            const uint64_t b = std::max<uint64_t>((n + kFp8BlockElems - 1) / kFp8BlockElems, 1);
            if (blocks + b > kMaxLaunchBlocks) {
                const int rc = flush();
                if (rc != AMSP_OK) return rc;
            }
            table.first_block[count] = (uint32_t)blocks;
            table.scale[count] = scale_index;
            table.master_off[count] = master_off + off;
            table.out_off[count] = out_off + off;
            table.s[count] = s;
            if (s.vectorised && (reinterpret_cast<uintptr_t>(out + out_off + off + s.head) & 15) == 0) table.wide |= 1u << count;
            blocks += b;
            return ++count == (uint32_t)kMaxNormSegs ? flush() : (int)AMSP_OK;
        });
    }
};

}  // namespace

// ---------------------------------------------------------------- the entry point that allocates nothing
// Block sums of amsp_grad_sqnorm_static: one copy of this array per GPU the library runs on, held until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress; the device address
// it yields (one per device) is what kernels and the batch logic are given.
static __device__ __align__(256) double scratch[kNormSlots + kSliceBlocks];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<double *> scratch_address[kMaxDevices];   // per device; null until first asked

// The current device's copy of `scratch`, looked up once per device.
int static_scratch(double **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AMSP_EDEVICE;
    double *p = scratch_address[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        void *addr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || addr == nullptr) {
            fprintf(stderr, "amsp: hipGetSymbolAddress(scratch) failed on device %d: %s\n", dev, hipGetErrorString(e));
            (void)hipGetLastError();
            return AMSP_EDEVICE;
        }
        p = static_cast<double *>(addr);
        scratch_address[dev].store(p, std::memory_order_release);   // any thread may store it: same value
    }
    *out = p;
    return AMSP_OK;
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
        case AMSP_ENOPLAN: return "no sharding plan is feasible";
        case AMSP_ESIZE: return "range longer than the entry point without a workspace supports";
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
    if (master == nullptr || param_bf16_out == nullptr) return AMSP_ENULL;
    if (misaligned(master, 4) || misaligned(param_bf16_out, 2)) return AMSP_EALIGN;
    clear_stale_error();
    return for_pieces(0, n, kMaxLaunchElems, [&](uint64_t off, uint64_t len) -> int {
        Stream16 st[2] = {{master + off, 4}, {param_bf16_out + off, 2}};
        Span s = make_span(len, st, 2, kVecRW);
        const RwLaunch L = rw_launch(s, 16, adamw_target(16));
        hipLaunchKernelGGL(cast_kernel, L.grid, L.block, L.lds, (hipStream_t)stream, master + off,
                           param_bf16_out + off, s);
        return launched();
    });
}

size_t amsp_reduce_workspace_bytes(uint64_t n, uint64_t bucket_elems) {
    return (size_t)(reduce_norm_slots(n, bucket_elems) + kSliceBlocks) * sizeof(double);
}

// Step 1 over a flat range, with step 2 fused in when d_sqnorm != NULL.
static int reduce_range(const uint16_t *const *partials, uint32_t k, uint64_t n, uint64_t bucket_elems,
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
    if (grad_out == nullptr) return AMSP_ENULL;
    if (misaligned(grad_out, 4)) return AMSP_EALIGN;
    uint64_t used = 0;   // block sums written so far, bucket after bucket
    const unsigned lane_bytes = (8 * k + (accumulate ? 16 : 0)) * reduce_rows((int)k);
    auto single = [&](uint64_t off, uint64_t len) -> int {
        PartialPtrs q = offset_partials(pp, k, off);
        Stream16 st[AMSP_MAX_K + 1];
        int ns = add_partial_streams(st, 0, q, k);
        st[ns++] = Stream16{grad_out + off, 4};
        Span s = make_span(len, st, ns, kVecRW);
        const Buckets none{};
        clear_stale_error();
        RwLaunch L = rw_launch(s, lane_bytes, reduce_target(k, accumulate != 0));
        if (s.vectorised) L.grid = dim3((unsigned)reduce_norm_grid(s, k));   // reduce_rows(k) vectors per lane
        if (!norm) {
            AMSP_DISPATCH_K(k, hipLaunchKernelGGL((reduce_kernel<KK, false>), L.grid, L.block, L.lds, hs, q, (int)k,
                                                  grad_out + off, accumulate, block_sums, s, none));
            return launched();
        }
        const uint64_t blocks = reduce_norm_grid(s, k);   // == L.grid.x on the vector path, capped on the other
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
        if (!make_buckets(len, U, st, ns, kVecRW, bk, reduce_rows((int)k)))
            return for_buckets(len, U, [&](uint64_t o, uint64_t l) { return single(off + o, l); });
        const dim3 grid((unsigned)(((len + U - 1) / U) * bk.blocks_per_bucket)), block(kRwThreads);
        const unsigned lds = occupancy_lds(lane_bytes, reduce_target(k, accumulate != 0));
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

int amsp_reduce_grad_shard(const uint16_t *const *partials, uint32_t k, uint64_t n, uint64_t bucket_elems,
                           float *grad_out, int accumulate, void *stream) {
    return reduce_range(partials, k, n, bucket_elems, grad_out, accumulate, nullptr, 0, nullptr, 0, stream);
}

int amsp_reduce_grad_sqnorm_shard(const uint16_t *const *partials, uint32_t k, uint64_t n, uint64_t bucket_elems,
                                  float *grad_out, int accumulate, double *d_sqnorm, int sqnorm_accumulate,
                                  void *workspace, size_t workspace_bytes, void *stream) {
    if (d_sqnorm == nullptr) return AMSP_ENULL;
    return reduce_range(partials, k, n, bucket_elems, grad_out, accumulate, d_sqnorm, sqnorm_accumulate, workspace,
                        workspace_bytes, stream);
}

// Step 2 over a flat range; `sums` is the block-sum buffer ((kNormSlots + kSliceBlocks) doubles, checked by the caller).
static int sqnorm_range(const uint16_t *const *partials, uint32_t k, const float *grad_f32, uint64_t n,
                        uint64_t bucket_elems, double *d_sqnorm, int accumulate, double *sums, void *stream) {
    PartialPtrs pp{};
    if (k > 0) {
        int rc = check_partials(partials, k, pp);
        if (rc != AMSP_OK) return rc;
    } else if (n > 0) {
        if (grad_f32 == nullptr) return AMSP_ENULL;
        if (misaligned(grad_f32, 4)) return AMSP_EALIGN;
    }
    if (d_sqnorm == nullptr) return AMSP_ENULL;
    if (misaligned(d_sqnorm, 8)) return AMSP_EALIGN;
    NormBatch batch{(hipStream_t)stream, sums, d_sqnorm, 0, accumulate != 0};
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

int amsp_grad_sqnorm(const uint16_t *const *partials, uint32_t k, const float *grad_f32, uint64_t n,
                     uint64_t bucket_elems, double *d_sqnorm, int accumulate, void *workspace,
                     size_t workspace_bytes, void *stream) {
    if (k > AMSP_MAX_K) return AMSP_EINVAL;
    if (workspace == nullptr) return AMSP_ENULL;
    if (misaligned(workspace, 8)) return AMSP_EALIGN;
    if (workspace_bytes < amsp_workspace_bytes()) return AMSP_EWORKSPACE;
    return sqnorm_range(partials, k, grad_f32, n, bucket_elems, d_sqnorm, accumulate, static_cast<double *>(workspace),
                        stream);
}

int amsp_grad_sqnorm_static(const uint16_t *const *partials, uint32_t k, const float *grad_f32, uint64_t n,
                            uint64_t bucket_elems, double *d_sqnorm, int accumulate, void *stream) {
    if (k > AMSP_MAX_K) return AMSP_EINVAL;
    if (n > AMSP_STATIC_MAX_ELEMS) {
        fprintf(stderr, "amsp_grad_sqnorm_static: n = %llu exceeds AMSP_STATIC_MAX_ELEMS = %llu; use amsp_grad_sqnorm "
                        "with a workspace\n", (unsigned long long)n, (unsigned long long)AMSP_STATIC_MAX_ELEMS);
        return AMSP_ESIZE;
    }
    double *sums = nullptr;
    const int rc = static_scratch(&sums);
    if (rc != AMSP_OK) return rc;
    return sqnorm_range(partials, k, grad_f32, n, bucket_elems, d_sqnorm, accumulate, sums, stream);
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
    }
    if (misaligned(grad_f32_local, 4)) return AMSP_EALIGN;
    hipStream_t hs = (hipStream_t)stream;
    TableBuilder tb;
    auto flush_table = [&]() -> int {
        if (tb.count == 0) return AMSP_OK;
        tb.pad();
        const unsigned lds = occupancy_lds(8 * k + (accumulate ? 16 : 0), reduce_target(k, accumulate != 0));
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
        rc = amsp_reduce_grad_shard(q.p, k, g.length, 0, grad_f32_local + g.local_offset, accumulate, stream);
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
        // at most 2^20 - 1 segments with maxima: the words stay 32-bit indexable and the folding
        // kernel's grid (one block per segment) far inside the grid limit
        if ((size_t)num_segments * kAmaxWordsPerSegment > 0xFFFFFFFFull) return AMSP_EINVAL;
        words = static_cast<uint32_t *>(amax_workspace);
    }
    for (uint32_t i = 0; i < num_segments; ++i) {
        if (segments[i].length == 0) continue;
        if (master_local == nullptr || exp_avg_local == nullptr || exp_avg_sq_local == nullptr ||
            (k == 0 && grad_f32_local == nullptr))
            return AMSP_ENULL;
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
                           (uint64_t)count, 0u);
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
    if (master == nullptr || d_scale == nullptr || param_fp8_out == nullptr) return AMSP_ENULL;
    if (misaligned(master, 4) || misaligned(d_scale, 4)) return AMSP_EALIGN;
    clear_stale_error();
    Fp8CastBatch batch(master, d_scale, param_fp8_out, (hipStream_t)stream);
    const int rc = batch.add(0, 0, n, 0);
    return rc != AMSP_OK ? rc : batch.flush();
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
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(kThreads), 0, hs, slots, (uint64_t)num_segments, 0u);
        if (launched() != AMSP_OK) return AMSP_EDEVICE;
        // segments the table does not take: kMaxNormSegs of them to a launch, the blocks of a resident grid
        // dealt out in proportion to the ranges' lengths (at least one each)
        AbsmaxTable at;
        int count = 0;
        uint64_t work = 0;
        auto flush_ranges = [&]() -> int {
            if (count == 0) return AMSP_OK;
            const uint64_t grid = (uint64_t)norm_grid(work, 0);
            uint32_t blocks = 0;
            for (int j = 0; j < kMaxNormSegs; ++j) {
                if (j >= count) {
                    at.first_block[j] = 0xFFFFFFFFu;
                    at.blocks[j] = 0; at.slot[j] = 0;
                    at.seg[j] = NormSeg{0, Span{0, 0, 0, 0, 0}};
                    continue;
                }
                const Span &sp = at.seg[j].s;
                const uint64_t w = sp.vectorised ? sp.nvec : sp.n;
                // round(grid * w / work); both factors are below 2^34 and 2^10
                uint64_t share = work ? (grid * w + work / 2) / work : 1;
                const uint64_t useful = (w + kNormThreads - 1) / kNormThreads;   // blocks that would have a vector
                if (share > useful) share = useful;
                at.first_block[j] = blocks;
                at.blocks[j] = (uint32_t)(share ? share : 1);
                blocks += at.blocks[j];
            }
            hipLaunchKernelGGL(absmax_kernel, dim3(blocks), dim3(kNormThreads), 0, hs, master_local, slots, at);
            count = 0;
            work = 0;
            return launched();
        };
        for (uint32_t i = 0; i < num_segments; ++i) {
            if (segments[i].length == 0) continue;
            if (tabled(i, false, &rc)) {
                if (rc != AMSP_OK) return rc;
                continue;
            }
            Stream16 st[1] = {{master_local + segments[i].local_offset, 4}};
            NormSeg &g = at.seg[count];
            g.base = segments[i].local_offset;
            g.s = make_span(segments[i].length, st, 1, 4);
            at.slot[count] = i;
            work += g.s.vectorised ? g.s.nvec : g.s.n;
            if (++count == kMaxNormSegs && (rc = flush_ranges()) != AMSP_OK) return rc;
        }
        rc = flush_ranges();
        if (rc != AMSP_OK) return rc;
        rc = flush_table(false);
        if (rc != AMSP_OK) return rc;
    }
    hipLaunchKernelGGL(fp8_scale_kernel, dim3(1), dim3(kThreads), 0, hs, d_amax, d_scale, num_segments);
    if (launched() != AMSP_OK) return AMSP_EDEVICE;
    Fp8CastBatch codes(master_local, d_scale, param_fp8_flat, hs);
    for (uint32_t i = 0; i < num_segments; ++i) {
        if (segments[i].length == 0) continue;
        if (tabled(i, true, &rc)) {
            if (rc != AMSP_OK) return rc;
            continue;
        }
        rc = codes.add(segments[i].local_offset, segments[i].flat_offset, segments[i].length, i);
        if (rc != AMSP_OK) return rc;
    }
    rc = codes.flush();
    return rc != AMSP_OK ? rc : flush_table(true);
}

}  // extern "C"
