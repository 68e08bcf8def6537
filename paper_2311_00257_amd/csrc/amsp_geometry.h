// Range geometry of the model-state kernels: how a launch over n elements of several streams splits
// into an element-wise head, aligned vector accesses and an element-wise tail, for a single range and
// for the buckets of one launch.  Plain integer arithmetic shared by the host code that sizes the
// launches and the kernels that walk them; it compiles as ordinary C++ too, so that the indexing can be
// checked exhaustively on a CPU.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define AMSP_HOST_DEVICE __host__ __device__
#else
#define AMSP_HOST_DEVICE
#endif

namespace amsp_geom {

constexpr int kWaveLanes = 64;   // one-wave workgroups: lanes per block on the vector path

// A launch covers n elements: `head` leading ones up to the element at which every stream is
// aligned (to a wave's piece when the streams allow it, else to a 128-byte line, else to its vector
// access), nvec groups of VEC taken with vector accesses, and `tail` < VEC trailing ones.  Head and
// tail are the "edge", done element-wise by the range's first block.  When the streams have no common
// phase the host sets vectorised = 0 and every element goes through the element-wise loop.
struct Span {
    uint64_t n;
    uint64_t nvec;
    uint32_t head;
    uint32_t tail;
    uint32_t vectorised;
};

// Element index of the t-th edge element, t < head + tail.
AMSP_HOST_DEVICE inline uint64_t edge_elem(const Span &s, uint32_t t, int vec) {
    return t < s.head ? (uint64_t)t : (uint64_t)s.head + s.nvec * (uint64_t)vec + (t - s.head);
}

// Several buckets in one launch.  Bucket b covers [b * bucket_elems, min((b + 1) * bucket_elems, n)) and
// is given blocks_per_bucket consecutive one-wave blocks (enough for its vectors at the launch's vectors per
// lane); its own head, vector count and tail follow
// from h0, the head of element 0, because alignment repeats every mask + 1 elements.
// bucket_elems == 0: the launch is a single range described by a Span.
struct Buckets {
    uint64_t bucket_elems;
    uint64_t n;
    uint32_t h0;
    uint32_t mask;
    uint32_t blocks_per_bucket;
};

// The range block `block` works on: its Span (relative to `off`), the range's first element `off`, and
// the block's index within the range.  With bucket_elems == 0, `s` is left as passed in.
AMSP_HOST_DEVICE inline void block_range(const Buckets &bk, uint32_t block, int vec, Span &s, uint64_t &off,
                                         uint32_t &local_block) {
    off = 0;
    local_block = block;
    if (bk.bucket_elems != 0) {
        const uint32_t b = block / bk.blocks_per_bucket;
        local_block = block - b * bk.blocks_per_bucket;
        off = (uint64_t)b * bk.bucket_elems;
        const uint64_t left = bk.n - off;
        const uint64_t len = left < bk.bucket_elems ? left : bk.bucket_elems;
        const uint32_t head = (bk.h0 - (uint32_t)off) & bk.mask;
        s.n = len;
        s.vectorised = 1;
        if (len < (uint64_t)head + (uint64_t)vec) {   // too short for one aligned vector: all of it is edge
            s.head = (uint32_t)len;
            s.nvec = 0;
            s.tail = 0;
        } else {
            s.head = head;
            s.nvec = (len - head) / (uint64_t)vec;
            s.tail = (uint32_t)(len - head - s.nvec * (uint64_t)vec);
        }
    }
}

// The read-only pass over a range's nvec vectors: a persistent grid of `grid` one-wave blocks.  Block b's
// trip t covers the U consecutive wave pieces (kWaveLanes vectors each) that start at vector
// (t * grid + b) * kWaveLanes * U, so that a trip of the whole grid is one contiguous window of every
// stream.  full(v): lane's vectors v, v + kWaveLanes, ..., v + (U - 1) kWaveLanes are all inside the range;
// part(v): the block's last trip when the range ends inside it (at most once per range): of those U
// vectors only the ones below nvec exist, the first (v) always does.  Both issue their loads together: a
// range of a few trips (a 25 M-element bucket is six) would otherwise spend as long on the pieces of its
// last trip, one memory round trip each, as on all the others.  Every vector in [0, nvec) is visited
// exactly once.
template <int U, typename Full, typename Part>
AMSP_HOST_DEVICE inline void norm_walk(uint64_t nvec, uint32_t grid, uint32_t block, uint32_t lane, Full full,
                                       Part part) {
    const uint64_t row = (uint64_t)grid * kWaveLanes;   // vectors the grid takes per piece index
    uint64_t v = (uint64_t)block * (kWaveLanes * U) + lane;
    for (; v + (uint64_t)(U - 1) * kWaveLanes < nvec; v += (uint64_t)U * row) full(v);
    if (U > 1 && v < nvec) part(v);
}

// ---------------------------------------------------------------- host side
struct Stream {
    const void *ptr;
    uint32_t elem;   // bytes per element: 1, 2 or 4
};

// Three alignments a launch may start its vector accesses at, best first:
//   kAlignWave   every stream on a multiple of what one wave takes from it per access (64 lanes x
//                vec elements: 512 B of bf16, 1 KiB of fp32 at vec = 4), so that a wave's piece is
//                aligned to its own size; pieces shifted by 128-384 B cost the fused step 4-5 %
//   kAlignLine   every stream on a 128-byte line (each piece is whole lines)
//   kAlignVector every stream aligned for its vector access only
// Alignment repeats every `period` elements; the head is the smallest element offset that reaches it.
enum AlignLevel { kAlignWave = 0, kAlignLine = 1, kAlignVector = 2 };

inline uintptr_t align_need(AlignLevel level, uint32_t elem, int vec) {
    if (level == kAlignWave) return (uintptr_t)kWaveLanes * vec * elem;
    if (level == kAlignLine) return 128;
    return (uintptr_t)vec * elem < 16 ? (uintptr_t)vec * elem : 16;
}

inline int align_period(AlignLevel level, const Stream *st, int ns, int vec) {
    if (level == kAlignWave) return kWaveLanes * vec;
    if (level == kAlignVector) return vec;
    uint32_t smallest = 4;
    for (int i = 0; i < ns; ++i)
        if (st[i].elem < smallest) smallest = st[i].elem;
    return (int)(128 / smallest);
}

// Smallest head at which every stream meets `level`, or -1.  Every stream's alignment repeats with a
// power-of-two period (in elements) that divides the longest one, so the only candidate below the
// longest period is the head of the stream that has it; the others either agree with it or no head exists.
inline int common_head(const Stream *st, int ns, int vec, AlignLevel level) {
    if (ns <= 0) return 0;
    int widest = 0;
    uintptr_t widest_period = 0;
    for (int i = 0; i < ns; ++i) {
        const uintptr_t period = align_need(level, st[i].elem, vec) / st[i].elem;
        if (period > widest_period) {
            widest_period = period;
            widest = i;
        }
    }
    const uintptr_t need = align_need(level, st[widest].elem, vec);
    const uintptr_t past = (uintptr_t)st[widest].ptr & (need - 1);   // bytes past the last aligned address
    if (past % st[widest].elem != 0) return -1;                      // not even element-aligned
    const uintptr_t h = ((need - past) & (need - 1)) / st[widest].elem;
    for (int i = 0; i < ns; ++i)
        if ((((uintptr_t)st[i].ptr + h * st[i].elem) & (align_need(level, st[i].elem, vec) - 1)) != 0) return -1;
    return (int)h;
}

inline Span make_span(uint64_t n, const Stream *st, int ns, int vec) {
    Span s{n, 0, 0, 0, 0};
    for (int level = kAlignWave; level <= kAlignVector; ++level) {
        const int h = common_head(st, ns, vec, (AlignLevel)level);
        if (h < 0 || n < (uint64_t)h + (uint64_t)vec) continue;
        s.head = (uint32_t)h;
        s.nvec = (n - (uint64_t)h) / (uint64_t)vec;
        s.tail = (uint32_t)(n - (uint64_t)h - s.nvec * (uint64_t)vec);
        s.vectorised = 1;
        break;
    }
    return s;
}

// A launch is given at most kMaxLaunchBlocks workgroups (2^25: 8.6e9 elements of the kernels that write,
// above the largest launch the workloads make, 2.6e7 workgroups; the hardware's own limit is 2^31 - 1).
// Longer ranges are cut on the host into consecutive pieces, each an ordinary launch with its own head and
// tail; a piece's length is a multiple of 1024 elements, so every piece after the first starts at the
// alignment phase of the range's own start.
constexpr uint64_t kMaxLaunchBlocks = 1ull << 25;
constexpr uint64_t kElemsPerBlock = (uint64_t)kWaveLanes * 4;   // one-wave workgroups, 4 elements per lane
constexpr uint64_t kMaxLaunchElems = kMaxLaunchBlocks * kElemsPerBlock;

// Calls f(off, len) for the pieces of [begin, begin + n): consecutive, disjoint, covering, each of at most
// `limit` elements (a multiple of 1024).  Stops at the first non-zero return and hands it on.
template <typename F>
inline int for_pieces(uint64_t begin, uint64_t n, uint64_t limit, F f) {
    for (uint64_t off = 0; off < n; off += limit) {
        const int rc = f(begin + off, n - off < limit ? n - off : limit);
        if (rc != 0) return rc;
    }
    return 0;
}

// Geometry of one launch over the buckets of [0, n) whose streams start at `st`; false when the streams
// have no common phase (then every bucket goes through the element-wise path, a launch each).
// `rows`: vectors per lane and block (a block covers rows consecutive wave pieces).
inline bool make_buckets(uint64_t n, uint64_t bucket_elems, const Stream *st, int ns, int vec, Buckets &bk,
                         int rows = 1) {
    for (int level = kAlignWave; level <= kAlignVector; ++level) {
        const int h = common_head(st, ns, vec, (AlignLevel)level);
        if (h < 0) continue;
        bk = Buckets{bucket_elems, n, (uint32_t)h, (uint32_t)align_period((AlignLevel)level, st, ns, vec) - 1u,
                     (uint32_t)(bucket_elems / ((uint64_t)kWaveLanes * vec * rows) + 1)};
        return true;
    }
    return false;
}

}  // namespace amsp_geom
