// Exhaustive CPU check of the range geometry the kernels walk: for random stream alignments, lengths
// and bucket sizes, emulate every block and lane of a launch and verify that
//   - every element of [0, n) is touched exactly once (head, vectors, tail; across all buckets),
//   - every vector access of every stream is aligned for its width,
//   - the best alignment level that exists is the one taken (a wave's piece, else a line, else a vector),
// and, for the persistent read-only pass, that the trips of all blocks and lanes visit every vector of a
// range exactly once, never one outside it, with the vectors of a "full" trip all inside the range.
// Prints "ok <cases>" and exits 0, or names the failing case and exits 1.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#include "amsp_geometry.h"

using namespace amsp_geom;

static uint64_t rng_state = 0x2311002570000001ull;
static uint64_t rnd() {   // splitmix64
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint64_t below(uint64_t m) { return rnd() % m; }

struct Case {
    std::vector<Stream> st;
    uint64_t n, bucket;
    int vec;
    int rows = 1;   // vectors per lane and block: a block covers `rows` consecutive wave pieces
};

static bool aligned(const Stream &s, uint64_t elem_index, uintptr_t need) {
    return (((uintptr_t)s.ptr + (uintptr_t)elem_index * s.elem) & (need - 1)) == 0;
}

// The alignment rules restated here, on purpose not taken from the header under test.
// level 0: what a wave takes from the stream per access (64 lanes x vec elements); 1: a 128-byte line;
// 2: the lane's own access, vec elements or 16 bytes, whichever is smaller.
static uintptr_t need_of(int level, uint32_t elem, int vec) {
    if (level == 0) return (uintptr_t)64 * vec * elem;
    if (level == 1) return 128;
    const uintptr_t lane = (uintptr_t)vec * elem;
    return lane < 16 ? lane : 16;
}
// Smallest h >= 0 such that element `from + h` of every stream meets `level`, or -1 (none within two wave pieces).
static int brute_head(const Case &c, int level, uint64_t from) {
    for (int h = 0; h < 2 * 64 * c.vec; ++h) {
        bool ok = true;
        for (const Stream &st : c.st) ok = ok && aligned(st, from + h, need_of(level, st.elem, c.vec));
        if (ok) return h;
    }
    return -1;
}

static int fail(const Case &c, const char *what, uint64_t at) {
    printf("FAIL: %s at %llu; n=%llu bucket=%llu vec=%d rows=%d streams:", what, (unsigned long long)at,
           (unsigned long long)c.n, (unsigned long long)c.bucket, c.vec, c.rows);
    for (const Stream &s : c.st) printf(" (%p,%u)", s.ptr, s.elem);
    printf("\n");
    return 1;
}

// Walk one range the way a kernel's blocks do; bump `seen` per element touched.
static int walk_range(const Case &c, const Span &s, uint64_t off, uint32_t local_block, std::vector<uint8_t> &seen) {
    for (int slot = 0; slot < kWaveLanes * c.rows; ++slot) {   // slot = row * 64 + lane
        const uint64_t v = (uint64_t)local_block * kWaveLanes * c.rows + slot;
        if (v < s.nvec) {
            const uint64_t e = off + s.head + v * c.vec;
            for (const Stream &st : c.st)
                if (!aligned(st, e, need_of(2, st.elem, c.vec))) return fail(c, "misaligned vector access", e);
            for (int q = 0; q < c.vec; ++q) {
                if (e + q >= c.n) return fail(c, "vector access out of range", e + q);
                ++seen[e + q];
            }
        }
    }
    if (local_block == 0)
        for (uint32_t t = 0; t < s.head + s.tail; ++t) {
            const uint64_t i = off + edge_elem(s, t, c.vec);
            if (i >= c.n) return fail(c, "edge element out of range", i);
            ++seen[i];
        }
    return 0;
}

static int check(const Case &c) {
    std::vector<uint8_t> seen(c.n, 0);
    const Stream *st = c.st.data();
    const int ns = (int)c.st.size();
    if (c.bucket == 0 || c.bucket >= c.n) {
        const Span s = make_span(c.n, st, ns, c.vec);
        // the best level that exists (and leaves room for one vector) decides the head
        int want = -1;
        for (int level = 0; level <= 2 && want < 0; ++level) {
            const int h = brute_head(c, level, 0);
            if (h >= 0 && c.n >= (uint64_t)h + c.vec) want = h;
        }
        if (!s.vectorised) {
            if (want >= 0) return fail(c, "vector path refused though a head exists", want);
            return 0;
        }
        if (want < 0) return fail(c, "vector path taken though no head exists", s.head);
        if ((uint32_t)want != s.head) return fail(c, "head is not that of the best alignment level", want);
        if (s.head + s.nvec * c.vec + s.tail != c.n || s.tail >= (uint32_t)c.vec) return fail(c, "span does not add up", s.head);
        const uint64_t per_block = (uint64_t)kWaveLanes * c.rows;
        const uint64_t blocks = (s.nvec + per_block - 1) / per_block;
        for (uint64_t b = 0; b < (blocks ? blocks : 1); ++b)
            if (walk_range(c, s, 0, (uint32_t)b, seen)) return 1;
    } else {
        Buckets bk;
        int level = 0;
        while (level <= 2 && brute_head(c, level, 0) < 0) ++level;   // the launch's level: the best that exists at all
        if (!make_buckets(c.n, c.bucket, st, ns, c.vec, bk, c.rows)) {
            if (level <= 2) return fail(c, "bucket launch refused though a head exists", 0);
            return 0;
        }
        if (level > 2) return fail(c, "bucket launch taken though no head exists", 0);
        const uint64_t nb = (c.n + c.bucket - 1) / c.bucket;
        for (uint64_t block = 0; block < nb * bk.blocks_per_bucket; ++block) {
            Span s{c.n, 0, 0, 0, 1};
            uint64_t off;
            uint32_t lb;
            block_range(bk, (uint32_t)block, c.vec, s, off, lb);
            if (off >= c.n || off + s.n > c.n) return fail(c, "bucket outside the range", off);
            if (s.head + s.nvec * c.vec + s.tail != s.n) return fail(c, "bucket span does not add up", off);
            const int bh = brute_head(c, level, off);
            if (s.nvec > 0 && (bh < 0 || (uint32_t)bh != s.head)) return fail(c, "bucket head is not the smallest aligned one", off);
            if (s.nvec == 0 && bh >= 0 && s.n >= (uint64_t)bh + c.vec) return fail(c, "bucket left to the edge loop though a vector fits", off);
            if (s.tail >= (uint32_t)c.vec && s.nvec > 0) return fail(c, "bucket tail as long as a vector", off);
            if ((uint64_t)bk.blocks_per_bucket * kWaveLanes * c.rows < s.nvec) return fail(c, "too few blocks per bucket", off);
            const uint64_t per_block = (uint64_t)kWaveLanes * c.rows * c.vec;   // elements
            if ((uint64_t)bk.blocks_per_bucket * per_block > c.bucket + 2 * per_block)
                return fail(c, "more blocks per bucket than its vectors need", off);
            if (walk_range(c, s, off, lb, seen)) return 1;
        }
    }
    for (uint64_t i = 0; i < c.n; ++i)
        if (seen[i] != 1) return fail(c, seen[i] ? "element touched twice" : "element never touched", i);
    return 0;
}

// The read-only pass: every (block, lane) of a persistent grid walks its trips; count the visits per vector.
template <int U>
static int check_norm_walk(uint64_t nvec, uint32_t grid) {
    std::vector<uint8_t> seen(nvec, 0);
    int bad = 0;
    for (uint32_t block = 0; block < grid && !bad; ++block)
        for (uint32_t lane = 0; lane < (uint32_t)kWaveLanes && !bad; ++lane) {
            int partial_trips = 0;
            norm_walk<U>(
                nvec, grid, block, lane,
                [&](uint64_t v) {
                    for (int u = 0; u < U; ++u) {
                        const uint64_t x = v + (uint64_t)u * kWaveLanes;
                        if (x >= nvec) { bad = 1; return; }
                        // the U pieces of a trip are consecutive: one contiguous window per block
                        if (x / kWaveLanes != v / kWaveLanes + (uint64_t)u || x % kWaveLanes != lane) { bad = 1; return; }
                        ++seen[x];
                    }
                },
                [&](uint64_t v) {   // the block's last, partial trip: at most one per block and range
                    if (U == 1 || v >= nvec || v % kWaveLanes != lane || ++partial_trips > 1) { bad = 1; return; }
                    if (v + (uint64_t)(U - 1) * kWaveLanes < nvec) { bad = 1; return; }   // it was a full trip
                    for (int u = 0; u < U; ++u) {
                        const uint64_t x = v + (uint64_t)u * kWaveLanes;
                        if (x < nvec) ++seen[x];
                    }
                });
        }
    for (uint64_t v = 0; v < nvec && !bad; ++v)
        if (seen[v] != 1) bad = 1;
    if (bad) printf("FAIL: norm walk U=%d nvec=%llu grid=%u\n", U, (unsigned long long)nvec, grid);
    return bad;
}

// Ranges longer than a launch: the pieces tile the range in order, none longer than the limit, and (the
// limit being a multiple of 1024 elements) every piece starts at the alignment phase of the range's start.
static int check_pieces(uint64_t begin, uint64_t n, uint64_t limit) {
    uint64_t next = begin, count = 0;
    const int rc = for_pieces(begin, n, limit, [&](uint64_t off, uint64_t len) -> int {
        if (off != next || len == 0 || len > limit || (off - begin) % 1024 != 0) return 7;
        next = off + len;
        ++count;
        return 0;
    });
    if (rc != 0 || next != begin + n || count != (n + limit - 1) / limit) {
        printf("FAIL: pieces begin=%llu n=%llu limit=%llu\n", (unsigned long long)begin, (unsigned long long)n,
               (unsigned long long)limit);
        return 1;
    }
    // an error stops the walk and is handed on
    int calls = 0;
    if (n > limit && (for_pieces(begin, n, limit, [&](uint64_t, uint64_t) { return ++calls == 1 ? -5 : 0; }) != -5 || calls != 1)) return 1;
    return 0;
}

int main() {
    static_assert(kMaxLaunchElems % 1024 == 0 && kMaxLaunchElems == kMaxLaunchBlocks * 256, "piece length");
    if (check_pieces(0, 0, kMaxLaunchElems) || check_pieces(5, 1, kMaxLaunchElems) ||
        check_pieces(0, kMaxLaunchElems, kMaxLaunchElems) || check_pieces(3, kMaxLaunchElems + 1, kMaxLaunchElems) ||
        check_pieces(0, 5 * kMaxLaunchElems - 1, kMaxLaunchElems) || check_pieces(1ull << 40, (1ull << 36) + 12345, kMaxLaunchElems))
        return 1;
    for (int iter = 0; iter < 2000; ++iter)
        if (check_pieces(below(1ull << 40), below(1ull << 20), 1024 * (1 + below(64)))) return 1;
    for (int iter = 0; iter < 3000; ++iter) {
        const uint64_t nvec = below(4) == 0 ? below(70) : below(30000);
        const uint32_t grid = 1 + (uint32_t)below(below(2) ? 8 : 48);
        if (check_norm_walk<1>(nvec, grid) || check_norm_walk<4>(nvec, grid) || check_norm_walk<8>(nvec, grid)) return 1;
    }

    const uint64_t lengths[] = {1, 2, 3, 4, 5, 63, 64, 65, 255, 256, 257, 258, 259, 260, 511, 512, 513, 1023, 1024, 1025};
    const uint64_t buckets[] = {0, 0, 1, 2, 3, 4, 5, 7, 63, 64, 255, 256, 257, 258, 259, 260, 261, 300, 511, 512, 513, 1000, 1025};
    int cases = 0;
    for (int iter = 0; iter < 60000; ++iter) {
        Case c;
        c.vec = below(4) == 0 ? 8 : 4;
        c.n = below(3) == 0 ? lengths[below(sizeof lengths / sizeof *lengths)] : 1 + below(6000);
        c.bucket = c.vec == 8 ? 0 : buckets[below(sizeof buckets / sizeof *buckets)];
        c.rows = c.vec == 8 ? 1 : (below(3) == 0 ? (below(2) ? 2 : 4) : 1);   // the reduction with few partials
        const int ns = 1 + (int)below(6);
        const int mode = (int)below(5);   // 0: unrelated small shifts; 1: a common shift plus whole lines; else: a common shift
        const uint64_t common = below(700);
        for (int i = 0; i < ns; ++i) {
            const uint32_t elem = c.vec == 8 ? 2u : (below(8) == 0 ? 1u : (below(2) ? 2u : 4u));
            // mode 1 leaves the streams line-aligned together but (mostly) not aligned to a wave's piece together
            const uint64_t shift = mode == 0 ? below(9) : (mode == 1 ? common + below(4) * (128 / elem) : common);
            const uintptr_t base = (uintptr_t)((1 + below(1000)) << 21);   // 2 MiB-aligned allocations
            c.st.push_back(Stream{(const void *)(base + shift * elem), elem});
        }
        if (check(c)) return 1;
        ++cases;
    }
    printf("ok %d\n", cases);
    return 0;
}
