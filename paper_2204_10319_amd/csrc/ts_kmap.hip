// Kernel-map construction (paper Sec. 2.1: output coordinates, Alg. 3; map search, Alg. 1).
//
// Pipeline on the device, one stream:
//   fill     one launch clears the hash table, the counters and (stride 1) the neighbour table
//   pack     (b,x,y,z) -> order-preserving 64-bit keys       (one integer per coordinate, Sec. 2.1.2)
//   stride>1: candidate keys (p - delta)/s, radix sort, unique -> P_out           (Alg. 3, stages 1-4)
//   insert   the searched point set into an open-addressing table (64-bit CAS)
//   search   s*q_k + delta_n for every output k and offset n (Alg. 1).  Stride 1, K = 3: one thread
//            per (point, offset below the centre), the mirrored entry written alongside
//            (Sec. 4.2.1), then a pass over the rows; otherwise one thread per output.  Leaves per
//            output the row of neighbour indices and its offset bitmask, and per 64 outputs and
//            offset a presence bitmap with its count
//   scan     per-offset exclusive scan of the block counts -> where each pair sits in the
//            offset-major lists, and the per-offset totals
// The host waits once, after `scan`, for the map sizes and error flags.
// The searched set can also be held in a coordinate grid (`grid` of Sec. 4.4: collision-free, one
// memory access per insertion and per lookup) when the caller states the bounds of its coordinates;
// Alg. 3's boundary check is applied where the candidates are formed.
//   compact  pair lists M[W_n] (in, out), ordered by output index inside an offset: derived from
//            the above when first asked for (ts_kmap_pairs, the explicit dataflow's gather)
//
// ts_kmap_sort_rows (optional, for maps that serve several layers) orders the output rows by
// offset bitmask: distinct bitmasks are counted in a small hash table, ranked, and every row
// goes to (first position of its bitmask) + (arrival rank).
#include "ts_internal.h"

#include <cstdlib>
#include <cstring>
#include <new>
#include <type_traits>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_select.hpp>

using namespace ts;


namespace {

constexpr int kThreads = 256;

// status words written by the kernels and read back once per build
enum {
    ST_RANGE = 0,       // a coordinate was outside the packable range
    ST_DUP = 1,         // two input rows held the same coordinate
    ST_DCOUNT = 2,      // distinct offset bitmasks seen (ts_kmap_sort_rows)
    ST_OVERFLOW = 3,    // the bitmask table could not hold them all
    ST_TOTALS = 8,      // [32] per-offset map sizes
    ST_WORDS = 40
};

// Error flags are raised with a plain store of 1: every writer stores the same value, and the word may
// live in pinned host memory (a build nobody waits for reports straight to the host, without a copy).
__device__ __forceinline__ void raise_flag(int *status, int which) { *reinterpret_cast<volatile int *>(&status[which]) = 1; }

// ---- coordinate hash table ------------------------------------------------------------------------
// Open addressing over two arrays: 64-bit keys (what lookups read) and 32-bit values (read on a
// hit only).  Random lookups cost about twice as much once the array they walk no longer fits a
// 4 MiB L2 slice, so the probed array is kept as small as the key allows.  8 keys form a 64-byte
// bucket addressed by the hash of the point's 2x2x2 block, the home slot inside the bucket by the
// three parity bits: the cells around a point share a few buckets.
struct Table {
    uint64_t *keys;
    int32_t *vals;
    uint32_t mask;   // capacity - 1 (capacity: power of two >= 4 * entries, >= 1024)
    int shift;       // 64 - log2(capacity / slots per bucket)
};

// The cells of a small box of space (2^kBx x 2^kBy x 2^kBz cells) share a bucket of consecutive slots,
// addressed by the hash of the box; the home slot inside the bucket is the cell's position in the box.
// 2 x 2 x 2 is the measured optimum on the LiDAR-like scenes from 153 k to 15 M points: boxes of 4 x 4 x 4
// (64 slots), 1 x 1 x 8 and 1 x 2 x 4 put the slots of points inserted by neighbouring lanes into the same
// cache lines, whose atomics are then served one after the other (insertion 1.4 to 1.9 times slower), and do
// not make the search faster; smaller boxes (2 x 2 x 1, 1 x 2 x 2, 1 x 1 x 2, none) make it slower (20.4, 21.0,
// 26.8 and 32.5 us against 17.3 on 153 k points: a point's 13 lookups then touch more cache lines).
constexpr int kBx = 1, kBy = 1, kBz = 1;
constexpr uint64_t kSubBits = ((1ull << kBz) - 1) | (((1ull << kBy) - 1) << kFieldBits) | (((1ull << kBx) - 1) << (2 * kFieldBits));
constexpr int kBucketLog2 = kBx + kBy + kBz;

__device__ __forceinline__ uint32_t home_sub(uint64_t key) {
    return ((uint32_t)key & ((1u << kBz) - 1)) | (((uint32_t)(key >> kFieldBits) & ((1u << kBy) - 1)) << kBz) |
           (((uint32_t)(key >> (2 * kFieldBits)) & ((1u << kBx) - 1)) << (kBz + kBy));
}
// (Placing the buckets of neighbouring boxes next to each other - hashing only a region of 4, 8 or 16 boxes
// per axis and using a box's position in its region as the low part of the bucket number - was measured as
// well, for the sake of the large scenes whose table no longer fits the caches: occupied boxes then crowd
// into few stretches of the table, probe chains grow, and both insertion and search take 1.3 to 6 times as
// long at every size from 20 k to 15 M points.  Scattering the boxes is worth more than keeping them together.)
__device__ __forceinline__ uint32_t home_slot(uint64_t key, int shift) {
    const uint64_t cell = key & ~kSubBits;
    return ((uint32_t)((cell * 0x9E3779B97F4A7C15ull) >> shift) << kBucketLog2) + home_sub(key);   // multiplicative (Fibonacci) hashing
}
// Slot after `slot` in a probe sequence: 9 further (next bucket, next position; odd, so the sequence
// visits every slot of the power-of-two table).  A miss ends at the first empty slot it meets, which
// for a point's absent neighbour is usually the home slot itself.  (The slot right after, in the same
// cache line, is the home of the cell's neighbour in z: a key put there displaces that neighbour in turn,
// and the line's atomics queue up; measured, insertion took 15.1 instead of 11.1 us on 153 k points and the
// search 19.5 instead of 17.3.)
// What decides the length of the chains is how many occupied boxes there are per bucket, not points per slot:
// a LiDAR-like scene fills a 2x2x2 box with 1.5 to 2 points, so at a load of 0.29 points per slot there were
// about 1.5 boxes per bucket.  Hence the table's size of four slots per point or more: against two it took
// the search of 153 k points from 18.8 to 17.3 us, their insertion from 13.2 to 11.1, and the build of 15 M
// points from 6.1 to 4.9 ms; eight slots per point gained nothing more at 153 k and cost clearing time.
__device__ __forceinline__ uint32_t next_slot(uint32_t slot, uint32_t mask) { return (slot + 9u) & mask; }

// Loads by 32-bit byte offset from the array base (capacity is at most 2^28 slots), which keeps
// one register per lookup for the address instead of two.
__device__ __forceinline__ uint64_t slot_key(const Table &t, uint32_t slot) {
    return *reinterpret_cast<const uint64_t *>(reinterpret_cast<const char *>(t.keys) + (slot << 3));
}
__device__ __forceinline__ int32_t slot_val(const Table &t, uint32_t slot) {
    return *reinterpret_cast<const int32_t *>(reinterpret_cast<const char *>(t.vals) + (slot << 2));
}

__device__ __forceinline__ void table_insert(const Table &t, uint64_t key, int32_t value, int *status) {
    uint32_t slot = home_slot(key, t.shift);
    for (;;) {
        unsigned long long prev = atomicCAS(reinterpret_cast<unsigned long long *>(&t.keys[slot]),
                                            (unsigned long long)kEmptyKey, (unsigned long long)key);
        if (prev == kEmptyKey) {
            t.vals[slot] = value;
            return;
        }
        if (prev == key) {
            raise_flag(status, ST_DUP);
            return;
        }
        slot = next_slot(slot, t.mask);   // the table is at most a quarter full, so an empty slot exists
    }
}

// First slot holding `want`'s value, or -1: a miss ends at the first empty slot.
__device__ __forceinline__ int32_t table_find(const Table &t, uint64_t want) {
    uint32_t slot = home_slot(want, t.shift);
    for (;;) {
        const uint64_t found = slot_key(t, slot);
        if (found == want) return slot_val(t, slot);
        if (found == kEmptyKey) return -1;
        slot = next_slot(slot, t.mask);
    }
}

// ---- coordinate grid ------------------------------------------------------------------------------------
// The collision-free table of Sec. 4.4 (`grid`): one int32 cell per coordinate of a box, holding the
// row of the point there or -1.  An insertion is one store, a lookup one load, whatever the
// occupancy; the price is the box's volume in memory.  The cells live in a buffer the library keeps
// between builds with every cell at -1: a build writes its points in, searches, and takes them out
// again, so it touches 2 N cells and never clears the volume.
struct Grid {
    int32_t *vals;      // [batches][ext x][ext y][ext z]
    int32_t lo[3];      // coordinate of cell 0 on each axis
    uint32_t ext[3];    // cells per axis
    uint32_t batches;
};

// Cell of a packed coordinate, or -1 outside the box.
__device__ __forceinline__ int64_t grid_cell(const Grid &g, uint64_t key) {
    int32_t c[4];
    unpack_key(key, c);
    const uint32_t x = (uint32_t)(c[1] - g.lo[0]), y = (uint32_t)(c[2] - g.lo[1]), z = (uint32_t)(c[3] - g.lo[2]);
    if ((uint32_t)c[0] >= g.batches || x >= g.ext[0] || y >= g.ext[1] || z >= g.ext[2]) return -1;
    return (((int64_t)c[0] * g.ext[0] + x) * g.ext[1] + y) * g.ext[2] + z;
}

__device__ __forceinline__ void table_insert(const Grid &g, uint64_t key, int32_t value, int *status) {
    const int64_t cell = grid_cell(g, key);
    if (cell < 0) {
        raise_flag(status, ST_RANGE);
        return;
    }
    if (atomicCAS(&g.vals[cell], -1, value) != -1) raise_flag(status, ST_DUP);
}

__device__ __forceinline__ int32_t table_find(const Grid &g, uint64_t want) {
    const int64_t cell = grid_cell(g, want);
    return cell < 0 ? -1 : g.vals[cell];
}

// Takes the points out again: the cells of `keys` go back to -1.
__global__ void k_grid_erase(const uint64_t *keys, int64_t n, Grid g) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint64_t key = keys[i];
    if (key == kEmptyKey) return;
    const int64_t cell = grid_cell(g, key);
    if (cell >= 0) g.vals[cell] = -1;
}

// Bounds the caller states for its coordinates (grid search); on == 0: none stated.
struct Box {
    int on;
    int32_t lo[3], hi[3];   // inclusive
    int32_t batches;
};
// Alg. 3's boundary: a candidate u is kept when 0 <= u < hi on every axis (hi = s * b); on == 0: no boundary.
struct Bound {
    int on;
    int32_t hi[3];
};

__device__ __forceinline__ bool coord_ok(int4 c) {
    return c.x >= 0 && c.x <= TS_BATCH_MAX && c.y >= TS_COORD_MIN && c.y <= TS_COORD_MAX &&
           c.z >= TS_COORD_MIN && c.z <= TS_COORD_MAX && c.w >= TS_COORD_MIN && c.w <= TS_COORD_MAX;
}

__host__ __device__ constexpr int offset_component(int K, int n, int axis) {
    const int r = (K - 1) / 2;
    return axis == 0 ? n / (K * K) - r : (axis == 1 ? (n / K) % K - r : n % K - r);
}

__device__ __forceinline__ bool in_box(int4 c, const Box &b) {
    return !b.on || (c.x < b.batches && c.y >= b.lo[0] && c.y <= b.hi[0] && c.z >= b.lo[1] && c.z <= b.hi[1] &&
                     c.w >= b.lo[2] && c.w <= b.hi[2]);
}

__host__ __device__ __forceinline__ int floor_div(int a, int s) { return a >= 0 ? a / s : -((-a + s - 1) / s); }

// ---- one launch for every buffer that must start at a known value -----------------------------------
struct FillSeg {
    uint4 *p;
    uint64_t n_vec;     // 16-byte vectors
    uint32_t value;     // replicated into every 32-bit word
};
struct FillArgs {
    FillSeg seg[8];
    int n = 0;
    void add(void *p, size_t bytes, uint32_t value) {
        if (bytes == 0) return;
        seg[n].p = static_cast<uint4 *>(p);
        seg[n].n_vec = (bytes + 15) / 16;
        seg[n].value = value;
        ++n;
    }
};

__global__ void k_fill(FillArgs a) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (int s = 0; s < a.n; ++s) {
        const uint32_t v = a.seg[s].value;
        const uint4 vv = make_uint4(v, v, v, v);
        for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.seg[s].n_vec; i += stride)
            a.seg[s].p[i] = vv;
    }
}

// Bounding box of the valid coordinates, for builds that choose their search by it: 64 partial boxes
// on cache lines of their own (atomics on one line are served one after the other), each 7 running
// maxima: -x, -y, -z, x, y, z, batch.  The host folds the 64.
constexpr int kBoxSlots = 64, kBoxSlotWords = 32;

// keys[i] = pack(coords[i]); out-of-range rows get the empty key and raise ST_RANGE.
__global__ void __launch_bounds__(kThreads) k_pack(const int4 *coords, int64_t n, uint64_t *keys, int *status, Box box, int32_t *bbox) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int32_t v[7];
#pragma unroll
    for (int q = 0; q < 7; ++q) v[q] = INT32_MIN;
    if (i < n) {
        int4 c = coords[i];
        if (!coord_ok(c) || !in_box(c, box)) {
            raise_flag(status, ST_RANGE);
            keys[i] = kEmptyKey;
        } else {
            keys[i] = pack_key(c.x, c.y, c.z, c.w);
            v[0] = -c.y, v[1] = -c.z, v[2] = -c.w, v[3] = c.y, v[4] = c.z, v[5] = c.w, v[6] = c.x;
        }
    }
    if (!bbox) return;
#pragma unroll
    for (int q = 0; q < 7; ++q)
        for (int d = 32; d >= 1; d >>= 1) v[q] = max(v[q], __shfl_xor(v[q], d, 64));
    const int lane = threadIdx.x & 63;
    const int slot = (int)((blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6)) % kBoxSlots);
    if (lane < 7) {
        int32_t mine = v[0];
#pragma unroll
        for (int q = 1; q < 7; ++q) mine = lane == q ? v[q] : mine;
        if (mine != INT32_MIN) atomicMax(&bbox[slot * kBoxSlotWords + lane], mine);
    }
}

// Insert (keys[i] -> i).
template <class TableT>
__global__ void k_insert(const uint64_t *keys, int64_t n, TableT t, int *status) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t key = keys[i];
    if (key == kEmptyKey) return;
    table_insert(t, key, (int32_t)i, status);
}

// Stride-1 front end in one pass: pack and insert (key -> i).  With `rows` (the neighbour table of a 3x3x3
// map, 8 16-byte vectors per point) the workgroup also sets its points' rows to "no neighbour": the symmetric
// search writes hits only, and these stores ride along with a kernel that waits for its atomics anyway
// instead of tripling what the clearing launch before it has to write.
template <class TableT>
__global__ void k_pack_insert(const int4 *coords, int64_t n, uint64_t *keys, TableT t, int *status, Box box, int4 *rows) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const int4 c = coords[i];
        if (!coord_ok(c) || !in_box(c, box)) {
            raise_flag(status, ST_RANGE);
            keys[i] = kEmptyKey;
        } else {
            const uint64_t key = pack_key(c.x, c.y, c.z, c.w);
            keys[i] = key;
            table_insert(t, key, (int32_t)i, status);
        }
    }
    // (after the insertion: stores issued before it would have to complete before the atomic's answer is seen)
    if (rows) {
        const int64_t first = (int64_t)blockIdx.x * blockDim.x * 8, end = n * 8;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int64_t at = first + (int64_t)k * blockDim.x + threadIdx.x;
            if (at < end) rows[at] = make_int4(-1, -1, -1, -1);
        }
    }
}

// Alg. 3 stages 1-4 in registers: candidate u = p - delta, modular check, boundary check, key of u/s.
// Along an axis the admissible offsets are those congruent to p modulo s, at most A = ceil(K/s) of
// the K; a thread takes one of the A^3 combinations of one input (blockIdx.y), so nothing is formed
// for the offsets the modular check would throw out.  Returns the empty key when the combination
// does not exist for this point or falls outside the boundary.
__device__ __forceinline__ uint64_t candidate_key(uint64_t key, int slot, int K, int s, int A, const Bound &bound) {
    if (key == kEmptyKey) return kEmptyKey;
    int32_t c[4];
    unpack_key(key, c);
    const int r = (K - 1) / 2;
    const int t[3] = {slot / (A * A), (slot / A) % A, slot % A};
    int32_t q[3];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        const int p = c[1 + a];
        const int first = -r + (((p + r) % s) + s) % s;   // smallest offset >= -r congruent to p
        const int d = first + t[a] * s;
        if (d > K - 1 - r) return kEmptyKey;
        const int u = p - d;                               // a multiple of s
        if (bound.on && (u < 0 || u >= bound.hi[a])) return kEmptyKey;
        q[a] = u / s;
    }
    return pack_key(c[0], q[0], q[1], q[2]);
}

__global__ void k_candidates(const uint64_t *keys, int64_t n, int K, int s, int A, Bound bound, uint64_t *cand) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    cand[i * (int64_t)gridDim.y + blockIdx.y] = candidate_key(keys[i], blockIdx.y, K, s, A, bound);
}

// The same candidates, marked in a bitmap over the box the outputs can lie in (one bit per cell, cells
// in (batch, x, y, z) order): Alg. 3's Unique() without a sort, for callers that state their bounds.
__global__ void k_candidates_mark(const uint64_t *keys, int64_t n, int K, int s, int A, Bound bound, Grid cbox,
                                  uint32_t *bits, int *status) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t cand = i < n ? candidate_key(keys[i], blockIdx.y, K, s, A, bound) : kEmptyKey;
    const int64_t cell = cand == kEmptyKey ? -1 : grid_cell(cbox, cand);
    // neighbours in row order are often neighbours in space: a lane whose predecessor marks the same cell stays silent
    const int64_t before = __shfl_up(cell, 1, 64);
    if (cand == kEmptyKey) return;
    if (cell < 0) {
        raise_flag(status, ST_RANGE);
        return;
    }
    if ((threadIdx.x & 63) != 0 && before == cell) return;
    atomicOr(&bits[cell >> 5], 1u << (cell & 31));
}

__global__ void k_drop_empty_key(const uint64_t *uniq, int64_t *count) {
    if (*count > 0 && uniq[*count - 1] == kEmptyKey) --*count;
}

__global__ void k_unpack(const uint64_t *keys, int64_t n, int4 *coords) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int32_t c[4];
    unpack_key(keys[i], c);
    coords[i] = make_int4(c[0], c[1], c[2], c[3]);
}

// ---- distinct offset bitmasks ------------------------------------------------------------------------
// A small open-addressing table bitmask -> number of rows.  Rows take an arrival rank from the
// counter; the distinct masks are ranked afterwards, so rows with equal masks end up adjacent.
// Which of those rows comes first depends on arrival order, which no result depends on: the
// compute kernels add a row's terms in offset order whatever tile the row sits in.
struct MaskHash {
    uint32_t *key;      // [cap]  0xFFFFFFFF = empty
    int32_t *cnt;       // [cap]  rows holding the mask
    int32_t *start;     // [cap]  first sorted position of the mask (filled by the rank step)
    int32_t *dlist;     // [dmax] slots in use, in arrival order
    uint32_t cap_mask;  // cap - 1
    int shift;          // 32 - log2(cap)
    int dmax;           // most distinct masks the fast path ranks
};
constexpr int kMaskHashCap = 1 << 16;
constexpr int kMaskHashMaxDistinct = 1 << 14;
constexpr int kMaskHashMaxSteps = 128;

__device__ __forceinline__ int mask_hash_insert(const MaskHash &mh, uint32_t mask, int *status) {
    // bitmasks are structured keys: mix all bits before taking the top ones
    uint32_t h = mask;
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    uint32_t sl = h >> mh.shift;
    for (int step = 0; step < kMaskHashMaxSteps; ++step) {
        // An ordinary (cached) load first: most masks are in the table already, and a key never
        // changes once set.  A stale "empty" only means the compare-and-swap below decides.
        uint32_t prev = mh.key[sl];
        if (prev == 0xFFFFFFFFu) prev = __hip_atomic_load(&mh.key[sl], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev == 0xFFFFFFFFu) prev = atomicCAS(&mh.key[sl], 0xFFFFFFFFu, mask);
        if (prev == 0xFFFFFFFFu) {
            const int id = atomicAdd(&status[ST_DCOUNT], 1);
            if (id < mh.dmax)
                mh.dlist[id] = (int32_t)sl;
            else
                atomicOr(&status[ST_OVERFLOW], 1);
            return (int)sl;
        }
        if (prev == mask) return (int)sl;
        sl = (sl + 1) & mh.cap_mask;
    }
    atomicOr(&status[ST_OVERFLOW], 1);   // too crowded: the build falls back to a radix sort of the masks
    return -1;
}

// Order in which distinct masks are laid out.  For K = 3 the bits of rarely present offsets
// (corners, then edges, then faces, then the centre) are made the most significant, so that
// neighbouring masks in the order differ in few offsets where rows of several masks share a tile.
struct BitPos27 {
    uint8_t p[27];
};
constexpr BitPos27 make_bitpos27() {
    BitPos27 b{};
    int next = 0;
    for (int cls = 0; cls <= 3; ++cls)
        for (int n = 0; n < 27; ++n) {
            const int nz = (n / 9 != 1) + ((n / 3) % 3 != 1) + (n % 3 != 1);
            if (nz == cls) b.p[n] = (uint8_t)next++;
        }
    return b;
}
__host__ __device__ __forceinline__ uint32_t mask_sort_key(uint32_t mask, int K3) {
    if (K3 != 27) return mask;
    constexpr BitPos27 bp = make_bitpos27();
    uint32_t key = 0;
#pragma unroll
    for (int n = 0; n < 27; ++n) key |= ((mask >> n) & 1u) << bp.p[n];
    return key;
}

// What every search kernel does once a thread knows the offset bitmask of its output row:
// presence bitmaps of the wave's 64 outputs, one per offset, their counts, and the wave's OR.
template <int K3>
__device__ __forceinline__ void finish_rows(uint32_t mask, uint64_t *__restrict__ colbits, int32_t *__restrict__ colcnt,
                                            uint32_t *__restrict__ wavemask, int64_t n_blocks) {
    const int lane = threadIdx.x & 63;
    const int64_t block64 = (int64_t)blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);   // wave-uniform
    uint64_t mine = 0;
#pragma unroll
    for (int n = 0; n < K3; ++n) {
        const uint64_t b = __ballot((mask >> n) & 1u);
        if (lane == n) mine = b;
    }
    if (lane < K3 && block64 < n_blocks) {
        colbits[(int64_t)lane * n_blocks + block64] = mine;
        colcnt[(int64_t)lane * n_blocks + block64] = __popcll(mine);
    }
    // offsets present anywhere in the wave's 64 rows (what a tile of the fused kernel has to visit)
    const uint64_t any = __ballot(lane < K3 && mine != 0);
    if (lane == 0 && block64 < n_blocks) wavemask[block64] = (uint32_t)any;
}

// ts_kmap_sort_rows, step 1: register every row's bitmask in the mask table; slot_rank[k] = (table
// slot, arrival rank among the rows of that mask).  Lanes of a wave holding the same mask share
// one counter update: first the wave's classes of equal masks (registers only), then every class
// leader talks to the table at once.
__global__ void __launch_bounds__(kThreads) k_register(const int32_t *__restrict__ nbr, int64_t n_out, int stride, int K3,
                                                       int *__restrict__ status, MaskHash mh, int2 *__restrict__ slot_rank) {
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const bool ok = k < n_out;
    const uint32_t mask = ok ? (uint32_t)nbr[k * stride + K3] : 0u;
    int my_leader = lane;
    uint64_t my_class = 0;
    uint64_t todo = __ballot(ok);
    while (todo) {
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const uint32_t lm = (uint32_t)__shfl((int)mask, leader, 64);
        const uint64_t same = __ballot(ok && mask == lm);
        if ((same >> lane) & 1ull) {
            my_leader = leader;
            my_class = same;
        }
        todo &= ~same;
    }
    int sl = -1, first = 0;
    if (ok && lane == my_leader) {
        sl = mask_hash_insert(mh, mask, status);
        if (sl >= 0) first = atomicAdd(&mh.cnt[sl], __popcll(my_class));
    }
    const int my_slot = __shfl(sl, my_leader, 64);
    const int my_rank = __shfl(first, my_leader, 64) + __popcll(my_class & ((1ull << lane) - 1ull));
    if (ok) slot_rank[k] = make_int2(my_slot, my_rank);
}

// ---- map search (Alg. 1) -------------------------------------------------------------------------------
enum { MODE_SUB = 0, MODE_FWD = 1, MODE_TR = 2 };

// One thread per output point k.
//   MODE_SUB  stride 1, odd K: neighbour key = key_k + key_delta(delta_n); the centre is k itself
//   MODE_FWD  stride s: input at s*q_k + delta_n
//   MODE_TR   transposed: coarse point (p_k - delta_n)/s when s divides the difference
// Writes nbr[k][0..K3) (input row or -1) and nbr[k][K3] = bitmask of the offsets present; per wave
// (64 consecutive outputs) and offset the presence bitmap and its popcount.  (No global counters
// here: atomics from every wave on one cache line are served one after the other.)
template <int MODE, int K, class TableT>
__global__ void __launch_bounds__(kThreads, 3) k_probe(const uint64_t *__restrict__ out_keys, int64_t n_out, TableT t, int s,
                                                    int32_t *__restrict__ nbr, uint64_t *__restrict__ colbits,
                                                    int32_t *__restrict__ colcnt, uint32_t *__restrict__ wavemask,
                                                    int64_t n_blocks) {
    constexpr int K3 = K * K * K, STRIDE = nbr_stride(K3), CENTRE = (K3 - 1) / 2;
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const uint64_t key = k < n_out ? out_keys[k] : kEmptyKey;
    const bool ok = key != kEmptyKey;
    int32_t c[4] = {0, 0, 0, 0};
    if (MODE != MODE_SUB && ok) unpack_key(key, c);

    // Key searched for offset n.  Stride 1 and forward maps: a base key plus the constant
    // key_delta(delta_n), so a loaded key is tested as (loaded - base == constant) and nothing per
    // offset stays in registers but the slot; transposed maps keep the searched keys.
    uint64_t base = key;
    if (MODE == MODE_FWD) base = pack_key(c[0], s * c[1], s * c[2], s * c[3]);
    auto delta_of = [](int n) -> int64_t {
        constexpr int r = (K - 1) / 2;
        return key_delta(n / (K * K) - r, (n / K) % K - r, n % K - r);
    };
    uint64_t want_tr[MODE == MODE_TR ? K3 : 1];
    auto is_wanted = [&](int n, uint64_t loaded) -> bool {
        if (MODE == MODE_TR) return loaded == want_tr[MODE == MODE_TR ? n : 0];
        return (int64_t)(loaded - base) == delta_of(n);
    };
    // All lookups advance together.  The first load of each (its key only) is issued before any
    // is examined; then rounds: lookups whose slot held another key move on together, so a wave
    // pays one memory access time per round, not per collision.  A finished lookup leaves the
    // slot it hit (or none); the values are fetched in one last batch.
    // searched key of offset n, and whether there is anything to search for
    auto wanted = [&](int n, bool *probe) -> uint64_t {
        *probe = ok && !(MODE == MODE_SUB && n == CENTRE);
        uint64_t want = base + (uint64_t)delta_of(n);
        if (MODE == MODE_TR) {
            constexpr int r = (K - 1) / 2;
            const int ux = c[1] - (n / (K * K) - r), uy = c[2] - ((n / K) % K - r), uz = c[3] - (n % K - r);
            *probe = ok && ux % s == 0 && uy % s == 0 && uz % s == 0;
            want = pack_key(c[0], ux / s, uy / s, uz / s);
        }
        return want;
    };
    int32_t j[K3];
    if constexpr (std::is_same<TableT, Grid>::value) {
        // a grid lookup is one load and the K3 loads of a thread do not depend on each other
#pragma unroll
        for (int n = 0; n < K3; ++n) {
            bool probe;
            const uint64_t want = wanted(n, &probe);
            j[n] = (MODE == MODE_SUB && n == CENTRE && ok) ? (int32_t)k : -1;
            if (probe) j[n] = table_find(t, want);
        }
    } else {
    constexpr uint32_t kNone = 0xFFFFFFFFu;
    uint32_t slot[K3];
    uint64_t got[K3];
    uint32_t pending = 0;   // bit n: lookup n has not ended yet
#pragma unroll
    for (int n = 0; n < K3; ++n) {
        bool probe;
        const uint64_t want = wanted(n, &probe);
        if (MODE == MODE_TR) want_tr[MODE == MODE_TR ? n : 0] = want;
        slot[n] = kNone;
        if (probe) {
            pending |= 1u << n;
            slot[n] = home_slot(want, t.shift);
            got[n] = slot_key(t, slot[n]);
        }
    }
    for (;;) {
#pragma unroll
        for (int n = 0; n < K3; ++n) {
            if ((pending >> n) & 1u) {
                if (is_wanted(n, got[n])) {
                    pending &= ~(1u << n);
                } else if (got[n] == kEmptyKey) {
                    pending &= ~(1u << n);
                    slot[n] = kNone;
                }
            }
        }
        if (__ballot(pending != 0) == 0) break;
#pragma unroll
        for (int n = 0; n < K3; ++n) {
            if ((pending >> n) & 1u) {
                slot[n] = next_slot(slot[n], t.mask);
                got[n] = slot_key(t, slot[n]);
            }
        }
    }
#pragma unroll
    for (int n = 0; n < K3; ++n) {
        j[n] = (MODE == MODE_SUB && n == CENTRE && ok) ? (int32_t)k : -1;
        if (slot[n] != kNone) j[n] = slot_val(t, slot[n]);
    }
    }
    uint32_t mask = 0;
#pragma unroll
    for (int n = 0; n < K3; ++n)
        if (j[n] >= 0) mask |= 1u << n;

    // the row of the out-major table
    if (k < n_out) {
        constexpr int CHUNKS = (K3 + 1 + 3) / 4;
        int4 *dst = reinterpret_cast<int4 *>(nbr + k * STRIDE);
#pragma unroll
        for (int ch = 0; ch < CHUNKS; ++ch) {
            int32_t v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int idx = ch * 4 + q;
                v[q] = idx < K3 ? j[idx < K3 ? idx : 0] : (idx == K3 ? (int32_t)mask : 0);
            }
            dst[ch] = make_int4(v[0], v[1], v[2], v[3]);
        }
    }

    finish_rows<K3>(mask, colbits, colcnt, wavemask, n_blocks);
}

// Map search for stride 1, K = 3, one lane per (point i, offset n) with n below the centre.
// A hit (j at p_i + delta_n) gives two entries: (j, i, n) in row i and, by symmetry (Sec. 4.2.1),
// (i, j, K^3-1-n) in row j; rows start out all -1.  One lookup per lane: a long probe chain
// delays one wave of 64 lookups, not a wave holding all 26 lookups of 64 points, and the many
// waves in flight hide the memory round trips.  The 13 offsets of a point sit in neighbouring lanes
// (16 lanes per point), so a point's own entries land in one cache line of the table: with a lane per
// point and the offset in the grid's y, every hit was a 4-byte write into a line of its own, and the
// kernel took 34 us instead of 22.
template <class TableT>
__global__ void k_probe_symmetric(const uint64_t *__restrict__ keys, int64_t n_pts, TableT t, int K,
                                  int32_t *__restrict__ nbr, int stride) {
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = g >> 4;
    const int n = (int)(g & 15), K3 = K * K * K;
    if (i >= n_pts || n >= K3 / 2) return;
    const uint64_t key = keys[i];
    if (key == kEmptyKey) return;
    const uint64_t want = (uint64_t)((int64_t)key + key_delta(offset_component(K, n, 0), offset_component(K, n, 1), offset_component(K, n, 2)));
    const int32_t j = table_find(t, want);
    if (j >= 0) {
        nbr[i * stride + n] = j;
        nbr[(int64_t)j * stride + (K3 - 1 - n)] = (int32_t)i;
    }
}

// Row pass over a neighbour table whose hits have been written into rows that started out as -1
// (the symmetric probe; the transposition of a forward map): a thread per output row reads its
// row, sets the centre entry where the map has one (stride 1: output k is input k) and the row's
// offset bitmask, and does what every search kernel does once the bitmask is known.
template <int K3, bool HAS_CENTRE>
__global__ void __launch_bounds__(kThreads) k_rows(int32_t *__restrict__ nbr, const uint64_t *__restrict__ keys, int64_t n_out,
                                                   uint64_t *__restrict__ colbits, int32_t *__restrict__ colcnt,
                                                   uint32_t *__restrict__ wavemask, int64_t n_blocks) {
    constexpr int STRIDE = nbr_stride(K3), CHUNKS = (K3 + 3) / 4, CENTRE = (K3 - 1) / 2;
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool ok = k < n_out && keys[k] != kEmptyKey;
    uint32_t mask = 0;
    if (ok) {
        int32_t j[CHUNKS * 4];
#pragma unroll
        for (int ch = 0; ch < CHUNKS; ++ch) {
            const int4 v = reinterpret_cast<const int4 *>(nbr + k * STRIDE)[ch];
            j[ch * 4 + 0] = v.x;
            j[ch * 4 + 1] = v.y;
            j[ch * 4 + 2] = v.z;
            j[ch * 4 + 3] = v.w;
        }
#pragma unroll
        for (int n = 0; n < K3; ++n)
            if ((HAS_CENTRE && n == CENTRE) || j[n] >= 0) mask |= 1u << n;
        if (HAS_CENTRE) nbr[k * STRIDE + CENTRE] = (int32_t)k;
        nbr[k * STRIDE + K3] = (int32_t)mask;
    } else if (k < n_out) {
        nbr[k * STRIDE + K3] = 0;   // a row of an invalid coordinate (the build reports the error) has no neighbours
    }
    finish_rows<K3>(mask, colbits, colcnt, wavemask, n_blocks);
}

// Transposition of a forward map: entry (input j, output k, offset n) of the forward table becomes
// entry (input k, output j, offset n).  A thread per forward output row.
template <int K3>
__global__ void __launch_bounds__(kThreads) k_transpose(const int32_t *__restrict__ fwd, int64_t n_fwd_out,
                                                        int32_t *__restrict__ tnbr) {
    constexpr int STRIDE = nbr_stride(K3), CHUNKS = (K3 + 3) / 4;
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (k >= n_fwd_out) return;
    int32_t j[CHUNKS * 4];
#pragma unroll
    for (int ch = 0; ch < CHUNKS; ++ch) {
        const int4 v = reinterpret_cast<const int4 *>(fwd + k * STRIDE)[ch];
        j[ch * 4 + 0] = v.x;
        j[ch * 4 + 1] = v.y;
        j[ch * 4 + 2] = v.z;
        j[ch * 4 + 3] = v.w;
    }
#pragma unroll
    for (int n = 0; n < K3; ++n)
        if (j[n] >= 0) tnbr[(int64_t)j[n] * STRIDE + n] = (int32_t)k;
}

template <int THREADS = kThreads>
__device__ __forceinline__ int block_exclusive_scan(int v, int *total) {
    __shared__ int wave_sums[THREADS / 64];
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
    for (int d = 1; d < 64; d <<= 1) {
        int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int base = 0, all = 0;
    for (int w = 0; w < THREADS / 64; ++w) {
        int sw = wave_sums[w];
        if (w < wave) base += sw;
        all += sw;
    }
    __syncthreads();
    *total = all;
    return base + incl - v;
}

// ---- marked cells -> sorted distinct keys ------------------------------------------------------------------
// Bits set per block of 256 words.
__global__ void __launch_bounds__(kThreads) k_bits_count(const uint64_t *__restrict__ words, int64_t n_words,
                                                         int32_t *__restrict__ block_total) {
    const int64_t w = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    int total;
    block_exclusive_scan(w < n_words ? __popcll(words[w]) : 0, &total);
    if (threadIdx.x == 0) block_total[blockIdx.x] = total;
}

// One block: block_total[] -> its exclusive prefix in place, and the grand total.
__global__ void __launch_bounds__(kThreads) k_bits_scan(int32_t *__restrict__ block_total, int64_t n, int64_t *__restrict__ count) {
    int64_t run = 0;
    for (int64_t base = 0; base < n; base += kThreads) {
        const int64_t i = base + threadIdx.x;
        const int v = i < n ? block_total[i] : 0;
        int total;
        const int before = block_exclusive_scan(v, &total);
        if (i < n) block_total[i] = (int32_t)(run + before);
        run += total;
    }
    if (threadIdx.x == 0) *count = run;
}

// Every set bit becomes the key of its cell, at the rank of the bit: cells are numbered in
// (batch, x, y, z) order, which is the order of the keys.  word_base[w] receives the rank of word w's
// first set bit (the number of set bits before the word): the rank of any marked cell is then one load
// of it, one of the word, and a popcount.  self_scan: block_total[] still holds the per-block counts and
// every block sums the ones before it itself (a few thousand L2-resident words), which saves the scan
// launch in between; the last block then also writes the grand total.
__global__ void __launch_bounds__(kThreads) k_bits_expand(const uint64_t *__restrict__ words, int64_t n_words,
                                                          const int32_t *__restrict__ block_base, Grid cbox,
                                                          uint64_t *__restrict__ out_keys, int32_t *__restrict__ word_base,
                                                          int self_scan, int64_t *__restrict__ count) {
    const int64_t w = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    uint64_t bits = w < n_words ? words[w] : 0;
    int64_t before = 0;
    if (self_scan) {
        int part = 0;
        for (int i = threadIdx.x; i < (int)blockIdx.x; i += kThreads) part += block_base[i];
        int sum;
        block_exclusive_scan(part, &sum);
        before = sum;
    } else {
        before = block_base[blockIdx.x];
    }
    int total;
    int64_t at = before + block_exclusive_scan(__popcll(bits), &total);
    if (self_scan && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *count = before + total;
    if (w < n_words) word_base[w] = (int32_t)at;
    if (bits == 0) return;
    // coordinates of the word's first cell once (a box holds at most 2^30 cells: 32-bit arithmetic),
    // then every set bit is that cell moved along z, carrying into y, x and the batch index
    uint32_t cell = (uint32_t)w * 64u;
    uint32_t z0 = cell % cbox.ext[2];
    cell /= cbox.ext[2];
    uint32_t y0 = cell % cbox.ext[1];
    cell /= cbox.ext[1];
    uint32_t x0 = cell % cbox.ext[0], b0 = cell / cbox.ext[0];
    // (the bits come in ascending order, so the cell only ever moves forward: a word costs 64 / ext z
    // carries in all, not that many per set bit, which on the flat boxes of coarse levels was the whole kernel)
    uint32_t z = z0, y = y0, x = x0, b = b0;
    int prev = 0;
    while (bits) {
        const int bit = __builtin_ctzll(bits);
        bits &= bits - 1;
        z += (uint32_t)(bit - prev);
        prev = bit;
        while (z >= cbox.ext[2]) {
            z -= cbox.ext[2];
            if (++y == cbox.ext[1]) {
                y = 0;
                if (++x == cbox.ext[0]) {
                    x = 0;
                    ++b;
                }
            }
        }
        out_keys[at++] = pack_key((int32_t)b, (int32_t)x + cbox.lo[0], (int32_t)y + cbox.lo[1], (int32_t)z + cbox.lo[2]);
    }
}

// Strided maps without a search.  Every admissible candidate (p_j - delta_n) / s of an input p_j that
// Alg. 3 keeps IS an output point, so the pair (j, k, n) of Alg. 1 follows from the candidate alone: k is
// the rank of the candidate's cell among the marked cells (outputs are numbered in cell order).  A lane per
// (input, admissible offset combination), as in k_candidates_mark.
//   forward     nbr[k][n] = j, written with a compare-and-swap against -1: two inputs with one coordinate
//               meet in one entry, which is how duplicates are found
//   transposed  nbr[j][n] = k (rows belong to the given fine points; the roles are swapped)
// Rows start out as -1; the row pass (k_rows) adds bitmasks and presence bitmaps afterwards.
template <bool TRANSPOSED>
__global__ void __launch_bounds__(kThreads) k_rank_scatter(const uint64_t *__restrict__ keys, int64_t n, int K, int s, int A,
                                                           Bound bound, Grid cbox, const uint64_t *__restrict__ words,
                                                           const int32_t *__restrict__ word_base, int32_t *__restrict__ nbr,
                                                           int stride, int *status) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint64_t key = keys[i];
    const uint64_t cand = candidate_key(key, blockIdx.y, K, s, A, bound);
    if (cand == kEmptyKey) return;
    const int64_t cell = grid_cell(cbox, cand);
    if (cell < 0) return;                       // k_candidates_mark has raised the flag
    const int32_t k = word_base[cell >> 6] + __popcll(words[cell >> 6] & ((1ull << (cell & 63)) - 1ull));
    // the offset: delta = p - s * q per axis
    int32_t p[4], q[4];
    unpack_key(key, p);
    unpack_key(cand, q);
    const int r = (K - 1) / 2;
    const int nidx = ((p[1] - s * q[1] + r) * K + (p[2] - s * q[2] + r)) * K + (p[3] - s * q[3] + r);
    if (TRANSPOSED) {
        nbr[i * stride + nidx] = k;
    } else {
        if (atomicCAS(&nbr[(int64_t)k * stride + nidx], -1, (int32_t)i) != -1) raise_flag(status, ST_DUP);
    }
}

// Block n: exclusive scan of colcnt[n][*] -> colbase[n][b] = pairs of offset n in the 64-row
// blocks before b (relative to the start of the offset's list), and the offset's total (the host
// turns the totals into offs[], the start of each offset's list, and hands them to later kernels
// by value).
constexpr int kScanThreads = 1024, kScanItems = 4;
__global__ void __launch_bounds__(kScanThreads) k_scan(const int32_t *__restrict__ colcnt, int32_t *__restrict__ colbase,
                                                       int64_t n_blocks, int *__restrict__ status, int K3,
                                                       const uint32_t *__restrict__ wavemask, int64_t n_tiles,
                                                       int32_t *__restrict__ tile_order) {
    if ((int)blockIdx.x == K3) {
        // The extra block: tiles of 128 outputs (two waves of the search) in descending order of
        // the number of offsets they meet, a counting sort.  The fused kernel takes tiles in this
        // order, so that the long ones do not start when everything else is done.
        __shared__ int hist[32], base[32];
        if (threadIdx.x < 32) hist[threadIdx.x] = 0;
        __syncthreads();
        auto offsets_of = [&](int64_t t) {
            const uint32_t a = wavemask[2 * t], b = 2 * t + 1 < n_blocks ? wavemask[2 * t + 1] : 0u;
            return __builtin_popcount(a | b);
        };
        for (int64_t t = threadIdx.x; t < n_tiles; t += kScanThreads) atomicAdd(&hist[offsets_of(t)], 1);
        __syncthreads();
        if (threadIdx.x == 0) {
            int at = 0;
            for (int c = 31; c >= 0; --c) {
                base[c] = at;
                at += hist[c];
            }
        }
        __syncthreads();
        for (int64_t t = threadIdx.x; t < n_tiles; t += kScanThreads) tile_order[atomicAdd(&base[offsets_of(t)], 1)] = (int32_t)t;
        return;
    }
    const int n = blockIdx.x;
    const int32_t *src = colcnt + (int64_t)n * n_blocks;
    int32_t *dst = colbase + (int64_t)n * n_blocks;
    int run = 0;
    for (int64_t base = 0; base < n_blocks; base += kScanThreads * kScanItems) {
        const int64_t i0 = base + (int64_t)threadIdx.x * kScanItems;
        int v[kScanItems], sum = 0;
#pragma unroll
        for (int e = 0; e < kScanItems; ++e) {
            v[e] = i0 + e < n_blocks ? src[i0 + e] : 0;
            sum += v[e];
        }
        int total;
        int at = run + block_exclusive_scan<kScanThreads>(sum, &total);
#pragma unroll
        for (int e = 0; e < kScanItems; ++e) {
            if (i0 + e < n_blocks) dst[i0 + e] = at;
            at += v[e];
        }
        run += total;
    }
    if (threadIdx.x == 0) status[ST_TOTALS + n] = run;
}

// ts_kmap_sort_rows, step 2: the distinct bitmasks as a dense list of (sort key, rows), followed
// by sentinel entries that sort last and hold no rows.
constexpr int kRankSlices = 32, kRankPer = 4, kRankUnroll = 16;
constexpr int kDensePad = kRankSlices * kRankUnroll;
__global__ void k_dense(const int *__restrict__ status, MaskHash mh, int K3, int2 *__restrict__ dense) {
    int D = status[ST_DCOUNT];
    D = D < mh.dmax ? D : mh.dmax;
    const int d = blockIdx.x * blockDim.x + threadIdx.x;
    if (d < D) {
        const int sl = mh.dlist[d];
        dense[d] = make_int2((int)mask_sort_key(mh.key[sl], K3), mh.cnt[sl]);
    } else if (d < mh.dmax + kDensePad) {
        dense[d] = make_int2(-1, 0);
    }
}

// ts_kmap_sort_rows, step 3: start of mask d = rows whose mask sorts lower.  Block (d-block, slice)
// adds up, for 1024 masks (4 per thread), the rows of the lower masks found in one slice of the
// list; k_rank_sum adds the slices.  The list is read with wave-uniform addresses (scalar loads),
// so the inner loop is compare / select / add only.
__global__ void __launch_bounds__(kThreads) k_rank_partial(const int2 *__restrict__ dense, const int *__restrict__ status,
                                                           int dmax, int32_t *__restrict__ partial) {
    const int rb = blockIdx.x, dblk = rb / kRankSlices, slice = rb % kRankSlices;
    int D = status[ST_DCOUNT];
    D = D < dmax ? D : dmax;
    if (dblk * kThreads * kRankPer >= D) return;
    // slices are whole groups of kRankUnroll entries; what lies behind the list are sentinels
    const int per = ((D + kRankSlices - 1) / kRankSlices + kRankUnroll - 1) / kRankUnroll * kRankUnroll;
    const int lo = slice * per, hi = lo + per;
    uint32_t my_key[kRankPer];
    int sum[kRankPer];
#pragma unroll
    for (int e = 0; e < kRankPer; ++e) {
        const int d = (dblk * kRankPer + e) * kThreads + threadIdx.x;
        my_key[e] = d < D ? (uint32_t)dense[d].x : 0u;
        sum[e] = 0;
    }
    for (int q = lo; q < hi; q += kRankUnroll) {
        int2 kc[kRankUnroll];   // same addresses in every lane; all loaded before the first use
#pragma unroll
        for (int u = 0; u < kRankUnroll; ++u) kc[u] = dense[q + u];
#pragma unroll
        for (int u = 0; u < kRankUnroll; ++u)
#pragma unroll
            for (int e = 0; e < kRankPer; ++e) sum[e] += (uint32_t)kc[u].x < my_key[e] ? kc[u].y : 0;
    }
#pragma unroll
    for (int e = 0; e < kRankPer; ++e) {
        const int d = (dblk * kRankPer + e) * kThreads + threadIdx.x;
        if (d < D) partial[(int64_t)slice * dmax + d] = sum[e];
    }
}

__global__ void k_rank_sum(const int32_t *__restrict__ partial, const int *__restrict__ status, MaskHash mh) {
    int D = status[ST_DCOUNT];
    D = D < mh.dmax ? D : mh.dmax;
    const int d = blockIdx.x * blockDim.x + threadIdx.x;
    if (d >= D) return;
    int sum = 0;
#pragma unroll
    for (int sl = 0; sl < kRankSlices; ++sl) sum += partial[(int64_t)sl * mh.dmax + d];
    mh.start[mh.dlist[d]] = sum;
}

// ts_kmap_sort_rows, step 4: perm[start of the row's mask + arrival rank] = row.
__global__ void k_place(const int2 *__restrict__ slot_rank, int64_t n_out, MaskHash mh, int32_t *__restrict__ perm) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_out) return;
    const int2 sr = slot_rank[k];
    if (sr.x < 0) return;
    const int64_t pos = (int64_t)mh.start[sr.x] + sr.y;
    if (pos >= 0 && pos < n_out) perm[pos] = (int32_t)k;   // (out of range only when the table overflowed)
}

// Pair lists: thread per output row; the pair (k, n) goes to offs[n] + colbase[n][k/64] + (outputs of the
// same 64-block with offset n before k), which keeps ascending output order inside an offset.
template <int K3>
__global__ void __launch_bounds__(kThreads) k_compact(const int32_t *__restrict__ nbr, int64_t n_out,
                                                      const int32_t *__restrict__ colbase, int64_t n_blocks,
                                                      Offs offs, int32_t *__restrict__ in_idx,
                                                      int32_t *__restrict__ out_idx) {
    constexpr int STRIDE = nbr_stride(K3), CHUNKS = (K3 + 3) / 4;
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const int64_t block64 = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    int base_mine = 0;
    if (lane < K3 && block64 < n_blocks) base_mine = offs.v[lane] + colbase[(int64_t)lane * n_blocks + block64];
    int32_t j[CHUNKS * 4];
#pragma unroll
    for (int ch = 0; ch < CHUNKS; ++ch) {
        int4 v = make_int4(-1, -1, -1, -1);
        if (k < n_out) v = reinterpret_cast<const int4 *>(nbr + k * STRIDE)[ch];
        j[ch * 4 + 0] = v.x;
        j[ch * 4 + 1] = v.y;
        j[ch * 4 + 2] = v.z;
        j[ch * 4 + 3] = v.w;
    }
#pragma unroll
    for (int n = 0; n < K3; ++n) {
        const bool has = j[n] >= 0;
        const uint64_t bal = __ballot(has);
        const int base = __shfl(base_mine, n, 64);
        if (has) {
            const int p = base + __popcll(bal & ((1ull << lane) - 1ull));
            in_idx[p] = j[n];
            out_idx[p] = (int32_t)k;
        }
    }
}

// Fallback ordering input: the sort key of each row's bitmask and the identity row list.
__global__ void k_extract_masks(const int32_t *__restrict__ nbr, int64_t n_out, int stride, int K3,
                                uint32_t *__restrict__ keys, int32_t *__restrict__ rows) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_out) return;
    keys[k] = mask_sort_key((uint32_t)nbr[k * stride + K3], K3);
    rows[k] = (int32_t)k;
}

inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

// Owns the temporaries of one build; everything goes back to the pool on scope exit.
struct Temps {
    void *p[48];
    int n = 0;
    template <class T>
    int get(T **out, size_t count) {
        int rc = alloc_n(out, count);
        if (rc == TS_OK) p[n++] = *out;
        return rc;
    }
    ~Temps() {
        for (int i = 0; i < n; ++i) dev_free(p[i]);
    }
};

int launch_fill(const FillArgs &f) {
    if (f.n == 0) return TS_OK;
    uint64_t most = 0;
    for (int i = 0; i < f.n; ++i) most = f.seg[i].n_vec > most ? f.seg[i].n_vec : most;
    unsigned blocks = blocks_for((int64_t)most, kThreads);
    if (blocks > 4096) blocks = 4096;
    TS_LAUNCH("k_fill", k_fill, dim3(blocks), dim3(kThreads), f);
    return TS_OK;
}

// Allocates the table; its clearing is added to `fill`.
int make_table(Temps &tmp, int64_t entries, Table *t, FillArgs *fill) {
    uint64_t cap = 1024;
    while (cap < (uint64_t)(4 * entries)) cap <<= 1;
    if (cap > (1ull << 28)) return fail(TS_ERR_UNSUPPORTED, "too many points for the hash table");
    TS_TRY(tmp.get(&t->keys, cap));
    TS_TRY(tmp.get(&t->vals, cap));
    t->mask = (uint32_t)(cap - 1);
    t->shift = 64 - __builtin_ctzll(cap >> kBucketLog2);
    fill->add(t->keys, cap * sizeof(uint64_t), 0xFFFFFFFFu);
    return TS_OK;
}

// How a build was asked to run.
struct BuildOpts {
    bool wait = true;
    bool measure = false;   // strided builds: measure the bounding box on the device and use the grid if it is small enough
    bool grid = false;      // hold the searched set in the coordinate grid instead of the hash table
    Box box = {};           // bounds stated for the caller's coordinates (grid search)
    Bound bound = {};       // Alg. 3's boundary, already multiplied by the stride
};

// The searched point set of a build: in the hash table or in the grid.
struct Searched {
    bool grid = false;
    Table t = {};
    Grid g = {};
};

// The grid's cells: kept between builds, every cell -1 whenever no build is using them.
constexpr uint64_t kMaxGridCells = 1ull << 30;    // 4 GiB of cells: what a caller may ask for
constexpr uint64_t kAutoGridCells = 1ull << 28;   // output cells (bits of the bitmap: 32 MiB) up to which a strided build
                                                  // that measures its own box marks its candidates instead of sorting them
int32_t *g_grid = nullptr;
uint64_t g_grid_cells = 0;
bool g_grid_dirty = false;   // a build put points in and did not get as far as taking them out

// A grid over batches x [lo, hi] (inclusive).  Grows the buffer when the box needs more cells than it
// has; clears it only when new or left dirty by a build that failed half way.
int acquire_grid(const int32_t lo[3], const int32_t hi[3], int batches, Grid *g) {
    uint64_t cells = (uint64_t)batches;
    for (int a = 0; a < 3; ++a) {
        const int64_t ext = (int64_t)hi[a] - lo[a] + 1;
        if (ext <= 0 || batches <= 0) return fail(TS_ERR_INVALID_ARG, "empty grid bounds");
        g->lo[a] = lo[a];
        g->ext[a] = (uint32_t)ext;
        cells *= (uint64_t)ext;
        if (cells > kMaxGridCells)
            return fail(TS_ERR_UNSUPPORTED, "the grid bounds span more than %llu cells", (unsigned long long)kMaxGridCells);
    }
    g->batches = (uint32_t)batches;
    if (cells > g_grid_cells) {
        if (g_grid) {
            TS_HIP(hipStreamSynchronize(stream()));
            (void)hipFree(g_grid);
            g_grid = nullptr;
            g_grid_cells = 0;
        }
        const uint64_t want = (cells + 3) & ~3ull;
        if (hipMalloc(&g_grid, want * sizeof(int32_t)) != hipSuccess) {
            (void)hipGetLastError();
            g_grid = nullptr;
            return fail(TS_ERR_OOM, "no memory for a grid of %llu cells", (unsigned long long)cells);
        }
        g_grid_cells = want;
        g_grid_dirty = true;
    }
    if (g_grid_dirty) {
        FillArgs f;
        f.add(g_grid, g_grid_cells * sizeof(int32_t), 0xFFFFFFFFu);
        TS_TRY(launch_fill(f));
    }
    g_grid_dirty = true;   // until this build has taken its points out again
    g->vals = g_grid;
    return TS_OK;
}

// Table or grid for `entries` points inside batches x [lo, hi].
int make_searched(Temps &tmp, const BuildOpts &o, int64_t entries, const int32_t lo[3], const int32_t hi[3], Searched *sd,
                  FillArgs *fill) {
    sd->grid = o.grid;
    if (o.grid) return acquire_grid(lo, hi, o.box.batches, &sd->g);
    return make_table(tmp, entries, &sd->t, fill);
}

int make_mask_hash(Temps &tmp, MaskHash *mh, FillArgs *fill) {
    int32_t *cnt_start;
    TS_TRY(tmp.get(&mh->key, (size_t)kMaskHashCap));
    TS_TRY(tmp.get(&cnt_start, (size_t)2 * kMaskHashCap));
    TS_TRY(tmp.get(&mh->dlist, (size_t)kMaskHashMaxDistinct));
    mh->cnt = cnt_start;
    mh->start = cnt_start + kMaskHashCap;
    mh->cap_mask = kMaskHashCap - 1;
    mh->shift = 32 - __builtin_ctz(kMaskHashCap);
    mh->dmax = kMaskHashMaxDistinct;
    fill->add(mh->key, (size_t)kMaskHashCap * sizeof(uint32_t), 0xFFFFFFFFu);
    // counts and first positions: a mask that entered the table after the list of distinct masks
    // was full is never ranked, and its rows must not be placed through a stale position
    fill->add(cnt_start, (size_t)2 * kMaskHashCap * sizeof(int32_t), 0u);
    return TS_OK;
}

// Pinned landing places for the status words of builds whose caller did not wait
// (ts_build_kmap_async), each with the event that says the copy has arrived.
struct StatusSlot {
    int32_t *host = nullptr;
    int32_t *dev = nullptr;     // the same words as kernels address them
    hipEvent_t ev = nullptr;
    bool busy = false;          // a copy is in flight or has not been read yet
    const ts_kmap *owner = nullptr;   // NULL while busy: the map was freed before anyone asked
};
constexpr int kStatusSlots = 64;
StatusSlot g_slots[kStatusSlots];

int slot_acquire() {
    static int32_t *mem = nullptr;
    if (!mem) {
        if (hipHostMalloc(&mem, kStatusSlots * ST_WORDS * sizeof(int32_t), hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            mem = nullptr;
            return -1;
        }
        void *dview = nullptr;
        if (hipHostGetDevicePointer(&dview, mem, 0) != hipSuccess) {
            (void)hipGetLastError();
            dview = nullptr;
        }
        for (int i = 0; i < kStatusSlots; ++i) {
            g_slots[i].host = mem + i * ST_WORDS;
            g_slots[i].dev = dview ? static_cast<int32_t *>(dview) + i * ST_WORDS : nullptr;
        }
    }
    for (int i = 0; i < kStatusSlots; ++i) {
        StatusSlot &s = g_slots[i];
        if (s.busy && !s.owner && hipEventQuery(s.ev) == hipSuccess) s.busy = false;   // orphan whose copy has landed
        if (s.busy) continue;
        if (!s.ev && hipEventCreateWithFlags(&s.ev, hipEventDisableTiming) != hipSuccess) {
            (void)hipGetLastError();
            s.ev = nullptr;
            return -1;
        }
        return i;
    }
    (void)hipGetLastError();   // hipEventQuery leaves hipErrorNotReady behind
    return -1;
}

// Status words on the host -> the map's sizes, or its error.
int take_status(ts_kmap *m, const int32_t *h) {
    if (h[ST_RANGE]) m->error = TS_ERR_COORD_RANGE;
    else if (h[ST_DUP]) m->error = TS_ERR_DUPLICATE_COORD;
    m->offs[0] = 0;
    for (int n = 0; n < m->K3; ++n) m->offs[n + 1] = m->offs[n] + h[ST_TOTALS + n];
    for (int n = 0; n < m->K3; ++n) m->sizes[n] = m->offs[n + 1] - m->offs[n];
    m->M = m->offs[m->K3];
    return m->error;
}

int report(const ts_kmap *m) {
    if (m->error == TS_ERR_COORD_RANGE)
        return fail(TS_ERR_COORD_RANGE, "coordinate outside batch [0,%d] / xyz [%d,%d], or outside the grid bounds given", TS_BATCH_MAX, TS_COORD_MIN, TS_COORD_MAX);
    if (m->error == TS_ERR_DUPLICATE_COORD) return fail(TS_ERR_DUPLICATE_COORD, "input coordinates are not distinct");
    return m->error;
}

// The map of a 1x1x1 convolution at stride 1 over n distinct points, written out directly: output k
// takes input k through the only offset (Eq. 1 with delta = 0).  One pass fills the neighbour rows
// (entry, then the bitmask word), the rank structure (every row present: bitmap words of ones, base 64 b)
// and the tile order.
__global__ void __launch_bounds__(kThreads) k_identity_map(int32_t *__restrict__ nbr, int stride, uint64_t *__restrict__ colbits,
                                                           int32_t *__restrict__ colbase, int32_t *__restrict__ tile_order,
                                                           int64_t n, int64_t n_blocks, int64_t n_tiles) {
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (g < n) {
        int4 row = make_int4((int32_t)g, 1, -1, -1);
        *reinterpret_cast<int4 *>(nbr + g * stride) = row;
    }
    if (g < n_blocks) {
        const int64_t left = n - g * 64;
        colbits[g] = left >= 64 ? ~0ull : ((1ull << left) - 1ull);
        colbase[g] = (int32_t)(g * 64);
    }
    if (g < n_tiles) tile_order[g] = (int32_t)g;
}

void destroy(ts_kmap *m) {
    if (!m) return;
    if (m->pending_slot >= 0) g_slots[m->pending_slot].owner = nullptr;   // the slot frees itself when its copy has landed
    if (m->d_out_keys != m->d_in_keys) dev_free(m->d_out_keys);
    dev_free(m->d_in_keys);
    dev_free(m->d_nbr);
    dev_free(m->d_in_idx);
    dev_free(m->d_out_idx);
    dev_free(m->d_colbits);
    dev_free(m->d_colbase);
    dev_free(m->d_perm);
    dev_free(m->d_sched);
    dev_free(m->d_tile_order);
    delete m;
}

int sort_keys(Temps &tmp, uint64_t *in, uint64_t *out, size_t n) {
    size_t bytes = 0;
    TS_HIP(rocprim::radix_sort_keys(nullptr, bytes, in, out, n, 0, 64, stream()));
    void *ws;
    TS_TRY(tmp.get((char **)&ws, bytes));
    ProfScope ps("sort_keys");
    TS_HIP(rocprim::radix_sort_keys(ws, bytes, in, out, n, 0, 64, stream()));
    return TS_OK;
}

template <int MODE, int K>
void launch_probe(const ts_kmap *m, const Searched &sd, int32_t *colcnt, uint32_t *wavemask) {
    if (sd.grid)
        TS_LAUNCH("k_probe_grid", (k_probe<MODE, K, Grid>), dim3(blocks_for(m->n_out, kThreads)), dim3(kThreads), m->d_out_keys,
                  m->n_out, sd.g, m->s, m->d_nbr, m->d_colbits, colcnt, wavemask, m->n_blocks);
    else
        TS_LAUNCH("k_probe", (k_probe<MODE, K, Table>), dim3(blocks_for(m->n_out, kThreads)), dim3(kThreads), m->d_out_keys,
                  m->n_out, sd.t, m->s, m->d_nbr, m->d_colbits, colcnt, wavemask, m->n_blocks);
}

// Map search and everything after it.  `table` holds the searched point set (the map's inputs);
// m->d_out_keys the outputs; the clearing of the status words (and of the neighbour table where the
// search writes hits only) has been enqueued.
int deliver_status(ts_kmap *m, int *d_status, bool wait);
int search_and_finish(ts_kmap *m, Temps &tmp, const Searched &table, int *d_status, bool wait, int early_slot = -1) {
    hipStream_t st = stream();
    const int K3 = m->K3, K = m->K;
    const int64_t n_out = m->n_out;
    int32_t *colcnt;
    uint32_t *wavemask;
    TS_TRY(tmp.get(&colcnt, (size_t)K3 * m->n_blocks));
    TS_TRY(tmp.get(&wavemask, (size_t)m->n_blocks));
    const int mode = m->s == 1 ? MODE_SUB : (m->transposed ? MODE_TR : MODE_FWD);
    // a grid gets its points taken out as soon as the search has been enqueued
    auto after_search = [&]() {
        if (!table.grid) return;
        TS_LAUNCH("k_grid_erase", k_grid_erase, dim3(blocks_for(m->n_in, kThreads)), dim3(kThreads), m->d_in_keys, m->n_in, table.g);
        g_grid_dirty = false;
    };
    if (mode == MODE_SUB && K == 1) launch_probe<MODE_SUB, 1>(m, table, colcnt, wavemask);
    else if (mode == MODE_SUB && K == 3) {
        // 16 lanes per point (13 at work): a point's own entries land in one cache line of the table
        const dim3 lanes(blocks_for(n_out * 16, kThreads));
        if (table.grid)
            TS_LAUNCH("k_probe_symmetric_grid", k_probe_symmetric<Grid>, lanes, dim3(kThreads), m->d_out_keys, n_out, table.g, K,
                      m->d_nbr, m->stride);
        else
            TS_LAUNCH("k_probe_symmetric", k_probe_symmetric<Table>, lanes, dim3(kThreads), m->d_out_keys, n_out, table.t, K,
                      m->d_nbr, m->stride);
        after_search();
        if (!wait) {
            // A caller that does not wait gets the map with its search done: what the fused layer
            // kernel reads.  The row pass and the scan (bitmask words, rank bitmaps, sizes, tile order)
            // run when something first needs them (ts::resolve).  Error flags are known already.
            // (early_slot: the kernels raised their flags in the slot's pinned words themselves.)
            const int slot = early_slot >= 0 ? early_slot : slot_acquire();
            if (slot >= 0) {
                StatusSlot &sl = g_slots[slot];
                if (early_slot < 0) TS_HIP(hipMemcpyAsync(sl.host, d_status, ST_WORDS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
                TS_HIP(hipEventRecord(sl.ev, st));
                sl.busy = true;
                sl.owner = m;
                m->pending_slot = slot;
                m->rows_done = false;
                TS_HIP(hipGetLastError());
                return TS_OK;
            }
        }
        TS_LAUNCH("k_rows", (k_rows<27, true>), dim3(blocks_for(n_out, kThreads)), dim3(kThreads), m->d_nbr, m->d_out_keys, n_out,
                  m->d_colbits, colcnt, wavemask, m->n_blocks);
    }
    else if (mode == MODE_FWD && K == 1) launch_probe<MODE_FWD, 1>(m, table, colcnt, wavemask);
    else if (mode == MODE_TR && K == 1) launch_probe<MODE_TR, 1>(m, table, colcnt, wavemask);
    else if (mode == MODE_FWD && K == 2) launch_probe<MODE_FWD, 2>(m, table, colcnt, wavemask);
    else if (mode == MODE_FWD && K == 3) launch_probe<MODE_FWD, 3>(m, table, colcnt, wavemask);
    else if (mode == MODE_TR && K == 2) launch_probe<MODE_TR, 2>(m, table, colcnt, wavemask);
    else if (mode == MODE_TR && K == 3) launch_probe<MODE_TR, 3>(m, table, colcnt, wavemask);
    else return fail(TS_ERR_UNSUPPORTED, "no map search for kernel_size %d, stride %d", K, m->s);
    if (!(mode == MODE_SUB && K == 3)) after_search();

    TS_LAUNCH("k_scan", k_scan, dim3(K3 + 1), dim3(kScanThreads), colcnt, m->d_colbase, m->n_blocks, d_status, K3, wavemask,
              m->n_tiles, m->d_tile_order);
    return deliver_status(m, d_status, wait);
}

// The one host round trip at the end of a build: error flags and map sizes.  A caller that does not wait
// gets them when it first asks (ts::resolve); the copy lands in a pinned slot of its own meanwhile.
int deliver_status(ts_kmap *m, int *d_status, bool wait) {
    hipStream_t st = stream();
    const int slot = wait ? -1 : slot_acquire();
    if (slot >= 0) {
        StatusSlot &sl = g_slots[slot];
        TS_HIP(hipMemcpyAsync(sl.host, d_status, ST_WORDS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        TS_HIP(hipEventRecord(sl.ev, st));
        sl.busy = true;
        sl.owner = m;
        m->pending_slot = slot;
    } else {
        int32_t *h = static_cast<int32_t *>(host_staging(ST_WORDS * sizeof(int32_t)));
        if (!h) return last_fail_code();
        TS_HIP(hipMemcpyAsync(h, d_status, ST_WORDS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        TS_HIP(hipStreamSynchronize(st));
        if (take_status(m, h) != TS_OK) return report(m);
    }

    TS_HIP(hipGetLastError());
    // temporaries go back to the pool when the caller's Temps dies; later work on the same
    // stream is ordered after the kernels above, so reuse is safe without another wait
    return TS_OK;
}

// Orders the output rows by offset bitmask (see the head of this file).
int sort_rows(ts_kmap *m) {
    hipStream_t st = stream();
    Temps tmp;
    const int K3 = m->K3;
    const int64_t n_out = m->n_out;
    int *d_status;
    int2 *slot_rank, *dense;
    int32_t *partial, *perm;
    MaskHash mh;
    FillArgs fill;
    const int64_t n_tiles = (n_out + kTileRows - 1) / kTileRows;
    TS_TRY(tmp.get(&d_status, ST_WORDS));
    TS_TRY(tmp.get(&slot_rank, (size_t)n_out));
    TS_TRY(alloc_n(&perm, (size_t)n_tiles * kTileRows));
    fill.add(d_status, ST_WORDS * sizeof(int), 0u);
    fill.add(perm, (size_t)n_tiles * kTileRows * sizeof(int32_t), 0xFFFFFFFFu);
    int rc = make_mask_hash(tmp, &mh, &fill);
    if (rc == TS_OK) rc = tmp.get(&dense, (size_t)mh.dmax + kDensePad);
    if (rc == TS_OK) rc = tmp.get(&partial, (size_t)kRankSlices * mh.dmax);
    int32_t *h = static_cast<int32_t *>(host_staging(ST_WORDS * sizeof(int32_t)));
    if (rc == TS_OK && !h) rc = TS_ERR_OOM;
    if (rc != TS_OK) {
        dev_free(perm);
        return rc;
    }
    auto body = [&]() -> int {
        TS_TRY(launch_fill(fill));
        const dim3 grid(blocks_for(n_out, kThreads)), block(kThreads);
        TS_LAUNCH("k_register", k_register, grid, block, m->d_nbr, n_out, m->stride, K3, d_status, mh, slot_rank);
        TS_LAUNCH("k_dense", k_dense, dim3(blocks_for(mh.dmax + kDensePad, kThreads)), block, d_status, mh, K3, dense);
        {
            const unsigned rank_blocks = (unsigned)(mh.dmax / (kThreads * kRankPer)) * kRankSlices;
            ProfScope ps("k_rank");
            hipLaunchKernelGGL(k_rank_partial, dim3(rank_blocks), block, 0, st, dense, d_status, mh.dmax, partial);
            hipLaunchKernelGGL(k_rank_sum, dim3(mh.dmax / kThreads), block, 0, st, partial, d_status, mh);
        }
        TS_LAUNCH("k_place", k_place, grid, block, slot_rank, n_out, mh, perm);
        TS_HIP(hipMemcpyAsync(h, d_status, ST_WORDS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        TS_HIP(hipStreamSynchronize(st));
        if (h[ST_OVERFLOW]) {
            // more distinct bitmasks than the table ranks: order the rows with a radix sort instead
            uint32_t *keys, *keys_sorted;
            int32_t *rows;
            TS_TRY(tmp.get(&keys, (size_t)n_out));
            TS_TRY(tmp.get(&keys_sorted, (size_t)n_out));
            TS_TRY(tmp.get(&rows, (size_t)n_out));
            TS_LAUNCH("k_extract_masks", k_extract_masks, grid, block, m->d_nbr, n_out, m->stride, K3, keys, rows);
            size_t bytes = 0;
            TS_HIP(rocprim::radix_sort_pairs(nullptr, bytes, keys, keys_sorted, rows, perm, (size_t)n_out, 0, K3, st));
            void *ws;
            TS_TRY(tmp.get((char **)&ws, bytes));
            ProfScope ps("sort_masks");
            TS_HIP(rocprim::radix_sort_pairs(ws, bytes, keys, keys_sorted, rows, perm, (size_t)n_out, 0, K3, st));
        }
        TS_HIP(hipGetLastError());
        return TS_OK;
    };
    rc = body();
    if (rc != TS_OK) {
        (void)hipStreamSynchronize(st);
        dev_free(perm);
        return rc;
    }
    m->d_perm = perm;
    return TS_OK;
}

// Allocations of the map that depend on n_out only.
int alloc_outputs(ts_kmap *m, FillArgs *fill, bool rows_cleared_later = false) {
    const int K3 = m->K3;
    m->stride = nbr_stride(K3);
    m->n_blocks = (m->n_out + 63) / 64;
    m->n_tiles = (m->n_out + kTileRows - 1) / kTileRows;
    if (!m->d_nbr) TS_TRY(alloc_n(&m->d_nbr, (size_t)m->n_out * m->stride));   // (a build may have made it early, for a bound on n_out)
    TS_TRY(alloc_n(&m->d_colbits, (size_t)K3 * m->n_blocks));
    TS_TRY(alloc_n(&m->d_colbase, (size_t)K3 * m->n_blocks));
    TS_TRY(alloc_n(&m->d_tile_order, (size_t)m->n_tiles));
    if (!m->d_sched) {
        TS_TRY(alloc_n(&m->d_sched, (size_t)kMaxSchedSlices * kSchedWords));
        fill->add(m->d_sched, (size_t)kMaxSchedSlices * kSchedWords * sizeof(int32_t), 0u);
    }
    if (m->s == 1 && K3 == 27 && !rows_cleared_later) fill->add(m->d_nbr, (size_t)m->n_out * m->stride * sizeof(int32_t), 0xFFFFFFFFu);   // the symmetric probe writes hits only
    return TS_OK;
}

int rows_and_scan(ts_kmap *m, Temps &tmp, int32_t *colcnt, int *d_status);   // defined below the build

int build(const int32_t *coords, int64_t N, int K, int s, int transposed, ts_kmap *m, const BuildOpts &asked) {
    BuildOpts opt = asked;   // a build that measures its bounding box may turn the grid on
    const bool wait = opt.wait;
    hipStream_t st = stream();
    Temps tmp;
    const int K3 = K * K * K;
    m->K = K;
    m->s = s;
    m->transposed = transposed;
    m->K3 = K3;
    m->stride = nbr_stride(K3);
    m->centre = (s == 1) ? (K3 - 1) / 2 : -1;
    if (N == 0) return TS_OK;

    int *d_status;
    TS_TRY(tmp.get(&d_status, ST_WORDS));
    FillArgs fill;
    fill.add(d_status, ST_WORDS * sizeof(int), 0u);

    uint64_t *given;   // keys of the caller's coordinates
    TS_TRY(alloc_n(&given, (size_t)N));
    m->d_in_keys = given;   // provisional owner, so that an early error frees it

    Searched table;
    const dim3 per_point(blocks_for(N, kThreads)), block(kThreads);
    int early_slot = -1;
    if (s == 1) {
        m->n_in = m->n_out = N;
        m->d_out_keys = given;
        if (!wait && K == 3) {
            // Nobody waits for this build: its error flags go straight into pinned host words (plain
            // stores, raised on bad input only), which saves the copy at the end of the build.
            const int slot = slot_acquire();
            if (slot >= 0 && g_slots[slot].dev) {
                std::memset(g_slots[slot].host, 0, ST_WORDS * sizeof(int32_t));
                d_status = g_slots[slot].dev;
                early_slot = slot;
            }
        }
        const bool rows_here = K == 3;   // the insertion kernel clears the neighbour rows of a 3x3x3 map
        TS_TRY(alloc_outputs(m, &fill, rows_here));
        TS_TRY(make_searched(tmp, opt, N, opt.box.lo, opt.box.hi, &table, &fill));
        TS_TRY(launch_fill(fill));
        int4 *rows = rows_here ? reinterpret_cast<int4 *>(m->d_nbr) : nullptr;
        if (table.grid)
            TS_LAUNCH("k_pack_insert_grid", k_pack_insert<Grid>, per_point, block, reinterpret_cast<const int4 *>(coords), N, given, table.g, d_status, opt.box, rows);
        else
            TS_LAUNCH("k_pack_insert", k_pack_insert<Table>, per_point, block, reinterpret_cast<const int4 *>(coords), N, given, table.t, d_status, opt.box, rows);
    } else {
        // coarse set: the distinct admissible candidates in ascending order (Alg. 3)
        const int A = (K + s - 1) / s, slots = A * A * A;
        const size_t n_cand = (size_t)N * slots;
        uint64_t *uniq;
        int64_t *d_count;
        TS_TRY(tmp.get(&uniq, n_cand));
        TS_TRY(tmp.get(&d_count, 1));
        int32_t *d_bbox = nullptr;
        if (opt.measure && !opt.grid) {
            TS_TRY(tmp.get(&d_bbox, (size_t)kBoxSlots * kBoxSlotWords));
            fill.add(d_bbox, (size_t)kBoxSlots * kBoxSlotWords * sizeof(int32_t), 0x80000000u);
        }
        // Box known before the first launch, one candidate per input (K <= s), forward map: there are at most N
        // outputs, so the neighbour table is made for N rows now and everything that must start at a known
        // value - status words, bitmap, table rows, tile counters - is cleared by the one launch below.
        const bool early = opt.grid && slots == 1 && !transposed && !opt.bound.on;
        Grid cbox = {};
        uint64_t *words = nullptr;
        int32_t *word_base = nullptr, *block_total = nullptr;
        int64_t n_words = 0, n_wblocks = 0;
        auto bitmap_over_box = [&]() -> int {
            // the coarse points lie in the box of the fine ones, moved by less than K and divided by s
            uint64_t cells = (uint64_t)opt.box.batches;
            for (int a = 0; a < 3; ++a) {
                cbox.lo[a] = floor_div(opt.box.lo[a] - K, s);
                cbox.ext[a] = (uint32_t)(floor_div(opt.box.hi[a] + K, s) - cbox.lo[a] + 1);
                cells *= cbox.ext[a];
                if (cells > kMaxGridCells)
                    return fail(TS_ERR_UNSUPPORTED, "the grid bounds span more than %llu cells", (unsigned long long)kMaxGridCells);
            }
            cbox.batches = (uint32_t)opt.box.batches;
            n_words = (int64_t)((cells + 63) / 64);
            n_wblocks = (n_words + kThreads - 1) / kThreads;
            TS_TRY(tmp.get(&words, (size_t)n_words));
            TS_TRY(tmp.get(&word_base, (size_t)n_words));
            TS_TRY(tmp.get(&block_total, (size_t)n_wblocks));
            fill.add(words, (size_t)n_words * sizeof(uint64_t), 0u);
            return TS_OK;
        };
        if (early) {
            TS_TRY(bitmap_over_box());
            m->stride = nbr_stride(K3);
            TS_TRY(alloc_n(&m->d_nbr, (size_t)N * m->stride));
            TS_TRY(alloc_n(&m->d_sched, (size_t)kMaxSchedSlices * kSchedWords));
            fill.add(m->d_nbr, (size_t)N * m->stride * sizeof(int32_t), 0xFFFFFFFFu);
            fill.add(m->d_sched, (size_t)kMaxSchedSlices * kSchedWords * sizeof(int32_t), 0u);
        }
        TS_TRY(launch_fill(fill));
        fill = FillArgs();
        TS_LAUNCH("k_pack", k_pack, per_point, block, reinterpret_cast<const int4 *>(coords), N, given, d_status, opt.box, d_bbox);
        if (d_bbox) {
            // one more host round trip buys a build without a sort and a search without collisions
            const size_t bytes = (size_t)kBoxSlots * kBoxSlotWords * sizeof(int32_t);
            int32_t *hb = static_cast<int32_t *>(host_staging(bytes));
            if (!hb) return last_fail_code();
            TS_HIP(hipMemcpyAsync(hb, d_bbox, bytes, hipMemcpyDeviceToHost, st));
            TS_HIP(hipStreamSynchronize(st));
            int32_t top[7];
            for (int q = 0; q < 7; ++q) {
                top[q] = INT32_MIN;
                for (int sl = 0; sl < kBoxSlots; ++sl) top[q] = hb[sl * kBoxSlotWords + q] > top[q] ? hb[sl * kBoxSlotWords + q] : top[q];
            }
            if (top[6] != INT32_MIN) {   // at least one valid point
                // the bitmap has one bit per cell of the box the outputs can lie in
                Box bx = {};
                uint64_t cells = (uint64_t)top[6] + 1;
                for (int a = 0; a < 3; ++a) {
                    bx.lo[a] = -top[a];
                    bx.hi[a] = top[3 + a];
                    cells *= (uint64_t)((int64_t)floor_div(bx.hi[a] + K, s) - floor_div(bx.lo[a] - K, s) + 1);
                    if (cells > kAutoGridCells) cells = kAutoGridCells + 1;
                }
                bx.batches = top[6] + 1;
                if (cells <= kAutoGridCells) {
                    opt.grid = true;
                    opt.box = bx;   // on stays 0: nothing to check, the box is the points' own
                }
            }
        }
        // the coarse points lie in the box of the fine ones, moved by less than K and divided by s
        int32_t clo[3] = {0, 0, 0}, chi[3] = {0, 0, 0};
        for (int a = 0; a < 3; ++a) {
            clo[a] = floor_div(opt.box.lo[a] - K, s);
            chi[a] = floor_div(opt.box.hi[a] + K, s);
        }
        const bool ranked = opt.grid;   // outputs found through the bitmap: the map follows without a search
        if (opt.grid) {
            // bounds are stated or measured: mark the candidates' cells in a bitmap and read the set bits
            // off in order, which sorts and removes duplicates at once
            if (!early) {
                TS_TRY(bitmap_over_box());
                TS_TRY(launch_fill(fill));
                fill = FillArgs();
            }
            TS_LAUNCH("k_candidates_mark", k_candidates_mark, dim3(blocks_for(N, kThreads), slots), block, given, N, K, s, A, opt.bound,
                      cbox, reinterpret_cast<uint32_t *>(words), d_status);
            TS_LAUNCH("k_bits_count", k_bits_count, dim3((unsigned)n_wblocks), block, words, n_words, block_total);
            // up to a few thousand blocks every block sums the totals before it by itself; beyond, a scan launch
            const int self_scan = n_wblocks <= 8192;
            if (!self_scan) TS_LAUNCH("k_bits_scan", k_bits_scan, dim3(1), block, block_total, n_wblocks, d_count);
            TS_LAUNCH("k_bits_expand", k_bits_expand, dim3((unsigned)n_wblocks), block, words, n_words, block_total, cbox, uniq,
                      word_base, self_scan, d_count);
        } else {
            // candidates -> sort -> unique (the empty key, if present, sorts last)
            uint64_t *cand, *sorted;
            TS_TRY(tmp.get(&cand, n_cand));
            TS_TRY(tmp.get(&sorted, n_cand));
            TS_LAUNCH("k_candidates", k_candidates, dim3(blocks_for(N, kThreads), slots), block, given, N, K, s, A, opt.bound, cand);
            TS_TRY(sort_keys(tmp, cand, sorted, n_cand));
            size_t bytes = 0;
            TS_HIP(rocprim::unique(nullptr, bytes, sorted, uniq, d_count, n_cand, rocprim::equal_to<uint64_t>(), st));
            void *ws;
            TS_TRY(tmp.get((char **)&ws, bytes));
            {
                ProfScope ps("unique_keys");
                TS_HIP(rocprim::unique(ws, bytes, sorted, uniq, d_count, n_cand, rocprim::equal_to<uint64_t>(), st));
            }
            // the empty key, if any candidate was rejected, is the last unique value: do not count it
            TS_LAUNCH("k_drop_empty_key", k_drop_empty_key, dim3(1), dim3(1), uniq, d_count);
        }
        int64_t *h = static_cast<int64_t *>(host_staging(64));
        if (!h) return last_fail_code();
        TS_HIP(hipMemcpyAsync(h, d_count, sizeof(int64_t), hipMemcpyDeviceToHost, st));
        TS_HIP(hipStreamSynchronize(st));
        const int64_t n_coarse = h[0];
        if (n_coarse == 0) {
            // No candidate passed the modular check (or every coordinate was out of range): a map
            // without pairs.  The inputs are still checked for duplicates and range.
            Table t0;
            int32_t *colcnt = nullptr;
            TS_TRY(make_table(tmp, N, &t0, &fill));
            if (!transposed) {
                m->n_in = N;
                m->n_out = 0;
            } else {
                m->n_in = 0;
                m->n_out = N;
                m->d_in_keys = nullptr;
                m->d_out_keys = given;
                TS_TRY(alloc_outputs(m, &fill));
                fill.add(m->d_nbr, (size_t)N * m->stride * sizeof(int32_t), 0xFFFFFFFFu);
                TS_TRY(tmp.get(&colcnt, (size_t)K3 * m->n_blocks));
            }
            TS_TRY(launch_fill(fill));
            TS_LAUNCH("k_insert", k_insert<Table>, per_point, block, given, N, t0, d_status);
            if (transposed) TS_TRY(rows_and_scan(m, tmp, colcnt, d_status));
            int32_t *hs = static_cast<int32_t *>(host_staging(ST_WORDS * sizeof(int32_t)));
            if (!hs) return last_fail_code();
            TS_HIP(hipMemcpyAsync(hs, d_status, ST_WORDS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
            TS_HIP(hipStreamSynchronize(st));
            if (hs[ST_RANGE]) m->error = TS_ERR_COORD_RANGE;
            else if (hs[ST_DUP]) m->error = TS_ERR_DUPLICATE_COORD;
            return report(m);
        }
        uint64_t *coarse;
        TS_TRY(alloc_n(&coarse, (size_t)n_coarse));
        TS_HIP(hipMemcpyAsync(coarse, uniq, (size_t)n_coarse * sizeof(uint64_t), hipMemcpyDeviceToDevice, st));
        if (ranked) {
            // No search: an input's admissible candidates are outputs, and an output's row number is the rank
            // of its cell among the marked ones (k_rank_scatter).  Neither hash table nor coordinate grid.
            const dim3 per_cand(blocks_for(N, kThreads), slots);
            int32_t *colcnt;
            if (!transposed) {
                m->n_in = N;
                m->n_out = n_coarse;
                m->d_out_keys = coarse;
            } else {
                m->n_in = n_coarse;
                m->n_out = N;
                m->d_in_keys = coarse;
                m->d_out_keys = given;
            }
            TS_TRY(alloc_outputs(m, &fill));
            if (!early) fill.add(m->d_nbr, (size_t)m->n_out * m->stride * sizeof(int32_t), 0xFFFFFFFFu);   // (early: cleared by the first launch)
            TS_TRY(tmp.get(&colcnt, (size_t)K3 * m->n_blocks));
            if (!transposed && !opt.bound.on) {
                TS_TRY(launch_fill(fill));
                TS_LAUNCH("k_rank_scatter", k_rank_scatter<false>, per_cand, block, given, N, K, s, A, opt.bound, cbox, words, word_base,
                          m->d_nbr, m->stride, d_status);
            } else if (!transposed) {
                // with a boundary an input may lose all its candidates and then meets nobody in the table: equal
                // points are found through a hash table here as well
                Table fine_table;
                TS_TRY(make_table(tmp, N, &fine_table, &fill));
                TS_TRY(launch_fill(fill));
                TS_LAUNCH("k_insert", k_insert<Table>, per_point, block, given, N, fine_table, d_status);
                TS_LAUNCH("k_rank_scatter", k_rank_scatter<false>, per_cand, block, given, N, K, s, A, opt.bound, cbox, words, word_base,
                          m->d_nbr, m->stride, d_status);
            } else {
                // rows belong to the given points here, so equal points do not meet in an entry: they are found
                // by inserting the points into a hash table, which nothing else uses
                Table fine_table;
                TS_TRY(make_table(tmp, N, &fine_table, &fill));
                TS_TRY(launch_fill(fill));
                TS_LAUNCH("k_insert", k_insert<Table>, per_point, block, given, N, fine_table, d_status);
                TS_LAUNCH("k_rank_scatter", k_rank_scatter<true>, per_cand, block, given, N, K, s, A, opt.bound, cbox, words, word_base,
                          m->d_nbr, m->stride, d_status);
            }
            // where the next level's points can lie, for a caller that builds a pyramid
            if (!transposed) {
                m->out_box_batches = (int32_t)cbox.batches;
                for (int a = 0; a < 3; ++a) {
                    m->out_box_lo[a] = cbox.lo[a];
                    m->out_box_hi[a] = cbox.lo[a] + (int32_t)cbox.ext[a] - 1;
                }
            }
            TS_TRY(rows_and_scan(m, tmp, colcnt, d_status));
            return deliver_status(m, d_status, wait);
        }
        if (!transposed) {
            m->n_in = N;
            m->n_out = n_coarse;
            m->d_out_keys = coarse;
            TS_TRY(alloc_outputs(m, &fill));
            TS_TRY(make_searched(tmp, opt, N, opt.box.lo, opt.box.hi, &table, &fill));
            TS_TRY(launch_fill(fill));
            if (table.grid) TS_LAUNCH("k_insert_grid", k_insert<Grid>, per_point, block, given, N, table.g, d_status);
            else TS_LAUNCH("k_insert", k_insert<Table>, per_point, block, given, N, table.t, d_status);
        } else {
            m->n_in = n_coarse;
            m->n_out = N;
            m->d_in_keys = coarse;
            m->d_out_keys = given;
            TS_TRY(alloc_outputs(m, &fill));
            // duplicates among the fine points are found by inserting them as well
            Table fine_table;
            TS_TRY(make_table(tmp, N, &fine_table, &fill));
            TS_TRY(make_searched(tmp, opt, n_coarse, clo, chi, &table, &fill));
            TS_TRY(launch_fill(fill));
            TS_LAUNCH("k_insert", k_insert<Table>, per_point, block, given, N, fine_table, d_status);
            const dim3 per_coarse(blocks_for(n_coarse, kThreads));
            if (table.grid) TS_LAUNCH("k_insert_grid", k_insert<Grid>, per_coarse, block, coarse, n_coarse, table.g, d_status);
            else TS_LAUNCH("k_insert", k_insert<Table>, per_coarse, block, coarse, n_coarse, table.t, d_status);
        }
    }
    TS_HIP(hipGetLastError());
    return search_and_finish(m, tmp, table, d_status, wait, early_slot);
}

}  // namespace

namespace {

// Row pass (bitmasks, presence bitmaps) and scan over a neighbour table that is already filled in.
int rows_and_scan(ts_kmap *m, Temps &tmp, int32_t *colcnt, int *d_status) {
    uint32_t *wavemask;
    TS_TRY(tmp.get(&wavemask, (size_t)m->n_blocks));
    const dim3 grid(blocks_for(m->n_out, kThreads)), block(kThreads);
    if (m->K3 == 27) TS_LAUNCH("k_rows", (k_rows<27, false>), grid, block, m->d_nbr, m->d_out_keys, m->n_out, m->d_colbits, colcnt, wavemask, m->n_blocks);
    else if (m->K3 == 8) TS_LAUNCH("k_rows", (k_rows<8, false>), grid, block, m->d_nbr, m->d_out_keys, m->n_out, m->d_colbits, colcnt, wavemask, m->n_blocks);
    else TS_LAUNCH("k_rows", (k_rows<1, false>), grid, block, m->d_nbr, m->d_out_keys, m->n_out, m->d_colbits, colcnt, wavemask, m->n_blocks);
    TS_LAUNCH("k_scan", k_scan, dim3(m->K3 + 1), dim3(kScanThreads), colcnt, m->d_colbase, m->n_blocks, d_status, m->K3, wavemask,
              m->n_tiles, m->d_tile_order);
    TS_HIP(hipGetLastError());
    return TS_OK;
}

// The transposed map of a forward strided map, derived from its neighbour table: no search, and no
// host round trip either, because the sizes are those of the forward map.
int transpose(const ts_kmap *f, ts_kmap *m) {
    hipStream_t st = stream();
    Temps tmp;
    const int K3 = f->K3;
    m->K = f->K;
    m->s = f->s;
    m->transposed = 1;
    m->K3 = K3;
    m->centre = -1;
    m->n_in = f->n_out;
    m->n_out = f->n_in;
    m->M = f->M;
    for (int n = 0; n < K3; ++n) m->sizes[n] = f->sizes[n];
    for (int n = 0; n <= K3; ++n) m->offs[n] = f->offs[n];
    if (m->n_out == 0) return TS_OK;
    TS_TRY(alloc_n(&m->d_in_keys, (size_t)m->n_in));
    TS_TRY(alloc_n(&m->d_out_keys, (size_t)m->n_out));
    if (m->n_in > 0) TS_HIP(hipMemcpyAsync(m->d_in_keys, f->d_out_keys, (size_t)m->n_in * sizeof(uint64_t), hipMemcpyDeviceToDevice, st));
    TS_HIP(hipMemcpyAsync(m->d_out_keys, f->d_in_keys, (size_t)m->n_out * sizeof(uint64_t), hipMemcpyDeviceToDevice, st));
    FillArgs fill;
    int *d_status;
    int32_t *colcnt;
    TS_TRY(tmp.get(&d_status, ST_WORDS));
    fill.add(d_status, ST_WORDS * sizeof(int), 0u);
    TS_TRY(alloc_outputs(m, &fill));
    fill.add(m->d_nbr, (size_t)m->n_out * m->stride * sizeof(int32_t), 0xFFFFFFFFu);
    TS_TRY(tmp.get(&colcnt, (size_t)K3 * m->n_blocks));
    TS_TRY(launch_fill(fill));
    if (f->n_out > 0) {
        const dim3 gf(blocks_for(f->n_out, kThreads)), block(kThreads);
        if (K3 == 27) TS_LAUNCH("k_transpose", k_transpose<27>, gf, block, f->d_nbr, f->n_out, m->d_nbr);
        else if (K3 == 8) TS_LAUNCH("k_transpose", k_transpose<8>, gf, block, f->d_nbr, f->n_out, m->d_nbr);
        else TS_LAUNCH("k_transpose", k_transpose<1>, gf, block, f->d_nbr, f->n_out, m->d_nbr);
    }
    return rows_and_scan(m, tmp, colcnt, d_status);
}

}  // namespace

namespace ts {

int resolve(const ts_kmap *kmap, bool need_sizes) {
    ts_kmap *m = const_cast<ts_kmap *>(kmap);
    if (m->pending_slot >= 0) {
        StatusSlot &sl = g_slots[m->pending_slot];
        TS_HIP(hipEventSynchronize(sl.ev));
        take_status(m, sl.host);
        sl.busy = false;
        sl.owner = nullptr;
        m->pending_slot = -1;
        if (m->rows_enqueued) {   // ts_kmap_prepare ran the row pass and the scan behind the build; their sizes came with the flags
            m->rows_enqueued = false;
            m->rows_done = true;
        }
    }
    if (need_sizes && !m->rows_done && m->error == TS_OK) {
        // the part of a stride-1 build that was put off: row pass, scan, sizes
        hipStream_t st = stream();
        Temps tmp;
        int *d_status;
        int32_t *colcnt;
        uint32_t *wavemask;
        TS_TRY(tmp.get(&d_status, ST_WORDS));
        TS_TRY(tmp.get(&colcnt, (size_t)m->K3 * m->n_blocks));
        TS_TRY(tmp.get(&wavemask, (size_t)m->n_blocks));
        FillArgs fill;
        fill.add(d_status, ST_WORDS * sizeof(int), 0u);
        TS_TRY(launch_fill(fill));
        TS_LAUNCH("k_rows", (k_rows<27, true>), dim3(blocks_for(m->n_out, kThreads)), dim3(kThreads), m->d_nbr, m->d_out_keys,
                  m->n_out, m->d_colbits, colcnt, wavemask, m->n_blocks);
        TS_LAUNCH("k_scan", k_scan, dim3(m->K3 + 1), dim3(kScanThreads), colcnt, m->d_colbase, m->n_blocks, d_status, m->K3, wavemask,
                  m->n_tiles, m->d_tile_order);
        int32_t *h = static_cast<int32_t *>(host_staging(ST_WORDS * sizeof(int32_t)));
        if (!h) return last_fail_code();
        TS_HIP(hipMemcpyAsync(h, d_status, ST_WORDS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        TS_HIP(hipStreamSynchronize(st));
        take_status(m, h);
        m->rows_done = true;
    }
    return m->error == TS_OK ? TS_OK : report(m);
}

void release_grid() {
    if (g_grid) (void)hipFree(g_grid);
    g_grid = nullptr;
    g_grid_cells = 0;
    g_grid_dirty = false;
}

// The part of a 3x3x3 stride-1 build that ts_build_kmap_async put off, enqueued without a wait: its
// sizes land in the pinned words the build's flags went to, and the event is recorded again behind it.
int prepare(const ts_kmap *kmap) {
    ts_kmap *m = const_cast<ts_kmap *>(kmap);
    if (m->rows_done || m->rows_enqueued || m->pending_slot < 0) return TS_OK;   // nothing put off, or resolve will do it
    StatusSlot &sl = g_slots[m->pending_slot];
    if (!sl.dev) return TS_OK;
    Temps tmp;
    int32_t *colcnt;
    uint32_t *wavemask;
    TS_TRY(tmp.get(&colcnt, (size_t)m->K3 * m->n_blocks));
    TS_TRY(tmp.get(&wavemask, (size_t)m->n_blocks));
    TS_LAUNCH("k_rows", (k_rows<27, true>), dim3(blocks_for(m->n_out, kThreads)), dim3(kThreads), m->d_nbr, m->d_out_keys,
              m->n_out, m->d_colbits, colcnt, wavemask, m->n_blocks);
    TS_LAUNCH("k_scan", k_scan, dim3(m->K3 + 1), dim3(kScanThreads), colcnt, m->d_colbase, m->n_blocks, sl.dev, m->K3, wavemask,
              m->n_tiles, m->d_tile_order);
    TS_HIP(hipEventRecord(sl.ev, stream()));
    TS_HIP(hipGetLastError());
    m->rows_enqueued = true;
    return TS_OK;
}

Offs offs_of(const ts_kmap *kmap) {
    Offs o;
    for (int n = 0; n <= kMaxK3; ++n) o.v[n] = n <= kmap->K3 ? (int32_t)kmap->offs[n] : (int32_t)kmap->offs[kmap->K3];
    return o;
}

// The offset-major pair lists are derived from the out-major table when something first asks for
// them (ts_kmap_pairs, the gather of the explicit dataflow); the fused kernel never does.
int ensure_pairs(const ts_kmap *kmap) {
    ts_kmap *m = const_cast<ts_kmap *>(kmap);
    TS_TRY(resolve(m));
    if (m->d_in_idx || m->M == 0) return TS_OK;
    int32_t *in_idx, *out_idx;
    TS_TRY(alloc_n(&in_idx, (size_t)m->M));
    if (alloc_n(&out_idx, (size_t)m->M) != TS_OK) {
        dev_free(in_idx);
        return TS_ERR_OOM;
    }
    const dim3 grid(blocks_for(m->n_out, kThreads)), block(kThreads);
    if (m->K3 == 27) TS_LAUNCH("k_compact", k_compact<27>, grid, block, m->d_nbr, m->n_out, m->d_colbase, m->n_blocks, offs_of(m), in_idx, out_idx);
    else if (m->K3 == 8) TS_LAUNCH("k_compact", k_compact<8>, grid, block, m->d_nbr, m->n_out, m->d_colbase, m->n_blocks, offs_of(m), in_idx, out_idx);
    else TS_LAUNCH("k_compact", k_compact<1>, grid, block, m->d_nbr, m->n_out, m->d_colbase, m->n_blocks, offs_of(m), in_idx, out_idx);
    m->d_in_idx = in_idx;
    m->d_out_idx = out_idx;
    TS_HIP(hipGetLastError());
    return TS_OK;
}

}  // namespace ts

extern "C" {

static int build_checked(const int32_t *coords, int64_t N, int kernel_size, int stride, int transposed, ts_kmap **out_kmap,
                         const BuildOpts &opt) {
    if (!out_kmap) return fail(TS_ERR_INVALID_ARG, "out_kmap is NULL");
    *out_kmap = nullptr;
    if (N < 0) return fail(TS_ERR_INVALID_ARG, "N is negative");
    if (N > 0 && !coords) return fail(TS_ERR_INVALID_ARG, "coords is NULL");
    if (N > 0 && (reinterpret_cast<uintptr_t>(coords) & 15)) return fail(TS_ERR_INVALID_ARG, "coords must be 16-byte aligned");
    if (kernel_size < 1 || kernel_size > 3) return fail(TS_ERR_INVALID_ARG, "kernel_size must be 1, 2 or 3");
    if (stride < 1 || stride > 2) return fail(TS_ERR_INVALID_ARG, "stride must be 1 or 2");
    if (stride == 1 && kernel_size % 2 == 0) return fail(TS_ERR_INVALID_ARG, "stride 1 needs an odd kernel_size");
    if (transposed != 0 && transposed != 1) return fail(TS_ERR_INVALID_ARG, "transposed must be 0 or 1");
    if (transposed && stride == 1) return fail(TS_ERR_INVALID_ARG, "a transposed map needs stride > 1");
    if (N > (int64_t)((1u << 31) - 1) / (ts::kMaxK3 + 5)) return fail(TS_ERR_UNSUPPORTED, "N too large for 32-bit pair indices");
    ts_kmap *m = new (std::nothrow) ts_kmap();
    if (!m) return fail(TS_ERR_OOM, "host allocation failed");
    int rc = build(coords, N, kernel_size, stride, transposed, m, opt);
    if (rc != TS_OK) {
        (void)hipStreamSynchronize(ts::stream());
        destroy(m);
        return rc;
    }
    *out_kmap = m;
    return TS_OK;
}

int ts_build_kmap(const int32_t *coords, int64_t N, int kernel_size, int stride, int transposed,
                  ts_kmap **out_kmap) {
    BuildOpts opt;
    opt.measure = true;
    return build_checked(coords, N, kernel_size, stride, transposed, out_kmap, opt);
}

int ts_build_kmap_async(const int32_t *coords, int64_t N, int kernel_size, int stride, int transposed,
                        ts_kmap **out_kmap) {
    BuildOpts opt;
    opt.wait = false;
    opt.measure = true;
    return build_checked(coords, N, kernel_size, stride, transposed, out_kmap, opt);
}

int ts_identity_kmap(int64_t n, ts_kmap **out_kmap) {
    if (!out_kmap) return fail(TS_ERR_INVALID_ARG, "out_kmap is NULL");
    *out_kmap = nullptr;
    if (n < 0 || n > INT32_MAX) return fail(TS_ERR_INVALID_ARG, "n must be in [0, 2^31)");
    ts_kmap *m = new (std::nothrow) ts_kmap();
    if (!m) return fail(TS_ERR_OOM, "host allocation failed");
    m->K = 1;
    m->s = 1;
    m->K3 = 1;
    m->centre = 0;
    m->stride = ts::nbr_stride(1);
    m->n_in = m->n_out = m->M = n;
    m->sizes[0] = n;
    m->offs[1] = n;
    auto body = [&]() -> int {
        if (n == 0) return TS_OK;
        FillArgs fill;
        TS_TRY(alloc_outputs(m, &fill));
        TS_TRY(launch_fill(fill));
        TS_LAUNCH("k_identity_map", k_identity_map, dim3(blocks_for(n, kThreads)), dim3(kThreads), m->d_nbr, m->stride,
                  m->d_colbits, m->d_colbase, m->d_tile_order, n, m->n_blocks, m->n_tiles);
        TS_HIP(hipGetLastError());
        return TS_OK;
    };
    const int rc = body();
    if (rc != TS_OK) {
        (void)hipStreamSynchronize(ts::stream());
        destroy(m);
        return rc;
    }
    *out_kmap = m;
    return TS_OK;
}

int ts_build_kmap_ex(const int32_t *coords, int64_t N, int kernel_size, int stride, int transposed,
                     const ts_kmap_options *options, ts_kmap **out_kmap) {
    BuildOpts opt;
    opt.measure = true;
    if (out_kmap) *out_kmap = nullptr;
    if (options) {
        opt.wait = options->wait != 0;
        opt.measure = options->search == TS_SEARCH_AUTO;
        if (options->search != TS_SEARCH_HASH && options->search != TS_SEARCH_GRID && options->search != TS_SEARCH_AUTO)
            return fail(TS_ERR_INVALID_ARG, "search must be TS_SEARCH_AUTO, TS_SEARCH_HASH or TS_SEARCH_GRID");
        // TS_SEARCH_AUTO with a box stated (grid_batches > 0): a strided build takes the box instead of measuring
        // one (one host round trip less); a stride-1 build stays on the hash table and ignores it
        const bool hinted = options->search == TS_SEARCH_AUTO && options->grid_batches > 0 && stride > 1;
        if (options->search == TS_SEARCH_GRID || hinted) {
            opt.grid = true;
            opt.box.on = 1;
            opt.box.batches = options->grid_batches;
            if (options->grid_batches < 1 || options->grid_batches > TS_BATCH_MAX + 1)
                return fail(TS_ERR_INVALID_ARG, "grid_batches must be in [1, %d]", TS_BATCH_MAX + 1);
            for (int a = 0; a < 3; ++a) {
                opt.box.lo[a] = options->grid_lo[a];
                opt.box.hi[a] = options->grid_hi[a];
                if (options->grid_lo[a] > options->grid_hi[a] || options->grid_lo[a] < TS_COORD_MIN || options->grid_hi[a] > TS_COORD_MAX)
                    return fail(TS_ERR_INVALID_ARG, "grid bounds must satisfy %d <= lo <= hi <= %d", TS_COORD_MIN, TS_COORD_MAX);
            }
        }
        if (options->has_boundary && stride > 1) {
            opt.bound.on = 1;
            for (int a = 0; a < 3; ++a) {
                if (options->boundary[a] < 1 || (int64_t)options->boundary[a] * stride > (int64_t)TS_COORD_MAX + 1)
                    return fail(TS_ERR_INVALID_ARG, "boundary must be positive and stride * boundary at most %d", TS_COORD_MAX + 1);
                opt.bound.hi[a] = options->boundary[a] * stride;
            }
        }
    }
    return build_checked(coords, N, kernel_size, stride, transposed, out_kmap, opt);
}

int ts_kmap_status(const ts_kmap *kmap) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    return ts::resolve(kmap, false);   // the verdict only: what a build put off stays put off
}

int ts_kmap_prepare(const ts_kmap *kmap) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    return ts::prepare(kmap);
}

void ts_free(ts_kmap *kmap) { destroy(kmap); }

int ts_kmap_transpose(const ts_kmap *forward, ts_kmap **out_kmap) {
    if (!out_kmap) return fail(TS_ERR_INVALID_ARG, "out_kmap is NULL");
    *out_kmap = nullptr;
    if (!forward) return fail(TS_ERR_INVALID_ARG, "forward is NULL");
    if (forward->s == 1 || forward->transposed) return fail(TS_ERR_INVALID_ARG, "a forward map with stride > 1 is needed");
    TS_TRY(ts::resolve(forward));
    ts_kmap *m = new (std::nothrow) ts_kmap();
    if (!m) return fail(TS_ERR_OOM, "host allocation failed");
    int rc = transpose(forward, m);
    if (rc != TS_OK) {
        (void)hipStreamSynchronize(ts::stream());
        destroy(m);
        return rc;
    }
    *out_kmap = m;
    return TS_OK;
}

int ts_kmap_sort_rows(ts_kmap *kmap) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    TS_TRY(ts::resolve(kmap));
    if (kmap->d_perm || kmap->n_out == 0) return TS_OK;
    return sort_rows(kmap);
}

int64_t ts_kmap_num_in(const ts_kmap *kmap) { return kmap ? kmap->n_in : -1; }
int64_t ts_kmap_num_out(const ts_kmap *kmap) { return kmap ? kmap->n_out : -1; }
int64_t ts_kmap_num_pairs(const ts_kmap *kmap) { return kmap && ts::resolve(kmap) == TS_OK ? kmap->M : -1; }
int ts_kmap_kernel_volume(const ts_kmap *kmap) { return kmap ? kmap->K3 : -1; }

int ts_kmap_out_coords(const ts_kmap *kmap, int32_t *dst) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    if (kmap->n_out == 0) return TS_OK;
    if (!kmap->d_out_keys) return fail(TS_ERR_UNSUPPORTED, "a map made by ts_identity_kmap holds no coordinates");
    if (!dst || (reinterpret_cast<uintptr_t>(dst) & 15)) return fail(TS_ERR_INVALID_ARG, "dst is NULL or not 16-byte aligned");
    TS_LAUNCH("k_unpack", k_unpack, dim3(blocks_for(kmap->n_out, kThreads)), dim3(kThreads), kmap->d_out_keys, kmap->n_out, reinterpret_cast<int4 *>(dst));
    TS_HIP(hipGetLastError());
    return TS_OK;
}

int ts_kmap_out_box(const ts_kmap *kmap, int32_t *lo, int32_t *hi, int32_t *batches) {
    if (!kmap || !lo || !hi || !batches) return fail(TS_ERR_INVALID_ARG, "NULL argument");
    if (kmap->out_box_batches <= 0) return fail(TS_ERR_UNSUPPORTED, "this map's build did not bound its output coordinates");
    for (int a = 0; a < 3; ++a) {
        lo[a] = kmap->out_box_lo[a];
        hi[a] = kmap->out_box_hi[a];
    }
    *batches = kmap->out_box_batches;
    return TS_OK;
}

int ts_kmap_in_coords(const ts_kmap *kmap, int32_t *dst) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    if (kmap->n_in == 0) return TS_OK;
    if (!kmap->d_in_keys) return fail(TS_ERR_UNSUPPORTED, "a map made by ts_identity_kmap holds no coordinates");
    if (!dst || (reinterpret_cast<uintptr_t>(dst) & 15)) return fail(TS_ERR_INVALID_ARG, "dst is NULL or not 16-byte aligned");
    TS_LAUNCH("k_unpack", k_unpack, dim3(blocks_for(kmap->n_in, kThreads)), dim3(kThreads), kmap->d_in_keys, kmap->n_in, reinterpret_cast<int4 *>(dst));
    TS_HIP(hipGetLastError());
    return TS_OK;
}

int ts_kmap_sizes(const ts_kmap *kmap, int64_t *dst) {
    if (!kmap || !dst) return fail(TS_ERR_INVALID_ARG, "NULL argument");
    TS_TRY(ts::resolve(kmap));
    for (int n = 0; n < kmap->K3; ++n) dst[n] = kmap->sizes[n];
    return TS_OK;
}

int ts_kmap_pairs(const ts_kmap *kmap, int32_t *in_idx, int32_t *out_idx) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    TS_TRY(ts::resolve(kmap));
    if (kmap->M == 0) return TS_OK;
    TS_TRY(ts::ensure_pairs(kmap));
    size_t bytes = (size_t)kmap->M * sizeof(int32_t);
    if (in_idx) TS_HIP(hipMemcpyAsync(in_idx, kmap->d_in_idx, bytes, hipMemcpyDeviceToDevice, ts::stream()));
    if (out_idx) TS_HIP(hipMemcpyAsync(out_idx, kmap->d_out_idx, bytes, hipMemcpyDeviceToDevice, ts::stream()));
    return TS_OK;
}

}  // extern "C"
