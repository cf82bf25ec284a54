// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/ts.h"
#include "../../include/ts_bench.h"

namespace ts {

// ---- errors -------------------------------------------------------------------------------
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
// The code of this thread's last fail(): what a caller returns when a helper that reports through a
// null pointer (dev_alloc, scratch, zero_row, host_staging) has failed.
int last_fail_code();

#define TS_HIP(call)                                                                        \
    do {                                                                                    \
        hipError_t ts_e_ = (call);                                                          \
        if (ts_e_ != hipSuccess)                                                            \
            return ts::fail(TS_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(ts_e_));  \
    } while (0)

#define TS_TRY(expr)                  \
    do {                              \
        int ts_rc_ = (expr);          \
        if (ts_rc_ != TS_OK) return ts_rc_; \
    } while (0)

// ---- runtime ------------------------------------------------------------------------------
hipStream_t stream();

// Pooled device memory: freed blocks are kept and handed out again, so steady-state
// calls do not reach hipMalloc/hipFree.  A block is handed out again only in stream order: at once on the
// stream it was freed on, after that stream has drained on another.  Returns nullptr on failure (error
// text is set).
void *dev_alloc(size_t bytes);
void dev_free(void *p);

// Grow-only scratch areas for ts_sparse_conv; an outgrown area is kept, unused, until ts_release_cache
// (enqueued work or a captured graph may still address it), and growth fails while the stream is being
// captured (slot 0: gather buffer F, 1: partial sums G,
// 2: packed weights, 3: padded features, 4: a two-part input concatenated where the kernels cannot read the
// parts in place).  Contents do not survive across calls.
void *scratch(int slot, size_t bytes);

// 4 KiB of device zeros (a feature row of any supported width), allocated once.
const void *zero_row();

// Pinned host staging area (at least `bytes` long), one per process.
void *host_staging(size_t bytes);

// Optional per-kernel timing (ts_profile_enable): an event pair around the enclosed launches.
struct ProfScope {
    explicit ProfScope(const char *name);
    ~ProfScope();
    int rec_;
};

// The same for a single kernel launch, without the two marker packets that recorded events put into the
// stream (each costs the stream a few microseconds between kernels): the launch itself carries the event
// pair, which then holds the dispatch's own start and end time.  Both null: this launch is not timed.
struct ProfPair {
    hipEvent_t a = nullptr, b = nullptr;
};
ProfPair prof_pair(const char *name);

// Launch on the library stream, timed under the kernel's name while per-kernel timing is on.
#define TS_LAUNCH_SHM(name, kernel, grid, block, shm, ...)                                                   \
    do {                                                                                                     \
        const ts::ProfPair ts_pp_ = ts::prof_pair(name);                                                     \
        if (ts_pp_.a) hipExtLaunchKernelGGL(kernel, grid, block, shm, ts::stream(), ts_pp_.a, ts_pp_.b, 0, __VA_ARGS__); \
        else hipLaunchKernelGGL(kernel, grid, block, shm, ts::stream(), __VA_ARGS__);                        \
    } while (0)
#define TS_LAUNCH(name, kernel, grid, block, ...) TS_LAUNCH_SHM(name, kernel, grid, block, 0, __VA_ARGS__)

template <class T>
inline int alloc_n(T **p, size_t n) {
    *p = static_cast<T *>(dev_alloc((n ? n : 1) * sizeof(T)));
    return *p ? TS_OK : last_fail_code();
}

// Waits, if it has not happened yet, for the sizes and error flags of a map built with
// ts_build_kmap_async, and fills in M / sizes / offs.  Returns TS_OK or the build's error.
// need_sizes == false: only the error flags are awaited; the put-off part of a stride-1 build is not run.
int resolve(const struct ::ts_kmap *kmap, bool need_sizes = true);

// Enqueues, without waiting, what an asynchronous build put off (ts_kmap_prepare).
int prepare(const struct ::ts_kmap *kmap);

// Makes sure the offset-major pair lists of a map exist (they are derived on first use).
int ensure_pairs(const struct ::ts_kmap *kmap);

// Frees the cells of the coordinate grid (the device must be idle).
void release_grid();

// ---- 64-bit coordinate keys ----------------------------------------------------------------
// key = batch<<51 | (x+B)<<34 | (y+B)<<17 | (z+B), B = 2^16: order-preserving in (b,x,y,z)
// (the hash key of a coordinate is one integer made of its components, paper Sec. 2.1.2).
// With x,y,z in [TS_COORD_MIN, TS_COORD_MAX] a field never borrows or carries when a kernel
// offset (|d| <= 7) is added, so key(p + d) = key(p) + key_delta(d).
constexpr int kFieldBits = 17;
constexpr int64_t kBias = 1 << 16;
constexpr uint64_t kFieldMask = (1u << kFieldBits) - 1;
constexpr uint64_t kEmptyKey = ~0ull;

__host__ __device__ inline uint64_t pack_key(int32_t b, int32_t x, int32_t y, int32_t z) {
    return ((uint64_t)(uint32_t)b << (3 * kFieldBits)) | ((uint64_t)(x + kBias) << (2 * kFieldBits)) |
           ((uint64_t)(y + kBias) << kFieldBits) | (uint64_t)(z + kBias);
}
__host__ __device__ inline void unpack_key(uint64_t k, int32_t c[4]) {
    c[3] = (int32_t)(k & kFieldMask) - (int32_t)kBias;
    c[2] = (int32_t)((k >> kFieldBits) & kFieldMask) - (int32_t)kBias;
    c[1] = (int32_t)((k >> (2 * kFieldBits)) & kFieldMask) - (int32_t)kBias;
    c[0] = (int32_t)(k >> (3 * kFieldBits));
}
__host__ __device__ inline int64_t key_delta(int dx, int dy, int dz) {
    return ((int64_t)dx << (2 * kFieldBits)) + ((int64_t)dy << kFieldBits) + (int64_t)dz;
}

constexpr int kMaxK3 = 27;      // kernel volumes up to 3^3 (one bit per offset in a 32-bit mask)

// Start of every offset's pair list (exclusive prefix of the map sizes), passed to kernels by value.
struct Offs {
    int32_t v[kMaxK3 + 1];
};
constexpr int kTileRows = 128;  // output rows per workgroup tile of the fused kernel
constexpr int kMaxSchedSlices = 32;   // output-channel slices of a layer that take tiles from counters of their own
constexpr int kSchedWords = 9 * 32;   // per slice: 8 tile counters (one per XCD) and a done count, 128 bytes apart

// Row stride (in int32) of the neighbour table for a kernel volume: K3 neighbour entries, then
// the row's offset bitmask at index K3, padded to a power of two (16-byte multiples).
__host__ __device__ constexpr int nbr_stride(int K3) { return K3 > 8 ? 32 : (K3 > 1 ? 16 : 4); }

}  // namespace ts

struct ts_kmap;
namespace ts {
Offs offs_of(const ::ts_kmap *kmap);   // the map's offs[] as a kernel argument
}

// The kernel map.  Everything with a d_ prefix is device memory owned by the map.
struct ts_kmap {
    int K = 0, s = 0, transposed = 0, K3 = 0;
    int centre = -1;            // index of the identity offset (odd K, stride 1), else -1
    int stride = 0;             // nbr_stride(K3)
    int64_t n_in = 0, n_out = 0, M = 0;   // M, sizes, offs: valid once ts::resolve has run
    bool rows_enqueued = false; // the put-off row pass and scan have been enqueued (ts_kmap_prepare); resolve only waits
    bool rows_done = true;      // false: the row pass (bitmask words, centre entries, rank bitmaps, tile order) and the
                                // scan have not run yet; ts::resolve runs them (the fused kernel needs none of it)
    int pending_slot = -1;      // >= 0: sizes and error flags are still on their way to the host
    int error = 0;              // TS_OK, or what the build found wrong with its input
    int32_t out_box_lo[3] = {0, 0, 0}, out_box_hi[3] = {0, 0, 0}, out_box_batches = 0;   // a box that holds every output
                                // coordinate (a strided forward build that marked its candidates in one); batches 0: unknown
    int64_t n_blocks = 0;       // ceil(n_out / 64): 64-row blocks of the rank structure
    int64_t sizes[ts::kMaxK3] = {0};      // |M[W_n]|
    int64_t offs[ts::kMaxK3 + 1] = {0};   // exclusive prefix of sizes
    uint64_t *d_in_keys = nullptr;        // [n_in]  packed input coordinates, row order of X_in
    uint64_t *d_out_keys = nullptr;       // [n_out] packed output coordinates (may alias d_in_keys)
    // Out-major view (what Alg. 1 yields per output): row k holds, for every offset n, the input
    // row feeding output k through W_n (or -1), then the bitmask of the offsets present.
    int32_t *d_nbr = nullptr;             // [n_out][stride]
    // Offset-major view M[W_n] (Sec. 2.1): pair lists ordered by output index inside an offset,
    // derived from the out-major table on first use (ts::ensure_pairs); NULL until then ...
    int32_t *d_in_idx = nullptr;          // [M]
    int32_t *d_out_idx = nullptr;         // [M]
    // ... and the link between the two views: the pair (k, n) sits at
    // offs[n] + colbase[n][k/64] + popcount(colbits[n][k/64] & ((1 << k%64) - 1)).
    uint64_t *d_colbits = nullptr;        // [K3][n_blocks] bit r: output 64*b + r has offset n
    int32_t *d_colbase = nullptr;         // [K3][n_blocks] pairs of offset n in the blocks before b
    // Optional (ts_kmap_sort_rows): output rows ordered by offset bitmask, so that the rows of a
    // tile of the output-stationary kernel share their offsets.  NULL = natural row order.
    int64_t n_tiles = 0;                  // ceil(n_out / kTileRows)
    int32_t *d_perm = nullptr;            // [n_tiles*kTileRows] sorted position -> output row, -1 = padding
    int32_t *d_tile_order = nullptr;      // [n_tiles] tiles (of rows in input order) by descending number of offsets met
    // Tile counters of the fused kernel, per output-channel slice; all zero between launches (the
    // last workgroup of a launch rearms them).
    int32_t *d_sched = nullptr;           // [kMaxSchedSlices][kSchedWords]
};
