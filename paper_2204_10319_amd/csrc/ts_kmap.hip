// Kernel-map construction (paper Sec. 2.1: output coordinates, Alg. 3; map search, Alg. 1).
//
// Pipeline on the device, one stream:
//   pack (b,x,y,z) -> 64-bit keys                      ("flattening the coordinate", Sec. 2.1.2)
//   stride>1: candidate keys (p - delta)/s, radix sort, unique -> P_out      (Alg. 3, fused 1-4)
//   insert the searched point set into an open-addressing hash table (64-bit CAS, linear probing)
//   probe s*q_k + delta_n for every output and offset -> neighbour table nbr[n][k]   (Alg. 1)
//       odd K, stride 1: only the first half of the offsets is probed, the mirrored entry
//       (k, j, K^3-1-n) is written alongside (Sec. 4.2.1), the centre map is the identity
//   per-offset compaction (count, scan, write) -> pair lists M[W_n], ordered by output index
//   outputs sorted by neighbour bitmask -> tiles for the output-stationary fused kernel
#include "ts_internal.h"

#include <cstring>
#include <new>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_select.hpp>

using namespace ts;

namespace {

constexpr int kThreads = 256;

// status words written by the kernels and read back once per build
enum { ST_RANGE = 0, ST_DUP = 1, ST_TOTALS = 8, ST_WORDS = 8 + 32 };   // ST_TOTALS: per-offset map sizes

struct Table {
    uint64_t *keys;
    int32_t *vals;
    uint32_t mask;   // capacity - 1 (capacity is a power of two >= 2 * entries)
    int shift;       // 64 - log2(capacity)
};

__device__ __forceinline__ uint32_t hash_slot(uint64_t key, int shift) {
    return (uint32_t)((key * 0x9E3779B97F4A7C15ull) >> shift);   // multiplicative (Fibonacci) hashing
}

__device__ __forceinline__ void table_insert(const Table &t, uint64_t key, int32_t value, int *status) {
    uint32_t slot = hash_slot(key, t.shift);
    for (;;) {
        unsigned long long prev =
            atomicCAS(reinterpret_cast<unsigned long long *>(&t.keys[slot]), (unsigned long long)kEmptyKey,
                      (unsigned long long)key);
        if (prev == kEmptyKey) {
            t.vals[slot] = value;
            return;
        }
        if (prev == key) {
            atomicOr(&status[ST_DUP], 1);
            return;
        }
        slot = (slot + 1) & t.mask;   // the table is at most half full, so an empty slot exists
    }
}

__device__ __forceinline__ int32_t table_find(const Table &t, uint64_t key) {
    uint32_t slot = hash_slot(key, t.shift);
    for (;;) {
        uint64_t k = t.keys[slot];
        if (k == key) return t.vals[slot];
        if (k == kEmptyKey) return -1;
        slot = (slot + 1) & t.mask;
    }
}

__device__ __forceinline__ bool coord_ok(int4 c) {
    return c.x >= 0 && c.x <= TS_BATCH_MAX && c.y >= TS_COORD_MIN && c.y <= TS_COORD_MAX &&
           c.z >= TS_COORD_MIN && c.z <= TS_COORD_MAX && c.w >= TS_COORD_MIN && c.w <= TS_COORD_MAX;
}

__device__ __forceinline__ void offset_of(int K, int n, int &dx, int &dy, int &dz) {
    int r = (K - 1) / 2;
    dx = n / (K * K) - r;
    dy = (n / K) % K - r;
    dz = n % K - r;
}

__device__ __forceinline__ int floor_div(int a, int s) { return a >= 0 ? a / s : -((-a + s - 1) / s); }

// keys[i] = pack(coords[i]); out-of-range rows get the empty key and raise ST_RANGE.
__global__ void k_pack(const int4 *coords, int64_t n, uint64_t *keys, int *status) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int4 c = coords[i];
    if (!coord_ok(c)) {
        atomicOr(&status[ST_RANGE], 1);
        keys[i] = kEmptyKey;
        return;
    }
    keys[i] = pack_key(c.x, c.y, c.z, c.w);
}

// Insert (keys[i] -> i).  With centre_row != nullptr also writes the identity map of the
// centre offset (stride 1: output i is input i).
__global__ void k_insert(const uint64_t *keys, int64_t n, Table t, int32_t *centre_row, int *status) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t key = keys[i];
    if (key == kEmptyKey) return;
    table_insert(t, key, (int32_t)i, status);
    if (centre_row) centre_row[i] = (int32_t)i;
}

// Stride-1 front end in one pass: pack, insert (key -> i) and write the identity map of the
// centre offset (output i is input i).
__global__ void k_pack_insert(const int4 *coords, int64_t n, uint64_t *keys, Table t, int32_t *centre_row,
                              int *status) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int4 c = coords[i];
    if (!coord_ok(c)) {
        atomicOr(&status[ST_RANGE], 1);
        keys[i] = kEmptyKey;
        return;
    }
    uint64_t key = pack_key(c.x, c.y, c.z, c.w);
    keys[i] = key;
    table_insert(t, key, (int32_t)i, status);
    centre_row[i] = (int32_t)i;
}

// Stride 1, odd K: blockIdx.y = offset index n < K^3/2.  A hit (j at p_i + delta_n) gives the
// entry (j, i, n) and its mirror (i, j, K^3-1-n).
__global__ void k_probe_symmetric(const uint64_t *keys, int64_t n_pts, Table t, int K, int32_t *nbr) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pts) return;
    int n = blockIdx.y, dx, dy, dz;
    offset_of(K, n, dx, dy, dz);
    uint64_t key = keys[i];
    if (key == kEmptyKey) return;
    int32_t j = table_find(t, (uint64_t)((int64_t)key + key_delta(dx, dy, dz)));
    if (j >= 0) {
        nbr[(int64_t)n * n_pts + i] = j;
        nbr[(int64_t)(K * K * K - 1 - n) * n_pts + j] = (int32_t)i;
    }
}

// Alg. 3 stages 1-4 in registers: candidate u = p - delta_n, modular check, key of u/s.
// One thread per (input, offset); rejected candidates become the empty key (sorts last).
__global__ void k_candidates(const uint64_t *keys, int64_t n, int K, int s, uint64_t *cand) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int nn = blockIdx.y, K3 = K * K * K, dx, dy, dz;
    offset_of(K, nn, dx, dy, dz);
    uint64_t key = keys[i], out = kEmptyKey;
    if (key != kEmptyKey) {
        int32_t c[4];
        unpack_key(key, c);
        int ux = c[1] - dx, uy = c[2] - dy, uz = c[3] - dz;
        if (ux % s == 0 && uy % s == 0 && uz % s == 0) out = pack_key(c[0], ux / s, uy / s, uz / s);
    }
    cand[i * K3 + nn] = out;
}

// K = s = 2: exactly one admissible offset per input (delta = p mod 2), output floor(p/2).
__global__ void k_candidates_k2s2(const uint64_t *keys, int64_t n, uint64_t *cand) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t key = keys[i], out = kEmptyKey;
    if (key != kEmptyKey) {
        int32_t c[4];
        unpack_key(key, c);
        out = pack_key(c[0], floor_div(c[1], 2), floor_div(c[2], 2), floor_div(c[3], 2));
    }
    cand[i] = out;
}

// Alg. 1, forward strided map: thread per (output k, offset n): look up s*q_k + delta_n among the inputs.
__global__ void k_probe_forward(const uint64_t *out_keys, int64_t n_out, Table t, int K, int s, int32_t *nbr) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n_out) return;
    int n = blockIdx.y, dx, dy, dz;
    offset_of(K, n, dx, dy, dz);
    int32_t c[4];
    unpack_key(out_keys[k], c);
    nbr[(int64_t)n * n_out + k] = table_find(t, pack_key(c[0], s * c[1] + dx, s * c[2] + dy, s * c[3] + dz));
}

// Transposed map: thread per (fine point j, offset n): the coarse point (p_j - delta_n)/s, if any.
__global__ void k_probe_transposed(const uint64_t *fine_keys, int64_t n_fine, Table coarse, int K, int s,
                                   int32_t *nbr) {
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_fine) return;
    int n = blockIdx.y, dx, dy, dz;
    offset_of(K, n, dx, dy, dz);
    int32_t found = -1;
    uint64_t key = fine_keys[j];
    if (key != kEmptyKey) {
        int32_t c[4];
        unpack_key(key, c);
        int ux = c[1] - dx, uy = c[2] - dy, uz = c[3] - dz;
        if (ux % s == 0 && uy % s == 0 && uz % s == 0)
            found = table_find(coarse, pack_key(c[0], ux / s, uy / s, uz / s));
    }
    nbr[(int64_t)n * n_fine + j] = found;
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

// ---- per-offset compaction -------------------------------------------------------------------
constexpr int kItems = 1;                        // entries per thread
constexpr int kChunk = kThreads * kItems;        // entries per block

__device__ __forceinline__ int block_exclusive_scan(int v, int *total) {
    __shared__ int wave_sums[kThreads / 64];
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
    for (int d = 1; d < 64; d <<= 1) {
        int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int base = 0, all = 0;
    for (int w = 0; w < kThreads / 64; ++w) {
        int sw = wave_sums[w];
        if (w < wave) base += sw;
        all += sw;
    }
    __syncthreads();
    *total = all;
    return base + incl - v;
}

// One pass over the neighbour table: blkcnt[n][b] = number of valid entries of
// nbr[n][b*kChunk .. +kChunk), and per output its neighbour bitmask (plus the identity row list
// that the mask sort permutes).
__global__ void k_count_masks(const int32_t *nbr, int64_t n_out, int nblk, int K3, int32_t *blkcnt, uint32_t *masks,
                              int32_t *rows, int *totals) {
    __shared__ int s_cnt[kMaxK3];
    static_assert(kItems == 1, "one output per thread");
    const int b = blockIdx.x;
    if (threadIdx.x < kMaxK3) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t k = (int64_t)b * kChunk + threadIdx.x;
    const int64_t kc = k < n_out ? k : n_out - 1;
    int32_t v[kMaxK3];
#pragma unroll
    for (int n = 0; n < kMaxK3; ++n) v[n] = nbr[(int64_t)(n < K3 ? n : K3 - 1) * n_out + kc];   // all loads first
    uint32_t m = 0;
#pragma unroll
    for (int n = 0; n < kMaxK3; ++n)
        if (n < K3 && k < n_out && v[n] >= 0) m |= 1u << n;
#pragma unroll
    for (int n = 0; n < kMaxK3; ++n) {
        const int c = __popcll(__ballot((m >> n) & 1));
        if ((threadIdx.x & 63) == 0 && c) atomicAdd(&s_cnt[n], c);
    }
    if (k < n_out) {
        masks[k] = m;
        rows[k] = (int32_t)k;
    }
    __syncthreads();
    if (threadIdx.x < K3) {
        blkcnt[(int64_t)threadIdx.x * nblk + b] = s_cnt[threadIdx.x];
        if (s_cnt[threadIdx.x]) atomicAdd(&totals[threadIdx.x], s_cnt[threadIdx.x]);
    }
}

// Exclusive scan of blkcnt (offset-major) in place, one block per offset: the start of offset n
// is the sum of the totals before it.  offs[n] = start of offset n, offs[K3] = |M|.
__global__ void k_scan_counts(int32_t *blkcnt, int nblk, int K3, const int *totals, int32_t *offs) {
    const int n = blockIdx.x;
    int start = 0;
    for (int q = 0; q < n; ++q) start += totals[q];
    int32_t *row = blkcnt + (int64_t)n * nblk;
    const int per = (nblk + kThreads - 1) / kThreads;
    const int lo = threadIdx.x * per, hi = lo + per < nblk ? lo + per : nblk;
    int sum = 0;
    for (int e = lo; e < hi; ++e) sum += row[e];
    int total;
    int run = start + block_exclusive_scan(sum, &total);
    for (int e = lo; e < hi; ++e) {
        int c = row[e];
        row[e] = run;
        run += c;
    }
    if (threadIdx.x == 0) {
        offs[n] = start;
        if (n == K3 - 1) offs[K3] = start + total;
    }
}

// Write pairs and positions.  Block (b, n) owns entries [b*kChunk, +kChunk) of offset n; its
// first output slot is blkbase[n][b]; inside the block entries keep ascending output order.
__global__ void k_compact(const int32_t *nbr, int64_t n_out, int nblk, const int32_t *blkbase, int32_t *in_idx,
                          int32_t *out_idx, int32_t *pos) {
    int n = blockIdx.y, b = blockIdx.x;
    const int32_t *row = nbr + (int64_t)n * n_out;
    int64_t k0 = (int64_t)b * kChunk + (int64_t)threadIdx.x * kItems;   // thread owns kItems consecutive outputs
    int32_t j[kItems];
    int c = 0;
    for (int it = 0; it < kItems; ++it) {
        int64_t k = k0 + it;
        j[it] = k < n_out ? row[k] : -1;
        if (j[it] >= 0) ++c;
    }
    int total;
    int p = blkbase[(int64_t)n * nblk + b] + block_exclusive_scan(c, &total);
    for (int it = 0; it < kItems; ++it) {
        int64_t k = k0 + it;
        if (k >= n_out) break;
        if (j[it] >= 0) {
            in_idx[p] = j[it];
            out_idx[p] = (int32_t)k;
            pos[(int64_t)n * n_out + k] = p++;
        } else {
            pos[(int64_t)n * n_out + k] = -1;
        }
    }
}

// ---- tiles for the output-stationary kernels ---------------------------------------------------
// One block per tile of kTileRows sorted outputs: records the output row of each slot, the
// tile's offset bitmask, and per group of 32 rows the neighbour rows in rank order (rank = position among the group's present offsets)
// with a 32-byte header {count, offset of rank 0, offset of rank 1, ...}.
__global__ void __launch_bounds__(kTileRows) k_build_tiles(const int32_t *nbr, int64_t n_out, int K3,
                                                            const uint32_t *sorted_masks,
                                                            const int32_t *sorted_rows, int32_t *perm,
                                                            uint32_t *tmask, uint32_t *tmask32, int32_t *gnbr, uint32_t *ghdr, uint32_t *work,
                                                            uint32_t *work_count, int thr1, int thr2) {
    __shared__ uint32_t s_mask;
    __shared__ int s_max_count;
    int64_t tile = blockIdx.x, r = tile * kTileRows + threadIdx.x;
    if (threadIdx.x == 0) {
        s_mask = 0;
        s_max_count = 0;
    }
    __syncthreads();
    int32_t k = r < n_out ? sorted_rows[r] : -1;
    uint32_t m = r < n_out ? sorted_masks[r] : 0;
    perm[r] = k;
    for (int d = 16; d >= 1; d >>= 1) m |= __shfl_xor(m, d, 64);
    const uint32_t gm = m;                  // mask of this thread's group of 32 rows
    const int64_t group = r >> 5;
    const int lane32 = threadIdx.x & 31;
    if (lane32 == 0) {
        tmask32[group] = gm;
        atomicOr(&s_mask, gm);
        atomicMax(&s_max_count, __popc(gm));
    }
    // header: byte 0 = count, byte 1+rank = offset index; lanes 0..7 write one word each
    if (lane32 < 8) {
        uint32_t word = 0;
        int rank = 0;
        for (int n = 0; n < K3; ++n) {
            if (!((gm >> n) & 1)) continue;
            int byte = 1 + rank;
            if ((byte >> 2) == lane32) word |= (uint32_t)n << (8 * (byte & 3));
            ++rank;
        }
        if (lane32 == 0) word |= (uint32_t)rank;
        ghdr[group * 8 + lane32] = word;
    }
    __syncthreads();
    uint32_t tm = s_mask;
    if (threadIdx.x == 0) {
        tmask[tile] = tm;
        // work items of the group kernel: a tile whose largest group has many offsets is given
        // to 2 or 4 workgroups (item = tile << 4 | part << 2 | log2(parts)); list order is
        // arbitrary and does not affect results
        const int c = s_max_count;
        const int lg = c <= thr1 ? 0 : (c <= thr2 ? 1 : 2);
        const uint32_t base = atomicAdd(work_count, 1u << lg);
        for (uint32_t i = 0; i < (1u << lg); ++i) work[base + i] = ((uint32_t)tile << 4) | (i << 2) | (uint32_t)lg;
    }
    int rank = 0;
    for (int n = 0; n < K3; ++n) {
        if (!((gm >> n) & 1)) continue;
        gnbr[(group * K3 + rank) * 32 + lane32] = k >= 0 ? nbr[(int64_t)n * n_out + k] : -1;
        ++rank;
    }
}

// Largest per-group offset count handled by 1 (which = 1) or 2 (which = 2) workgroups per tile
// (measured on ~150k-voxel scans: chains of more than ~6 dependent offsets per wave dominate).
inline int split_thr(int which) { return which == 1 ? 6 : 12; }

inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

// Owns the temporaries of one build; everything goes back to the pool on scope exit.
struct Temps {
    void *p[40];
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

int make_table(Temps &tmp, int64_t entries, Table *t) {
    uint64_t cap = 1024;
    while (cap < (uint64_t)(2 * entries)) cap <<= 1;
    if (cap > (1ull << 31)) return fail(TS_ERR_UNSUPPORTED, "too many points for the hash table");
    TS_TRY(tmp.get(&t->keys, cap));
    TS_TRY(tmp.get(&t->vals, cap));
    t->mask = (uint32_t)(cap - 1);
    t->shift = 64 - __builtin_ctzll(cap);
    ProfScope ps("memset_table");
    TS_HIP(hipMemsetAsync(t->keys, 0xFF, cap * sizeof(uint64_t), stream()));
    return TS_OK;
}

void destroy(ts_kmap *m) {
    if (!m) return;
    if (m->d_out_keys != m->d_in_keys) dev_free(m->d_out_keys);
    dev_free(m->d_in_keys);
    dev_free(m->d_nbr);
    dev_free(m->d_pos);
    dev_free(m->d_in_idx);
    dev_free(m->d_out_idx);
    dev_free(m->d_offs);
    dev_free(m->d_perm);
    dev_free(m->d_tmask);
    dev_free(m->d_tmask32);
    dev_free(m->d_gnbr);
    dev_free(m->d_ghdr);
    dev_free(m->d_work);
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

// From the neighbour table to pair lists, positions and fused-kernel tiles.
int finish_map(ts_kmap *m, Temps &tmp, int *d_status) {
    hipStream_t st = stream();
    const int K3 = m->K3;
    const int64_t n_out = m->n_out;
    const int nblk = (int)blocks_for(n_out, kChunk);
    int32_t *blkcnt;
    TS_TRY(tmp.get(&blkcnt, (size_t)K3 * nblk));
    TS_TRY(alloc_n(&m->d_offs, K3 + 1));
    uint32_t *masks, *masks_sorted;
    int32_t *rows, *rows_sorted;
    TS_TRY(tmp.get(&masks, (size_t)n_out));
    TS_TRY(tmp.get(&masks_sorted, (size_t)n_out));
    TS_TRY(tmp.get(&rows, (size_t)n_out));
    TS_TRY(tmp.get(&rows_sorted, (size_t)n_out));
    TS_LAUNCH("k_count_masks", k_count_masks, dim3(nblk), dim3(kThreads), m->d_nbr, n_out, nblk, K3, blkcnt, masks, rows, d_status + ST_TOTALS);
    TS_LAUNCH("k_scan_counts", k_scan_counts, dim3(K3), dim3(kThreads), blkcnt, nblk, K3, d_status + ST_TOTALS, m->d_offs);

    // the one host round trip: status flags and the per-offset starts
    int32_t *h = static_cast<int32_t *>(host_staging((ST_WORDS + kMaxK3 + 1) * sizeof(int32_t)));
    if (!h) return TS_ERR_OOM;
    TS_HIP(hipMemcpyAsync(h, d_status, ST_WORDS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    TS_HIP(hipMemcpyAsync(h + ST_WORDS, m->d_offs, (K3 + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    TS_HIP(hipStreamSynchronize(st));
    if (h[ST_RANGE])
        return fail(TS_ERR_COORD_RANGE, "coordinate outside batch [0,%d] / xyz [%d,%d]", TS_BATCH_MAX,
                    TS_COORD_MIN, TS_COORD_MAX);
    if (h[ST_DUP]) return fail(TS_ERR_DUPLICATE_COORD, "input coordinates are not distinct");
    for (int n = 0; n <= K3; ++n) m->offs[n] = h[ST_WORDS + n];
    for (int n = 0; n < K3; ++n) m->sizes[n] = m->offs[n + 1] - m->offs[n];
    m->M = m->offs[K3];

    TS_TRY(alloc_n(&m->d_in_idx, (size_t)m->M));
    TS_TRY(alloc_n(&m->d_out_idx, (size_t)m->M));
    TS_TRY(alloc_n(&m->d_pos, (size_t)K3 * n_out));
    TS_LAUNCH("k_compact", k_compact, dim3(nblk, K3), dim3(kThreads), m->d_nbr, n_out, nblk, blkcnt, m->d_in_idx, m->d_out_idx, m->d_pos);

    // tiles: outputs ordered by neighbour bitmask so that a tile's rows share their offsets
    size_t bytes = 0;
    TS_HIP(rocprim::radix_sort_pairs(nullptr, bytes, masks, masks_sorted, rows, rows_sorted, (size_t)n_out, 0, K3,
                                     st));
    void *ws;
    TS_TRY(tmp.get((char **)&ws, bytes));
    {
        ProfScope ps("sort_masks");
        TS_HIP(rocprim::radix_sort_pairs(ws, bytes, masks, masks_sorted, rows, rows_sorted, (size_t)n_out, 0, K3, st));
    }
    m->n_tiles = (n_out + kTileRows - 1) / kTileRows;
    TS_TRY(alloc_n(&m->d_perm, (size_t)m->n_tiles * kTileRows));
    TS_TRY(alloc_n(&m->d_tmask, (size_t)m->n_tiles));
    TS_TRY(alloc_n(&m->d_tmask32, (size_t)m->n_tiles * (kTileRows / 32)));
    TS_TRY(alloc_n(&m->d_gnbr, (size_t)m->n_tiles * K3 * kTileRows));
    TS_TRY(alloc_n(&m->d_ghdr, (size_t)m->n_tiles * (kTileRows / 32) * 8));
    TS_TRY(alloc_n(&m->d_work, (size_t)m->n_tiles * 4 + 1));
    TS_HIP(hipMemsetAsync(m->d_work + m->n_tiles * 4, 0, sizeof(uint32_t), st));
    TS_LAUNCH("k_build_tiles", k_build_tiles, dim3((unsigned)m->n_tiles), dim3(kTileRows), m->d_nbr, n_out, K3, masks_sorted, rows_sorted, m->d_perm, m->d_tmask, m->d_tmask32, m->d_gnbr, m->d_ghdr, m->d_work, m->d_work + m->n_tiles * 4, split_thr(1), split_thr(2));
    TS_HIP(hipGetLastError());
    // temporaries go back to the pool when the caller's Temps dies; later work on the same
    // stream is ordered after the kernels above, so reuse is safe without another wait
    return TS_OK;
}

int build(const int32_t *coords, int64_t N, int K, int s, int transposed, ts_kmap *m) {
    hipStream_t st = stream();
    Temps tmp;
    const int K3 = K * K * K;
    m->K = K;
    m->s = s;
    m->transposed = transposed;
    m->K3 = K3;
    m->centre = (s == 1) ? (K3 - 1) / 2 : -1;
    if (N == 0) return TS_OK;

    int *d_status;
    TS_TRY(tmp.get(&d_status, ST_WORDS));
    TS_HIP(hipMemsetAsync(d_status, 0, ST_WORDS * sizeof(int), st));

    uint64_t *given;   // keys of the caller's coordinates
    TS_TRY(alloc_n(&given, (size_t)N));
    m->d_in_keys = given;   // provisional owner, so that an early error frees it
    if (s != 1)
        TS_LAUNCH("k_pack", k_pack, dim3(blocks_for(N, kThreads)), dim3(kThreads), reinterpret_cast<const int4 *>(coords), N, given, d_status);

    Table table;
    if (s == 1) {
        m->n_in = m->n_out = N;
        m->d_out_keys = given;
        TS_TRY(alloc_n(&m->d_nbr, (size_t)K3 * N));
        {
            ProfScope ps("memset_nbr");
            TS_HIP(hipMemsetAsync(m->d_nbr, 0xFF, (size_t)K3 * N * sizeof(int32_t), st));
        }
        TS_TRY(make_table(tmp, N, &table));
        TS_LAUNCH("k_pack_insert", k_pack_insert, dim3(blocks_for(N, kThreads)), dim3(kThreads), reinterpret_cast<const int4 *>(coords), N, given, table, m->d_nbr + (int64_t)m->centre * N, d_status);
        if (K3 > 1)
            TS_LAUNCH("k_probe_symmetric", k_probe_symmetric, dim3(blocks_for(N, kThreads), K3 / 2), dim3(kThreads), given, N, table, K, m->d_nbr);
    } else {
        // coarse set: candidates -> sort -> unique (the empty key, if present, sorts last)
        const bool one_each = (K == 2 && s == 2);
        const size_t n_cand = one_each ? (size_t)N : (size_t)N * K3;
        uint64_t *cand, *sorted, *uniq;
        int64_t *d_count;
        TS_TRY(tmp.get(&cand, n_cand));
        TS_TRY(tmp.get(&sorted, n_cand));
        TS_TRY(tmp.get(&uniq, n_cand));
        TS_TRY(tmp.get(&d_count, 1));
        if (one_each)
            TS_LAUNCH("k_candidates_k2s2", k_candidates_k2s2, dim3(blocks_for(N, kThreads)), dim3(kThreads), given, N, cand);
        else
            TS_LAUNCH("k_candidates", k_candidates, dim3(blocks_for(N, kThreads), K3), dim3(kThreads), given, N, K, s, cand);
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
        int64_t *h = static_cast<int64_t *>(host_staging(64));
        if (!h) return TS_ERR_OOM;
        TS_HIP(hipMemcpyAsync(h, d_count, sizeof(int64_t), hipMemcpyDeviceToHost, st));
        TS_HIP(hipStreamSynchronize(st));
        const int64_t n_coarse = h[0];
        uint64_t *coarse;
        TS_TRY(alloc_n(&coarse, (size_t)n_coarse));
        TS_HIP(hipMemcpyAsync(coarse, uniq, (size_t)n_coarse * sizeof(uint64_t), hipMemcpyDeviceToDevice, st));
        if (!transposed) {
            m->n_in = N;
            m->n_out = n_coarse;
            m->d_out_keys = coarse;
            if (n_coarse == 0) {   // only possible when every coordinate was rejected
                return fail(TS_ERR_COORD_RANGE, "no valid input coordinate");
            }
            TS_TRY(alloc_n(&m->d_nbr, (size_t)K3 * n_coarse));
            TS_TRY(make_table(tmp, N, &table));
            TS_LAUNCH("k_insert", k_insert, dim3(blocks_for(N, kThreads)), dim3(kThreads), given, N, table, (int32_t *)nullptr, d_status);
            TS_LAUNCH("k_probe_forward", k_probe_forward, dim3(blocks_for(n_coarse, kThreads), K3), dim3(kThreads), coarse, n_coarse, table, K, s, m->d_nbr);
        } else {
            m->n_in = n_coarse;
            m->n_out = N;
            m->d_in_keys = coarse;
            m->d_out_keys = given;
            if (n_coarse == 0) return fail(TS_ERR_COORD_RANGE, "no valid input coordinate");
            TS_TRY(alloc_n(&m->d_nbr, (size_t)K3 * N));
            // duplicates among the fine points are found by inserting them as well
            Table fine_table;
            TS_TRY(make_table(tmp, N, &fine_table));
            TS_LAUNCH("k_insert", k_insert, dim3(blocks_for(N, kThreads)), dim3(kThreads), given, N, fine_table, (int32_t *)nullptr, d_status);
            TS_TRY(make_table(tmp, n_coarse, &table));
            TS_LAUNCH("k_insert", k_insert, dim3(blocks_for(n_coarse, kThreads)), dim3(kThreads), coarse, n_coarse, table, (int32_t *)nullptr, d_status);
            TS_LAUNCH("k_probe_transposed", k_probe_transposed, dim3(blocks_for(N, kThreads), K3), dim3(kThreads), given, N, table, K, s, m->d_nbr);
        }
    }
    TS_HIP(hipGetLastError());
    return finish_map(m, tmp, d_status);
}

}  // namespace

extern "C" {

int ts_build_kmap(const int32_t *coords, int64_t N, int kernel_size, int stride, int transposed,
                  ts_kmap **out_kmap) {
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
    if (N > (int64_t)((1u << 31) - 1) / (ts::kMaxK3 + 1)) return fail(TS_ERR_UNSUPPORTED, "N too large for 32-bit pair indices");
    ts_kmap *m = new (std::nothrow) ts_kmap();
    if (!m) return fail(TS_ERR_OOM, "host allocation failed");
    int rc = build(coords, N, kernel_size, stride, transposed, m);
    if (rc != TS_OK) {
        (void)hipStreamSynchronize(ts::stream());
        destroy(m);
        return rc;
    }
    *out_kmap = m;
    return TS_OK;
}

void ts_free(ts_kmap *kmap) { destroy(kmap); }

int64_t ts_kmap_num_in(const ts_kmap *kmap) { return kmap ? kmap->n_in : -1; }
int64_t ts_kmap_num_out(const ts_kmap *kmap) { return kmap ? kmap->n_out : -1; }
int64_t ts_kmap_num_pairs(const ts_kmap *kmap) { return kmap ? kmap->M : -1; }
int ts_kmap_kernel_volume(const ts_kmap *kmap) { return kmap ? kmap->K3 : -1; }

int ts_kmap_out_coords(const ts_kmap *kmap, int32_t *dst) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    if (kmap->n_out == 0) return TS_OK;
    if (!dst || (reinterpret_cast<uintptr_t>(dst) & 15)) return fail(TS_ERR_INVALID_ARG, "dst is NULL or not 16-byte aligned");
    TS_LAUNCH("k_unpack", k_unpack, dim3(blocks_for(kmap->n_out, kThreads)), dim3(kThreads), kmap->d_out_keys, kmap->n_out, reinterpret_cast<int4 *>(dst));
    TS_HIP(hipGetLastError());
    return TS_OK;
}

int ts_kmap_in_coords(const ts_kmap *kmap, int32_t *dst) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    if (kmap->n_in == 0) return TS_OK;
    if (!dst || (reinterpret_cast<uintptr_t>(dst) & 15)) return fail(TS_ERR_INVALID_ARG, "dst is NULL or not 16-byte aligned");
    TS_LAUNCH("k_unpack", k_unpack, dim3(blocks_for(kmap->n_in, kThreads)), dim3(kThreads), kmap->d_in_keys, kmap->n_in, reinterpret_cast<int4 *>(dst));
    TS_HIP(hipGetLastError());
    return TS_OK;
}

int ts_kmap_sizes(const ts_kmap *kmap, int64_t *dst) {
    if (!kmap || !dst) return fail(TS_ERR_INVALID_ARG, "NULL argument");
    for (int n = 0; n < kmap->K3; ++n) dst[n] = kmap->sizes[n];
    return TS_OK;
}

int ts_kmap_pairs(const ts_kmap *kmap, int32_t *in_idx, int32_t *out_idx) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    if (kmap->M == 0) return TS_OK;
    size_t bytes = (size_t)kmap->M * sizeof(int32_t);
    if (in_idx) TS_HIP(hipMemcpyAsync(in_idx, kmap->d_in_idx, bytes, hipMemcpyDeviceToDevice, ts::stream()));
    if (out_idx) TS_HIP(hipMemcpyAsync(out_idx, kmap->d_out_idx, bytes, hipMemcpyDeviceToDevice, ts::stream()));
    return TS_OK;
}

}  // extern "C"
