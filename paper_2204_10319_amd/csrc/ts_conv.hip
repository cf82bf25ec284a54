// Feature computation of the sparse-convolution layer (paper Sec. 2.2, Alg. 2; Eq. 1).
//
// Two dataflows over the same kernel map:
//
//  explicit  - Alg. 2 in three launches for all offsets at once ("fused" gather / scatter of
//              Sec. 4.3.2): gather rows into the offset-major buffer F, grouped matmul
//              G = F_n * W_n scheduled as tiles over (offset, row block) without padding,
//              output-stationary reduction of G into X_out (each row reduced in registers,
//              written once).
//  fused     - one output-stationary kernel.  A workgroup owns 128 outputs (sorted by
//              neighbour bitmask so that they share offsets), walks the offsets present in
//              the tile, stages W_n in LDS, loads the neighbours' feature rows straight into
//              the MFMA operand registers and keeps the sum over offsets in the accumulators.
//              Neither F nor G exists; every output row is written once.
//
// MFMA orientation: D[co][m] += Wt[co][ci] * X[m][ci]  (32x32 tiles, "A" = transposed weights
// from LDS, "B" = gathered feature rows).  A lane then owns 4 consecutive output channels of
// one row per accumulator quad, which makes the stores 8-16 bytes wide.
#include "ts_internal.h"

#include <new>
#include <type_traits>
#include <utility>

using namespace ts;

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kWaveRows = 32;                 // rows (MFMA columns) per wave
static_assert(kWaves * kWaveRows == kTileRows, "tile = 4 waves x 32 rows");

// Per-dtype constants.  A lane moves 16-byte vectors of VEC elements.  One operand step covers
// KSTEP = 2*VEC input channels (lane halves h = 0/1 take VEC each).
template <class T> struct Elem;
template <> struct Elem<_Float16> {
    typedef half8 vec;
    static constexpr int VEC = 8, KSTEP = 16;
};
template <> struct Elem<float> {
    typedef floatx4 vec;
    static constexpr int VEC = 4, KSTEP = 8;
};

// Kernel shape: NCB blocks of 32 output channels per workgroup, input channels consumed in
// chunks of KC (KC divides C_in, so every chunk is full and the inner code is branch-free).
// LDS holds a [NCB*32][KC + VEC] slab of transposed weights; the VEC-element row padding
// makes the 16 lanes of a ds_read_b128 phase hit distinct bank groups.
template <class T, int NCB, int KC_>
struct Shape {
    typedef typename Elem<T>::vec vec;
    static constexpr int VEC = Elem<T>::VEC, KSTEP = Elem<T>::KSTEP, KC = KC_;
    static constexpr int NKB = KC / KSTEP;            // operand steps per chunk
    static constexpr int STRIDE = KC + VEC;           // LDS row stride in elements
    static constexpr int VPR = KC / VEC;              // 16-byte vectors per slab row
    static constexpr int ROWS = NCB * 32;
    static constexpr int TOTAL = ROWS * VPR;          // vectors per slab
    static constexpr int WV = (TOTAL + kThreads - 1) / kThreads;   // vectors per thread
    static constexpr int SLAB = ROWS * STRIDE;        // elements per slab
};

__device__ __forceinline__ void mma_step(const half8 &a, const half8 &b, floatx16 &acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_step(const floatx4 &a, const floatx4 &b, floatx16 &acc) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], acc, 0, 0, 0);
}

// Global -> registers: this thread's share of the weight slab of (offset n, channels k0..k0+KC).
// Threads past the end of a small slab repeat its last vector (same value to the same place).
template <class S, class T>
__device__ __forceinline__ void load_w_regs(typename S::vec (&wreg)[S::WV], const T *__restrict__ Wt, int n, int co0,
                                            int k0, int cin, int cout) {
    const T *src = Wt + ((int64_t)n * cout + co0) * cin + k0;
#pragma unroll
    for (int i = 0; i < S::WV; ++i) {
        int v = threadIdx.x + i * kThreads;
        v = v < S::TOTAL ? v : S::TOTAL - 1;
        int row = v / S::VPR, col = v % S::VPR;
        wreg[i] = *reinterpret_cast<const typename S::vec *>(src + (int64_t)row * cin + col * S::VEC);
    }
}

// Registers -> LDS, same mapping.
template <class S, class T>
__device__ __forceinline__ void store_w_regs(const typename S::vec (&wreg)[S::WV], T *lds) {
#pragma unroll
    for (int i = 0; i < S::WV; ++i) {
        int v = threadIdx.x + i * kThreads;
        v = v < S::TOTAL ? v : S::TOTAL - 1;
        int row = v / S::VPR, col = v % S::VPR;
        *reinterpret_cast<typename S::vec *>(lds + row * S::STRIDE + col * S::VEC) = wreg[i];
    }
}

// Global -> registers: the lane's operand vectors for channels [k0, k0+KC) of the row at `row`
// (already offset to the lane's half).  No predication: absent neighbours point at a zero row.
template <class S, class T>
__device__ __forceinline__ void load_x_regs(typename S::vec (&b)[S::NKB], const T *row) {
#pragma unroll
    for (int kb = 0; kb < S::NKB; ++kb) b[kb] = *reinterpret_cast<const typename S::vec *>(row + kb * S::KSTEP);
}

// acc[cb] += slab[cb*32 .. +32][0 .. KC) * b^T.
template <class S, class T, int NCB>
__device__ __forceinline__ void mma_stage(const T *lds, const typename S::vec (&b)[S::NKB], floatx16 (&acc)[NCB]) {
    const int lane = threadIdx.x & 63, m = lane & 31, h = lane >> 5;
    const T *base = lds + m * S::STRIDE + h * S::VEC;
#pragma unroll
    for (int kb = 0; kb < S::NKB; ++kb) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            typename S::vec a = *reinterpret_cast<const typename S::vec *>(base + cb * 32 * S::STRIDE + kb * S::KSTEP);
            mma_step(a, b[kb], acc[cb]);
        }
    }
}

// Store the wave's accumulators: lane (m, h) holds, for block cb and quad g, the channels
// co0 + cb*32 + g*8 + h*4 + {0..3} of row m.
template <class TO, int NCB>
__device__ __forceinline__ void store_rows(TO *out, int64_t row, int cout, int co0, const floatx16 (&acc)[NCB]) {
    const int lane = threadIdx.x & 63, h = lane >> 5;
    if (row < 0) return;
    TO *dst = out + row * cout + co0 + h * 4;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if constexpr (sizeof(TO) == 2) {
                half4 v = {(_Float16)acc[cb][g * 4 + 0], (_Float16)acc[cb][g * 4 + 1], (_Float16)acc[cb][g * 4 + 2],
                           (_Float16)acc[cb][g * 4 + 3]};
                *reinterpret_cast<half4 *>(dst + cb * 32 + g * 8) = v;
            } else {
                floatx4 v = {acc[cb][g * 4 + 0], acc[cb][g * 4 + 1], acc[cb][g * 4 + 2], acc[cb][g * 4 + 3]};
                *reinterpret_cast<floatx4 *>(dst + cb * 32 + g * 8) = v;
            }
        }
    }
}

// ---- fused output-stationary kernel ---------------------------------------------------------
// grid = (tiles, cout / (NCB*32)); cin is a multiple of KC.  A "stage" is one (offset n,
// channel chunk k0) pair of the tile.  Software pipeline with one barrier per stage: while the
// MFMAs of stage s read LDS slab `cur` and the operand registers loaded one stage earlier,
// the global loads of stage s+1 (weight slab, neighbour rows) are in flight; the slab goes to
// the other LDS buffer after the MFMAs.  All loads are unconditional so that the compiler can
// count them: rows without a neighbour read `zero_row` instead.
template <class T, int NCB, int KC, int G>
__global__ void __launch_bounds__(kThreads) k_fused(const T *__restrict__ X, const T *__restrict__ Wt,
                                                    const int32_t *__restrict__ nbr, int stride,
                                                    const int32_t *__restrict__ perm, int64_t n_out,
                                                    T *__restrict__ out, const T *__restrict__ zero_row, int cin,
                                                    int cout, int K3, int centre) {
    typedef Shape<T, NCB, KC> S;
    typedef typename S::vec vec;
    __shared__ __attribute__((aligned(16))) T lds_w[2][G][S::SLAB];
    __shared__ int32_t lds_j[kMaxK3][kTileRows];
    __shared__ uint32_t s_mask;
    const int64_t tile = blockIdx.x;
    const int co0 = blockIdx.y * NCB * 32;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, m = lane & 31, h = lane >> 5;
    const int slot = wave * kWaveRows + m;
    floatx16 acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
        for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;

    // Neighbour rows of the tile's outputs -> LDS (offset-major), and the OR of their offset
    // bitmasks.  Two threads share an output row and read half of its table row each, all
    // loads issued before the first is used.
    if (threadIdx.x == 0) s_mask = 0;
    __syncthreads();
    {
        const int half = threadIdx.x >> 7, col = threadIdx.x & 127;
        const int64_t pos = tile * kTileRows + col;
        const int32_t k = perm ? perm[pos] : (pos < n_out ? (int32_t)pos : -1);
        const int chunks = stride / 4, cph = chunks >= 2 ? chunks / 2 : 1;
        const int4 *src = reinterpret_cast<const int4 *>(nbr + (int64_t)(k >= 0 ? k : 0) * stride);
        int4 v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ch = half * cph + i;
            v[i] = make_int4(-1, -1, -1, -1);
            if (k >= 0 && i < cph && ch < chunks) v[i] = src[ch];
        }
        uint32_t mm = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ch = half * cph + i;
            if (i < cph && ch < chunks) {
                const int32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = ch * 4 + q;
                    // the row's offsets are read off its entries (the bitmask word of the table and
                    // the centre entry may not have been written yet: a map's row pass runs on demand)
                    if (idx < K3) {
                        const int32_t j = idx == centre ? k : (k >= 0 ? e[q] : -1);
                        lds_j[idx][col] = j;
                        if (j >= 0) mm |= 1u << idx;
                    }
                }
            }
        }
        for (int d = 32; d >= 1; d >>= 1) mm |= (uint32_t)__shfl_xor((int)mm, d, 64);
        if (lane == 0 && mm) atomicOr(&s_mask, mm);
    }
    __syncthreads();   // lds_j and s_mask complete
    const uint32_t mask = s_mask;

    if (mask) {
        // Iterator over the tile's (offset, chunk) pairs; a stage takes the next G of them.
        // Past the end it keeps returning the last pair with live = false (loads stay
        // unconditional and in bounds, the MFMAs are skipped).
        uint32_t rem = mask;
        int it_n = __builtin_ctz(rem), it_k = 0;
        bool it_live = true;
        rem &= rem - 1;
        auto next_pair = [&](int &n, int &k0, bool &live) {
            n = it_n;
            k0 = it_k;
            live = it_live;
            if (it_k + KC < cin) {
                it_k += KC;
            } else if (rem) {
                it_k = 0;
                it_n = __builtin_ctz(rem);
                rem &= rem - 1;
            } else {
                it_live = false;
            }
        };
        vec wreg[G][S::WV], bx_a[G][S::NKB], bx_b[G][S::NKB];
        int32_t j_a[G], j_b[G];
        bool live_a[G], live_b[G];
        auto issue_loads = [&](vec(&b)[G][S::NKB], int32_t(&j)[G], bool(&live)[G]) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                int n, k0;
                next_pair(n, k0, live[g]);
                load_w_regs<S, T>(wreg[g], Wt, n, co0, k0, cin, cout);
                j[g] = live[g] ? lds_j[n][slot] : -1;
                load_x_regs<S, T>(b[g], (j[g] >= 0 ? X + (int64_t)j[g] * cin + k0 : zero_row) + h * S::VEC);
            }
        };
        issue_loads(bx_a, j_a, live_a);
#pragma unroll
        for (int g = 0; g < G; ++g) store_w_regs<S, T>(wreg[g], lds_w[0][g]);
        int cur = 0;
        // One stage.  The two operand register sets swap roles between calls, so prefetched
        // registers are never copied (a copy would wait for the loads at once).
        auto stage = [&](vec(&b_now)[G][S::NKB], int32_t(&j_now)[G], bool(&live_now)[G], vec(&b_next)[G][S::NKB],
                         int32_t(&j_next)[G], bool(&live_next)[G]) -> bool {
            __syncthreads();   // slabs `cur` are complete; nobody still reads the other buffer
            const bool more = it_live;
            issue_loads(b_next, j_next, live_next);
#pragma unroll
            for (int g = 0; g < G; ++g)
                if (live_now[g] && __ballot(j_now[g] >= 0) != 0) mma_stage<S, T, NCB>(lds_w[cur][g], b_now[g], acc);
#pragma unroll
            for (int g = 0; g < G; ++g) store_w_regs<S, T>(wreg[g], lds_w[cur ^ 1][g]);
            cur ^= 1;
            return more;
        };
        for (;;) {
            if (!stage(bx_a, j_a, live_a, bx_b, j_b, live_b)) break;
            if (!stage(bx_b, j_b, live_b, bx_a, j_a, live_a)) break;
        }
    }
    {
        const int64_t pos = tile * kTileRows + slot;
        store_rows<T, NCB>(out, perm ? perm[pos] : (pos < n_out ? pos : -1), cout, co0, acc);
    }
}

// ---- fused output-stationary kernel, fp16, deep software pipeline ---------------------------------
// D[co][m] += Wt[co][ci] * X[m][ci] with v_mfma_f32_16x16x32_f16: lane l of a wave holds, of the
// "B" operand, 8 consecutive input channels (8 * (l / 16) + 0..7 of a 32-channel step) of
// output row l % 16, i.e. 16 contiguous bytes of the neighbour's feature row, so gathered rows
// go from memory straight into the operand registers, 4 lanes per 64 bytes of a row.  A wave owns
// 32 output rows (two 16-column blocks), a workgroup 128; the accumulators hold NCO blocks of 16
// output channels.  A stage is one (offset, KC-channel chunk) of the tile: its weight slab, kept
// in global memory in operand order, goes global -> registers -> LDS once for the four waves.
// What a wave pays for is dependent memory round trips, so the loads of a stage are issued DEPTH
// stages before their use and rotate through DEPTH register sets; one barrier per stage.
// Rows of an output are added in offset order whatever the tile holds, so results do not depend
// on how rows are grouped.
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vector: arrays of it stay in registers

// Calls fn(std::integral_constant<int, 0>{}) ... fn(std::integral_constant<int, N-1>{}): the index
// is a constant expression inside fn, so arrays indexed with it stay in registers.
template <class Fn, int... I>
__device__ __forceinline__ void static_for_impl(Fn &&fn, std::integer_sequence<int, I...>) {
    (fn(std::integral_constant<int, I>{}), ...);
}
template <int N, class Fn>
__device__ __forceinline__ void static_for(Fn &&fn) {
    static_for_impl(fn, std::make_integer_sequence<int, N>{});
}

// (Three waves per SIMD are asked for wherever the accumulators leave room: left to itself the compiler
// takes a few registers more than that allows for the six- and eight-block single-step variants.)
template <int NCO, int KSTEPS, int DEPTH, bool TWO = false>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(NCO * KSTEPS <= 8 ? 3 : 2))) k_conv_tile(const _Float16 *__restrict__ X, const u32x4 *__restrict__ Wf,
                                                        const int32_t *__restrict__ nbr, int stride,
                                                        const int32_t *__restrict__ perm,
                                                        const int32_t *__restrict__ tile_order, int64_t n_out,
                                                        _Float16 *__restrict__ out, int *__restrict__ sched,
                                                        int cin, int cout, int K3, const _Float16 *__restrict__ bias,
                                                        const _Float16 *__restrict__ residual, int relu, int x_bytes,
                                                        int w_bytes, int centre, const _Float16 *__restrict__ X2,
                                                        int x2_bytes, int cin1) {
    // TWO: the layer's input is the channel concatenation [X | X2], which is never formed: input channels
    // below cin1 are read from X (rows of cin1 channels), the others from X2 (rows of cin - cin1 channels);
    // cin1 is a multiple of 32, so each 32-channel operand step lies in one of the two.  Otherwise X2,
    // x2_bytes are unused and cin1 = cin.
    constexpr int KC = KSTEPS * 32, FRAGS = NCO * KSTEPS, SLAB = FRAGS * 64;   // slab in 16-byte vectors
    constexpr int WV = (SLAB + kThreads - 1) / kThreads;
    __shared__ u32x4 lds_w[2][SLAB];
    __shared__ int32_t lds_j[kMaxK3][kTileRows];
    __shared__ uint32_t s_mask;
    __shared__ int s_tile;
    // The launch holds as many workgroups as stay resident at once.  Workgroup b starts with tile b;
    // the tiles beyond the grid are handed out through counters, so nobody waits for a second
    // round of workgroups.  One counter per XCD (blockIdx % 8), on cache lines of their own:
    // atomics on one address are served one after the other.
    const int64_t n_tiles = (n_out + kTileRows - 1) / kTileRows;
    sched += kSchedWords * blockIdx.y;
    const int xcd = blockIdx.x & 7;
    const int cb0 = blockIdx.y * NCO;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, m16 = lane & 15, g = lane >> 4;
    const int r0 = wave * kWaveRows + m16, r1 = r0 + 16;   // the lane's two output rows (tile slots)
    // Longest tiles first, so that they do not start when everything else is done: by the order
    // the map build prepared (tiles of rows in input order by descending number of offsets); rows
    // sorted by bitmask put the tiles with the most offsets last, so those are taken from the end.
    int64_t turn = blockIdx.x;
    while (turn < n_tiles) {
    const int64_t tile = perm ? n_tiles - 1 - turn : (tile_order ? tile_order[turn] : turn);
    // ask for the next tile now; the answer is needed when this one is done
    int ticket = 0;
    if (threadIdx.x == 0) ticket = atomicAdd(&sched[xcd * 32], 1);

    // Neighbour rows of the tile's outputs -> LDS (offset-major), and the OR of their offset
    // bitmasks.  The 16-byte chunks of a table row go to neighbouring lanes, so that one load
    // instruction covers whole rows (a row touched by several instructions costs a request each).
    if (threadIdx.x == 0) s_mask = 0;
    __syncthreads();
    {
        const int chunks = stride / 4;                       // 8, 4 or 1 lanes per row
        const int ch = threadIdx.x % chunks, sub = threadIdx.x / chunks;
        const int rows_per_pass = kThreads / chunks;         // 32, 64 or 256
        int4 v[4];
        int32_t kk[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int col = i * rows_per_pass + sub;
            const int64_t pos = tile * kTileRows + col;
            kk[i] = -2;                                      // -2: no row of the tile in this pass
            if (col < kTileRows) kk[i] = perm ? perm[pos] : (pos < n_out ? (int32_t)pos : -1);
            v[i] = make_int4(-1, -1, -1, -1);
            if (kk[i] >= 0) v[i] = reinterpret_cast<const int4 *>(nbr + (int64_t)kk[i] * stride)[ch];
        }
        uint32_t mm = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (kk[i] == -2) continue;
            const int col = i * rows_per_pass + sub;
            const int32_t k = kk[i];
            const int32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int idx = ch * 4 + q;
                // the row's offsets are read off its entries (the bitmask word of the table and
                // the centre entry may not have been written yet: a map's row pass runs on demand)
                if (idx < K3) {
                    const int32_t j = idx == centre ? k : (k >= 0 ? e[q] : -1);
                    lds_j[idx][col] = j;
                    if (j >= 0) mm |= 1u << idx;
                }
            }
        }
        for (int d = 32; d >= 1; d >>= 1) mm |= (uint32_t)__shfl_xor((int)mm, d, 64);
        if (lane == 0 && mm) atomicOr(&s_mask, mm);
    }
    __syncthreads();
    // the offsets present in the tile, as a bitmask in a scalar register: the stages walk its set bits
    const uint32_t mask = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_mask);
    const int nchunks = cin / KC;
    const int nstage = __builtin_popcount(mask) * nchunks;
    const int cblocks = cout / 16;

    floatx4 acc[NCO][2];
#pragma unroll
    for (int cb = 0; cb < NCO; ++cb)
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) acc[cb][c2] = floatx4{0.f, 0.f, 0.f, 0.f};

    u32x4 wreg[DEPTH][WV];
    half8v xreg[DEPTH][2][KSTEPS];
    bool xlive[DEPTH];
    // Issue the loads of stage s into register set d (d is a compile-time constant at every call).
    // Every call issues the same number of loads, unconditionally (past the last stage it repeats
    // that stage; rows without the offset read the zero row): the compiler counts outstanding
    // loads to place its waits, and a load it cannot count would make every wait a full drain.
    // Loads go through buffer descriptors: a 32-bit byte offset per lane plus a wave-uniform one, no
    // 64-bit address arithmetic in the loop, and an offset beyond the buffer reads as zero without
    // touching memory, which is what a row without the offset must contribute.  The loop body is
    // short on purpose: with ~200 vector instructions per stage around 16 MFMAs this kernel was
    // bound by instruction issue.
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16 *>(X), 0, x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t xrsrc2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16 *>(TWO ? X2 : X), 0, TWO ? x2_bytes : x_bytes, 0x00020000);
    const int row_bytes2 = (cin - cin1) * 2;
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4 *>(Wf), 0, w_bytes, 0x00020000);
    constexpr int kNoRow = (int)0x80000000u;   // beyond any buffer this kernel is launched with
    const int row_bytes = cin1 * 2, xlane = g * 16;
    int wlane[WV];
#pragma unroll
    for (int v = 0; v < WV; ++v) {
        int idx = threadIdx.x + v * kThreads;
        if (SLAB % kThreads != 0) idx = idx < SLAB ? idx : SLAB - 1;   // surplus threads repeat the last vector
        wlane[v] = idx * 16;
    }
    uint32_t it_rem = mask ? mask : 1u;   // offsets not issued yet; the lowest set bit is the one being issued
    int it_ch = 0;                        // its chunk
    // neighbour rows of the lane's two outputs for the stage issued next: read out of LDS one stage
    // ahead, so that no stage waits for them
    int32_t pj0 = lds_j[__builtin_ctz(it_rem)][r0], pj1 = lds_j[__builtin_ctz(it_rem)][r1];
    // Issue the loads of stage s into register set d (a compile-time constant at every call).
    // Every call issues the same loads, unconditionally (past the last stage it repeats that
    // stage): the compiler counts outstanding loads to place its waits, and a load it cannot count
    // makes every wait a full drain.
    auto issue = [&](int s, auto dc) __attribute__((always_inline)) {
        constexpr int d = decltype(dc)::value;
        const bool real = s < nstage;
        const int ch = it_ch, n = __builtin_ctz(it_rem);   // scalar: the weight slab's address stays in scalar registers
        const int32_t j0 = pj0, j1 = pj1;
        if (s + 1 < nstage) {   // stages are issued in order: step the pair, stay on the last one past the end
            if (++it_ch == nchunks) {
                it_ch = 0;
                it_rem &= it_rem - 1;
            }
        }
        pj0 = lds_j[__builtin_ctz(it_rem)][r0];
        pj1 = lds_j[__builtin_ctz(it_rem)][r1];
        const int wsoff = (((n * nchunks + ch) * cblocks + cb0) * KSTEPS) * 1024;
#pragma unroll
        for (int v = 0; v < WV; ++v) wreg[d][v] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane[v], wsoff, 0);
        xlive[d] = real && __ballot(j0 >= 0 || j1 >= 0) != 0;   // false: none of the wave's rows has this offset
        const int off0 = j0 >= 0 ? j0 * row_bytes + xlane : kNoRow;
        const int off1 = j1 >= 0 ? j1 * row_bytes + xlane : kNoRow;
        const int xsoff = ch * (KC * 2);
        int offb0 = 0, offb1 = 0;
        if constexpr (TWO) {
            offb0 = j0 >= 0 ? j0 * row_bytes2 + xlane : kNoRow;
            offb1 = j1 >= 0 ? j1 * row_bytes2 + xlane : kNoRow;
        }
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            u32x4 v0, v1;
            if constexpr (TWO) {
                const int c0 = ch * KC + ks * 32;        // first input channel of this operand step
                const bool second = c0 >= cin1;          // wave-uniform: the step lies in X2
                const int so = second ? (c0 - cin1) * 2 : c0 * 2;
                v0 = __builtin_amdgcn_raw_buffer_load_b128(second ? xrsrc2 : xrsrc, second ? offb0 : off0, so, 0);
                v1 = __builtin_amdgcn_raw_buffer_load_b128(second ? xrsrc2 : xrsrc, second ? offb1 : off1, so, 0);
            } else {
                v0 = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off0, xsoff + ks * 64, 0);
                v1 = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off1, xsoff + ks * 64, 0);
            }
            __builtin_memcpy(&xreg[d][0][ks], &v0, 16);
            __builtin_memcpy(&xreg[d][1][ks], &v1, 16);
        }
    };
    auto run = [&](int s, auto dc) __attribute__((always_inline)) {
        constexpr int d = decltype(dc)::value;
        u32x4 *slab = lds_w[s & 1];
#pragma unroll
        for (int v = 0; v < WV; ++v) slab[wlane[v] >> 4] = wreg[d][v];
        __syncthreads();   // slab complete; everybody is done with the other slab
        if (xlive[d]) {
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                // all weight fragments of the step out of LDS first, then the MFMAs: a read placed
                // right before its MFMA costs one LDS latency per fragment
                u32x4 raw[NCO];
#pragma unroll
                for (int cb = 0; cb < NCO; ++cb) raw[cb] = slab[(cb * KSTEPS + ks) * 64 + lane];
                __builtin_amdgcn_s_setprio(1);
#pragma unroll
                for (int cb = 0; cb < NCO; ++cb) {
                    half8v a;
                    __builtin_memcpy(&a, &raw[cb], 16);
                    acc[cb][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, xreg[d][0][ks], acc[cb][0], 0, 0, 0);
                    acc[cb][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, xreg[d][1][ks], acc[cb][1], 0, 0, 0);
                }
                __builtin_amdgcn_s_setprio(0);
            }
        }
        issue(s + DEPTH, dc);
    };
    if (nstage > 0) {
        static_for<DEPTH>([&](auto dc) __attribute__((always_inline)) { issue(decltype(dc)::value, dc); });
        // whole rounds of DEPTH stages; stages past the end only repeat loads and skip the MFMAs
        for (int s0 = 0; s0 < nstage; s0 += DEPTH) static_for<DEPTH>([&](auto dc) __attribute__((always_inline)) { run(s0 + decltype(dc)::value, dc); });
    }

    // lane l holds, per block, output channels 4 * (l / 16) + 0..3 of rows r0 (c2 = 0) and r1 (c2 = 1).
    // What the tail adds is asked for in one go per kind (all blocks' bias words, then all blocks' residual
    // words of a row) and used afterwards: a load placed next to its use costs a round trip per block.
    half4 bv[NCO];
#pragma unroll
    for (int cb = 0; cb < NCO; ++cb) bv[cb] = half4{(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
    if (bias) {
        // (the pointer is made opaque per tile: loads the compiler can prove the same for every tile move to the
        // top of the kernel and hold registers through the stage loop, which has none to spare)
        const _Float16 *bp = bias;
        asm volatile("" : "+s"(bp));
#pragma unroll
        for (int cb = 0; cb < NCO; ++cb) bv[cb] = *reinterpret_cast<const half4 *>(bp + cb0 * 16 + cb * 16 + g * 4);
    }
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2) {
        const int64_t pos = tile * kTileRows + (c2 ? r1 : r0);
        const int64_t row = perm ? perm[pos] : (pos < n_out ? pos : -1);
        if (row < 0) continue;
        const int64_t at = row * cout + cb0 * 16 + g * 4;
        // the layer's own result, rounded once to fp16 (the accumulators' registers are free from here on) ...
        half4 v[NCO];
#pragma unroll
        for (int cb = 0; cb < NCO; ++cb)
            v[cb] = half4{(_Float16)acc[cb][c2][0], (_Float16)acc[cb][c2][1], (_Float16)acc[cb][c2][2], (_Float16)acc[cb][c2][3]};
        // ... then, if asked for, what ts_bias_act would do with it: fp32 sum, ReLU, one rounding
        if (bias || residual || relu) {
            half4 rv[NCO];
#pragma unroll
            for (int cb = 0; cb < NCO; ++cb) rv[cb] = half4{(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
            if (residual) {
#pragma unroll
                for (int cb = 0; cb < NCO; ++cb) rv[cb] = *reinterpret_cast<const half4 *>(residual + at + cb * 16);
            }
#pragma unroll
            for (int cb = 0; cb < NCO; ++cb) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float f = (float)v[cb][e];
                    if (bias) f += (float)bv[cb][e];
                    if (residual) f += (float)rv[cb][e];
                    v[cb][e] = (_Float16)(relu && f < 0.f ? 0.f : f);
                }
            }
        }
#pragma unroll
        for (int cb = 0; cb < NCO; ++cb) *reinterpret_cast<half4 *>(out + at + cb * 16) = v[cb];
    }
    if (threadIdx.x == 0) s_tile = ticket;
    __syncthreads();   // the tile's LDS is free; s_tile is set
    turn = (int64_t)gridDim.x + xcd + 8 * (int64_t)s_tile;
    }
    // the last workgroup to leave rearms the counters for the next launch on this map
    if (threadIdx.x == 0 && atomicAdd(&sched[8 * 32], 1) == (int)gridDim.x - 1) {
        for (int i = 0; i <= 8; ++i) sched[i * 32] = 0;
    }
}

// ---- fused kernel for narrow layers: all weights resident in LDS -----------------------------------
// With C_in = 32 KSTEPS and a slice of 16 NCO output channels the weights, in operand order, are
// K^3 NCO KSTEPS KiB (used with C_in <= 32 and C_out = 32 or 64: 54 or 108 KiB):
// it is loaded into LDS once per workgroup and stays.  Nothing is shared between waves after that,
// so there is no barrier in the loop and the unit of work is a wave's own 32 output rows: its
// neighbour rows sit in a slice of LDS that only this wave touches, the offsets it walks are the
// ones its own 32 rows have (fewer than a 128-row tile has), and units are handed to waves, not to
// workgroups.  Operand layout, accumulation order (offsets ascending per output) and epilogue are
// those of k_conv_tile: the two kernels give the same bits.
// (8 to 16 waves per workgroup and 2 to 8 stages of loads in flight all land within 10 % of each other on
// 153 k points; 12 waves with 3 stages was the fastest.)
constexpr int kResWaves = 12, kResDepth = 3, kResThreads = kResWaves * 64, kResRows = 32;
template <int FRAGS>
constexpr size_t res_lds_bytes() {
    return (size_t)kMaxK3 * FRAGS * 64 * 16 + (size_t)kResWaves * kMaxK3 * kResRows * 4;
}

template <int NCO, int KSTEPS, int DEPTH>
__global__ void __launch_bounds__(kResThreads) k_conv_res(const _Float16 *__restrict__ X, const u32x4 *__restrict__ Wf,
                                                          const int32_t *__restrict__ nbr, int stride,
                                                          const int32_t *__restrict__ perm, int64_t n_out,
                                                          _Float16 *__restrict__ out, int *__restrict__ sched, int K3, int cout,
                                                          const _Float16 *__restrict__ bias,
                                                          const _Float16 *__restrict__ residual, int relu, int x_bytes,
                                                          int centre) {
    extern __shared__ u32x4 lds_res[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, m16 = lane & 15, g = lane >> 4;
    constexpr int FRAGS = NCO * KSTEPS;
    const int cb0 = blockIdx.y * NCO, cblocks = cout / 16;
    sched += kSchedWords * blockIdx.y;
    u32x4 *lds_w = lds_res;                                                         // [K3][NCO][KSTEPS][64]
    int32_t *lds_j = reinterpret_cast<int32_t *>(lds_res + kMaxK3 * FRAGS * 64) + wave * (kMaxK3 * kResRows);   // [K3][32], this wave's
    // the fragments of this slice of output channels are contiguous within an offset
    for (int i = threadIdx.x; i < K3 * FRAGS * 64; i += kResThreads) {
        const int n = i / (FRAGS * 64), rem = i % (FRAGS * 64);
        lds_w[i] = Wf[(n * cblocks + cb0) * KSTEPS * 64 + rem];
    }
    __syncthreads();

    constexpr int row_bytes = KSTEPS * 64;
    const int64_t n_units = (n_out + kResRows - 1) / kResRows;
    const int64_t n_waves = (int64_t)gridDim.x * kResWaves;
    const int xcd = blockIdx.x & 7;
    const int r0 = m16, r1 = m16 + 16;
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16 *>(X), 0, x_bytes, 0x00020000);
    constexpr int kNoRow = (int)0x80000000u;
    const int xlane = g * 16;
    // A wave starts with unit (its index in the launch); the units beyond the launch come from the
    // per-XCD counters, as tiles do in k_conv_tile.
    int64_t turn = (int64_t)blockIdx.x * kResWaves + wave;
    while (turn < n_units) {
        const int64_t unit = perm ? n_units - 1 - turn : turn;
        int ticket = 0;
        if (lane == 0) ticket = atomicAdd(&sched[xcd * 32], 1);
        uint32_t mm = 0;
        {
            const int chunks = stride / 4;                       // 8, 4 or 1 lanes per table row
            const int ch = lane % chunks, sub = lane / chunks;
            const int rows_per_pass = 64 / chunks;               // 8, 16 or 64
            int4 v[4];
            int32_t kk[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int col = i * rows_per_pass + sub;
                const int64_t pos = unit * kResRows + col;
                kk[i] = -2;                                      // -2: no row of the unit in this pass
                if (col < kResRows) kk[i] = perm ? perm[pos] : (pos < n_out ? (int32_t)pos : -1);
                v[i] = make_int4(-1, -1, -1, -1);
                if (kk[i] >= 0) v[i] = reinterpret_cast<const int4 *>(nbr + (int64_t)kk[i] * stride)[ch];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (kk[i] == -2) continue;
                const int col = i * rows_per_pass + sub;
                const int32_t k = kk[i];
                const int32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = ch * 4 + q;
                    if (idx < K3) {
                        const int32_t j = idx == centre ? k : (k >= 0 ? e[q] : -1);
                        lds_j[idx * kResRows + col] = j;
                        if (j >= 0) mm |= 1u << idx;
                    }
                }
            }
            for (int d = 32; d >= 1; d >>= 1) mm |= (uint32_t)__shfl_xor((int)mm, d, 64);
        }
        // LDS serves a wave's accesses in order: what its lanes wrote above is what they read below
        __builtin_amdgcn_wave_barrier();
        const uint32_t mask = (uint32_t)__builtin_amdgcn_readfirstlane((int)mm);
        const int nstage = __builtin_popcount(mask);

        floatx4 acc[NCO][2];
#pragma unroll
        for (int cb = 0; cb < NCO; ++cb)
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2) acc[cb][c2] = floatx4{0.f, 0.f, 0.f, 0.f};
        half8v xreg[DEPTH][2][KSTEPS];
        int nn[DEPTH];
        bool xlive[DEPTH];
        uint32_t it_rem = mask ? mask : 1u;
        int32_t pj0 = lds_j[__builtin_ctz(it_rem) * kResRows + r0], pj1 = lds_j[__builtin_ctz(it_rem) * kResRows + r1];
        // the same loads at every call (past the last stage they repeat it), so the compiler can count them
        auto issue = [&](int s, auto dc) __attribute__((always_inline)) {
            constexpr int d = decltype(dc)::value;
            xlive[d] = s < nstage;
            nn[d] = __builtin_ctz(it_rem);
            const int32_t j0 = pj0, j1 = pj1;
            if (s + 1 < nstage) it_rem &= it_rem - 1;
            pj0 = lds_j[__builtin_ctz(it_rem) * kResRows + r0];
            pj1 = lds_j[__builtin_ctz(it_rem) * kResRows + r1];
            const int off0 = j0 >= 0 ? j0 * row_bytes + xlane : kNoRow;
            const int off1 = j1 >= 0 ? j1 * row_bytes + xlane : kNoRow;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off0, ks * 64, 0);
                const u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off1, ks * 64, 0);
                __builtin_memcpy(&xreg[d][0][ks], &v0, 16);
                __builtin_memcpy(&xreg[d][1][ks], &v1, 16);
            }
        };
        auto run = [&](int s, auto dc) __attribute__((always_inline)) {
            constexpr int d = decltype(dc)::value;
            if (xlive[d]) {
                u32x4 raw[NCO][KSTEPS];
#pragma unroll
                for (int cb = 0; cb < NCO; ++cb)
#pragma unroll
                    for (int ks = 0; ks < KSTEPS; ++ks) raw[cb][ks] = lds_w[((nn[d] * NCO + cb) * KSTEPS + ks) * 64 + lane];
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
                    for (int cb = 0; cb < NCO; ++cb) {
                        half8v a;
                        __builtin_memcpy(&a, &raw[cb][ks], 16);
                        acc[cb][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, xreg[d][0][ks], acc[cb][0], 0, 0, 0);
                        acc[cb][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, xreg[d][1][ks], acc[cb][1], 0, 0, 0);
                    }
            }
            issue(s + DEPTH, dc);
        };
        if (nstage > 0) {
            static_for<DEPTH>([&](auto dc) __attribute__((always_inline)) { issue(decltype(dc)::value, dc); });
            for (int s0 = 0; s0 < nstage; s0 += DEPTH) static_for<DEPTH>([&](auto dc) __attribute__((always_inline)) { run(s0 + decltype(dc)::value, dc); });
        }
        // the reads of lds_j issued last belong to no stage: they must have returned before the next unit overwrites it
        __builtin_amdgcn_wave_barrier();

#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) {
            const int64_t pos = unit * kResRows + (c2 ? r1 : r0);
            const int64_t row = perm ? perm[pos] : (pos < n_out ? pos : -1);
            if (row < 0) continue;
            const int64_t at = row * cout + cb0 * 16 + g * 4;
#pragma unroll
            for (int cb = 0; cb < NCO; ++cb) {
                half4 v = {(_Float16)acc[cb][c2][0], (_Float16)acc[cb][c2][1], (_Float16)acc[cb][c2][2], (_Float16)acc[cb][c2][3]};
                if (bias || residual || relu) {
                    float f[4] = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
                    if (bias) {
                        const half4 b = *reinterpret_cast<const half4 *>(bias + cb0 * 16 + cb * 16 + g * 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) f[e] += (float)b[e];
                    }
                    if (residual) {
                        const half4 r = *reinterpret_cast<const half4 *>(residual + at + cb * 16);
#pragma unroll
                        for (int e = 0; e < 4; ++e) f[e] += (float)r[e];
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (_Float16)(relu && f[e] < 0.f ? 0.f : f[e]);
                }
                *reinterpret_cast<half4 *>(out + at + cb * 16) = v;
            }
        }
        ticket = __builtin_amdgcn_readfirstlane(ticket);
        turn = n_waves + xcd + 8 * (int64_t)ticket;
    }
    __syncthreads();   // all waves of the workgroup are done
    // the last workgroup to leave rearms the counters for the next launch on this map
    if (threadIdx.x == 0 && atomicAdd(&sched[8 * 32], 1) == (int)gridDim.x - 1) {
        for (int i = 0; i <= 8; ++i) sched[i * 32] = 0;
    }
}

// Weights in the operand order of k_conv_tile:
// Wf[n][chunk][cb][ks][lane][e] = W[n][ci][co], co = cb*16 + lane%16, ci = chunk*KC + ks*32 + 8*(lane/16) + e
// (0 for ci >= cin).  One (n, chunk, cb, ks) fragment is 64 lanes x 16 bytes, contiguous.
__global__ void k_pack_weights_tile(const _Float16 *__restrict__ W, _Float16 *__restrict__ Wf, int K3, int cin,
                                    int cin_pad, int cout, int ksteps) {
    const int64_t gidx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)K3 * cout * cin_pad;
    if (gidx >= total) return;
    const int kc = ksteps * 32, nchunks = cin_pad / kc, cblocks = cout / 16;
    int64_t r = gidx;
    const int e = (int)(r % 8); r /= 8;
    const int lane = (int)(r % 64); r /= 64;
    const int ks = (int)(r % ksteps); r /= ksteps;
    const int cb = (int)(r % cblocks); r /= cblocks;
    const int chunk = (int)(r % nchunks); r /= nchunks;
    const int n = (int)r;
    const int co = cb * 16 + (lane & 15);
    const int ci = chunk * kc + ks * 32 + 8 * (lane >> 4) + e;
    Wf[gidx] = ci < cin ? W[((int64_t)n * cin + ci) * cout + co] : (_Float16)0;
}

// ---- explicit dataflow ------------------------------------------------------------------------
// Gather (Alg. 2, "F[m] <- X_in[j]") for all offsets: a thread moves kGatherPer 16-byte vectors,
// one each of rows a workgroup-stride apart, all loaded before the first store.  F is written
// once and read once by the matmul, so its stores bypass the caches and leave them to X, every row
// of which is gathered several times.
constexpr int kGatherPer = 2;
__global__ void __launch_bounds__(kThreads) k_gather(const u32x4 *__restrict__ X, const int32_t *__restrict__ in_idx,
                                                     u32x4 *__restrict__ F, int64_t M, int vec_per_row, int64_t skip_lo,
                                                     int64_t skip_hi) {
    const int64_t base = (int64_t)blockIdx.x * (kThreads * kGatherPer) + threadIdx.x;
    u32x4 v[kGatherPer];
    int64_t at[kGatherPer];
#pragma unroll
    for (int u = 0; u < kGatherPer; ++u) {
        const int64_t g = base + (int64_t)u * kThreads;
        const int64_t p = g / vec_per_row;
        const int c = (int)(g - p * vec_per_row);
        at[u] = (p < M && !(p >= skip_lo && p < skip_hi)) ? g : -1;
        if (at[u] >= 0) v[u] = X[(int64_t)in_idx[p] * vec_per_row + c];
    }
#pragma unroll
    for (int u = 0; u < kGatherPer; ++u)
        if (at[u] >= 0) __builtin_nontemporal_store(v[u], &F[at[u]]);
}

// The same gather in input-stationary order (the locality-aware order of Sec. 4.3.2: an input row is read
// once and written to every place it is needed), for 3x3x3 stride-1 maps.  VPR lanes share an input row j
// and hold 16 bytes of it each.  By the symmetry of Sec. 4.2.1 row j of the out-major table also lists
// where j is an input: nbr[j][n'] = k means input j feeds output k through offset n = 26 - n', and that
// pair's row in F is offs[n] + (rank of k among the outputs with offset n), read off the rank bitmaps.
// The lanes of a group first work out those rows for the offsets they own (n' = c, c + VPR, ...), all
// lookups in flight together, then the group walks the 27 offsets and stores.  Reads X sequentially and
// once; F's rows are written whole but scattered.  Centre rows are left out, as in k_gather.
template <int VPR>
__global__ void __launch_bounds__(kThreads) k_gather_in(const u32x4 *__restrict__ X, const int32_t *__restrict__ nbr,
                                                        const uint64_t *__restrict__ colbits,
                                                        const int32_t *__restrict__ colbase, Offs offs, int64_t n_blocks,
                                                        u32x4 *__restrict__ F, int64_t n_in) {
    constexpr int K3 = 27, STRIDE = 32, PER = (K3 + VPR - 1) / VPR;
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t j = t / VPR;
    const int c = (int)(t % VPR), lane = threadIdx.x & 63, first = lane - c;   // first: the group's lane 0
    const bool ok = j < n_in;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (ok) v = X[j * VPR + c];
    int32_t pos[PER];
#pragma unroll
    for (int r = 0; r < PER; ++r) {
        const int np = c + r * VPR;     // this lane's offset n' of row j
        pos[r] = -1;
        if (ok && np < K3 && np != K3 / 2) {
            const int32_t k = nbr[j * STRIDE + np];
            if (k >= 0) {
                const int n = K3 - 1 - np;
                const int64_t b = (int64_t)n * n_blocks + (k >> 6);
                pos[r] = offs.v[n] + colbase[b] + __popcll(colbits[b] & ((1ull << (k & 63)) - 1ull));
            }
        }
    }
#pragma unroll
    for (int np = 0; np < K3; ++np) {
        const int32_t p = __shfl(pos[np / VPR], first + np % VPR, 64);
        if (p >= 0) __builtin_nontemporal_store(v, &F[(int64_t)p * VPR + c]);
    }
}

// One launch of the grouped matmul: the offsets it covers and how many 128-row blocks each gets.
// An offset given more blocks than its list fills stands for a list padded to a longer one
// (the batched matmul of Appendix B, Alg. 4): the surplus blocks multiply zero rows and store nothing.
struct MmPlan {
    int32_t count;
    int32_t n[kMaxK3];
    int32_t tiles[kMaxK3];
};

// Grouped matmul: block -> (offset n, 128-row block) by walking the plan's block counts.
// Rows of the centre offset of an identity map come from X itself.  Rows past the end of an
// offset's list read `zero_row` and are not stored.
template <class T, int NCB, int KC>
__global__ void __launch_bounds__(kThreads) k_grouped_mm(const T *__restrict__ F, const T *__restrict__ X,
                                                         const T *__restrict__ Wt, Offs offs, MmPlan plan,
                                                         float *__restrict__ G, const T *__restrict__ zero_row,
                                                         int cin, int cout, int centre,
                                                         const int32_t *__restrict__ in_idx,
                                                         const T *__restrict__ X2, int cin1) {
    // X2 != nullptr (rows fetched through the map only: F is not used then): the input is the channel
    // concatenation [X | X2], never formed; channels below cin1 come from X, the others from X2.
    typedef Shape<T, NCB, KC> S;
    typedef typename S::vec vec;
    __shared__ __attribute__((aligned(16))) T lds_w[S::SLAB];
    int t = blockIdx.x, i = 0;
    for (; i < plan.count; ++i) {
        if (t < plan.tiles[i]) break;
        t -= plan.tiles[i];
    }
    if (i >= plan.count) return;
    const int n = plan.n[i];
    const int lo = offs.v[n], hi = offs.v[n + 1];
    const int co0 = blockIdx.y * NCB * 32;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, m = lane & 31, h = lane >> 5;
    const int64_t p = (int64_t)lo + (int64_t)t * kTileRows + wave * kWaveRows + m;   // row of F and G
    const bool valid = p < hi;
    const int64_t j = !valid ? 0 : (n == centre ? p - lo : (in_idx ? (int64_t)in_idx[p] : p));
    const T *src = !valid ? zero_row : ((n == centre || in_idx) ? X + j * cin1 : F + p * cin);
    const T *src2 = (!valid || !X2) ? zero_row : X2 + j * (cin - cin1) - cin1;   // indexed with k0 >= cin1
    const int kstride = valid ? 1 : 0;   // the zero row is one chunk long
    floatx16 acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
        for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;
    vec wreg[S::WV], bx[S::NKB];
    for (int k0 = 0; k0 < cin; k0 += KC) {
        load_w_regs<S, T>(wreg, Wt, n, co0, k0, cin, cout);
        load_x_regs<S, T>(bx, (k0 < cin1 ? src : src2) + k0 * kstride + h * S::VEC);
        __syncthreads();
        store_w_regs<S, T>(wreg, lds_w);
        __syncthreads();
        mma_stage<S, T, NCB>(lds_w, bx, acc);
    }
    store_rows<float, NCB>(G, valid ? p : -1, cout, co0, acc);
}

// Scatter-accumulate, output-stationary: thread = (output row, 4 channels); partial sums are
// added in offset order in fp32 registers and the row is written once.  The row of G that holds
// the pair (k, n) follows from the offset's start, the base of k's 64-row block and the block's
// presence bitmap.
template <class T>
__global__ void __launch_bounds__(kThreads) k_scatter_reduce(const float *__restrict__ G, const int32_t *__restrict__ nbr,
                                                             int stride, const uint64_t *__restrict__ colbits,
                                                             const int32_t *__restrict__ colbase, Offs offs,
                                                             int64_t n_blocks,
                                                             T *__restrict__ out, int64_t n_out, int cout, int K3,
                                                             const T *__restrict__ bias, const T *__restrict__ residual,
                                                             int relu) {
    const int quads = cout / 4;
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t k = g / quads;
    int q = (int)(g - k * quads);
    if (k >= n_out) return;
    uint32_t mask = (uint32_t)nbr[k * stride + K3];
    const int64_t b = k >> 6;
    const uint64_t before = (1ull << (k & 63)) - 1ull;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    // four offsets at a time: their positions first, then their rows of G (read once: streamed
    // past the caches), then the adds in offset order
    while (mask) {
        int64_t p[4];
        floatx4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            p[u] = -1;
            if (mask) {
                const int n = __builtin_ctz(mask);
                mask &= mask - 1;
                p[u] = offs.v[n] + colbase[n * n_blocks + b] + __popcll(colbits[n * n_blocks + b] & before);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (p[u] >= 0) v[u] = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(G + p[u] * cout + q * 4));
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (p[u] >= 0) acc += v[u];
    }
    // the layer's own result in T, then, if asked for, what ts_bias_act would do with it: fp32 sum
    // (bias first, then the residual), ReLU, one rounding
    const int64_t at = k * cout + q * 4;
    const bool tail = bias || residual || relu;
    if constexpr (sizeof(T) == 2) {
        half4 v = {(_Float16)acc[0], (_Float16)acc[1], (_Float16)acc[2], (_Float16)acc[3]};
        if (tail) {
            float f[4] = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
            if (bias) {
                const half4 b = *reinterpret_cast<const half4 *>(bias + q * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) f[e] += (float)b[e];
            }
            if (residual) {
                const half4 r = *reinterpret_cast<const half4 *>(residual + at);
#pragma unroll
                for (int e = 0; e < 4; ++e) f[e] += (float)r[e];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (_Float16)(relu && f[e] < 0.f ? 0.f : f[e]);
        }
        *reinterpret_cast<half4 *>(out + at) = v;
    } else {
        if (tail) {
            if (bias) acc += *reinterpret_cast<const floatx4 *>(bias + q * 4);
            if (residual) acc += *reinterpret_cast<const floatx4 *>(residual + at);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = relu && acc[e] < 0.f ? 0.f : acc[e];
        }
        *reinterpret_cast<floatx4 *>(out + at) = acc;
    }
}

// ---- operand preparation ----------------------------------------------------------------------
// Wt[n][co][ci'] = W[n][ci'][co] for ci' < cin, 0 for cin <= ci' < cin_pad.
template <class T>
__global__ void k_pack_weights(const T *__restrict__ W, T *__restrict__ Wt, int K3, int cin, int cin_pad, int cout) {
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)K3 * cout * cin_pad;
    if (g >= total) return;
    int ci = (int)(g % cin_pad);
    int co = (int)((g / cin_pad) % cout);
    int n = (int)(g / ((int64_t)cin_pad * cout));
    Wt[g] = ci < cin ? W[((int64_t)n * cin + ci) * cout + co] : (T)0;
}

// Xp[row][c] = X[row][c] for c < cin, 0 up to cin_pad.
// A thread writes 8 consecutive elements of a padded row (cin_pad is a multiple of 8) with 16-byte stores.
template <class T>
__global__ void k_pad_rows(const T *__restrict__ X, T *__restrict__ Xp, int64_t rows, int cin, int cin_pad) {
    const int per_row = cin_pad / 8;
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= rows * per_row) return;
    int64_t r = g / per_row;
    const int c0 = (int)(g - r * per_row) * 8;
    T v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = c0 + e < cin ? X[r * cin + c0 + e] : (T)0;
    u32x4 raw[sizeof(T) / 2];
    __builtin_memcpy(raw, v, sizeof(v));
    u32x4 *dst = reinterpret_cast<u32x4 *>(Xp + r * cin_pad + c0);
#pragma unroll
    for (unsigned i = 0; i < sizeof(T) / 2; ++i) dst[i] = raw[i];
}

inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }
inline size_t elem_size(int dtype) { return dtype == TS_F16 ? 2 : 4; }
inline int kstep(int dtype) { return dtype == TS_F16 ? Elem<_Float16>::KSTEP : Elem<float>::KSTEP; }

// Output-channel blocks of 32 handled by one workgroup: the largest of 4,3,2,1 dividing cout/32.
inline int pick_ncb(int cout) {
    int blocks = cout / 32;
    for (int ncb = 4; ncb >= 1; --ncb)
        if (blocks % ncb == 0) return ncb;
    return 1;
}

}  // namespace

// Weights of one layer in the layouts the kernels read (ts_weights_prepare); device memory owned
// by the object.
struct ts_weights {
    int K3 = 0, cin = 0, cout = 0, dtype = 0;
    void *wt = nullptr;     // [K3][cout][cin rounded up to the operand step], for k_fused / k_grouped_mm
    void *tile = nullptr;   // fp16: operand order of k_conv_tile (see k_pack_weights_tile)
};

namespace {

struct Prepared {
    const void *x;    // features, rows padded to cin_pad channels
    const void *wt;   // transposed, padded weights
    int cin_pad;
};

int check_tensor(const ts_tensor *t, const char *name) {
    if (!t) return fail(TS_ERR_INVALID_ARG, "%s is NULL", name);
    if (t->dtype != TS_F32 && t->dtype != TS_F16) return fail(TS_ERR_INVALID_ARG, "%s: unknown dtype %d", name, t->dtype);
    if (t->rows < 0 || t->cols <= 0) return fail(TS_ERR_SHAPE, "%s: bad shape [%lld, %d]", name, (long long)t->rows, t->cols);
    if (t->rows > 0 && !t->data) return fail(TS_ERR_INVALID_ARG, "%s: data is NULL", name);
    if (reinterpret_cast<uintptr_t>(t->data) & 15) return fail(TS_ERR_INVALID_ARG, "%s: data must be 16-byte aligned", name);
    return TS_OK;
}

int check_layer(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, const ts_tensor *out) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    if (kmap->pending_slot < 0 && kmap->error != TS_OK) return resolve(kmap);   // a map whose build found bad input
    TS_TRY(check_tensor(feats, "feats"));
    TS_TRY(check_tensor(weights, "weights"));
    TS_TRY(check_tensor(out, "out"));
    if (feats->dtype != weights->dtype || feats->dtype != out->dtype)
        return fail(TS_ERR_SHAPE, "feats, weights and out must share one dtype");
    if (feats->rows != kmap->n_in) return fail(TS_ERR_SHAPE, "feats has %lld rows, the map expects %lld", (long long)feats->rows, (long long)kmap->n_in);
    if (out->rows != kmap->n_out) return fail(TS_ERR_SHAPE, "out has %lld rows, the map produces %lld", (long long)out->rows, (long long)kmap->n_out);
    if (weights->rows != (int64_t)kmap->K3 * feats->cols)
        return fail(TS_ERR_SHAPE, "weights must be [K^3*C_in, C_out] = [%lld, .], got %lld rows", (long long)kmap->K3 * feats->cols, (long long)weights->rows);
    if (weights->cols != out->cols) return fail(TS_ERR_SHAPE, "weights has %d columns, out has %d", weights->cols, out->cols);
    if (out->cols % 32 != 0 || out->cols > 1024) return fail(TS_ERR_UNSUPPORTED, "C_out must be a multiple of 32 (<= 1024), got %d", out->cols);
    if (feats->cols > 1024) return fail(TS_ERR_UNSUPPORTED, "C_in must be <= 1024, got %d", feats->cols);
    return TS_OK;
}

// Transpose/pad the weights into scratch, and pad the features when C_in is not a multiple of
// the operand step.
template <class T>
int prepare(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, Prepared *pr,
            const ts_weights *pw = nullptr, void *wbuf = nullptr) {
    const int cin = feats->cols, cout = weights->cols, ks = Elem<T>::KSTEP;
    const int cin_pad = (cin + ks - 1) / ks * ks;
    pr->cin_pad = cin_pad;
    if (wbuf && cin_pad != cin) return fail(TS_ERR_UNSUPPORTED, "C_in must be a multiple of %d here", ks);
    if (pw) {
        pr->wt = pw->wt;
    } else {
        size_t wn = (size_t)kmap->K3 * cout * cin_pad;
        T *wt = static_cast<T *>(wbuf ? wbuf : scratch(2, wn * sizeof(T)));
        if (!wt) return last_fail_code();
        TS_LAUNCH("k_pack_weights", k_pack_weights<T>, dim3(blocks_for((int64_t)wn, kThreads)), dim3(kThreads), static_cast<const T *>(weights->data), wt, kmap->K3, cin, cin_pad, cout);
        pr->wt = wt;
    }
    pr->x = feats->data;
    if (cin_pad != cin && feats->rows > 0) {
        size_t xn = (size_t)feats->rows * cin_pad;
        T *xp = static_cast<T *>(scratch(3, xn * sizeof(T)));
        if (!xp) return last_fail_code();
        TS_LAUNCH("k_pad_rows", k_pad_rows<T>, dim3(blocks_for((int64_t)xn / 8, kThreads)), dim3(kThreads), static_cast<const T *>(feats->data), xp, feats->rows, cin, cin_pad);
        pr->x = xp;
    }
    return TS_OK;
}

// Largest chunk of {8,4,2} operand steps (KC = 64/32/16 for fp16, 32/16/8 for fp32) that divides cin.
inline int pick_ksteps(int cin, int kstep_elems) {
    int steps = cin / kstep_elems;
    if (steps % 4 == 0) return 4;
    if (steps % 2 == 0) return 2;
    return 1;
}

// Run `fn.template operator()<NCB, KSTEPS>()` for the runtime pair (ncb, ksteps).
template <class Fn>
void dispatch_shape(int ncb, int ksteps, Fn &&fn) {
#define TS_CASE(N, K)                     \
    if (ncb == N && ksteps == K) {        \
        fn.template operator()<N, K>();   \
        return;                           \
    }
    TS_CASE(1, 1) TS_CASE(1, 2) TS_CASE(1, 4) TS_CASE(2, 1) TS_CASE(2, 2) TS_CASE(2, 4)
    TS_CASE(3, 1) TS_CASE(3, 2) TS_CASE(3, 4) TS_CASE(4, 1) TS_CASE(4, 2) TS_CASE(4, 4)
#undef TS_CASE
}

// (offset, chunk) pairs per pipeline stage of k_fused: narrow shapes have little MFMA work
// per pair, so several are batched between barriers to shorten the chain of memory latencies.
constexpr int fused_group(int ncb, int ksteps) {
    return ncb * ksteps <= 2 ? 4 : (ncb * ksteps <= 8 ? 3 : 1);
}

template <class T>
struct FusedLaunch {
    const Prepared &pr;
    const ts_kmap *kmap;
    ts_tensor *out;
    const T *zero;
    template <int NCB, int KSTEPS>
    void operator()() const {
        constexpr int KC = KSTEPS * Elem<T>::KSTEP;
        constexpr int G = fused_group(NCB, KSTEPS);
        dim3 grid((unsigned)kmap->n_tiles, out->cols / (NCB * 32));
        TS_LAUNCH("k_fused", (k_fused<T, NCB, KC, G>), grid, dim3(kThreads), static_cast<const T *>(pr.x),
                  static_cast<const T *>(pr.wt), kmap->d_nbr, kmap->stride, kmap->d_perm, kmap->n_out,
                  static_cast<T *>(out->data), zero, pr.cin_pad, out->cols, kmap->K3, kmap->centre);
    }
};

template <class T>
int run_fused_staged(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, ts_tensor *out,
                     const ts_weights *pw = nullptr, void *wbuf = nullptr, const void *zeros = nullptr) {
    Prepared pr;
    TS_TRY(prepare<T>(feats, weights, kmap, &pr, pw, wbuf));
    const T *zero = static_cast<const T *>(zeros ? zeros : zero_row());
    if (!zero) return last_fail_code();
    dispatch_shape(pick_ncb(out->cols), pick_ksteps(pr.cin_pad, Elem<T>::KSTEP), FusedLaunch<T>{pr, kmap, out, zero});
    TS_HIP(hipGetLastError());
    return TS_OK;
}

constexpr int kTileDepth = 3;

// What follows the layer's sum, if anything: y = act(conv + bias + residual) (see ts_sparse_conv_act).
struct Epilogue {
    const void *bias = nullptr;
    const void *residual = nullptr;
    int relu = 0;
    bool any() const { return bias || residual || relu; }
};

inline int compute_units() {
    static int n = 0;
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n = prop.multiProcessorCount;
        if (n <= 0) n = 256;
    }
    return n;
}

// The second half of a layer input that is the channel concatenation [x | x2] of two tensors (never
// formed): x has cin1 channels per row, x2 the rest.  x2 == nullptr: one tensor, as usual.
struct Second {
    const void *x2 = nullptr;
    int cin1 = 0;
};

template <int NCO, int KSTEPS, bool TWO = false>
void launch_conv_tile(const _Float16 *x, const _Float16 *wf, const ts_kmap *kmap, ts_tensor *out, int cin_pad,
                      const Epilogue &ep, const Second &sec = Second()) {
    // as many workgroups as stay resident at once, fewer for small maps
    static int per_cu = 0;   // per instantiation
    if (per_cu == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_conv_tile<NCO, KSTEPS, kTileDepth, TWO>, kThreads, 0) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            n = 2;
        }
        per_cu = n;
    }
    const int64_t resident = (int64_t)compute_units() * per_cu;
    dim3 grid((unsigned)(kmap->n_tiles < resident ? kmap->n_tiles : resident), out->cols / (NCO * 16));
    const int cin1 = TWO ? sec.cin1 : cin_pad;
    TS_LAUNCH("k_conv_tile", (k_conv_tile<NCO, KSTEPS, kTileDepth, TWO>), grid, dim3(kThreads), x,
              reinterpret_cast<const u32x4 *>(wf), kmap->d_nbr, kmap->stride, kmap->d_perm, kmap->rows_done ? kmap->d_tile_order : nullptr,
              kmap->n_out, static_cast<_Float16 *>(out->data), kmap->d_sched, cin_pad, out->cols, kmap->K3,
              static_cast<const _Float16 *>(ep.bias), static_cast<const _Float16 *>(ep.residual), ep.relu,
              (int)((size_t)kmap->n_in * cin1 * 2), (int)((size_t)kmap->K3 * cin_pad * out->cols * 2), kmap->centre,
              static_cast<const _Float16 *>(sec.x2), (int)((size_t)kmap->n_in * (cin_pad - cin1) * 2), cin1);
}

// Narrow layers (C_in <= 32, C_out = 32): the kernel that keeps all weights in LDS.  False if this
// device does not give a workgroup that much LDS: the caller then takes k_conv_tile.
template <int NCO, int KSTEPS>
bool launch_conv_res(const _Float16 *x, const _Float16 *wf, const ts_kmap *kmap, ts_tensor *out, const Epilogue &ep) {
    static int usable = -1;   // per instantiation
    constexpr size_t lds = res_lds_bytes<NCO * KSTEPS>();
    if (usable < 0) {
        usable = hipFuncSetAttribute(reinterpret_cast<const void *>(k_conv_res<NCO, KSTEPS, kResDepth>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
        if (!usable) (void)hipGetLastError();
    }
    if (!usable) return false;
    const int64_t n_units = (kmap->n_out + kResRows - 1) / kResRows;
    const int64_t wgs = (n_units + kResWaves - 1) / kResWaves;
    const int64_t cus = compute_units();
    TS_LAUNCH_SHM("k_conv_res", (k_conv_res<NCO, KSTEPS, kResDepth>), dim3((unsigned)(wgs < cus ? wgs : cus), out->cols / (NCO * 16)), dim3(kResThreads), lds,
                       x, reinterpret_cast<const u32x4 *>(wf), kmap->d_nbr, kmap->stride, kmap->d_perm, kmap->n_out,
                       static_cast<_Float16 *>(out->data), kmap->d_sched, kmap->K3, out->cols, static_cast<const _Float16 *>(ep.bias),
                       static_cast<const _Float16 *>(ep.residual), ep.relu, (int)((size_t)kmap->n_in * KSTEPS * 64), kmap->centre);
    return true;
}

// fp16: input channels padded to a multiple of 32 (one MFMA step), chunks of 64 where possible.
// feats->cols is the layer's C_in; with sec.x2 set, feats->data holds only the first sec.cin1 channels of
// every row (both parts multiples of 32 channels: nothing is padded then).
int run_fused_f16(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, ts_tensor *out,
                  const Epilogue &ep, const ts_weights *pw = nullptr, void *wbuf = nullptr, const Second &sec = Second()) {
    typedef _Float16 T;
    const int cin = feats->cols, cout = out->cols;
    const int cin_pad = (cin + 31) / 32 * 32;
    const int ksteps = cin_pad % 64 == 0 ? 2 : 1;
    // the kernel addresses features and weights with 31-bit byte offsets
    if ((size_t)kmap->n_in * cin_pad * 2 >= (1ull << 31) || (size_t)kmap->K3 * cin_pad * cout * 2 >= (1ull << 31)) {
        if (ep.any()) return fail(TS_ERR_UNSUPPORTED, "feature matrix of 2 GiB or more: call ts_sparse_conv and ts_bias_act");
        if (wbuf) return fail(TS_ERR_UNSUPPORTED, "feature matrix of 2 GiB or more");
        return run_fused_staged<_Float16>(feats, weights, kmap, out, pw);
    }
    if (wbuf && cin_pad != cin) return fail(TS_ERR_UNSUPPORTED, "C_in must be a multiple of 32 here");
    const T *wf = pw ? static_cast<const T *>(pw->tile) : nullptr;
    if (!wf) {
        const size_t wn = (size_t)kmap->K3 * cout * cin_pad;
        T *buf = static_cast<T *>(wbuf ? wbuf : scratch(2, wn * sizeof(T)));
        if (!buf) return last_fail_code();
        TS_LAUNCH("k_pack_weights", k_pack_weights_tile, dim3(blocks_for((int64_t)wn, kThreads)), dim3(kThreads),
                  static_cast<const T *>(weights->data), buf, kmap->K3, cin, cin_pad, cout, ksteps);
        wf = buf;
    }
    const T *x = static_cast<const T *>(feats->data);
    if (cin_pad != cin) {
        const size_t xn = (size_t)feats->rows * cin_pad;
        T *xp = static_cast<T *>(scratch(3, xn * sizeof(T)));
        if (!xp) return last_fail_code();
        TS_LAUNCH("k_pad_rows", k_pad_rows<T>, dim3(blocks_for((int64_t)xn / 8, kThreads)), dim3(kThreads), x, xp, feats->rows, cin, cin_pad);
        x = xp;
    }
    const int cblocks = cout / 16;
    // 32 input channels and 27 offsets: the kernel with resident weights (for 2x2x2 maps and for 64 -> 32 it
    // measured no faster than k_conv_tile, and 64 -> 64 in two slices of output channels much slower: every
    // slice gathers all rows again)
    if (cin_pad == 32 && kmap->K3 > 8 && kmap->n_out > 0 && (cout == 32 || cout == 64) && !sec.x2) {
        const bool done = cout == 32 ? launch_conv_res<2, 1>(x, wf, kmap, out, ep) : launch_conv_res<4, 1>(x, wf, kmap, out, ep);
        if (done) {
            TS_HIP(hipGetLastError());
            return TS_OK;
        }
    }
    // Output channels per workgroup: as many as divide C_out (every slice gathers the rows again), fewer
    // when the launch would leave most of the chip idle: a lone workgroup per CU walks its stages one
    // after the other, and a stage of eight output blocks takes twice as long as one of four.
    int nco = 2, cap = 8;
    const int64_t cus = compute_units(), wgs8 = kmap->n_tiles * ((cblocks + 7) / 8);
    if (wgs8 <= cus / 2 || (wgs8 <= cus && kmap->K3 > 8)) cap = 4;
    if (cap == 4 && kmap->n_tiles * ((cblocks + 3) / 4) <= cus / 2) cap = 2;
    for (int c : {8, 6, 4, 2})
        if (c <= cap && cblocks % c == 0) {
            nco = c;
            break;
        }
#define TS_TILE_CASE(N)                                                                            \
    if (nco == N) {                                                                                \
        if (sec.x2) {                                                                              \
            if (ksteps == 2) launch_conv_tile<N, 2, true>(x, wf, kmap, out, cin_pad, ep, sec);    \
            else launch_conv_tile<N, 1, true>(x, wf, kmap, out, cin_pad, ep, sec);                \
        } else if (ksteps == 2) launch_conv_tile<N, 2>(x, wf, kmap, out, cin_pad, ep);            \
        else launch_conv_tile<N, 1>(x, wf, kmap, out, cin_pad, ep);                                \
    }
    TS_TILE_CASE(8) TS_TILE_CASE(6) TS_TILE_CASE(4) TS_TILE_CASE(2)
#undef TS_TILE_CASE
    static_assert(1024 / 32 <= kMaxSchedSlices, "C_out <= 1024 in slices of at least 32 channels");
    TS_HIP(hipGetLastError());
    return TS_OK;
}

template <class T>
int run_fused(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, ts_tensor *out,
              const ts_weights *pw = nullptr) {
    if constexpr (sizeof(T) == 2) return run_fused_f16(feats, weights, kmap, out, Epilogue(), pw);
    return run_fused_staged<T>(feats, weights, kmap, out, pw);
}

int64_t mm_tiles(int64_t rows) { return (rows + kTileRows - 1) / kTileRows; }

// Every offset with the blocks its own list needs: no padding, one launch.
MmPlan whole_plan(const ts_kmap *kmap) {
    MmPlan plan;
    plan.count = 0;
    for (int n = 0; n < kmap->K3; ++n) {
        if (kmap->sizes[n] == 0) continue;
        plan.n[plan.count] = n;
        plan.tiles[plan.count++] = (int32_t)mm_tiles(kmap->sizes[n]);
    }
    return plan;
}

int64_t plan_tiles(const MmPlan &plan) {
    int64_t t = 0;
    for (int i = 0; i < plan.count; ++i) t += plan.tiles[i];
    return t;
}

template <class T>
struct GroupedLaunch {
    const T *F, *X, *wt;
    const ts_kmap *kmap;
    MmPlan plan;
    float *G;
    const T *zero;
    int cin_pad, cout;
    const int32_t *in_idx;
    const T *X2;
    int cin1;
    template <int NCB, int KSTEPS>
    void operator()() const {
        constexpr int KC = KSTEPS * Elem<T>::KSTEP;
        dim3 grid((unsigned)plan_tiles(plan), cout / (NCB * 32));
        TS_LAUNCH("k_grouped_mm", (k_grouped_mm<T, NCB, KC>), grid, dim3(kThreads), F, X, wt, offs_of(kmap), plan, G, zero,
                  cin_pad, cout, kmap->centre, in_idx, X2, cin1);
    }
};

// order: 0 = the library's choice, 1 = output order (k_gather), 2 = input-stationary (k_gather_in) where it applies.
int gather_impl(const void *x, int64_t /*rows*/, int cin_pad, int dtype, const ts_kmap *kmap, void *F, int order = 0) {
    if (kmap->M == 0) return TS_OK;
    const int vec_per_row = (int)(cin_pad * elem_size(dtype) / 16);
    // Input-stationary order reads every input row once instead of once per pair, and writes whole rows of F
    // at scattered places.  Measured on the LiDAR-like scene at 153 k, 1.5 M and 15 M points: with rows of 128
    // bytes or more it wins at every size (C = 64: 31 against 35 us at 153 k, 3.0 against 4.4 ms at 15 M;
    // C = 128: 51 against 67 us, 5.4 against 8.8 ms); with 64-byte rows (half a cache line per scattered
    // write) only once the feature matrix no longer fits the 256 MB last-level cache.
    const bool can_in = kmap->K3 == 27 && kmap->centre >= 0 && kmap->stride == 32 &&
                        (vec_per_row == 4 || vec_per_row == 8 || vec_per_row == 16 || vec_per_row == 32) &&
                        kmap->M < (int64_t)1 << 31;
    const size_t x_bytes = (size_t)kmap->n_in * vec_per_row * 16;
    if (can_in && (order == 2 || (order == 0 && (vec_per_row >= 8 || x_bytes > ((size_t)256 << 20))))) {
        TS_TRY(resolve(kmap));
        const int64_t threads = kmap->n_in * vec_per_row;
        const dim3 grid(blocks_for(threads, kThreads)), block(kThreads);
        const u32x4 *xs = static_cast<const u32x4 *>(x);
        u32x4 *fs = static_cast<u32x4 *>(F);
#define TS_GATHER_IN(V) TS_LAUNCH("k_gather_in", k_gather_in<V>, grid, block, xs, kmap->d_nbr, kmap->d_colbits, kmap->d_colbase, offs_of(kmap), kmap->n_blocks, fs, kmap->n_in)
        if (vec_per_row == 4) TS_GATHER_IN(4);
        else if (vec_per_row == 8) TS_GATHER_IN(8);
        else if (vec_per_row == 16) TS_GATHER_IN(16);
        else TS_GATHER_IN(32);
#undef TS_GATHER_IN
        TS_HIP(hipGetLastError());
        return TS_OK;
    }
    TS_TRY(ensure_pairs(kmap));
    int64_t lo = 0, hi = 0;
    if (kmap->centre >= 0) {
        lo = kmap->offs[kmap->centre];
        hi = kmap->offs[kmap->centre + 1];
    }
    TS_LAUNCH("k_gather", k_gather, dim3(blocks_for(kmap->M * vec_per_row, kThreads * kGatherPer)), dim3(kThreads), static_cast<const u32x4 *>(x), kmap->d_in_idx, static_cast<u32x4 *>(F), kmap->M, vec_per_row, lo, hi);
    TS_HIP(hipGetLastError());
    return TS_OK;
}

template <class T>
int grouped_mm_launch(const void *F, const void *X, const void *wt, const ts_kmap *kmap, const MmPlan &plan, float *G,
                      int cin_pad, int cout, const int32_t *in_idx = nullptr, const Second &sec = Second()) {
    if (plan_tiles(plan) == 0) return TS_OK;
    const T *zero = static_cast<const T *>(zero_row());
    if (!zero) return last_fail_code();
    // the chunk of input channels a step takes must divide both parts of a two-part input
    int ksteps = pick_ksteps(cin_pad, Elem<T>::KSTEP);
    const int cin1 = sec.x2 ? sec.cin1 : cin_pad;
    if (sec.x2) {
        const int k1 = pick_ksteps(cin1, Elem<T>::KSTEP), k2 = pick_ksteps(cin_pad - cin1, Elem<T>::KSTEP);
        ksteps = k1 < k2 ? k1 : k2;
    }
    dispatch_shape(pick_ncb(cout), ksteps,
                   GroupedLaunch<T>{static_cast<const T *>(F), static_cast<const T *>(X), static_cast<const T *>(wt),
                                    kmap, plan, G, zero, cin_pad, cout, in_idx, static_cast<const T *>(sec.x2), cin1});
    TS_HIP(hipGetLastError());
    return TS_OK;
}

template <class T>
int grouped_mm_impl(const void *F, const void *X, const void *wt, const ts_kmap *kmap, float *G, int cin_pad,
                    int cout) {
    return grouped_mm_launch<T>(F, X, wt, kmap, whole_plan(kmap), G, cin_pad, cout);
}

// Consecutive indices are grouped while the padded share of the group, 1 - n_min / n_max, stays within
// epsilon (Appendix B, Alg. 4, first loop).  group_of[i] = number of the group index i falls in.
int partition_by_size(const int64_t *sizes, int count, double epsilon, int32_t *group_of) {
    int groups = 0;
    for (int first = 0; first < count;) {
        int64_t lo = sizes[first], hi = sizes[first];
        int next = first + 1;
        for (; next < count; ++next) {
            const int64_t l = sizes[next] < lo ? sizes[next] : lo, h = sizes[next] > hi ? sizes[next] : hi;
            const double padded = h == 0 ? 0.0 : 1.0 - (double)l / (double)h;
            if (padded > epsilon) break;
            lo = l;
            hi = h;
        }
        for (int i = first; i < next; ++i) group_of[i] = groups;
        ++groups;
        first = next;
    }
    return groups;
}

// The grouped matmul the way Appendix B, Alg. 4 schedules it: per group one batched launch with every
// member padded to the longest when that length is below S, else one launch per member.  With an odd
// kernel at stride 1 index i and its mirror K^3-1-i have maps of one size and always share a launch
// (symmetric grouping, Sec. 4.2.3), the groups are formed over the first half of the indices, and the
// centre is a launch of its own.  epsilon < 0: no grouping at all, one launch per offset.
template <class T>
int grouped_mm_adaptive(const void *F, const void *X, const void *wt, const ts_kmap *kmap, float *G, int cin_pad, int cout,
                        double epsilon, int64_t S, int64_t *stats) {
    const int K3 = kmap->K3;
    const bool mirrored = kmap->centre >= 0 && epsilon >= 0;
    const int count = mirrored ? K3 / 2 : K3;
    int32_t group_of[kMaxK3];
    int groups;
    if (epsilon < 0) {
        for (int i = 0; i < count; ++i) group_of[i] = i;
        groups = count;
    } else {
        groups = partition_by_size(kmap->sizes, count, epsilon, group_of);
    }
    int64_t launches = 0, padded_rows = 0;
    auto launch = [&](const MmPlan &plan) -> int {
        if (plan_tiles(plan) == 0) return TS_OK;
        ++launches;
        return grouped_mm_launch<T>(F, X, wt, kmap, plan, G, cin_pad, cout);
    };
    auto add = [&](MmPlan &plan, int n, int64_t rows) {
        plan.n[plan.count] = n;
        plan.tiles[plan.count++] = (int32_t)mm_tiles(rows);
        padded_rows += rows;
    };
    for (int g = 0, first = 0; g < groups; ++g) {
        int next = first;
        int64_t n_max = 0;
        for (; next < count && group_of[next] == g; ++next) n_max = kmap->sizes[next] > n_max ? kmap->sizes[next] : n_max;
        const bool batched = n_max < S;
        MmPlan plan;
        plan.count = 0;
        for (int i = first; i < next; ++i) {
            if (!batched) plan.count = 0;
            const int64_t rows = batched ? n_max : kmap->sizes[i];
            add(plan, i, rows);
            if (mirrored) add(plan, K3 - 1 - i, rows);
            if (!batched) TS_TRY(launch(plan));
        }
        if (batched) TS_TRY(launch(plan));
        first = next;
    }
    if (mirrored) {
        MmPlan plan;
        plan.count = 0;
        add(plan, kmap->centre, kmap->sizes[kmap->centre]);
        TS_TRY(launch(plan));
    }
    if (stats) {
        stats[0] = launches;
        stats[1] = groups;
        stats[2] = padded_rows;
        stats[3] = kmap->M;
    }
    return TS_OK;
}

template <class T>
int reduce_impl(const float *G, const ts_kmap *kmap, ts_tensor *out, const Epilogue &ep = Epilogue()) {
    if (kmap->n_out == 0) return TS_OK;
    int64_t threads = kmap->n_out * (out->cols / 4);
    TS_LAUNCH("k_scatter_reduce", k_scatter_reduce<T>, dim3(blocks_for(threads, kThreads)), dim3(kThreads), G, kmap->d_nbr, kmap->stride, kmap->d_colbits, kmap->d_colbase, offs_of(kmap), kmap->n_blocks, static_cast<T *>(out->data), kmap->n_out, out->cols, kmap->K3, static_cast<const T *>(ep.bias), static_cast<const T *>(ep.residual), ep.relu);
    TS_HIP(hipGetLastError());
    return TS_OK;
}

template <class T>
int run_explicit(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, ts_tensor *out,
                 const ts_weights *pw = nullptr, bool fetch = false, const Epilogue &ep = Epilogue(),
                 const Second &sec = Second()) {
    TS_TRY(resolve(kmap));
    Prepared pr;
    TS_TRY(prepare<T>(feats, weights, kmap, &pr, pw));
    if (sec.x2 && (!fetch || pr.cin_pad != feats->cols)) return fail(TS_ERR_UNSUPPORTED, "a two-part input needs the fetch-on-demand dataflow and unpadded rows");
    const int64_t M = kmap->M;
    float *G = static_cast<float *>(scratch(1, (size_t)(M ? M : 1) * out->cols * sizeof(float)));
    if (!G) return last_fail_code();
    if (fetch) {   // the matmul reads X_in[j] through the pair lists: no buffer F, no gather launch
        if (M == 0) return reduce_impl<T>(G, kmap, out, ep);
        TS_TRY(ensure_pairs(kmap));
        TS_TRY(grouped_mm_launch<T>(nullptr, pr.x, pr.wt, kmap, whole_plan(kmap), G, pr.cin_pad, out->cols, kmap->d_in_idx, sec));
        return reduce_impl<T>(G, kmap, out, ep);
    }
    void *F = scratch(0, (size_t)(M ? M : 1) * pr.cin_pad * sizeof(T));
    if (!F) return last_fail_code();
    TS_TRY(gather_impl(pr.x, feats->rows, pr.cin_pad, feats->dtype, kmap, F));
    TS_TRY(grouped_mm_impl<T>(F, pr.x, pr.wt, kmap, G, pr.cin_pad, out->cols));
    return reduce_impl<T>(G, kmap, out, ep);
}

}  // namespace

// TS_DATAFLOW_AUTO.  The fused kernel re-reads a layer's weights for every tile of 128 outputs
// (about 20 of the 27 offsets meet an input somewhere in a tile); the explicit dataflow reads
// them once but moves every pair's rows through the buffer G (and F, unless the matmul fetches
// the rows itself, which is the form taken here).  Wide layers on point sets too
// small to fill the machine with tiles (the coarse levels of a U-Net) are cheaper explicit,
// everything else fused; the factor and the size limit come from timing both on the layers of
// the MinkUNet-style benchmark network.
bool prefer_explicit(const ts_kmap *kmap, int cin, int cout, size_t elem) {
    if (kmap->n_tiles > compute_units()) return false;
    if (resolve(kmap) != TS_OK) return false;   // needs the number of pairs
    const double tile_offsets = kmap->K3 < 20 ? kmap->K3 : 20;
    const double fused_weight_bytes = (double)kmap->n_tiles * tile_offsets * cin * cout * elem;
    const double explicit_bytes = (double)kmap->M * (2.0 * cin * elem + 2.0 * cout * sizeof(float));
    return fused_weight_bytes > 0.6 * explicit_bytes;
}

// ---- the layer for callers that cannot allocate -----------------------------------------------------------
// ts_sparse_conv's kernels take two pieces of memory beyond their inputs and outputs: the weights repacked
// into operand order (a staging buffer written by k_pack_weights* and read by the layer kernel) and, for
// TS_F32, a row of zeros that stands in for absent neighbours.  Here both live in one array that is part of
// the library's code object, so that a call reaches no allocator: [0, 4 KiB) zeros, then the packed weights.
constexpr size_t kStaticZeroBytes = 4096;
constexpr size_t kStaticWeightBytes = size_t(4) << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticZeroBytes + kStaticWeightBytes];

namespace {
constexpr int kMaxDevices = 64;
unsigned char *g_static_ptr[kMaxDevices] = {nullptr};   // per device: where that device holds its copy of the array

__global__ void k_clear_words(uint32_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// The device address of the array on the current device (looked up once per device).
int static_scratch(unsigned char **ptr) {
    int dev = -1;
    TS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(TS_ERR_UNSUPPORTED, "device ordinal %d is beyond %d", dev, kMaxDevices - 1);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        TS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)));
        if (!p) return fail(TS_ERR_HIP, "hipGetSymbolAddress gave no address");
        g_static_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *ptr = g_static_ptr[dev];
    return TS_OK;
}
}  // namespace

extern "C" {

int ts_sparse_conv_static(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, ts_tensor *out) {
    TS_TRY(check_layer(feats, weights, kmap, out));
    const bool f16 = feats->dtype == TS_F16;
    const int cin = feats->cols, cout = out->cols, step = f16 ? 32 : Elem<float>::KSTEP;
    if (cin % step != 0) return fail(TS_ERR_UNSUPPORTED, "ts_sparse_conv_static: C_in must be a multiple of %d, got %d (ts_sparse_conv pads narrower rows, in memory it allocates)", step, cin);
    const size_t wbytes = (size_t)kmap->K3 * cin * cout * (f16 ? 2 : 4);
    if (wbytes > kStaticWeightBytes)
        return fail(TS_ERR_UNSUPPORTED, "ts_sparse_conv_static: the weights take %zu bytes, the static area holds %zu (K^3 * C_in * C_out * element size)", wbytes, kStaticWeightBytes);
    if (kmap->n_out == 0) return TS_OK;
    unsigned char *base = nullptr;
    TS_TRY(static_scratch(&base));
    void *wbuf = base + kStaticZeroBytes;
    if (f16) return run_fused_f16(feats, weights, kmap, out, Epilogue(), nullptr, wbuf);
    // the zeros are never written by a layer kernel; they are cleared all the same, so that nothing rests on
    // what an earlier user of the array left there (a fill kernel, not a memset: a caller may be capturing)
    TS_LAUNCH("k_clear_words", k_clear_words, dim3((unsigned)(kStaticZeroBytes / 4 / kThreads)), dim3(kThreads), reinterpret_cast<uint32_t *>(base), (int)(kStaticZeroBytes / 4));
    return run_fused_staged<float>(feats, weights, kmap, out, nullptr, wbuf, base);
}

int ts_sparse_conv_ex(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, ts_tensor *out,
                      int dataflow) {
    TS_TRY(check_layer(feats, weights, kmap, out));
    if (dataflow != TS_DATAFLOW_AUTO && dataflow != TS_DATAFLOW_EXPLICIT && dataflow != TS_DATAFLOW_FUSED &&
        dataflow != TS_DATAFLOW_FUSED_STAGED && dataflow != TS_DATAFLOW_FETCH)
        return fail(TS_ERR_INVALID_ARG, "unknown dataflow %d", dataflow);
    if (kmap->n_out == 0) return TS_OK;
    const bool f16 = feats->dtype == TS_F16;
    if (dataflow == TS_DATAFLOW_AUTO && prefer_explicit(kmap, feats->cols, out->cols, f16 ? 2 : 4)) dataflow = TS_DATAFLOW_FETCH;
    if (dataflow == TS_DATAFLOW_EXPLICIT || dataflow == TS_DATAFLOW_FETCH) {
        const bool fetch = dataflow == TS_DATAFLOW_FETCH;
        return f16 ? run_explicit<_Float16>(feats, weights, kmap, out, nullptr, fetch)
                   : run_explicit<float>(feats, weights, kmap, out, nullptr, fetch);
    }
    if (dataflow == TS_DATAFLOW_FUSED_STAGED)
        return f16 ? run_fused_staged<_Float16>(feats, weights, kmap, out) : run_fused_staged<float>(feats, weights, kmap, out);
    return f16 ? run_fused<_Float16>(feats, weights, kmap, out) : run_fused<float>(feats, weights, kmap, out);
}

int ts_sparse_conv(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, ts_tensor *out) {
    return ts_sparse_conv_ex(feats, weights, kmap, out, TS_DATAFLOW_AUTO);
}

// The layer with its optional elementwise tail; pw, when given, holds the weights already packed.
static int conv_act(const ts_tensor *feats_in, const ts_tensor *weights, const ts_weights *pw, const ts_kmap *kmap,
                    const void *bias, const ts_tensor *residual, int relu, ts_tensor *out,
                    const ts_tensor *feats2 = nullptr) {
    // With feats2 the layer's input is [feats_in | feats2] along the channels.  Where the kernels can read
    // the two parts in place (fp16 fused: both parts multiples of 32 channels; fetch-on-demand: multiples of
    // the operand step) the concatenation is never formed; otherwise it is formed in scratch memory first.
    ts_tensor cat;
    const ts_tensor *feats = feats_in;
    Second sec;
    if (feats2) {
        TS_TRY(check_tensor(feats_in, "feats"));
        TS_TRY(check_tensor(feats2, "feats2"));
        if (feats2->rows != feats_in->rows || feats2->dtype != feats_in->dtype)
            return fail(TS_ERR_SHAPE, "feats2 must have the rows and dtype of feats");
        cat = *feats_in;
        cat.cols = feats_in->cols + feats2->cols;
        feats = &cat;
        sec.x2 = feats2->data;
        sec.cin1 = feats_in->cols;
    }
    TS_TRY(check_layer(feats, weights, kmap, out));
    if (residual) {
        TS_TRY(check_tensor(residual, "residual"));
        if (residual->rows != out->rows || residual->cols != out->cols || residual->dtype != out->dtype)
            return fail(TS_ERR_SHAPE, "residual must have the shape and dtype of out");
        if (residual->data == out->data) return fail(TS_ERR_INVALID_ARG, "residual must not alias out");
    }
    if (bias && (reinterpret_cast<uintptr_t>(bias) & 15)) return fail(TS_ERR_INVALID_ARG, "bias must be 16-byte aligned");
    if (kmap->n_out == 0) return TS_OK;
    const bool f16 = feats->dtype == TS_F16;
    const bool go_explicit = prefer_explicit(kmap, feats->cols, out->cols, f16 ? 2 : 4);
    if (feats2) {
        const int step = go_explicit ? kstep(feats->dtype) : 32;
        const bool in_place = (f16 || go_explicit) && feats_in->cols % step == 0 && feats2->cols % step == 0 &&
                              (go_explicit || ((size_t)kmap->n_in * feats->cols * 2 < (1ull << 31)));
        if (!in_place) {
            void *buf = scratch(4, (size_t)(feats->rows ? feats->rows : 1) * feats->cols * (f16 ? 2 : 4));
            if (!buf) return last_fail_code();
            cat.data = buf;
            TS_TRY(ts_concat_cols(feats_in, feats2, &cat));
            sec = Second();
        }
    }
    Epilogue ep;
    ep.bias = bias;
    ep.residual = residual ? residual->data : nullptr;
    ep.relu = relu != 0;
    if (f16 && !go_explicit) return run_fused_f16(feats, weights, kmap, out, ep, pw, nullptr, sec);
    // fetch-on-demand: the tail runs in the scatter-accumulate kernel
    if (go_explicit)
        return f16 ? run_explicit<_Float16>(feats, weights, kmap, out, pw, true, ep, sec) : run_explicit<float>(feats, weights, kmap, out, pw, true, ep, sec);
    // otherwise (fp32, fused): the layer, then the elementwise step on its output
    TS_TRY(run_fused<float>(feats, weights, kmap, out, pw));
    if (!bias && !residual && !relu) return TS_OK;
    return ts_bias_act(out, bias, residual, relu, out);
}

int ts_sparse_conv_act(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, const void *bias,
                       const ts_tensor *residual, int relu, ts_tensor *out) {
    return conv_act(feats, weights, nullptr, kmap, bias, residual, relu, out);
}

int ts_weights_prepare(const ts_tensor *weights, int kernel_volume, ts_weights **out_weights) {
    if (!out_weights) return fail(TS_ERR_INVALID_ARG, "out_weights is NULL");
    *out_weights = nullptr;
    TS_TRY(check_tensor(weights, "weights"));
    if (kernel_volume != 1 && kernel_volume != 8 && kernel_volume != 27) return fail(TS_ERR_INVALID_ARG, "kernel_volume must be 1, 8 or 27");
    if (weights->rows <= 0 || weights->rows % kernel_volume != 0) return fail(TS_ERR_SHAPE, "weights must be [K^3*C_in, C_out]");
    const int cin = (int)(weights->rows / kernel_volume), cout = weights->cols;
    if (cout % 32 != 0 || cout > 1024 || cin > 1024) return fail(TS_ERR_UNSUPPORTED, "C_out must be a multiple of 32, C_in and C_out at most 1024");
    ts_weights *w = new (std::nothrow) ts_weights();
    if (!w) return fail(TS_ERR_OOM, "host allocation failed");
    w->K3 = kernel_volume;
    w->cin = cin;
    w->cout = cout;
    w->dtype = weights->dtype;
    const bool f16 = weights->dtype == TS_F16;
    const int ks = f16 ? Elem<_Float16>::KSTEP : Elem<float>::KSTEP;
    const int cin_wt = (cin + ks - 1) / ks * ks;
    const size_t n_wt = (size_t)kernel_volume * cout * cin_wt;
    w->wt = dev_alloc(n_wt * elem_size(weights->dtype));
    if (!w->wt) {
        delete w;
        return TS_ERR_OOM;
    }
    if (f16)
        TS_LAUNCH("k_pack_weights", k_pack_weights<_Float16>, dim3(blocks_for((int64_t)n_wt, kThreads)), dim3(kThreads), static_cast<const _Float16 *>(weights->data), static_cast<_Float16 *>(w->wt), kernel_volume, cin, cin_wt, cout);
    else
        TS_LAUNCH("k_pack_weights", k_pack_weights<float>, dim3(blocks_for((int64_t)n_wt, kThreads)), dim3(kThreads), static_cast<const float *>(weights->data), static_cast<float *>(w->wt), kernel_volume, cin, cin_wt, cout);
    if (f16) {
        const int cin_tile = (cin + 31) / 32 * 32, ksteps = cin_tile % 64 == 0 ? 2 : 1;
        const size_t n_tile = (size_t)kernel_volume * cout * cin_tile;
        w->tile = dev_alloc(n_tile * 2);
        if (!w->tile) {
            dev_free(w->wt);
            delete w;
            return TS_ERR_OOM;
        }
        TS_LAUNCH("k_pack_weights", k_pack_weights_tile, dim3(blocks_for((int64_t)n_tile, kThreads)), dim3(kThreads), static_cast<const _Float16 *>(weights->data), static_cast<_Float16 *>(w->tile), kernel_volume, cin, cin_tile, cout, ksteps);
    }
    TS_HIP(hipGetLastError());
    *out_weights = w;
    return TS_OK;
}

void ts_weights_free(ts_weights *w) {
    if (!w) return;
    dev_free(w->wt);
    dev_free(w->tile);
    delete w;
}

int ts_sparse_conv_prepared(const ts_tensor *feats, const ts_weights *w, const ts_kmap *kmap, const void *bias,
                            const ts_tensor *residual, int relu, ts_tensor *out) {
    if (!w) return fail(TS_ERR_INVALID_ARG, "weights is NULL");
    if (kmap && w->K3 != kmap->K3) return fail(TS_ERR_SHAPE, "weights were prepared for kernel volume %d, the map has %d", w->K3, kmap->K3);
    const ts_tensor desc = {w->wt, (int64_t)w->K3 * w->cin, w->cout, w->dtype};   // shape and dtype for the checks
    return conv_act(feats, &desc, w, kmap, bias, residual, relu, out);
}

int ts_sparse_conv_prepared2(const ts_tensor *feats, const ts_tensor *feats2, const ts_weights *w, const ts_kmap *kmap,
                             const void *bias, const ts_tensor *residual, int relu, ts_tensor *out) {
    if (!w) return fail(TS_ERR_INVALID_ARG, "weights is NULL");
    if (kmap && w->K3 != kmap->K3) return fail(TS_ERR_SHAPE, "weights were prepared for kernel volume %d, the map has %d", w->K3, kmap->K3);
    const ts_tensor desc = {w->wt, (int64_t)w->K3 * w->cin, w->cout, w->dtype};
    return conv_act(feats, &desc, w, kmap, bias, residual, relu, out, feats2);
}

int ts_gather_ex(const ts_tensor *feats, const ts_kmap *kmap, ts_tensor *F, int order) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    if (order != TS_GATHER_AUTO && order != TS_GATHER_OUTPUT_ORDER && order != TS_GATHER_INPUT_STATIONARY)
        return fail(TS_ERR_INVALID_ARG, "unknown gather order %d", order);
    TS_TRY(resolve(kmap));
    TS_TRY(check_tensor(feats, "feats"));
    TS_TRY(check_tensor(F, "F"));
    if (feats->rows != kmap->n_in) return fail(TS_ERR_SHAPE, "feats has %lld rows, the map expects %lld", (long long)feats->rows, (long long)kmap->n_in);
    if (F->rows != kmap->M || F->cols != feats->cols || F->dtype != feats->dtype)
        return fail(TS_ERR_SHAPE, "F must be [num_pairs, C_in] of the dtype of feats");
    if ((feats->cols * elem_size(feats->dtype)) % 16 != 0)
        return fail(TS_ERR_UNSUPPORTED, "rows must be a multiple of 16 bytes");
    return gather_impl(feats->data, feats->rows, feats->cols, feats->dtype, kmap, F->data, order);
}

int ts_gather(const ts_tensor *feats, const ts_kmap *kmap, ts_tensor *F) { return ts_gather_ex(feats, kmap, F, TS_GATHER_AUTO); }

int ts_adaptive_groups(const int64_t *sizes, int32_t count, double epsilon, int32_t *group_of, int32_t *num_groups) {
    if (!sizes || !group_of || !num_groups) return fail(TS_ERR_INVALID_ARG, "sizes, group_of and num_groups must not be NULL");
    if (count < 0 || count > kMaxK3) return fail(TS_ERR_INVALID_ARG, "count must be in [0, %d]", kMaxK3);
    if (!(epsilon >= 0.0 && epsilon <= 1.0)) return fail(TS_ERR_INVALID_ARG, "epsilon must be in [0, 1]");
    for (int i = 0; i < count; ++i)
        if (sizes[i] < 0) return fail(TS_ERR_INVALID_ARG, "sizes[%d] is negative", i);
    *num_groups = partition_by_size(sizes, count, epsilon, group_of);
    return TS_OK;
}

static int grouped_matmul_checked(const ts_tensor *F, const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap,
                                  ts_tensor *G, bool adaptive, double epsilon, int64_t S, int64_t *stats) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    TS_TRY(resolve(kmap));
    TS_TRY(check_tensor(F, "F"));
    TS_TRY(check_tensor(weights, "weights"));
    TS_TRY(check_tensor(G, "G"));
    if (kmap->centre >= 0) {
        TS_TRY(check_tensor(feats, "feats"));
        if (feats->rows != kmap->n_in || feats->cols != F->cols || feats->dtype != F->dtype)
            return fail(TS_ERR_SHAPE, "feats must be [num_in, C_in] of the dtype of F");
    }
    if (F->rows != kmap->M || G->rows != kmap->M) return fail(TS_ERR_SHAPE, "F and G must have num_pairs rows");
    if (weights->dtype != F->dtype || G->dtype != TS_F32) return fail(TS_ERR_SHAPE, "weights must match F; G must be TS_F32");
    if (weights->rows != (int64_t)kmap->K3 * F->cols || weights->cols != G->cols)
        return fail(TS_ERR_SHAPE, "weights must be [K^3*C_in, C_out]");
    if (G->cols % 32 != 0 || F->cols % kstep(F->dtype) != 0)
        return fail(TS_ERR_UNSUPPORTED, "C_out must be a multiple of 32 and C_in of %d", kstep(F->dtype));
    // weights only: the rows of F are already in the operand layout
    ts_tensor none = {nullptr, 0, F->cols, F->dtype};
    Prepared pr;
    const void *X = feats ? feats->data : nullptr;
    float *g = static_cast<float *>(G->data);
    if (F->dtype == TS_F16) {
        TS_TRY(prepare<_Float16>(&none, weights, kmap, &pr));
        return adaptive ? grouped_mm_adaptive<_Float16>(F->data, X, pr.wt, kmap, g, F->cols, G->cols, epsilon, S, stats)
                        : grouped_mm_impl<_Float16>(F->data, X, pr.wt, kmap, g, F->cols, G->cols);
    }
    TS_TRY(prepare<float>(&none, weights, kmap, &pr));
    return adaptive ? grouped_mm_adaptive<float>(F->data, X, pr.wt, kmap, g, F->cols, G->cols, epsilon, S, stats)
                    : grouped_mm_impl<float>(F->data, X, pr.wt, kmap, g, F->cols, G->cols);
}

int ts_grouped_matmul(const ts_tensor *F, const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap,
                      ts_tensor *G) {
    return grouped_matmul_checked(F, feats, weights, kmap, G, false, 0.0, 0, nullptr);
}

int ts_grouped_matmul_adaptive(const ts_tensor *F, const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap,
                               double epsilon, int64_t S, ts_tensor *G, int64_t *stats) {
    if (!(epsilon <= 1.0)) return fail(TS_ERR_INVALID_ARG, "epsilon must be at most 1 (negative: no grouping)");
    if (S < 0) return fail(TS_ERR_INVALID_ARG, "S must not be negative");
    return grouped_matmul_checked(F, feats, weights, kmap, G, true, epsilon, S, stats);
}

int ts_scatter_reduce(const ts_tensor *G, const ts_kmap *kmap, ts_tensor *out) {
    if (!kmap) return fail(TS_ERR_INVALID_ARG, "kmap is NULL");
    TS_TRY(resolve(kmap));
    TS_TRY(check_tensor(G, "G"));
    TS_TRY(check_tensor(out, "out"));
    if (G->dtype != TS_F32 || G->rows != kmap->M) return fail(TS_ERR_SHAPE, "G must be TS_F32 [num_pairs, C_out]");
    if (out->rows != kmap->n_out || out->cols != G->cols) return fail(TS_ERR_SHAPE, "out must be [num_out, C_out]");
    if (out->cols % 4 != 0) return fail(TS_ERR_UNSUPPORTED, "C_out must be a multiple of 4");
    return out->dtype == TS_F16 ? reduce_impl<_Float16>(static_cast<const float *>(G->data), kmap, out)
                                : reduce_impl<float>(static_cast<const float *>(G->data), kmap, out);
}

}  // extern "C"
