/*
 * ts.h - C ABI of the MI355X sparse-convolution library (libts.so).
 *
 * One layer of a sparse CNN on a voxelized point cloud, as the paper states it
 * (Sec. 2): inputs are integer coordinates P_in with features X_in, weights
 * W[K^3][C_in][C_out], kernel size K and stride s; "mapping" takes coordinates
 * only and yields the output coordinates P_out and the kernel maps
 * M = {(j, k, n)} with p_j = s*q_k + delta_n (Sec. 2.1, Alg. 1 and Alg. 3);
 * the compute takes X_in, W and M and yields
 *     x_out[k] = sum_n sum_j 1[p_j = s*q_k + delta_n] x_in[j] * W_n     (Eq. 1)
 * by gather, per-offset matmul and scatter-accumulate (Sec. 2.2, Alg. 2).
 *
 * Conventions (fixed by this library where the paper is silent):
 *   coords   int32 [N][4], columns (batch, x, y, z); rows are distinct.
 *   offsets  Delta^3(K) = {-r..K-1-r}^3, r = floor((K-1)/2); weight index
 *            n = ((dx+r)*K + (dy+r))*K + (dz+r)  (x slowest).  K=3: {-1,0,1}^3,
 *            K=2: {0,1}^3.
 *   stride 1: P_out = P_in, same row order (output k is input k).
 *   stride>1: P_out = distinct candidates (p - delta)/s with s | (p - delta),
 *            in ascending (batch, x, y, z) order; clipped to the grid [0, b) when
 *            a boundary b is given (Alg. 3; ts_build_kmap_ex), else not at all.
 *   transposed: coords are the FINE coordinates (the outputs of the transposed
 *            layer).  The map is the forward (K, s) map fine -> coarse with the
 *            roles swapped: inputs are the coarse points in ascending order,
 *            x_out[j] = sum over (k, n) with p_j = s*q_k + delta_n of x_in[k]*W_n.
 *
 * Memory: every pointer documented "device" is HIP device memory on the
 * current device; "host" is ordinary host memory.  The caller owns all
 * tensors passed in; they must stay alive until the stream has passed the
 * call.  The library owns everything behind ts_kmap* until ts_free().
 *
 * Errors: every int-returning function returns TS_OK (0) or a negative
 * ts_status; ts_last_error() gives thread-local text for the last failure.
 * No exception crosses this boundary.  There is no CPU fallback: without a
 * usable HIP device every call fails with TS_ERR_HIP.
 *
 * Threading/streams: work is enqueued on the stream set by ts_set_stream()
 * (default: the null stream).  The stream, the scratch areas and the memory pool are per process: one
 * stream is in use at a time.  Changing the stream is allowed between calls; memory the library freed
 * on the previous stream is reused on the new one only after the previous stream has drained (the
 * library waits for it then, except under stream capture, where it allocates instead).  A ts_kmap must
 * be used on the stream it was built on, or after that stream has been synchronised.  Calls from several
 * host threads at once are not supported.
 */
#ifndef TS_H
#define TS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ts_status {
    TS_OK = 0,
    TS_ERR_INVALID_ARG = -1,     /* null pointer, negative size, unsupported K / stride            */
    TS_ERR_SHAPE = -2,           /* rows / cols / dtype do not match the kernel map or each other   */
    TS_ERR_COORD_RANGE = -3,     /* a coordinate is outside the packable range below                */
    TS_ERR_DUPLICATE_COORD = -4, /* two input rows hold the same (batch, x, y, z)                   */
    TS_ERR_OOM = -5,             /* device or host allocation failed                                */
    TS_ERR_HIP = -6,             /* a HIP runtime call failed (text in ts_last_error)               */
    TS_ERR_UNSUPPORTED = -7      /* valid request outside what the kernels cover                    */
} ts_status;

/* Element types of feature / weight / output tensors. */
enum { TS_F32 = 0, TS_F16 = 1 };

/* Packable coordinate range: batch in [0, TS_BATCH_MAX], x,y,z in [TS_COORD_MIN, TS_COORD_MAX]. */
#define TS_BATCH_MAX 8190
#define TS_COORD_MIN (-65528)
#define TS_COORD_MAX 65527

/* How ts_sparse_conv_ex computes Eq. 1. */
enum {
    TS_DATAFLOW_AUTO = 0,     /* library's choice (the fused kernel where it applies)                     */
    TS_DATAFLOW_EXPLICIT = 1, /* Alg. 2 as three launches: gather -> grouped matmul -> scatter-accumulate */
    TS_DATAFLOW_FUSED = 2,    /* one output-stationary kernel: gather into the MFMA operand, accumulate
                                 over offsets in registers, write each output row once                    */
    TS_DATAFLOW_FUSED_STAGED = 3, /* the same dataflow by the older kernel that stages weight slabs and
                                 neighbour indices per tile in LDS with 32x32 MFMAs: what TS_F32 always
                                 runs, and TS_F16 when features or weights reach 2 GiB                    */
    TS_DATAFLOW_FETCH = 4     /* Alg. 2 without the buffer F: the grouped matmul fetches X_in[j] through
                                 the map itself (the fetch-on-demand dataflow that Sec. 5.2 and the
                                 related work name as the better one on small workloads), then the
                                 scatter-accumulate: two launches.  Same bits as TS_DATAFLOW_EXPLICIT.
                                 TS_DATAFLOW_AUTO takes it for wide layers on small maps.                 */
};

/* Dense row-major matrix: rows x cols elements of dtype, device memory. */
typedef struct ts_tensor {
    void   *data;   /* device */
    int64_t rows;
    int32_t cols;
    int32_t dtype;  /* TS_F32 or TS_F16 */
} ts_tensor;

/* Opaque, immutable, device-resident kernel map (Sec. 2.1: the maps M plus P_out). */
typedef struct ts_kmap ts_kmap;

/* ---- mapping (Sec. 2.1; Alg. 1, Alg. 3) ---------------------------------------------------- */

/*
 * Build the kernel map of a (kernel_size, stride) convolution over N input points.
 *   coords       device, int32 [N][4] (batch, x, y, z); not modified; N >= 0.
 *   kernel_size  1, 2 or 3 (stride 1 requires odd kernel_size); stride 1 or 2.
 *   transposed   0 or 1 (1 requires stride > 1), see the header comment.
 *   out_kmap     receives the new map; *out_kmap = NULL on error.
 * Internally: pack coordinates to 64-bit keys, insert inputs into an open-addressing hash
 * table, probe s*q_k + delta_n for every output and offset (one row of neighbour indices
 * per output), count per offset.  A strided build first finds its output coordinates
 * (Alg. 3) and chooses its route by the bounding box of its input, see ts_build_kmap_ex
 * (TS_SEARCH_AUTO).  The
 * per-offset pair lists are derived from that when first asked for (ts_kmap_pairs, the
 * explicit dataflow).  Synchronises the stream (it must learn N_out and the map sizes and
 * report bad input).  The map may be reused by any number of ts_sparse_conv calls.
 */
int ts_build_kmap(const int32_t *coords, int64_t N, int kernel_size, int stride, int transposed,
                  ts_kmap **out_kmap);

/*
 * ts_build_kmap without the wait at the end, where the build allows it: the map is returned as soon
 * as its kernels are enqueued, and its sizes and the error flags of its input (duplicate or
 * out-of-range coordinates) reach the host when something first needs them: ts_kmap_status,
 * ts_kmap_num_pairs / _sizes / _pairs, the explicit dataflow, ts_kmap_sort_rows, ts_kmap_transpose.
 * For a 3x3x3 stride-1 map the part of the build that only those need (the pass that counts each
 * offset's pairs) is put off until then as well.  The fused layer kernel needs none of it, so a
 * build followed by ts_sparse_conv runs on the device without a host round trip in between.  A map whose input was bad is safe to use (rows of
 * bad points have no neighbours) but its results are meaningless: call ts_kmap_status before
 * trusting them.  Strided maps still wait once inside (for the number of output points).
 */
int ts_build_kmap_async(const int32_t *coords, int64_t N, int kernel_size, int stride, int transposed,
                        ts_kmap **out_kmap);
/* Waits for an asynchronous build's verdict: TS_OK, TS_ERR_DUPLICATE_COORD or TS_ERR_COORD_RANGE. */
int ts_kmap_status(const ts_kmap *kmap);
/*
 * Optional, for a map from ts_build_kmap_async that will serve more than a fused layer: enqueues, without
 * waiting, the part of the build that was put off (the pass that counts each offset's pairs), so that a
 * later ts_kmap_status / accessor / explicit-dataflow call only waits instead of running it then.  A caller
 * that builds several maps calls this on each and then ts_kmap_status on each: the waits overlap.
 * No effect on maps that have nothing put off.
 */
int ts_kmap_prepare(const ts_kmap *kmap);

/*
 * The map of a 1x1x1 convolution at stride 1 over n distinct points, made without coordinates: by
 * Eq. 1 with delta = 0 output k takes input k and nothing else, so M = {(k, k, 0)} whatever the points
 * are, as long as no two of them coincide (which the caller knows from any other build on the same
 * points; nothing is checked here).  n_in = n_out = |M| = n, kernel volume 1.  Two launches, no host
 * wait, no search; every layer call accepts the map.  It holds no coordinates: ts_kmap_out_coords and
 * ts_kmap_in_coords fail on it with TS_ERR_UNSUPPORTED.  Errors: TS_ERR_INVALID_ARG (NULL out_kmap, n < 0
 * or n >= 2^31), TS_ERR_OOM.  Free with ts_free.
 */
int ts_identity_kmap(int64_t n, ts_kmap **out_kmap);

/*
 * ts_build_kmap with the choices the paper leaves to each layer (Sec. 4.4; Alg. 3).  options == NULL
 * is ts_build_kmap.  The map built is the same whatever `search` says.
 *   search        TS_SEARCH_AUTO (what ts_build_kmap does): stride 1 searches the hash table.  A strided
 *                 build measures the bounding box of its coordinates on the device (one more host
 *                 round trip; none if the caller states the box: grid_batches > 0 with grid_lo / grid_hi
 *                 as below, ignored at stride 1) and, when its outputs can lie in at most 2^28 cells,
 *                 marks its candidates in a bitmap over those cells (32 MiB at most, a temporary) and
 *                 reads the set bits off in order: the sorted distinct outputs without a sort.  The map
 *                 then follows without a search either: every kept candidate of an input is an output,
 *                 whose row number is the rank of its cell among the marked ones.  Larger boxes take the
 *                 hash route.
 *                 TS_SEARCH_HASH: the open-addressing table (a temporary of the build: a power of two
 *                 of 12-byte slots, four per searched point or more; at most 2^26 points); a strided
 *                 build finds its output coordinates by sorting the candidates.  TS_SEARCH_GRID: the collision-free
 *                 grid of Sec. 4.4, one int32 cell per coordinate of the box the caller states
 *                 with grid_lo / grid_hi (inclusive bounds of x, y, z over the rows of `coords`) and
 *                 grid_batches (batch indices are below it): one memory access per insertion and per
 *                 lookup; a strided build with a stated box takes the bitmap route described above
 *                 (no cells of the grid are involved).
 *                 A coordinate outside the stated box is TS_ERR_COORD_RANGE.  The box may
 *                 span at most 2^30 cells (TS_ERR_UNSUPPORTED beyond).  The cells are library memory
 *                 kept between builds (4 bytes per cell of the largest box seen, until
 *                 ts_release_cache): a build writes its points in and takes them out again, so it
 *                 never clears the volume.  Builds on different streams must not overlap.
 *   wait          0: do not wait at the end (ts_build_kmap_async).
 *   has_boundary  != 0 with stride > 1: Alg. 3's boundary check.  A candidate u = p - delta becomes an
 *                 output only if 0 <= u < stride * boundary on every axis, so the outputs lie on the
 *                 grid [0, boundary) (x, y, z; each positive).  Ignored at stride 1, where the outputs
 *                 are the inputs.  Inputs all of whose candidates are cut feed no output (forward) or
 *                 get no contribution (transposed).
 */
enum { TS_SEARCH_AUTO = 0, TS_SEARCH_HASH = 1, TS_SEARCH_GRID = 2 };
typedef struct ts_kmap_options {
    int32_t search;
    int32_t wait;
    int32_t has_boundary;
    int32_t boundary[3];
    int32_t grid_lo[3];
    int32_t grid_hi[3];
    int32_t grid_batches;
} ts_kmap_options;
int ts_build_kmap_ex(const int32_t *coords, int64_t N, int kernel_size, int stride, int transposed,
                     const ts_kmap_options *options, ts_kmap **out_kmap);

/*
 * The transposed map of `forward` (built with stride > 1, transposed = 0): the same map that
 * ts_build_kmap(fine coords, kernel_size, stride, 1) yields for the coordinates `forward` was built
 * from, derived from `forward` without another search.  A network's upsampling layer takes this
 * instead of building its map from coordinates (maps are shared between layers, Sec. 2.3).
 * `forward` is not modified and need not outlive the result.  Does not synchronise.
 */
int ts_kmap_transpose(const ts_kmap *forward, ts_kmap **out_kmap);

/*
 * Optional.  Orders the output rows of a map by their offset bitmask (which offsets meet an input),
 * so that the 128 rows a workgroup of the output-stationary kernel handles share their offsets and
 * absent ones are skipped per tile (Sec. 4.2 argues the same way for grouping by map size).  It
 * costs about as much as the search itself, so it pays for maps that serve several layers; results
 * of ts_sparse_conv do not depend on it bit for bit.  Idempotent.  Synchronises the stream.
 */
int ts_kmap_sort_rows(ts_kmap *kmap);

/* Release a map and everything it owns.  NULL is allowed. */
void ts_free(ts_kmap *kmap);

int64_t ts_kmap_num_in(const ts_kmap *kmap);        /* rows of X_in the map expects               */
int64_t ts_kmap_num_out(const ts_kmap *kmap);       /* rows of X_out it produces                  */
int64_t ts_kmap_num_pairs(const ts_kmap *kmap);     /* |M| = sum of the per-offset sizes          */
int     ts_kmap_kernel_volume(const ts_kmap *kmap); /* K^3                                        */

/* Output coordinates P_out: dst is device int32 [num_out][4].  (For a transposed map: the fine coords.) */
int ts_kmap_out_coords(const ts_kmap *kmap, int32_t *dst);
/*
 * A box that holds every output coordinate of a strided forward map, known on the host without a wait
 * when the build marked its candidates in a bitmap over such a box (the default route and TS_SEARCH_GRID):
 * lo, hi (host, 3 values each, inclusive x, y, z) and *batches (batch indices are below it).  It is what
 * the build of the next level of a pyramid can be given as its box (ts_kmap_options: TS_SEARCH_AUTO with
 * grid_lo / grid_hi / grid_batches stated), which then need not measure one.  TS_ERR_UNSUPPORTED for maps
 * whose build bounded nothing (stride 1, transposed, the sort route, empty inputs).
 */
int ts_kmap_out_box(const ts_kmap *kmap, int32_t *lo, int32_t *hi, int32_t *batches);
/* Input coordinates in the row order X_in must have: dst is device int32 [num_in][4]. */
int ts_kmap_in_coords(const ts_kmap *kmap, int32_t *dst);
/* Per-offset map sizes |M[W_n]|: dst is HOST int64 [K^3]. */
int ts_kmap_sizes(const ts_kmap *kmap, int64_t *dst);
/*
 * The maps as index pairs, offset-major: entries [off_n, off_n + size_n) belong to offset n,
 * off_n = sum of sizes before n; within an offset, pairs are ordered by output index.
 * in_idx/out_idx are device int32 [num_pairs]; either may be NULL.
 */
int ts_kmap_pairs(const ts_kmap *kmap, int32_t *in_idx, int32_t *out_idx);

/* ---- compute (Sec. 2.2, Alg. 2; Eq. 1) ------------------------------------------------------ */

/*
 * out = sparse convolution of feats with weights over kmap (Eq. 1).
 *   feats    [num_in][C_in], weights [K^3 * C_in][C_out] (i.e. [K^3][C_in][C_out] flattened),
 *   out      [num_out][C_out], caller-allocated, fully overwritten.
 * All three share one dtype.  TS_F16 multiplies fp16 operands and accumulates in fp32 over
 * C_in and over all offsets, rounding once when the row is stored; TS_F32 uses fp32 throughout.
 * C_out must be a multiple of 32; C_in may be anything (rows narrower than the kernels' operand step -
 * 32 channels for TS_F16, 8 for TS_F32 - are zero-extended in library scratch: the 4-channel stem of a
 * network); both at most 1024 (TS_ERR_UNSUPPORTED beyond).
 * Never synchronises.  Uses library-owned scratch memory (repacked weights, padded features, the
 * buffers F and G of the explicit dataflows) that grows on demand with hipMalloc; an outgrown area stays
 * allocated, unused, until ts_release_cache, because work already enqueued or a HIP graph captured earlier
 * may still address it.  While the stream is being captured nothing can grow: a call that would need to
 * fails with TS_ERR_UNSUPPORTED, so run the same call once eagerly before capturing (or take
 * ts_sparse_conv_static, which owns no growable memory).
 */
int ts_sparse_conv(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap,
                   ts_tensor *out);

/*
 * out = act(sparse convolution + bias + residual): ts_sparse_conv followed by ts_bias_act (below)
 * in one call.  bias (device, [C_out], dtype of out) and residual ([num_out][C_out], dtype of out,
 * must not alias out) may be NULL; relu != 0 clamps at zero.  The result equals, bit for bit, that
 * of the two calls made one after the other (the layer's sum is rounded to the I/O dtype first).
 * It is computed where the layer's sums are formed - the fused kernel's epilogue (TS_F16), or the
 * scatter-accumulate kernel where the library takes the fetch-on-demand dataflow - so the
 * activation tensor is written once and not read back (the paper's Principle II: data movement is
 * what to cut, Sec. 3); only TS_F32 layers that run fused take a second launch for it.
 */
int ts_sparse_conv_act(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap,
                       const void *bias, const ts_tensor *residual, int relu, ts_tensor *out);

/*
 * Weights of a layer, repacked once into the layouts the kernels read (the layer calls above do this
 * on every call; a network whose weights do not change between calls prepares them once).
 *   weights        [K^3 * C_in][C_out] as for ts_sparse_conv; not needed after the call returns
 *                  (the copy is made on the stream).
 *   kernel_volume  K^3 of the maps the weights will be used with: 1, 8 or 27.
 * ts_sparse_conv_prepared is ts_sparse_conv_act with such weights; results are bit-identical.
 * ts_weights_free releases them (NULL allowed; not before the stream has passed their last use).
 */
typedef struct ts_weights ts_weights;
int  ts_weights_prepare(const ts_tensor *weights, int kernel_volume, ts_weights **out_weights);
void ts_weights_free(ts_weights *weights);
int  ts_sparse_conv_prepared(const ts_tensor *feats, const ts_weights *weights, const ts_kmap *kmap,
                             const void *bias, const ts_tensor *residual, int relu, ts_tensor *out);

/*
 * ts_sparse_conv_prepared on an input that is the channel concatenation [feats | feats2] of two tensors
 * (a U-Net decoder's skip connection), without forming it: the layer kernels read input channels below
 * feats->cols from feats and the others from feats2 (the paper's Principle II, Sec. 3: data movement is what
 * to cut; the concatenated tensor would be written once and read by every layer that takes it).
 *   feats   [num_in][C1], feats2 [num_in][C2], same dtype; weights prepared from [K^3 * (C1 + C2)][C_out],
 *           rows of a weight slice in the order of the concatenation.
 * The result equals, bit for bit, ts_sparse_conv_prepared on the concatenated tensor.  The parts are read in
 * place when C1 and C2 are multiples of 32 (TS_F16) or, where the library takes the fetch-on-demand dataflow,
 * of 16 (TS_F16) / 8 (TS_F32); any other pair of widths is concatenated into library scratch first.
 * feats2 == NULL is ts_sparse_conv_prepared.
 */
int ts_sparse_conv_prepared2(const ts_tensor *feats, const ts_tensor *feats2, const ts_weights *weights,
                             const ts_kmap *kmap, const void *bias, const ts_tensor *residual, int relu,
                             ts_tensor *out);

/* Same as ts_sparse_conv, with the dataflow chosen by the caller (TS_DATAFLOW_*). */
int ts_sparse_conv_ex(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap,
                      ts_tensor *out, int dataflow);

/*
 * ts_sparse_conv for callers that cannot allocate: code under HIP graph capture, serving loops and
 * harnesses that forbid hipMalloc.  Same arguments, same kernels (the fused dataflow), same bits; but the one
 * piece of memory ts_sparse_conv takes from the library's grow-on-demand scratch - the weights repacked
 * into the order the kernels read, plus a row of zeros for TS_F32 - lives in a fixed array inside the
 * library's code object (4 MiB + 4 KiB on every GPU the library runs on, held until the process ends).
 * The call reaches no hipMalloc, hipFree or other allocating routine, and never synchronises.
 * Limits (TS_ERR_UNSUPPORTED beyond them, with the figures in ts_last_error):
 *   K^3 * C_in * C_out * element size <= 4 MiB (e.g. 27 x 256 x 256 fp16, 27 x 192 x 192 fp32);
 *   C_in a multiple of 32 (TS_F16) or 8 (TS_F32): narrower rows would need a padded copy of feats;
 *   features and weights below 2 GiB each.
 * The map must come from a build that has finished its own allocations (any map ts_build_kmap* returned).
 * The first call on a device looks the array's address up (hipGetSymbolAddress); make that call outside a
 * capture.  Every call on a GPU shares that GPU's array and overwrites it: calls that overlap on one GPU
 * (two streams, two host threads) race; calls on one stream are ordered and safe.
 */
int ts_sparse_conv_static(const ts_tensor *feats, const ts_tensor *weights, const ts_kmap *kmap, ts_tensor *out);

/*
 * The three stages of Alg. 2 on their own (what TS_DATAFLOW_EXPLICIT runs), for per-stage
 * tests and timing.  The buffers F and G are offset-major like ts_kmap_pairs.
 *
 * ts_gather:        F[off_n + m] = feats[in_n[m]] for every offset in one launch.
 *                   F is [num_pairs][C_in], dtype of feats.  For an odd-K stride-1 map the rows
 *                   of the centre offset are left untouched: its map is the identity and
 *                   ts_grouped_matmul reads feats directly (Sec. 4.2.1).
 * ts_grouped_matmul: G[off_n + m] = F[off_n + m] * W_n for every offset in one launch, tiles
 *                   scheduled over (offset, row block) with no zero padding.  feats is needed
 *                   for the centre offset only and may be NULL when the map has none.
 *                   G is [num_pairs][C_out] TS_F32 (partial sums stay fp32).
 * ts_scatter_reduce: out[k] = sum of G rows whose pair has output k (output-stationary: each
 *                   row is reduced in registers in offset order and written once).
 */
int ts_gather(const ts_tensor *feats, const ts_kmap *kmap, ts_tensor *F);
/*
 * ts_gather with the order of the copy chosen by the caller; F is the same whatever the order.
 *   TS_GATHER_OUTPUT_ORDER      walks F's rows in order and fetches each pair's input row (sequential
 *                               writes, gathered reads: an input row is read once per pair it is in).
 *   TS_GATHER_INPUT_STATIONARY  the locality-aware order of Sec. 4.3.2: walks the input rows in order,
 *                               reads each once and writes it to every row of F it belongs in
 *                               (positions from the map's rank bitmaps).  Built for 3x3x3 stride-1 maps
 *                               and rows of 64, 128, 256 or 512 bytes; other requests run in output order.
 *   TS_GATHER_AUTO              what ts_gather and the explicit dataflow do: input-stationary where it is
 *                               built and rows have 128 bytes or more, or the feature matrix exceeds the
 *                               256 MB last-level cache (every re-read of a 64-byte row then comes from
 *                               memory); else output order.
 */
enum { TS_GATHER_AUTO = 0, TS_GATHER_OUTPUT_ORDER = 1, TS_GATHER_INPUT_STATIONARY = 2 };
int ts_gather_ex(const ts_tensor *feats, const ts_kmap *kmap, ts_tensor *F, int order);
int ts_grouped_matmul(const ts_tensor *F, const ts_tensor *feats, const ts_tensor *weights,
                      const ts_kmap *kmap, ts_tensor *G);
int ts_scatter_reduce(const ts_tensor *G, const ts_kmap *kmap, ts_tensor *out);

/*
 * Adaptive grouping (Sec. 4.2.3; Appendix B, Alg. 4), kept for comparison with the single
 * tile-scheduled launch of ts_grouped_matmul, which needs neither padding nor tuning.
 *
 * ts_adaptive_groups: host arithmetic only (no GPU call).  sizes[count] (host, count <= 27, all >= 0)
 *   are the map sizes of consecutive weight indices; group_of[count] (host, written) receives the
 *   number of the group each index falls in, *num_groups the number of groups.  A group starts at the
 *   first index not yet grouped and takes the following ones while 1 - n_min / n_max <= epsilon over
 *   its sizes (the share of padding a batched matmul of the group would carry; two empty maps count as
 *   equal).  epsilon in [0, 1]: 0 groups equal sizes only, 1 makes one group.
 *
 * ts_grouped_matmul_adaptive: the same result as ts_grouped_matmul (bit for bit), computed in the
 *   launches Alg. 4 prescribes.  For an odd-K stride-1 map the groups are formed over the first
 *   floor(K^3/2) indices, index i always shares its launch with its mirror K^3-1-i (equal sizes:
 *   symmetric grouping), and the centre offset is a launch of its own; otherwise over all K^3 indices.
 *   A group whose longest map has fewer than S rows is one batched launch with every member padded to
 *   that length (the padding rows are multiplied and thrown away: the redundant computation the
 *   tolerance buys regularity with); any other group is one launch per member.  epsilon < 0 disables
 *   grouping altogether: one launch per non-empty offset (the separate baseline of Sec. 4.2.3).
 *   stats (host, 4 values, may be NULL) receives: launches made, groups formed, rows multiplied
 *   including padding, rows needed (num_pairs).
 */
int ts_adaptive_groups(const int64_t *sizes, int32_t count, double epsilon, int32_t *group_of,
                       int32_t *num_groups);
int ts_grouped_matmul_adaptive(const ts_tensor *F, const ts_tensor *feats, const ts_tensor *weights,
                               const ts_kmap *kmap, double epsilon, int64_t S, ts_tensor *G,
                               int64_t *stats);

/* ---- elementwise steps between layers (not in the paper; needed to chain layers into a network) ---- */

/*
 * out[r][c] = act(x[r][c] + bias[c] + residual[r][c]): bias (device, [cols], dtype of x) and
 * residual (same shape and dtype as x) may be NULL; relu != 0 clamps at zero.  fp32
 * arithmetic, one rounding at the store.  out may alias x or residual.
 */
int ts_bias_act(const ts_tensor *x, const void *bias, const ts_tensor *residual, int relu, ts_tensor *out);
/* out[r] = [a[r], b[r]]: channel concatenation of two tensors with equal rows and dtype. */
int ts_concat_cols(const ts_tensor *a, const ts_tensor *b, ts_tensor *out);

/* ---- runtime ---------------------------------------------------------------------------------- */

/* Stream (hipStream_t) all later calls enqueue on; NULL = the null stream. */
int ts_set_stream(void *hip_stream);
/*
 * Lets the caller's allocator own the library's device memory (for PyTorch: its caching allocator, so that
 * the memory shows in its statistics and is shared with the rest of the program).  From the call on every
 * block the library needs - map storage, temporaries of a build, scratch areas when they grow - is asked
 * for with alloc(bytes, ctx), which returns device memory aligned to 256 bytes or NULL (reported as
 * TS_ERR_OOM), and given back with release(ptr, ctx) when the library is done with it; the library's own
 * pool is bypassed.  The allocator must make a released block safe to hand out again in stream order, as a
 * caching allocator keyed on the current stream does: the library releases a block as soon as the work
 * that uses it has been enqueued on its stream.  alloc == release == NULL goes back to the library's pool.
 * Blocks are returned to where they came from, so the setting may change while maps exist.  The
 * coordinate grid of TS_SEARCH_GRID and the fixed array of ts_sparse_conv_static are not covered.
 */
int ts_set_allocator(void *(*alloc)(size_t bytes, void *ctx), void (*release)(void *ptr, void *ctx), void *ctx);
/* Free the library's cached scratch and pooled device memory (synchronises the device). */
int ts_release_cache(void);

/* Text of the last error on this thread ("" if none). Valid until the next failing call. */
const char *ts_last_error(void);
/* Library version string. */
const char *ts_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TS_H */
