// Host-side checks of libts's C ABI that need no GPU: argument validation, error texts, the host
// arithmetic of ts_adaptive_groups, NULL-safe releases.  Built against a copy of the library whose host
// code is compiled with AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_host_sanitizers.py),
// so that a bad read in these paths stops the run instead of passing by luck.  Where a call needs a
// device it must fail with an error code, never crash: this program also runs on machines without one.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include <hip/hip_runtime_api.h>

#include "../../include/ts.h"
#include "../../include/ts_bench.h"

static int failures = 0;
#define CHECK(cond)                                                                \
    do {                                                                           \
        if (!(cond)) {                                                             \
            std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);          \
            ++failures;                                                            \
        }                                                                          \
    } while (0)

int main() {
    CHECK(std::strncmp(ts_version(), "libts", 5) == 0);

    // ---- Appendix B, Alg. 4 (first loop): the partition is host arithmetic
    {
        const int64_t sizes[6] = {100, 90, 60, 55, 10, 10};
        int32_t group_of[6], groups = -1;
        CHECK(ts_adaptive_groups(sizes, 6, 0.0, group_of, &groups) == TS_OK);
        CHECK(groups == 5 && group_of[4] == group_of[5] && group_of[0] != group_of[1]);
        CHECK(ts_adaptive_groups(sizes, 6, 1.0, group_of, &groups) == TS_OK);
        CHECK(groups == 1);
        CHECK(ts_adaptive_groups(sizes, 6, 0.15, group_of, &groups) == TS_OK);
        CHECK(groups == 3 && group_of[0] == 0 && group_of[1] == 0 && group_of[2] == 1 && group_of[3] == 1 && group_of[4] == 2);
        CHECK(ts_adaptive_groups(sizes, 0, 0.5, group_of, &groups) == TS_OK && groups == 0);
        CHECK(ts_adaptive_groups(sizes, 28, 0.5, group_of, &groups) == TS_ERR_INVALID_ARG);
        CHECK(ts_adaptive_groups(sizes, 6, 1.5, group_of, &groups) == TS_ERR_INVALID_ARG);
        CHECK(ts_adaptive_groups(nullptr, 6, 0.5, group_of, &groups) == TS_ERR_INVALID_ARG);
        const int64_t neg[2] = {3, -1};
        CHECK(ts_adaptive_groups(neg, 2, 0.5, group_of, &groups) == TS_ERR_INVALID_ARG);
        CHECK(std::strlen(ts_last_error()) > 0);
    }

    // ---- mapping: argument validation comes before any device work
    {
        ts_kmap *m = reinterpret_cast<ts_kmap *>(0x1);
        alignas(16) int32_t coords[8] = {0, 1, 2, 3, 0, 4, 5, 6};
        CHECK(ts_build_kmap(coords, 2, 3, 1, 0, nullptr) == TS_ERR_INVALID_ARG);
        CHECK(ts_build_kmap(coords, -1, 3, 1, 0, &m) == TS_ERR_INVALID_ARG && m == nullptr);
        CHECK(ts_build_kmap(nullptr, 2, 3, 1, 0, &m) == TS_ERR_INVALID_ARG);
        CHECK(ts_build_kmap(coords, 2, 4, 1, 0, &m) == TS_ERR_INVALID_ARG);
        CHECK(ts_build_kmap(coords, 2, 2, 1, 0, &m) == TS_ERR_INVALID_ARG);      // stride 1 needs an odd kernel
        CHECK(ts_build_kmap(coords, 2, 3, 3, 0, &m) == TS_ERR_INVALID_ARG);
        CHECK(ts_build_kmap(coords, 2, 3, 1, 1, &m) == TS_ERR_INVALID_ARG);      // transposed needs a stride
        CHECK(ts_build_kmap(reinterpret_cast<const int32_t *>(reinterpret_cast<const char *>(coords) + 4), 1, 3, 1, 0, &m) == TS_ERR_INVALID_ARG);
        ts_kmap_options opt;
        std::memset(&opt, 0, sizeof(opt));
        opt.search = 7;
        CHECK(ts_build_kmap_ex(coords, 2, 3, 1, 0, &opt, &m) == TS_ERR_INVALID_ARG);
        opt.search = TS_SEARCH_GRID;
        opt.grid_batches = 0;
        CHECK(ts_build_kmap_ex(coords, 2, 3, 1, 0, &opt, &m) == TS_ERR_INVALID_ARG);
        opt.grid_batches = 1;
        opt.grid_lo[0] = 5;
        opt.grid_hi[0] = 4;
        CHECK(ts_build_kmap_ex(coords, 2, 3, 1, 0, &opt, &m) == TS_ERR_INVALID_ARG);
        std::memset(&opt, 0, sizeof(opt));
        opt.has_boundary = 1;
        CHECK(ts_build_kmap_ex(coords, 2, 3, 2, 0, &opt, &m) == TS_ERR_INVALID_ARG);   // boundary 0
        CHECK(ts_identity_kmap(-1, &m) == TS_ERR_INVALID_ARG);
        CHECK(ts_identity_kmap(5, nullptr) == TS_ERR_INVALID_ARG);
        // an empty input is a valid, empty map, and needs no device
        CHECK(ts_build_kmap(nullptr, 0, 3, 1, 0, &m) == TS_OK && m != nullptr);
        if (m) {
            CHECK(ts_kmap_num_in(m) == 0 && ts_kmap_num_out(m) == 0 && ts_kmap_kernel_volume(m) == 27);
            int64_t sizes[27];
            CHECK(ts_kmap_sizes(m, sizes) == TS_OK && sizes[13] == 0);
            CHECK(ts_kmap_status(m) == TS_OK);
            int32_t lo[3], hi[3], b;
            CHECK(ts_kmap_out_box(m, lo, hi, &b) == TS_ERR_UNSUPPORTED);
            ts_free(m);
        }
    }

    // ---- NULL handles and NULL-safe releases
    {
        CHECK(ts_kmap_num_in(nullptr) == -1 && ts_kmap_num_out(nullptr) == -1 && ts_kmap_num_pairs(nullptr) == -1);
        CHECK(ts_kmap_kernel_volume(nullptr) == -1);
        CHECK(ts_kmap_status(nullptr) == TS_ERR_INVALID_ARG);
        CHECK(ts_kmap_prepare(nullptr) == TS_ERR_INVALID_ARG);
        CHECK(ts_kmap_sort_rows(nullptr) == TS_ERR_INVALID_ARG);
        ts_kmap *t = nullptr;
        CHECK(ts_kmap_transpose(nullptr, &t) == TS_ERR_INVALID_ARG);
        ts_free(nullptr);
        ts_weights_free(nullptr);
    }

    // ---- compute: shape and argument checks
    {
        ts_tensor x = {nullptr, 0, 32, TS_F16}, w = {nullptr, 0, 32, TS_F16}, y = {nullptr, 0, 32, TS_F16};
        CHECK(ts_sparse_conv(&x, &w, nullptr, &y) == TS_ERR_INVALID_ARG);
        CHECK(ts_sparse_conv_static(&x, &w, nullptr, &y) == TS_ERR_INVALID_ARG);
        CHECK(ts_sparse_conv_prepared(&x, nullptr, nullptr, nullptr, nullptr, 0, &y) == TS_ERR_INVALID_ARG);
        CHECK(ts_gather(&x, nullptr, &y) == TS_ERR_INVALID_ARG);
        CHECK(ts_scatter_reduce(&x, nullptr, &y) == TS_ERR_INVALID_ARG);
        ts_weights *pw = nullptr;
        CHECK(ts_weights_prepare(nullptr, 27, &pw) == TS_ERR_INVALID_ARG && pw == nullptr);
        alignas(16) static uint16_t wdata[27 * 16 * 32];
        ts_tensor wt = {wdata, 27 * 16, 32, TS_F16};
        CHECK(ts_weights_prepare(&wt, 5, &pw) == TS_ERR_INVALID_ARG);
        ts_tensor odd = {wdata, 27 * 16 + 1, 32, TS_F16};
        CHECK(ts_weights_prepare(&odd, 27, &pw) == TS_ERR_SHAPE);
        ts_tensor narrow = {wdata, 27 * 16, 24, TS_F16};
        CHECK(ts_weights_prepare(&narrow, 27, &pw) == TS_ERR_UNSUPPORTED);
        ts_kmap *m = nullptr;
        CHECK(ts_build_kmap(nullptr, 0, 3, 1, 0, &m) == TS_OK);
        if (m) {
            ts_tensor x0 = {nullptr, 0, 16, TS_F16}, w0 = {wdata, 27 * 16, 32, TS_F16}, y0 = {nullptr, 0, 32, TS_F16};
            CHECK(ts_sparse_conv(&x0, &w0, m, &y0) == TS_OK);                       // zero rows: nothing to launch
            ts_tensor y1 = {nullptr, 3, 32, TS_F16};
            CHECK(ts_sparse_conv(&x0, &w0, m, &y1) == TS_ERR_INVALID_ARG);          // rows without data
            ts_tensor wbad = {wdata, 26 * 16, 32, TS_F16};
            CHECK(ts_sparse_conv(&x0, &wbad, m, &y0) == TS_ERR_SHAPE);
            ts_tensor y32 = {nullptr, 0, 32, TS_F32};
            CHECK(ts_sparse_conv(&x0, &w0, m, &y32) == TS_ERR_SHAPE);
            CHECK(ts_sparse_conv_ex(&x0, &w0, m, &y0, 99) == TS_ERR_INVALID_ARG);
            CHECK(ts_gather_ex(&x0, m, &y0, 9) == TS_ERR_INVALID_ARG);
            ts_free(m);
        }
    }

    // ---- the caller's allocator: every block handed out comes back, whatever happens to the call
    {
        static int handed_out = 0, returned = 0;
        auto alloc = [](size_t bytes, void *ctx) -> void * {
            ++*static_cast<int *>(ctx);
            return std::malloc(bytes ? bytes : 1);      // host memory: without a device nothing ever touches it
        };
        auto release = [](void *p, void *) {
            ++returned;
            std::free(p);
        };
        CHECK(ts_set_allocator(alloc, nullptr, nullptr) == TS_ERR_INVALID_ARG);
        CHECK(ts_set_allocator(nullptr, release, nullptr) == TS_ERR_INVALID_ARG);
        CHECK(ts_set_allocator(alloc, release, &handed_out) == TS_OK);
        alignas(16) static int32_t coords[4 * 64];
        for (int i = 0; i < 64; ++i) {
            coords[4 * i] = 0;
            coords[4 * i + 1] = i;
            coords[4 * i + 2] = 2 * i;
            coords[4 * i + 3] = 3;
        }
        ts_kmap *m = nullptr;
        // with a device this pointer would have to be device memory; here the build can only fail (no device)
        // or, should a device be present after all, is not attempted
        int dev_count = 0;
        const bool no_device = hipGetDeviceCount(&dev_count) != hipSuccess || dev_count == 0;
        if (no_device) {
            const int rc = ts_build_kmap(coords, 64, 3, 1, 0, &m);
            CHECK(rc != TS_OK && m == nullptr);
            const int rc2 = ts_build_kmap(coords, 64, 2, 2, 0, &m);
            CHECK(rc2 != TS_OK && m == nullptr);
            CHECK(handed_out > 0);
        }
        CHECK(ts_set_allocator(nullptr, nullptr, nullptr) == TS_OK);
        (void)ts_release_cache();
        CHECK(handed_out == returned);
    }

    // ---- measurement helpers
    {
        char buf[8];
        CHECK(ts_profile_enable(0, nullptr) == TS_OK);
        CHECK(ts_profile_read(nullptr, 0) == TS_ERR_INVALID_ARG);
        CHECK(ts_copy_bytes(nullptr, buf, 16) == TS_ERR_INVALID_ARG);
        double flops = 0;
        CHECK(ts_mfma_loop(0, buf, &flops) == TS_ERR_INVALID_ARG);
    }

    if (failures) {
        std::printf("%d host check(s) failed\n", failures);
        return 1;
    }
    std::printf("host checks ok\n");
    return 0;
}
