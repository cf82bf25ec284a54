// Runtime pieces of libts: error text, stream, pooled device memory, scratch areas.
#include "ts_internal.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

namespace ts {

static thread_local std::string g_error;
static thread_local int g_error_code = TS_OK;
static hipStream_t g_stream = nullptr;

int fail(int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_error = buf;
    g_error_code = code;
    return code;
}

int last_fail_code() { return g_error_code != TS_OK ? g_error_code : TS_ERR_OOM; }

hipStream_t stream() { return g_stream; }

// ---- pooled device memory -------------------------------------------------------------------
namespace {
std::mutex g_pool_mu;
struct FreeBlock {
    void *p;
    hipStream_t stream;   // the library stream when the block was given back: work enqueued there may still use it
};
std::multimap<size_t, FreeBlock> g_free_blocks;       // size -> block
std::unordered_map<void *, size_t> g_live_blocks;     // block -> size
// The caller's allocator, if one is set (ts_set_allocator): every block then comes from it and goes back to it,
// and the pool above is not used.  A block remembers where it came from, so the setting may change while
// blocks are out.
struct Foreign {
    void (*release)(void *, void *);
    void *ctx;
};
void *(*g_user_alloc)(size_t, void *) = nullptr;
void (*g_user_release)(void *, void *) = nullptr;
void *g_user_ctx = nullptr;
std::unordered_map<void *, Foreign> g_foreign_blocks;  // block -> how to give it back
struct Retired {
    void *p;
    bool foreign;
    Foreign how;
};
std::vector<Retired> g_retired;                       // outgrown scratch areas, kept until ts_release_cache

// Round a request so that similar sizes land in the same bin: 256 B granules below 1 MiB,
// then 1/8-octave steps.
size_t bin_size(size_t bytes) {
    if (bytes < 256) return 256;
    if (bytes <= (1u << 20)) return (bytes + 255) & ~size_t(255);
    size_t p = size_t(1) << (63 - __builtin_clzll(bytes));
    size_t step = p >> 3;
    return (bytes + step - 1) / step * step;
}

struct Scratch {
    void *p = nullptr;
    size_t bytes = 0;
    bool foreign = false;
    Foreign how = {nullptr, nullptr};
};
Scratch g_scratch[8];
void *g_host = nullptr;
size_t g_host_bytes = 0;

bool capturing() {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(g_stream, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}
}  // namespace

// A freed block goes back to work only in stream order.  Blocks given back on the stream the library is on
// now are reused at once (later work on that stream comes after whatever still uses them).  A block given
// back on another stream is taken only after that stream has drained, and never while the current stream
// is being captured (a wait is not allowed there): then fresh memory is asked for instead.
void *dev_alloc(size_t bytes) {
    size_t sz = bin_size(bytes);
    if (g_user_alloc) {
        void *p = g_user_alloc(sz, g_user_ctx);
        if (!p) {
            fail(TS_ERR_OOM, "the caller's allocator returned NULL for %zu bytes", sz);
            return nullptr;
        }
        std::lock_guard<std::mutex> lk(g_pool_mu);
        g_foreign_blocks[p] = Foreign{g_user_release, g_user_ctx};
        return p;
    }
    {
        std::unique_lock<std::mutex> lk(g_pool_mu);
        auto foreign = g_free_blocks.end();
        for (auto it = g_free_blocks.lower_bound(sz); it != g_free_blocks.end() && it->first <= sz + sz / 4; ++it) {
            if (it->second.stream == g_stream) {
                void *p = it->second.p;
                g_live_blocks[p] = it->first;
                g_free_blocks.erase(it);
                return p;
            }
            if (foreign == g_free_blocks.end()) foreign = it;
        }
        if (foreign != g_free_blocks.end() && !capturing()) {
            const FreeBlock b = foreign->second;
            const size_t bsz = foreign->first;
            g_free_blocks.erase(foreign);
            g_live_blocks[b.p] = bsz;
            lk.unlock();
            if (hipStreamSynchronize(b.stream) != hipSuccess) {   // e.g. a stream that no longer exists
                (void)hipGetLastError();
                (void)hipDeviceSynchronize();
            }
            return b.p;
        }
    }
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, sz);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        fail(e == hipErrorOutOfMemory ? TS_ERR_OOM : TS_ERR_HIP, "hipMalloc(%zu) failed: %s", sz,
             hipGetErrorString(e));
        return nullptr;
    }
    std::lock_guard<std::mutex> lk(g_pool_mu);
    g_live_blocks[p] = sz;
    return p;
}

void dev_free(void *p) {
    if (!p) return;
    {
        std::unique_lock<std::mutex> lk(g_pool_mu);
        auto f = g_foreign_blocks.find(p);
        if (f != g_foreign_blocks.end()) {
            const Foreign how = f->second;
            g_foreign_blocks.erase(f);
            lk.unlock();
            if (how.release) how.release(p, how.ctx);
            return;
        }
    }
    std::lock_guard<std::mutex> lk(g_pool_mu);
    auto it = g_live_blocks.find(p);
    if (it == g_live_blocks.end()) return;
    g_free_blocks.emplace(it->second, FreeBlock{p, g_stream});
    g_live_blocks.erase(it);
}

// A scratch area that is too small is replaced by a larger one (half as large again, so that the areas
// left behind add up to less than twice the last).  The old area is NOT reused for anything until
// ts_release_cache: work already enqueued, or a HIP graph captured earlier, may still address it.  Nothing
// waits here.  While the stream is being captured no memory can be asked for: the call fails instead, and
// the caller sizes the areas with one eager pass first.
void *scratch(int slot, size_t bytes) {
    Scratch &s = g_scratch[slot];
    if (s.bytes >= bytes && s.p) return s.p;
    if (capturing()) {
        fail(TS_ERR_UNSUPPORTED, "library scratch area %d must grow to %zu bytes, which cannot happen while the stream is being captured: run the same call once before capturing", slot, bytes);
        return nullptr;
    }
    size_t want = bytes + bytes / 2;
    void *p = nullptr;
    bool foreign = false;
    Foreign how = {nullptr, nullptr};
    if (g_user_alloc) {
        p = g_user_alloc(want, g_user_ctx);
        if (!p) {
            fail(TS_ERR_OOM, "the caller's allocator returned NULL for %zu bytes", want);
            return nullptr;
        }
        foreign = true;
        how = Foreign{g_user_release, g_user_ctx};
    } else {
        hipError_t e = hipMalloc(&p, want);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            want = bytes;
            e = hipMalloc(&p, want);
        }
        if (e != hipSuccess) {
            (void)hipGetLastError();
            fail(e == hipErrorOutOfMemory ? TS_ERR_OOM : TS_ERR_HIP, "hipMalloc(%zu) failed: %s", want, hipGetErrorString(e));
            return nullptr;
        }
    }
    if (s.p) {
        std::lock_guard<std::mutex> lk(g_pool_mu);
        g_retired.push_back(Retired{s.p, s.foreign, s.how});
    }
    s.p = p;
    s.bytes = want;
    s.foreign = foreign;
    s.how = how;
    return s.p;
}

const void *zero_row() {
    static void *z = nullptr;
    if (z) return z;
    void *p = nullptr;
    if (hipMalloc(&p, 4096) != hipSuccess || hipMemset(p, 0, 4096) != hipSuccess) {
        (void)hipGetLastError();
        fail(TS_ERR_OOM, "allocating the zero row failed");
        return nullptr;
    }
    z = p;
    return z;
}

void *host_staging(size_t bytes) {
    if (g_host_bytes >= bytes) return g_host;
    if (g_host) (void)hipHostFree(g_host);
    g_host = nullptr;
    g_host_bytes = 0;
    size_t want = bytes < 4096 ? 4096 : bytes;
    if (hipHostMalloc(&g_host, want, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        fail(TS_ERR_OOM, "hipHostMalloc(%zu) failed", want);
        return nullptr;
    }
    g_host_bytes = want;
    return g_host;
}

// ---- per-kernel timing --------------------------------------------------------------------------
namespace {
struct ProfRec {
    const char *name;
    hipEvent_t a, b;
};
bool g_prof_on = false;
std::string g_prof_filter;
std::vector<ProfRec> g_prof_recs;
std::vector<hipEvent_t> g_prof_free_events;

hipEvent_t prof_event() {
    if (!g_prof_free_events.empty()) {
        hipEvent_t e = g_prof_free_events.back();
        g_prof_free_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}
}  // namespace

ProfScope::ProfScope(const char *name) : rec_(-1) {
    if (!g_prof_on) return;
    if (!g_prof_filter.empty() && strncmp(name, g_prof_filter.c_str(), g_prof_filter.size()) != 0) return;
    ProfRec r{name, prof_event(), prof_event()};
    if (!r.a || !r.b) return;
    (void)hipEventRecord(r.a, g_stream);
    g_prof_recs.push_back(r);
    rec_ = (int)g_prof_recs.size() - 1;
}

ProfScope::~ProfScope() {
    if (rec_ >= 0) (void)hipEventRecord(g_prof_recs[rec_].b, g_stream);
}

ProfPair prof_pair(const char *name) {
    ProfPair pp;
    if (!g_prof_on) return pp;
    if (!g_prof_filter.empty() && strncmp(name, g_prof_filter.c_str(), g_prof_filter.size()) != 0) return pp;
    ProfRec r{name, prof_event(), prof_event()};
    if (!r.a || !r.b) return pp;
    g_prof_recs.push_back(r);
    pp.a = r.a;
    pp.b = r.b;
    return pp;
}

}  // namespace ts

// Plain streaming copy, 16 bytes per thread per step (grid-stride).
__global__ void k_copy_bytes(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n_vec) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n_vec; i += stride) dst[i] = src[i];
}

// Register-only loop of fp16 MFMAs (v_mfma_f32_16x16x32_f16), eight independent accumulators per wave:
// what the matrix pipes sustain when nothing else is in the way.
typedef _Float16 mfma_half8 __attribute__((ext_vector_type(8)));
typedef float mfma_float4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) k_mfma_loop(int iters, float *__restrict__ sink) {
    mfma_half8 a, b;
    for (int e = 0; e < 8; ++e) {
        a[e] = (_Float16)(0.001f * (float)((threadIdx.x + e) & 7));
        b[e] = (_Float16)(0.002f * (float)((threadIdx.x * 3 + e) & 7));
    }
    mfma_float4 acc[8];
    for (int q = 0; q < 8; ++q) acc[q] = mfma_float4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[q], 0, 0, 0);
    }
    float total = 0.f;
    for (int q = 0; q < 8; ++q) total += acc[q][0] + acc[q][1] + acc[q][2] + acc[q][3];
    if (total == -1.f) sink[blockIdx.x * blockDim.x + threadIdx.x] = total;   // never true: keeps the loop alive
}

extern "C" {

int ts_mfma_loop(int iters, void *sink, double *flops) {
    if (!sink || !flops) return ts::fail(TS_ERR_INVALID_ARG, "NULL pointer");
    if (iters < 1 || iters > (1 << 20)) return ts::fail(TS_ERR_INVALID_ARG, "iters must be in [1, 2^20]");
    const int blocks = 256 * 4;   // four workgroups of four waves per CU: four waves per SIMD
    TS_LAUNCH("k_mfma_loop", k_mfma_loop, dim3(blocks), dim3(256), iters, static_cast<float *>(sink));
    TS_HIP(hipGetLastError());
    *flops = (double)blocks * 4.0 * (double)iters * 8.0 * (2.0 * 16 * 16 * 32);
    return TS_OK;
}

int ts_copy_bytes(void *dst, const void *src, size_t bytes) {
    if (!dst || !src) return ts::fail(TS_ERR_INVALID_ARG, "NULL pointer");
    if ((bytes & 15) || (reinterpret_cast<uintptr_t>(dst) & 15) || (reinterpret_cast<uintptr_t>(src) & 15))
        return ts::fail(TS_ERR_INVALID_ARG, "pointers and size must be multiples of 16 bytes");
    if (bytes == 0) return TS_OK;
    const size_t n_vec = bytes / 16;
    size_t blocks = (n_vec + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;   // 32 workgroups per CU, grid-stride beyond that
    TS_LAUNCH("k_copy_bytes", k_copy_bytes, dim3((unsigned)blocks), dim3(256), static_cast<const uint4 *>(src),
              static_cast<uint4 *>(dst), n_vec);
    TS_HIP(hipGetLastError());
    return TS_OK;
}

int ts_profile_enable(int on, const char *only) {
    ts::g_prof_on = on != 0;
    ts::g_prof_filter = only ? only : "";
    return TS_OK;
}

int ts_profile_read(char *buf, size_t cap) {
    if (!buf || cap == 0) return ts::fail(TS_ERR_INVALID_ARG, "buf is NULL or empty");
    TS_HIP(hipStreamSynchronize(ts::g_stream));
    std::map<std::string, std::pair<long, double>> agg;
    std::vector<std::string> order;
    for (auto &r : ts::g_prof_recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) {
            (void)hipGetLastError();
            ms = 0.f;
        }
        auto it = agg.find(r.name);
        if (it == agg.end()) {
            order.push_back(r.name);
            agg[r.name] = {1, (double)ms};
        } else {
            it->second.first += 1;
            it->second.second += ms;
        }
        ts::g_prof_free_events.push_back(r.a);
        ts::g_prof_free_events.push_back(r.b);
    }
    ts::g_prof_recs.clear();
    std::string text;
    char line[256];
    for (auto &name : order) {
        snprintf(line, sizeof(line), "%s %ld %.6f\n", name.c_str(), agg[name].first, agg[name].second);
        text += line;
    }
    if (text.size() + 1 > cap) return ts::fail(TS_ERR_INVALID_ARG, "buffer too small: need %zu bytes", text.size() + 1);
    memcpy(buf, text.c_str(), text.size() + 1);
    return TS_OK;
}

int ts_set_stream(void *hip_stream) {
    ts::g_stream = static_cast<hipStream_t>(hip_stream);
    return TS_OK;
}

int ts_set_allocator(void *(*alloc)(size_t, void *), void (*release)(void *, void *), void *ctx) {
    if ((alloc == nullptr) != (release == nullptr)) return ts::fail(TS_ERR_INVALID_ARG, "alloc and release must both be given, or both be NULL");
    std::lock_guard<std::mutex> lk(ts::g_pool_mu);
    ts::g_user_alloc = alloc;
    ts::g_user_release = release;
    ts::g_user_ctx = ctx;
    return TS_OK;
}

int ts_release_cache(void) {
    TS_HIP(hipDeviceSynchronize());
    ts::release_grid();
    std::lock_guard<std::mutex> lk(ts::g_pool_mu);
    for (auto &s : ts::g_scratch) {
        if (s.p) {
            if (s.foreign) {
                if (s.how.release) s.how.release(s.p, s.how.ctx);
            } else {
                (void)hipFree(s.p);
            }
        }
        s = ts::Scratch();
    }
    for (auto &r : ts::g_retired) {
        if (r.foreign) {
            if (r.how.release) r.how.release(r.p, r.how.ctx);
        } else {
            (void)hipFree(r.p);
        }
    }
    ts::g_retired.clear();
    for (auto &kv : ts::g_free_blocks) (void)hipFree(kv.second.p);
    ts::g_free_blocks.clear();
    return TS_OK;
}

const char *ts_last_error(void) { return ts::g_error.c_str(); }

const char *ts_version(void) { return "libts 0.1 (gfx950)"; }

}  // extern "C"
