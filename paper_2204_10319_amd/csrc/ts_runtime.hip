// Runtime pieces of libts: error text, stream, pooled device memory, scratch areas.
#include "ts_internal.h"

#include <cstdarg>
#include <cstdio>
#include <map>
#include <mutex>
#include <string>
#include <unordered_map>

namespace ts {

static thread_local std::string g_error;
static hipStream_t g_stream = nullptr;

int fail(int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_error = buf;
    return code;
}

hipStream_t stream() { return g_stream; }

// ---- pooled device memory -------------------------------------------------------------------
namespace {
std::mutex g_pool_mu;
std::multimap<size_t, void *> g_free_blocks;          // size -> block
std::unordered_map<void *, size_t> g_live_blocks;     // block -> size

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
};
Scratch g_scratch[8];
void *g_host = nullptr;
size_t g_host_bytes = 0;
}  // namespace

void *dev_alloc(size_t bytes) {
    size_t sz = bin_size(bytes);
    {
        std::lock_guard<std::mutex> lk(g_pool_mu);
        auto it = g_free_blocks.lower_bound(sz);
        if (it != g_free_blocks.end() && it->first <= sz + sz / 4) {
            void *p = it->second;
            g_live_blocks[p] = it->first;
            g_free_blocks.erase(it);
            return p;
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
    std::lock_guard<std::mutex> lk(g_pool_mu);
    auto it = g_live_blocks.find(p);
    if (it == g_live_blocks.end()) return;
    g_free_blocks.emplace(it->second, p);
    g_live_blocks.erase(it);
}

void *scratch(int slot, size_t bytes) {
    Scratch &s = g_scratch[slot];
    if (s.bytes >= bytes && s.p) return s.p;
    // Work already enqueued may still read the old area: stream-ordered reuse is safe through
    // the pool only after the stream has drained.
    if (s.p) {
        (void)hipStreamSynchronize(g_stream);
        dev_free(s.p);
        s.p = nullptr;
        s.bytes = 0;
    }
    size_t want = bytes + bytes / 8;
    s.p = dev_alloc(want);
    if (s.p) s.bytes = want;
    return s.p;
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

}  // namespace ts

extern "C" {

int ts_set_stream(void *hip_stream) {
    ts::g_stream = static_cast<hipStream_t>(hip_stream);
    return TS_OK;
}

int ts_release_cache(void) {
    TS_HIP(hipDeviceSynchronize());
    std::lock_guard<std::mutex> lk(ts::g_pool_mu);
    for (auto &s : ts::g_scratch) {
        if (s.p) {
            auto it = ts::g_live_blocks.find(s.p);
            if (it != ts::g_live_blocks.end()) ts::g_live_blocks.erase(it);
            (void)hipFree(s.p);
        }
        s.p = nullptr;
        s.bytes = 0;
    }
    for (auto &kv : ts::g_free_blocks) (void)hipFree(kv.second);
    ts::g_free_blocks.clear();
    return TS_OK;
}

const char *ts_last_error(void) { return ts::g_error.c_str(); }

const char *ts_version(void) { return "libts 0.1 (gfx950)"; }

}  // extern "C"
