// Elementwise steps between sparse-convolution layers of a network (not in the paper, which
// covers the convolution only): per-channel bias + optional residual + optional ReLU, and
// channel concatenation for skip connections.  fp32 arithmetic, one rounding at the store.
#include "ts_internal.h"

using namespace ts;

namespace {

constexpr int kThreads = 256;

template <class T> __device__ __forceinline__ float to_f(T v) { return (float)v; }

// out[r][c] = act(x[r][c] + bias[c] + res[r][c]); bias / res may be null.
template <class T>
__global__ void k_bias_act(const T *__restrict__ x, const T *__restrict__ bias, const T *__restrict__ res,
                           T *__restrict__ out, int64_t total, int cols, int relu) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    float v = to_f(x[i]);
    if (bias) v += to_f(bias[i % cols]);
    if (res) v += to_f(res[i]);
    if (relu && v < 0.f) v = 0.f;
    out[i] = (T)v;
}

// out[r] = [a[r], b[r]]
template <class T>
__global__ void k_concat_cols(const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ out, int64_t rows,
                              int ca, int cb) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int c = ca + cb;
    if (i >= rows * c) return;
    int64_t r = i / c;
    int col = (int)(i - r * c);
    out[i] = col < ca ? a[r * ca + col] : b[r * cb + (col - ca)];
}

// The same in 16-byte vectors, when both widths are whole vectors: va, vb = vectors per row of a, b.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ void k_concat_cols_vec(const u32x4 *__restrict__ a, const u32x4 *__restrict__ b, u32x4 *__restrict__ out,
                                  int64_t rows, int va, int vb) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int v = va + vb;
    if (i >= rows * v) return;
    int64_t r = i / v;
    int col = (int)(i - r * v);
    out[i] = col < va ? a[r * va + col] : b[r * vb + (col - va)];
}

int check(const ts_tensor *t, const char *name) {
    if (!t) return fail(TS_ERR_INVALID_ARG, "%s is NULL", name);
    if (t->dtype != TS_F32 && t->dtype != TS_F16) return fail(TS_ERR_INVALID_ARG, "%s: unknown dtype", name);
    if (t->rows < 0 || t->cols <= 0) return fail(TS_ERR_SHAPE, "%s: bad shape", name);
    if (t->rows > 0 && !t->data) return fail(TS_ERR_INVALID_ARG, "%s: data is NULL", name);
    return TS_OK;
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

}  // namespace

extern "C" {

int ts_bias_act(const ts_tensor *x, const void *bias, const ts_tensor *residual, int relu, ts_tensor *out) {
    TS_TRY(check(x, "x"));
    TS_TRY(check(out, "out"));
    if (out->rows != x->rows || out->cols != x->cols || out->dtype != x->dtype)
        return fail(TS_ERR_SHAPE, "out must have the shape and dtype of x");
    if (residual) {
        TS_TRY(check(residual, "residual"));
        if (residual->rows != x->rows || residual->cols != x->cols || residual->dtype != x->dtype)
            return fail(TS_ERR_SHAPE, "residual must have the shape and dtype of x");
    }
    const int64_t total = x->rows * x->cols;
    if (total == 0) return TS_OK;
    if (x->dtype == TS_F16)
        TS_LAUNCH("k_bias_act", k_bias_act<_Float16>, dim3(blocks_for(total)), dim3(kThreads),
                  static_cast<const _Float16 *>(x->data), static_cast<const _Float16 *>(bias),
                  residual ? static_cast<const _Float16 *>(residual->data) : nullptr,
                  static_cast<_Float16 *>(out->data), total, x->cols, relu);
    else
        TS_LAUNCH("k_bias_act", k_bias_act<float>, dim3(blocks_for(total)), dim3(kThreads),
                  static_cast<const float *>(x->data), static_cast<const float *>(bias),
                  residual ? static_cast<const float *>(residual->data) : nullptr, static_cast<float *>(out->data),
                  total, x->cols, relu);
    TS_HIP(hipGetLastError());
    return TS_OK;
}

int ts_concat_cols(const ts_tensor *a, const ts_tensor *b, ts_tensor *out) {
    TS_TRY(check(a, "a"));
    TS_TRY(check(b, "b"));
    TS_TRY(check(out, "out"));
    if (a->rows != b->rows || out->rows != a->rows || out->cols != a->cols + b->cols || a->dtype != b->dtype ||
        out->dtype != a->dtype)
        return fail(TS_ERR_SHAPE, "out must be [rows, cols(a) + cols(b)] of the common dtype");
    const int64_t total = out->rows * out->cols;
    if (total == 0) return TS_OK;
    const size_t elem = a->dtype == TS_F16 ? 2 : 4;
    const bool whole_vectors = a->cols * elem % 16 == 0 && b->cols * elem % 16 == 0 &&
                               ((reinterpret_cast<uintptr_t>(a->data) | reinterpret_cast<uintptr_t>(b->data) |
                                 reinterpret_cast<uintptr_t>(out->data)) & 15) == 0;
    if (whole_vectors) {
        const int va = (int)(a->cols * elem / 16), vb = (int)(b->cols * elem / 16);
        TS_LAUNCH("k_concat_cols", k_concat_cols_vec, dim3(blocks_for(out->rows * (va + vb))), dim3(kThreads),
                  static_cast<const u32x4 *>(a->data), static_cast<const u32x4 *>(b->data),
                  static_cast<u32x4 *>(out->data), out->rows, va, vb);
    } else if (a->dtype == TS_F16)
        TS_LAUNCH("k_concat_cols", k_concat_cols<_Float16>, dim3(blocks_for(total)), dim3(kThreads),
                  static_cast<const _Float16 *>(a->data), static_cast<const _Float16 *>(b->data),
                  static_cast<_Float16 *>(out->data), out->rows, a->cols, b->cols);
    else
        TS_LAUNCH("k_concat_cols", k_concat_cols<float>, dim3(blocks_for(total)), dim3(kThreads),
                  static_cast<const float *>(a->data), static_cast<const float *>(b->data),
                  static_cast<float *>(out->data), out->rows, a->cols, b->cols);
    TS_HIP(hipGetLastError());
    return TS_OK;
}

}  // extern "C"
