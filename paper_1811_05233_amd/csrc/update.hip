// Momentum SGD over the flat parameter buffer and the FP32 -> FP16 parameter cast.
// Pure HBM streaming: 20 bytes per parameter (read g 2, w 4, v 4; write w 4, v 4, w16 2).
// Plain (temporal) 16-byte accesses: non-temporal hints measured 15-25 % slower here.
//
// Floating-point contraction is off in this file: the update is evaluated exactly as written
// (separately rounded FP32 multiplies and adds), so it matches an FP32 host evaluation bit for bit.
#include "common.h"
#include "prof.h"
#pragma clang fp contract(off)

thread_local int rn50_tls_hip_error = 0;

extern "C" int rn50_last_hip_error(void) { return rn50_tls_hip_error; }

extern "C" const char* rn50_status_string(int s) {
    switch (s) {
        case RN50_OK: return "ok";
        case RN50_ERR_NULL: return "null pointer";
        case RN50_ERR_SHAPE: return "bad or unsupported shape";
        case RN50_ERR_DTYPE: return "unsupported storage type";
        case RN50_ERR_WORKSPACE: return "workspace missing or too small";
        case RN50_ERR_ALIGN: return "pointer not 16-byte aligned";
        case RN50_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

namespace {

constexpr int kThreads = 256;

template <bool kWriteLowp>
__global__ __launch_bounds__(kThreads) void sgd_momentum_kernel(
    size_t n, const h16* __restrict__ g, float grad_scale, float* __restrict__ w, float* __restrict__ v,
    h16* __restrict__ w16, float lr, float mu, float wd)
{
    const size_t nvec = n / 8;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        const h16x8 gv = reinterpret_cast<const h16x8*>(g)[i];
        f32x4 w0 = reinterpret_cast<const f32x4*>(w)[2 * i];
        f32x4 w1 = reinterpret_cast<const f32x4*>(w)[2 * i + 1];
        f32x4 v0 = reinterpret_cast<const f32x4*>(v)[2 * i];
        f32x4 v1 = reinterpret_cast<const f32x4*>(v)[2 * i + 1];
        h16x8 lo;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float gp = (float)gv[j] * grad_scale + wd * w0[j];
            v0[j] = mu * v0[j] + gp;
            w0[j] = w0[j] - lr * v0[j];
            lo[j] = (h16)w0[j];
            gp = (float)gv[4 + j] * grad_scale + wd * w1[j];
            v1[j] = mu * v1[j] + gp;
            w1[j] = w1[j] - lr * v1[j];
            lo[4 + j] = (h16)w1[j];
        }
        reinterpret_cast<f32x4*>(w)[2 * i] = w0;
        reinterpret_cast<f32x4*>(w)[2 * i + 1] = w1;
        reinterpret_cast<f32x4*>(v)[2 * i] = v0;
        reinterpret_cast<f32x4*>(v)[2 * i + 1] = v1;
        if (kWriteLowp) reinterpret_cast<h16x8*>(w16)[i] = lo;
    }
    // ragged tail (n not a multiple of 8): one thread per element
    const size_t tail0 = nvec * 8;
    const size_t t = tail0 + (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (t < n) {
        const float gp = (float)g[t] * grad_scale + wd * w[t];
        const float vn = mu * v[t] + gp;
        const float wn = w[t] - lr * vn;
        v[t] = vn;
        w[t] = wn;
        if (kWriteLowp) w16[t] = (h16)wn;
    }
}

__global__ __launch_bounds__(kThreads) void cast_params_kernel(size_t n, const float* __restrict__ w,
                                                               h16* __restrict__ w16)
{
    const size_t nvec = n / 8;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += stride) {
        const f32x4 a = reinterpret_cast<const f32x4*>(w)[2 * i];
        const f32x4 b = reinterpret_cast<const f32x4*>(w)[2 * i + 1];
        h16x8 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) { o[j] = (h16)a[j]; o[4 + j] = (h16)b[j]; }
        reinterpret_cast<h16x8*>(w16)[i] = o;
    }
    const size_t t = nvec * 8 + (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (t < n) w16[t] = (h16)w[t];
}

int stream_grid(size_t n)
{
    const size_t nvec = n / 8 + 1;
    size_t blocks = (nvec + kThreads - 1) / kThreads;
    // one 8-element group per thread: measured faster than a capped grid with a grid-stride loop
    // (6.7 vs 5.0 TB/s on the 25.6 M-parameter buffer); the loop only matters beyond 2^31 threads
    const size_t cap = (size_t)1 << 22;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

}  // namespace

extern "C" int sgd_momentum_flat(size_t n, const void* grad, int grad_dt, float grad_scale,
                                 float* master_w, float* momentum, void* w_lowp_out,
                                 float lr, float mu, float wd, void* stream)
{
    if (grad_dt != RN50_F16) return RN50_ERR_DTYPE;
    if (n == 0) return RN50_OK;
    RN50_REQUIRE_PTR(grad); RN50_REQUIRE_PTR(master_w); RN50_REQUIRE_PTR(momentum);
    RN50_REQUIRE_ALIGNED(grad); RN50_REQUIRE_ALIGNED(master_w); RN50_REQUIRE_ALIGNED(momentum);
    RN50_REQUIRE_ALIGNED(w_lowp_out);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = stream_grid(n);
    ProfScope ps(RN50_K_SGD, 0.0, (w_lowp_out ? 20.0 : 18.0) * (double)n, s);
    if (w_lowp_out)
        sgd_momentum_kernel<true><<<grid, kThreads, 0, s>>>(n, static_cast<const h16*>(grad), grad_scale, master_w,
                                                            momentum, static_cast<h16*>(w_lowp_out), lr, mu, wd);
    else
        sgd_momentum_kernel<false><<<grid, kThreads, 0, s>>>(n, static_cast<const h16*>(grad), grad_scale, master_w,
                                                             momentum, nullptr, lr, mu, wd);
    return rn50_check_launch();
}

extern "C" int rn50_cast_params(size_t n, const float* master_w, void* w_lowp, int dt, void* stream)
{
    if (dt != RN50_F16) return RN50_ERR_DTYPE;
    if (n == 0) return RN50_OK;
    RN50_REQUIRE_PTR(master_w); RN50_REQUIRE_PTR(w_lowp);
    RN50_REQUIRE_ALIGNED(master_w); RN50_REQUIRE_ALIGNED(w_lowp);
    ProfScope ps(RN50_K_CAST, 0.0, 6.0 * (double)n, static_cast<hipStream_t>(stream));
    cast_params_kernel<<<stream_grid(n), kThreads, 0, static_cast<hipStream_t>(stream)>>>(
        n, master_w, static_cast<h16*>(w_lowp));
    return rn50_check_launch();
}
