// LARS with momentum over the flat parameter buffer (the optimizer of the paper's training configuration,
// Sec. 3.2: coefficient 0.01, eps 1e-6, FP32 arithmetic on FP16 gradients).
//
// Per layer tensor (segment) l, with g' = float(g)*grad_scale:
//     rate_l = eta*||w_l|| / (||g'_l|| + wd*||w_l|| + eps)           (1 if either norm is zero)
//     v <- mu*v + lr*rate_l*(g' + wd*w) ;  w <- w - v
// and for segments excluded from the layer-wise scaling (BN scale / shift, biases):
//     v <- mu*v + lr*g' ;  w <- w - v
//
// Three launches: (1) every workgroup covers up to 2048 consecutive elements of ONE segment and leaves
// (sum w^2, sum g'^2) of them; (2) one wavefront per segment adds its workgroups' sums in a fixed order in
// double and turns them into the segment's step scale lr*rate_l and decay; (3) the same workgroup table
// drives the streaming update.  26 bytes per parameter (6 for the norms, 20 for the update) with an FP16
// gradient; no atomics, so results do not depend on timing.
//
// Contraction is off so that the update arithmetic is evaluated as written (as in the momentum-SGD kernel).
#include <algorithm>
#include <utility>
#include <vector>

#include "common.h"
#include "misc_internal.h"
#include "prof.h"
#pragma clang fp contract(off)

struct LarsBlock { unsigned long long begin; unsigned count; int seg; };

struct lars_plan {
    int nseg = 0, nblocks = 0;
    LarsBlock* blocks = nullptr;          // device, nblocks
    int* seg_first = nullptr;             // device, nseg + 1: first workgroup of every segment
    int* seg_use = nullptr;               // device, nseg: layer-wise scaling on / off
    float* partial = nullptr;             // device, nblocks x 2
    float* scale = nullptr;               // device, nseg x 2: (lr*rate, decay)
    double covered = 0;                   // elements in all segments
};

namespace {

constexpr int kThreads = 256;
constexpr unsigned kBlockElems = kThreads * 8;

struct Layout { size_t blocks_off, first_off, use_off, partial_off, scale_off, total; int nblocks; };

bool lars_layout(const rn50_lars_segment* segs, int nseg, Layout& L)
{
    long long nb = 0;
    for (int i = 0; i < nseg; ++i) {
        if (segs[i].offset % 8 != 0) return false;
        nb += (long long)((segs[i].count + kBlockElems - 1) / kBlockElems);
    }
    if (nb > (1ll << 30)) return false;
    L.nblocks = (int)nb;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += rn50_round_up(bytes, 256); return o; };
    L.blocks_off = take((size_t)(nb > 0 ? nb : 1) * sizeof(LarsBlock));
    L.first_off = take((size_t)(nseg + 1) * sizeof(int));
    L.use_off = take((size_t)(nseg > 0 ? nseg : 1) * sizeof(int));
    L.partial_off = take((size_t)(nb > 0 ? nb : 1) * 2 * sizeof(float));
    L.scale_off = take((size_t)(nseg > 0 ? nseg : 1) * 2 * sizeof(float));
    L.total = off;
    return true;
}

__device__ __forceinline__ void load8(const h16* g, size_t i, float (&out)[8])
{
    const h16x8 gh = *reinterpret_cast<const h16x8*>(g + i);
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = (float)gh[j];
}

__global__ __launch_bounds__(kThreads) void lars_norm_kernel(const LarsBlock* __restrict__ blocks,
                                                             const int* __restrict__ seg_use, const h16* __restrict__ g,
                                                             float grad_scale, const float* __restrict__ w,
                                                             float* __restrict__ partial)
{
    __shared__ float red[2][kThreads / 64];
    const LarsBlock b = blocks[blockIdx.x];
    if (!seg_use[b.seg]) return;                       // plain segment: no norms needed
    const unsigned e0 = threadIdx.x * 8;
    float sw = 0.f, sg = 0.f;
    if (e0 + 8 <= b.count) {
        const size_t i = (size_t)b.begin + e0;
        float gv[8];
        load8(g, i, gv);
        const f32x4 w0 = *reinterpret_cast<const f32x4*>(w + i), w1 = *reinterpret_cast<const f32x4*>(w + i + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = gv[j] * grad_scale, c = gv[4 + j] * grad_scale;
            sw += w0[j] * w0[j]; sw += w1[j] * w1[j];
            sg += a * a; sg += c * c;
        }
    } else {
        for (unsigned e = e0; e < b.count; ++e) {
            const float a = (float)g[(size_t)b.begin + e] * grad_scale;
            const float x = w[(size_t)b.begin + e];
            sw += x * x; sg += a * a;
        }
    }
    sw = wave_sum(sw); sg = wave_sum(sg);
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = sw; red[1][threadIdx.x >> 6] = sg; }
    __syncthreads();
    if (threadIdx.x < 2) {
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < kThreads / 64; ++k) s += red[threadIdx.x][k];
        partial[(size_t)blockIdx.x * 2 + threadIdx.x] = s;
    }
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// one wavefront per segment
__global__ __launch_bounds__(64) void lars_rate_kernel(int nseg, const int* __restrict__ seg_first,
                                                       const int* __restrict__ seg_use, const float* __restrict__ partial,
                                                       float lr, float wd, float eta, float eps, float* __restrict__ scale,
                                                       float* __restrict__ rates_out)
{
    const int seg = blockIdx.x;
    const int lane = threadIdx.x;
    float rate = 1.f, decay = 0.f;
    if (seg_use[seg]) {
        double sw = 0.0, sg = 0.0;
        for (int k = seg_first[seg] + lane; k < seg_first[seg + 1]; k += 64) {
            sw += (double)partial[(size_t)k * 2];
            sg += (double)partial[(size_t)k * 2 + 1];
        }
        sw = wave_sum_f64(sw); sg = wave_sum_f64(sg);
        const float nw = (float)sqrt(sw), ng = (float)sqrt(sg);
        if (nw > 0.f && ng > 0.f) rate = eta * nw / (ng + wd * nw + eps);
        decay = wd;
    }
    if (lane == 0) {
        scale[seg * 2] = lr * rate;
        scale[seg * 2 + 1] = decay;
        if (rates_out) rates_out[seg] = rate;
    }
}

template <bool kWriteLowp>
__global__ __launch_bounds__(kThreads) void lars_update_kernel(const LarsBlock* __restrict__ blocks,
                                                               const float* __restrict__ scale, const h16* __restrict__ g,
                                                               float grad_scale, float* __restrict__ w,
                                                               float* __restrict__ v, h16* __restrict__ w16, float mu)
{
    const LarsBlock b = blocks[blockIdx.x];
    const float step = scale[b.seg * 2], decay = scale[b.seg * 2 + 1];
    const unsigned e0 = threadIdx.x * 8;
    if (e0 + 8 <= b.count) {
        const size_t i = (size_t)b.begin + e0;
        float gv[8];
        h16x8 lo;
        load8(g, i, gv);
        f32x4 w0 = *reinterpret_cast<const f32x4*>(w + i), w1 = *reinterpret_cast<const f32x4*>(w + i + 4);
        f32x4 v0 = *reinterpret_cast<const f32x4*>(v + i), v1 = *reinterpret_cast<const f32x4*>(v + i + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float gp = gv[j] * grad_scale + decay * w0[j];
            v0[j] = mu * v0[j] + step * gp;
            w0[j] = w0[j] - v0[j];
            lo[j] = (h16)w0[j];
            gp = gv[4 + j] * grad_scale + decay * w1[j];
            v1[j] = mu * v1[j] + step * gp;
            w1[j] = w1[j] - v1[j];
            lo[4 + j] = (h16)w1[j];
        }
        *reinterpret_cast<f32x4*>(w + i) = w0; *reinterpret_cast<f32x4*>(w + i + 4) = w1;
        *reinterpret_cast<f32x4*>(v + i) = v0; *reinterpret_cast<f32x4*>(v + i + 4) = v1;
        if (kWriteLowp) *reinterpret_cast<h16x8*>(w16 + i) = lo;
    } else {
        for (unsigned e = e0; e < b.count; ++e) {
            const size_t i = (size_t)b.begin + e;
            const float gp = (float)g[i] * grad_scale + decay * w[i];
            const float vn = mu * v[i] + step * gp;
            const float wn = w[i] - vn;
            v[i] = vn; w[i] = wn;
            if (kWriteLowp) w16[i] = (h16)wn;
        }
    }
}

}  // namespace

extern "C" size_t lars_workspace_bytes(const rn50_lars_segment* segs, int nseg)
{
    Layout L;
    if ((nseg > 0 && !segs) || nseg < 0 || !lars_layout(segs, nseg, L)) return 0;
    return L.total;
}

extern "C" int lars_plan_create(lars_plan** out, const rn50_lars_segment* segs, int nseg, void* workspace,
                                size_t workspace_bytes)
{
    if (!out) return RN50_ERR_NULL;
    *out = nullptr;
    if (nseg < 0 || (nseg > 0 && !segs)) return RN50_ERR_NULL;
    Layout L;
    if (!lars_layout(segs, nseg, L)) return RN50_ERR_SHAPE;
    if (!workspace || workspace_bytes < L.total) return RN50_ERR_WORKSPACE;
    if (!rn50_aligned16(workspace)) return RN50_ERR_ALIGN;
    // segments must not overlap (two workgroups would update the same element)
    {
        std::vector<std::pair<size_t, size_t>> iv;
        for (int i = 0; i < nseg; ++i) if (segs[i].count) iv.push_back({segs[i].offset, segs[i].offset + segs[i].count});
        std::sort(iv.begin(), iv.end());
        for (size_t i = 1; i < iv.size(); ++i) if (iv[i].first < iv[i - 1].second) return RN50_ERR_SHAPE;
    }
    std::vector<LarsBlock> blocks;
    std::vector<int> first(nseg + 1, 0), use(nseg > 0 ? nseg : 1, 0);
    size_t covered = 0;
    for (int i = 0; i < nseg; ++i) {
        first[i] = (int)blocks.size();
        use[i] = segs[i].use_lars ? 1 : 0;
        for (size_t o = 0; o < segs[i].count; o += kBlockElems) {
            const size_t c = segs[i].count - o < kBlockElems ? segs[i].count - o : kBlockElems;
            blocks.push_back({(unsigned long long)(segs[i].offset + o), (unsigned)c, i});
        }
        covered += segs[i].count;
    }
    first[nseg] = (int)blocks.size();
    lars_plan* p = new lars_plan();
    char* base = static_cast<char*>(workspace);
    p->nseg = nseg; p->nblocks = (int)blocks.size();
    p->blocks = reinterpret_cast<LarsBlock*>(base + L.blocks_off);
    p->seg_first = reinterpret_cast<int*>(base + L.first_off);
    p->seg_use = reinterpret_cast<int*>(base + L.use_off);
    p->partial = reinterpret_cast<float*>(base + L.partial_off);
    p->scale = reinterpret_cast<float*>(base + L.scale_off);
    p->covered = (double)covered;
    hipError_t e = hipSuccess;
    if (!blocks.empty()) e = hipMemcpy(p->blocks, blocks.data(), blocks.size() * sizeof(LarsBlock), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(p->seg_first, first.data(), first.size() * sizeof(int), hipMemcpyHostToDevice);
    if (e == hipSuccess && nseg > 0) e = hipMemcpy(p->seg_use, use.data(), (size_t)nseg * sizeof(int), hipMemcpyHostToDevice);
    if (e != hipSuccess) { delete p; return rn50_hip_fail(e); }
    *out = p;
    return RN50_OK;
}

extern "C" void lars_plan_destroy(lars_plan* plan) { delete plan; }

int rn50_lars_launch(const lars_plan* p, const h16* grad, float grad_scale, float* w, float* v, h16* w16, float lr, float mu,
                     float wd, float eta, float eps, float* rates_out, hipStream_t s)
{
    if (p->nblocks == 0) return RN50_OK;
    {
        ProfScope ps(RN50_K_LARS_NORM, 0.0, 6.0 * p->covered, s);
        lars_norm_kernel<<<p->nblocks, kThreads, 0, s>>>(p->blocks, p->seg_use, grad, grad_scale, w, p->partial);
        RN50_TRY(rn50_check_launch());
    }
    {
        ProfScope ps(RN50_K_LARS_RATE, 0.0, 8.0 * p->nblocks, s);
        lars_rate_kernel<<<p->nseg, 64, 0, s>>>(p->nseg, p->seg_first, p->seg_use, p->partial, lr, wd, eta, eps, p->scale, rates_out);
        RN50_TRY(rn50_check_launch());
    }
    ProfScope ps(RN50_K_LARS_UPDATE, 0.0, (18.0 + (w16 ? 2.0 : 0.0)) * p->covered, s);
    if (w16) lars_update_kernel<true><<<p->nblocks, kThreads, 0, s>>>(p->blocks, p->scale, grad, grad_scale, w, v, w16, mu);
    else lars_update_kernel<false><<<p->nblocks, kThreads, 0, s>>>(p->blocks, p->scale, grad, grad_scale, w, v, nullptr, mu);
    return rn50_check_launch();
}

extern "C" int lars_momentum_flat(const lars_plan* plan, const void* grad, int grad_dt, float grad_scale, float* master_w,
                                  float* momentum, void* w_lowp_out, float lr, float mu, float wd, float eta, float eps,
                                  float* rates_out, void* stream)
{
    RN50_REQUIRE_PTR(plan);
    if (grad_dt != RN50_F16) return RN50_ERR_DTYPE;
    if (plan->nblocks == 0) return RN50_OK;
    RN50_REQUIRE_PTR(grad); RN50_REQUIRE_PTR(master_w); RN50_REQUIRE_PTR(momentum);
    RN50_REQUIRE_ALIGNED(grad); RN50_REQUIRE_ALIGNED(master_w); RN50_REQUIRE_ALIGNED(momentum);
    RN50_REQUIRE_ALIGNED(w_lowp_out);
    if (!(eta > 0.f) || eps < 0.f) return RN50_ERR_SHAPE;
    return rn50_lars_launch(plan, static_cast<const h16*>(grad), grad_scale, master_w, momentum, static_cast<h16*>(w_lowp_out),
                            lr, mu, wd, eta, eps, rates_out, static_cast<hipStream_t>(stream));
}
