// Softmax cross-entropy with label smoothing: loss and gradient w.r.t. the logits in one
// launch.  One workgroup of 16 wavefronts; each wavefront owns rows i = wave, wave+16, ...
// and keeps its partial loss in a fixed order, so the result is deterministic.
#include "common.h"
#include "prof.h"

namespace {

constexpr int kWaves = 16;
constexpr int kCache = 16;   // logits per lane kept in registers (rows of up to 1024 classes)

__global__ __launch_bounds__(kWaves * 64) void ls_xent_kernel(
    int batch, int classes, const float* __restrict__ logits, const int32_t* __restrict__ labels,
    float eps, float grad_scale, float* __restrict__ loss_mean, float* __restrict__ loss_per_sample,
    h16* __restrict__ dlogits)
{
    __shared__ float wave_total[kWaves];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float q_off = eps / (float)classes;
    float my_total = 0.f;   // identical on every lane of the wave
    for (int i = wave; i < batch; i += kWaves) {
        const float* z = logits + (size_t)i * classes;
        // the lane's logits are read once into registers when the row is short enough (<= 64*kCache)
        float zc[kCache];
        const bool cached = classes <= 64 * kCache;
        float m = -INFINITY;
        if (cached) {
#pragma unroll
            for (int u = 0; u < kCache; ++u) {
                const int k = lane + 64 * u;
                zc[u] = k < classes ? z[k] : -INFINITY;
                m = fmaxf(m, zc[u]);
            }
        } else {
            for (int k = lane; k < classes; k += 64) m = fmaxf(m, z[k]);
        }
        m = wave_max(m);
        float se = 0.f;
        if (cached) {
#pragma unroll
            for (int u = 0; u < kCache; ++u) se += expf(zc[u] - m);      // exp(-inf) = 0 for the padding
        } else {
            for (int k = lane; k < classes; k += 64) se += expf(z[k] - m);
        }
        se = wave_sum(se);
        const float lse = m + logf(se);
        const int label = labels[i];
        float li = 0.f;
        auto one = [&](int k, float zk) {
            const float logp = zk - lse;
            const float q = (k == label ? 1.f - eps : 0.f) + q_off;
            li -= q * logp;
            dlogits[(size_t)i * classes + k] = (h16)((expf(logp) - q) * grad_scale);
        };
        if (cached) {
#pragma unroll
            for (int u = 0; u < kCache; ++u) {
                const int k = lane + 64 * u;
                if (k < classes) one(k, zc[u]);
            }
        } else {
            for (int k = lane; k < classes; k += 64) one(k, z[k]);
        }
        li = wave_sum(li);
        if (loss_per_sample && lane == 0) loss_per_sample[i] = li;
        my_total += li;
    }
    if (lane == 0) wave_total[wave] = my_total;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < kWaves; ++w) t += wave_total[w];
        *loss_mean = t / (float)batch;
    }
}

}  // namespace

extern "C" int ls_xent_fwd_bwd(int batch, int classes, const float* logits, const int32_t* labels,
                               float eps, float grad_scale, float* loss_mean, float* loss_per_sample,
                               void* dlogits, int dlogits_dt, void* stream)
{
    if (dlogits_dt != RN50_F16) return RN50_ERR_DTYPE;
    if (batch < 1 || batch > 65536 || classes < 2 || classes > 65536) return RN50_ERR_SHAPE;
    RN50_REQUIRE_PTR(logits); RN50_REQUIRE_PTR(labels); RN50_REQUIRE_PTR(loss_mean); RN50_REQUIRE_PTR(dlogits);
    RN50_REQUIRE_ALIGNED(logits); RN50_REQUIRE_ALIGNED(dlogits);
    ProfScope ps(RN50_K_LOSS, 0.0, 6.0 * batch * classes, static_cast<hipStream_t>(stream));
    ls_xent_kernel<<<1, kWaves * 64, 0, static_cast<hipStream_t>(stream)>>>(
        batch, classes, logits, labels, eps, grad_scale, loss_mean, loss_per_sample, static_cast<h16*>(dlogits));
    return rn50_check_launch();
}
