// Max-pool 3x3/2, global average pool and the fully connected layer (forward and backward).
// All of them are small next to the convolutions; they are written for coalesced 16-byte
// accesses on NHWC data (a thread owns 8 consecutive channels).
#include "common.h"
#include "misc_internal.h"
#include "prof.h"

namespace {

constexpr int kThreads = 256;

// y = max over the 3x3 window (stride 2, pad 1); padding never wins.  arg = index (r*3+s) of the
// FIRST maximum in row-major window order, kept for the backward pass.
__global__ __launch_bounds__(kThreads) void maxpool_fwd_kernel(int N, int H, int W, int C, int P, int Q,
                                                               const h16* __restrict__ x, h16* __restrict__ y,
                                                               uint8_t* __restrict__ arg)
{
    const int G = C / 8;
    const size_t total = (size_t)N * P * Q * G;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
        const int g = (int)(i % G);
        size_t t = i / G;
        const int q = (int)(t % Q); t /= Q;
        const int p = (int)(t % P);
        const int n = (int)(t / P);
        h16x8 best;
        uint8_t bi[8];
        bool have = false;
        for (int r = 0; r < 3; ++r) {
            const int ih = 2 * p - 1 + r;
            if ((unsigned)ih >= (unsigned)H) continue;
            for (int s = 0; s < 3; ++s) {
                const int iw = 2 * q - 1 + s;
                if ((unsigned)iw >= (unsigned)W) continue;
                const h16x8 v = *reinterpret_cast<const h16x8*>(x + (((size_t)n * H + ih) * W + iw) * C + g * 8);
                if (!have) {
                    best = v;
#pragma unroll
                    for (int j = 0; j < 8; ++j) bi[j] = (uint8_t)(r * 3 + s);
                    have = true;
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (v[j] > best[j]) { best[j] = v[j]; bi[j] = (uint8_t)(r * 3 + s); }
                }
            }
        }
        *reinterpret_cast<h16x8*>(y + i * 8) = best;
        uint2 packed;
        packed.x = bi[0] | (bi[1] << 8) | (bi[2] << 16) | ((uint32_t)bi[3] << 24);
        packed.y = bi[4] | (bi[5] << 8) | (bi[6] << 16) | ((uint32_t)bi[7] << 24);
        *reinterpret_cast<uint2*>(arg + i * 8) = packed;
    }
}

// dx[n,h,w,c] = sum of dy over the (at most 4) windows whose recorded first maximum is (h,w).
// One workgroup row (blockIdx.x) per image row; all four candidate windows are requested at once (an even
// coordinate has one candidate per axis: the second request then repeats the first and is ignored).
__global__ __launch_bounds__(kThreads) void maxpool_bwd_kernel(int H, int W, int C, int P, int Q,
                                                               const h16* __restrict__ dy,
                                                               const uint8_t* __restrict__ arg, h16* __restrict__ dx)
{
    const int G = C / 8;
    const int idx = blockIdx.y * kThreads + threadIdx.x;
    if (idx >= W * G) return;
    const int w = idx / G, g = idx - w * G;
    const int n = blockIdx.x / H, h = blockIdx.x - n * H;
    // windows p with 2p-1 <= h <= 2p+1: h/2 and, for odd h, (h+1)/2
    const int p0 = h >> 1, p1 = (h + 1) >> 1, q0 = w >> 1, q1 = (w + 1) >> 1;
    const bool vp[2] = {p0 < P, p1 != p0 && p1 < P};
    const bool vq[2] = {q0 < Q, q1 != q0 && q1 < Q};
    const int pp[2] = {vp[0] ? p0 : 0, vp[1] ? p1 : 0}, qq[2] = {vq[0] ? q0 : 0, vq[1] ? q1 : 0};
    uint2 packed[4];
    h16x8 d[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const size_t o = (((size_t)n * P + pp[k >> 1]) * Q + qq[k & 1]) * C + g * 8;
        packed[k] = *reinterpret_cast<const uint2*>(arg + o);
        d[k] = *reinterpret_cast<const h16x8*>(dy + o);
    }
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 4; ++k) {                           // same order as the window loops: p outer, q inner
        if (!(vp[k >> 1] && vq[k & 1])) continue;
        const int r = h - (2 * pp[k >> 1] - 1), sx = w - (2 * qq[k & 1] - 1);
        const uint32_t me = (uint32_t)(r * 3 + sx);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t a = ((j < 4 ? packed[k].x : packed[k].y) >> ((j & 3) * 8)) & 0xffu;
            if (a == me) acc[j] += (float)d[k][j];
        }
    }
    h16x8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (h16)acc[j];
    *reinterpret_cast<h16x8*>(dx + (((size_t)n * H + h) * W + w) * C + g * 8) = o;
}

__global__ __launch_bounds__(kThreads) void avgpool_fwd_kernel(int N, int HW, int C, const h16* __restrict__ x,
                                                               h16* __restrict__ y)
{
    const int G = C / 8;
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N * G) return;
    const int g = i % G, n = i / G;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int k = 0;
    for (; k + 7 <= HW; k += 7) {                       // 7 independent loads in flight
        h16x8 v[7];
#pragma unroll
        for (int u = 0; u < 7; ++u) v[u] = *reinterpret_cast<const h16x8*>(x + ((size_t)n * HW + k + u) * C + g * 8);
#pragma unroll
        for (int u = 0; u < 7; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += (float)v[u][j];
    }
    for (; k < HW; ++k) {
        const h16x8 v = *reinterpret_cast<const h16x8*>(x + ((size_t)n * HW + k) * C + g * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += (float)v[j];
    }
    h16x8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (h16)(acc[j] / (float)HW);
    *reinterpret_cast<h16x8*>(y + (size_t)i * 8) = o;
}

// z[i,j] = sum_c a[i,c]*Wt[j,c] + b[j].  One wavefront per (output column j, group of 8 rows): the
// lane's chunks of the weight row stay in registers, the 8 rows' loads are independent, and each dot
// product is finished by a wavefront reduction.  Cin must be a multiple of 8.
constexpr int kFcRows = 8;
__global__ __launch_bounds__(kThreads) void fc_fwd_kernel(int B, int Cin, int Cout, const h16* __restrict__ a,
                                                          const h16* __restrict__ Wt, const float* __restrict__ bias,
                                                          float* __restrict__ z)
{
    const int lane = threadIdx.x & 63;
    const int row_groups = (B + kFcRows - 1) / kFcRows;
    const int w = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (w >= Cout * row_groups) return;
    const int j = w / row_groups, i0 = (w % row_groups) * kFcRows;
    const int chunks = Cin / 8;
    float acc[kFcRows];
#pragma unroll
    for (int r = 0; r < kFcRows; ++r) acc[r] = 0.f;
    for (int c = lane; c < chunks; c += 64) {
        const h16x8 wv = *reinterpret_cast<const h16x8*>(Wt + (size_t)j * Cin + c * 8);
        h16x8 av[kFcRows];
#pragma unroll
        for (int r = 0; r < kFcRows; ++r) {
            const int i = i0 + r < B ? i0 + r : B - 1;
            av[r] = *reinterpret_cast<const h16x8*>(a + (size_t)i * Cin + c * 8);
        }
#pragma unroll
        for (int r = 0; r < kFcRows; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r] += (float)wv[e] * (float)av[r][e];
    }
#pragma unroll
    for (int r = 0; r < kFcRows; ++r) {
        const float s = wave_sum(acc[r]);
        if (lane == 0 && i0 + r < B) z[(size_t)(i0 + r) * Cout + j] = s + bias[j];
    }
}

// dWt[j,c] = sum_i dz[i,j]*a[i,c];  db[j] = sum_i dz[i,j]  (FP32 sums, stored as half)
__global__ __launch_bounds__(kThreads) void fc_bwd_w_kernel(int B, int Cin, int Cout, const h16* __restrict__ a,
                                                            const h16* __restrict__ dz, h16* __restrict__ dWt,
                                                            h16* __restrict__ db)
{
    const int G = Cin / 8;
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (size_t)Cout * G) return;
    const int g = (int)(i % G), j = (int)(i / G);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float sb = 0.f;
    for (int r = 0; r < B; ++r) {
        const float d = (float)dz[(size_t)r * Cout + j];
        const h16x8 av = *reinterpret_cast<const h16x8*>(a + (size_t)r * Cin + g * 8);
        sb += d;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += d * (float)av[e];
    }
    h16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (h16)acc[e];
    *reinterpret_cast<h16x8*>(dWt + (size_t)j * Cin + g * 8) = o;
    if (g == 0) db[j] = (h16)sb;
}

// da[i,c] = sum_j dz[i,j]*Wt[j,c] rounded to half, then spread over the HW positions of the
// average pool: dx[i,hw,c] = half(da/HW).  Workgroup = (image i, slab of 16 channel groups);
// 16 row-lanes split the classes (4 independent loads in flight each) and are combined through LDS in
// a fixed order.
__global__ __launch_bounds__(kThreads) void fc_bwd_a_avgpool_bwd_kernel(int Cin, int Cout, int HW,
                                                                        const h16* __restrict__ Wt,
                                                                        const h16* __restrict__ dz,
                                                                        h16* __restrict__ dx)
{
    __shared__ float red[16][16][8];
    const int G = Cin / 8;
    const int slabs = (G + 15) / 16;
    const int i = blockIdx.x / slabs, slab = blockIdx.x % slabs;
    const int gl = threadIdx.x & 15, jl = threadIdx.x >> 4;
    const int g = slab * 16 + gl;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (g < G) {
        int j = jl;
        for (; j + 48 < Cout; j += 64) {
            h16x8 wv[4];
            float d[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                d[u] = (float)dz[(size_t)i * Cout + j + 16 * u];
                wv[u] = *reinterpret_cast<const h16x8*>(Wt + (size_t)(j + 16 * u) * Cin + g * 8);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += d[u] * (float)wv[u][e];
        }
        for (; j < Cout; j += 16) {
            const float d = (float)dz[(size_t)i * Cout + j];
            const h16x8 wv = *reinterpret_cast<const h16x8*>(Wt + (size_t)j * Cin + g * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += d * (float)wv[e];
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[jl][gl][e] = acc[e];
    __syncthreads();
    if (g < G) {
        h16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float s = 0.f;
            for (int k = 0; k < 16; ++k) s += red[k][gl][e];
            const h16 da = (h16)s;
            o[e] = (h16)((float)da / (float)HW);
        }
        for (int k = jl; k < HW; k += 16) *reinterpret_cast<h16x8*>(dx + ((size_t)i * HW + k) * Cin + g * 8) = o;
    }
}

int grid_for(size_t items) {
    size_t b = (items + kThreads - 1) / kThreads;
    if (b > 256 * 16) b = 256 * 16;
    return b < 1 ? 1 : (int)b;
}

}  // namespace

int rn50_maxpool_fwd(int N, int H, int W, int C, const h16* x, h16* y, uint8_t* arg, hipStream_t s)
{
    const int P = (H + 2 - 3) / 2 + 1, Q = (W + 2 - 3) / 2 + 1;
    ProfScope ps(RN50_K_POOL, 0.0, 2.0 * N * C * ((double)H * W + 1.5 * P * Q), s);
    maxpool_fwd_kernel<<<grid_for((size_t)N * P * Q * (C / 8)), kThreads, 0, s>>>(N, H, W, C, P, Q, x, y, arg);
    return rn50_check_launch();
}

int rn50_maxpool_bwd(int N, int H, int W, int C, const h16* dy, const uint8_t* arg, h16* dx, hipStream_t s)
{
    const int P = (H + 2 - 3) / 2 + 1, Q = (W + 2 - 3) / 2 + 1;
    ProfScope ps(RN50_K_POOL, 0.0, 2.0 * N * C * ((double)H * W + 1.5 * P * Q), s);
    const dim3 grid((unsigned)(N * H), (unsigned)rn50_cdiv((long long)W * (C / 8), kThreads));
    maxpool_bwd_kernel<<<grid, kThreads, 0, s>>>(H, W, C, P, Q, dy, arg, dx);
    return rn50_check_launch();
}

int rn50_avgpool_fwd(int N, int HW, int C, const h16* x, h16* y, hipStream_t s)
{
    ProfScope ps(RN50_K_POOL, 0.0, 2.0 * N * C * (HW + 1.0), s);
    avgpool_fwd_kernel<<<rn50_cdiv((long long)N * (C / 8), kThreads), kThreads, 0, s>>>(N, HW, C, x, y);
    return rn50_check_launch();
}

int rn50_fc_fwd(int B, int Cin, int Cout, const h16* a, const h16* Wt, const float* bias, float* z, hipStream_t s)
{
    ProfScope ps(RN50_K_FC, 2.0 * B * Cin * Cout, 2.0 * Cin * (B + Cout) + 4.0 * B * Cout, s);
    fc_fwd_kernel<<<rn50_cdiv((long long)Cout * ((B + kFcRows - 1) / kFcRows), kThreads / 64), kThreads, 0, s>>>(B, Cin, Cout, a,
                                                                                                                Wt, bias, z);
    return rn50_check_launch();
}

// The two halves of the FC backward pass only share dz: the weight gradient (dWt, db) may run on another stream than
// the activation gradient that the rest of the backward pass waits for.
int rn50_fc_bwd(int B, int Cin, int Cout, int HW, const h16* a, const h16* Wt, const h16* dz, h16* dWt, h16* db,
                h16* dx, hipStream_t s_weights, hipStream_t s)
{
    {
        ProfScope ps(RN50_K_FC, 2.0 * B * Cin * Cout, 2.0 * Cin * B + 2.0 * Cin * Cout, s_weights);
        fc_bwd_w_kernel<<<rn50_cdiv((long long)Cout * (Cin / 8), kThreads), kThreads, 0, s_weights>>>(B, Cin, Cout, a, dz, dWt, db);
    }
    ProfScope ps(RN50_K_FC, 2.0 * B * Cin * Cout, 2.0 * Cin * Cout + 2.0 * B * Cin * HW, s);
    const int slabs = (Cin / 8 + 15) / 16;
    fc_bwd_a_avgpool_bwd_kernel<<<B * slabs, kThreads, 0, s>>>(Cin, Cout, HW, Wt, dz, dx);
    return rn50_check_launch();
}
