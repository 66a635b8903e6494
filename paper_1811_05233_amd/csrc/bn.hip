// Fused BatchNorm (+residual) (+ReLU), forward and backward, batch statistics only.
// Tensors are [m, c] half with c contiguous; a thread owns one group of 8 channels
// (one 16-byte chunk per row) and walks rows, so every access is a coalesced 16-byte
// load/store and per-channel parameters stay in registers.
//
// Reductions are two-stage and deterministic: every workgroup writes per-channel FP32 partial
// sums to the workspace, a second stage combines them in a fixed order: FP32 within a row
// lane, double across lanes, waves and for everything that follows (mean, variance).
// When the partial sums come from a convolution epilogue and there are at most 400 row tiles,
// the apply kernels combine them themselves (per 64-channel slice, in double) and no second
// kernel runs.
// The stand-alone forward statistics (bn_relu_fwd, bn_batch_moments) are accumulated around a
// per-channel pivot (row 0) so that E[x^2]-E[x]^2 does not cancel when |mean| >> sigma.  The
// partial sums a convolution epilogue leaves (whole-step path) are plain sum x / sum x^2 of
// at most 256 rows per tile in FP32 (pivot 0): with |mean| = r*sigma the variance carries a
// relative error of about r^2 * 2^-24 per tile, i.e. 1/sqrt(var+eps) is good to 1e-4 up to
// r of about 40 and degrades as r^2 beyond; BN inputs here are zero-mean-ish conv outputs.
#include "common.h"
#include "misc_internal.h"
#include "prof.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 2048;

struct RowMap {
    int gp;         // 16-byte channel groups per row (c / 8)
    int gpb;        // channel groups handled by one pass of a workgroup: min(gp, 256)
    int rows_par;   // rows handled in parallel by a workgroup: 256 / gpb
};

__host__ __device__ inline RowMap make_rowmap(int c) {
    RowMap r;
    r.gp = c / 8;
    r.gpb = r.gp < kThreads ? r.gp : kThreads;
    r.rows_par = kThreads / r.gpb;
    return r;
}

// Sum the kThreads/gpb row-lanes that share a channel group.  vals: this thread's NV values.
// After the call thread (row lane 0) holds the totals.
template <int NV>
__device__ __forceinline__ void reduce_row_lanes(float (&vals)[NV], float* smem, const RowMap& rm) {
    if (rm.rows_par == 1) return;
    const int tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < NV; ++j) smem[j * kThreads + tid] = vals[j];
    __syncthreads();
    if (tid < rm.gpb) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            float s = 0.f;
            for (int r = 0; r < rm.rows_par; ++r) s += smem[j * kThreads + r * rm.gpb + tid];
            vals[j] = s;
        }
    }
}

// Row loops are unrolled by kUnroll so that several 16-byte loads per tensor are in flight per thread.
constexpr int kUnroll = 4;

// ------------------------------------------------------------------ forward statistics
// part[(blk*2+0)*c + ch] = sum (x - pivot), part[(blk*2+1)*c + ch] = sum (x - pivot)^2
__global__ __launch_bounds__(kThreads) void bn_stats_kernel(long long m, int c, const h16* __restrict__ x,
                                                            float* __restrict__ part, int rows_per_block)
{
    __shared__ float smem[16 * kThreads];
    const RowMap rm = make_rowmap(c);
    const int tid = threadIdx.x;
    const int cgl = tid % rm.gpb, rl = tid / rm.gpb;
    const long long row0 = (long long)blockIdx.x * rows_per_block;
    long long row1 = row0 + rows_per_block;
    if (row1 > m) row1 = m;
    const int rp = rm.rows_par;
    for (int cg = cgl; cg < rm.gp; cg += rm.gpb) {
        const h16x8 pv = *reinterpret_cast<const h16x8*>(x + (size_t)cg * 8);
        const h16* xc = x + (size_t)cg * 8;
        float acc[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = 0.f;
        long long r = row0 + rl;
        for (; r + (kUnroll - 1) * rp < row1; r += kUnroll * rp) {
            h16x8 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) v[u] = *reinterpret_cast<const h16x8*>(xc + (size_t)(r + u * rp) * c);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float d = (float)v[u][j] - (float)pv[j];
                    acc[j] += d;
                    acc[8 + j] += d * d;
                }
        }
        for (; r < row1; r += rp) {
            const h16x8 v = *reinterpret_cast<const h16x8*>(xc + (size_t)r * c);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float d = (float)v[j] - (float)pv[j];
                acc[j] += d;
                acc[8 + j] += d * d;
            }
        }
        reduce_row_lanes<16>(acc, smem, rm);
        if (rl == 0) {
            float* p0 = part + ((size_t)blockIdx.x * 2) * c + (size_t)cg * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) { p0[j] = acc[j]; p0[c + j] = acc[8 + j]; }
        }
        if (rm.gp > rm.gpb) __syncthreads();
    }
}

// Column sums of the partials matrix [nblk][2][c] and what follows from them.  A workgroup owns 16
// channels (both sums): 8 lanes x 16 bytes cover one row's two 64-byte segments, the other lanes take
// further rows, every thread keeps several rows in flight.  Row lanes are combined in a fixed order
// (wave shuffles, then across waves in double), so the result does not depend on timing.
//   kMode 0 (forward): partials are sum (x - pivot), sum (x - pivot)^2 -> mean, 1/sqrt(var + eps);
//                      pivot_row: first row of x, or nullptr for pivot 0
//   kMode 1 (backward): partials are sum g, sum g*xhat -> sums[0..c) = d beta, sums[c..2c) = d gamma, plus the
//                      optional half copies (slices of the flat FP16 gradient)
//   kMode 2 (moments):  as kMode 0 but out0[0..c) = mean, out0[c..2c) = mean of squares (what GPUs exchange)
template <int kMode, int kNT>
__global__ __launch_bounds__(kNT) void bn_finalize_kernel(long long m, int c, float eps, int nblk,
                                                          const h16* __restrict__ pivot_row,
                                                          const float* __restrict__ part, float* __restrict__ out0,
                                                          float* __restrict__ out1, h16* __restrict__ dgamma,
                                                          h16* __restrict__ dbeta)
{
    constexpr int kRowLanes = kNT / 8, kWaves = kNT / 64, kBatch = 8;
    __shared__ float red[kWaves][32];
    __shared__ double fin[32];
    const int tid = threadIdx.x;
    const int cl = tid & 7, rl = tid >> 3;
    const int which = cl >> 2, ch0 = blockIdx.x * 16 + (cl & 3) * 4;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (ch0 < c) {
        const float* p = part + (size_t)which * c + ch0;
        const size_t pitch = 2 * (size_t)c;
        for (int r0 = rl; r0 < nblk; r0 += kRowLanes * kBatch) {
            f32x4 v[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int r = r0 + u * kRowLanes;
                v[u] = r < nblk ? *reinterpret_cast<const f32x4*>(p + (size_t)r * pitch) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) acc += v[u];
        }
    }
#pragma unroll
    for (int o = 8; o < 64; o <<= 1)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] += __shfl_xor(acc[j], o, 64);
    if ((tid & 63) < 8) {
#pragma unroll
        for (int j = 0; j < 4; ++j) red[tid >> 6][cl * 4 + j] = acc[j];
    }
    __syncthreads();
    if (tid < 32) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += (double)red[w][tid];
        fin[tid] = s;
    }
    __syncthreads();
    const int ch = blockIdx.x * 16 + tid;
    if (tid < 16 && ch < c) {
        const double sa = fin[tid], sb = fin[16 + tid];
        if (kMode == 0) {
            const double pivot = pivot_row ? (double)(float)pivot_row[ch] : 0.0;
            const double md = sa / (double)m;
            double var = sb / (double)m - md * md;
            if (var < 0.0) var = 0.0;
            out0[ch] = (float)(pivot + md);
            out1[ch] = (float)(1.0 / sqrt(var + (double)eps));
        } else if (kMode == 2) {
            // E[x] = p + E[x-p];  E[x^2] = E[(x-p)^2] + 2p E[x-p] + p^2
            const double pivot = pivot_row ? (double)(float)pivot_row[ch] : 0.0;
            const double md = sa / (double)m;
            out0[ch] = (float)(pivot + md);
            out0[c + ch] = (float)(sb / (double)m + 2.0 * pivot * md + pivot * pivot);
        } else {
            out0[ch] = (float)sa;
            out0[c + ch] = (float)sb;
            if (dbeta) dbeta[ch] = (h16)(float)sa;
            if (dgamma) dgamma[ch] = (h16)(float)sb;
        }
    }
}

// many partial rows: 1024 threads (128 row lanes), else 256
template <int kMode>
void launch_bn_finalize(long long m, int c, float eps, int nblk, const h16* pivot_row, const float* part, float* out0,
                        float* out1, h16* dgamma, h16* dbeta, hipStream_t s)
{
    const int grid = rn50_cdiv(c, 16);
    if (nblk > 256)
        bn_finalize_kernel<kMode, 1024><<<grid, 1024, 0, s>>>(m, c, eps, nblk, pivot_row, part, out0, out1, dgamma, dbeta);
    else
        bn_finalize_kernel<kMode, 256><<<grid, 256, 0, s>>>(m, c, eps, nblk, pivot_row, part, out0, out1, dgamma, dbeta);
}

// ------------------------------------------------------------------ forward apply
template <bool kRelu, bool kRes>
__global__ __launch_bounds__(kThreads) void bn_apply_kernel(long long m, int c, const h16* __restrict__ x,
                                                            const float* __restrict__ gamma,
                                                            const float* __restrict__ beta,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ invstd,
                                                            const h16* __restrict__ res, h16* __restrict__ y,
                                                            int rows_per_block)
{
    const RowMap rm = make_rowmap(c);
    const int tid = threadIdx.x;
    const int cgl = tid % rm.gpb, rl = tid / rm.gpb;
    const long long row0 = (long long)blockIdx.x * rows_per_block;
    long long row1 = row0 + rows_per_block;
    if (row1 > m) row1 = m;
    const int rp = rm.rows_par;
    for (int cg = cgl; cg < rm.gp; cg += rm.gpb) {
        float g[8], b[8], mu[8], is[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            g[j] = gamma[cg * 8 + j]; b[j] = beta[cg * 8 + j];
            mu[j] = mean[cg * 8 + j]; is[j] = invstd[cg * 8 + j];
        }
        auto one = [&](const h16x8& v, const h16x8& rv) {
            h16x8 o;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float t = g[j] * (((float)v[j] - mu[j]) * is[j]) + b[j];
                if (kRes) t += (float)rv[j];
                if (kRelu) t = t > 0.f ? t : 0.f;
                o[j] = (h16)t;
            }
            return o;
        };
        long long r = row0 + rl;
        for (; r + (kUnroll - 1) * rp < row1; r += kUnroll * rp) {
            h16x8 v[kUnroll], rv[kUnroll] = {};
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const size_t off = (size_t)(r + u * rp) * c + (size_t)cg * 8;
                v[u] = *reinterpret_cast<const h16x8*>(x + off);
                if (kRes) rv[u] = *reinterpret_cast<const h16x8*>(res + off);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                *reinterpret_cast<h16x8*>(y + (size_t)(r + u * rp) * c + (size_t)cg * 8) = one(v[u], rv[u]);
        }
        for (; r < row1; r += rp) {
            const size_t off = (size_t)r * c + (size_t)cg * 8;
            const h16x8 v = *reinterpret_cast<const h16x8*>(x + off);
            h16x8 rv = {0, 0, 0, 0, 0, 0, 0, 0};
            if (kRes) rv = *reinterpret_cast<const h16x8*>(res + off);
            *reinterpret_cast<h16x8*>(y + off) = one(v, rv);
        }
    }
}

// ------------------------------------------------------------------ backward reductions
// part[(blk*2+0)*c + ch] = sum g, part[(blk*2+1)*c + ch] = sum g*xhat
template <bool kRelu>
__global__ __launch_bounds__(kThreads) void bn_bwd_reduce_kernel(long long m, int c, const h16* __restrict__ dy,
                                                                 const h16* __restrict__ x,
                                                                 const h16* __restrict__ y,
                                                                 const float* __restrict__ mean,
                                                                 const float* __restrict__ invstd,
                                                                 float* __restrict__ part, int rows_per_block)
{
    __shared__ float smem[16 * kThreads];
    const RowMap rm = make_rowmap(c);
    const int tid = threadIdx.x;
    const int cgl = tid % rm.gpb, rl = tid / rm.gpb;
    const long long row0 = (long long)blockIdx.x * rows_per_block;
    long long row1 = row0 + rows_per_block;
    if (row1 > m) row1 = m;
    const int rp = rm.rows_par;
    for (int cg = cgl; cg < rm.gp; cg += rm.gpb) {
        float mu[8], is[8], acc[16];
#pragma unroll
        for (int j = 0; j < 8; ++j) { mu[j] = mean[cg * 8 + j]; is[j] = invstd[cg * 8 + j]; }
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = 0.f;
        auto one = [&](const h16x8& d, const h16x8& xv, const h16x8& yv) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float g = (float)d[j];
                if (kRelu) g = (float)yv[j] > 0.f ? g : 0.f;
                acc[j] += g;
                acc[8 + j] += g * (((float)xv[j] - mu[j]) * is[j]);
            }
        };
        long long r = row0 + rl;
        for (; r + (kUnroll - 1) * rp < row1; r += kUnroll * rp) {
            h16x8 d[kUnroll], xv[kUnroll], yv[kUnroll] = {};
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const size_t off = (size_t)(r + u * rp) * c + (size_t)cg * 8;
                d[u] = *reinterpret_cast<const h16x8*>(dy + off);
                xv[u] = *reinterpret_cast<const h16x8*>(x + off);
                if (kRelu) yv[u] = *reinterpret_cast<const h16x8*>(y + off);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) one(d[u], xv[u], yv[u]);
        }
        for (; r < row1; r += rp) {
            const size_t off = (size_t)r * c + (size_t)cg * 8;
            const h16x8 d = *reinterpret_cast<const h16x8*>(dy + off);
            const h16x8 xv = *reinterpret_cast<const h16x8*>(x + off);
            h16x8 yv = {0, 0, 0, 0, 0, 0, 0, 0};
            if (kRelu) yv = *reinterpret_cast<const h16x8*>(y + off);
            one(d, xv, yv);
        }
        reduce_row_lanes<16>(acc, smem, rm);
        if (rl == 0) {
            float* p0 = part + ((size_t)blockIdx.x * 2) * c + (size_t)cg * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) { p0[j] = acc[j]; p0[c + j] = acc[8 + j]; }
        }
        if (rm.gp > rm.gpb) __syncthreads();
    }
}

template <bool kRelu, bool kRes>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(long long m, int c, const h16* __restrict__ dy,
                                                                const h16* __restrict__ x,
                                                                const h16* __restrict__ y,
                                                                const float* __restrict__ gamma,
                                                                const float* __restrict__ mean,
                                                                const float* __restrict__ invstd,
                                                                const float* __restrict__ sums,
                                                                h16* __restrict__ dx, h16* __restrict__ dres,
                                                                int rows_per_block, float inv_m)
{
    const RowMap rm = make_rowmap(c);
    const int tid = threadIdx.x;
    const int cgl = tid % rm.gpb, rl = tid / rm.gpb;
    const long long row0 = (long long)blockIdx.x * rows_per_block;
    long long row1 = row0 + rows_per_block;
    if (row1 > m) row1 = m;
    const int rp = rm.rows_par;
    for (int cg = cgl; cg < rm.gp; cg += rm.gpb) {
        float mu[8], is[8], sc[8], mb[8], mg[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            mu[j] = mean[cg * 8 + j]; is[j] = invstd[cg * 8 + j];
            sc[j] = gamma[cg * 8 + j] * is[j];
            mb[j] = sums[cg * 8 + j] * inv_m;
            mg[j] = sums[c + cg * 8 + j] * inv_m;
        }
        auto one = [&](const h16x8& d, const h16x8& xv, const h16x8& yv, size_t off) {
            h16x8 o, go;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float g = (float)d[j];
                if (kRelu) g = (float)yv[j] > 0.f ? g : 0.f;
                go[j] = (h16)g;
                const float xh = ((float)xv[j] - mu[j]) * is[j];
                o[j] = (h16)(sc[j] * (g - mb[j] - xh * mg[j]));
            }
            *reinterpret_cast<h16x8*>(dx + off) = o;
            if (kRes) *reinterpret_cast<h16x8*>(dres + off) = go;
        };
        long long r = row0 + rl;
        for (; r + (kUnroll - 1) * rp < row1; r += kUnroll * rp) {
            h16x8 d[kUnroll], xv[kUnroll], yv[kUnroll] = {};
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const size_t off = (size_t)(r + u * rp) * c + (size_t)cg * 8;
                d[u] = *reinterpret_cast<const h16x8*>(dy + off);
                xv[u] = *reinterpret_cast<const h16x8*>(x + off);
                if (kRelu) yv[u] = *reinterpret_cast<const h16x8*>(y + off);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) one(d[u], xv[u], yv[u], (size_t)(r + u * rp) * c + (size_t)cg * 8);
        }
        for (; r < row1; r += rp) {
            const size_t off = (size_t)r * c + (size_t)cg * 8;
            const h16x8 d = *reinterpret_cast<const h16x8*>(dy + off);
            const h16x8 xv = *reinterpret_cast<const h16x8*>(x + off);
            h16x8 yv = {0, 0, 0, 0, 0, 0, 0, 0};
            if (kRelu) yv = *reinterpret_cast<const h16x8*>(y + off);
            one(d, xv, yv, off);
        }
    }
}

// ------------------------------------------------------------------ finalize + apply in one launch
// For layers with few row tiles (small feature maps) a separate finalize launch costs more than the work it
// does.  Here every workgroup owns a 64-channel slice and kSliceRows rows, first adds up the partials of its own
// 64 channels (redundantly with the other workgroups of the slice: ntiles x 512 bytes from L2) and then applies.
// The first row chunk of each slice also stores the per-channel results.
constexpr int kSliceRows = 128;          // 32 row lanes x 4 rows in flight
constexpr int kFusedMaxTiles = 400;      // beyond this the redundant summing costs more than the finalize launch (measured: 128, 400, 800)

// Column sums of part[ntiles][2][c] for channels [ch0, ch0 + 64): s[0..63] = first sums, s[64..127] = second sums.
__device__ __forceinline__ void slice_partial_sums(const float* __restrict__ part, int c, int ntiles, int ch0, double* s)
{
    __shared__ double red[4][128];
    const int tid = threadIdx.x;
    const int cl = tid & 31, rl = tid >> 5;                       // 32 x 16-byte columns, 8 row lanes
    const float* p = part + (size_t)(cl >> 4) * c + ch0 + (cl & 15) * 4;
    const size_t pitch = 2 * (size_t)c;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int r0 = rl; r0 < ntiles; r0 += 64) {
        f32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = r0 + u * 8;
            v[u] = r < ntiles ? *reinterpret_cast<const f32x4*>(p + (size_t)r * pitch) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] += (double)v[u][j];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] += __shfl_xor(acc[j], 32, 64);
    if ((tid & 63) < 32) {
#pragma unroll
        for (int j = 0; j < 4; ++j) red[tid >> 6][cl * 4 + j] = acc[j];
    }
    __syncthreads();
    if (tid < 128) s[tid] = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
    __syncthreads();
}

template <bool kRelu, bool kRes>
__global__ __launch_bounds__(kThreads) void bn_fused_apply_kernel(long long m, int c, float eps, int ntiles,
                                                                  const float* __restrict__ part,
                                                                  const h16* __restrict__ x,
                                                                  const float* __restrict__ gamma,
                                                                  const float* __restrict__ beta,
                                                                  const h16* __restrict__ res, h16* __restrict__ y,
                                                                  float* __restrict__ save_mean,
                                                                  float* __restrict__ save_invstd)
{
    __shared__ double sums[128];
    __shared__ float s_mean[64], s_inv[64];
    const int tid = threadIdx.x;
    const int ch0 = blockIdx.y * 64;
    const int cg = tid & 7, rl = tid >> 3;                         // 8 channel groups of 8, 32 row lanes
    const long long row0 = (long long)blockIdx.x * kSliceRows + rl;
    const size_t col = (size_t)ch0 + cg * 8;
    // the rows of x (and the residual) are requested before the statistics are known
    h16x8 v[4], rv[4] = {};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const long long r = row0 + u * 32;
        v[u] = r < m ? *reinterpret_cast<const h16x8*>(x + (size_t)r * c + col) : h16x8{0, 0, 0, 0, 0, 0, 0, 0};
        if (kRes && r < m) rv[u] = *reinterpret_cast<const h16x8*>(res + (size_t)r * c + col);
    }
    slice_partial_sums(part, c, ntiles, ch0, sums);
    if (tid < 64) {
        const double md = sums[tid] / (double)m;
        double var = sums[64 + tid] / (double)m - md * md;
        if (var < 0.0) var = 0.0;
        const float mean = (float)md, inv = (float)(1.0 / sqrt(var + (double)eps));
        s_mean[tid] = mean; s_inv[tid] = inv;
        if (blockIdx.x == 0) { save_mean[ch0 + tid] = mean; save_invstd[ch0 + tid] = inv; }
    }
    __syncthreads();
    float g[8], b[8], mu[8], is[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        g[j] = gamma[col + j]; b[j] = beta[col + j];
        mu[j] = s_mean[cg * 8 + j]; is[j] = s_inv[cg * 8 + j];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const long long r = row0 + u * 32;
        if (r >= m) continue;
        h16x8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float t = g[j] * (((float)v[u][j] - mu[j]) * is[j]) + b[j];
            if (kRes) t += (float)rv[u][j];
            if (kRelu) t = t > 0.f ? t : 0.f;
            o[j] = (h16)t;
        }
        *reinterpret_cast<h16x8*>(y + (size_t)r * c + col) = o;
    }
}

// backward: partials are (sum g | sum g*xhat) of the already masked gradient g; dx = gamma*invstd*(g - mean(g) - xhat*mean(g*xhat))
__global__ __launch_bounds__(kThreads) void bn_bwd_fused_apply_kernel(long long m, int c, int ntiles,
                                                                      const float* __restrict__ part,
                                                                      const h16* __restrict__ gr,
                                                                      const h16* __restrict__ x,
                                                                      const float* __restrict__ gamma,
                                                                      const float* __restrict__ mean,
                                                                      const float* __restrict__ invstd,
                                                                      h16* __restrict__ dx, h16* __restrict__ dgamma,
                                                                      h16* __restrict__ dbeta)
{
    __shared__ double sums[128];
    const int tid = threadIdx.x;
    const int ch0 = blockIdx.y * 64;
    const int cg = tid & 7, rl = tid >> 3;
    const long long row0 = (long long)blockIdx.x * kSliceRows + rl;
    const size_t col = (size_t)ch0 + cg * 8;
    h16x8 gv[4], xv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const long long r = row0 + u * 32;
        gv[u] = r < m ? *reinterpret_cast<const h16x8*>(gr + (size_t)r * c + col) : h16x8{0, 0, 0, 0, 0, 0, 0, 0};
        xv[u] = r < m ? *reinterpret_cast<const h16x8*>(x + (size_t)r * c + col) : h16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    slice_partial_sums(part, c, ntiles, ch0, sums);
    if (blockIdx.x == 0 && tid < 64) {
        if (dbeta) dbeta[ch0 + tid] = (h16)(float)sums[tid];
        if (dgamma) dgamma[ch0 + tid] = (h16)(float)sums[64 + tid];
    }
    const float inv_m = 1.f / (float)m;
    float mu[8], is[8], sc[8], mb[8], mg[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        mu[j] = mean[col + j]; is[j] = invstd[col + j];
        sc[j] = gamma[col + j] * is[j];
        mb[j] = (float)sums[cg * 8 + j] * inv_m;
        mg[j] = (float)sums[64 + cg * 8 + j] * inv_m;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const long long r = row0 + u * 32;
        if (r >= m) continue;
        h16x8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float g = (float)gv[u][j];
            const float xh = ((float)xv[u][j] - mu[j]) * is[j];
            o[j] = (h16)(sc[j] * (g - mb[j] - xh * mg[j]));
        }
        *reinterpret_cast<h16x8*>(dx + (size_t)r * c + col) = o;
    }
}

// (mean, mean of squares) -> (mean, 1/sqrt(var + eps)) with var = max(E[x^2] - mean^2, 0), in double
__global__ __launch_bounds__(kThreads) void bn_moments_to_stats_kernel(int c, float eps, const float* __restrict__ moments,
                                                                       float* __restrict__ save_mean,
                                                                       float* __restrict__ save_invstd)
{
    const int ch = blockIdx.x * kThreads + threadIdx.x;
    if (ch >= c) return;
    const double mean = (double)moments[ch];
    double var = (double)moments[c + ch] - mean * mean;
    if (var < 0.0) var = 0.0;
    save_mean[ch] = (float)mean;
    save_invstd[ch] = (float)(1.0 / sqrt(var + (double)eps));
}

struct BnPlan { int nblk; int rows_per_block; };

// Elementwise passes: 4 rows per thread (one unrolled batch), as many workgroups as that takes.
BnPlan plan_rows_apply(long long m, int c)
{
    const RowMap rm = make_rowmap(c);
    const long long rows = (long long)rm.rows_par * kUnroll;
    BnPlan p;
    p.nblk = (int)((m + rows - 1) / rows);
    p.rows_per_block = (int)rows;
    return p;
}

// Reducing passes: partials cost a second kernel, so fewer, fatter workgroups.
BnPlan plan_rows(long long m, int c)
{
    const RowMap rm = make_rowmap(c);
    // about 8 row iterations per thread, at most kMaxBlocks workgroups
    long long rows = (long long)rm.rows_par * 8;
    long long nblk = (m + rows - 1) / rows;
    if (nblk > kMaxBlocks) {
        rows = (m + kMaxBlocks - 1) / kMaxBlocks;
        rows = (rows + rm.rows_par - 1) / rm.rows_par * rm.rows_par;
        nblk = (m + rows - 1) / rows;
    }
    BnPlan p;
    p.nblk = (int)nblk;
    p.rows_per_block = (int)rows;
    return p;
}

int validate(const bn_desc* d)
{
    RN50_REQUIRE_PTR(d);
    if (d->dt != RN50_F16) return RN50_ERR_DTYPE;
    if (d->m < 1 || d->c < 8 || d->c % 8 != 0 || d->m > (1ll << 40)) return RN50_ERR_SHAPE;
    const int gp = d->c / 8;
    if (!(kThreads % gp == 0 || gp % kThreads == 0)) return RN50_ERR_SHAPE;
    return RN50_OK;
}

}  // namespace

// partials of up to kMaxBlocks workgroups (2 rows of c floats each) + 2c floats of totals
int rn50_bn_fused_max_tiles() { return kFusedMaxTiles; }
size_t rn50_bn_ws_floats(int c) { return (size_t)kMaxBlocks * 2 * c + 2 * (size_t)c; }

extern "C" size_t bn_workspace_bytes(const bn_desc* d)
{
    if (validate(d) != RN50_OK) return 0;
    return rn50_bn_ws_floats(d->c) * sizeof(float);
}

// Internal entry points, also used by the whole-step driver.
int rn50_bn_fwd_launch(long long m, int c, float eps, bool relu, const h16* x, const float* gamma, const float* beta,
                       const h16* res, h16* y, float* save_mean, float* save_invstd, float* ws, hipStream_t s)
{
    const BnPlan p = plan_rows(m, c);
    const double elems = (double)m * c;
    {
        ProfScope ps(RN50_K_BN_STATS, 0.0, 2.0 * elems, s);
        bn_stats_kernel<<<p.nblk, kThreads, 0, s>>>(m, c, x, ws, p.rows_per_block);
    }
    {
        ProfScope ps(RN50_K_BN_STATS_FINALIZE, 0.0, 8.0 * p.nblk * c, s);
        launch_bn_finalize<0>(m, c, eps, p.nblk, x, ws, save_mean, save_invstd, nullptr, nullptr, s);
    }
    ProfScope ps(RN50_K_BN_APPLY, 0.0, (res ? 6.0 : 4.0) * elems, s);
    const BnPlan pa = plan_rows_apply(m, c);
#define RN50_BN_APPLY(R, Z) bn_apply_kernel<R, Z><<<pa.nblk, kThreads, 0, s>>>(m, c, x, gamma, beta, save_mean, \
                                                                               save_invstd, res, y, pa.rows_per_block)
    if (relu) { if (res) RN50_BN_APPLY(true, true); else RN50_BN_APPLY(true, false); }
    else      { if (res) RN50_BN_APPLY(false, true); else RN50_BN_APPLY(false, false); }
#undef RN50_BN_APPLY
    return rn50_check_launch();
}

// Forward for a tensor whose per-row-tile partial sums (pivot 0) were already written by the producing
// convolution: part[(tile*2+0)*c + ch] = sum x, part[(tile*2+1)*c + ch] = sum x^2 over the tile's rows.
int rn50_bn_fwd_from_partials_launch(long long m, int c, float eps, bool relu, const h16* x, const float* gamma,
                                     const float* beta, const h16* res, h16* y, float* save_mean, float* save_invstd,
                                     const float* part, int ntiles, hipStream_t s)
{
    const double elems = (double)m * c;
    if (ntiles <= kFusedMaxTiles && c % 64 == 0) {
        ProfScope ps(RN50_K_BN_FUSED_APPLY, 0.0, (res ? 6.0 : 4.0) * elems, s);
        const dim3 grid((unsigned)rn50_cdiv(m, kSliceRows), (unsigned)(c / 64));
#define RN50_BN_FUSED(R, Z) bn_fused_apply_kernel<R, Z><<<grid, kThreads, 0, s>>>(m, c, eps, ntiles, part, x, gamma, beta, res, \
                                                                                y, save_mean, save_invstd)
        if (relu) { if (res) RN50_BN_FUSED(true, true); else RN50_BN_FUSED(true, false); }
        else      { if (res) RN50_BN_FUSED(false, true); else RN50_BN_FUSED(false, false); }
#undef RN50_BN_FUSED
        return rn50_check_launch();
    }
    {
        ProfScope ps(RN50_K_BN_STATS_FINALIZE, 0.0, 8.0 * ntiles * c, s);
        launch_bn_finalize<0>(m, c, eps, ntiles, nullptr, part, save_mean, save_invstd, nullptr, nullptr, s);
    }
    ProfScope ps(RN50_K_BN_APPLY, 0.0, (res ? 6.0 : 4.0) * elems, s);
    const BnPlan pa = plan_rows_apply(m, c);
#define RN50_BN_APPLY(R, Z) bn_apply_kernel<R, Z><<<pa.nblk, kThreads, 0, s>>>(m, c, x, gamma, beta, save_mean, \
                                                                               save_invstd, res, y, pa.rows_per_block)
    if (relu) { if (res) RN50_BN_APPLY(true, true); else RN50_BN_APPLY(true, false); }
    else      { if (res) RN50_BN_APPLY(false, true); else RN50_BN_APPLY(false, false); }
#undef RN50_BN_APPLY
    return rn50_check_launch();
}

int rn50_bn_bwd_launch(long long m, int c, bool relu, const h16* dy, const h16* x, const h16* y, const float* gamma,
                       const float* save_mean, const float* save_invstd, h16* dx, h16* dres,
                       h16* dgamma, h16* dbeta, float* ws, hipStream_t s)
{
    const BnPlan p = plan_rows(m, c);
    float* sums = ws + (size_t)kMaxBlocks * 2 * c;
    const double elems = (double)m * c;
    {
        ProfScope ps(RN50_K_BN_BWD_REDUCE, 0.0, (relu ? 6.0 : 4.0) * elems, s);
        if (relu) bn_bwd_reduce_kernel<true><<<p.nblk, kThreads, 0, s>>>(m, c, dy, x, y, save_mean, save_invstd, ws, p.rows_per_block);
        else      bn_bwd_reduce_kernel<false><<<p.nblk, kThreads, 0, s>>>(m, c, dy, x, y, save_mean, save_invstd, ws, p.rows_per_block);
    }
    {
        ProfScope ps(RN50_K_BN_BWD_FINALIZE, 0.0, 8.0 * p.nblk * c, s);
        launch_bn_finalize<1>(m, c, 0.f, p.nblk, nullptr, ws, sums, nullptr, dgamma, dbeta, s);
    }
    ProfScope ps(RN50_K_BN_BWD_APPLY, 0.0, ((relu ? 6.0 : 4.0) + 2.0 + (dres ? 2.0 : 0.0)) * elems, s);
    const BnPlan pa = plan_rows_apply(m, c);
#define RN50_BN_BWD(R, Z) bn_bwd_apply_kernel<R, Z><<<pa.nblk, kThreads, 0, s>>>(m, c, dy, x, y, gamma, save_mean, \
                                                                                 save_invstd, sums, dx, dres, pa.rows_per_block, 1.f / (float)m)
    if (relu) { if (dres) RN50_BN_BWD(true, true); else RN50_BN_BWD(true, false); }
    else      { if (dres) RN50_BN_BWD(false, true); else RN50_BN_BWD(false, false); }
#undef RN50_BN_BWD
    return rn50_check_launch();
}

// Backward for a layer whose masked incoming gradient g and per-row-tile partial sums (sum g, sum g*xhat)
// were already produced by the data gradient that wrote g: combine the partials, then dx.  sums: 2c floats.
int rn50_bn_bwd_from_partials_launch(long long m, int c, const h16* g, const h16* x, const float* gamma,
                                     const float* save_mean, const float* save_invstd, h16* dx,
                                     h16* dgamma, h16* dbeta, const float* part, int ntiles, float* sums,
                                     hipStream_t s)
{
    const double elems = (double)m * c;
    if (ntiles <= kFusedMaxTiles && c % 64 == 0) {
        ProfScope ps(RN50_K_BN_BWD_FUSED_APPLY, 0.0, 6.0 * elems, s);
        const dim3 grid((unsigned)rn50_cdiv(m, kSliceRows), (unsigned)(c / 64));
        bn_bwd_fused_apply_kernel<<<grid, kThreads, 0, s>>>(m, c, ntiles, part, g, x, gamma, save_mean, save_invstd, dx,
                                                            dgamma, dbeta);
        return rn50_check_launch();
    }
    {
        ProfScope ps(RN50_K_BN_BWD_FINALIZE, 0.0, 8.0 * ntiles * c, s);
        launch_bn_finalize<1>(m, c, 0.f, ntiles, nullptr, part, sums, nullptr, dgamma, dbeta, s);
    }
    ProfScope ps(RN50_K_BN_BWD_APPLY, 0.0, 6.0 * elems, s);
    const BnPlan pa = plan_rows_apply(m, c);
    bn_bwd_apply_kernel<false, false><<<pa.nblk, kThreads, 0, s>>>(m, c, g, x, nullptr, gamma, save_mean, save_invstd,
                                                                   sums, dx, nullptr, pa.rows_per_block, 1.f / (float)m);
    return rn50_check_launch();
}

extern "C" int bn_relu_fwd(const bn_desc* d, const void* x, const float* gamma, const float* beta,
                           const void* residual, void* y, float* save_mean, float* save_invstd,
                           void* ws, size_t ws_bytes, void* stream)
{
    RN50_TRY(validate(d));
    RN50_REQUIRE_PTR(x); RN50_REQUIRE_PTR(gamma); RN50_REQUIRE_PTR(beta); RN50_REQUIRE_PTR(y);
    RN50_REQUIRE_PTR(save_mean); RN50_REQUIRE_PTR(save_invstd);
    if (d->has_residual) RN50_REQUIRE_PTR(residual);
    if (!ws || ws_bytes < bn_workspace_bytes(d)) return RN50_ERR_WORKSPACE;
    RN50_REQUIRE_ALIGNED(x); RN50_REQUIRE_ALIGNED(y); RN50_REQUIRE_ALIGNED(residual); RN50_REQUIRE_ALIGNED(ws);
    return rn50_bn_fwd_launch(d->m, d->c, d->eps, d->relu != 0, static_cast<const h16*>(x), gamma, beta,
                              d->has_residual ? static_cast<const h16*>(residual) : nullptr, static_cast<h16*>(y),
                              save_mean, save_invstd, static_cast<float*>(ws), static_cast<hipStream_t>(stream));
}

extern "C" int bn_relu_bwd(const bn_desc* d, const void* dy, const void* x, const void* y, const float* gamma,
                           const float* save_mean, const float* save_invstd, void* dx, void* dresidual,
                           void* dgamma, void* dbeta, void* ws, size_t ws_bytes, void* stream)
{
    RN50_TRY(validate(d));
    RN50_REQUIRE_PTR(dy); RN50_REQUIRE_PTR(x); RN50_REQUIRE_PTR(gamma); RN50_REQUIRE_PTR(save_mean);
    RN50_REQUIRE_PTR(save_invstd); RN50_REQUIRE_PTR(dx); RN50_REQUIRE_PTR(dgamma); RN50_REQUIRE_PTR(dbeta);
    if (d->relu) RN50_REQUIRE_PTR(y);
    if (d->has_residual) RN50_REQUIRE_PTR(dresidual);
    if (!ws || ws_bytes < bn_workspace_bytes(d)) return RN50_ERR_WORKSPACE;
    RN50_REQUIRE_ALIGNED(dy); RN50_REQUIRE_ALIGNED(x); RN50_REQUIRE_ALIGNED(y); RN50_REQUIRE_ALIGNED(dx);
    RN50_REQUIRE_ALIGNED(dresidual); RN50_REQUIRE_ALIGNED(ws);
    return rn50_bn_bwd_launch(d->m, d->c, d->relu != 0, static_cast<const h16*>(dy), static_cast<const h16*>(x),
                              static_cast<const h16*>(y), gamma, save_mean, save_invstd, static_cast<h16*>(dx),
                              d->has_residual ? static_cast<h16*>(dresidual) : nullptr, static_cast<h16*>(dgamma),
                              static_cast<h16*>(dbeta), static_cast<float*>(ws), static_cast<hipStream_t>(stream));
}


// ---- bn_relu_fwd for callers that cannot hand over (or allocate) a workspace ----
// Same kernels as bn_relu_fwd; the partial sums of the statistics pass live in a file-scope device array
// instead of a workspace argument.  Every GPU holds its own copy of the array; its device address is looked
// up once per device and kept.  All calls on one GPU share the array, so calls that overlap in time on one
// GPU race (every call overwrites the part it reads, nothing has to start at zero).
namespace {
constexpr int kStaticMaxC = RN50_BN_STATIC_MAX_C;
constexpr size_t kStaticFloats = (size_t)kMaxBlocks * 2 * kStaticMaxC + 2 * (size_t)kStaticMaxC;
__device__ __align__(256) float scratch[kStaticFloats];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices];      // per device: address of that device's copy of `scratch` (nullptr: not looked up yet)

int static_scratch(float** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return rn50_hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return RN50_ERR_SHAPE;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return rn50_hip_fail(e);
        if (!p) return RN50_ERR_HIP;
        g_scratch_ptr[dev] = static_cast<float*>(p);
    }
    *out = g_scratch_ptr[dev];
    return RN50_OK;
}
}  // namespace

extern "C" int bn_relu_fwd_static(const bn_desc* d, const void* x, const float* gamma, const float* beta,
                                  const void* residual, void* y, float* save_mean, float* save_invstd, void* stream)
{
    RN50_TRY(validate(d));
    if (d->c > kStaticMaxC) return RN50_ERR_WORKSPACE;      // the static scratch holds the partials of at most this many channels
    RN50_REQUIRE_PTR(x); RN50_REQUIRE_PTR(gamma); RN50_REQUIRE_PTR(beta); RN50_REQUIRE_PTR(y);
    RN50_REQUIRE_PTR(save_mean); RN50_REQUIRE_PTR(save_invstd);
    if (d->has_residual) RN50_REQUIRE_PTR(residual);
    RN50_REQUIRE_ALIGNED(x); RN50_REQUIRE_ALIGNED(y); RN50_REQUIRE_ALIGNED(residual);
    float* ws = nullptr;
    RN50_TRY(static_scratch(&ws));
    return rn50_bn_fwd_launch(d->m, d->c, d->eps, d->relu != 0, static_cast<const h16*>(x), gamma, beta,
                              d->has_residual ? static_cast<const h16*>(residual) : nullptr, static_cast<h16*>(y),
                              save_mean, save_invstd, ws, static_cast<hipStream_t>(stream));
}

// ---- the same operators split at the points where GPUs exchange statistics (synchronised BN) ----
extern "C" int bn_batch_moments(const bn_desc* d, const void* x, float* moments, void* ws, size_t ws_bytes, void* stream)
{
    RN50_TRY(validate(d));
    RN50_REQUIRE_PTR(x); RN50_REQUIRE_PTR(moments);
    if (!ws || ws_bytes < bn_workspace_bytes(d)) return RN50_ERR_WORKSPACE;
    RN50_REQUIRE_ALIGNED(x); RN50_REQUIRE_ALIGNED(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const BnPlan p = plan_rows(d->m, d->c);
    const h16* xh = static_cast<const h16*>(x);
    float* part = static_cast<float*>(ws);
    {
        ProfScope ps(RN50_K_BN_STATS, 0.0, 2.0 * (double)d->m * d->c, s);
        bn_stats_kernel<<<p.nblk, kThreads, 0, s>>>(d->m, d->c, xh, part, p.rows_per_block);
    }
    ProfScope ps(RN50_K_BN_STATS_FINALIZE, 0.0, 8.0 * p.nblk * d->c, s);
    launch_bn_finalize<2>(d->m, d->c, 0.f, p.nblk, xh, part, moments, nullptr, nullptr, nullptr, s);
    return rn50_check_launch();
}

extern "C" int bn_relu_fwd_from_moments(const bn_desc* d, const void* x, const float* gamma, const float* beta,
                                        const void* residual, void* y, const float* moments, float* save_mean,
                                        float* save_invstd, void* stream)
{
    RN50_TRY(validate(d));
    RN50_REQUIRE_PTR(x); RN50_REQUIRE_PTR(gamma); RN50_REQUIRE_PTR(beta); RN50_REQUIRE_PTR(y); RN50_REQUIRE_PTR(moments);
    RN50_REQUIRE_PTR(save_mean); RN50_REQUIRE_PTR(save_invstd);
    if (d->has_residual) RN50_REQUIRE_PTR(residual);
    RN50_REQUIRE_ALIGNED(x); RN50_REQUIRE_ALIGNED(y); RN50_REQUIRE_ALIGNED(residual);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const long long m = d->m;
    const int c = d->c;
    bn_moments_to_stats_kernel<<<rn50_cdiv(c, kThreads), kThreads, 0, s>>>(c, d->eps, moments, save_mean, save_invstd);
    RN50_TRY(rn50_check_launch());
    const h16* res = d->has_residual ? static_cast<const h16*>(residual) : nullptr;
    ProfScope ps(RN50_K_BN_APPLY, 0.0, (res ? 6.0 : 4.0) * (double)m * c, s);
    const BnPlan pa = plan_rows_apply(m, c);
#define RN50_BN_APPLY(R, Z) bn_apply_kernel<R, Z><<<pa.nblk, kThreads, 0, s>>>(m, c, static_cast<const h16*>(x), gamma, beta, \
                                                                               save_mean, save_invstd, res, static_cast<h16*>(y), \
                                                                               pa.rows_per_block)
    if (d->relu) { if (res) RN50_BN_APPLY(true, true); else RN50_BN_APPLY(true, false); }
    else         { if (res) RN50_BN_APPLY(false, true); else RN50_BN_APPLY(false, false); }
#undef RN50_BN_APPLY
    return rn50_check_launch();
}

extern "C" int bn_relu_bwd_sums(const bn_desc* d, const void* dy, const void* x, const void* y, const float* save_mean,
                                const float* save_invstd, float* sums, void* ws, size_t ws_bytes, void* stream)
{
    RN50_TRY(validate(d));
    RN50_REQUIRE_PTR(dy); RN50_REQUIRE_PTR(x); RN50_REQUIRE_PTR(save_mean); RN50_REQUIRE_PTR(save_invstd); RN50_REQUIRE_PTR(sums);
    if (d->relu) RN50_REQUIRE_PTR(y);
    if (!ws || ws_bytes < bn_workspace_bytes(d)) return RN50_ERR_WORKSPACE;
    RN50_REQUIRE_ALIGNED(dy); RN50_REQUIRE_ALIGNED(x); RN50_REQUIRE_ALIGNED(y); RN50_REQUIRE_ALIGNED(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const long long m = d->m;
    const int c = d->c;
    const BnPlan p = plan_rows(m, c);
    float* part = static_cast<float*>(ws);
    const h16 *dyh = static_cast<const h16*>(dy), *xh = static_cast<const h16*>(x), *yh = static_cast<const h16*>(y);
    {
        ProfScope ps(RN50_K_BN_BWD_REDUCE, 0.0, (d->relu ? 6.0 : 4.0) * (double)m * c, s);
        if (d->relu) bn_bwd_reduce_kernel<true><<<p.nblk, kThreads, 0, s>>>(m, c, dyh, xh, yh, save_mean, save_invstd, part, p.rows_per_block);
        else         bn_bwd_reduce_kernel<false><<<p.nblk, kThreads, 0, s>>>(m, c, dyh, xh, yh, save_mean, save_invstd, part, p.rows_per_block);
    }
    ProfScope ps(RN50_K_BN_BWD_FINALIZE, 0.0, 8.0 * p.nblk * c, s);
    launch_bn_finalize<1>(m, c, 0.f, p.nblk, nullptr, part, sums, nullptr, nullptr, nullptr, s);
    return rn50_check_launch();
}

extern "C" int bn_relu_bwd_from_sums(const bn_desc* d, const void* dy, const void* x, const void* y, const float* gamma,
                                     const float* save_mean, const float* save_invstd, const float* sums,
                                     long long total_rows, void* dx, void* dresidual, void* stream)
{
    RN50_TRY(validate(d));
    RN50_REQUIRE_PTR(dy); RN50_REQUIRE_PTR(x); RN50_REQUIRE_PTR(gamma); RN50_REQUIRE_PTR(save_mean);
    RN50_REQUIRE_PTR(save_invstd); RN50_REQUIRE_PTR(sums); RN50_REQUIRE_PTR(dx);
    if (d->relu) RN50_REQUIRE_PTR(y);
    if (d->has_residual) RN50_REQUIRE_PTR(dresidual);
    if (total_rows < d->m) return RN50_ERR_SHAPE;
    RN50_REQUIRE_ALIGNED(dy); RN50_REQUIRE_ALIGNED(x); RN50_REQUIRE_ALIGNED(y); RN50_REQUIRE_ALIGNED(dx); RN50_REQUIRE_ALIGNED(dresidual);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const long long m = d->m;
    const int c = d->c;
    h16* dres = d->has_residual ? static_cast<h16*>(dresidual) : nullptr;
    ProfScope ps(RN50_K_BN_BWD_APPLY, 0.0, ((d->relu ? 6.0 : 4.0) + 2.0 + (dres ? 2.0 : 0.0)) * (double)m * c, s);
    const BnPlan pa = plan_rows_apply(m, c);
    const float inv_m = (float)(1.0 / (double)total_rows);
#define RN50_BN_BWD(R, Z) bn_bwd_apply_kernel<R, Z><<<pa.nblk, kThreads, 0, s>>>(m, c, static_cast<const h16*>(dy), \
        static_cast<const h16*>(x), static_cast<const h16*>(y), gamma, save_mean, save_invstd, sums, static_cast<h16*>(dx), dres, \
        pa.rows_per_block, inv_m)
    if (d->relu) { if (dres) RN50_BN_BWD(true, true); else RN50_BN_BWD(true, false); }
    else         { if (dres) RN50_BN_BWD(false, true); else RN50_BN_BWD(false, false); }
#undef RN50_BN_BWD
    return rn50_check_launch();
}
