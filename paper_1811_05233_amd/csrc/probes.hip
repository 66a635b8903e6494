// Hardware probes: small kernels that measure the machine figures the convolution design is argued from --
// matrix-unit throughput from registers, the rate at which tiles arrive in the compute units from L2 / the
// Infinity Cache / HBM (through LDS-DMA and through plain vector loads), a streaming copy, and the cost of a
// dependent empty launch.  Measurement aids only; nothing of the training path calls them.
#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kTileBytes = 16384;            // one probe tile: 16 wave-wide 1 KB loads
constexpr int kTileHalfs = kTileBytes / 2;
constexpr int kStages = 4;

#define RN50_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xf) | 0x0f70 | (((n) >> 4) << 14))
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// four independent accumulators per wavefront, operands never leave the registers
__global__ __launch_bounds__(kThreads) void probe_mfma_kernel(float* out, int iters)
{
    h16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (h16)(threadIdx.x * 0.001f + i); b[i] = (h16)(1.0f - i * 0.01f); }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
    out[(size_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

// Every workgroup pulls `iters` consecutive tiles of 16 KB, starting at tile blockIdx.x * start_stride, out of a
// buffer of `ntiles` tiles (tile index wraps, so the buffer size and the stride set where the data comes from) into a four-stage LDS ring with buffer_load ... lds, three tiles in flight,
// and reads one 16-byte word per lane from each tile so that the loads cannot be dropped.
__global__ __launch_bounds__(kThreads) void probe_tile_dma_kernel(const h16* src, unsigned src_bytes, unsigned ntiles,
                                                                  unsigned start_stride, int iters, float* out)
{
    __shared__ __attribute__((aligned(16))) h16 lds[kStages * kTileHalfs];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(src), 0, src_bytes, 0x00020000);
    unsigned tile = (unsigned)(((unsigned long long)blockIdx.x * start_stride) % ntiles);
    auto issue = [&](int stage) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned voff = tile * (unsigned)kTileBytes + (unsigned)((wave + 4 * j) * 1024 + lane * 16);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(lds + stage * kTileHalfs + (wave + 4 * j) * 512), 16,
                                                     (int)voff, 0, 0, 0);
        }
        if (++tile == ntiles) tile = 0;
    };
    for (int p = 0; p < kStages - 1; ++p)
        if (p < iters) issue(p);
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        if (it + kStages - 2 < iters) RN50_WAIT_VMCNT(4 * (kStages - 2)); else RN50_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        if (it + kStages - 1 < iters) issue((it + kStages - 1) % kStages);
        const h16x8 v = *reinterpret_cast<const h16x8*>(lds + (it % kStages) * kTileHalfs + tid * 8);
        acc += (float)v[0];
    }
    out[(size_t)blockIdx.x * kThreads + tid] = acc;
}

// The same traffic through plain 16-byte vector loads into registers (four per thread and tile, one tile ahead);
// all four words of every load enter an XOR checksum, so that no part of a load can be dropped.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(kThreads) void probe_tile_vec_kernel(const h16* src, unsigned ntiles, unsigned start_stride,
                                                                  int iters, float* out)
{
    const int tid = threadIdx.x;
    unsigned tile = (unsigned)(((unsigned long long)blockIdx.x * start_stride) % ntiles);
    unsigned acc = 0u;
    u32x4 cur[4], nxt[4];
    auto load = [&](u32x4 (&r)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) r[j] = *reinterpret_cast<const u32x4*>(src + (size_t)tile * kTileHalfs + j * 2048 + tid * 8);
        if (++tile == ntiles) tile = 0;
    };
    load(cur);
    for (int it = 0; it < iters; ++it) {
        if (it + 1 < iters) load(nxt);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc ^= cur[j][0] ^ cur[j][1] ^ cur[j][2] ^ cur[j][3];
        if (it + 1 < iters) {
#pragma unroll
            for (int j = 0; j < 4; ++j) cur[j] = nxt[j];
        }
    }
    reinterpret_cast<unsigned*>(out)[(size_t)blockIdx.x * kThreads + tid] = acc;
}

// four 16-byte words per thread and pass, all requested before the first is stored
__global__ __launch_bounds__(kThreads) void probe_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += 4 * stride) {
        f32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * stride < n16) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * stride < n16) dst[i + u * stride] = v[u];
    }
}

__global__ void probe_empty_kernel(int* sink)
{
    if (sink == nullptr) return;
    if (threadIdx.x == 0 && blockIdx.x == 0) sink[0] = 1;
}

}  // namespace

extern "C" int rn50_probe_mfma(int blocks, int iters, float* out, void* stream)
{
    RN50_REQUIRE_PTR(out);
    if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 24)) return RN50_ERR_SHAPE;
    probe_mfma_kernel<<<blocks, kThreads, 0, static_cast<hipStream_t>(stream)>>>(out, iters);
    return rn50_check_launch();
}

extern "C" int rn50_probe_tile_load(const void* src, size_t src_bytes, int blocks, int iters, int start_stride,
                                    int through_lds, float* out, void* stream)
{
    RN50_REQUIRE_PTR(src); RN50_REQUIRE_PTR(out); RN50_REQUIRE_ALIGNED(src);
    if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 20) || start_stride < 0) return RN50_ERR_SHAPE;
    if (src_bytes < (size_t)kTileBytes || src_bytes % kTileBytes != 0 || src_bytes > 0x7fffc000u) return RN50_ERR_SHAPE;
    const unsigned ntiles = (unsigned)(src_bytes / kTileBytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (through_lds)
        probe_tile_dma_kernel<<<blocks, kThreads, 0, s>>>(static_cast<const h16*>(src), (unsigned)src_bytes, ntiles,
                                                         (unsigned)start_stride, iters, out);
    else
        probe_tile_vec_kernel<<<blocks, kThreads, 0, s>>>(static_cast<const h16*>(src), ntiles, (unsigned)start_stride, iters, out);
    return rn50_check_launch();
}

extern "C" int rn50_probe_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    RN50_REQUIRE_PTR(src); RN50_REQUIRE_PTR(dst); RN50_REQUIRE_ALIGNED(src); RN50_REQUIRE_ALIGNED(dst);
    if (bytes < 16 || bytes % 16 != 0) return RN50_ERR_SHAPE;
    probe_copy_kernel<<<256 * 16, kThreads, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const f32x4*>(src),
                                                                                  static_cast<f32x4*>(dst), bytes / 16);
    return rn50_check_launch();
}

extern "C" int rn50_probe_empty(int count, void* stream)
{
    if (count < 1 || count > 100000) return RN50_ERR_SHAPE;
    for (int i = 0; i < count; ++i) probe_empty_kernel<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>(nullptr);
    return rn50_check_launch();
}
