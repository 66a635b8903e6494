// Internal helpers shared by the HIP translation units of librn50 (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "rn50.h"

typedef _Float16 h16;
typedef h16 h16x2 __attribute__((ext_vector_type(2)));
typedef h16 h16x4 __attribute__((ext_vector_type(4)));
typedef h16 h16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

extern thread_local int rn50_tls_hip_error;

static inline int rn50_hip_fail(hipError_t e) {
    rn50_tls_hip_error = (int)e;
    return RN50_ERR_HIP;
}
// Call after a kernel launch: turns a launch failure into RN50_ERR_HIP.
static inline int rn50_check_launch() {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? RN50_OK : rn50_hip_fail(e);
}
static inline bool rn50_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define RN50_REQUIRE_PTR(p) do { if ((p) == nullptr) return RN50_ERR_NULL; } while (0)
#define RN50_REQUIRE_ALIGNED(p) do { if (!rn50_aligned16(p)) return RN50_ERR_ALIGN; } while (0)
#define RN50_TRY(expr) do { int rn50_rc_ = (expr); if (rn50_rc_ != RN50_OK) return rn50_rc_; } while (0)

static inline size_t rn50_round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int rn50_cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  This maps the hardware index
// to a logical one such that every XCD gets a contiguous range of logical indices, so that neighbouring
// tiles, which share operands, share an L2.
__device__ __forceinline__ int rn50_xcd_remap(int bid, int nblk) {
    const int full = nblk & ~7;
    if (bid >= full) return bid;
    return (bid & 7) * (full >> 3) + (bid >> 3);
}
