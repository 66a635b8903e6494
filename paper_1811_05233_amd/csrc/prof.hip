// Per-kernel HIP-event timing behind rn50_profile_begin / rn50_profile_end.
#include <vector>

#include "prof.h"

namespace {

const char* const kNames[RN50_K_COUNT] = {
    "gather_gemm_kernel<128,128,32,4,2>", "gather_gemm_kernel<128,64,32,4,2>", "gather_gemm_kernel<64,64,64,4,2>",
    "gather_gemm_kernel<64,64,64,2,4>", "gather_gemm_kernel<64,64,32,4,4>", "gather_gemm_kernel<128,64,32,2,4>",
    "gather_gemm_kernel<128,128,32,2,3>", "gather_gemm_kernel<256,64,32,3,2>", "gather_gemm_kernel<128,64,64,3,2>",
    "gather_gemm_kernel<64,64,128,2,2>", "gather_gemm_kernel<128,64,128,2,1>", "gather_gemm_kernel<64,64,256,2,1>",
    "gather_gemm_kernel<128,128,64,2,2>", "gather_gemm_kernel<256,64,64,2,2>", "gather_gemm_kernel<256,128,64,2,1>",
    "strip_gemm_kernel<256,4,1,2,1>", "strip_gemm_kernel<128,2,2,2,1>", "strip_gemm_kernel<64,2,2,2,1>",
    "strip_gemm_kernel<256,4,1,1,2>", "strip_gemm_kernel<128,2,2,1,3>", "strip_gemm_kernel<64,2,2,1,3>",
    "gather_gemm_kernel<128,128,32,2,4>",
    "gather_gemm_kernel (stem forward)",
    "wgrad_kernel<128,128,4,64,false,32>", "wgrad_kernel<64,64,4,64,false,32>", "wgrad_kernel<64,128,4,64,false,32>",
    "wgrad_kernel<128,64,4,64,false,32>", "wgrad_kernel<64,64,3,64,false,64>", "wgrad_kernel<64,64,2,64,false,64>",
    "wgrad_kernel<64,64,2,64,false,128>", "wgrad_kernel<64,128,3,64,false,64>", "wgrad_kernel<128,64,3,64,false,64>",
    "wgrad_kernel<128,128,2,64,false,64>", "wgrad_strip_kernel", "wgrad_kernel<64,64,4,32,true,32> (stem)",
    "wgrad_reduce_kernel",
    "bn_stats_kernel", "bn_finalize_kernel<0,*> (forward statistics)", "bn_apply_kernel", "bn_fused_apply_kernel (finalize + apply)",
    "bn_bwd_reduce_kernel", "bn_finalize_kernel<1,*> (backward sums)", "bn_bwd_apply_kernel", "bn_bwd_fused_apply_kernel (finalize + apply)",
    "sgd_momentum_kernel", "lars_norm_kernel", "lars_rate_kernel", "lars_update_kernel", "cast_f32_to_h16_kernel", "fill_zero_kernel", "transpose_all_kernel",
    "maxpool/avgpool kernels", "fc kernels", "ls_xent_kernel", "stem pad/pack/unpack kernels"};

struct Span { int kernel; double flops, bytes; hipEvent_t e0, e1; bool side; };

struct Profiler {
    bool active = false;
    std::vector<hipEvent_t> pool;     // recycled events
    std::vector<Span> spans;
    std::vector<hipStream_t> side_streams;   // library-owned second streams (their launches overlap the caller's chain)
    Span cur;
};

Profiler g_prof;

hipEvent_t take_event()
{
    if (!g_prof.pool.empty()) { hipEvent_t e = g_prof.pool.back(); g_prof.pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

}  // namespace

bool rn50_prof_active() { return g_prof.active; }

void rn50_prof_note_side_stream(hipStream_t s, bool add)
{
    std::vector<hipStream_t>& v = g_prof.side_streams;
    for (size_t i = 0; i < v.size(); ++i)
        if (v[i] == s) { if (!add) v.erase(v.begin() + i); return; }
    if (add) v.push_back(s);
}

void rn50_prof_record_begin(int kernel, double flops, double bytes, hipStream_t s)
{
    bool side = false;
    for (hipStream_t t : g_prof.side_streams) side = side || t == s;
    g_prof.cur = {kernel, flops, bytes, take_event(), take_event(), side};
    (void)hipEventRecord(g_prof.cur.e0, s);
}

void rn50_prof_record_end(hipStream_t s)
{
    (void)hipEventRecord(g_prof.cur.e1, s);
    g_prof.spans.push_back(g_prof.cur);
}

extern "C" int rn50_profile_begin(void)
{
    for (Span& sp : g_prof.spans) { g_prof.pool.push_back(sp.e0); g_prof.pool.push_back(sp.e1); }
    g_prof.spans.clear();
    g_prof.active = true;
    return RN50_OK;
}

extern "C" int rn50_profile_end(rn50_profile_entry* out, int max_entries, int* n_out)
{
    if (!out || !n_out) return RN50_ERR_NULL;
    g_prof.active = false;
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return rn50_hip_fail(e);
    double ms[RN50_K_COUNT] = {0}, fl[RN50_K_COUNT] = {0}, by[RN50_K_COUNT] = {0};
    long long cnt[RN50_K_COUNT] = {0}, side[RN50_K_COUNT] = {0};
    for (Span& sp : g_prof.spans) {
        float t = 0.f;
        e = hipEventElapsedTime(&t, sp.e0, sp.e1);
        if (e != hipSuccess) return rn50_hip_fail(e);
        ms[sp.kernel] += t; fl[sp.kernel] += sp.flops; by[sp.kernel] += sp.bytes; cnt[sp.kernel] += 1; side[sp.kernel] += sp.side ? 1 : 0;
        g_prof.pool.push_back(sp.e0); g_prof.pool.push_back(sp.e1);
    }
    g_prof.spans.clear();
    int n = 0;
    for (int k = 0; k < RN50_K_COUNT && n < max_entries; ++k) {
        if (!cnt[k]) continue;
        out[n].name = kNames[k];
        out[n].launches = cnt[k];
        out[n].total_ms = ms[k];
        out[n].flops = fl[k];
        out[n].bytes = by[k];
        out[n].side_launches = side[k];
        ++n;
    }
    *n_out = n;
    return RN50_OK;
}
