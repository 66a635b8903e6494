// Optional per-kernel timing with HIP events (off unless rn50_profile_begin was called).
// Every launcher wraps its launch in a ProfScope naming the kernel and its algorithmic work.
#pragma once
#include "common.h"

enum Rn50Kernel {
    RN50_K_GATHER_TILE0 = 0,        // conv forward / data gradient: one id per tile variant (RN50_TILE_* order)
    RN50_K_GATHER_TILE_LAST = 21,
    RN50_K_GATHER_STEM,             // stem forward (32-wide K slabs, any of the tiles that fit it)
    RN50_K_WGRAD_TILE0,             // filter gradient: one id per tile variant
    RN50_K_WGRAD_TILE_LAST = RN50_K_WGRAD_TILE0 + 10,
    RN50_K_WGRAD_STEM,
    RN50_K_WGRAD_REDUCE,
    RN50_K_BN_STATS,
    RN50_K_BN_STATS_FINALIZE,
    RN50_K_BN_APPLY,
    RN50_K_BN_FUSED_APPLY,
    RN50_K_BN_BWD_REDUCE,
    RN50_K_BN_BWD_FINALIZE,
    RN50_K_BN_BWD_APPLY,
    RN50_K_BN_BWD_FUSED_APPLY,
    RN50_K_SGD,
    RN50_K_LARS_NORM,
    RN50_K_LARS_RATE,
    RN50_K_LARS_UPDATE,
    RN50_K_CAST,
    RN50_K_FILL,
    RN50_K_TRANSPOSE,
    RN50_K_POOL,
    RN50_K_FC,
    RN50_K_LOSS,
    RN50_K_STEM_MISC,
    RN50_K_COUNT
};

bool rn50_prof_active();
// a context's second stream is announced (add) and withdrawn (!add), so that launches on it can be told apart
void rn50_prof_note_side_stream(hipStream_t s, bool add);
void rn50_prof_record_begin(int kernel, double flops, double bytes, hipStream_t s);
void rn50_prof_record_end(hipStream_t s);

struct ProfScope {
    hipStream_t s;
    bool on;
    ProfScope(int kernel, double flops, double bytes, hipStream_t stream) : s(stream), on(rn50_prof_active()) {
        if (on) rn50_prof_record_begin(kernel, flops, bytes, s);
    }
    ~ProfScope() { if (on) rn50_prof_record_end(s); }
};
