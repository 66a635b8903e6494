// Whole-iteration driver: walks the ResNet-50 v1.5 layer table and enqueues forward, loss,
// backward and the momentum-SGD (or LARS) update with no host synchronisation.  The caller's
// stream carries the dependent chain; a second stream owned by the context takes the work that
// only branches off it (projection shortcuts, filter gradients, the filter re-layout) and is
// joined back before the update.  The context is a host object; every device byte lives in the
// caller's workspace.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "common.h"
#include "conv_internal.h"
#include "misc_internal.h"
#include "prof.h"

namespace {

constexpr int kThreads = 256;

struct Segment { size_t offset, count; int kind, fan_in; };

struct ConvLayer {
    std::string name;
    conv_desc d;
    int P, Q;
    size_t w_off, gamma_off, beta_off;   // element offsets into the flat parameter layout
    size_t wt_off;                       // element offset into the transposed-filter buffer
    // workspace tensors
    h16* conv_out = nullptr;
    h16* bn_out = nullptr;
    float* mean = nullptr;
    float* invstd = nullptr;
    h16* dconv = nullptr;                // gradient w.r.t. the conv output (BN backward result)
    h16* din = nullptr;                  // gradient w.r.t. the conv input (data-gradient result)
    bool din_compact = false;            // strided 1x1 (projection): din holds the (even, even) input pixels only,
                                         //   [n][P][Q][c]; the gradient is zero at all other pixels
    h16* dres = nullptr;                 // conv3 only: masked gradient handed to the shortcut
    // kernel variants (RN50_TILE_AUTO until rn50_autotune has measured them)
    int fwd_tile = RN50_TILE_AUTO, dgrad_tile = RN50_TILE_AUTO, wgrad_variant = RN50_TILE_AUTO;
    size_t in_elems() const { return (size_t)d.n * d.h * d.w * d.c; }
    size_t out_elems() const { return (size_t)d.n * P * Q * d.k; }
};

struct Block { int c1, c2, c3, proj; };   // indices into layers (proj = -1 if none)

struct Layout {
    std::vector<Segment> segments;
    std::vector<ConvLayer> layers;
    std::vector<Block> blocks;
    size_t param_count = 0;
    size_t fcw_off = 0, fcb_off = 0;
    int feat = 0, final_h = 0, final_w = 0;
    int pool_in_h = 0, pool_in_w = 0, pool_h = 0, pool_w = 0;
};

bool config_ok(const rn50_config* c)
{
    if (!c) return false;
    if (c->dt != RN50_F16) return false;
    if (c->batch < 1 || c->batch > 4096 || c->image_h < 1 || c->image_w < 1) return false;
    if (c->num_stages < 1 || c->num_stages > 4) return false;
    for (int s = 0; s < c->num_stages; ++s) if (c->blocks[s] < 1 || c->blocks[s] > 64) return false;
    if (c->base_width < 64 || c->base_width % 64 != 0 || c->base_width > 1024) return false;
    if (c->classes < 8 || c->classes % 8 != 0 || c->classes > 65536) return false;
    if (c->has_stem && (c->image_h % 2 != 0 || c->image_w % 2 != 0)) return false;
    if (!(c->bn_eps > 0.f) || !(c->loss_scale > 0.f) || c->ls_eps < 0.f || c->ls_eps >= 1.f) return false;
    return true;
}

int out_dim(int h, int pad, int r, int stride) { return (h + 2 * pad - r) / stride + 1; }

// Builds segments, layers and blocks; returns false if some layer has an unsupported shape.
bool build_layout(const rn50_config& c, Layout& L)
{
    size_t off = 0, wt_off = 0;
    auto add_seg = [&](size_t count, int kind, int fan_in) {
        L.segments.push_back({off, count, kind, fan_in});
        off += count;
        return off - count;
    };
    auto add_conv = [&](const std::string& name, int h, int w, int cin, int cout, int r, int stride, int pad) -> int {
        ConvLayer l;
        l.name = name;
        l.d = {c.batch, h, w, cin, cout, r, r, stride, pad, RN50_F16};
        l.P = out_dim(h, pad, r, stride);
        l.Q = out_dim(w, pad, r, stride);
        l.w_off = add_seg((size_t)cout * r * r * cin, RN50_KIND_CONV, cin * r * r);
        l.gamma_off = add_seg(cout, RN50_KIND_GAMMA, 0);
        l.beta_off = add_seg(cout, RN50_KIND_BETA, 0);
        l.wt_off = wt_off;
        if (cin != 3) wt_off += (size_t)cout * r * r * cin;
        L.layers.push_back(l);
        return (int)L.layers.size() - 1;
    };
    int h = c.image_h, w = c.image_w;
    if (c.has_stem) {
        const int i = add_conv("stem", h, w, 3, c.base_width, 7, 2, 3);
        L.pool_in_h = L.layers[i].P; L.pool_in_w = L.layers[i].Q;
        h = out_dim(L.pool_in_h, 1, 3, 2); w = out_dim(L.pool_in_w, 1, 3, 2);
        L.pool_h = h; L.pool_w = w;
    }
    int cin = c.base_width;
    for (int s = 0; s < c.num_stages; ++s) {
        const int width = c.base_width << s, cout = 4 * width;
        for (int b = 0; b < c.blocks[s]; ++b) {
            const int stride = (b == 0 && s > 0) ? 2 : 1;
            const std::string nm = "s" + std::to_string(s + 1) + "b" + std::to_string(b);
            Block blk;
            blk.c1 = add_conv(nm + "c1", h, w, cin, width, 1, 1, 0);
            blk.c2 = add_conv(nm + "c2", h, w, width, width, 3, stride, 1);
            const int h2 = L.layers[blk.c2].P, w2 = L.layers[blk.c2].Q;
            blk.c3 = add_conv(nm + "c3", h2, w2, width, cout, 1, 1, 0);
            blk.proj = (b == 0) ? add_conv(nm + "p", h, w, cin, cout, 1, stride, 0) : -1;
            if (blk.proj >= 0 && stride == 2) L.layers[blk.proj].din_compact = true;
            L.blocks.push_back(blk);
            h = h2; w = w2; cin = cout;
        }
    }
    L.feat = cin; L.final_h = h; L.final_w = w;
    L.fcw_off = add_seg((size_t)c.classes * cin, RN50_KIND_FCW, cin);
    L.fcb_off = add_seg((size_t)c.classes, RN50_KIND_FCB, cin);
    L.param_count = off;
    for (const ConvLayer& l : L.layers)
        if (rn50_conv_validate(&l.d) != RN50_OK || l.P < 1 || l.Q < 1) return false;
    return h >= 1 && w >= 1;
}

// ---- batched filter transpose: every non-stem filter KRSC -> CRSK in one launch ----
struct TransposeJob { unsigned long long src_off, dst_off; int K, T, C, block_end; };

__global__ __launch_bounds__(kThreads) void transpose_all_kernel(const h16* __restrict__ w, h16* __restrict__ wt,
                                                                 const TransposeJob* __restrict__ jobs, int njobs)
{
    __shared__ h16 tile[32][33];
    int lo = 0, hi = njobs - 1;
    const int b = blockIdx.x;
    while (lo < hi) {                     // first job whose block_end exceeds b
        const int mid = (lo + hi) >> 1;
        if (jobs[mid].block_end > b) hi = mid; else lo = mid + 1;
    }
    const TransposeJob j = jobs[lo];
    int lb = b - (lo ? jobs[lo - 1].block_end : 0);
    const int tiles_c = j.C / 32, tiles_k = j.K / 32;
    const int tc = lb % tiles_c; lb /= tiles_c;
    const int tk = lb % tiles_k;
    const int t = lb / tiles_k;
    const h16* src = w + j.src_off;
    h16* dst = wt + j.dst_off;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        tile[ty + i * 8][tx] = src[((size_t)(tk * 32 + ty + i * 8) * j.T + t) * j.C + tc * 32 + tx];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i)
        dst[((size_t)(tc * 32 + ty + i * 8) * j.T + t) * j.K + tk * 32 + tx] = tile[tx][ty + i * 8];
}

}  // namespace

struct rn50_ctx {
    rn50_config cfg;
    Layout L;
    // workspace carve-up
    char* ws = nullptr;
    size_t ws_bytes = 0;
    h16* stem_padded = nullptr;
    h16* stem_packed = nullptr;
    float* stem_wacc = nullptr;
    h16* pool_out = nullptr;
    uint8_t* pool_arg = nullptr;
    h16* feat = nullptr;
    float* logits = nullptr;
    h16* dlogits = nullptr;
    h16* wt_all = nullptr;        // transposed filters
    float* bn_ws = nullptr;
    float* bn_ws_side = nullptr;  // BN partial sums of the projection branch (forward, side stream)
    float* wgrad_part = nullptr;  // per-split partial tiles of the filter gradient
    void* lars_ws = nullptr;      // device tables and scratch of the LARS plan
    size_t lars_ws_bytes = 0;
    lars_plan* lars = nullptr;
    h16* head_din = nullptr;      // gradient w.r.t. the last block's output (from the FC / avg-pool backward)
    h16* pool_din = nullptr;      // gradient w.r.t. the stem's BN output (from the max-pool backward)
    TransposeJob* jobs = nullptr;
    int njobs = 0, transpose_blocks = 0;
    // filter gradients run on a second stream, next to the data-gradient / BN-backward chain
    hipStream_t side = nullptr;
    std::vector<hipEvent_t> fork_events;   // one per conv layer: "d(conv output) is ready"
    hipEvent_t join_event = nullptr;
    hipEvent_t transpose_fork = nullptr, transpose_done = nullptr;
    bool tuning = false;                   // rn50_autotune: every conv launch site times its variants
    std::string tune_report;               // what the last rn50_autotune measured, one line per launch site and candidate
    hipEvent_t tune_e0 = nullptr, tune_e1 = nullptr;
    size_t max_act = 0, wt_elems = 0;
};

namespace {

// Layer-wise scaling applies to the convolution filters and the FC weight; BN scale / shift and the FC bias
// are updated with plain momentum.
std::vector<rn50_lars_segment> lars_segments(const Layout& L)
{
    std::vector<rn50_lars_segment> segs;
    for (const Segment& sg : L.segments)
        segs.push_back({sg.offset, sg.count, (sg.kind == RN50_KIND_CONV || sg.kind == RN50_KIND_FCW) ? 1 : 0});
    return segs;
}

// Lays the workspace out; with base == nullptr only the size is computed.
size_t carve(rn50_ctx& c, char* base)
{
    size_t off = 0;
    auto take = [&](size_t bytes) -> char* {
        char* p = base ? base + off : nullptr;
        off += rn50_round_up(bytes, 256);
        return p;
    };
    const rn50_config& cfg = c.cfg;
    Layout& L = c.L;
    size_t max_act = (size_t)cfg.batch * cfg.image_h * cfg.image_w * (cfg.has_stem ? 4 : cfg.base_width);
    size_t wt_elems = 0;
    int max_c = cfg.base_width;
    for (ConvLayer& l : L.layers) {
        l.conv_out = reinterpret_cast<h16*>(take(l.out_elems() * sizeof(h16)));
        l.bn_out = reinterpret_cast<h16*>(take(l.out_elems() * sizeof(h16)));
        l.mean = reinterpret_cast<float*>(take(l.d.k * sizeof(float)));
        l.invstd = reinterpret_cast<float*>(take(l.d.k * sizeof(float)));
        if (l.out_elems() > max_act) max_act = l.out_elems();
        if (l.in_elems() > max_act && l.d.c != 3) max_act = l.in_elems();
        if (l.d.c != 3) wt_elems += (size_t)l.d.k * l.d.r * l.d.s * l.d.c;
        if (l.d.k > max_c) max_c = l.d.k;
    }
    c.max_act = max_act; c.wt_elems = wt_elems;
    if (cfg.has_stem) {
        const ConvLayer& st = L.layers[0];
        c.stem_padded = reinterpret_cast<h16*>(take(rn50_stem_padded_bytes(st.d)));
        c.stem_packed = reinterpret_cast<h16*>(take(rn50_stem_packed_filter_bytes(st.d)));
        c.stem_wacc = reinterpret_cast<float*>(take(rn50_wgrad_acc_floats(st.d) * sizeof(float)));
        const size_t pool_elems = (size_t)cfg.batch * L.pool_h * L.pool_w * cfg.base_width;
        c.pool_out = reinterpret_cast<h16*>(take(pool_elems * sizeof(h16)));
        c.pool_arg = reinterpret_cast<uint8_t*>(take(pool_elems));
    }
    c.feat = reinterpret_cast<h16*>(take((size_t)cfg.batch * L.feat * sizeof(h16)));
    c.logits = reinterpret_cast<float*>(take((size_t)cfg.batch * cfg.classes * sizeof(float)));
    c.dlogits = reinterpret_cast<h16*>(take((size_t)cfg.batch * cfg.classes * sizeof(h16)));
    c.wt_all = reinterpret_cast<h16*>(take(wt_elems * sizeof(h16)));
    size_t bn_ws_floats = rn50_bn_ws_floats(max_c);
    for (const ConvLayer& l : L.layers) {
        if (rn50_conv_stats_floats(l.d) > bn_ws_floats) bn_ws_floats = rn50_conv_stats_floats(l.d);
        if (l.d.c != 3 && rn50_dgrad_stats_floats(l.d) + 2 * (size_t)l.d.c > bn_ws_floats)
            bn_ws_floats = rn50_dgrad_stats_floats(l.d) + 2 * (size_t)l.d.c;
    }
    c.bn_ws = reinterpret_cast<float*>(take(bn_ws_floats * sizeof(float)));
    c.bn_ws_side = reinterpret_cast<float*>(take(bn_ws_floats * sizeof(float)));
    size_t part_floats = 4;
    for (const ConvLayer& l : L.layers)
        if (rn50_wgrad_partial_floats(l.d) > part_floats) part_floats = rn50_wgrad_partial_floats(l.d);
    c.wgrad_part = reinterpret_cast<float*>(take(part_floats * sizeof(float)));
    // Activation gradients.  Normally five rotating buffers (two alternate as block-input gradients,
    // one holds the shortcut gradient, two are scratch inside a block) plus d(conv output) per layer;
    // with keep_grads every gradient tensor gets its own buffer so that it can be inspected afterwards.
    const int nb = (int)L.blocks.size();
    if (cfg.keep_grads) {
        for (ConvLayer& l : L.layers) {
            l.dconv = reinterpret_cast<h16*>(take(l.out_elems() * sizeof(h16)));
            l.din = reinterpret_cast<h16*>(take(l.in_elems() * sizeof(h16)));
        }
        for (const Block& b : L.blocks)
            L.layers[b.c3].dres = reinterpret_cast<h16*>(take(L.layers[b.c3].out_elems() * sizeof(h16)));
        c.head_din = reinterpret_cast<h16*>(take(L.layers[L.blocks[nb - 1].c3].out_elems() * sizeof(h16)));
        c.pool_din = cfg.has_stem ? reinterpret_cast<h16*>(take(L.layers[0].out_elems() * sizeof(h16))) : nullptr;
    } else {
        // d(conv output) keeps a buffer of its own per layer: the filter gradient reads it on the side
        // stream while the main stream already produces the next layer's gradients
        for (ConvLayer& l : L.layers) l.dconv = reinterpret_cast<h16*>(take(l.out_elems() * sizeof(h16)));
        h16* g[5];
        for (int i = 0; i < 5; ++i) g[i] = reinterpret_cast<h16*>(take(max_act * sizeof(h16)));
        for (int bi = 0; bi < nb; ++bi) {
            const Block& b = L.blocks[bi];
            L.layers[b.c3].dres = g[2];
            L.layers[b.c3].din = g[3];
            L.layers[b.c2].din = g[3];
            L.layers[b.c1].din = g[bi % 2];
            if (b.proj >= 0) L.layers[b.proj].din = g[4];
        }
        c.head_din = g[nb % 2];
        if (cfg.has_stem) c.pool_din = g[3];
    }
    // conv3's masked shortcut gradient is the (masked) block-output gradient itself whenever that was
    // produced by the next block's conv1 data gradient; only the last block keeps a buffer of its own
    for (int bi = 0; bi + 1 < nb; ++bi) L.layers[L.blocks[bi].c3].dres = L.layers[L.blocks[bi + 1].c1].din;
    c.jobs = reinterpret_cast<TransposeJob*>(take(L.layers.size() * sizeof(TransposeJob)));
    {
        const std::vector<rn50_lars_segment> segs = lars_segments(L);
        c.lars_ws_bytes = lars_workspace_bytes(segs.data(), (int)segs.size());
        c.lars_ws = take(c.lars_ws_bytes);
    }
    return off;
}

}  // namespace

extern "C" size_t rn50_param_count(const rn50_config* cfg)
{
    Layout L;
    if (!config_ok(cfg) || !build_layout(*cfg, L)) return 0;
    return L.param_count;
}

extern "C" int rn50_num_segments(const rn50_config* cfg)
{
    Layout L;
    if (!config_ok(cfg) || !build_layout(*cfg, L)) return 0;
    return (int)L.segments.size();
}

extern "C" int rn50_param_layout(const rn50_config* cfg, int idx, size_t* offset, size_t* count, int* kind, int* fan_in)
{
    Layout L;
    if (!cfg) return RN50_ERR_NULL;
    if (!config_ok(cfg) || !build_layout(*cfg, L)) return RN50_ERR_SHAPE;
    if (idx < 0 || idx >= (int)L.segments.size()) return RN50_ERR_SHAPE;
    const Segment& s = L.segments[idx];
    if (offset) *offset = s.offset;
    if (count) *count = s.count;
    if (kind) *kind = s.kind;
    if (fan_in) *fan_in = s.fan_in;
    return RN50_OK;
}

extern "C" size_t rn50_workspace_bytes(const rn50_config* cfg)
{
    if (!config_ok(cfg)) return 0;
    rn50_ctx c;
    c.cfg = *cfg;
    if (!build_layout(*cfg, c.L)) return 0;
    return carve(c, nullptr);
}

extern "C" int rn50_create(rn50_ctx** out, const rn50_config* cfg, void* workspace, size_t workspace_bytes)
{
    if (!out || !cfg) return RN50_ERR_NULL;
    *out = nullptr;
    if (cfg->dt != RN50_F16) return RN50_ERR_DTYPE;
    if (!config_ok(cfg)) return RN50_ERR_SHAPE;
    rn50_ctx* c = new rn50_ctx();
    c->cfg = *cfg;
    if (!build_layout(*cfg, c->L)) { delete c; return RN50_ERR_SHAPE; }
    const size_t need = carve(*c, nullptr);
    if (!workspace || workspace_bytes < need) { delete c; return RN50_ERR_WORKSPACE; }
    if (!rn50_aligned16(workspace)) { delete c; return RN50_ERR_ALIGN; }
    c->ws = static_cast<char*>(workspace);
    c->ws_bytes = workspace_bytes;
    carve(*c, c->ws);
    // job table of the batched filter transpose (uploaded once, synchronously)
    std::vector<TransposeJob> jobs;
    int blocks = 0;
    for (const ConvLayer& l : c->L.layers) {
        if (l.d.c == 3) continue;
        const int T = l.d.r * l.d.s;
        blocks += (l.d.c / 32) * (l.d.k / 32) * T;
        jobs.push_back({(unsigned long long)l.w_off, (unsigned long long)l.wt_off, l.d.k, T, l.d.c, blocks});
    }
    c->njobs = (int)jobs.size();
    c->transpose_blocks = blocks;
    if (!jobs.empty()) {
        hipError_t e = hipMemcpy(c->jobs, jobs.data(), jobs.size() * sizeof(TransposeJob), hipMemcpyHostToDevice);
        if (e != hipSuccess) { delete c; return rn50_hip_fail(e); }
    }
    {
        const std::vector<rn50_lars_segment> segs = lars_segments(c->L);
        const int rc = lars_plan_create(&c->lars, segs.data(), (int)segs.size(), c->lars_ws, c->lars_ws_bytes);
        if (rc != RN50_OK) { delete c; return rc; }
    }
    hipError_t e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->join_event, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->transpose_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->transpose_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreate(&c->tune_e0);
    if (e == hipSuccess) e = hipEventCreate(&c->tune_e1);
    c->fork_events.assign(c->L.layers.size(), nullptr);
    for (size_t i = 0; e == hipSuccess && i < c->fork_events.size(); ++i)
        e = hipEventCreateWithFlags(&c->fork_events[i], hipEventDisableTiming);
    if (e != hipSuccess) { rn50_destroy(c); return rn50_hip_fail(e); }
    rn50_prof_note_side_stream(c->side, true);
    *out = c;
    return RN50_OK;
}

extern "C" void rn50_destroy(rn50_ctx* ctx)
{
    if (!ctx) return;
    for (hipEvent_t ev : ctx->fork_events) if (ev) (void)hipEventDestroy(ev);
    if (ctx->join_event) (void)hipEventDestroy(ctx->join_event);
    if (ctx->transpose_fork) (void)hipEventDestroy(ctx->transpose_fork);
    if (ctx->transpose_done) (void)hipEventDestroy(ctx->transpose_done);
    if (ctx->tune_e0) (void)hipEventDestroy(ctx->tune_e0);
    if (ctx->tune_e1) (void)hipEventDestroy(ctx->tune_e1);
    if (ctx->side) { rn50_prof_note_side_stream(ctx->side, false); (void)hipStreamDestroy(ctx->side); }
    lars_plan_destroy(ctx->lars);
    delete ctx;
}

extern "C" int rn50_tensor(rn50_ctx* ctx, const char* name, void** ptr, size_t* elems, int* elem_bytes)
{
    if (!ctx || !name || !ptr || !elems || !elem_bytes) return RN50_ERR_NULL;
    const rn50_config& cfg = ctx->cfg;
    const std::string nm(name);
    auto set = [&](void* p, size_t n, int eb) { *ptr = p; *elems = n; *elem_bytes = eb; return RN50_OK; };
    if (nm == "feat") return set(ctx->feat, (size_t)cfg.batch * ctx->L.feat, 2);
    if (nm == "logits") return set(ctx->logits, (size_t)cfg.batch * cfg.classes, 4);
    if (nm == "dlogits") return set(ctx->dlogits, (size_t)cfg.batch * cfg.classes, 2);
    if (nm == "pool.out" && cfg.has_stem)
        return set(ctx->pool_out, (size_t)cfg.batch * ctx->L.pool_h * ctx->L.pool_w * cfg.base_width, 2);
    if (cfg.keep_grads) {
        if (nm == "head.din") return set(ctx->head_din, ctx->L.layers[ctx->L.blocks.back().c3].out_elems(), 2);
        if (nm == "pool.din" && cfg.has_stem) return set(ctx->pool_din, ctx->L.layers[0].out_elems(), 2);
    }
    const size_t dot = nm.rfind('.');
    if (dot == std::string::npos) return RN50_ERR_SHAPE;
    const std::string layer = nm.substr(0, dot), what = nm.substr(dot + 1);
    for (ConvLayer& l : ctx->L.layers) {
        if (l.name != layer) continue;
        if (what == "conv") return set(l.conv_out, l.out_elems(), 2);
        if (what == "out") return set(l.bn_out, l.out_elems(), 2);
        if (what == "mean") return set(l.mean, (size_t)l.d.k, 4);
        if (what == "invstd") return set(l.invstd, (size_t)l.d.k, 4);
        if (cfg.keep_grads) {
            if (what == "dconv") return set(l.dconv, l.out_elems(), 2);
            if (what == "din" && l.d.c != 3)
                return set(l.din, l.din_compact ? (size_t)l.d.n * l.P * l.Q * l.d.c : l.in_elems(), 2);
            if (what == "dres" && l.dres) return set(l.dres, l.out_elems(), 2);
        }
    }
    return RN50_ERR_SHAPE;
}

namespace {
// Launch site with variants.  Normally launches variant *choice.  In tuning mode it times every variant
// (one warm-up, two timed launches, device-synchronous) on stream s, stores the fastest in *choice and
// leaves its (identical) result in place.
inline float no_penalty(int) { return 0.f; }

// A convolution whose epilogue leaves more row tiles of BatchNorm partial sums than the apply kernel combines by
// itself costs one more (small, dependent) launch afterwards: charged to the tile variants that cause it.
inline float finalize_penalty(long long rows, int tile)
{
    const int per = rn50_gather_tile_rows(tile);
    return (rows + per - 1) / per > rn50_bn_fused_max_tiles() ? 0.008f : 0.f;
}

// penalty_ms(cand) is added to a candidate's measured time (cost the timing in isolation does not show).
// cand_flag is or-ed to every candidate while tuning (RN50_TILE_STRICT: candidates that do not apply are skipped).
template <class F, class G = float (*)(int)>
int launch_or_tune(rn50_ctx& c, hipStream_t s, int ncand, int* choice, F launch, const char* what = "", const char* layer = "",
                   G penalty_ms = no_penalty, int cand_flag = 0)
{
    if (!c.tuning) {
        if (*choice >= 0 && cand_flag) {
            // a table entry that does not apply to this shape is replaced by the heuristic, visibly (rn50_get_tuning)
            const int rc = launch(*choice | cand_flag);
            if (rc != RN50_ERR_SHAPE) return rc;
            *choice = RN50_TILE_AUTO;
        }
        return launch(*choice);
    }
    char line[160];
    float best_ms = 1e30f;
    int best = RN50_TILE_AUTO;
    for (int cand = 0; cand < ncand; ++cand) {
        const int first = launch(cand | cand_flag);
        if (first == RN50_ERR_SHAPE && cand_flag) continue;       // not applicable to this shape
        RN50_TRY(first);
        hipError_t e = hipEventRecord(c.tune_e0, s);
        if (e != hipSuccess) return rn50_hip_fail(e);
        RN50_TRY(launch(cand | cand_flag));
        RN50_TRY(launch(cand | cand_flag));
        e = hipEventRecord(c.tune_e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(c.tune_e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, c.tune_e0, c.tune_e1);
        if (e != hipSuccess) return rn50_hip_fail(e);
        ms = ms * 0.5f + penalty_ms(cand);
        if (ms < best_ms) { best_ms = ms; best = cand; }
        snprintf(line, sizeof line, "tune %s %s cand %d: %.1f us\n", layer, what, cand, ms * 1000.f);
        c.tune_report += line;
    }
    snprintf(line, sizeof line, "tune %s %s -> %d (%.1f us)\n", layer, what, best, best_ms * 1000.f);
    c.tune_report += line;
    *choice = best;
    return launch(best);
}
}  // namespace

extern "C" int rn50_step(rn50_ctx* ctx, const void* images, const int32_t* labels, float* master_w, float* momentum,
                         void* w_lowp, void* grad_lowp, const rn50_hparams* hp, float* loss_out, void* stream)
{
    RN50_REQUIRE_PTR(ctx); RN50_REQUIRE_PTR(images); RN50_REQUIRE_PTR(labels); RN50_REQUIRE_PTR(master_w);
    RN50_REQUIRE_PTR(w_lowp); RN50_REQUIRE_PTR(grad_lowp); RN50_REQUIRE_PTR(loss_out);
    if (hp) RN50_REQUIRE_PTR(momentum);
    RN50_REQUIRE_ALIGNED(images); RN50_REQUIRE_ALIGNED(master_w); RN50_REQUIRE_ALIGNED(momentum);
    RN50_REQUIRE_ALIGNED(w_lowp); RN50_REQUIRE_ALIGNED(grad_lowp);
    hipStream_t s = static_cast<hipStream_t>(stream);
    rn50_ctx& c = *ctx;
    const rn50_config& cfg = c.cfg;
    Layout& L = c.L;
    const h16* w16 = static_cast<const h16*>(w_lowp);
    h16* g16 = static_cast<h16*>(grad_lowp);      // every gradient kernel stores its slice of the flat FP16 gradient itself
    const int B = cfg.batch;

    // ---- per-step preparation: re-lay the filters for the data gradient.  Only the backward pass needs
    // them, so this runs on the side stream next to the forward pass. ----
    if (c.njobs > 0) {
        hipError_t e = hipEventRecord(c.transpose_fork, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(c.side, c.transpose_fork, 0);
        if (e != hipSuccess) return rn50_hip_fail(e);
        {
            ProfScope ps(RN50_K_TRANSPOSE, 0.0, 4.0 * c.wt_elems, c.side);
            transpose_all_kernel<<<c.transpose_blocks, kThreads, 0, c.side>>>(w16, c.wt_all, c.jobs, c.njobs);
            RN50_TRY(rn50_check_launch());
        }
        e = hipEventRecord(c.transpose_done, c.side);
        if (e != hipSuccess) return rn50_hip_fail(e);
    }

    // convolution (its epilogue also leaves the BatchNorm partial sums of every row tile), then BN
    auto conv_bn_fwd = [&](ConvLayer& l, const h16* x, const h16* wts, bool relu, const h16* residual,
                           hipStream_t st, float* part) -> int {
        int tiles = 0;
        RN50_TRY(launch_or_tune(c, st, RN50_NUM_GATHER_TILES, &l.fwd_tile, [&](int tile) {
            return rn50_conv_fwd_launch(l.d, x, wts, l.conv_out, st, part, &tiles, tile);
        }, "fwd", l.name.c_str(), [&](int tile) { return finalize_penalty((long long)l.d.n * l.P * l.Q, tile); },
        RN50_TILE_STRICT));
        return rn50_bn_fwd_from_partials_launch((long long)l.d.n * l.P * l.Q, l.d.k, cfg.bn_eps, relu, l.conv_out,
                                                master_w + l.gamma_off, master_w + l.beta_off, residual, l.bn_out,
                                                l.mean, l.invstd, part, tiles, st);
    };

    // ================= forward =================
    const h16* x = static_cast<const h16*>(images);
    if (cfg.has_stem) {
        ConvLayer& st = L.layers[0];
        RN50_TRY(rn50_stem_pad_image(st.d, x, c.stem_padded, s));
        RN50_TRY(rn50_stem_pack_filter(st.d, w16 + st.w_off, c.stem_packed, s));
        RN50_TRY(conv_bn_fwd(st, c.stem_padded, c.stem_packed, true, nullptr, s, c.bn_ws));
        RN50_TRY(rn50_maxpool_fwd(B, st.P, st.Q, st.d.k, st.bn_out, c.pool_out, c.pool_arg, s));
        x = c.pool_out;
    }
    std::vector<const h16*> block_in(L.blocks.size());
    for (size_t bi = 0; bi < L.blocks.size(); ++bi) {
        const Block& b = L.blocks[bi];
        block_in[bi] = x;
        const h16* shortcut = x;
        if (b.proj >= 0) {
            // the projection shortcut (conv + BN) only depends on the block input: run it on the side
            // stream next to conv1 -> conv2 and join before conv3's BN adds it
            ConvLayer& lp = L.layers[b.proj];
            hipEvent_t ev = c.fork_events[b.proj];
            hipError_t e = hipEventRecord(ev, s);
            if (e == hipSuccess) e = hipStreamWaitEvent(c.side, ev, 0);
            if (e != hipSuccess) return rn50_hip_fail(e);
            RN50_TRY(conv_bn_fwd(lp, x, w16 + lp.w_off, false, nullptr, c.side, c.bn_ws_side));
            e = hipEventRecord(c.join_event, c.side);
            if (e != hipSuccess) return rn50_hip_fail(e);
            shortcut = lp.bn_out;
        }
        RN50_TRY(conv_bn_fwd(L.layers[b.c1], x, w16 + L.layers[b.c1].w_off, true, nullptr, s, c.bn_ws));
        RN50_TRY(conv_bn_fwd(L.layers[b.c2], L.layers[b.c1].bn_out, w16 + L.layers[b.c2].w_off, true, nullptr, s, c.bn_ws));
        if (b.proj >= 0) {
            hipError_t e = hipStreamWaitEvent(s, c.join_event, 0);
            if (e != hipSuccess) return rn50_hip_fail(e);
        }
        RN50_TRY(conv_bn_fwd(L.layers[b.c3], L.layers[b.c2].bn_out, w16 + L.layers[b.c3].w_off, true, shortcut, s, c.bn_ws));
        x = L.layers[b.c3].bn_out;
    }
    const int HW = L.final_h * L.final_w;
    RN50_TRY(rn50_avgpool_fwd(B, HW, L.feat, x, c.feat, s));
    RN50_TRY(rn50_fc_fwd(B, L.feat, cfg.classes, c.feat, w16 + L.fcw_off, master_w + L.fcb_off, c.logits, s));

    // ================= loss =================
    RN50_TRY(ls_xent_fwd_bwd(B, cfg.classes, c.logits, labels, cfg.ls_eps, cfg.loss_scale / (float)B, loss_out,
                             nullptr, c.dlogits, RN50_F16, stream));

    // ================= backward =================
    if (c.njobs > 0) {
        hipError_t e = hipStreamWaitEvent(s, c.transpose_done, 0);
        if (e != hipSuccess) return rn50_hip_fail(e);
    }
    {   // the FC weight gradient joins the filter gradients on the side stream (dlogits is ready from here on)
        hipError_t e = hipEventRecord(c.transpose_fork, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(c.side, c.transpose_fork, 0);
        if (e != hipSuccess) return rn50_hip_fail(e);
    }
    RN50_TRY(rn50_fc_bwd(B, L.feat, cfg.classes, HW, c.feat, w16 + L.fcw_off, c.dlogits, g16 + L.fcw_off, g16 + L.fcb_off,
                         c.head_din, c.side, s));

    // The filter gradient of a conv is queued on the side stream as soon as d(conv output) exists (it only
    // needs that and forward activations), so that it overlaps with the data-gradient / BN-backward chain.
    auto fork_wgrad = [&](ConvLayer& l, const h16* in, h16* out16, float* out32) -> int {
        hipEvent_t ev = c.fork_events[&l - &L.layers[0]];
        hipError_t e = hipEventRecord(ev, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(c.side, ev, 0);
        if (e != hipSuccess) return rn50_hip_fail(e);
        return launch_or_tune(c, c.side, l.d.c == 3 ? 3 : RN50_NUM_WGRAD_VARIANTS, &l.wgrad_variant, [&](int variant) {
            return rn50_conv_wgrad_launch(l.d, in, l.dconv, out16, out32, c.wgrad_part, c.side, variant);
        }, "wgrad", l.name.c_str(), [&](int variant) {
            // the partial tiles of a pixel split are written and read back through HBM, which the rest of the
            // step competes for; timing the variant on its own does not show that, so the traffic is charged at
            // a nominal 1.5 TB/s (the value that gave the shortest step among 0.7 .. 6 TB/s)
            const float gbs = 1500.f;
            return 2.f * (float)rn50_wgrad_variant_partial_bytes(l.d, variant) / (gbs * 1e6f);
        });
    };
    // BN backward, stand-alone form (reduce, finalize, apply): dy -> l.dconv (and dres)
    auto bn_bwd_std = [&](ConvLayer& l, const h16* dy, bool relu, h16* dres) -> int {
        return rn50_bn_bwd_launch((long long)l.d.n * l.P * l.Q, l.d.k, relu, dy, l.conv_out, l.bn_out,
                                  master_w + l.gamma_off, l.mean, l.invstd, l.dconv, dres, g16 + l.gamma_off,
                                  g16 + l.beta_off, c.bn_ws, s);
    };
    // BN backward when the data gradient that produced g already applied the ReLU mask and left the
    // per-tile sums (sum g, sum g*xhat) in c.bn_ws: finalize + apply only
    int fused_tiles = 0, proj_tiles = 0;    // row tiles of the sums waiting in c.bn_ws / c.bn_ws_side
    auto bn_bwd_fused = [&](ConvLayer& l, const h16* g) -> int {
        float* sums = c.bn_ws + (size_t)fused_tiles * 2 * l.d.k;
        return rn50_bn_bwd_from_partials_launch((long long)l.d.n * l.P * l.Q, l.d.k, g, l.conv_out,
                                                master_w + l.gamma_off, l.mean, l.invstd, l.dconv,
                                                g16 + l.gamma_off, g16 + l.beta_off, c.bn_ws, fused_tiles, sums, s);
    };
    // data gradient of conv l into l.din.  prev (nullable) = the layer whose BN+ReLU output `in` is l's input:
    // then the result is masked by in > 0 and the BN-backward sums of prev are formed in the epilogue.
    // `compact_addend`: addend holds only the (even, even) pixels (see ConvLayer::din_compact).
    // prev2 (nullable): a second BN that receives the same gradient (the projection shortcut of the block below);
    // its sums go to c.bn_ws_side, which only the forward pass uses otherwise.
    auto dgrad = [&](ConvLayer& l, const h16* addend, ConvLayer* prev, const h16* in, bool compact_addend = false,
                     ConvLayer* prev2 = nullptr) -> int {
        DgradBnFuse f = {in, prev ? prev->conv_out : nullptr, prev ? prev->mean : nullptr,
                         prev ? prev->invstd : nullptr, c.bn_ws};
        if (prev && prev2) { f.bn_x2 = prev2->conv_out; f.mean2 = prev2->mean; f.invstd2 = prev2->invstd; f.part2 = c.bn_ws_side; }
        // a strided 1x1 convolution only reaches the (even, even) input pixels: its data gradient is the
        // stride-1 data gradient on the output grid, stored compactly
        conv_desc d = l.d;
        if (l.din_compact) { d.h = l.P; d.w = l.Q; d.stride = 1; }
        return launch_or_tune(c, s, RN50_NUM_GATHER_TILES, &l.dgrad_tile, [&](int tile) {
            return rn50_conv_dgrad_launch(d, l.dconv, c.wt_all + l.wt_off, addend, l.din, s, prev ? &f : nullptr,
                                          prev ? &fused_tiles : nullptr, tile, compact_addend);
        }, "dgrad", l.name.c_str(), [&](int tile) {
            return (prev && d.stride == 1) ? finalize_penalty((long long)d.n * d.h * d.w, tile) : 0.f;
        }, RN50_TILE_STRICT);
    };

    const h16* dY = c.head_din;
    bool dY_fused = false;   // dY is already masked and conv3's BN sums are waiting in c.bn_ws
    for (int bi = (int)L.blocks.size() - 1; bi >= 0; --bi) {
        const Block& b = L.blocks[bi];
        ConvLayer &l1 = L.layers[b.c1], &l2 = L.layers[b.c2], &l3 = L.layers[b.c3];
        ConvLayer* below = bi > 0 ? &L.layers[L.blocks[bi - 1].c3] : nullptr;   // produced this block's input
        ConvLayer* below_proj = (bi > 0 && L.blocks[bi - 1].proj >= 0) ? &L.layers[L.blocks[bi - 1].proj] : nullptr;
        const bool need_in = cfg.has_stem || bi > 0;
        const h16* gres;                                              // masked gradient for the shortcut
        if (dY_fused) { RN50_TRY(bn_bwd_fused(l3, dY)); gres = dY; }
        else { RN50_TRY(bn_bwd_std(l3, dY, true, l3.dres)); gres = l3.dres; }
        RN50_TRY(fork_wgrad(l3, l2.bn_out, g16 + l3.w_off, nullptr));
        RN50_TRY(dgrad(l3, nullptr, &l2, l2.bn_out));
        RN50_TRY(bn_bwd_fused(l2, l3.din));
        RN50_TRY(fork_wgrad(l2, l1.bn_out, g16 + l2.w_off, nullptr));
        RN50_TRY(dgrad(l2, nullptr, &l1, l1.bn_out));
        RN50_TRY(bn_bwd_fused(l1, l2.din));
        RN50_TRY(fork_wgrad(l1, block_in[bi], g16 + l1.w_off, nullptr));
        if (b.proj >= 0) {
            ConvLayer& lp = L.layers[b.proj];
            if (dY_fused) {
                // the data gradient that produced gres also left this BN's sums (in c.bn_ws_side, same tile count)
                RN50_TRY(rn50_bn_bwd_from_partials_launch((long long)lp.d.n * lp.P * lp.Q, lp.d.k, gres, lp.conv_out,
                                                          master_w + lp.gamma_off, lp.mean, lp.invstd, lp.dconv,
                                                          g16 + lp.gamma_off, g16 + lp.beta_off, c.bn_ws_side,
                                                          proj_tiles, c.bn_ws_side + (size_t)proj_tiles * 2 * lp.d.k, s));
            } else {
                RN50_TRY(bn_bwd_std(lp, gres, false, nullptr));
            }
            RN50_TRY(fork_wgrad(lp, block_in[bi], g16 + lp.w_off, nullptr));
            if (need_in) {
                RN50_TRY(dgrad(lp, nullptr, nullptr, nullptr));
                RN50_TRY(dgrad(l1, lp.din, below, block_in[bi], lp.din_compact, below_proj));   // main path + projection shortcut
            }
        } else {
            RN50_TRY(dgrad(l1, gres, below, block_in[bi], false, below_proj));   // main path + identity shortcut
        }
        if (below_proj) proj_tiles = fused_tiles;
        dY = l1.din;
        dY_fused = below != nullptr;
    }
    if (cfg.has_stem) {
        ConvLayer& st = L.layers[0];
        RN50_TRY(rn50_maxpool_bwd(B, st.P, st.Q, st.d.k, dY, c.pool_arg, c.pool_din, s));
        RN50_TRY(rn50_bn_bwd_launch((long long)B * st.P * st.Q, st.d.k, true, c.pool_din, st.conv_out, st.bn_out,
                                    master_w + st.gamma_off, st.mean, st.invstd, st.dconv, nullptr, g16 + st.gamma_off,
                                    g16 + st.beta_off, c.bn_ws, s));
        RN50_TRY(fork_wgrad(st, c.stem_padded, nullptr, c.stem_wacc));
        RN50_TRY(rn50_stem_unpack_wgrad(st.d, c.stem_wacc, g16 + st.w_off, c.side));
    }
    {   // join: everything queued on the side stream precedes the update
        hipError_t e = hipEventRecord(c.join_event, c.side);
        if (e == hipSuccess) e = hipStreamWaitEvent(s, c.join_event, 0);
        if (e != hipSuccess) return rn50_hip_fail(e);
    }

    // ================= update (the flat FP16 gradient is complete) =================
    if (hp && hp->lars_eta > 0.f)
        return rn50_lars_launch(c.lars, g16, hp->grad_scale, master_w, momentum, static_cast<h16*>(w_lowp), hp->lr,
                                hp->momentum, hp->wd, hp->lars_eta, hp->lars_eps, nullptr, s);
    if (hp)
        return sgd_momentum_flat(L.param_count, g16, RN50_F16, hp->grad_scale, master_w, momentum, w_lowp, hp->lr, hp->momentum,
                                 hp->wd, stream);
    return RN50_OK;
}

extern "C" int rn50_autotune(rn50_ctx* ctx, const void* images, const int32_t* labels, float* master_w, void* w_lowp,
                             void* grad_lowp, float* loss_out, void* stream)
{
    RN50_REQUIRE_PTR(ctx);
    ctx->tune_report.clear();
    ctx->tuning = true;
    const int rc = rn50_step(ctx, images, labels, master_w, nullptr, w_lowp, grad_lowp, nullptr, loss_out, stream);
    ctx->tuning = false;
    if (rc != RN50_OK) return rc;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    return e == hipSuccess ? RN50_OK : rn50_hip_fail(e);
}

// Kernel variants in use, three numbers per convolution in network order: forward tile, data-gradient tile,
// filter-gradient variant (RN50_TILE_AUTO = the launcher's heuristic).
extern "C" int rn50_get_tuning(rn50_ctx* ctx, int* table, int capacity)
{
    RN50_REQUIRE_PTR(ctx);
    const int n = 3 * (int)ctx->L.layers.size();
    if (!table) return n;
    if (capacity < n) return RN50_ERR_SHAPE;
    for (size_t i = 0; i < ctx->L.layers.size(); ++i) {
        const ConvLayer& l = ctx->L.layers[i];
        table[3 * i] = l.fwd_tile; table[3 * i + 1] = l.dgrad_tile;
        table[3 * i + 2] = rn50_wgrad_canonical_variant(l.d, l.wgrad_variant);      // an autotuned pick may be an alias
    }
    return n;
}

extern "C" int rn50_set_tuning(rn50_ctx* ctx, const int* table, int n)
{
    RN50_REQUIRE_PTR(ctx); RN50_REQUIRE_PTR(table);
    if (n != 3 * (int)ctx->L.layers.size()) return RN50_ERR_SHAPE;
    for (int i = 0; i < n; ++i) {
        const int limit = (i % 3 == 2) ? RN50_NUM_WGRAD_VARIANTS : RN50_NUM_GATHER_TILES;
        if (table[i] < RN50_TILE_AUTO || table[i] >= limit) return RN50_ERR_SHAPE;
    }
    for (size_t i = 0; i < ctx->L.layers.size(); ++i) {
        ConvLayer& l = ctx->L.layers[i];
        l.fwd_tile = table[3 * i]; l.dgrad_tile = table[3 * i + 1];
        l.wgrad_variant = rn50_wgrad_canonical_variant(l.d, table[3 * i + 2]);     // the variant that will actually run
    }
    return RN50_OK;
}

// Text of what the last rn50_autotune on this context measured.  Copies at most cap-1 characters (NUL-terminated)
// and returns the full length.
extern "C" size_t rn50_tuning_report(rn50_ctx* ctx, char* buf, size_t cap)
{
    if (!ctx) return 0;
    if (buf && cap > 0) {
        const size_t n = ctx->tune_report.size() < cap - 1 ? ctx->tune_report.size() : cap - 1;
        memcpy(buf, ctx->tune_report.data(), n);
        buf[n] = 0;
    }
    return ctx->tune_report.size();
}
