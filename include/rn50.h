/*
 * rn50.h -- C ABI of the MI355X (gfx950) library that runs one GPU's share of a
 * synchronous data-parallel ResNet-50 SGD iteration: forward and backward over
 * the local mini-batch, label-smoothed softmax cross-entropy, and the
 * momentum-SGD update of the flat parameter buffer.
 *
 * Source of the problem statement: the paper's Sec. 2 (every GPU runs
 * forward/backward on its own mini-batch, gradients are averaged, weights are
 * updated), Sec. 2.1 (label smoothing), Sec. 3.2 (ResNet-50; FP16
 * forward/backward, FP32 optimizer arithmetic, batch normalisation from the
 * batch mean and batch squared mean in FP32 without moving averages;
 * per-worker mini-batch 16 or 32, Table 3).  The gradient all-reduce between
 * backward and update is not part of this library.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers owned by the caller, 16-byte
 *     aligned.  The library allocates no device memory.  Descriptor structs
 *     and out-parameters of the *_bytes / *_layout queries are HOST memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Every
 *     call only enqueues work on that stream and returns; nothing synchronises.
 *   - Return value: RN50_OK (0) or a negative rn50_status.  Arguments are
 *     validated before anything is launched; on error nothing is enqueued.
 *   - Layouts: activations NHWC, filters KRSC (out-channel, row, col,
 *     in-channel), all dense.  "half" below is IEEE binary16 (RN50_F16).
 *   - Workspaces: `ws` must hold at least the number of bytes the matching
 *     *_workspace_bytes query returns, else RN50_ERR_WORKSPACE.  Contents are
 *     scratch; two calls that overlap in time must not share a workspace.
 */
#ifndef RN50_H
#define RN50_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RN50_OK = 0,
    RN50_ERR_NULL = -1,      /* a required pointer is NULL */
    RN50_ERR_SHAPE = -2,     /* a size is non-positive or unsupported by the kernels */
    RN50_ERR_DTYPE = -3,     /* storage type not supported */
    RN50_ERR_WORKSPACE = -4, /* workspace missing or too small */
    RN50_ERR_ALIGN = -5,     /* a pointer is not 16-byte aligned */
    RN50_ERR_HIP = -6        /* a HIP runtime call failed (see rn50_last_hip_error) */
} rn50_status;

typedef enum { RN50_F16 = 0, RN50_BF16 = 1 } rn50_dtype; /* only RN50_F16 is implemented */

const char* rn50_status_string(int status);
int rn50_last_hip_error(void); /* hipError_t of the most recent RN50_ERR_HIP on this thread */

/* ------------------------------------------------------------------------------------------
 * Convolution (Sec. 3.2: the convolutions of ResNet-50, FP16 storage, FP32 accumulation).
 * x [n,h,w,c] half, w [k,r,s,c] half, y [n,p,q,k] half with p=(h+2*pad-r)/stride+1 (q alike).
 * Supported: c and k multiples of 64 with r=s in {1,3}, stride in {1,2}; and the stem
 * shape c=3, r=s=7, stride=2, pad=3 (k multiple of 64; no conv_dgrad for the stem).
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    int n, h, w, c; /* input  NHWC */
    int k, r, s;    /* filter KRSC */
    int stride, pad;
    int dt;         /* rn50_dtype */
} conv_desc;

enum { RN50_CONV_FWD = 0, RN50_CONV_DGRAD = 1, RN50_CONV_WGRAD = 2 };
/* The three stand-alone calls below choose among the library's kernel variants (tile shapes, pipeline depths,
 * split counts) by a shape heuristic; all variants compute the same result up to summation order.  The
 * *_variant forms (for tests and tuning) name one: 0 .. rn50_conv_variant_count(which)-1; a value that is out
 * of range or does not fit the shape leaves the heuristic in charge. */
size_t conv_workspace_bytes(const conv_desc* d, int which);
int rn50_conv_variant_count(int which);
/* 1 if variant is a kernel of its own for this convolution (which: 0 forward, 1 data gradient, 2 filter gradient),
 * 0 if the shape heuristic or a fallback would run in its place (or d is invalid).  Host only, launches nothing. */
int rn50_conv_variant_applies(const conv_desc* d, int which, int variant);

/* y[n,p,q,k] = sum_{r,s,c} x[n,p*stride+r-pad,q*stride+s-pad,c] * w[k,r,s,c]  (zero padding) */
int conv_fwd(const conv_desc* d, const void* x, const void* w, void* y,
             void* ws, size_t ws_bytes, void* stream);
/* dx[n,h,w,c] = sum over (k,r,s) with h+pad-r = p*stride, w+pad-s = q*stride of
 *               dy[n,p,q,k] * w[k,r,s,c].  Every element of dx is written. */
int conv_dgrad(const conv_desc* d, const void* dy, const void* w, void* dx,
               void* ws, size_t ws_bytes, void* stream);
int conv_fwd_variant(const conv_desc* d, const void* x, const void* w, void* y,
                     void* ws, size_t ws_bytes, int variant, void* stream);
int conv_dgrad_variant(const conv_desc* d, const void* dy, const void* w, void* dx,
                       void* ws, size_t ws_bytes, int variant, void* stream);
/* dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n,p*stride+r-pad,q*stride+s-pad,c], stored as
 * half.  FP32 partial sums of different pixel ranges are added in a fixed order, so the
 * result is deterministic. */
int conv_wgrad(const conv_desc* d, const void* x, const void* dy, void* dw,
               void* ws, size_t ws_bytes, void* stream);
int conv_wgrad_variant(const conv_desc* d, const void* x, const void* dy, void* dw,
                       void* ws, size_t ws_bytes, int variant, void* stream);

/* ------------------------------------------------------------------------------------------
 * Batch normalisation over m = N*H*W rows of c channels with batch statistics only
 * (Sec. 3.2, "Batch Normalization without Moving Average": batch mean and batch squared
 * mean in FP32 => biased variance), optional residual add, optional ReLU.
 *   mean_c = E[x], var_c = E[x^2]-mean^2 (clamped at 0), invstd = 1/sqrt(var+eps)
 *   y = gamma*(x-mean)*invstd + beta (+ residual);  y = max(y,0) if relu
 * c: a power of two from 8 to 2048, or a multiple of 2048 (a thread owns 8 channels and a 256-thread
 * workgroup covers whole rows or a whole number of 2048-channel passes); anything else: RN50_ERR_SHAPE.
 * x, y, residual, dy, dx, dresidual: half [m,c].
 * gamma, beta, save_mean, save_invstd: float [c].  dgamma, dbeta: half [c] (slices of
 * the flat FP16 gradient).
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    long long m;
    int c;
    float eps;
    int relu;         /* 0/1 */
    int has_residual; /* 0/1 */
    int dt;           /* rn50_dtype */
} bn_desc;

size_t bn_workspace_bytes(const bn_desc* d);
int bn_relu_fwd(const bn_desc* d, const void* x, const float* gamma, const float* beta,
                const void* residual /* NULL unless has_residual */, void* y,
                float* save_mean, float* save_invstd, void* ws, size_t ws_bytes, void* stream);
/* bn_relu_fwd for callers that cannot allocate or pass a workspace (code under HIP graph capture, serving
 * loops, harnesses that forbid hipMalloc): same arguments without ws, same kernels, same result bit for bit.
 * The partial sums live in a device array inside the library (RN50_BN_STATIC_MAX_C channels, 4.2 MB per GPU,
 * held until the process ends); c above that limit returns RN50_ERR_WORKSPACE.  The call allocates nothing.
 * All calls on one GPU share that array: calls that overlap in time on the same GPU race. */
#define RN50_BN_STATIC_MAX_C 256
int bn_relu_fwd_static(const bn_desc* d, const void* x, const float* gamma, const float* beta,
                       const void* residual /* NULL unless has_residual */, void* y,
                       float* save_mean, float* save_invstd, void* stream);
/* g = dy*[y>0] if relu else dy;  dresidual = g (written iff has_residual);
 * dbeta = sum g; dgamma = sum g*xhat; dx = gamma*invstd*(g - dbeta/m - xhat*dgamma/m). */
int bn_relu_bwd(const bn_desc* d, const void* dy, const void* x, const void* y /* NULL unless relu */,
                const float* gamma, const float* save_mean, const float* save_invstd,
                void* dx, void* dresidual /* NULL unless has_residual */, void* dgamma, void* dbeta,
                void* ws, size_t ws_bytes, void* stream);

/* The same two operators split at the points where GPUs exchange statistics (Sec. 3.2: batch mean and
 * batch squared mean are synchronised in FP32): every GPU computes its local moments / sums, the caller
 * combines them across GPUs (row-weighted average of the moments, sum of the backward sums), and every GPU
 * applies with the combined values.
 *   bn_batch_moments:          moments[0..c) = E[x], moments[c..2c) = E[x^2] over this GPU's m rows
 *   bn_relu_fwd_from_moments:  bn_relu_fwd with mean = moments[0..c), var = max(moments[c..2c) - mean^2, 0);
 *                              also writes save_mean / save_invstd for the backward pass
 *   bn_relu_bwd_sums:          sums[0..c) = sum g, sums[c..2c) = sum g*xhat over this GPU's rows (g as above)
 *   bn_relu_bwd_from_sums:     dx = gamma*invstd*(g - sums[0..c)/M - xhat*sums[c..2c)/M), M = total_rows over all
 *                              GPUs (>= m, else RN50_ERR_SHAPE); dresidual = g.  d gamma / d beta are the
 *                              combined sums themselves.
 * moments, sums: float [2c], device.  ws: bn_workspace_bytes(d). */
int bn_batch_moments(const bn_desc* d, const void* x, float* moments, void* ws, size_t ws_bytes, void* stream);
int bn_relu_fwd_from_moments(const bn_desc* d, const void* x, const float* gamma, const float* beta,
                             const void* residual /* NULL unless has_residual */, void* y, const float* moments,
                             float* save_mean, float* save_invstd, void* stream);
int bn_relu_bwd_sums(const bn_desc* d, const void* dy, const void* x, const void* y /* NULL unless relu */,
                     const float* save_mean, const float* save_invstd, float* sums, void* ws, size_t ws_bytes,
                     void* stream);
int bn_relu_bwd_from_sums(const bn_desc* d, const void* dy, const void* x, const void* y /* NULL unless relu */,
                          const float* gamma, const float* save_mean, const float* save_invstd, const float* sums,
                          long long total_rows, void* dx, void* dresidual /* NULL unless has_residual */, void* stream);

/* ------------------------------------------------------------------------------------------
 * Softmax cross-entropy with label smoothing (Sec. 2.1).  Target q = (1-eps)*onehot + eps/K.
 *   l_i = -sum_k q_k log softmax(logits_i)_k ; *loss_mean = mean_i l_i
 *   dlogits[i,k] = (softmax(logits_i)_k - q_k) * grad_scale   (half)
 * logits float [batch,classes]; labels int32 [batch], each in [0,classes) (not checked on
 * the device: out-of-range labels are treated as "no true class").  loss_per_sample
 * (float [batch]) may be NULL.  1 <= batch <= 65536, 2 <= classes <= 65536.
 * ---------------------------------------------------------------------------------------- */
int ls_xent_fwd_bwd(int batch, int classes, const float* logits, const int32_t* labels,
                    float eps, float grad_scale, float* loss_mean, float* loss_per_sample,
                    void* dlogits, int dlogits_dt, void* stream);

/* ------------------------------------------------------------------------------------------
 * Momentum SGD over the flat buffer (Sec. 3.2: FP32 optimizer arithmetic on FP16 gradients;
 * the paper's LARS scaling is not applied).  For every i < n, in FP32:
 *   g' = float(grad[i])*grad_scale + wd*w[i];  v[i] = mu*v[i] + g';  w[i] -= lr*v[i]
 *   w_lowp_out[i] = half(w[i])   (skipped if w_lowp_out is NULL)
 * master_w and momentum are updated in place.
 * ---------------------------------------------------------------------------------------- */
int sgd_momentum_flat(size_t n, const void* grad, int grad_dt, float grad_scale,
                      float* master_w, float* momentum, void* w_lowp_out,
                      float lr, float mu, float wd, void* stream);

/* ------------------------------------------------------------------------------------------
 * LARS with momentum over the flat buffer (Sec. 3.2, training configurations: the optimizer the
 * paper used, coefficient eta = 0.01, eps = 1e-6, computed in FP32 on the FP16 gradient).  The
 * paper prints no formula; the published layer-wise rule is used.  Per segment l (one layer
 * tensor), with g' = float(grad)*grad_scale and the 2-norms taken over the segment:
 *   rate_l = eta*||w_l|| / (||g'_l|| + wd*||w_l|| + eps)        (1 if either norm is zero)
 *   v = mu*v + lr*rate_l*(g' + wd*w);  w -= v;  w_lowp_out = half(w)
 * Segments with use_lars == 0 (BN scale / shift, biases) take  v = mu*v + lr*g';  w -= v.
 * Note that lr sits inside the momentum buffer here, unlike sgd_momentum_flat.
 *
 * A plan turns the segment table into device tables once; lars_plan_create copies them into
 * `workspace` (device memory, lars_workspace_bytes(...) bytes, 16-byte aligned, owned by the
 * caller and in use until lars_plan_destroy) with synchronous copies.  Segment offsets must be
 * multiples of 8 elements and segments must not overlap (RN50_ERR_SHAPE otherwise); elements
 * outside every segment are not touched.  lars_momentum_flat enqueues three kernels on `stream`
 * and allocates nothing; rates_out (nullable, device, one float per segment) receives rate_l.
 * Calls that share a plan must not overlap (they share its scratch).
 * ---------------------------------------------------------------------------------------- */
typedef struct { size_t offset, count; int use_lars; } rn50_lars_segment;
typedef struct lars_plan lars_plan; /* host object */
size_t lars_workspace_bytes(const rn50_lars_segment* segments, int nseg); /* 0 on a bad table */
int lars_plan_create(lars_plan** out, const rn50_lars_segment* segments /* host */, int nseg,
                     void* workspace, size_t workspace_bytes);
void lars_plan_destroy(lars_plan* plan);
int lars_momentum_flat(const lars_plan* plan, const void* grad, int grad_dt, float grad_scale,
                       float* master_w, float* momentum, void* w_lowp_out,
                       float lr, float mu, float wd, float eta, float eps, float* rates_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Training recipe, host-side pure functions (Sec. 3.2 "Training Configurations": the printed formulas of
 * configuration B, and Table 3).  epoch = processed samples / data-set size, a real number in [0, 90].
 *   LR(epoch)         = 0.2 + (29 - 0.2)*epoch/5            epoch < 5
 *                       29*(1 - epoch/90)^2                 epoch < 30
 *                       50*(1 - epoch/90)^2                 otherwise
 *   NoiseScale(epoch) = LR(epoch)*32*1024/(1 - 0.9)
 *   Momentum(epoch)   = 1 - LR(epoch)*B/NoiseScale(epoch),  B = total mini-batch size
 * rn50_sched_batch: per-worker and total mini-batch size of Table 3's experiments (0 = Reference, 1..4) at
 * `epoch`; RN50_ERR_SHAPE for an unknown experiment or an epoch outside [0, 90].  Configuration A is not
 * offered: the paper states only its warm-up (34 epochs from 1e-5 to 34.0) and refers elsewhere for the rest.
 * ---------------------------------------------------------------------------------------- */
double rn50_sched_lr_b(double epoch);
double rn50_sched_noise_scale_b(double epoch);
double rn50_sched_momentum_b(double epoch, double total_batch);
int rn50_sched_batch(int experiment, double epoch, int* per_worker, int* total);

/* ------------------------------------------------------------------------------------------
 * Whole iteration (Sec. 2 + Sec. 3.2) on a ResNet-50 v1.5 style network:
 *   [stem 7x7/2 conv 3->base_width, BN, ReLU, 3x3/2 max-pool]  (iff has_stem)
 *   num_stages stages of blocks[s] bottleneck blocks (1x1, 3x3, 1x1; widths w,w,4w with
 *   w = base_width<<s; stride 2 on the 3x3 of the first block of stages >= 1; 1x1
 *   projection shortcut + BN on the first block of every stage; ReLU after the add),
 *   global average pool, FC to `classes`, label-smoothed loss, backward, momentum SGD.
 * ResNet-50: has_stem=1, image 224x224, num_stages=4, blocks={3,4,6,3}, base_width=64,
 * classes=1000.  Without a stem the input is [batch,image_h,image_w,base_width] half and
 * receives no gradient.
 *
 * Flat parameter layout (used by master_w, momentum, w_lowp, grad_lowp alike), network
 * order: per conv its filter KRSC, then BN gamma, then BN beta; inside a block conv1,
 * conv2, conv3, projection; then FC weight [classes,C], then FC bias.  rn50_param_layout
 * walks it.  Forward uses w_lowp for filters and the FC weight, master_w for gamma,
 * beta and the FC bias.  On entry w_lowp must equal half(master_w) (rn50_cast_params).
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    int batch;
    int image_h, image_w;
    int has_stem;
    int num_stages;   /* 1..4 */
    int blocks[4];
    int base_width;   /* multiple of 64 */
    int classes;      /* multiple of 8 */
    int dt;           /* rn50_dtype */
    float bn_eps;
    float ls_eps;
    float loss_scale; /* dlogits = loss_scale*(p-q)/batch; the update multiplies by grad_scale */
    int keep_grads;   /* 0: activation gradients live in a few rotating buffers.  1: every one keeps its
                         own buffer (larger workspace) and rn50_tensor can return it; for checking. */
} rn50_config;

/* lars_eta == 0: momentum SGD as in sgd_momentum_flat.  lars_eta > 0: LARS as in lars_momentum_flat, with
 * layer-wise scaling on the convolution filters and the FC weight and plain momentum (no weight decay) on
 * BN scale / shift and the FC bias. */
typedef struct { float lr, momentum, wd, grad_scale, lars_eta, lars_eps; } rn50_hparams;

typedef struct rn50_ctx rn50_ctx; /* host object: descriptors + pointers into the workspace */

enum { RN50_KIND_CONV = 0, RN50_KIND_GAMMA = 1, RN50_KIND_BETA = 2, RN50_KIND_FCW = 3, RN50_KIND_FCB = 4 };

size_t rn50_param_count(const rn50_config* cfg); /* 25557032 for ResNet-50; 0 on a bad config */
int rn50_num_segments(const rn50_config* cfg);
/* idx-th segment of the flat layout: element offset, element count, RN50_KIND_*, fan-in
 * (c*r*s for filters, C for the FC weight, 0 otherwise). */
int rn50_param_layout(const rn50_config* cfg, int idx, size_t* offset, size_t* count, int* kind, int* fan_in);

size_t rn50_workspace_bytes(const rn50_config* cfg); /* activations, gradients, statistics, scratch */
/* Binds a context to a caller-owned device workspace (kept until rn50_destroy). */
int rn50_create(rn50_ctx** out, const rn50_config* cfg, void* workspace, size_t workspace_bytes);
void rn50_destroy(rn50_ctx* ctx);

/* w_lowp[i] = half(master_w[i]) for the whole flat buffer. */
int rn50_cast_params(size_t n, const float* master_w, void* w_lowp, int dt, void* stream);

/* One iteration.  images half [batch,image_h,image_w,3] (or [..,base_width] without stem),
 * labels int32 [batch].  master_w, momentum float [P] updated in place; w_lowp half [P]
 * read, then overwritten with half(new master_w); grad_lowp half [P] receives the
 * (loss_scale-scaled) flat gradient; loss_out: one float on the device.
 * If hp is NULL the update is skipped (forward, loss and backward only). */
int rn50_step(rn50_ctx* ctx, const void* images, const int32_t* labels,
              float* master_w, float* momentum, void* w_lowp, void* grad_lowp,
              const rn50_hparams* hp, float* loss_out, void* stream);

/* Optional: measures, for every convolution of the network and each of its three kernels, the kernel
 * variants the library has (tile shapes, pipeline depths, split counts) on the real tensors of one
 * forward+backward pass, and makes later rn50_step calls on this context use the fastest.  Arguments as
 * for rn50_step without the update.  Unlike every other call this one SYNCHRONISES (it times kernels
 * with HIP events) and must not run under stream capture.  Results of later steps stay within the
 * documented tolerances but may differ in the last bits from an untuned context (summation order). */
int rn50_autotune(rn50_ctx* ctx, const void* images, const int32_t* labels, float* master_w, void* w_lowp,
                  void* grad_lowp, float* loss_out, void* stream);

/* The variants in use on a context, three ints per convolution in network order (forward, data gradient, filter
 * gradient; -1 = shape heuristic), so that a tuning can be stored and a later context (another process, a
 * profiler run) executes exactly the same kernels.  rn50_get_tuning(ctx, NULL, 0) returns the table length; with
 * a table it fills it and returns the length (RN50_ERR_SHAPE if capacity is too small).  rn50_set_tuning checks
 * the length and every entry's range.  An entry whose variant does not apply to its convolution's shape is not an
 * error: the library runs the shape heuristic (forward, data gradient) or a fallback tile with the same pixel split
 * (filter gradient) instead, and rn50_get_tuning reports what actually runs (the filter-gradient entries at once,
 * the others after the first rn50_step).  paper_1811_05233_amd/tune_in_situ.py searches the table by the measured
 * time of the whole step; the table it found for full ResNet-50 at batch 32 ships beside it.  rn50_tuning_report copies the text of what the last rn50_autotune measured
 * (one line per launch site and candidate, microseconds) into buf (host, at most cap-1 characters, NUL-terminated)
 * and returns its full length. */
int rn50_get_tuning(rn50_ctx* ctx, int* table /* host */, int capacity);
int rn50_set_tuning(rn50_ctx* ctx, const int* table /* host */, int n);
size_t rn50_tuning_report(rn50_ctx* ctx, char* buf /* host */, size_t cap);

/* Device address of a tensor the last rn50_step left in the workspace, for parity checks.
 * name: "<conv>.conv" (conv output), "<conv>.out" (BN output), "<conv>.mean",
 * "<conv>.invstd", "pool.out", "feat", "logits", "dlogits"; with keep_grads also
 * "<conv>.dconv" (gradient w.r.t. the conv output), "<conv>.din" (w.r.t. its input; for conv1
 * it includes the shortcut's share; where the input is a ReLU output inside the network the
 * stored tensor is already multiplied by the ReLU mask [input > 0]),
 * "<conv3>.dres" (masked gradient given to the shortcut),
 * "head.din" (w.r.t. the last block's output), "pool.din" (w.r.t. the stem's BN output);
 * <conv> = "stem" or "s<stage>b<block>{c1,c2,c3,p}" (stage from 1).  *elems = element count,
 * *elem_bytes = 2 or 4.  Unknown name: RN50_ERR_SHAPE. */
int rn50_tensor(rn50_ctx* ctx, const char* name, void** ptr, size_t* elems, int* elem_bytes);

/* ------------------------------------------------------------------------------------------
 * Measurement aid (not part of the training path).  Between rn50_profile_begin and
 * rn50_profile_end every kernel launch of this library is bracketed by a pair of HIP events on
 * its stream.  rn50_profile_end synchronises the device and returns, per kernel, the number of
 * launches, the summed event-to-event time, and the summed ALGORITHMIC work of those launches:
 * flops = 2*M*N*K of the convolution as defined (live taps only), bytes = compulsory HBM
 * traffic (each operand read once, each result written once).  An event pair of a launch on a
 * context's second stream also contains the time the launch waited for compute units held by
 * the caller's stream.  Process-wide, not thread-safe.
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    const char* name;   /* kernel name as it appears in a rocprofv3 kernel trace (abbreviated) */
    long long launches;
    double total_ms;
    double flops;
    double bytes;
    long long side_launches;   /* how many of the launches ran on a context's second stream, next to the caller's chain */
} rn50_profile_entry;
int rn50_profile_begin(void);
int rn50_profile_end(rn50_profile_entry* out, int max_entries, int* n_out);

/* ------------------------------------------------------------------------------------------
 * Hardware probes (measurement aids, not part of the training path): the machine figures that
 * the tile shapes of the convolutions (Sec. 3.2: FP16 forward/backward) are weighed against.
 * All pointers are device pointers owned by the caller; every call only enqueues one kernel.
 *   rn50_probe_mfma: blocks workgroups of 4 wavefronts, each issuing 4*iters independent
 *     32x32x16 FP16 MFMAs from registers (flops = blocks*4*iters*4*32768); out: blocks*256 floats.
 *   rn50_probe_tile_load: workgroup b fetches iters consecutive tiles of 16 KB out of src, starting at
 *     tile (b * start_stride) mod (src_bytes / 16384) and wrapping (src_bytes a multiple of 16384, at most
 *     2 GiB - 16 KB; the working-set size and the stride decide whether the tiles come from L2, the Infinity
 *     Cache or HBM: start_stride = iters with blocks*iters tiles in src reads every tile exactly once),
 *     through_lds != 0: global -> LDS directly with three tiles in flight (out[b*256+t] = sum over the tiles of
 *     half t*8 of the tile), else with 16-byte vector loads into registers (out, read as unsigned: XOR of all
 *     32-bit words the thread loaded: words t*4..t*4+3 of each 4 KB quarter of each tile);
 *     bytes moved = blocks*iters*16384; out: blocks*256 elements.
 *   rn50_probe_copy: streaming copy of bytes (a multiple of 16) from src to dst.
 *   rn50_probe_empty: count kernels that do nothing, one after the other on the stream (cost of a
 *     dependent launch).
 * RN50_ERR_SHAPE for sizes outside the stated ranges (blocks 1..65536, iters >= 1).
 * ---------------------------------------------------------------------------------------- */
int rn50_probe_mfma(int blocks, int iters, float* out, void* stream);
int rn50_probe_tile_load(const void* src, size_t src_bytes, int blocks, int iters, int start_stride, int through_lds,
                         float* out, void* stream);
int rn50_probe_copy(const void* src, void* dst, size_t bytes, void* stream);
int rn50_probe_empty(int count, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RN50_H */
