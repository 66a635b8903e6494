// Internal launchers: pooling, FC, batch norm (used by the whole-step driver).
#pragma once
#include "common.h"

int rn50_maxpool_fwd(int N, int H, int W, int C, const h16* x, h16* y, uint8_t* arg, hipStream_t s);
int rn50_maxpool_bwd(int N, int H, int W, int C, const h16* dy, const uint8_t* arg, h16* dx, hipStream_t s);
int rn50_avgpool_fwd(int N, int HW, int C, const h16* x, h16* y, hipStream_t s);
int rn50_fc_fwd(int B, int Cin, int Cout, const h16* a, const h16* Wt, const float* bias, float* z, hipStream_t s);
// dWt, db: half (slices of the flat FP16 gradient)
int rn50_fc_bwd(int B, int Cin, int Cout, int HW, const h16* a, const h16* Wt, const h16* dz, h16* dWt, h16* db,
                h16* dx, hipStream_t s_weights, hipStream_t s);

int rn50_bn_fwd_launch(long long m, int c, float eps, bool relu, const h16* x, const float* gamma, const float* beta,
                       const h16* res, h16* y, float* save_mean, float* save_invstd, float* ws, hipStream_t s);
// dgamma / dbeta: half (slices of the flat FP16 gradient)
int rn50_bn_bwd_launch(long long m, int c, bool relu, const h16* dy, const h16* x, const h16* y, const float* gamma,
                       const float* save_mean, const float* save_invstd, h16* dx, h16* dres,
                       h16* dgamma, h16* dbeta, float* ws, hipStream_t s);
size_t rn50_bn_ws_floats(int c);
// most row tiles of partial sums that the from_partials launchers combine inside the apply kernel; beyond this
// they run a separate finalize kernel first
int rn50_bn_fused_max_tiles();
int rn50_bn_fwd_from_partials_launch(long long m, int c, float eps, bool relu, const h16* x, const float* gamma,
                                     const float* beta, const h16* res, h16* y, float* save_mean, float* save_invstd,
                                     const float* part, int ntiles, hipStream_t s);
int rn50_bn_bwd_from_partials_launch(long long m, int c, const h16* g, const h16* x, const float* gamma,
                                     const float* save_mean, const float* save_invstd, h16* dx,
                                     h16* dgamma, h16* dbeta, const float* part, int ntiles, float* sums,
                                     hipStream_t s);
struct lars_plan;
int rn50_lars_launch(const lars_plan* p, const h16* grad, float grad_scale, float* w, float* v, h16* w16, float lr, float mu,
                     float wd, float eta, float eps, float* rates_out, hipStream_t s);
