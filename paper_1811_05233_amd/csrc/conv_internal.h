// Kernel argument blocks and internal launchers of the convolution kernels.
#pragma once
#include "common.h"

// Tile variants of the gather GEMM (rows x columns of the output tile, K-slab, ring stages) and of the
// filter gradient (tile x split target); RN50_TILE_AUTO lets the launcher's heuristic choose.
enum {
    RN50_TILE_AUTO = -1,
    RN50_TILE_128x128 = 0,     // 128x128, 32-wide slabs, 4 stages (needs output channels % 128 == 0)
    RN50_TILE_128x64,          // 128x64, 32-wide slabs, 4 stages
    RN50_TILE_64x64_DEEP,      // 64x64, 64-wide slabs, 4 stages, 2 workgroups per compute unit
    RN50_TILE_64x64_WIDE,      // 64x64, 64-wide slabs, 2 stages, 4 workgroups per compute unit
    RN50_TILE_64x64_K32,       // 64x64, 32-wide slabs, 4 stages, 4 workgroups per compute unit
    RN50_TILE_128x64_SHORT,    // 128x64, 32-wide slabs, 2 stages, 4 workgroups per compute unit (short reductions)
    RN50_TILE_128x128_SHORT,   // 128x128, 32-wide slabs, 2 stages, 3 workgroups per compute unit
    RN50_TILE_256x64,          // 256x64, 32-wide slabs, 3 stages
    RN50_TILE_128x64_K64,      // 128x64, 64-wide slabs, 3 stages
    RN50_TILE_64x64_K128,      // 64x64, 128-wide slabs, 2 stages (reduction length a multiple of 128)
    RN50_TILE_128x64_K128,     // 128x64, 128-wide slabs, 2 stages (reduction length a multiple of 128)
    RN50_TILE_64x64_K256,      // 64x64, 256-wide slabs, 2 stages (reduction length a multiple of 256)
    RN50_TILE_128x128_K64,     // 128x128, 64-wide slabs, 2 stages, 2 workgroups per compute unit
    RN50_TILE_256x64_K64,      // 256x64, 64-wide slabs, 2 stages
    RN50_TILE_256x128_K64,     // 256x128, 64-wide slabs, 2 stages, 1 workgroup per compute unit
    RN50_TILE_STRIP_256,       // 3x3 / stride 1 only: 256 pixels x 64 columns, one input strip per 32-channel slab for all 9 taps
    RN50_TILE_STRIP_128,       //   the same with 128 pixels
    RN50_TILE_STRIP_64,        //   the same with 64 pixels
    RN50_TILE_STRIP_256_S1,    //   single-stage forms of the three (smaller LDS footprint: 2-3 workgroups per compute unit
    RN50_TILE_STRIP_128_S1,    //   overlap each other's loads and MFMAs instead of a two-stage ring inside one)
    RN50_TILE_STRIP_64_S1,
    RN50_TILE_128x128_OCC4,    // 128x128, 32-wide slabs, 2 stages, 4 workgroups per compute unit (784 tiles fit one round of 1024)
    RN50_NUM_GATHER_TILES,
    RN50_TILE_STRICT = 0x1000,  // flag on a tile id: fail with RN50_ERR_SHAPE instead of falling back when it does not apply
    RN50_TILE_QUERY = 0x2000,   // flag on a tile id: launch nothing, only report RN50_OK / RN50_ERR_SHAPE (pointers may be null)
    RN50_WGRAD_TILE_STRIP = 10, // filter-gradient tile index of the 3x3 strip kernel (the ten before it: kWgradTiles)
    RN50_NUM_WGRAD_TILES = 11,
    RN50_NUM_WGRAD_VARIANTS = 3 * RN50_NUM_WGRAD_TILES      // tile x split target
};

struct GatherArgs {
    const h16* A;        // gathered NHWC tensor
    const h16* B;        // [NO][T][CR]
    h16* out;            // NHWC output, NO channels
    const h16* addend;   // nullable, same layout as out (or, with add_sub, the compact form below)
    int add_sub;         // 1: addend holds only out's even pixels, [NB][add_h][add_w][NO]; odd pixels add nothing
    int add_h, add_w;
    float* stats_part;   // nullable: per row tile, two per-channel sums of the stored output, [tile][2][NO]
    const h16* mask_y;   // nullable (data gradient): zero the output where this tensor (out's layout) is <= 0
    const h16* bn_x;     // nullable (data gradient): input of the BN that produced mask_y; switches the sums
    const float* bn_mean;    //   to sum g and sum g*xhat with xhat = (bn_x - mean) * invstd
    const float* bn_invstd;
    const h16* bn_x2;    // nullable: a second BN fed by the same gradient (a projection shortcut's): its input,
    const float* bn_mean2;   //   statistics, and the place of its sums [tile][2][NO] (sum g again, sum g*xhat2)
    const float* bn_invstd2;
    float* stats_part2;
    int NB;              // images
    int IH, IW;          // spatial size of A
    int lda;             // halfs between adjacent pixels of A
    int CR;              // reduction length per tap
    int T;               // taps in B's layout
    int NO;              // output channels
    int OH, OW;          // spatial size of out
    int a_mul, a_off;    // A coordinate = sub-grid coordinate * a_mul + a_off + tap offset
    int o_mul;           // out coordinate = sub-grid coordinate * o_mul + class offset
    int ncls;            // 1, or stride^2 parity classes for the strided data gradient
    int cOHs[4], cOWs[4];
    int oph[4], opw[4];
    int mt_end[4];       // running end of each class's row tiles (filled by the launcher)
    int ntaps[4];
    float inv_oh[4], inv_ow[4];   // reciprocals of cOHs / cOWs (filled by the launcher)
    unsigned a_bytes, b_bytes;    // sizes of A and B in bytes (buffer range checks)
    int tap[4][9];       // per class and live tap: dh | dw << 8 (signed bytes, A-pixel offset) | filter tap << 16
    int xcd_split_cols;  // 1: an XCD owns a range of column tiles (all row tiles); 0: a range of row tiles.  Set by the launcher
};

struct WgradArgs {
    const h16* x;
    const h16* dy;
    float* out;          // [nsplit][K][NG*G] FP32 partial tiles (or the final tile when there is one split)
    int K;               // output channels (row length of dy)
    int C;               // input channels (row length of x; 4 for the padded stem image)
    int H, W;            // spatial size of x (padded size for the stem)
    int P, Q;            // spatial size of dy
    int R, S, stride, pad;
    int NG;              // granules per output row
    int direct;          // 1x1 stride 1: x pixel index == dy pixel index
    int npix;            // N*P*Q
    int pix_per_split;
    float inv_p, inv_q;
    unsigned x_bytes, dy_bytes;
    size_t split_stride; // floats between consecutive splits' tiles
};

bool rn50_conv_is_stem(const conv_desc& d);
int rn50_gather_tile_rows(int tile);
int rn50_conv_validate(const conv_desc* d);
size_t rn50_stem_padded_bytes(const conv_desc& d);
size_t rn50_stem_packed_filter_bytes(const conv_desc& d);
int rn50_stem_pad_image(const conv_desc& d, const h16* img, h16* padded, hipStream_t s);
int rn50_stem_pack_filter(const conv_desc& d, const h16* w, h16* packed, hipStream_t s);
int rn50_transpose_filter(const conv_desc& d, const h16* w, h16* wt, hipStream_t s);
int rn50_fill_zero(float* p, size_t n, hipStream_t s);
int rn50_cast_f32_to_h16(const float* src, h16* dst, size_t n, hipStream_t s);
// stats_part (nullable): receives per-row-tile BatchNorm partial sums; *stats_tiles = number of row tiles
int rn50_conv_fwd_launch(const conv_desc& d, const h16* x, const h16* w, h16* y, hipStream_t s, float* stats_part,
                         int* stats_tiles, int tile);
size_t rn50_conv_stats_floats(const conv_desc& d);
// Optional fusion of the ReLU mask and the BN-backward reductions of the layer that produced this
// convolution's input into the data gradient's epilogue.
struct DgradBnFuse {
    const h16* mask_y;     // the convolution's own input (a ReLU output)
    const h16* bn_x;       // conv output the BN normalised to produce mask_y
    const float* mean;
    const float* invstd;
    float* part;           // [row tile][sum g | sum g*xhat][channels], rn50_dgrad_stats_floats(d) floats
    // optional second BN that receives the same (masked) gradient, e.g. the projection shortcut's: its sums go to
    // part2, same layout and size
    const h16* bn_x2 = nullptr;
    const float* mean2 = nullptr;
    const float* invstd2 = nullptr;
    float* part2 = nullptr;
};
// addend (nullable) has dx's layout, or with addend_even_only its (even row, even column) pixels only,
// [n][ceil(h/2)][ceil(w/2)][c] (the data gradient of a strided 1x1 convolution is zero elsewhere).
int rn50_conv_dgrad_launch(const conv_desc& d, const h16* dy, const h16* wt, const h16* addend, h16* dx, hipStream_t s,
                           const DgradBnFuse* fuse, int* tiles_out, int tile, bool addend_even_only = false);
size_t rn50_dgrad_stats_floats(const conv_desc& d);
size_t rn50_wgrad_acc_floats(const conv_desc& d);
size_t rn50_wgrad_partial_floats(const conv_desc& d);
size_t rn50_wgrad_variant_partial_bytes(const conv_desc& d, int variant);
int rn50_wgrad_canonical_variant(const conv_desc& d, int variant);
// sum of the per-split partial tiles -> out16 (half) or out32 (FP32); exactly one of the two is given
int rn50_conv_wgrad_launch(const conv_desc& d, const h16* x, const h16* dy, h16* out16, float* out32, float* partials,
                           hipStream_t s, int variant);
int rn50_stem_unpack_wgrad(const conv_desc& d, const float* acc, h16* out, hipStream_t s);
