// Convolution forward / data-gradient / filter-gradient as implicit GEMM on the gfx950 matrix
// cores (v_mfma_f32_32x32x16_f16: FP16 operands, FP32 accumulation), LDS-staged NHWC tiles.
//
// Forward and data-gradient share one "gather GEMM":
//     out[m, j] = sum_{tap} sum_{c < CR} A[pixel(m, tap), c] * B[j, tap, c]
// where m enumerates output pixels, A is an NHWC tensor whose pixel rows are gathered with zero
// fill outside the image, and B is [NO][T][CR] (reduction index contiguous).
//   forward:        A = x,  B = w (KRSC as given),        pixel = (n, p*stride - pad + r, q*stride - pad + s)
//   data-gradient:  A = dy, B = w transposed to CRSK,     pixel = (n, (h + pad - r)/stride, (w + pad - s)/stride)
// For stride 2 the data-gradient rows are split into the four (h%2, w%2) parity classes; each
// class only visits the filter taps that can reach it, so no multiply hits an inserted zero.
//
// The filter gradient reduces over pixels, which is the strided dimension of both operands: its
// tiles go to LDS as they lie in memory and the MFMA operands are read with the transposing LDS
// read (ds_read_b64_tr_b16).  The pixel range is split over workgroups; their partial tiles are
// added in a fixed order.
//
// Every kernel exists in several variants (tile shape, K-slab depth, ring stages, residency);
// the whole-step driver times them per layer, the stand-alone entry points use a shape heuristic.
#include "common.h"
#include "conv_internal.h"
#include "prof.h"

namespace {

constexpr int kThreads = 256;

// LDS tile of ROWS rows x KW halfs (KW = 32, 64, 128 or 256), addressed in 16-byte chunks.  A ds_read_b128 is served
// 16 lanes at a time (16 lanes x 16 bytes = the 64 banks), and the 16 lanes of such a group read 16 consecutive rows
// at one chunk index; the chunk index is therefore XOR-ed with a function of the row that gives those 16 rows 16
// different 16-byte slots of the 256-byte bank space:
//   KW = 32  (64-byte rows, four rows per bank space): rows r, r+4, r+8, r+12 share a quarter -> chunk ^ ((r >> 2) & 3)
//   KW = 64  (128-byte rows, two per bank space):       even / odd rows share a half           -> chunk ^ ((r ^ (r >> 3)) & 7)
//   KW >= 128 (every row spans the whole bank space):                                           -> chunk ^ (r & 15)
// (the first holds for any 16 consecutive rows, which the strip kernel's shifted reads need).
template <int KW>
__device__ __forceinline__ int lds_swz(int row) {
    if (KW == 32) return (row >> 2) & 3;
    if (KW == 64) return (row ^ (row >> 3)) & 7;
    return row & 15;
}
template <int KW>
__device__ __forceinline__ int lds_off(int row, int chunk) {
    if (KW == 32) {
        // two rows share a 128-byte line
        const int line = row >> 1;
        const int slot = ((row & 1) << 2) | ((chunk ^ lds_swz<32>(row)) & 3);
        return line * 64 + slot * 8;
    }
    return row * KW + (chunk ^ lds_swz<KW>(row)) * 8;   // XOR touches only the low bits of the chunk index
}

// ------------------------------------------------------------------------------------------------
// gather GEMM (forward, data-gradient)
// ------------------------------------------------------------------------------------------------
// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14])
#define RN50_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xf) | 0x0f70 | (((n) >> 4) << 14))
#define RN50_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xc07f)

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// m = q*d + r with 0 <= r < d, for 0 <= m < 2^24, using the precomputed float reciprocal of d.
__device__ __forceinline__ void fast_divmod(int m, int d, float inv_d, int& q, int& r) {
    q = (int)((float)m * inv_d);
    r = m - q * d;
    const int fix = (r >= d ? 1 : 0) - (r < 0 ? 1 : 0);     // the float quotient is off by at most one; no branches
    q += fix;
    r -= fix * d;
}

// Accumulator start: zero, or the addend at the tile's output positions (out = addend + A*B, rounded once).
// row_pix(row, n, oh, ow) -> bool maps a tile row to its output pixel (false: the row is outside the tensor).
template <int BN, int TM, int TN, class RowPix>
__device__ __forceinline__ void gather_init_acc(const GatherArgs& a, f32x16 (&acc)[TM][TN], int wm0, int wn0, int li, int lg,
                                                int nt, RowPix row_pix)
{
    if (a.addend) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            int n, oh, ow;
            bool ok = row_pix(wm0 + tm * 32 + li, n, oh, ow);
            size_t opix = 0;
            if (ok) {
                if (a.add_sub) {
                    ok = ((oh | ow) & 1) == 0;
                    opix = ((size_t)n * a.add_h + (oh >> 1)) * a.add_w + (ow >> 1);
                } else {
                    opix = ((size_t)n * a.OH + oh) * a.OW + ow;
                }
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    h16x4 v = {0, 0, 0, 0};
                    if (ok) v = *reinterpret_cast<const h16x4*>(a.addend + opix * a.NO + nt * BN + wn0 + tn * 32 + q * 8 + lg * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[tm][tn][q * 4 + e] = (float)v[e];
                }
        }
    } else {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;
    }
}

// The extra operands of the data gradient's epilogue for one chunk of a thread's rows: ReLU mask source and BN inputs.
template <int CH>
struct EpiOperands {
    size_t gidx[CH];
    bool ok[CH];
    h16x8 yv[CH], xv[CH], xw[CH];
};
template <int BM, int BN>
struct EpiShape {
    static constexpr int OCPR = BN / 8;                 // output chunks per row
    static constexpr int ORPP = kThreads / OCPR;        // rows covered by one pass of the workgroup
    static constexpr int NR = BM / ORPP;                // rows per thread
    static constexpr int CH = NR < 2 ? NR : 2;          // rows whose extra operands are requested together
    static constexpr int NC = NR / CH;
    static_assert(NR % CH == 0, "rows per thread must split into whole chunks");
};
// Requests chunk c of this thread's rows.  A row past the end of the tensor reads element 0 (never used).
template <int BM, int BN, class RowPix>
__device__ __forceinline__ void gather_epi_request(const GatherArgs& a, EpiOperands<EpiShape<BM, BN>::CH>& o, int c, int tid,
                                                   int nt, RowPix row_pix)
{
    using S = EpiShape<BM, BN>;
    const int oc = tid % S::OCPR, orl = tid / S::OCPR;
#pragma unroll
    for (int i = 0; i < S::CH; ++i) {
        int n, oh, ow;
        o.ok[i] = row_pix(orl + (c * S::CH + i) * S::ORPP, n, oh, ow);
        o.gidx[i] = o.ok[i] ? (((size_t)n * a.OH + oh) * a.OW + ow) * a.NO + nt * BN + oc * 8 : 0;
    }
    if (a.mask_y) {
#pragma unroll
        for (int i = 0; i < S::CH; ++i) o.yv[i] = *reinterpret_cast<const h16x8*>(a.mask_y + o.gidx[i]);
    }
    if (a.bn_x) {
#pragma unroll
        for (int i = 0; i < S::CH; ++i) o.xv[i] = *reinterpret_cast<const h16x8*>(a.bn_x + o.gidx[i]);
        if (a.bn_x2) {
#pragma unroll
            for (int i = 0; i < S::CH; ++i) o.xw[i] = *reinterpret_cast<const h16x8*>(a.bn_x2 + o.gidx[i]);
        }
    }
}

// Epilogue: FP32 -> half, through LDS so that global stores are full 16-byte rows, plus the optional per-channel
// sums over the tile's rows.  Forward: sum and sum of squares of the stored halves (BN statistics of the layer that
// follows).  Data gradient with bn_x set: the stored gradient g is first masked by the ReLU of the tensor it belongs
// to (mask_y), then sum g and sum g*xhat are formed for the backward pass of the BN that produced that tensor.
// The caller has made sure that no wave still reads the part of LDS used here.  tile_row: index of the row tile
// (first index of the partial sums).
// first: the operands of the thread's first chunk of rows, requested by the caller at the start of the kernel (they
// arrive with the first K-slab); later chunks are requested here, one chunk ahead of their use.
// kAlias: the statistics scratch takes the place of the staged tile (one more barrier, less LDS) instead of lying
// behind it.
template <int BM, int BN, int TM, int TN, int LDS_HALFS, bool kAlias, class RowPix>
__device__ __forceinline__ void gather_epilogue(const GatherArgs& a, h16* lds, f32x16 (&acc)[TM][TN], int wm0, int wn0, int li,
                                                int lg, int tid, int nt, int tile_row, RowPix row_pix,
                                                EpiOperands<EpiShape<BM, BN>::CH>& first)
{
    using S = EpiShape<BM, BN>;
    constexpr int EP = BN + 8;                   // row pitch of the staged tile in halfs
    constexpr int ORPP = S::ORPP, CH = S::CH, NC = S::NC;
    const int oc = tid % S::OCPR, orl = tid / S::OCPR;
    const bool bwd_stats = a.bn_x != nullptr;
    const bool second = bwd_stats && a.bn_x2 != nullptr;
    const bool masked = a.mask_y != nullptr;
    EpiOperands<CH> other;
    if (NC > 1) gather_epi_request<BM, BN>(a, other, 1, tid, nt, row_pix);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                h16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (h16)acc[tm][tn][q * 4 + e];
                *reinterpret_cast<h16x4*>(lds + (wm0 + tm * 32 + li) * EP + wn0 + tn * 32 + q * 8 + lg * 4) = v;
            }
    __syncthreads();
    // Backward sums are taken as sum g and sum g*x over the tile; xhat = (x - mean) * invstd is linear in x, so the
    // tile's sum g*xhat = invstd * (sum g*x - mean * sum g) is formed once per column below.
    float st[16], st2[8];
#pragma unroll
    for (int j = 0; j < 16; ++j) st[j] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) st2[j] = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        EpiOperands<CH>& cur = (c & 1) ? other : first;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            if (!cur.ok[i]) continue;            // a row past the end of the tensor
            const int row = orl + (c * CH + i) * ORPP;
            h16x8 v = *reinterpret_cast<const h16x8*>(lds + row * EP + oc * 8);
            if (masked) {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = (float)cur.yv[i][j] > 0.f ? v[j] : (h16)0.f;
            }
            *reinterpret_cast<h16x8*>(a.out + cur.gidx[i]) = v;
            if (bwd_stats) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float g = (float)v[j];
                    st[j] += g;
                    st[8 + j] += g * (float)cur.xv[i][j];
                }
                if (second) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) st2[j] += (float)v[j] * (float)cur.xw[i][j];
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) { const float f = (float)v[j]; st[j] += f; st[8 + j] += f * f; }
            }
        }
        if (c + 2 < NC) gather_epi_request<BM, BN>(a, cur, c + 2, tid, nt, row_pix);     // two chunks stay in flight
    }
    if (a.stats_part) {
        // per-channel sums of this row tile, added in a fixed order: [tile][first | second sum][channel].  The
        // scratch (ORPP x 2 x BN floats) lies behind the staged tile, or takes its place once every thread has
        // read its rows.
        float* red = reinterpret_cast<float*>(kAlias ? lds : lds + BM * EP);
        constexpr int RP = 2 * BN;          // (an odd pitch would spread the scalar writes over the banks; measured slower)
        static_assert((kAlias ? 0 : BM * EP * 2) + ORPP * RP * 4 <= LDS_HALFS * 2, "statistics scratch must fit in LDS");
        if (kAlias) __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            red[orl * RP + oc * 8 + j] = st[j];
            red[orl * RP + BN + oc * 8 + j] = st[8 + j];
        }
        __syncthreads();
        float sum_g = 0.f;                  // kept by the threads of the second half for the second BN
        if (tid < 2 * BN) {
            const int which = tid / BN, col = tid % BN;
            float sum = 0.f;
            for (int r = 0; r < ORPP; ++r) sum += red[r * RP + which * BN + col];
            if (bwd_stats) {
                for (int r = 0; r < ORPP; ++r) sum_g += red[r * RP + col];
                if (which == 1) sum = a.bn_invstd[nt * BN + col] * (sum - a.bn_mean[nt * BN + col] * sum_g);
            }
            a.stats_part[((size_t)tile_row * 2 + which) * a.NO + nt * BN + col] = sum;
            if (second && which == 0) a.stats_part2[((size_t)tile_row * 2) * a.NO + nt * BN + col] = sum;
        }
        if (second) {                       // the second BN's sum g*xhat2, through the same scratch
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) red[orl * RP + oc * 8 + j] = st2[j];
            __syncthreads();
            if (tid >= BN && tid < 2 * BN) {
                const int col = tid - BN;
                float sum = 0.f;
                for (int r = 0; r < ORPP; ++r) sum += red[r * RP + col];
                a.stats_part2[((size_t)tile_row * 2 + 1) * a.NO + nt * BN + col] =
                    a.bn_invstd2[nt * BN + col] * (sum - a.bn_mean2[nt * BN + col] * sum_g);
            }
        }
    }
}

// K-slabs travel global memory -> LDS directly (buffer_load ... lds, 16 bytes per lane, no staging
// registers) into a ring of NST stages, so that NST-1 slabs are in flight while one is consumed.
// Rows outside the image (zero padding, ragged last tile) use an out-of-range buffer offset, which
// the hardware turns into zeros.  One workgroup barrier per K-slab.
template <int BM, int BN, int BK, int NST, int OCC>
__global__ __launch_bounds__(kThreads, OCC) void gather_gemm_kernel(const GatherArgs a)
{
    constexpr int WR = 2, WC = 2;
    constexpr int CPR = BK / 8;            // 16-byte chunks per tile row
    constexpr int RPI = 64 / CPR;          // tile rows written by one wave-wide load (1 KB of LDS)
    constexpr int NA = BM / RPI / 4, NB = BN / RPI / 4;   // loads per thread and K-slab
    constexpr int NL = NA + NB;
    constexpr int WM = BM / WR, WN = BN / WC, TM = WM / 32, TN = WN / 32;
    constexpr int KS = BK / 16;
    constexpr int STAGE = (BM + BN) * BK;
    constexpr int EP = BN + 8;             // epilogue row pitch in halfs (see gather_epilogue)
    constexpr int EPI_STATS = (kThreads / (BN / 8)) * 2 * BN * 2;            // statistics scratch (floats) in halfs
    constexpr bool kAliasStats = BN == 128 && OCC == 4;                      // the variant that needs 4 x its LDS per unit
    constexpr int EPI_HALFS = kAliasStats ? (BM * EP > EPI_STATS ? BM * EP : EPI_STATS) : BM * EP + EPI_STATS;
    constexpr int LDS_HALFS = (NST * STAGE > EPI_HALFS) ? NST * STAGE : EPI_HALFS;
    constexpr unsigned kOutOfRange = 0x80000000u;
    __shared__ __attribute__((aligned(16))) h16 lds[LDS_HALFS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index as a scalar
    const int li = lane & 31, lg = lane >> 5;
    const int wm0 = (wave / WC) * WM, wn0 = (wave % WC) * WN;

    // ---- which tile ----
    // Workgroups are dealt round-robin to the 8 XCDs.  Normally every XCD takes a contiguous range of row tiles
    // with all their column tiles (its L2 then holds that range's A rows and all of B); when B is the larger
    // operand every XCD takes one eighth of the column tiles with all row tiles instead.
    const int n_tiles = a.NO / BN;
    int nt, mt;
    if (a.xcd_split_cols) {
        const int per = n_tiles >> 3, p = blockIdx.x >> 3;
        nt = (blockIdx.x & 7) * per + p % per;
        mt = p / per;
    } else {
        const int bid = rn50_xcd_remap(blockIdx.x, gridDim.x);
        nt = bid % n_tiles;
        mt = bid / n_tiles;
    }
    const int tile_row = mt;
    int cls = 0;
    while (cls < a.ncls - 1 && mt >= a.mt_end[cls]) ++cls;
    if (cls > 0) mt -= a.mt_end[cls - 1];
    const int OHs = a.cOHs[cls], OWs = a.cOWs[cls];
    const float inv_oh = a.inv_oh[cls], inv_ow = a.inv_ow[cls];
    const int M = a.NB * OHs * OWs;
    const int ntaps = a.ntaps[cls];
    const int IH = a.IH, IW = a.IW, lda = a.lda, CR = a.CR;

    // ---- this lane's place in a wave-wide load: row inside the group of RPI rows, logical chunk ----
    int row_in_grp, phys;
    if (BK >= 64) { row_in_grp = lane / CPR; phys = lane % CPR; }
    else { row_in_grp = 2 * (lane >> 3) + ((lane & 7) >> 2); phys = lane & 3; }
    auto logical_chunk = [&](int row) { return phys ^ lds_swz<BK>(row); };

    int a_h0[NA], a_w0[NA];
    unsigned a_voff[NA], b_voff[NB];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int row = (wave + 4 * j) * RPI + row_in_grp;
        const int m = mt * BM + row;
        if (m < M) {
            int t, wq, n, hq;
            fast_divmod(m, OWs, inv_ow, t, wq);
            fast_divmod(t, OHs, inv_oh, n, hq);
            a_h0[j] = hq * a.a_mul + a.a_off;
            a_w0[j] = wq * a.a_mul + a.a_off;
            a_voff[j] = (unsigned)(((n * IH + a_h0[j]) * IW + a_w0[j]) * lda) * 2u + logical_chunk(row) * 16;
        } else {
            a_h0[j] = -(1 << 20); a_w0[j] = 0; a_voff[j] = 0;
        }
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int row = (wave + 4 * j) * RPI + row_in_grp;
        b_voff[j] = (unsigned)((nt * BN + row) * a.T * CR) * 2u + logical_chunk(row) * 16;
    }
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(a.A), 0, a.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(a.B), 0, a.b_bytes, 0x00020000);

    const int KC = CR / BK;
    const int kiters = ntaps * KC;
    int ld_ti = 0, ld_cc = 0, ld_stage = 0;      // next slab to load: tap, channel slab, ring stage (wave-uniform)
    // The tap table lives in the kernel-argument segment.  The entry of the tap being loaded is held in a register
    // and replaced when the tap changes, so that no slab waits on a scalar memory read.
    int ld_tap = a.tap[cls][0];                  // packed: dh | dw << 8 | filter tap << 16

    auto issue_slab = [&]() {
        const int tap = ld_tap;
        const int dh = (int)(signed char)(tap & 0xff), dw = (int)(signed char)((tap >> 8) & 0xff), bt = tap >> 16;
        const int a_delta = ((dh * IW + dw) * lda + ld_cc * BK) * 2;          // bytes, wave-uniform
        const unsigned b_delta = (unsigned)(bt * CR + ld_cc * BK) * 2u;
        h16* sa = lds + ld_stage * STAGE;
        h16* sb = sa + BM * BK;
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const int ih = a_h0[j] + dh, iw = a_w0[j] + dw;
            const bool ok = (unsigned)ih < (unsigned)IH && (unsigned)iw < (unsigned)IW;
            const unsigned voff = ok ? a_voff[j] + (unsigned)a_delta : kOutOfRange;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)(sa + (wave + 4 * j) * 512), 16, (int)voff, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < NB; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)(sb + (wave + 4 * j) * 512), 16,
                                                     (int)(b_voff[j] + b_delta), 0, 0, 0);
        if (++ld_cc == KC) { ld_cc = 0; ++ld_ti; ld_tap = a.tap[cls][ld_ti < ntaps ? ld_ti : 0]; }
        if (++ld_stage == NST) ld_stage = 0;
    };

    // start the ring before touching anything else
#pragma unroll
    for (int p = 0; p < NST - 1; ++p)
        if (p < kiters) issue_slab();

    // tile row -> output pixel
    auto row_pix = [&](int row, int& n, int& oh, int& ow) -> bool {
        const int m = mt * BM + row;
        if (m >= M) return false;
        int t, wq, hq;
        fast_divmod(m, OWs, inv_ow, t, wq);
        fast_divmod(t, OHs, inv_oh, n, hq);
        oh = hq * a.o_mul + a.oph[cls];
        ow = wq * a.o_mul + a.opw[cls];
        return true;
    };
    f32x16 acc[TM][TN];
    gather_init_acc<BN>(a, acc, wm0, wn0, li, lg, nt, row_pix);
    // The epilogue's extra operands for the thread's first rows are requested here, so that they arrive together
    // with the first K-slab -- except in the variants whose occupancy leaves no registers for it.
    constexpr bool kEarlyEpi = !(BM == 64 && BN == 64 && BK == 64 && OCC == 4) && !(BN == 128 && OCC == 4);
    EpiOperands<EpiShape<BM, BN>::CH> epi_first;
    if (kEarlyEpi) gather_epi_request<BM, BN>(a, epi_first, 0, tid, nt, row_pix);

    int cur = 0;
    for (int kit = 0; kit < kiters; ++kit) {
        // slab `kit` has landed once at most the NST-2 younger slabs are outstanding
        if (kit + NST - 2 < kiters) RN50_WAIT_VMCNT(NL * (NST - 2));
        else RN50_WAIT_VMCNT(0);
        RN50_WAIT_LGKMCNT0();                 // this wave's LDS reads of the previous slab are done
        __builtin_amdgcn_s_barrier();         // everyone's part of slab kit is in LDS; stage (kit-1)%NST is free
        if (kit + NST - 1 < kiters) issue_slab();
        const h16* sa = lds + cur * STAGE;
        const h16* sb = sa + BM * BK;
        // Operand reads run one group of k-steps (at least four MFMAs' worth) ahead of the MFMAs that use them, in
        // two register sets, so that a wave keeps its matrix unit busy while its next LDS reads are in flight.
        constexpr int GE = (TM * TN >= 4 || KS == 1) ? 1 : ((TM * TN == 2 || KS == 2) ? 2 : 4);
        constexpr int NG = KS / GE;
        h16x8 fa[2][GE][TM], fb[2][GE][TN];
        auto read_group = [&](int g, int buf) {
#pragma unroll
            for (int e = 0; e < GE; ++e) {
                const int ks = g * GE + e;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    fa[buf][e][tm] = *reinterpret_cast<const h16x8*>(sa + lds_off<BK>(wm0 + tm * 32 + li, ks * 2 + lg));
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    fb[buf][e][tn] = *reinterpret_cast<const h16x8*>(sb + lds_off<BK>(wn0 + tn * 32 + li, ks * 2 + lg));
            }
        };
        read_group(0, 0);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int buf = g & 1;
            if (g + 1 < NG) read_group(g + 1, buf ^ 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = 0; e < GE; ++e)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        // operands swapped: the accumulator holds out^T, i.e. every lane owns one pixel
                        // (lane%32) and runs of 4 consecutive output channels
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[buf][e][tn], fa[buf][e][tm], acc[tm][tn], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (++cur == NST) cur = 0;
    }
    if (!kEarlyEpi) gather_epi_request<BM, BN>(a, epi_first, 0, tid, nt, row_pix);
    RN50_WAIT_LGKMCNT0();
    __builtin_amdgcn_s_barrier();             // all waves are done reading the ring before it is reused

    gather_epilogue<BM, BN, TM, TN, LDS_HALFS, kAliasStats>(a, lds, acc, wm0, wn0, li, lg, tid, nt, tile_row, row_pix, epi_first);
}

// ------------------------------------------------------------------------------------------------
// 3x3, stride 1, pad 1 (forward, and the data gradient of such a layer)
// ------------------------------------------------------------------------------------------------
// With stride 1 and "same" padding, consecutive output pixels (flat index m over n, h, w) read consecutive input
// pixels: tap (dh, dw) of output pixel m is input pixel m + dh*W + dw.  One strip of BM + 2W + 2 input pixels
// therefore serves all nine taps of a tile of BM output pixels; it is loaded once per 32-channel slab instead of
// nine times (the gather kernel above loads every tap's rows separately).  Where a tap falls outside the image
// (top / bottom row, left / right column) the strip holds a neighbouring pixel instead of the zero padding; the
// A fragment of such a row is cleared in registers (a row is one lane of the fragment).  The nine filter taps of
// the slab sit next to the strip, [tap][column][32 channels].  Two stages: the next slab's strip and taps are in
// flight while the 9 x 2 x TM x TN MFMAs of the current one run.
constexpr int kStripMaxW = 56;      // widest image row the strip buffer is sized for

template <int BM, int WR, int WC, int NST, int OCC>
__global__ __launch_bounds__(kThreads, OCC) void strip_gemm_kernel(const GatherArgs a)
{
    constexpr int BN = 64, BK = 32, T = 9;
    constexpr int SROWS = (BM + 2 * kStripMaxW + 2 + 15) / 16 * 16;    // strip rows per stage, whole 1 KB DMA blocks
    constexpr int BROWS = T * BN;
    constexpr int NAJ = SROWS / 16 / 4, NBJ = BROWS / 16 / 4;          // DMA loads per thread and slab
    constexpr int STAGE = (SROWS + BROWS) * BK;                        // halfs
    constexpr int WM = BM / WR, WN = BN / WC, TM = WM / 32, TN = WN / 32;
    constexpr int KS = BK / 16;
    constexpr int EP = BN + 8;
    constexpr int EPI_HALFS = BM * EP + (kThreads / (BN / 8)) * 2 * BN * 2;
    constexpr int LDS_HALFS = (NST * STAGE > EPI_HALFS) ? NST * STAGE : EPI_HALFS;
    constexpr unsigned kOutOfRange = 0x80000000u;
    static_assert(WR * WC == 4 && TM >= 1 && TN >= 1 && SROWS % 64 == 0, "four waves; strip rows in whole rounds of the four waves");
    __shared__ __attribute__((aligned(16))) h16 lds[LDS_HALFS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lg = lane >> 5;
    const int wm0 = (wave / WC) * WM, wn0 = (wave % WC) * WN;

    const int n_tiles = a.NO / BN;
    const int bid = rn50_xcd_remap(blockIdx.x, gridDim.x);
    const int nt = bid % n_tiles, mt = bid / n_tiles;
    const int H = a.IH, W = a.IW, lda = a.lda, CR = a.CR;
    const int M = a.NB * H * W;
    const int m0 = mt * BM;
    const int p0 = m0 - (W + 1);                   // flat input pixel held by strip row 0
    const int naw = (BM + 2 * W + 2 + 15) >> 4;    // 16-row DMA blocks the strip needs for this image width

    // ---- this lane's place in a wave-wide load (16 rows of 64 bytes, two rows per 128-byte line) ----
    const int row_in_grp = 2 * (lane >> 3) + ((lane & 7) >> 2), phys = lane & 3;
    unsigned a_voff[NAJ], b_voff[NBJ];
#pragma unroll
    for (int j = 0; j < NAJ; ++j) {
        const int row = (wave + 4 * j) * 16 + row_in_grp;
        const int p = p0 + row;
        const int chunk = phys ^ lds_swz<BK>(row);
        a_voff[j] = ((unsigned)p < (unsigned)M) ? (unsigned)(p * lda) * 2u + chunk * 16 : kOutOfRange;
    }
#pragma unroll
    for (int j = 0; j < NBJ; ++j) {
        const int row = (wave + 4 * j) * 16 + row_in_grp;          // = tap slot * 64 + column
        const int slot = row >> 6, col = row & 63;
        const int bt = a.tap[0][slot] >> 16;                       // filter tap of this slot
        const int chunk = phys ^ lds_swz<BK>(row);
        b_voff[j] = (unsigned)(((nt * BN + col) * T + bt) * CR) * 2u + chunk * 16;
    }
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(a.A), 0, a.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(a.B), 0, a.b_bytes, 0x00020000);

    const int KC = CR / BK;
    int ld_cc = 0, ld_stage = 0;
    auto issue_slab = [&]() {
        h16* sa = lds + ld_stage * STAGE;
        h16* sb = sa + SROWS * BK;
        const unsigned delta = (unsigned)(ld_cc * BK) * 2u;
#pragma unroll
        for (int j = 0; j < NBJ; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)(sb + (wave + 4 * j) * 512), 16, (int)(b_voff[j] + delta), 0, 0, 0);
#pragma unroll
        for (int j = 0; j < NAJ; ++j)
            if (wave + 4 * j < naw) {      // wave-uniform
                const unsigned voff = a_voff[j] == kOutOfRange ? kOutOfRange : a_voff[j] + delta;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)(sa + (wave + 4 * j) * 512), 16, (int)voff, 0, 0, 0);
            }
        ++ld_cc;
        if (NST == 2) ld_stage ^= 1;
    };
    issue_slab();

    auto row_pix = [&](int row, int& n, int& oh, int& ow) -> bool {
        const int m = m0 + row;
        if (m >= M) return false;
        int t;
        fast_divmod(m, W, a.inv_ow[0], t, ow);
        fast_divmod(t, H, a.inv_oh[0], n, oh);
        return true;
    };

    // ---- per tap: where this lane's A rows sit in the strip, and whether the tap leaves the image there ----
    int fa_off[T][TM];         // halfs, k-step 0 (k-step 1: ^ 16)
    unsigned inval[TM];        // bit t: tap slot t reads outside the image for this lane's row
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        int n, oh, ow;
        const bool live = row_pix(wm0 + tm * 32 + li, n, oh, ow);
        unsigned bad = live ? 0u : 0x1ffu;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int tap = a.tap[0][t];
            const int dh = (int)(signed char)(tap & 0xff), dw = (int)(signed char)((tap >> 8) & 0xff);
            if (live && ((unsigned)(oh + dh) >= (unsigned)H || (unsigned)(ow + dw) >= (unsigned)W)) bad |= 1u << t;
            fa_off[t][tm] = lds_off<BK>(wm0 + tm * 32 + li + dh * W + dw + W + 1, lg);
        }
        inval[tm] = bad;
    }
    int fb_off[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) fb_off[tn] = lds_off<BK>(wn0 + tn * 32 + li, lg);

    f32x16 acc[TM][TN];
    gather_init_acc<BN>(a, acc, wm0, wn0, li, lg, nt, row_pix);
    EpiOperands<EpiShape<BM, BN>::CH> epi_first;

    int cur = 0;
    for (int kit = 0; kit < KC; ++kit) {
        RN50_WAIT_VMCNT(0);                   // this wave's part of slab kit has landed
        RN50_WAIT_LGKMCNT0();
        __builtin_amdgcn_s_barrier();         // everyone's part has; the other stage is free
        if (NST == 2 && kit + 1 < KC) issue_slab();
        const h16* sa = lds + cur * STAGE;
        const h16* sb = sa + SROWS * BK;
        // The operands of tap t+1 are requested before the MFMAs of tap t are issued (two register sets), so that
        // with a single wave per SIMD the LDS latency hides behind a whole tap's worth of matrix work.
        h16x8 fa[2][KS][TM], fb[2][KS][TN];
        auto read_tap = [&](int t, int buf) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    fa[buf][ks][tm] = *reinterpret_cast<const h16x8*>(sa + (fa_off[t][tm] ^ (ks * 16)));
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    fb[buf][ks][tn] = *reinterpret_cast<const h16x8*>(sb + t * (BN * BK) + (fb_off[tn] ^ (ks * 16)));
            }
        };
        read_tap(0, 0);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int buf = t & 1;
            if (t + 1 < T) read_tap(t + 1, buf ^ 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    if ((inval[tm] >> t) & 1u) fa[buf][ks][tm] = h16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[buf][ks][tn], fa[buf][ks][tm], acc[tm][tn], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (NST == 2) cur ^= 1;
        else if (kit + 1 < KC) {
            // single stage (several workgroups per compute unit overlap each other's loads and MFMAs instead):
            // the next slab overwrites this one once every wave is done reading it
            RN50_WAIT_LGKMCNT0();
            __builtin_amdgcn_s_barrier();
            issue_slab();
        }
    }
    gather_epi_request<BM, BN>(a, epi_first, 0, tid, nt, row_pix);     // in flight while the tile is staged
    RN50_WAIT_LGKMCNT0();
    __builtin_amdgcn_s_barrier();

    gather_epilogue<BM, BN, TM, TN, LDS_HALFS, false>(a, lds, acc, wm0, wn0, li, lg, tid, nt, mt, row_pix, epi_first);
}

// ------------------------------------------------------------------------------------------------
// filter gradient
// ------------------------------------------------------------------------------------------------
// out[k][g][c] = sum_{pix in this split} dy[pix][k] * X[pix, g][c], g = granule of G columns.
// Regular mode (G = 64): granule = (tap, 64-channel slab of x).  Stem mode (G = 32): granule = filter
// row r; the 32 columns are the 8 consecutive padded-image pixels x 4 channels starting at column 2q.
//
// Both operands are pixel-major in memory while the MFMA wants 8 consecutive pixels per lane.  The
// tiles travel global -> LDS untouched ([pixel][channel], same ring as the gather GEMM) and the
// operands are read with ds_read_b64_tr_b16, which transposes 4x4 blocks of halves across lanes:
// within 16 lanes, lane 4*r+e receives element e of the 8-byte words read by lanes r, 4+r, 8+r, 12+r.
// Lanes 4*j..4*j+3 therefore read 16 consecutive channels of pixel j, and lane L ends up with
// channel L of pixels 0..3.  Each workgroup reduces its own pixel range and stores an FP32 partial
// tile; a second kernel adds the partials in a fixed order (deterministic, no atomics).
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

// 8 bytes per lane through the transposing LDS read, as four halves
__device__ __forceinline__ h16x4 lds_read_tr(const h16* p) {
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(const_cast<h16*>(p)));
    return __builtin_bit_cast(h16x4, v);
}

template <int BM, int BN, int NST, int G, bool kStem, int BKP>      // BKP: pixels per K-slab
__global__ __launch_bounds__(kThreads, 2) void wgrad_kernel(const WgradArgs a)
{
    constexpr int A_LPR = BM / 8, A_RPI = 64 / A_LPR, NA = BKP / A_RPI / 4;
    constexpr int B_LPR = BN / 8, B_RPI = 64 / B_LPR, NB = BKP / B_RPI / 4;
    constexpr int NL = NA + NB;
    constexpr int STAGE = (BM + BN) * BKP;
    constexpr int WR = 2, WC = 2;
    constexpr int WM = BM / WR, WN = BN / WC, TM = WM / 32, TN = WN / 32;
    constexpr unsigned kOutOfRange = 0x80000000u;
    __shared__ __attribute__((aligned(16))) h16 lds[NST * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int wm0 = (wave / WC) * WM, wn0 = (wave % WC) * WN;

    const int m_tiles = a.K / BM, n_tiles = a.NG * G / BN;
    int bid = rn50_xcd_remap(blockIdx.x, gridDim.x);   // the tiles of one pixel range share the range's dy / x rows: same L2
    const int nt = bid % n_tiles; bid /= n_tiles;
    const int mt = bid % m_tiles;
    const int split = bid / m_tiles;
    const int pix_begin = split * a.pix_per_split;
    int pix_end = pix_begin + a.pix_per_split;
    if (pix_end > a.npix) pix_end = a.npix;
    const int kiters = (pix_end - pix_begin + BKP - 1) / BKP;

    // ---- this lane's part of the wave-wide loads ----
    // dy tile: [pixel][BM channels]; chunk index XOR-ed with 2*(pixel & 3) (conflict-free transposing reads)
    const int a_pl = lane / A_LPR, a_chunk = (lane % A_LPR) ^ ((a_pl & 3) << 1);
    const unsigned a_col = (unsigned)(mt * BM + a_chunk * 8) * 2u;
    const int b_pl = lane / B_LPR, b_chunk = (lane % B_LPR) ^ ((b_pl & 3) << 1);
    const int gran = nt * (BN / G) + (b_chunk * 8) / G;
    const int gcol = (b_chunk * 8) % G;
    int tap_r = 0, tap_s = 0, c0 = 0;
    bool gran_ok = true;
    if (kStem) { tap_r = gran; gran_ok = gran < a.R; }
    else {
        const int gpt = a.C / G;     // granules per tap
        const int tap = gran / gpt;
        tap_r = tap / a.S; tap_s = tap % a.S;
        c0 = (gran % gpt) * G + gcol;
    }
    const bool direct = a.direct != 0;   // 1x1 stride 1: x pixel index == dy pixel index
    const int K = a.K, C = a.C, H = a.H, W = a.W, P = a.P, Q = a.Q;
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(a.dy), 0, a.dy_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(a.x), 0, a.x_bytes, 0x00020000);

    int ld_pix = pix_begin, ld_stage = 0;
    auto issue_slab = [&]() {
        h16* sa = lds + ld_stage * STAGE;
        h16* sb = sa + BM * BKP;
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const int pix = ld_pix + (wave + 4 * j) * A_RPI + a_pl;
            const unsigned voff = pix < pix_end ? (unsigned)(pix * K) * 2u + a_col : kOutOfRange;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)(sa + (wave + 4 * j) * 512), 16, (int)voff, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int pix = ld_pix + (wave + 4 * j) * B_RPI + b_pl;
            bool ok = pix < pix_end && gran_ok;
            unsigned voff;
            if (direct) {
                voff = (unsigned)(pix * C + c0) * 2u;
            } else {
                int t, q, n, p;
                fast_divmod(pix, Q, a.inv_q, t, q);
                fast_divmod(t, P, a.inv_p, n, p);
                if (kStem) {
                    voff = (unsigned)(((n * H + 2 * p + tap_r) * W + 2 * q) * 4 + gcol) * 2u;   // padded image: in bounds
                } else {
                    const int ih = p * a.stride - a.pad + tap_r, iw = q * a.stride - a.pad + tap_s;
                    ok = ok && (unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W;
                    voff = (unsigned)(((n * H + ih) * W + iw) * C + c0) * 2u;
                }
            }
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)(sb + (wave + 4 * j) * 512), 16,
                                                     (int)(ok ? voff : kOutOfRange), 0, 0, 0);
        }
        ld_pix += BKP;
        if (++ld_stage == NST) ld_stage = 0;
    };

#pragma unroll
    for (int p = 0; p < NST - 1; ++p)
        if (p < kiters) issue_slab();

    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

    // transposing-read addresses: 16-lane group g4 serves channels 16*(g4&1).. and pixels 8*(g4>>1)..;
    // inside the group lane 4*jj+r reads channels 4r..4r+3 of pixel jj
    const int g4 = lane >> 4, jj = (lane >> 2) & 3, rr = lane & 3;
    int fa_off[TM], fb_off[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int ch = wm0 + tm * 32 + 16 * (g4 & 1) + 4 * rr;
        fa_off[tm] = (8 * (g4 >> 1) + jj) * BM + ((((ch >> 3) ^ (jj << 1)) << 3) | (ch & 7));
    }
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int ch = wn0 + tn * 32 + 16 * (g4 & 1) + 4 * rr;
        fb_off[tn] = (8 * (g4 >> 1) + jj) * BN + ((((ch >> 3) ^ (jj << 1)) << 3) | (ch & 7));
    }

    int cur = 0;
    for (int kit = 0; kit < kiters; ++kit) {
        if (kit + NST - 2 < kiters) RN50_WAIT_VMCNT(NL * (NST - 2));
        else RN50_WAIT_VMCNT(0);
        RN50_WAIT_LGKMCNT0();
        __builtin_amdgcn_s_barrier();
        if (kit + NST - 1 < kiters) issue_slab();
        h16* sa = lds + cur * STAGE;
        h16* sb = sa + BM * BKP;
#pragma unroll
        for (int ks = 0; ks < BKP / 16; ++ks) {
            h16x8 fa[TM], fb[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const h16x4 lo = lds_read_tr(sa + fa_off[tm] + (ks * 16) * BM);
                const h16x4 hi = lds_read_tr(sa + fa_off[tm] + (ks * 16 + 4) * BM);
                fa[tm] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const h16x4 lo = lds_read_tr(sb + fb_off[tn] + (ks * 16) * BN);
                const h16x4 hi = lds_read_tr(sb + fb_off[tn] + (ks * 16 + 4) * BN);
                fb[tn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[tm], fb[tn], acc[tm][tn], 0, 0, 0);
        }
        if (++cur == NST) cur = 0;
    }

    // ---- FP32 partial tile: lane owns column li, rows 8*(v/4) + 4*lg + v%4 ----
    const int row_len = a.NG * G;      // columns per output row
    float* out = a.out + (size_t)split * a.split_stride;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int col = nt * BN + wn0 + tn * 32 + li;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = mt * BM + wm0 + tm * 32 + (v / 4) * 8 + lg * 4 + (v % 4);
                out[(size_t)row * row_len + col] = acc[tm][tn][v];
            }
        }
}

// Filter gradient of a 3x3 / stride 1 / pad 1 convolution with operand reuse across the nine taps.
// Pixels are enumerated in PADDED coordinates (h+1, w+1) of an (H+2) x (W+2) frame per image; positions on the
// frame's border hold zeros (the DMA leaves them to the out-of-range zero fill, nothing is padded in memory).  In
// these coordinates tap (r, s) of output position pp is input position pp + (r-1)*(W+2) + (s-1) for every pp,
// border included (there dy is zero), so one slab of dy positions and ONE strip of x positions (the slab's range
// widened by W+3 on either side) serve all nine taps: a workgroup owns 64 output channels x 9 taps x 64 input
// channels, reads each dy fragment once per k-step for nine MFMAs, and moves 4-6 times fewer bytes from L2 into
// LDS per MFMA than the tile-per-tap kernel above.  No masks are needed.
// A K-slab is RPS = floor(64 / (W+2)) whole frame rows of one image (padded with zero rows to 64 positions), so
// that a lane's place inside a slab (frame row, frame column) never changes and the per-slab address arithmetic is
// scalar; the reduction gets up to 30 % longer for it (frame border + slab padding).  Slab ranges are split over
// workgroups as above (partial tiles, fixed-order sum).
constexpr int kWStripMaxW = 56, kWStripMinW = 10;                 // narrower images waste most of a 64-position slab
constexpr int kWStripPix = 64;                                    // positions per K-slab
constexpr int kWStripRows = 192;                                  // x strip rows per stage: 64 + 2*(56+2) + 2 = 182, in whole rounds of 32

__global__ __launch_bounds__(kThreads, 2) void wgrad_strip_kernel(const WgradArgs a)
{
    constexpr int BKP = kWStripPix, SROWS = kWStripRows, NST = 2, T = 9;
    constexpr int NA = BKP / 8 / 4, NB = SROWS / 8 / 4;            // wave-wide loads (8 rows of 128 bytes) per thread and slab
    constexpr int STAGE = (BKP + SROWS) * 64;                      // halfs
    constexpr unsigned kOutOfRange = 0x80000000u;
    __shared__ __attribute__((aligned(16))) h16 lds[NST * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lg = lane >> 5;
    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;

    const int K = a.K, C = a.C, H = a.H, W = a.W;
    const int WP = W + 2;
    const int rps = a.P, spi = a.Q;                                // frame rows per slab, slabs per image (set by the launcher)
    const int m_tiles = K / 64, n_tiles = C / 64;
    int bid = rn50_xcd_remap(blockIdx.x, gridDim.x);               // the tiles of one slab range share its dy / x rows: same L2
    const int nt = bid % n_tiles; bid /= n_tiles;
    const int mt = bid % m_tiles;
    const int split = bid / m_tiles;
    const int slab_begin = split * a.pix_per_split;                // in slabs
    int slab_end = slab_begin + a.pix_per_split;
    if (slab_end > a.npix) slab_end = a.npix;                      // npix: slabs in all
    const int kiters = slab_end - slab_begin;
    const int nbw = (BKP + 2 * WP + 2 + 7) >> 3;                   // wave-wide loads the strip needs

    // ---- this lane's fixed place in every slab: frame row (relative to the slab's first) and frame column ----
    const int pl = lane >> 3, chunk = (lane & 7) ^ ((pl & 3) << 1);       // row inside a wave-wide load, swizzled 16-byte chunk
    int a_row[NA], b_row[NB];
    unsigned a_off[NA], b_off[NB];
    bool a_ok[NA], b_ok[NB];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int i = (wave + 4 * j) * 8 + pl;                     // slab position
        const int rr = i / WP, wp = i - rr * WP;
        a_row[j] = rr;
        a_ok[j] = rr < rps && wp >= 1 && wp <= W;
        a_off[j] = (unsigned)((rr * W + wp) * K + mt * 64 + chunk * 8) * 2u;
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int sr = (wave + 4 * j) * 8 + pl;                    // strip row: slab position sr - (WP + 1)
        const int t = sr + WP - 1, q = t / WP, wp = t - q * WP;
        b_row[j] = q - 2;
        b_ok[j] = wp >= 1 && wp <= W;
        b_off[j] = (unsigned)(((q - 2) * W + wp) * C + nt * 64 + chunk * 8) * 2u;
    }
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(a.dy), 0, a.dy_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(const_cast<h16*>(a.x), 0, a.x_bytes, 0x00020000);

    int ld_n = slab_begin / spi, ld_si = slab_begin - ld_n * spi, ld_stage = 0;     // image and slab-in-image of the next slab to load
    auto issue_slab = [&]() {
        h16* sa = lds + ld_stage * STAGE;
        h16* sb = sa + BKP * 64;
        const int hp0 = ld_si * rps;                                                // frame row of slab position 0
        const int pix0 = (ld_n * H + hp0 - 1) * W - 1;                              // pixel index of frame position (hp0, 0), may be negative
        const unsigned base_a = (unsigned)(pix0 * K) * 2u, base_b = (unsigned)(pix0 * C) * 2u;
#pragma unroll
        for (int j = 0; j < NA; ++j) {
            const bool ok = a_ok[j] && (unsigned)(hp0 + a_row[j] - 1) < (unsigned)H;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)(sa + (wave + 4 * j) * 512), 16,
                                                     (int)(ok ? base_a + a_off[j] : kOutOfRange), 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < NB; ++j)
            if (wave + 4 * j < nbw) {          // wave-uniform
                const bool ok = b_ok[j] && (unsigned)(hp0 + b_row[j] - 1) < (unsigned)H;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)(sb + (wave + 4 * j) * 512), 16,
                                                         (int)(ok ? base_b + b_off[j] : kOutOfRange), 0, 0, 0);
            }
        if (++ld_si == spi) { ld_si = 0; ++ld_n; }
        ld_stage ^= 1;
    };
    if (kiters > 0) issue_slab();

    f32x16 acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    // transposing-read addresses (see wgrad_kernel): lane 4*jj+r of a 16-lane group reads channels 4r..4r+3 of pixel jj
    const int g4 = lane >> 4, jj = (lane >> 2) & 3, rr = lane & 3;
    const int cha = wm0 + 16 * (g4 & 1) + 4 * rr, chb = wn0 + 16 * (g4 & 1) + 4 * rr;
    const int fa_off = (8 * (g4 >> 1) + jj) * 64 + ((((cha >> 3) ^ (jj << 1)) << 3) | (cha & 7));
    int fb_off[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int row = 8 * (g4 >> 1) + jj + (t / 3) * WP + (t % 3);        // strip row 0 is slab position - (W+2) - 1
        fb_off[t] = row * 64 + ((((chb >> 3) ^ ((row & 3) << 1)) << 3) | (chb & 7));
    }

    int cur = 0;
    for (int kit = 0; kit < kiters; ++kit) {
        RN50_WAIT_VMCNT(0);
        RN50_WAIT_LGKMCNT0();
        __builtin_amdgcn_s_barrier();
        if (kit + 1 < kiters) issue_slab();
        h16* sa = lds + cur * STAGE;
        h16* sb = sa + BKP * 64;
#pragma unroll
        for (int ks = 0; ks < BKP / 16; ++ks) {
            const h16x4 alo = lds_read_tr(sa + fa_off + (ks * 16) * 64);
            const h16x4 ahi = lds_read_tr(sa + fa_off + (ks * 16 + 4) * 64);
            const h16x8 fa = __builtin_shufflevector(alo, ahi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const h16x4 lo = lds_read_tr(sb + fb_off[t] + (ks * 16) * 64);
                const h16x4 hi = lds_read_tr(sb + fb_off[t] + (ks * 16 + 4) * 64);
                const h16x8 fb = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa, fb, acc[t], 0, 0, 0);
            }
        }
        cur ^= 1;
    }

    // ---- FP32 partial tile [K][9][C]: lane owns column li, rows 8*(v/4) + 4*lg + v%4 ----
    const int row_len = T * C;
    float* out = a.out + (size_t)split * a.split_stride;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int col = t * C + nt * 64 + wn0 + li;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = mt * 64 + wm0 + (v / 4) * 8 + lg * 4 + (v % 4);
            out[(size_t)row * row_len + col] = acc[t][v];
        }
    }
}

// out[i] = sum over splits of part[s][i], stored as FP32 or rounded to half (the flat FP16 gradient).  A workgroup
// owns 16 consecutive float4 elements; 16 split lanes each add every 16th split in order, and their sums are
// combined in a fixed order through LDS.
template <bool kHalfOut>
__global__ __launch_bounds__(kThreads) void wgrad_reduce_kernel(const f32x4* __restrict__ part, void* __restrict__ out,
                                                                size_t n4, int nsplit, size_t stride4)
{
    __shared__ f32x4 red[16][16];
    const int il = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const size_t i = (size_t)blockIdx.x * 16 + il;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (i < n4)
        for (int k = sl; k < nsplit; k += 16) s += part[(size_t)k * stride4 + i];
    red[sl][il] = s;
    __syncthreads();
    if (sl == 0 && i < n4) {
        for (int k = 1; k < 16; ++k) s += red[k][il];
        if (kHalfOut) {
            h16x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = (h16)s[j];
            static_cast<h16x4*>(out)[i] = o;
        } else {
            static_cast<f32x4*>(out)[i] = s;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// small helpers: fills, casts, weight re-layouts, stem image staging
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void fill_zero_kernel(f32x4* p, size_t n4)
{
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (size_t)gridDim.x * kThreads) p[i] = z;
}

__global__ __launch_bounds__(kThreads) void cast_f32_to_h16_kernel(const float* __restrict__ src, h16* __restrict__ dst, size_t n)
{
    const size_t n8 = n / 8;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n8; i += (size_t)gridDim.x * kThreads) {
        const f32x4 u = reinterpret_cast<const f32x4*>(src)[2 * i], w = reinterpret_cast<const f32x4*>(src)[2 * i + 1];
        h16x8 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) { o[j] = (h16)u[j]; o[4 + j] = (h16)w[j]; }
        reinterpret_cast<h16x8*>(dst)[i] = o;
    }
    const size_t t = n8 * 8 + (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (t < n) dst[t] = (h16)src[t];
}

// KRSC -> CRSK for one filter: dst[c][t][k] = src[k][t][c].  32x32 tiles through LDS.
__global__ __launch_bounds__(kThreads) void transpose_filter_kernel(const h16* __restrict__ src, h16* __restrict__ dst,
                                                                    int K, int T, int C)
{
    __shared__ h16 tile[32][33];
    const int tiles_c = C / 32, tiles_k = K / 32;
    int b = blockIdx.x;
    const int tc = b % tiles_c; b /= tiles_c;
    const int tk = b % tiles_k;
    const int t = b / tiles_k;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int k = tk * 32 + ty + i * 8, c = tc * 32 + tx;
        tile[ty + i * 8][tx] = src[((size_t)k * T + t) * C + c];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tc * 32 + ty + i * 8, k = tk * 32 + tx;
        dst[((size_t)c * T + t) * K + k] = tile[tx][ty + i * 8];
    }
}

// stem: images [N,H,W,3] -> zero-padded [N,H+6,W+6,4] (3 pixels of padding on every side, 4th channel 0)
__global__ __launch_bounds__(kThreads) void stem_pad_image_kernel(const h16* __restrict__ img, h16* __restrict__ dst,
                                                                  int N, int H, int W)
{
    const int HP = H + 6, WP = W + 6;
    const size_t total = (size_t)N * HP * WP;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
        const int wp = (int)(i % WP);
        const size_t t = i / WP;
        const int hp = (int)(t % HP), n = (int)(t / HP);
        const int h = hp - 3, w = wp - 3;
        h16x4 v = {0, 0, 0, 0};
        if ((unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W) {
            const h16* s = img + (((size_t)n * H + h) * W + w) * 3;
            v[0] = s[0]; v[1] = s[1]; v[2] = s[2];
        }
        reinterpret_cast<h16x4*>(dst)[i] = v;
    }
}

// stem filter [K][7][7][3] -> [K][7][32]: column s*4+c, zero for s = 7 or c = 3
__global__ __launch_bounds__(kThreads) void stem_pack_filter_kernel(const h16* __restrict__ w, h16* __restrict__ dst, int K)
{
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= K * 7 * 32) return;
    const int col = i % 32, r = (i / 32) % 7, k = i / (32 * 7);
    const int s = col / 4, c = col % 4;
    dst[i] = (s < 7 && c < 3) ? w[(((size_t)k * 7 + r) * 7 + s) * 3 + c] : (h16)0.f;
}

// stem filter gradient: acc [K][8][32] (row r, column s*4+c, FP32) -> out [K][7][7][3] (half)
__global__ __launch_bounds__(kThreads) void stem_unpack_wgrad_kernel(const float* __restrict__ acc, h16* __restrict__ out, int K)
{
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= K * 147) return;
    const int c = i % 3, s = (i / 3) % 7, r = (i / 21) % 7, k = i / 147;
    out[i] = (h16)acc[((size_t)k * 8 + r) * 32 + s * 4 + c];
}

int grid_for(size_t work_items)
{
    size_t b = (work_items + kThreads - 1) / kThreads;
    if (b > 256 * 8) b = 256 * 8;
    return b < 1 ? 1 : (int)b;
}

inline int floordiv(int a, int b) { return (a >= 0) ? a / b : -((-a + b - 1) / b); }
inline int pack_tap(int dh, int dw, int bt) { return (dh & 0xff) | ((dw & 0xff) << 8) | (bt << 16); }

template <int BM, int BN, int BK, int NST, int OCC>
int launch_gather(GatherArgs& a, hipStream_t s, int kid, double flops, double bytes)
{
    int total = 0;
    for (int c = 0; c < a.ncls; ++c) {
        const long long M = (long long)a.NB * a.cOHs[c] * a.cOWs[c];
        total += (int)((M + BM - 1) / BM);
        a.mt_end[c] = total;
        a.inv_oh[c] = 1.0f / (float)(a.cOHs[c] > 0 ? a.cOHs[c] : 1);
        a.inv_ow[c] = 1.0f / (float)(a.cOWs[c] > 0 ? a.cOWs[c] : 1);
    }
    if (total == 0) return RN50_OK;
    const int grid = total * (a.NO / BN);
    a.xcd_split_cols = (a.b_bytes > a.a_bytes && (a.NO / BN) % 8 == 0) ? 1 : 0;
    ProfScope ps(kid, flops, bytes, s);
    gather_gemm_kernel<BM, BN, BK, NST, OCC><<<grid, kThreads, 0, s>>>(a);
    return rn50_check_launch();
}

template <int BM, int WR, int WC, int NST, int OCC>
int launch_strip(GatherArgs& a, hipStream_t s, int kid, double flops, double bytes)
{
    const long long M = (long long)a.NB * a.cOHs[0] * a.cOWs[0];
    const int total = (int)((M + BM - 1) / BM);
    a.mt_end[0] = total;
    a.inv_oh[0] = 1.0f / (float)a.cOHs[0];
    a.inv_ow[0] = 1.0f / (float)a.cOWs[0];
    if (total == 0) return RN50_OK;
    ProfScope ps(kid, flops, bytes, s);
    strip_gemm_kernel<BM, WR, WC, NST, OCC><<<total * (a.NO / 64), kThreads, 0, s>>>(a);
    return rn50_check_launch();
}

// the strip kernel covers 3x3 / stride 1 / pad 1 in either direction: nine taps in one class, output grid = input grid
bool strip_ok(const GatherArgs& a)
{
    return a.ncls == 1 && a.ntaps[0] == 9 && a.T == 9 && a.a_mul == 1 && a.o_mul == 1 && a.a_off == 0 && a.IH == a.OH &&
           a.IW == a.OW && a.IW <= kStripMaxW && a.lda == a.CR && a.CR % 32 == 0 && a.NO % 64 == 0 && a.IH >= 1;
}

bool gather_tile_ok(const GatherArgs& a, int tile)
{
    if (tile < 0 || tile >= RN50_NUM_GATHER_TILES) return false;
    if (tile >= RN50_TILE_STRIP_256 && tile <= RN50_TILE_STRIP_64_S1) return strip_ok(a);
    if (tile == RN50_TILE_128x128_K64 || tile == RN50_TILE_256x128_K64) return a.NO % 128 == 0 && a.CR % 64 == 0;
    if (tile == RN50_TILE_256x64_K64) return a.CR % 64 == 0;
    if (tile == RN50_TILE_64x64_K128 || tile == RN50_TILE_128x64_K128) return a.CR % 128 == 0;
    if (tile == RN50_TILE_64x64_K256) return a.CR % 256 == 0;
    return (tile != RN50_TILE_128x128 && tile != RN50_TILE_128x128_SHORT && tile != RN50_TILE_128x128_OCC4) || a.NO % 128 == 0;
}

// default choice when no tuned tile is given (what the autotuner picks most often for such shapes): the large
// tiles while they still yield about two workgroups per compute unit; else 64x64 tiles, with the deepest K-slab
// the reduction length allows when there are too few workgroups to cover the load latency by numbers
int gather_tile_heuristic(const GatherArgs& a)
{
    long long rows = 0;
    for (int c = 0; c < a.ncls; ++c) rows += (long long)a.NB * a.cOHs[c] * a.cOWs[c];
    if (a.NO % 128 == 0 && (rows / 128) * (a.NO / 128) >= 400) return RN50_TILE_128x128_SHORT;
    if ((rows / 128) * (a.NO / 64) >= 400) return RN50_TILE_128x64_SHORT;
    const long long small = ((rows + 63) / 64) * (a.NO / 64);
    if (small <= 256 && a.CR % 256 == 0) return RN50_TILE_64x64_K256;
    if (small <= 512 && a.CR % 128 == 0) return RN50_TILE_64x64_K128;
    return RN50_TILE_64x64_WIDE;
}

int dispatch_gather(GatherArgs& a, hipStream_t s, double flops, double bytes, int tile)
{
    // RN50_TILE_STRICT (tuning): a variant that does not apply to this shape is an error instead of a fallback;
    // RN50_TILE_QUERY: only say whether it applies
    const bool strict = tile >= 0 && (tile & RN50_TILE_STRICT) != 0;
    const bool query = tile >= 0 && (tile & RN50_TILE_QUERY) != 0;
    if (tile >= 0) tile &= ~(RN50_TILE_STRICT | RN50_TILE_QUERY);
    if (a.CR == 32) {               // stem forward (one 32-wide slab per filter row): the 32-wide tiles with 64 columns
        const bool ok = tile == RN50_TILE_128x64 || tile == RN50_TILE_128x64_SHORT || tile == RN50_TILE_64x64_K32 ||
                        tile == RN50_TILE_256x64;
        if (query || (strict && !ok)) return ok ? RN50_OK : RN50_ERR_SHAPE;
        switch (ok ? tile : RN50_TILE_128x64) {
            case RN50_TILE_128x64_SHORT: return launch_gather<128, 64, 32, 2, 4>(a, s, RN50_K_GATHER_STEM, flops, bytes);
            case RN50_TILE_64x64_K32: return launch_gather<64, 64, 32, 4, 4>(a, s, RN50_K_GATHER_STEM, flops, bytes);
            case RN50_TILE_256x64: return launch_gather<256, 64, 32, 3, 2>(a, s, RN50_K_GATHER_STEM, flops, bytes);
            default: return launch_gather<128, 64, 32, 4, 2>(a, s, RN50_K_GATHER_STEM, flops, bytes);
        }
    }
    if (!gather_tile_ok(a, tile)) {
        if (strict || query) return RN50_ERR_SHAPE;
        tile = gather_tile_heuristic(a);
    }
    if (query) return RN50_OK;
    static_assert(RN50_K_GATHER_TILE_LAST - RN50_K_GATHER_TILE0 + 1 == RN50_NUM_GATHER_TILES, "one profile id per tile variant");
    const int kid = RN50_K_GATHER_TILE0 + tile;
    switch (tile) {
        case RN50_TILE_128x128: return launch_gather<128, 128, 32, 4, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_128x64: return launch_gather<128, 64, 32, 4, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_64x64_DEEP: return launch_gather<64, 64, 64, 4, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_64x64_WIDE: return launch_gather<64, 64, 64, 2, 4>(a, s, kid, flops, bytes);
        case RN50_TILE_128x64_SHORT: return launch_gather<128, 64, 32, 2, 4>(a, s, kid, flops, bytes);
        case RN50_TILE_128x128_SHORT: return launch_gather<128, 128, 32, 2, 3>(a, s, kid, flops, bytes);
        case RN50_TILE_256x64: return launch_gather<256, 64, 32, 3, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_128x64_K64: return launch_gather<128, 64, 64, 3, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_64x64_K128: return launch_gather<64, 64, 128, 2, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_128x64_K128: return launch_gather<128, 64, 128, 2, 1>(a, s, kid, flops, bytes);
        case RN50_TILE_64x64_K256: return launch_gather<64, 64, 256, 2, 1>(a, s, kid, flops, bytes);
        case RN50_TILE_128x128_K64: return launch_gather<128, 128, 64, 2, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_256x64_K64: return launch_gather<256, 64, 64, 2, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_256x128_K64: return launch_gather<256, 128, 64, 2, 1>(a, s, kid, flops, bytes);
        case RN50_TILE_STRIP_256: return launch_strip<256, 4, 1, 2, 1>(a, s, kid, flops, bytes);
        case RN50_TILE_STRIP_128: return launch_strip<128, 2, 2, 2, 1>(a, s, kid, flops, bytes);
        case RN50_TILE_STRIP_64: return launch_strip<64, 2, 2, 2, 1>(a, s, kid, flops, bytes);
        case RN50_TILE_STRIP_256_S1: return launch_strip<256, 4, 1, 1, 2>(a, s, kid, flops, bytes);
        case RN50_TILE_STRIP_128_S1: return launch_strip<128, 2, 2, 1, 3>(a, s, kid, flops, bytes);
        case RN50_TILE_STRIP_64_S1: return launch_strip<64, 2, 2, 1, 3>(a, s, kid, flops, bytes);
        case RN50_TILE_128x128_OCC4: return launch_gather<128, 128, 32, 2, 4>(a, s, kid, flops, bytes);
        default: tile = RN50_TILE_64x64_K32; return launch_gather<64, 64, 32, 4, 4>(a, s, RN50_K_GATHER_TILE0 + tile, flops, bytes);
    }
}

}  // namespace

// output rows (pixels) per workgroup of a gather-GEMM tile variant
int rn50_gather_tile_rows(int tile)
{
    switch (tile) {
        case RN50_TILE_64x64_DEEP: case RN50_TILE_64x64_WIDE: case RN50_TILE_64x64_K32: case RN50_TILE_64x64_K128:
        case RN50_TILE_64x64_K256: case RN50_TILE_STRIP_64: case RN50_TILE_STRIP_64_S1: return 64;
        case RN50_TILE_256x64: case RN50_TILE_256x64_K64: case RN50_TILE_256x128_K64: case RN50_TILE_STRIP_256:
        case RN50_TILE_STRIP_256_S1: return 256;
        default: return 128;
    }
}

namespace {
// algorithmic work of one convolution (either direction): 2*M*N*K flops; bytes = input pixels actually
// needed + filter + output, 2 bytes each
double conv_flops(const conv_desc& d, int P, int Q) { return 2.0 * d.n * P * Q * (double)d.k * d.r * d.s * d.c; }
double conv_bytes(const conv_desc& d, int P, int Q, bool with_addend)
{
    const double in = (d.r == 1 && d.stride > 1) ? (double)d.n * P * Q * d.c : (double)d.n * d.h * d.w * d.c;
    double b = 2.0 * (in + (double)d.k * d.r * d.s * d.c + (double)d.n * P * Q * d.k);
    if (with_addend) b += 2.0 * d.n * d.h * d.w * d.c;
    return b;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// internal entry points (also used by the whole-step driver)
// ------------------------------------------------------------------------------------------------
bool rn50_conv_is_stem(const conv_desc& d) { return d.c == 3 && d.r == 7 && d.s == 7 && d.stride == 2 && d.pad == 3; }

int rn50_conv_validate(const conv_desc* d)
{
    if (!d) return RN50_ERR_NULL;
    if (d->dt != RN50_F16) return RN50_ERR_DTYPE;
    if (d->n < 1 || d->h < 1 || d->w < 1 || d->k < 64 || d->k % 64 != 0) return RN50_ERR_SHAPE;
    // tensors stay below 2 GiB (32-bit buffer offsets) and pixel counts below 2^24 (float reciprocal division)
    if ((long long)d->n * (d->h + 6) * (d->w + 6) * (d->c > d->k ? d->c : d->k) >= (1ll << 30)) return RN50_ERR_SHAPE;
    if ((long long)d->n * d->h * d->w >= (1ll << 24)) return RN50_ERR_SHAPE;
    if (rn50_conv_is_stem(*d)) return (d->h % 2 == 0 && d->w % 2 == 0) ? RN50_OK : RN50_ERR_SHAPE;
    if (d->c < 64 || d->c % 64 != 0) return RN50_ERR_SHAPE;
    if (d->r != d->s || (d->r != 1 && d->r != 3)) return RN50_ERR_SHAPE;
    if (d->stride != 1 && d->stride != 2) return RN50_ERR_SHAPE;
    if (d->pad != (d->r - 1) / 2) return RN50_ERR_SHAPE;
    if (d->h + 2 * d->pad < d->r || d->w + 2 * d->pad < d->s) return RN50_ERR_SHAPE;
    return RN50_OK;
}

static inline int out_dim(int h, int pad, int r, int stride) { return (h + 2 * pad - r) / stride + 1; }

size_t rn50_stem_padded_bytes(const conv_desc& d) { return rn50_round_up((size_t)d.n * (d.h + 6) * (d.w + 6) * 4 * sizeof(h16), 256); }
size_t rn50_stem_packed_filter_bytes(const conv_desc& d) { return rn50_round_up((size_t)d.k * 7 * 32 * sizeof(h16), 256); }

int rn50_stem_pad_image(const conv_desc& d, const h16* img, h16* padded, hipStream_t s)
{
    ProfScope ps(RN50_K_STEM_MISC, 0.0, (double)d.n * d.h * d.w * 6 + (double)d.n * (d.h + 6) * (d.w + 6) * 8, s);
    stem_pad_image_kernel<<<grid_for((size_t)d.n * (d.h + 6) * (d.w + 6)), kThreads, 0, s>>>(img, padded, d.n, d.h, d.w);
    return rn50_check_launch();
}

int rn50_stem_pack_filter(const conv_desc& d, const h16* w, h16* packed, hipStream_t s)
{
    ProfScope ps(RN50_K_STEM_MISC, 0.0, (double)d.k * (147 + 224) * 2, s);
    stem_pack_filter_kernel<<<rn50_cdiv(d.k * 7 * 32, kThreads), kThreads, 0, s>>>(w, packed, d.k);
    return rn50_check_launch();
}

int rn50_transpose_filter(const conv_desc& d, const h16* w, h16* wt, hipStream_t s)
{
    const int T = d.r * d.s;
    ProfScope ps(RN50_K_TRANSPOSE, 0.0, 4.0 * d.k * T * d.c, s);
    transpose_filter_kernel<<<(d.c / 32) * (d.k / 32) * T, kThreads, 0, s>>>(w, wt, d.k, T, d.c);
    return rn50_check_launch();
}

int rn50_fill_zero(float* p, size_t n, hipStream_t s)
{
    // n must be a multiple of 4 floats
    ProfScope ps(RN50_K_FILL, 0.0, 4.0 * n, s);
    fill_zero_kernel<<<grid_for(n / 4), kThreads, 0, s>>>(reinterpret_cast<f32x4*>(p), n / 4);
    return rn50_check_launch();
}

int rn50_cast_f32_to_h16(const float* src, h16* dst, size_t n, hipStream_t s)
{
    ProfScope ps(RN50_K_CAST, 0.0, 6.0 * n, s);
    cast_f32_to_h16_kernel<<<grid_for(n / 8 + 1), kThreads, 0, s>>>(src, dst, n);
    return rn50_check_launch();
}

// Forward.  For the stem, x is the padded 4-channel image and w the packed filter.
int rn50_conv_fwd_launch(const conv_desc& d, const h16* x, const h16* w, h16* y, hipStream_t s, float* stats_part,
                         int* stats_tiles, int tile)
{
    GatherArgs a = {};
    a.stats_part = stats_part;
    const int P = out_dim(d.h, d.pad, d.r, d.stride), Q = out_dim(d.w, d.pad, d.s, d.stride);
    a.A = x; a.B = w; a.out = y; a.addend = nullptr;
    a.NB = d.n; a.NO = d.k; a.OH = P; a.OW = Q; a.o_mul = 1;
    a.ncls = 1; a.cOHs[0] = P; a.cOWs[0] = Q; a.oph[0] = 0; a.opw[0] = 0;
    a.a_mul = d.stride;
    if (rn50_conv_is_stem(d)) {
        a.a_bytes = (unsigned)((size_t)d.n * (d.h + 6) * (d.w + 6) * 4 * sizeof(h16));
        a.b_bytes = (unsigned)((size_t)d.k * 7 * 32 * sizeof(h16));
        a.IH = d.h + 6; a.IW = d.w + 6; a.lda = 4; a.CR = 32; a.T = 7; a.a_off = 0;
        a.ntaps[0] = 7;
        for (int r = 0; r < 7; ++r) a.tap[0][r] = pack_tap(r, 0, r);
    } else {
        a.a_bytes = (unsigned)((size_t)d.n * d.h * d.w * d.c * sizeof(h16));
        a.b_bytes = (unsigned)((size_t)d.k * d.r * d.s * d.c * sizeof(h16));
        a.IH = d.h; a.IW = d.w; a.lda = d.c; a.CR = d.c; a.T = d.r * d.s; a.a_off = 0;
        a.ntaps[0] = d.r * d.s;
        for (int r = 0; r < d.r; ++r)
            for (int q = 0; q < d.s; ++q) {
                const int t = r * d.s + q;
                a.tap[0][t] = pack_tap(r - d.pad, q - d.pad, t);
            }
    }
    const int rc = dispatch_gather(a, s, conv_flops(d, P, Q), conv_bytes(d, P, Q, false), tile);
    if (stats_tiles) *stats_tiles = a.mt_end[0];
    return rc;
}

// Data gradient.  wt is the filter transposed to [C][R][S][K].  addend (nullable) has dx's layout.
int rn50_conv_dgrad_launch(const conv_desc& d, const h16* dy, const h16* wt, const h16* addend, h16* dx, hipStream_t s,
                           const DgradBnFuse* fuse, int* tiles_out, int tile, bool addend_even_only)
{
    GatherArgs a = {};
    if (fuse) {
        a.mask_y = fuse->mask_y; a.bn_x = fuse->bn_x; a.bn_mean = fuse->mean; a.bn_invstd = fuse->invstd;
        a.stats_part = fuse->part;
        if (fuse->bn_x2 && fuse->part2) {
            a.bn_x2 = fuse->bn_x2; a.bn_mean2 = fuse->mean2; a.bn_invstd2 = fuse->invstd2; a.stats_part2 = fuse->part2;
        }
    }
    const int P = out_dim(d.h, d.pad, d.r, d.stride), Q = out_dim(d.w, d.pad, d.s, d.stride);
    a.A = dy; a.B = wt; a.out = dx; a.addend = addend;
    a.add_sub = (addend && addend_even_only) ? 1 : 0; a.add_h = (d.h + 1) / 2; a.add_w = (d.w + 1) / 2;
    a.a_bytes = (unsigned)((size_t)d.n * P * Q * d.k * sizeof(h16));
    a.b_bytes = (unsigned)((size_t)d.k * d.r * d.s * d.c * sizeof(h16));
    a.NB = d.n; a.IH = P; a.IW = Q; a.lda = d.k; a.CR = d.k; a.T = d.r * d.s; a.NO = d.c;
    a.OH = d.h; a.OW = d.w; a.a_mul = 1; a.a_off = 0; a.o_mul = d.stride;
    a.ncls = d.stride * d.stride;
    for (int ph = 0; ph < d.stride; ++ph)
        for (int pw = 0; pw < d.stride; ++pw) {
            const int c = ph * d.stride + pw;
            a.oph[c] = ph; a.opw[c] = pw;
            a.cOHs[c] = (d.h - ph + d.stride - 1) / d.stride;
            a.cOWs[c] = (d.w - pw + d.stride - 1) / d.stride;
            int nt = 0;
            for (int r = 0; r < d.r; ++r) {
                const int eh = ph + d.pad - r;
                if (((eh % d.stride) + d.stride) % d.stride != 0) continue;
                for (int q = 0; q < d.s; ++q) {
                    const int ew = pw + d.pad - q;
                    if (((ew % d.stride) + d.stride) % d.stride != 0) continue;
                    a.tap[c][nt] = pack_tap(floordiv(eh, d.stride), floordiv(ew, d.stride), r * d.s + q);
                    ++nt;
                }
            }
            a.ntaps[c] = nt;
        }
    // A strided 1x1 convolution reaches only the (even, even) input pixels: the other three parity classes of dx are
    // plain zeros.  Without an addend or a fused epilogue they are cleared by a fill of the whole tensor and only the
    // first class goes through the GEMM.
    if (d.r == 1 && d.stride == 2 && !addend && !fuse) {
        const bool query = tile >= 0 && (tile & RN50_TILE_QUERY) != 0;       // a query launches nothing
        if (!query) RN50_TRY(rn50_fill_zero(reinterpret_cast<float*>(dx), (size_t)d.n * d.h * d.w * d.c / 2, s));
        a.ncls = 1;
    }
    // a strided 1x1 data gradient still writes every pixel of dx
    const double bytes = conv_bytes(d, P, Q, addend != nullptr) +
                         ((d.r == 1 && d.stride > 1) ? 2.0 * d.n * ((double)d.h * d.w - (double)P * Q) * d.c : 0.0);
    const int rc = dispatch_gather(a, s, conv_flops(d, P, Q), bytes + (fuse ? 4.0 * d.n * d.h * d.w * d.c : 0.0), tile);
    if (tiles_out) *tiles_out = a.mt_end[a.ncls - 1];
    return rc;
}

// upper bound of the floats a fused data gradient writes to DgradBnFuse::part: one row tile per 64 pixels
// (plus one ragged tile per parity class), two sums per input channel
size_t rn50_dgrad_stats_floats(const conv_desc& d)
{
    const long long rows = (long long)d.n * d.h * d.w;
    return (size_t)((rows + 63) / 64 + 4) * 2 * d.c;
}

// upper bound of the floats conv_fwd writes to stats_part: (smallest tile = 64 rows) x 2 x k
size_t rn50_conv_stats_floats(const conv_desc& d)
{
    const long long M = (long long)d.n * out_dim(d.h, d.pad, d.r, d.stride) * out_dim(d.w, d.pad, d.s, d.stride);
    return (size_t)((M + 63) / 64) * 2 * d.k;
}

size_t rn50_wgrad_acc_floats(const conv_desc& d)
{
    if (rn50_conv_is_stem(d)) return (size_t)d.k * 8 * 32;
    return (size_t)d.k * d.r * d.s * d.c;
}

namespace {
// Tile variants of the filter gradient: (filters) x (filter-element columns), ring stages, pixels per K-slab.
// A shape that does not allow a 128-wide side runs the 64x64 tile of the same slab depth instead.
struct WgradTile { int BM, BN, NST, BKP; };
constexpr WgradTile kWgradTiles[RN50_WGRAD_TILE_STRIP] = {
    {128, 128, 4, 32}, {64, 64, 4, 32}, {64, 128, 4, 32}, {128, 64, 4, 32},
    {64, 64, 3, 64}, {64, 64, 2, 64}, {64, 64, 2, 128}, {64, 128, 3, 64}, {128, 64, 3, 64}, {128, 128, 2, 64}};
constexpr int kWgradFallback32 = 1, kWgradFallback64 = 4, kWgradFallback128 = 6;   // the 64x64 tile per slab depth

struct WgradPlan { int tile, BM, BN, G, NG, tiles, nsplit, pix_per_split; bool stem, strip; };

// the strip kernel covers 3x3 / stride 1 / pad 1 with image rows of at most kWStripMaxW pixels
bool wgrad_strip_ok(const conv_desc& d)
{
    return d.r == 3 && d.s == 3 && d.stride == 1 && d.pad == 1 && d.w <= kWStripMaxW && d.w >= kWStripMinW && d.c % 64 == 0 &&
           d.k % 64 == 0;
}
// frame rows per 64-position slab, slabs per image
inline int wstrip_rps(const conv_desc& d) { return kWStripPix / (d.w + 2); }
inline int wstrip_spi(const conv_desc& d) { return (d.h + 2 + wstrip_rps(d) - 1) / wstrip_rps(d); }

// variant: RN50_TILE_AUTO, or tile_index * 3 + split_index: a kWgradTiles entry and a split target of 256, 512 or
// 1024 workgroups
WgradPlan wgrad_plan(const conv_desc& d, int variant)
{
    WgradPlan p;
    // without a tuned variant: 64x64 tiles with 128-pixel slabs, 256 workgroups (the autotuner's most frequent pick)
    const int want_blocks = variant < 0 ? 256 : 256 << (variant % 3);
    p.tile = variant < 0 ? kWgradFallback128 : variant / 3;
    const int P = out_dim(d.h, d.pad, d.r, d.stride), Q = out_dim(d.w, d.pad, d.s, d.stride);
    const long long npix = (long long)d.n * P * Q;
    p.stem = rn50_conv_is_stem(d);
    p.strip = false;
    if (!p.stem && p.tile == RN50_WGRAD_TILE_STRIP) {
        if (wgrad_strip_ok(d)) {
            // 64 filters x 9 taps x 64 channels per workgroup; 128, 256 or 512 workgroups; ranges of padded positions
            p.strip = true;
            p.BM = 64; p.BN = 64; p.G = 64; p.NG = 9 * d.c / 64;
            p.tiles = (d.k / 64) * (d.c / 64);
            const long long slabs_s = (long long)d.n * wstrip_spi(d);
            long long want_s = ((128 << (variant % 3)) + p.tiles - 1) / p.tiles;
            long long per = (slabs_s + want_s - 1) / want_s;
            if (per < 4) per = slabs_s < 4 ? slabs_s : 4;
            p.pix_per_split = (int)per;                    // in slabs
            p.nsplit = (int)((slabs_s + per - 1) / per);
            return p;
        }
        p.tile = kWgradFallback128;
    }
    if (p.stem) { p.tile = -1; p.BM = 64; p.BN = 64; p.G = 32; p.NG = 8; }
    else {
        p.G = 64; p.NG = d.r * d.s * d.c / 64;
        const WgradTile& t = kWgradTiles[p.tile];
        if ((t.BM == 128 && d.k % 128 != 0) || (t.BN == 128 && p.NG % 2 != 0))
            p.tile = t.BKP == 32 ? kWgradFallback32 : t.BKP == 64 ? kWgradFallback64 : kWgradFallback128;
        p.BM = kWgradTiles[p.tile].BM; p.BN = kWgradTiles[p.tile].BN;
    }
    p.tiles = (d.k / p.BM) * (p.NG * p.G / p.BN);
    // pixel splits: about want_blocks workgroups, but at least 8 K-slabs of 32 pixels each
    const long long slabs = (npix + 31) / 32;
    long long want = (want_blocks + p.tiles - 1) / p.tiles;
    long long slabs_per = (slabs + want - 1) / want;
    if (slabs_per < 8) slabs_per = slabs < 8 ? slabs : 8;
    p.pix_per_split = (int)(slabs_per * 32);
    p.nsplit = (int)((slabs + slabs_per - 1) / slabs_per);
    return p;
}

template <int TILE>
void launch_wgrad_tile(const WgradArgs& a, int grid, hipStream_t s)
{
    constexpr WgradTile t = kWgradTiles[TILE];
    wgrad_kernel<t.BM, t.BN, t.NST, 64, false, t.BKP><<<grid, kThreads, 0, s>>>(a);
}
}  // namespace

// floats of scratch rn50_conv_wgrad_launch needs for its per-split partial tiles
size_t rn50_wgrad_partial_floats(const conv_desc& d)
{
    size_t most = 0;
    for (int v = RN50_TILE_AUTO; v < RN50_NUM_WGRAD_VARIANTS; ++v) {
        const WgradPlan p = wgrad_plan(d, v);
        const size_t f = (size_t)p.nsplit * rn50_wgrad_acc_floats(d);
        if (f > most) most = f;
    }
    return most;
}

// A filter-gradient variant whose tile does not apply to the shape runs a fallback tile with the same split target;
// this returns the id of what actually runs (so that a stored table names it).
int rn50_wgrad_canonical_variant(const conv_desc& d, int variant)
{
    if (variant < 0 || rn50_conv_is_stem(d)) return variant;
    return wgrad_plan(d, variant).tile * 3 + variant % 3;
}

// bytes of partial tiles that variant `variant` writes (and the sum kernel reads back)
size_t rn50_wgrad_variant_partial_bytes(const conv_desc& d, int variant)
{
    const WgradPlan p = wgrad_plan(d, variant);
    return (size_t)p.nsplit * rn50_wgrad_acc_floats(d) * sizeof(float);
}

// Filter gradient: every pixel split leaves an FP32 partial tile in `partials` (rn50_wgrad_partial_floats(d) floats);
// their sum goes to out16 as half (layout [K][R][S][C], a slice of the flat FP16 gradient) or, for the stem, to
// out32 in FP32 (layout [K][8][32], unpacked afterwards).  Exactly one of out16 / out32 is given; every element is
// written.  For the stem, x is the padded 4-channel image.
int rn50_conv_wgrad_launch(const conv_desc& d, const h16* x, const h16* dy, h16* out16, float* out32, float* partials,
                           hipStream_t s, int variant)
{
    WgradArgs a = {};
    const WgradPlan p = wgrad_plan(d, variant);
    const int P = out_dim(d.h, d.pad, d.r, d.stride), Q = out_dim(d.w, d.pad, d.s, d.stride);
    a.x = x; a.dy = dy;
    a.K = d.k; a.P = P; a.Q = Q; a.npix = d.n * P * Q;
    a.inv_p = 1.0f / (float)P; a.inv_q = 1.0f / (float)Q;
    a.stride = d.stride; a.pad = d.pad; a.R = d.r; a.S = d.s; a.NG = p.NG;
    a.dy_bytes = (unsigned)((size_t)a.npix * d.k * sizeof(h16));
    if (p.stem) {
        a.H = d.h + 6; a.W = d.w + 6; a.C = 4; a.direct = 0;
        a.x_bytes = (unsigned)((size_t)d.n * a.H * a.W * 4 * sizeof(h16));
    } else {
        a.H = d.h; a.W = d.w; a.C = d.c; a.direct = (d.r == 1 && d.stride == 1) ? 1 : 0;
        a.x_bytes = (unsigned)((size_t)d.n * d.h * d.w * d.c * sizeof(h16));
    }
    a.pix_per_split = p.pix_per_split;
    a.split_stride = rn50_wgrad_acc_floats(d);
    a.out = partials;
    const int grid = p.tiles * p.nsplit;
    if (p.strip) {      // the reduction runs over slabs of whole frame rows: P = frame rows per slab, Q = slabs per image
        a.P = wstrip_rps(d); a.Q = wstrip_spi(d);
        a.npix = d.n * a.Q;
    }
    {
        const double bytes = 2.0 * ((double)d.n * d.h * d.w * d.c + (double)d.n * P * Q * d.k) + 4.0 * d.k * d.r * d.s * d.c;
        static_assert(RN50_K_WGRAD_TILE_LAST - RN50_K_WGRAD_TILE0 + 1 == RN50_NUM_WGRAD_TILES, "one profile id per tile variant");
        ProfScope ps(p.stem ? RN50_K_WGRAD_STEM : RN50_K_WGRAD_TILE0 + p.tile, conv_flops(d, P, Q), bytes, s);
        if (p.strip) wgrad_strip_kernel<<<grid, kThreads, 0, s>>>(a);
        else switch (p.tile) {
            case -1: wgrad_kernel<64, 64, 4, 32, true, 32><<<grid, kThreads, 0, s>>>(a); break;
            case 0: launch_wgrad_tile<0>(a, grid, s); break;
            case 1: launch_wgrad_tile<1>(a, grid, s); break;
            case 2: launch_wgrad_tile<2>(a, grid, s); break;
            case 3: launch_wgrad_tile<3>(a, grid, s); break;
            case 4: launch_wgrad_tile<4>(a, grid, s); break;
            case 5: launch_wgrad_tile<5>(a, grid, s); break;
            case 6: launch_wgrad_tile<6>(a, grid, s); break;
            case 7: launch_wgrad_tile<7>(a, grid, s); break;
            case 8: launch_wgrad_tile<8>(a, grid, s); break;
            default: launch_wgrad_tile<9>(a, grid, s); break;
        }
        RN50_TRY(rn50_check_launch());
    }
    {
        const size_t n4 = a.split_stride / 4;
        const unsigned rgrid = (unsigned)((n4 + 15) / 16);
        ProfScope ps(RN50_K_WGRAD_REDUCE, 0.0, a.split_stride * (4.0 * p.nsplit + (out16 ? 2.0 : 4.0)), s);
        if (out16)
            wgrad_reduce_kernel<true><<<rgrid, kThreads, 0, s>>>(reinterpret_cast<const f32x4*>(partials), out16, n4, p.nsplit, n4);
        else
            wgrad_reduce_kernel<false><<<rgrid, kThreads, 0, s>>>(reinterpret_cast<const f32x4*>(partials), out32, n4, p.nsplit, n4);
        RN50_TRY(rn50_check_launch());
    }
    return RN50_OK;
}

int rn50_stem_unpack_wgrad(const conv_desc& d, const float* acc, h16* out, hipStream_t s)
{
    ProfScope ps(RN50_K_STEM_MISC, 0.0, (double)d.k * (147 * 2 + 256 * 4), s);
    stem_unpack_wgrad_kernel<<<rn50_cdiv(d.k * 147, kThreads), kThreads, 0, s>>>(acc, out, d.k);
    return rn50_check_launch();
}

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
extern "C" size_t conv_workspace_bytes(const conv_desc* d, int which)
{
    if (rn50_conv_validate(d) != RN50_OK) return 0;
    const bool stem = rn50_conv_is_stem(*d);
    switch (which) {
        case RN50_CONV_FWD:
            return stem ? rn50_stem_padded_bytes(*d) + rn50_stem_packed_filter_bytes(*d) : 0;
        case RN50_CONV_DGRAD:
            return stem ? 0 : rn50_round_up((size_t)d->k * d->r * d->s * d->c * sizeof(h16), 256);
        case RN50_CONV_WGRAD: {
            size_t b = rn50_round_up(rn50_wgrad_partial_floats(*d) * sizeof(float), 256);
            if (stem) b += rn50_round_up(rn50_wgrad_acc_floats(*d) * sizeof(float), 256) + rn50_stem_padded_bytes(*d);
            return b;
        }
        default: return 0;
    }
}

static int check_common(const conv_desc* d, const void* p0, const void* p1, const void* p2, void* ws, size_t ws_bytes, int which)
{
    RN50_TRY(rn50_conv_validate(d));
    RN50_REQUIRE_PTR(p0); RN50_REQUIRE_PTR(p1); RN50_REQUIRE_PTR(p2);
    const size_t need = conv_workspace_bytes(d, which);
    if (need > 0 && (!ws || ws_bytes < need)) return RN50_ERR_WORKSPACE;
    RN50_REQUIRE_ALIGNED(p0); RN50_REQUIRE_ALIGNED(p1); RN50_REQUIRE_ALIGNED(p2); RN50_REQUIRE_ALIGNED(ws);
    return RN50_OK;
}

extern "C" int rn50_conv_variant_count(int which)
{
    if (which == RN50_CONV_FWD || which == RN50_CONV_DGRAD) return RN50_NUM_GATHER_TILES;
    return which == RN50_CONV_WGRAD ? RN50_NUM_WGRAD_VARIANTS : 0;
}

// The stand-alone entry points pick a kernel variant by a shape heuristic; the *_variant forms name one
// (a value that is out of range or does not fit the shape leaves the heuristic in charge).
extern "C" int conv_fwd_variant(const conv_desc* d, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, int variant,
                                void* stream)
{
    RN50_TRY(check_common(d, x, w, y, ws, ws_bytes, RN50_CONV_FWD));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (rn50_conv_is_stem(*d)) {
        h16* padded = static_cast<h16*>(ws);
        h16* packed = reinterpret_cast<h16*>(static_cast<char*>(ws) + rn50_stem_padded_bytes(*d));
        RN50_TRY(rn50_stem_pad_image(*d, static_cast<const h16*>(x), padded, s));
        RN50_TRY(rn50_stem_pack_filter(*d, static_cast<const h16*>(w), packed, s));
        return rn50_conv_fwd_launch(*d, padded, packed, static_cast<h16*>(y), s, nullptr, nullptr, variant);
    }
    return rn50_conv_fwd_launch(*d, static_cast<const h16*>(x), static_cast<const h16*>(w), static_cast<h16*>(y), s, nullptr,
                                nullptr, variant);
}

// 1 if the variant id is a kernel of its own for this shape, 0 if the heuristic (forward, data gradient) or a
// fallback tile (filter gradient) would run in its place.
extern "C" int rn50_conv_variant_applies(const conv_desc* d, int which, int variant)
{
    if (!d || rn50_conv_validate(d) != RN50_OK || variant < 0) return 0;
    if (which == RN50_CONV_FWD) {
        if (variant >= RN50_NUM_GATHER_TILES) return 0;
        return rn50_conv_fwd_launch(*d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, variant | RN50_TILE_QUERY) == RN50_OK;
    }
    if (which == RN50_CONV_DGRAD) {
        if (variant >= RN50_NUM_GATHER_TILES || rn50_conv_is_stem(*d)) return 0;
        return rn50_conv_dgrad_launch(*d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, variant | RN50_TILE_QUERY) ==
               RN50_OK;
    }
    if (which == RN50_CONV_WGRAD) return variant < RN50_NUM_WGRAD_VARIANTS && rn50_wgrad_canonical_variant(*d, variant) == variant;
    return 0;
}

extern "C" int conv_fwd(const conv_desc* d, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, void* stream)
{
    return conv_fwd_variant(d, x, w, y, ws, ws_bytes, RN50_TILE_AUTO, stream);
}

extern "C" int conv_dgrad_variant(const conv_desc* d, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes,
                                  int variant, void* stream)
{
    RN50_TRY(rn50_conv_validate(d));
    if (rn50_conv_is_stem(*d)) return RN50_ERR_SHAPE;   // the images need no gradient
    RN50_TRY(check_common(d, dy, w, dx, ws, ws_bytes, RN50_CONV_DGRAD));
    hipStream_t s = static_cast<hipStream_t>(stream);
    h16* wt = static_cast<h16*>(ws);
    RN50_TRY(rn50_transpose_filter(*d, static_cast<const h16*>(w), wt, s));
    return rn50_conv_dgrad_launch(*d, static_cast<const h16*>(dy), wt, nullptr, static_cast<h16*>(dx), s, nullptr, nullptr,
                                  variant);
}

extern "C" int conv_dgrad(const conv_desc* d, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes, void* stream)
{
    return conv_dgrad_variant(d, dy, w, dx, ws, ws_bytes, RN50_TILE_AUTO, stream);
}

extern "C" int conv_wgrad_variant(const conv_desc* d, const void* x, const void* dy, void* dw, void* ws, size_t ws_bytes,
                                  int variant, void* stream)
{
    RN50_TRY(check_common(d, x, dy, dw, ws, ws_bytes, RN50_CONV_WGRAD));
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* partials = static_cast<float*>(ws);
    char* p = static_cast<char*>(ws) + rn50_round_up(rn50_wgrad_partial_floats(*d) * sizeof(float), 256);
    if (rn50_conv_is_stem(*d)) {
        float* acc = reinterpret_cast<float*>(p);
        h16* padded = reinterpret_cast<h16*>(p + rn50_round_up(rn50_wgrad_acc_floats(*d) * sizeof(float), 256));
        RN50_TRY(rn50_stem_pad_image(*d, static_cast<const h16*>(x), padded, s));
        RN50_TRY(rn50_conv_wgrad_launch(*d, padded, static_cast<const h16*>(dy), nullptr, acc, partials, s, RN50_TILE_AUTO));
        return rn50_stem_unpack_wgrad(*d, acc, static_cast<h16*>(dw), s);
    }
    return rn50_conv_wgrad_launch(*d, static_cast<const h16*>(x), static_cast<const h16*>(dy), static_cast<h16*>(dw), nullptr,
                                  partials, s, (variant >= 0 && variant < RN50_NUM_WGRAD_VARIANTS) ? variant : RN50_TILE_AUTO);
}

extern "C" int conv_wgrad(const conv_desc* d, const void* x, const void* dy, void* dw, void* ws, size_t ws_bytes, void* stream)
{
    return conv_wgrad_variant(d, x, dy, dw, ws, ws_bytes, RN50_TILE_AUTO, stream);
}
