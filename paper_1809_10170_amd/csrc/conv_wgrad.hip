// Weight gradient of the convolution layer for gfx950 (MI355X), fp32 MFMA, no workspace.
//
//   dw[k][c][r][s] = sum over n, p, q of  dy[n][k][p][q] * x[n][c][p*stride + r - pad][q*stride + s - pad]
//
// (taps outside the image contribute nothing).  The paper names the backward pass with
// respect to the filter as a direction (closing section) and gives no algorithm; this is
// the same direct scheme turned around: a dense contraction whose reduction runs over the
// output pixels, computed from the plain tensors with the input window of a row of
// pixels staged in LDS, so that the S taps of a filter row read it at S constant offsets
// and no lowered copy of x exists.
//
// v_mfma_f32_32x32x2_f32 with rows = output channels k (A = dy), columns = input channels
// c (B = x), the two k-lanes = two neighbouring output pixels.  One wave owns the 32 x 32
// results of one k-block for CBW channel blocks and the S taps of ONE filter row r:
// CBW*S accumulator blocks.  A workgroup of WK waves (32*WK output channels) walks over
// chunks of PXC consecutive pixels of one output row: per chunk it stages dy[32*WK][PXC]
// and x[32*CBW][(PXC-1)*ST + S] (input row p*ST + r - pad) into LDS with LDS-direct loads
// (out-of-range pixels read zeros), double-buffered: the loads of chunk i+1 are in flight
// while chunk i multiplies.
//
// The reduction over all N*P*Q pixels is split over `splits` workgroups per result tile
// (each takes every splits-th image) so that the grid fills the chip; their partial sums
// meet in dw itself by fp32 atomic adds (dw is cleared by a fill kernel first).  No
// workspace, but the order of those additions, and with it the last bits, varies.  With
// splits = 1 (the deterministic plans) a result tile has one workgroup, which stores it
// plainly: no fill, no atomics, the same bits every run.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "conv_dma_kernel.h"   // CONVD_LDS, uniform_ptr, vector types
#include "wgrad.h"

namespace convd {

//
// PACK > 0 (layers with very few input channels, C*S <= 32*PACK): the MFMA columns are the
// (input channel, filter column) pairs c*S + s packed into PACK blocks of 32, instead of 32
// channels per block and one block per filter column; with C = 3 that fills 21 of 32 columns
// (S = 7) instead of 3.
//
// QW > 0 (small maps whose output rows are QW pixels wide, QW fixed at compile time): a chunk
// is RPC = PXC / QW whole output rows instead of a piece of one, so that a 13-pixel row does
// not leave 19 of 32 pixel slots empty.  The dy pixels of such a chunk are still one
// contiguous run; the input rows they need sit in LDS one after the other, 32 words apart.
//
// S = 0: the fallback for any filter width and any stride up to ST (which then only sizes the LDS):
// the filter column becomes one more grid dimension, a wave owns CBW blocks of one tap, and the
// stride is read at run time.
//
// AR = 1 (square filters, stride 1): a wave owns ALL S*S taps of 32*CBW input channels instead of the S
// taps of one filter row, and the MFMA columns are the flattened (channel, tap) indices c*S*S + r*S + s
// in blocks of 32.  The filter row is then no grid dimension: a chunk stages the S input rows its output
// row needs (dy is staged once for all of them), and, above all, the 32 lanes of an accumulator row hold
// 32 CONSECUTIVE floats of dw[k][.][.][.], so that a wave's atomic additions cover two 128-byte lines
// instead of some twenty.  In LDS an input row is RP words and a channel S*RP words with RP = S (mod 32):
// the 32 columns of a block then read 32 different banks.
//
// WC > 1: the waves of a workgroup also spread over WC groups of 32*CBW input channels (wave = k-block +
// WK * channel group), which all read the same staged dy: a tile of 32*WK output x 32*CBW*WC input
// channels whose accumulators are shared out over WK*WC waves.
//
// WB > 1 (all-rows mode): the column blocks of the workgroup's channels are dealt out to WB waves per
// k-block (block wb, wb + WB, ...), for filters whose S*S taps times 32 channels are more blocks than one
// wave can hold (25 for 5x5).  A wave whose last block does not exist computes it on any valid operands
// and drops it.
template <int S_, int ST_, int CBW_, int WK_, int PXC_, int PACK_ = 0, int QW_ = 0, int AR_ = 0, int WC_ = 1, int WB_ = 1>
struct WgGeom {
    static constexpr int S = S_, ST = ST_, CBW = CBW_, WK = WK_, PXC = PXC_, PACK = PACK_, QW = QW_, AR = AR_, WC = WC_, WB = WB_;
    static constexpr int NW = WK_ * WC_ * WB_;           // waves per workgroup
    static constexpr bool RT = S_ == 0;
    static constexpr int SB = RT ? 1 : S_;               // filter columns a wave owns
    static constexpr int NR = AR ? S_ : 1;               // filter rows a wave owns
    static constexpr int NCOLB = PACK ? PACK : CBW * SB * NR; // column blocks of the wave's channels
    static constexpr int NBLK = (NCOLB + WB - 1) / WB;        // accumulator blocks per wave
    static constexpr int RPC = QW ? PXC / QW : 1;        // output rows per chunk
    static constexpr int NPX = QW ? RPC * QW : PXC;      // pixels per chunk
    static constexpr int PXR = AR_ ? 32 + S_ : 32;       // QW: LDS words from one input row to the next (all-rows mode: = S mod 32)
    static constexpr int XROWS = QW ? RPC + NR - 1 : NR; // input rows a chunk stages per channel
    static constexpr int NT = 64 * NW;
    static constexpr int KT = 32 * WK;                    // output channels per workgroup
    static constexpr int CT = (PACK && AR) ? 4 : 32 * CBW * WC;   // input channels per workgroup (packed all-rows mode:
                                                          // the C <= 4 channels of a first layer)
    // LDS pitch of a dy row: odd, so that the 32 rows one half-wave reads at the same pixel fall into
    // 32 different banks.  A 32-pixel chunk is staged by the first 32 lanes only, so that two
    // workgroups fit the LDS of a CU.
    static constexpr int PA = PXC <= 32 ? 33 : 65;
    static constexpr bool HALF_A = PA == 33;
    // chunks of at most 31 pixels: one 64-lane load stages TWO dy rows (lanes 0.. the first, lanes 33.. the second,
    // which starts 33 words on; the lanes between and behind load zeros into words no one reads)
    static constexpr bool DUAL_A = HALF_A && (QW_ ? (PXC_ / QW_) * QW_ : PXC_) <= 31 && (32 * WK_ / (WK_ * WC_ * WB_)) % 2 == 0;
    static constexpr int WX = ((QW ? QW : PXC) - 1) * ST + SB;  // input columns a chunk needs (fallback: at most)
    static_assert(!RT || (PACK == 0 && QW == 0), "the fallback uses plain row chunks");
    static constexpr int NLX = (WX + 63) / 64;            // 64-lane loads per input channel (row chunks)
    static constexpr int RP = WX + ((S_ - WX) % 32 + 32) % 32;     // AR: LDS pitch of an input row, = S (mod 32)
    // LDS pitch of an input channel: odd (32 channels, 32 banks); all-rows mode: = S*S (mod 32), like the columns
    static constexpr int PX = AR ? (QW ? XROWS * PXR + ((NR * S_ - XROWS * PXR) % 32 + 32) % 32 : NR * RP)
                                 : QW ? RPC * PXR + 1 : NLX * 64 + 1;
    static_assert(!AR || (!RT && (QW == 0 || (ST == 1 && PACK == 0))), "all-rows mode: small-map chunks at stride 1, unpacked");
    static_assert(WC == 1 || (PACK == 0 && 32 % WC == 0), "channel groups of waves: whole dy rows per wave");
    static_assert(WB == 1 || (AR && WC == 1 && 32 % WB == 0), "column blocks dealt out to waves: all-rows mode");
    static_assert(!QW || (WX <= PXR && RPC >= 1 && PACK == 0), "small-map chunks: an input row fits 32 words");
    // small-map chunks: one 64-lane load stages TWO input rows of a channel (the second starts PXR words on)
    static constexpr bool DUAL_X = QW_ != 0 && XROWS % 2 == 0 && WX + PXR <= 64;
    // All-rows variants stage without lane masks: every load writes 64 consecutive LDS words, and what a load writes
    // past its own row (zeros) lands in the row after it, which the SAME wave loads next (a wave's loads reach LDS in
    // the order they were issued).  So a wave stages consecutive dy rows and consecutive input channels, in rising
    // address order, and behind each wave's block lies a slack no one reads.
    static constexpr int RPWV = KT / NW > 0 ? KT / NW : 1;     // dy rows a wave stages
    static constexpr int CPWV = CT / NW > 0 ? CT / NW : 1;     // input channels a wave stages (packed first layers: one of CT <= NW)
    static constexpr int ASL = (AR && HALF_A && !DUAL_A) ? 32 : 0;   // slack (floats) behind a wave's dy rows
    static constexpr int XSL = AR ? 64 : 0;                           // ... behind a wave's input channels
    static constexpr int ABUF = KT * PA + NW * ASL, XBUF = CT * PX + NW * XSL;  // floats
    static constexpr int BUF = ABUF + XBUF;
    static constexpr size_t LDS_BYTES = sizeof(float) * (2 * (size_t)BUF + 64);   // (+ slack: an odd last pixel pair reads
                                                                                  // a few words past the last input row)
    static_assert(PXC <= 64 && PXC % 2 == 0, "a dy row segment is staged by one 64-lane load");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
    // workgroups per CU the kernel is sized for: two if their LDS fits and they are at most four waves each
    static constexpr int PER_CU = (LDS_BYTES <= 80 * 1024 && NW <= 4) ? 2 : 1;
    static constexpr int WPE = PER_CU * NW >= 4 ? PER_CU * NW / 4 : 1;   // waves per SIMD the register budget must allow
};

// element (k, c, tap) of dw in the blocked weight layout [K/32][C/4][R][S][4][32] (RS taps per channel pair)
__device__ inline size_t dw_blocked_index(int k, int c, int tap, int C, int RS)
{
    return ((((size_t)(k >> 5) * ((C + 3) / 4) + (c >> 2)) * RS + tap) * 4 + (c & 3)) * 32 + (k & 31);
}

template <class G>
__global__ void __launch_bounds__(G::NT, G::WPE) conv_wgrad_kernel(const WgradArgs a)
{
    extern __shared__ __align__(16) float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    __builtin_assume(wave >= 0 && wave < G::NW);
    const int wk = wave % G::WK, wc = (wave / G::WK) % G::WC, wb = wave / (G::WK * G::WC);   // k-block, channel group, first column block
    const int h = lane >> 5, j = lane & 31;
    const int N = a.s.N, C = a.s.C, H = a.s.H, W = a.s.W, K = a.s.K, R = a.s.R, P = a.s.P, Q = a.s.Q, pad = a.s.pad;
    const int st = G::RT ? a.s.stride : G::ST;       // (a compile-time constant except in the fallback)
    // (scalars, not the argument struct, go into the lambdas below: a struct captured by reference
    // ends up in private memory)
    const float *const xp = a.x, *const dyp = a.dy;
    float *const dwp = a.dw;
    const int splits = a.splits, cgroups = a.cgroups, ktiles = a.ktiles, SFILT = a.s.S;
    // Layouts (run-time flags; the staging transposes either into the same LDS arrays).  Blocked activations
    // [N][channels/4][rows][cols][4]: a pixel step is 4 floats, a channel step inside a group of 4 one float, and a
    // step of 4 channels 4 planes -- the same as in the plain layout.
    const int xbl = a.x_blocked, ybl = a.dy_blocked, wbl = a.dw_blocked;
    const int CI = xbl ? (C + 3) / 4 * 4 : C, KI = ybl ? (K + 3) / 4 * 4 : K;   // channels an image occupies in memory
    const int xpx = xbl ? 4 : 1, ypx = ybl ? 4 : 1;                             // floats from one pixel to the next
    const int plane_dy = P * Q * 4, plane_x = H * W * 4;                        // bytes of a channel plane (plain layout)
    const int y_c1 = ybl ? 4 : plane_dy, x_c1 = xbl ? 4 : plane_x;              // bytes from a channel to the next (inside a group of 4)
    // byte offset of channel ch, counted from a channel that is a multiple of 4 (k0, c0)
    auto ych = [&](int ch) { return (ch >> 2) * (4 * plane_dy) + (ch & 3) * y_c1; };
    auto xch = [&](int ch) { return (ch >> 2) * (4 * plane_x) + (ch & 3) * x_c1; };

    // workgroup -> (pixel split, filter row, channel group, k tile); neighbours share dy
    // (consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2: regroup
    // them so that the workgroups that read the same dy rows run on one XCD)
    unsigned bid = blockIdx.x;
    {
        const unsigned g8 = gridDim.x & ~7u;
        if (bid < g8) bid = (bid & 7u) * (g8 >> 3) + (bid >> 3);
    }
    int s0 = 0;                                      // fallback: the filter column of this workgroup
    if (G::RT) { s0 = bid % SFILT;  bid /= SFILT; }
    const int cg = bid % cgroups;  bid /= cgroups;
    int r = 0;                                       // (all-rows mode: no such grid dimension)
    if (!G::AR) { r = bid % R;  bid /= R; }
    const int kt = bid % ktiles;
    const int ps = bid / ktiles;
    const int k0 = kt * G::KT, c0 = cg * G::CT;

    // The reduction runs over output rows u = n*P + p of all images; this workgroup takes rows
    // ps, ps + splits, ...  A chunk: image n, output row p, first column q0.
    // (small-map chunks: the unit is a group of RPC output rows, p its first row, one chunk per unit)
    const int PG = G::QW ? (P + G::RPC - 1) / G::RPC : P;   // units per image
    const int rows_all = N * PG;
    int u = ps, n = 0, p = 0, q0 = 0;
    // the slack behind the second buffer is read (times a zero of dy) when a chunk has an odd number of pixels
    if (threadIdx.x < 64) lds[2 * G::BUF + threadIdx.x] = 0.f;
    auto settle = [&]() __attribute__((always_inline)) {   // move u forward to the next unit of this split (row chunks: whose input row exists)
        for (; u < rows_all; u += splits) {
            n = u / PG;
            p = (u - n * PG) * G::RPC;
            if (G::QW || G::AR || (unsigned)(p * st + r - pad) < (unsigned)H) break;
        }
        if (u >= rows_all) n = N;
    };
    // (all-rows variants take every unit: the step from one unit of this split to the next is the same every time and
    // needs no division)
    const int step_n = splits / PG, step_g = splits - step_n * PG;
    int ug = 0;                                              // the unit's index within its image (all-rows variants)
    auto advance = [&]() __attribute__((always_inline)) {
        q0 += G::PXC;
        if (G::QW || q0 >= Q) {
            q0 = 0;
            u += splits;
            if constexpr (G::AR != 0) {
                ug += step_g;
                n += step_n;
                if (ug >= PG) { ug -= PG; ++n; }
                p = ug * G::RPC;
                if (u >= rows_all) n = N;
            } else {
                settle();
            }
        }
    };
    settle();
    if (G::AR) ug = u - n * PG;

    // Stage the chunk (n, p, q0) into buffer b: dy rows wave, wave+WK, ... and input
    // channels likewise; lanes past the row's end or outside the image load zeros; rows
    // of output channels >= K and input channels >= C are skipped (they feed results
    // that are never written).
    auto stage = [&](int b, int sn, int sp, int sq0) __attribute__((always_inline)) {
        float *abuf = lds + b * G::BUF, *xbuf = abuf + G::ABUF;
        {
            // pixels of the chunk that exist: the rest of the row, or whole rows down to the image's last
            const int npix = G::QW ? (P - sp < G::RPC ? P - sp : G::RPC) * G::QW : Q - sq0;
            const unsigned voff = lane < npix ? (unsigned)(lane * ypx) * 4u : 0x80000000u;
            const float *base = dyp + ((size_t)sn * KI + k0) * P * Q + (size_t)(sp * Q + sq0) * ypx;
            __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(base), 0, 0x7fffffff, 0x00020000);
            if constexpr (G::DUAL_A) {
                const int l2 = lane - G::PA;                      // lane's pixel in the second row of its pair
                const int np = npix < G::NPX ? npix : G::NPX;     // (the rest of a long row is more than a chunk)
                const unsigned voff2 = lane < np ? (unsigned)(lane * ypx) * 4u
                                       : (l2 >= 0 && l2 < np) ? (unsigned)y_c1 + (unsigned)(l2 * ypx) * 4u : 0x80000000u;   // (the pair's second row: an odd channel)
#pragma unroll
                for (int i = 0; i < G::KT / G::NW / 2; ++i) {
                    const int row = (i * G::NW + wave) * 2;
                    if (k0 + row < K)   // (a second row past K is not loaded: the single-row offsets)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, CONVD_LDS(abuf + row * G::PA), 4,
                                                                 k0 + row + 1 < K ? voff2 : voff, ych(row), 0, 0);
                }
            } else if (!G::HALF_A || lane < 32) {   // (a disabled lane writes nothing: rows 33 words apart do not overlap)
#pragma unroll
                for (int i = 0; i < G::KT / G::NW; ++i) {
                    const int row = i * G::NW + wave;
                    if (k0 + row < K)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, CONVD_LDS(abuf + row * G::PA), 4, voff, ych(row), 0, 0);
                }
            }
        }
        if constexpr (G::QW != 0) {
            // RPC input rows per channel, 32 words apart: only the first 32 lanes take part in a load
            // (a disabled lane writes nothing), lanes past the row's columns or outside the image load zeros
            const float *base = xp + ((size_t)sn * CI + c0) * H * W;
            __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(base), 0, 0x7fffffff, 0x00020000);
            const int iw = lane - pad;
            const bool colok = lane < G::WX && (unsigned)iw < (unsigned)W;
            if constexpr (G::DUAL_X) {
                const int l2 = lane - G::PXR, iw2 = l2 - pad;      // the lane's column in the second row of a pair
                const bool colok2 = l2 >= 0 && l2 < G::WX && (unsigned)iw2 < (unsigned)W;
#pragma unroll
                for (int i = 0; i < G::CT / G::NW; ++i) {
                    const int ch = i * G::NW + wave;
                    if (c0 + ch < C) {
#pragma unroll
                        for (int ri = 0; ri < G::XROWS; ri += 2) {
                            const int ih0 = (sp + ri) * G::ST + r - pad, ih1 = ih0 + G::ST;
                            const bool ok0 = (unsigned)ih0 < (unsigned)H, ok1 = (unsigned)ih1 < (unsigned)H;
                            const unsigned voff = (colok && ok0)    ? (unsigned)((ih0 * W + iw) * xpx) * 4u
                                                  : (colok2 && ok1) ? (unsigned)((ih1 * W + iw2) * xpx) * 4u
                                                                    : 0x80000000u;
                            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, CONVD_LDS(xbuf + ch * G::PX + ri * G::PXR), 4, voff,
                                                                     xch(ch), 0, 0);
                        }
                    }
                }
            } else if (lane < G::PXR) {
#pragma unroll
                for (int i = 0; i < G::CT / G::NW; ++i) {
                    const int ch = i * G::NW + wave;
                    if (c0 + ch < C) {
#pragma unroll
                        for (int ri = 0; ri < G::XROWS; ++ri) {   // (all-rows mode: the halo rows of all taps too)
                            const int ih = (sp + ri) * G::ST + r - pad;
                            const bool rowok = (unsigned)ih < (unsigned)H;
                            const unsigned voff = (colok && rowok) ? (unsigned)(iw * xpx) * 4u : 0x80000000u;
                            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, CONVD_LDS(xbuf + ch * G::PX + ri * G::PXR), 4, voff,
                                                                     xch(ch) + (rowok ? ih : 0) * W * xpx * 4, 0, 0);
                        }
                    }
                }
            }
        } else {
            const int ih = sp * st + r - pad;              // exists (the chunk list skips rows without one)
            const int iw0 = sq0 * st - pad + s0;
            const int wx = (G::PXC - 1) * st + G::SB;      // columns the chunk needs
            const float *base = xp + ((size_t)sn * CI + c0) * H * W + (size_t)ih * W * xpx;
            __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(base), 0, 0x7fffffff, 0x00020000);
            unsigned voff[G::NLX];
#pragma unroll
            for (int u = 0; u < G::NLX; ++u) {
                const int col = u * 64 + lane, iw = iw0 + col;
                voff[u] = (col < wx && (unsigned)iw < (unsigned)W) ? (unsigned)(iw * xpx) * 4u : 0x80000000u;
            }
#pragma unroll
            for (int i = 0; i < G::CT / G::NW; ++i) {
                const int ch = i * G::NW + wave;
                if (c0 + ch < C) {
#pragma unroll
                    for (int u = 0; u < G::NLX; ++u)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, CONVD_LDS(xbuf + ch * G::PX + u * 64), 4, voff[u],
                                                                 xch(ch), 0, 0);
                }
            }
        }
    };

    // ---- all-rows variants: staging without vector ALU work per load, metered into the MFMA loop ----
    // A wave that stages shares its SIMD with a wave that multiplies (or with its own MFMAs), and the
    // address work of a chunk's 30-odd loads, done in one block behind the barrier, kept the matrix pipe
    // waiting for a sixth of the time.  Here everything that differs from load to load is a scalar:
    //   * a buffer resource that ends where the image's last channel ends, so that rows of output channels
    //     >= K and input channels >= C read zeros (the range check covers the scalar offset too);
    //   * for an input row outside the image, a scalar offset as large as the resource, which puts the whole load out of range;
    //   * per-lane offsets that depend on the chunk only through its column position (recomputed once per
    //     chunk: a handful of instructions) or not at all.
    // and the loads of the next chunk are issued a few at a time between the MFMAs of this one.
    struct ArSrc {
        __amdgpu_buffer_rsrc_t ra, rx;          // dy, input
        unsigned va;                            // dy: the lane's offset in its row (pair)
        unsigned vx[G::NLX > 0 ? G::NLX : 1];   // input, row chunks: the lane's column
        unsigned sx[G::XROWS];                  // input: scalar offset of each staged row from the resource's base; for a
                                                // row outside the image the resource's size, which sends the load out of range
        unsigned vd[G::XROWS / 2 > 0 ? G::XROWS / 2 : 1];   // small maps, two rows per load: the lane's offset per row pair
    };
    // per-lane constants of the dy loads: the lane's pixel, full chunk / ragged last chunk of a row or image
    auto dy_voff = [&](int np) -> unsigned {
        if (G::DUAL_A) {
            const int l2 = lane - G::PA;
            return lane < np ? (unsigned)(lane * ypx) * 4u : (l2 >= 0 && l2 < np) ? (unsigned)y_c1 + (unsigned)(l2 * ypx) * 4u : 0x80000000u;
        }
        return lane < np ? (unsigned)(lane * ypx) * 4u : 0x80000000u;
    };
    const int np_rag = G::QW ? (P % G::RPC) * G::QW : Q % G::PXC;       // pixels of a ragged last chunk (0: there is none)
    const unsigned va_full = dy_voff(G::NPX), va_rag = dy_voff(np_rag);
    // small maps: per-lane parts of a load of two input rows (the second starts PXR words on)
    unsigned vd_both = 0x80000000u, vd_first = 0x80000000u, vd_second = 0x80000000u;
    if (G::QW != 0) {
        const int iw = lane - pad, l2 = lane - G::PXR, iw2 = l2 - pad;
        const bool c1 = lane < G::WX && lane < G::PXR && (unsigned)iw < (unsigned)W;
        const bool c2 = l2 >= 0 && l2 < G::WX && (unsigned)iw2 < (unsigned)W;
        vd_first = c1 ? (unsigned)(iw * xpx) * 4u : 0x80000000u;
        vd_second = (G::DUAL_X && c2) ? (unsigned)((G::ST * W + iw2) * xpx) * 4u : 0x80000000u;
        vd_both = c1 ? vd_first : vd_second;
    }
    // (offsets inside one image fit 31 bits: conv_direct_create_wgrad refuses layers whose K*P*Q*4 or C*H*W*4 does not)
    const int img_dy = (KI - k0) * P * Q, img_x = (CI - c0) * H * W;   // floats from the workgroup's first channel to the image's end
    auto ar_source = [&](ArSrc &src, int sn, int sp, int sq0, bool more) __attribute__((always_inline)) {
        // dy: from (sn, k0, sp, sq0) to the end of the image's last channel
        const int a_in = (sp * Q + sq0) * ypx;
        src.ra = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(dyp + ((size_t)sn * KI + k0) * P * Q + a_in), 0, more ? (img_dy - a_in) * 4 : 0,
                                                   0x00020000);
        const int npix = G::QW ? (P - sp < G::RPC ? P - sp : G::RPC) * G::QW : Q - sq0;
        src.va = npix >= G::NPX ? va_full : va_rag;
        // input: from row ih0 (possibly above the image), column iw0 (row chunks: possibly left of it: the lanes there are
        // sent out of range) of channel c0, to the end of the image's last channel
        const int ih0 = sp * G::ST - pad, iw0 = G::QW ? 0 : sq0 * G::ST - pad;
        const int x_in = (ih0 * W + iw0) * xpx;                            // (may be negative)
        const unsigned nrx = more ? (unsigned)(img_x - x_in) * 4u : 0u;
        src.rx = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(xp + ((long long)sn * CI + c0) * H * W + x_in), 0, (int)nrx, 0x00020000);
        bool okx[G::XROWS];
#pragma unroll
        for (int ri = 0; ri < G::XROWS; ++ri) {
            const int ih = ih0 + ri * (G::QW ? G::ST : 1);
            okx[ri] = (unsigned)ih < (unsigned)H;
            src.sx[ri] = (okx[ri] || (G::QW && G::DUAL_X)) ? (unsigned)(ih - ih0) * (unsigned)(W * xpx) * 4u : nrx;
        }
        if (G::QW == 0) {
#pragma unroll
            for (int u = 0; u < G::NLX; ++u) {
                const int col = u * 64 + lane, iw = iw0 + col;
                src.vx[u] = (col < G::WX && (unsigned)iw < (unsigned)W) ? (unsigned)(col * xpx) * 4u : 0x80000000u;
            }
        } else if (G::DUAL_X) {
#pragma unroll
            for (int rp = 0; rp < G::XROWS / 2; ++rp) {
                const bool o0 = okx[2 * rp], o1 = okx[2 * rp + 1];
                src.vd[rp] = (o0 && o1) ? vd_both : o0 ? vd_first : o1 ? vd_second : 0x80000000u;
            }
        }
    };
    // loads number [PART * NL / NPARTS, (PART + 1) * NL / NPARTS) of the NL loads of a chunk, into buffer b
    constexpr int AR_NA = G::DUAL_A ? G::KT / G::NW / 2 : G::KT / G::NW;                 // dy loads of a wave
    constexpr int AR_XR = G::QW ? (G::DUAL_X ? G::XROWS / 2 : G::XROWS) : G::NR * (G::NLX > 0 ? G::NLX : 1);   // input loads per channel
    constexpr int AR_NX = (G::CT / G::NW > 0 ? G::CT / G::NW : 1) * AR_XR;
    constexpr int AR_NL = AR_NA + AR_NX;
    auto ar_stage = [&](auto part_tag, auto nparts_tag, int b, const ArSrc &src) __attribute__((always_inline)) {
        constexpr int PART = decltype(part_tag)::value, NPARTS = decltype(nparts_tag)::value;
        constexpr int L0 = PART * AR_NL / NPARTS, L1 = (PART + 1) * AR_NL / NPARTS;
        float *abuf = lds + b * G::BUF + wave * G::ASL, *xbuf = lds + b * G::BUF + G::ABUF + wave * G::XSL;
        // (no lane is masked: see the note on the slack in the geometry)
#pragma unroll
        for (int i = 0; i < AR_NA; ++i)
            if (i >= L0 && i < L1) {
                const int row = (wave * AR_NA + i) * (G::DUAL_A ? 2 : 1);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(src.ra, CONVD_LDS(abuf + row * G::PA), 4, src.va, ych(row), 0, 0);
            }
#pragma unroll
        for (int i = 0; i < G::CPWV; ++i) {
            const int ch = wave * G::CPWV + i;
#pragma unroll
            for (int xr = 0; xr < AR_XR; ++xr) {
                const int li = AR_NA + i * AR_XR + xr;
                if (li >= L0 && li < L1 && (G::CT >= G::NW || ch < G::CT)) {
                    if (G::QW == 0) {
                        const int ri = xr / (G::NLX > 0 ? G::NLX : 1), u = xr % (G::NLX > 0 ? G::NLX : 1);
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(src.rx, CONVD_LDS(xbuf + ch * G::PX + ri * G::RP + u * 64), 4, src.vx[u],
                                                                 xch(ch) + src.sx[ri], 0, 0);
                    } else if (G::DUAL_X) {
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(src.rx, CONVD_LDS(xbuf + ch * G::PX + 2 * xr * G::PXR), 4, src.vd[xr],
                                                                 xch(ch) + src.sx[2 * xr], 0, 0);
                    } else {
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(src.rx, CONVD_LDS(xbuf + ch * G::PX + xr * G::PXR), 4, vd_first,
                                                                 xch(ch) + src.sx[xr], 0, 0);
                    }
                }
            }
        }
    };

    dma_floatx16 acc[G::NBLK];
#pragma unroll
    for (int b = 0; b < G::NBLK; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

    // LDS addresses are one register plus an immediate: the buffer's base goes into the per-lane
    // registers (one set per buffer, the chunk loop is unrolled over the two buffers), the step's
    // part into the immediate -- no vector ALU work per fetch, which a wave between its own MFMAs
    // would wait some 20 clocks for each time.
    // lane (k = j, pixel parity h; small maps, all-rows variants: pixel half h); the slack behind the rows of the waves before
    const int aoff = (wk * 32 + j) * G::PA + h * ((G::QW != 0 && G::AR != 0) ? (G::NPX + 1) / 2 : 1) + ((wk * 32 + j) / G::RPWV) * G::ASL;
    // LDS offset of the lane's B operand of block b at pixel pair 0: column j of the block is input
    // channel cb*32 + j at filter column s (b = cb*S + s), or the packed pair (c, s) = divmod(b*32 + j, S)
    int xoff[G::NBLK];
#pragma unroll
    for (int b = 0; b < G::NBLK; ++b) {
        if (G::PACK && !G::AR) {
            const int col = b * 32 + j < C * G::S ? b * 32 + j : 0;   // (columns past C*S: any valid position, discarded)
            xoff[b] = (col / G::S) * G::PX + col % G::S + h * G::ST;
        } else if (G::AR) {
            constexpr int SS = G::SB * G::NR;                         // taps per channel
            // (packed: the columns are all C*S*S (channel, tap) pairs; those past them read any valid position)
            const int colb = (wb + G::WB * b) * 32 + j;               // (blocks dealt out to WB waves)
            const int col = ((!G::PACK || colb < C * SS) && colb < G::NCOLB * 32) ? colb : 0, tap = col % SS;
            const int chn = wc * 32 * G::CBW + col / SS;             // channel of the workgroup's CT
            xoff[b] = chn * G::PX + (chn / G::CPWV) * G::XSL + (tap / G::SB) * (G::QW ? G::PXR : G::RP) + tap % G::SB +
                      (G::QW ? h * (((G::NPX + 1) / 2) / (G::QW ? G::QW : 1)) * G::PXR : h * G::ST);   // (small maps: the lane's half of the rows)
        } else {
            xoff[b] = ((wc * G::CBW + b / G::SB) * 32 + j) * G::PX + b % G::SB + (G::QW ? 0 : h * st);
        }
    }

    int aoffB[2], xoffB[2][G::NBLK];
#pragma unroll
    for (int bf = 0; bf < 2; ++bf) {
        aoffB[bf] = bf * G::BUF + aoff;
#pragma unroll
        for (int bb = 0; bb < G::NBLK; ++bb) xoffB[bf][bb] = bf * G::BUF + G::ABUF + xoff[bb];
    }
    constexpr int NST = (G::NPX + 1) / 2;
    // Small maps, all-rows variants: the two k-lanes of step t take pixels t and t + NST of the chunk (not 2t and
    // 2t + 1): with whole rows in each half (NST a multiple of QW) the second pixel lies a constant number of LDS
    // rows below the first, so the lane's half is part of its base address and a step adds a compile-time constant.
    constexpr bool HALVES = G::QW != 0 && G::AR != 0;
    static_assert(!HALVES || (NST % (G::QW ? G::QW : 1) == 0 && G::NPX % 2 == 0), "small-map chunks: an even number of whole rows");
    auto pix_off = [&](int t) {
        // LDS offset of the step's two pixels: along the row, or (small maps) row and column of
        // pixels 2t and 2t+1 of the chunk, the lane's one picked by its pixel parity
        if (HALVES) {
            constexpr int QWc = G::QW ? G::QW : 1;
            return (t / QWc) * G::PXR + (t % QWc) * G::ST;
        }
        if (G::QW) {
            constexpr int QWc = G::QW ? G::QW : 1;
            const int o0 = (2 * t / QWc) * G::PXR + (2 * t % QWc) * G::ST;
            const int o1 = ((2 * t + 1) / QWc) * G::PXR + ((2 * t + 1) % QWc) * G::ST;
            return h ? o1 : o0;
        }
        return 2 * t * st;
    };
    // one chunk out of buffer bf, whose per-lane LDS offsets are aoffc and xoffc: meet, send the next
    // chunk's loads, multiply
    auto chunk_body = [&](int bf, int aoffc, const int (&xoffc)[G::NBLK]) __attribute__((always_inline)) {
        advance();                                            // (n, p, q0) is now the next chunk
        wait_vmem_done();  // this wave's loads of chunk bf (the only ones in flight) have landed
        __syncthreads();   // chunk bf is complete and every wave has left the other buffer
        if (n < N) stage(bf ^ 1, n, p, q0);
        // operands of step t+1 are fetched from LDS while step t multiplies
        float an = lds[aoffc], bn[G::NBLK];
        {
            const int po = pix_off(0);
#pragma unroll
            for (int bb = 0; bb < G::NBLK; ++bb) bn[bb] = lds[xoffc[bb] + po];
        }
#pragma unroll
        for (int t = 0; t < NST; ++t) {
            const float av = an;
            float bv[G::NBLK];
#pragma unroll
            for (int bb = 0; bb < G::NBLK; ++bb) bv[bb] = bn[bb];
            if (t + 1 < NST) {
                an = lds[aoffc + 2 * (t + 1)];
                const int po = pix_off(t + 1);
#pragma unroll
                for (int bb = 0; bb < G::NBLK; ++bb) bn[bb] = lds[xoffc[bb] + po];
            }
#pragma unroll
            for (int bb = 0; bb < G::NBLK; ++bb)
                acc[bb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[bb], acc[bb], 0, 0, 0);
        }
    };
    if constexpr (G::AR != 0) {
        // One loop body for both buffers (the buffer's base is added to the per-lane offsets once per
        // chunk): with nine accumulator blocks a loop unrolled over the two buffers, whose second half
        // can be left early, costs a second set of accumulator registers.
        {
            ArSrc src;
            ar_source(src, n, p, q0, n < N);
            ar_stage(IntTag<0>{}, IntTag<1>{}, 0, src);
        }
        int bf = 0;
        while (n < N) {
            int xoffc[G::NBLK];
#pragma unroll
            for (int bb = 0; bb < G::NBLK; ++bb) xoffc[bb] = xoff[bb] + bf * G::BUF + G::ABUF;
            const int aoffc = aoff + bf * G::BUF;
            wait_vmem_done();  // this wave's loads of chunk bf (the only ones in flight) have landed
            __syncthreads();   // chunk bf is complete and every wave has left the other buffer
            ArSrc src;
            // operands of step t+1 are fetched from LDS while step t multiplies; the next chunk's loads go out a few per
            // step from step 1 on, their scalar preparation (which chunk comes next, where it lies) behind the MFMAs of step 0
            float an = lds[aoffc], bn[G::NBLK];
            {
                const int po = pix_off(0);
#pragma unroll
                for (int bb = 0; bb < G::NBLK; ++bb) bn[bb] = lds[xoffc[bb] + po];
            }
            static_for<0, NST>([&](auto t_tag) {
                constexpr int t = decltype(t_tag)::value;
                const float av = an;
                float bv[G::NBLK];
#pragma unroll
                for (int bb = 0; bb < G::NBLK; ++bb) bv[bb] = bn[bb];
                if (t + 1 < NST) {
                    an = lds[aoffc + (HALVES ? 1 : 2) * (t + 1)];
                    const int po = pix_off(t + 1);
#pragma unroll
                    for (int bb = 0; bb < G::NBLK; ++bb) bn[bb] = lds[xoffc[bb] + po];
                }
                if constexpr (t > 0) ar_stage(IntTag<t - 1>{}, IntTag<NST - 1>{}, bf ^ 1, src);
#pragma unroll
                for (int bb = 0; bb < G::NBLK; ++bb)
                    acc[bb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[bb], acc[bb], 0, 0, 0);
                if constexpr (t == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    advance();                                    // (n, p, q0) is now the next chunk
                    ar_source(src, n, p, q0, n < N);
                    __builtin_amdgcn_sched_barrier(0);
                }
            });
            bf ^= 1;
        }
    } else {
        if (n < N) stage(0, n, p, q0);
        // (the loop is unrolled over the two buffers, whose offsets are then constants of each half)
        while (n < N) {
            chunk_body(0, aoffB[0], xoffB[0]);
            if (!(n < N)) break;
            chunk_body(1, aoffB[1], xoffB[1]);
        }
    }

    // partial sums of this pixel split -> dw (cleared before the launch)
    const int SF = G::RT ? SFILT : G::S;             // filter width
    const int RS = R * SF;
    if (wbl) {
        // Blocked dw [K/32][C/4][R][S][4][32]: the 32 output channels of a block are the contiguous index, but an
        // accumulator row (32 lanes) holds 32 columns of ONE output channel, 128 bytes or more apart.  Each wave
        // turns its blocks round through LDS (the stage buffers, free now) so that 32 lanes hold the 32 output
        // channels of one column: an atomic instruction then covers two 128-byte lines instead of 32.
        static_assert(2 * G::BUF >= G::NW * 32 * 33, "the stage buffers hold one 32 x 33 tile per wave");
        wait_vmem_done();    // (the loads issued for a chunk past the end write zeros into the stage buffers)
        __syncthreads();     // every wave has left the chunk loop
        float *tb = lds + wave * (32 * 33);
        const int k = k0 + wk * 32 + j;
#pragma unroll
        for (int b = 0; b < G::NBLK; ++b) {
#pragma unroll
            for (int v = 0; v < 16; ++v) tb[(8 * (v >> 2) + 4 * h + (v & 3)) * 33 + j] = acc[b][v];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int jc = 2 * i + h;                       // column of the block this lane handles now
                const float val = tb[j * 33 + jc];              // (the wave's LDS operations complete in order)
                int c, tap;
                bool ok;
                if (G::AR) {
                    constexpr int SS = G::SB * G::NR;
                    const int col = (wb + G::WB * b) * 32 + jc;
                    c = c0 + wc * 32 * G::CBW + col / SS;       // (packed first layers: c0 = wc = 0)
                    tap = col % SS;
                    ok = col < G::NCOLB * 32 && (G::PACK ? col < C * SS : c < C);
                } else {
                    const int col = b * 32 + jc;
                    c = G::PACK ? col / G::SB : c0 + (wc * G::CBW + b / G::SB) * 32 + jc;
                    tap = r * SF + (G::PACK ? col % G::SB : G::RT ? s0 : b % G::SB);
                    ok = c < C;
                }
                if (k < K && ok) {
                    float *d = dwp + dw_blocked_index(k, c, tap, C, RS);
                    if (splits == 1) *d = val;
                    else unsafeAtomicAdd(d, val);
                }
            }
        }
        return;
    }
    if constexpr (G::AR != 0) {
        // column b*32 + j is float b*32 + j of the run dw[k][c0 .. c0 + CT)[.][.]
#pragma unroll
        for (int b = 0; b < G::NBLK; ++b) {
            const int col = (wb + G::WB * b) * 32 + j;
            const bool cok = col < G::NCOLB * 32 &&
                             (G::PACK ? col < C * G::SB * G::NR : c0 + wc * 32 * G::CBW + col / (G::SB * G::NR) < C);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = k0 + wk * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (k < K && cok) {
                    float *d = dwp + ((size_t)k * C + c0 + wc * 32 * G::CBW) * (G::SB * G::NR) + col;
                    if (splits == 1) *d = acc[b][v];          // the tile's only workgroup: a plain store, the same bits every run
                    else unsafeAtomicAdd(d, acc[b][v]);
                }
            }
        }
        return;
    }
#pragma unroll
    for (int b = 0; b < G::NBLK; ++b) {
        const int col = b * 32 + j;
        const int c = G::PACK ? col / G::SB : c0 + (wc * G::CBW + b / G::SB) * 32 + j;
        const int s = G::PACK ? col % G::SB : G::RT ? s0 : b % G::SB;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + wk * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (k < K && c < C) {
                float *d = dwp + ((size_t)k * C + c) * RS + r * SF + s;
                if (splits == 1) *d = acc[b][v];
                else unsafeAtomicAdd(d, acc[b][v]);
            }
        }
    }
}

__global__ void __launch_bounds__(256) wgrad_clear_kernel(float *dw, long long elems)
{
    for (long long t = blockIdx.x * 256ll + threadIdx.x; t < elems; t += gridDim.x * 256ll) dw[t] = 0.f;
}

template <class G>
static hipError_t launch_wg(const WgradArgs &a, unsigned grid, hipStream_t stream)
{
    static std::atomic<unsigned long long> raised{0};
    if (hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(&conv_wgrad_kernel<G>), G::LDS_BYTES, raised); e != hipSuccess)
        return e;
    hipLaunchKernelGGL((conv_wgrad_kernel<G>), dim3(grid), dim3(G::NT), G::LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class G>
constexpr WgradVariant make_wg(const char *name)
{
    return WgradVariant{name, G::S, G::ST, G::CBW, G::WK, G::PXC, G::PACK, G::QW, G::PER_CU, &launch_wg<G>, G::AR, G::WC, G::WB};
}

// name: w<S>s<stride>_c<channels per workgroup>_k<output channels per workgroup>_p<pixels per chunk>
static WgradVariant g_wgrad[] = {
    make_wg<WgGeom<3, 1, 2, 4, 64>>("w3s1_c64_k128_p64"),
    make_wg<WgGeom<3, 1, 2, 4, 32>>("w3s1_c64_k128_p32"),
    make_wg<WgGeom<3, 1, 2, 2, 64>>("w3s1_c64_k64_p64"),
    make_wg<WgGeom<3, 1, 2, 2, 32>>("w3s1_c64_k64_p32"),
    make_wg<WgGeom<3, 2, 2, 4, 32>>("w3s2_c64_k128_p32"),
    make_wg<WgGeom<5, 1, 1, 4, 32>>("w5s1_c32_k128_p32"),
    make_wg<WgGeom<5, 1, 1, 4, 64>>("w5s1_c32_k128_p64"),
    make_wg<WgGeom<1, 1, 4, 4, 64>>("w1s1_c128_k128_p64"),
    make_wg<WgGeom<1, 1, 4, 2, 64>>("w1s1_c128_k64_p64"),
    make_wg<WgGeom<7, 2, 1, 2, 64>>("w7s2_c32_k64_p64"),
    make_wg<WgGeom<11, 4, 1, 4, 32>>("w11s4_c32_k128_p32"),
    // all S*S taps per wave, columns = consecutive floats of dw (coalesced atomic additions)
    make_wg<WgGeom<3, 1, 1, 4, 32, 0, 0, 1>>("w3s1_ar_c32_k128_p32"),
    make_wg<WgGeom<3, 1, 1, 2, 32, 0, 0, 1, 2>>("w3s1_ar_c64_k64_p32"),
    make_wg<WgGeom<3, 1, 1, 4, 28, 0, 0, 1>>("w3s1_ar_c32_k128_p28"),
    // eight waves, one workgroup per CU: dy staged once for 64 channels
    make_wg<WgGeom<3, 1, 1, 4, 28, 0, 0, 1, 2>>("w3s1_ar_c64_k128_p28"),
    make_wg<WgGeom<3, 1, 1, 4, 32, 0, 0, 1, 2>>("w3s1_ar_c64_k128_p32"),
    // 1x1: small chunks, two workgroups per CU (these layers are bound by reading x and dy once)
    make_wg<WgGeom<1, 1, 2, 2, 32, 0, 0, 1, 2>>("w1s1_ar_c128_k64_p32"),
    make_wg<WgGeom<1, 1, 2, 2, 28, 0, 0, 1, 2>>("w1s1_ar_c128_k64_p28"),
    make_wg<WgGeom<1, 1, 2, 4, 32, 0, 0, 1, 1>>("w1s1_ar_c64_k128_p32"),
    make_wg<WgGeom<1, 1, 2, 4, 28, 0, 0, 1, 1>>("w1s1_ar_c64_k128_p28"),
    make_wg<WgGeom<5, 1, 1, 2, 32, 0, 0, 1, 1, 4>>("w5s1_ar_c32_k64_p32"),
    make_wg<WgGeom<5, 1, 1, 2, 28, 0, 0, 1, 1, 4>>("w5s1_ar_c32_k64_p28"),
    make_wg<WgGeom<5, 2, 1, 2, 32, 0, 0, 1, 1, 4>>("w5s2_ar_c32_k64_p32"),
    make_wg<WgGeom<5, 2, 1, 2, 28, 0, 0, 1, 1, 4>>("w5s2_ar_c32_k64_p28"),
    // 4x4: 16 column blocks, two waves per k-block
    make_wg<WgGeom<4, 1, 1, 4, 32, 0, 0, 1, 1, 2>>("w4s1_ar_c32_k128_p32"),
    make_wg<WgGeom<4, 1, 1, 4, 28, 0, 0, 1, 1, 2>>("w4s1_ar_c32_k128_p28"),
    make_wg<WgGeom<4, 2, 1, 4, 32, 0, 0, 1, 1, 2>>("w4s2_ar_c32_k128_p32"),
    make_wg<WgGeom<4, 2, 1, 4, 28, 0, 0, 1, 1, 2>>("w4s2_ar_c32_k128_p28"),
    make_wg<WgGeom<3, 2, 1, 4, 28, 0, 0, 1>>("w3s2_ar_c32_k128_p28"),
    make_wg<WgGeom<3, 2, 1, 4, 32, 0, 0, 1>>("w3s2_ar_c32_k128_p32"),
    // first layers: all (channel, tap) pairs of C <= 4 channels packed into blocks of 32 columns
    make_wg<WgGeom<7, 2, 1, 2, 64, 5, 0, 1>>("w7s2_arpack5_k64_p64"),
    make_wg<WgGeom<7, 2, 1, 2, 56, 5, 0, 1>>("w7s2_arpack5_k64_p56"),
    make_wg<WgGeom<11, 4, 1, 4, 32, 12, 0, 1>>("w11s4_arpack12_k128_p32"),
    make_wg<WgGeom<11, 4, 1, 4, 28, 12, 0, 1>>("w11s4_arpack12_k128_p28"),
    make_wg<WgGeom<3, 1, 1, 4, 32, 1, 0, 1>>("w3s1_arpack1_k128_p32"),
    // ... their column blocks dealt out to two waves per k-block (more waves per CU: a lone wave per SIMD has nobody to cover its waits)
    make_wg<WgGeom<7, 2, 1, 2, 56, 5, 0, 1, 1, 2>>("w7s2_arpack5_k64_p56b2"),
    make_wg<WgGeom<7, 2, 1, 2, 28, 5, 0, 1, 1, 2>>("w7s2_arpack5_k64_p28b2"),
    make_wg<WgGeom<11, 4, 1, 3, 28, 12, 0, 1, 1, 2>>("w11s4_arpack12_k96_p28b2"),
    make_wg<WgGeom<11, 4, 1, 4, 28, 12, 0, 1, 1, 2>>("w11s4_arpack12_k128_p28b2"),
    make_wg<WgGeom<3, 1, 1, 2, 28, 0, 0, 1, 2>>("w3s1_ar_c64_k64_p28"),
    make_wg<WgGeom<3, 1, 1, 4, 56, 0, 7, 1>>("w3s1_ar_c32_k128_q7"),
    make_wg<WgGeom<3, 1, 1, 4, 32, 0, 13, 1>>("w3s1_ar_c32_k128_q13h"),
    make_wg<WgGeom<3, 1, 1, 4, 32, 0, 14, 1>>("w3s1_ar_c32_k128_q14h"),
    make_wg<WgGeom<3, 1, 1, 4, 32, 0, 7, 1>>("w3s1_ar_c32_k128_q7h"),
    // any filter width, any stride up to 4
    make_wg<WgGeom<0, 4, 2, 4, 32>>("w_any_c64_k128_p32"),
    // small maps: chunks of whole output rows of a fixed width
    make_wg<WgGeom<3, 1, 2, 4, 64, 0, 13>>("w3s1_c64_k128_q13"),
    make_wg<WgGeom<3, 1, 2, 4, 64, 0, 14>>("w3s1_c64_k128_q14"),
    make_wg<WgGeom<3, 1, 2, 4, 64, 0, 28>>("w3s1_c64_k128_q28"),
    make_wg<WgGeom<3, 1, 1, 4, 64, 0, 7>>("w3s1_c32_k128_q7"),
    make_wg<WgGeom<5, 1, 1, 4, 64, 0, 27>>("w5s1_c32_k128_q27"),
    // packed (channel, filter column) columns for layers with very few input channels
    make_wg<WgGeom<3, 1, 1, 4, 64, 1>>("w3s1_pack1_k128_p64"),
    make_wg<WgGeom<7, 2, 1, 2, 64, 1>>("w7s2_pack1_k64_p64"),
    make_wg<WgGeom<11, 4, 1, 4, 32, 2>>("w11s4_pack2_k128_p32"),
};

const WgradVariant *wgrad_table(int *count)
{
    *count = (int)(sizeof(g_wgrad) / sizeof(g_wgrad[0]));
    return g_wgrad;
}

hipError_t wgrad_clear(float *dw, long long elems, hipStream_t stream)
{
    long long blocks = (elems + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(wgrad_clear_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, dw, elems);
    return hipGetLastError();
}

}  // namespace convd
