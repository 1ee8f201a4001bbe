// Direct-convolution forward kernel for gfx950 (MI355X), row-pair family: layers
// with very few input channels (the first layer of a network: C <= CM, large
// filters, stride 1, 2 or 4).  Same computation and operand mapping as
// conv_dma_kernel.h (paper: Section 3, Algorithm 1; blocking after Section 3.1.2),
// with two differences that keep the MFMA reduction depth useful when C is tiny:
//
//   * the two k-lanes of v_mfma_f32_32x32x2_f32 take filter rows r and r + R2
//     (R2 = ceil(R/2)) of one input channel; for odd R the first half's last row has no
//     partner: the second half multiplies a zero weight there.  The reduction runs
//     over (channel, row pair, filter column);
//   * the input window of ALL channels of the workgroup's pixel tile is staged into
//     LDS once (it is small when C is small), so the main loop has no barrier at
//     all; the filter streams through registers, RG rows per lane at a time.
//
// For stride > 1 the window is stored split by column phase, [phase][row][col/stride]
// (rows padded to whole 64-lane loads),
// so that the 32 pixels of an MFMA column block read consecutive LDS words for every
// tap (stride-ST words would collide on the LDS banks).  The split costs nothing:
// LDS-direct loads take an arbitrary global address per lane.
#pragma once
#include "conv_dma_kernel.h"

namespace convd {

template <int R_, int S_, int ST_, int TP_, int TQ_, int KBW_, int PBW_, int WK_, int WP_, int CM_, int RG_, int OCC_,
          int NFULL_ = 0>
struct RowGeom {
    static constexpr int R = R_, S = S_, ST = ST_, TP = TP_, TQ = TQ_;
    static constexpr int KBW = KBW_, PBW = PBW_, WK = WK_, WP = WP_, CM = CM_, RG = RG_, OCC = OCC_;
    static constexpr int CB = CM;                        // reported as the channel block
    static constexpr int PAIR = PAIR_R;
    static constexpr int NT = 64 * WK * WP;
    static constexpr int WPE = (OCC * WK * WP + 3) / 4;
    static constexpr int KT = 32 * KBW * WK;            // a wave owns KBW x PBW 32x32 results
    // Unequal waves (NFULL > 0): only the first NFULL pixel groups own PBW blocks, the others
    // PBW - 1.  Waves are numbered k-group fastest, so with WK odd every SIMD of the CU still
    // gets its share of both kinds.
    static constexpr int NFULL = NFULL_;
    static constexpr int NPB = NFULL_ ? NFULL_ + (PBW_ - 1) * WP_ : PBW_ * WP_;
    static constexpr int NPIX = TP * TQ;
    static constexpr int R2 = (R + 1) / 2;               // filter rows per k-lane half
    static constexpr int NSUB = R2 / RG;                 // register sub-chunks per channel
    static constexpr int LH = (TP - 1) * ST + R;         // window rows
    static constexpr int LW = (TQ - 1) * ST + S;         // window columns
    static constexpr int LWQ = (LW + ST - 1) / ST;       // columns per phase
    static constexpr int NSEGR = (LWQ + 63) / 64;        // 64-lane loads per window row
    static constexpr int LWP = NSEGR * 64;               // LDS row pitch: whole loads, so that a row's last
                                                         // load cannot spill into the next row
    static constexpr int PH = LH * LWP;                  // floats of one phase plane
    static constexpr int PS = ST * PH;                   // floats of one channel's window
    static constexpr int PSP = PS;                       // LDS stride between channels
    static constexpr int HOFF = R2 * LWP;                // LDS offset of the second k-lane half
    static constexpr int NA = RG * S;                    // filter values per lane and sub-chunk
    static constexpr int NW = NT / 64;
    static constexpr int ROWS_IT = (CM * LH + NW - 1) / NW;   // window rows per wave, phase and row segment
    static constexpr size_t LDS_BYTES = sizeof(float) * (size_t)CM * PSP;
    static_assert(R2 % RG == 0 && NSUB % 2 == 0, "row groups must tile R2 an even number of times");
    static_assert(NPB * 32 >= NPIX, "pixel blocks must cover the tile");
    static_assert(NFULL == 0 || (NFULL < WP && PBW > 1), "unequal waves: some groups of each kind");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
};

// Stage the whole input window of a pixel tile (all channels) into LDS, once.
// One LDS-direct load brings 64 columns of one window row (channel, phase, row).
// Which row is a scalar matter: its byte offset goes into the instruction's scalar
// offset, rows outside the image take an all-lanes-unreachable vector offset.  The
// vector offsets (column part; unreachable outside the image) are computed once per
// phase and segment.  So the loop below costs no vector ALU work per load, which
// matters: the wave shares its SIMD with waves issuing MFMAs back to back and gets
// very few vector issue slots.  G supplies ST, LH, LWQ, NSEGR, LWP, CM and NW.
template <class G>
__device__ __forceinline__ void rows_stage_window(float *lds, const float *in, int n, int C, int H, int W, int ih0, int iw0,
                                                  int wave, int lane)
{
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        uniform_ptr(in + (size_t)n * C * H * W), 0, (int)((unsigned)(C * H * W) * 4u), 0x00020000);
    unsigned voffc[G::ST][G::NSEGR];
#pragma unroll
    for (int ph = 0; ph < G::ST; ++ph)
#pragma unroll
        for (int sg = 0; sg < G::NSEGR; ++sg) {
            const int cq = sg * 64 + lane, iw = iw0 + cq * G::ST + ph;
            voffc[ph][sg] = ((cq < G::LWQ) & ((unsigned)iw < (unsigned)W)) ? (unsigned)iw * 4u : 0x80000000u;
        }
    const unsigned voob = 0x80000000u;
#pragma unroll 1
    for (int i = 0; i < G::ROWS_IT; ++i) {
        const int row = i * G::NW + wave;            // (channel, window row), scalar
        const int cc = row / G::LH, hh = row - cc * G::LH;
        const int ih = ih0 + hh;
        const bool ok = (cc < C) & ((unsigned)ih < (unsigned)H);
        const int soff = ok ? ((cc * H + ih) * W) * 4 : 0;
        if (cc < G::CM) {
#pragma unroll
            for (int ph = 0; ph < G::ST; ++ph)
#pragma unroll
                for (int sg = 0; sg < G::NSEGR; ++sg) {
                    float *dst = lds + ((cc * G::ST + ph) * G::LH + hh) * G::LWP + sg * 64;
                    if (ok) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, CONVD_LDS(dst), 4, voffc[ph][sg], soff, 0, 0);
                    else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, CONVD_LDS(dst), 4, voob, 0, 0, 0);
                }
        }
    }
}

template <class G, bool FUSED>
__global__ void __launch_bounds__(G::NT, G::WPE) conv_rows_kernel(const KernelArgs a)
{
    extern __shared__ __align__(16) float lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    __builtin_assume(wave >= 0 && wave < G::NT / 64);
    const int wk = wave % G::WK, wp = wave / G::WK;
    const int h = lane >> 5, j = lane & 31;

    const int C = a.s.C, H = a.s.H, W = a.s.W, K = a.s.K, P = a.s.P, Q = a.s.Q;

    unsigned bid = blockIdx.x;
    {
        const unsigned g8 = gridDim.x & ~7u;
        if (bid < g8) bid = (bid & 7u) * (g8 >> 3) + (bid >> 3);
    }
    const int kt = bid % a.ktiles;  bid /= a.ktiles;
    const int tq = bid % a.tilesQ;  bid /= a.tilesQ;
    const int tp = bid % a.tilesP;
    const int n = bid / a.tilesP;
    const int p0 = tp * G::TP, q0 = tq * G::TQ, k0 = kt * G::KT;
    const int ih0 = p0 * G::ST - a.s.pad, iw0 = q0 * G::ST - a.s.pad;

    rows_stage_window<G>(lds, a.in, n, C, H, W, ih0, iw0, wave, lane);

    // Everything below depends on how many pixel blocks the wave owns (see NFULL): the
    // body is compiled once per count and the wave takes its own.
    auto body = [&](auto pbw_tag) __attribute__((always_inline)) {
    constexpr int PBW = decltype(pbw_tag)::value;
    // first pixel block of the wave
    const int pb0 = G::NFULL ? wp * (G::PBW - 1) + (wp < G::NFULL ? wp : G::NFULL) : wp * G::PBW;

        // per-lane LDS read offsets (floats): pixel position (phase 0) plus the k-lane half.
        // For odd R the second half has no partner for the first half's last row: there its
        // weight is zero and it reads the SAME window position as the first half (bsame), a
        // position inside the output's own window, so that the zero never meets a value
        // (an Inf, say) that the true sum does not contain.
        int bbase[PBW], bsame[PBW];
    #pragma unroll
        for (int pb = 0; pb < PBW; ++pb) {
            const int t = (pb0 + pb) * 32 + j;
            const int py = t / G::TQ, px = t - py * G::TQ;
            const int pix = t < G::NPIX ? py * G::ST * G::LWP + px : 0;
            bbase[pb] = pix + h * G::HOFF;
            bsame[pb] = pix;
        }

        // Filter values of this lane for sub-chunk (c, g): rows g*RG + h*R2 .. + RG of
        // w[k][c], RG*S consecutive floats.  Rows past R (second half, odd R) are zeros and
        // are not read.
        const float *w_lane[G::KBW];
    #pragma unroll
        for (int kb = 0; kb < G::KBW; ++kb) {
            int krow = k0 + (wk * G::KBW + kb) * 32 + j;
            krow = krow < K ? krow : K - 1;
            w_lane[kb] = a.w + (size_t)krow * C * G::R * G::S + h * G::R2 * G::S;
        }
        auto load_a = [&](float (&dst)[G::KBW][G::NA], int c, int g) {
    #pragma unroll
            for (int kb = 0; kb < G::KBW; ++kb) {
            const float *p = w_lane[kb] + ((size_t)c * G::R + g * G::RG) * G::S;
    #pragma unroll
            for (int i = 0; i < G::RG; ++i) {
                const float *pr = p + i * G::S;
                float *d = dst[kb] + i * G::S;
                // row g*RG + i + h*R2 exists for both halves iff it exists for the second
                const bool both = g * G::RG + i + G::R2 < G::R;
                const bool ok = both | (h == 0);
                const float *q = ok ? pr : a.w;     // lanes without a row read a valid address
                constexpr int N4 = G::S / 4, REM = G::S % 4;
    #pragma unroll
                for (int u = 0; u < N4; ++u) {
                    const dma_f4u v = *reinterpret_cast<const dma_f4u *>(q + 4 * u);
                    d[4 * u] = v[0]; d[4 * u + 1] = v[1]; d[4 * u + 2] = v[2]; d[4 * u + 3] = v[3];
                }
                if (REM >= 2) {
                    const dma_f2u v = *reinterpret_cast<const dma_f2u *>(q + 4 * N4);
                    d[4 * N4] = v[0]; d[4 * N4 + 1] = v[1];
                }
                if (REM & 1) d[G::S - 1] = q[G::S - 1];
                if (!both) {
    #pragma unroll
                    for (int u = 0; u < G::S; ++u) d[u] = ok ? d[u] : 0.f;
                }
            }
            }
        };

        dma_floatx16 acc[G::KBW][PBW];
    #pragma unroll
        for (int kb = 0; kb < G::KBW; ++kb)
    #pragma unroll
            for (int pb = 0; pb < PBW; ++pb)
    #pragma unroll
                for (int v = 0; v < 16; ++v) acc[kb][pb][v] = 0.f;

        // RG*S rank-2 updates: rows g*RG .. of the first half, columns 0 .. S-1
        auto compute = [&](const float *chan, int g, const float (&av)[G::KBW][G::NA]) {
    #pragma unroll
            for (int i = 0; i < G::RG; ++i)
    #pragma unroll
                for (int s = 0; s < G::S; ++s) {
                    const int boff = (s % G::ST) * G::PH + (g * G::RG + i) * G::LWP + s / G::ST;
                    const bool both = g * G::RG + i + G::R2 < G::R;   // the second half has this row too
                    float bv[PBW];
    #pragma unroll
                    for (int pb = 0; pb < PBW; ++pb) bv[pb] = chan[(both ? bbase[pb] : bsame[pb]) + boff];
    #pragma unroll
                    for (int kb = 0; kb < G::KBW; ++kb)
    #pragma unroll
                        for (int pb = 0; pb < PBW; ++pb)
                            acc[kb][pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[kb][i * G::S + s], bv[pb], acc[kb][pb], 0, 0, 0);
                }
        };

        float a0[G::KBW][G::NA], a1[G::KBW][G::NA];
        load_a(a0, 0, 0);
        wait_vmem_done();  // this wave's part of the staged window has landed
        __syncthreads();   // ... and so has everybody else's
        for (int c = 0; c < C; ++c) {
            const float *chan = lds + c * G::PSP;
    #pragma unroll
            for (int g = 0; g < G::NSUB; g += 2) {
                load_a(a1, c, g + 1);
                compute(chan, g, a0);
                {
                    // next sub-chunk: same channel, or the first of the next channel (clamped at the end)
                    const bool last = g + 2 == G::NSUB;
                    const int cn = last ? (c + 1 < C ? c + 1 : c) : c;
                    load_a(a0, cn, last ? 0 : g + 2);
                }
                compute(chan, g + 1, a1);
            }
        }

        // ---- epilogue (see write_block) ----
        const int KO = a.out_blocked ? (K + 3) / 4 * 4 : K;
        float *out_n = a.out + (size_t)n * KO * P * Q;
        __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(out_n), 0, 0x7fffffff, 0x00020000);
        const bool fits = (long long)KO * P * Q * 4 < (1ll << 31);
        const Tail tail{a.bias, a.residual ? a.residual + (size_t)n * KO * P * Q : nullptr, a.relu};
    #pragma unroll
        for (int pb = 0; pb < PBW; ++pb) {
            const int t = (pb0 + pb) * 32 + j;
            const int py = t / G::TQ, px = t - py * G::TQ;
            const int p = p0 + py, q = q0 + px;
            const bool live = t < G::NPIX && p < P && q < Q;
    #pragma unroll
            for (int kb = 0; kb < G::KBW; ++kb) {
                const int kw = k0 + (wk * G::KBW + kb) * 32;
                write_block<FUSED>(a.out_blocked != 0, fits & (kw + 32 <= K), orsrc, out_n, K, P * Q, kw, h, live, 0, p * Q + q,
                            acc[kb][pb], tail);
            }
        }
    };
    if (G::NFULL > 0 && wp >= G::NFULL) body(IntTag<(G::NFULL > 0 ? G::PBW - 1 : G::PBW)>{});
    else body(IntTag<G::PBW>{});
}

template <class G, bool FUSED>
static hipError_t launch_rows_f(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    static std::atomic<unsigned long long> raised{0};
    if (hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(&conv_rows_kernel<G, FUSED>), G::LDS_BYTES, raised);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((conv_rows_kernel<G, FUSED>), dim3(grid), dim3(G::NT), G::LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class G>
static hipError_t launch_rows(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    if (a.s.C > G::CM) return hipErrorInvalidValue;   // the planner never asks for this
    return has_tail(a) ? launch_rows_f<G, true>(a, grid, stream) : launch_rows_f<G, false>(a, grid, stream);
}

template <class G>
static size_t lds_rows(const Shape &) { return G::LDS_BYTES; }

template <class G>
constexpr Variant make_rows_variant(const char *name)
{
    return Variant{name, G::R, G::S, G::ST, G::TP, G::TQ, G::KT, G::NPB, G::CM, G::PAIR, G::NT, G::OCC,
                   G::PSP, 0, 0, &lds_rows<G>, &launch_rows<G>, 0, 0};
}

}  // namespace convd
