// Direct-convolution forward kernel for gfx950 (MI355X), single-tap family: layers with
// very few input channels whose output channels come in pairs of 32-channel blocks (the
// first layer of a network with K = 64, 128, ...).  Same computation as the other
// families (paper: Section 3, Algorithm 1) and the same staging as the row-pair family
// (the input window of all channels of the workgroup's pixel tile sits in LDS, split by
// column phase for strided layers; the filter streams through registers, one filter row
// per lane at a time).
//
// What differs is the MFMA: v_mfma_f32_32x32x1_f32 computes TWO independent 32 x 32 x 1
// products per instruction (lanes 0-31 feed the first, lanes 32-63 the second; 32
// accumulator registers), at the same flop rate as v_mfma_f32_32x32x2_f32.  With the two
// products taken as two blocks of OUTPUT channels over the same 32 pixels, an instruction
// needs ONE filter tap, not a pair: the reduction runs over exactly C*R*S taps.  Pairing
// two reduction indices (two rows of an odd filter: 8 for 7, 12 for 11) issues 14 % and
// 9 % more MFMAs than the layer has work for; this family issues none.
//
// Operands: lane (j, h) supplies A = w[k0 + 32*h + j][c][r][s] and B = the window value
// of pixel j (the same for both halves, which read the same LDS word); accumulator
// register v of lane (j, h) is channel 32*(v/16) + 8*((v%16)/4) + 4*h + v%4 of pixel j.
#pragma once
#include "conv_rows_kernel.h"

namespace convd {

typedef float taps_floatx32 __attribute__((ext_vector_type(32)));

// KPW pairs of 32-channel blocks and PBW pixel blocks per wave; WP pixel groups of waves
// (the first NFULL of them own PBW blocks, the others PBW - 1, when NFULL > 0).
template <int R_, int S_, int ST_, int TP_, int TQ_, int KPW_, int PBW_, int WK_, int WP_, int CM_, int OCC_, int NFULL_ = 0>
struct TapGeom {
    static constexpr int R = R_, S = S_, ST = ST_, TP = TP_, TQ = TQ_;
    static constexpr int KPW = KPW_, PBW = PBW_, WK = WK_, WP = WP_, CM = CM_, OCC = OCC_, NFULL = NFULL_;
    static constexpr int CB = CM;                        // reported as the channel block
    static constexpr int PAIR = PAIR_T;                  // one tap per MFMA; stages all channels at once (C <= CM)
    static constexpr int NT = 64 * WK * WP;
    static constexpr int WPE = (OCC * WK * WP + 3) / 4;
    static constexpr int KT = 64 * KPW * WK;             // output channels per workgroup
    static constexpr int NPB = NFULL_ ? NFULL_ + (PBW_ - 1) * WP_ : PBW_ * WP_;
    static constexpr int NPIX = TP * TQ;
    static constexpr int LH = (TP - 1) * ST + R;         // window rows
    static constexpr int LW = (TQ - 1) * ST + S;         // window columns
    static constexpr int LWQ = (LW + ST - 1) / ST;       // columns per phase
    static constexpr int NSEGR = (LWQ + 63) / 64;        // 64-lane loads per window row
    static constexpr int LWP = NSEGR * 64;               // LDS row pitch: whole loads
    static constexpr int PH = LH * LWP;                  // floats of one phase plane
    static constexpr int PS = ST * PH;                   // floats of one channel's window
    static constexpr int PSP = PS;
    static constexpr int NW = NT / 64;
    static constexpr int ROWS_IT = (CM * LH + NW - 1) / NW;
    static constexpr size_t LDS_BYTES = sizeof(float) * (size_t)CM * PSP;
    static_assert(NPB * 32 >= NPIX, "pixel blocks must cover the tile");
    static_assert(NFULL == 0 || (NFULL < WP && PBW > 1), "unequal waves: some groups of each kind");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
};

template <class G, bool FUSED>
__global__ void __launch_bounds__(G::NT, G::WPE) conv_taps_kernel(const KernelArgs a)
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
        const int pb0 = G::NFULL ? wp * (G::PBW - 1) + (wp < G::NFULL ? wp : G::NFULL) : wp * G::PBW;

        // per-lane LDS read offsets (floats): the pixel's window origin in phase 0 (both halves alike)
        int bbase[PBW];
#pragma unroll
        for (int pb = 0; pb < PBW; ++pb) {
            const int t = (pb0 + pb) * 32 + j;
            const int py = t / G::TQ, px = t - py * G::TQ;
            bbase[pb] = t < G::NPIX ? py * G::ST * G::LWP + px : 0;
        }

        // Filter values of this lane: row r of channel c of output channel k0 + (wk*KPW + kp)*64 + 32*h + j, S
        // consecutive floats (clamped: channels past K are computed and discarded)
        const float *w_lane[G::KPW];
#pragma unroll
        for (int kp = 0; kp < G::KPW; ++kp) {
            int krow = k0 + (wk * G::KPW + kp) * 64 + 32 * h + j;
            krow = krow < K ? krow : K - 1;
            w_lane[kp] = a.w + (size_t)krow * C * G::R * G::S;
        }
        auto load_a = [&](float (&dst)[G::KPW][G::S], int c, int r) {
#pragma unroll
            for (int kp = 0; kp < G::KPW; ++kp) {
                const float *q = w_lane[kp] + ((size_t)c * G::R + r) * G::S;
                float *d = dst[kp];
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
            }
        };

        taps_floatx32 acc[G::KPW][PBW];
#pragma unroll
        for (int kp = 0; kp < G::KPW; ++kp)
#pragma unroll
            for (int pb = 0; pb < PBW; ++pb)
#pragma unroll
                for (int v = 0; v < 32; ++v) acc[kp][pb][v] = 0.f;

        // the S taps of filter row r of one channel: one MFMA per tap, channel-block pair and pixel block
        auto compute = [&](const float *chan, int r, const float (&av)[G::KPW][G::S]) {
#pragma unroll
            for (int s = 0; s < G::S; ++s) {
                const int boff = (s % G::ST) * G::PH + r * G::LWP + s / G::ST;
                float bv[PBW];
#pragma unroll
                for (int pb = 0; pb < PBW; ++pb) bv[pb] = chan[bbase[pb] + boff];
#pragma unroll
                for (int kp = 0; kp < G::KPW; ++kp)
#pragma unroll
                    for (int pb = 0; pb < PBW; ++pb)
                        acc[kp][pb] = __builtin_amdgcn_mfma_f32_32x32x1f32(av[kp][s], bv[pb], acc[kp][pb], 0, 0, 0);
            }
        };

        // Filter rows stream through two register sets; which set a row uses alternates, so with an odd filter
        // height the roles swap from one channel to the next (the channel loop handles channels in pairs).
        float a0[G::KPW][G::S], a1[G::KPW][G::S];
        load_a(a0, 0, 0);
        wait_vmem_done();  // this wave's part of the staged window has landed
        __syncthreads();   // ... and so has everybody else's
        auto channel = [&](int c, float (&cur)[G::KPW][G::S], float (&nxt)[G::KPW][G::S]) {
            const float *chan = lds + c * G::PSP;
#pragma unroll
            for (int r = 0; r < G::R; ++r) {
                // next row: of this channel, or the first of the next channel (past the end: this one again)
                const bool lastr = r + 1 == G::R;
                const int cn = lastr ? (c + 1 < C ? c + 1 : c) : c, rn = lastr ? 0 : r + 1;
                if ((r & 1) == 0) {
                    load_a(nxt, cn, rn);
                    compute(chan, r, cur);
                } else {
                    load_a(cur, cn, rn);
                    compute(chan, r, nxt);
                }
            }
        };
        if constexpr (G::R % 2 == 0) {
            for (int c = 0; c < C; ++c) channel(c, a0, a1);
        } else {
            for (int c = 0; c < C; c += 2) {
                channel(c, a0, a1);                   // ends with the next row in a1
                if (c + 1 < C) channel(c + 1, a1, a0);
            }
        }

        // ---- epilogue (see write_block): registers 0-15 are the pair's first channel block, 16-31 its second ----
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
            for (int kp = 0; kp < G::KPW; ++kp)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int kw = k0 + (wk * G::KPW + kp) * 64 + 32 * b;
                    dma_floatx16 blk;
#pragma unroll
                    for (int v = 0; v < 16; ++v) blk[v] = acc[kp][pb][16 * b + v];
                    if (kw < K)   // (a pair's second block may lie wholly past K)
                        write_block<FUSED>(a.out_blocked != 0, fits & (kw + 32 <= K), orsrc, out_n, K, P * Q, kw, h, live, 0, p * Q + q, blk, tail);
                }
        }
    };
    if (G::NFULL > 0 && wp >= G::NFULL) body(IntTag<(G::NFULL > 0 ? G::PBW - 1 : G::PBW)>{});
    else body(IntTag<G::PBW>{});
}

template <class G, bool FUSED>
static hipError_t launch_taps_f(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    static std::atomic<unsigned long long> raised{0};
    if (hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(&conv_taps_kernel<G, FUSED>), G::LDS_BYTES, raised);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((conv_taps_kernel<G, FUSED>), dim3(grid), dim3(G::NT), G::LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class G>
static hipError_t launch_taps(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    if (a.s.C > G::CM) return hipErrorInvalidValue;   // the planner never asks for this
    return has_tail(a) ? launch_taps_f<G, true>(a, grid, stream) : launch_taps_f<G, false>(a, grid, stream);
}

template <class G>
static size_t lds_taps(const Shape &) { return G::LDS_BYTES; }

template <class G>
constexpr Variant make_taps_variant(const char *name)
{
    return Variant{name, G::R, G::S, G::ST, G::TP, G::TQ, G::KT, G::NPB, G::CM, G::PAIR, G::NT, G::OCC,
                   G::PSP, 0, 0, &lds_taps<G>, &launch_taps<G>, 0, 0};
}

}  // namespace convd
