// Direct-convolution forward kernel for gfx950 (MI355X), channel-pair family:
// fp32 MFMA, input halo tiles brought into LDS by LDS-direct buffer loads, filter
// values read straight into registers, no workspace.
//
// The computation is the paper's Algorithm 1 (Section 3): six loops around one
// multiply-accumulate.  The paper blocks the output-channel and output-column loops
// for the register file, the input-channel loop for the cache, and runs output
// channels in parallel (Section 3.1.2, Section 3.2, Algorithm 3).  Here:
//   * register block -> a 32 x (32*PBW) accumulator tile per wave (32x32 MFMA
//     results; rows = output channels, columns = output pixels);
//   * cache block    -> CB input channels per step: the input halo window of the
//     workgroup's pixel tile sits in LDS, every filter tap reads it at a different
//     constant offset, so no lowered (im2col) matrix ever exists (Sections 1, 2.2);
//   * parallel loop  -> the grid: every (image, pixel tile, channel tile) is an
//     independent workgroup.
//
// v_mfma_f32_32x32x2_f32 operand layout: lane l supplies A[i = l%32][kk = l/32] and
// B[kk = l/32][j = l%32]; accumulator register v of lane l holds
// D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].  A = filter (i = output channel),
// B = input (j = output pixel).  The two kk lanes of an instruction take input
// channels c and c + CB/2 of the chunk at one filter tap, so the filter values one
// lane needs for a chunk are (CB/2)*R*S consecutive floats of w[k][c..][.][.]: they
// are loaded from global memory directly into registers and never touch LDS.  Any
// order of the C*R*S additions is a correct convolution (Section 3, "any
// permutation of the loops").
//
// Input staging uses buffer_load_dword ... lds: 64 lanes write 64 consecutive LDS
// words, out-of-range lanes (zero padding, channels past C) read past the buffer
// resource's end and therefore store zeros.  No registers, address arithmetic or LDS
// store instructions are spent per element.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "variant.h"

namespace convd {

typedef float dma_floatx16 __attribute__((ext_vector_type(16)));
typedef float dma_f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float dma_f2u __attribute__((ext_vector_type(2), aligned(4)));

template <int R_, int S_, int ST_, int TP_, int TQ_, int PBW_, int WK_, int WP_, int CB_, int OCC_>
struct DmaGeom {
    static constexpr int R = R_, S = S_, ST = ST_, TP = TP_, TQ = TQ_;
    static constexpr int PBW = PBW_, WK = WK_, WP = WP_, CB = CB_, OCC = OCC_;
    static constexpr int PAIR = PAIR_C;
    static constexpr int NT = 64 * WK * WP;              // threads per workgroup
    static constexpr int WPE = (OCC * WK * WP + 3) / 4;  // waves per SIMD the register budget must allow
    static constexpr int KT = 32 * WK;                   // output channels per workgroup
    static constexpr int NPB = PBW * WP;                 // 32-pixel blocks per workgroup
    static constexpr int NPIX = TP * TQ;                 // real pixels in the tile
    static constexpr int RS = R * S;
    static constexpr int LH = (TP - 1) * ST + R;         // halo window rows
    static constexpr int LW = (TQ - 1) * ST + S;         // halo window columns = LDS row pitch
    static constexpr int PS = LH * LW;                   // floats of one channel's window
    static constexpr int NSEG = (PS + 63) / 64;          // 64-lane loads per channel
    static constexpr int PSP = NSEG * 64;                // LDS stride between channels
    static constexpr int HC = CB / 2;                    // channels per kk half
    static constexpr int HOFF = HC * PSP + 32;           // LDS offset of the second half (other banks)
    static constexpr int BUF = CB * PSP + 32;            // floats per stage buffer
    static constexpr int ITEMS = (CB * PSP + NT - 1) / NT;   // 64-lane loads per wave and chunk
    static constexpr int NA = HC * RS;                   // filter values per lane and chunk
    static constexpr int STEPS = HC * RS;                // MFMA k-steps per chunk
    static constexpr size_t LDS_BYTES = sizeof(float) * 2 * (size_t)BUF;
    static_assert(CB % 2 == 0, "channel pairing needs an even chunk");
    static_assert(NPB * 32 >= NPIX, "pixel blocks must cover the tile");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
};

#define CONVD_LDS(p) ((__attribute__((address_space(3))) void *)(p))

template <class G>
__global__ void __launch_bounds__(G::NT, G::WPE) conv_dma_kernel(const KernelArgs a)
{
    extern __shared__ __align__(16) float lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    __builtin_assume(wave >= 0 && wave < G::NT / 64);
    const int wk = wave % G::WK, wp = wave / G::WK;
    const int h = lane >> 5, j = lane & 31;

    const int C = a.s.C, H = a.s.H, W = a.s.W, K = a.s.K, P = a.s.P, Q = a.s.Q;

    // Workgroup -> tile.  Consecutive workgroup ids are dealt round-robin to the 8
    // XCDs, each with its own L2; the ids are first regrouped so that one XCD works
    // on neighbouring tiles (all channel tiles of a pixel tile share their input).
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

    // per-lane LDS read offsets (floats): pixel position plus the kk half
    int bbase[G::PBW];
#pragma unroll
    for (int pb = 0; pb < G::PBW; ++pb) {
        const int t = (wp * G::PBW + pb) * 32 + j;
        const int py = t / G::TQ, px = t - py * G::TQ;
        const int pix = t < G::NPIX ? py * G::ST * G::LW + px * G::ST : 0;
        bbase[pb] = pix + h * G::HOFF;
    }

    // Input staging plan: thread tid owns positions tid + i*NT of the chunk's
    // [CB][PSP] window array; its byte offset from the chunk's first channel, or an
    // offset no buffer can reach where the window lies outside the image.
    unsigned goff[G::ITEMS];
#pragma unroll
    for (int i = 0; i < G::ITEMS; ++i) {
        const int f = i * G::NT + tid;
        const int cc = f / G::PSP, pos = f - cc * G::PSP;
        const int hh = pos / G::LW, col = pos - hh * G::LW;
        const int ih = ih0 + hh, iw = iw0 + col;
        const bool ok = (f < G::CB * G::PSP) & (pos < G::PS) & ((unsigned)ih < (unsigned)H) &
                        ((unsigned)iw < (unsigned)W);
        goff[i] = ok ? (unsigned)(((cc * H + ih) * W + iw) * 4) : 0x80000000u;
    }
    const float *in_n = a.in + (size_t)n * C * H * W;
    const unsigned chan_bytes = (unsigned)(H * W) * 4u;

    // Stage the input window of channels [c0, c0 + CB) into buf.  The resource ends
    // at the image's last channel, so channels past C read as zeros.
    auto stage_b = [&](float *buf, int c0) {
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(in_n + (size_t)c0 * H * W), 0, (int)((unsigned)(C - c0) * chan_bytes), 0x00020000);
#pragma unroll
        for (int i = 0; i < G::ITEMS; ++i) {
            const int f0 = i * G::NT + wave * 64;           // first position of this wave's 64
            if (f0 < G::CB * G::PSP) {
                float *dst = buf + f0 + (f0 >= G::HC * G::PSP ? 32 : 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, CONVD_LDS(dst), 4, goff[i], 0, 0, 0);
            }
        }
    };

    // Filter values of this lane: output channel k0 + wk*32 + j (clamped: rows past K
    // are computed and discarded), input channels c0 + h*HC .. + HC, all taps.
    int krow = k0 + wk * 32 + j;
    krow = krow < K ? krow : K - 1;
    const float *w_lane = a.w + ((size_t)krow * C + h * G::HC) * G::RS;
    auto load_a = [&](float (&dst)[G::NA], int c0) {
        const float *p = w_lane + (size_t)c0 * G::RS;
        if (c0 + G::CB <= C) {
            constexpr int N4 = G::NA / 4, REM = G::NA % 4;
#pragma unroll
            for (int i = 0; i < N4; ++i) {
                const dma_f4u v = *reinterpret_cast<const dma_f4u *>(p + 4 * i);
                dst[4 * i] = v[0]; dst[4 * i + 1] = v[1]; dst[4 * i + 2] = v[2]; dst[4 * i + 3] = v[3];
            }
            if (REM >= 2) {
                const dma_f2u v = *reinterpret_cast<const dma_f2u *>(p + 4 * N4);
                dst[4 * N4] = v[0]; dst[4 * N4 + 1] = v[1];
            }
            if (REM & 1) dst[G::NA - 1] = p[G::NA - 1];
        } else {
            // last, partial chunk: channels past C contribute zero weights
#pragma unroll
            for (int e = 0; e < G::NA; ++e) {
                const bool ok = c0 + h * G::HC + e / G::RS < C;
                const float v = *(ok ? p + e : a.w);
                dst[e] = ok ? v : 0.f;
            }
        }
    };

    dma_floatx16 acc[G::PBW];
#pragma unroll
    for (int pb = 0; pb < G::PBW; ++pb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[pb][v] = 0.f;

    // The reduction over one staged chunk: STEPS rank-2 updates of the wave's tile.
    auto compute = [&](const float *buf, const float (&av)[G::NA]) {
#pragma unroll
        for (int cc = 0; cc < G::HC; ++cc)
#pragma unroll
            for (int r = 0; r < G::R; ++r)
#pragma unroll
                for (int s = 0; s < G::S; ++s) {
                    const int boff = cc * G::PSP + r * G::LW + s;
                    const float aval = av[(cc * G::R + r) * G::S + s];
#pragma unroll
                    for (int pb = 0; pb < G::PBW; ++pb)
                        acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(aval, buf[bbase[pb] + boff], acc[pb], 0, 0, 0);
                }
    };

    // Two stage buffers and two register sets, used alternately: chunk i+1 is in
    // flight (LDS-direct loads and filter loads) while chunk i is reduced.
    float *buf0 = lds, *buf1 = lds + G::BUF;
    float a0[G::NA], a1[G::NA];
    const int nch = (C + G::CB - 1) / G::CB;
    stage_b(buf0, 0);
    load_a(a0, 0);
    __syncthreads();
    for (int ci = 0;; ci += 2) {
        if (ci + 1 < nch) {
            stage_b(buf1, (ci + 1) * G::CB);
            load_a(a1, (ci + 1) * G::CB);
        }
        compute(buf0, a0);
        __syncthreads();
        if (ci + 1 >= nch) break;
        if (ci + 2 < nch) {
            stage_b(buf0, (ci + 2) * G::CB);
            load_a(a0, (ci + 2) * G::CB);
        }
        compute(buf1, a1);
        __syncthreads();
        if (ci + 2 >= nch) break;
    }

    // ---- epilogue: each output element is written exactly once ----
    float *out_n = a.out + (size_t)n * K * P * Q;
#pragma unroll
    for (int pb = 0; pb < G::PBW; ++pb) {
        const int t = (wp * G::PBW + pb) * 32 + j;
        const int py = t / G::TQ, px = t - py * G::TQ;
        const int p = p0 + py, q = q0 + px;
        if (t < G::NPIX && p < P && q < Q) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = k0 + wk * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (k < K) out_n[((size_t)k * P + p) * Q + q] = acc[pb][v];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side: launcher and the table entry of one compiled variant.
// ---------------------------------------------------------------------------
template <class G>
static hipError_t launch_dma(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    if (G::LDS_BYTES > 64 * 1024) {
        // workgroups above the 64 KB default need the limit raised (no allocation involved)
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_dma_kernel<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((conv_dma_kernel<G>), dim3(grid), dim3(G::NT), G::LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class G>
static size_t lds_dma(const Shape &) { return G::LDS_BYTES; }

template <class G>
constexpr Variant make_dma_variant(const char *name)
{
    return Variant{name, G::R, G::S, G::ST, G::TP, G::TQ, G::KT, G::NPB, G::CB, G::PAIR, G::NT, G::OCC,
                   &lds_dma<G>, &launch_dma<G>};
}

}  // namespace convd
