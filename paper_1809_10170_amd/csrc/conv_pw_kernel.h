// Direct-convolution forward kernel for gfx950 (MI355X), pointwise family: 1x1 filter,
// stride 1, no padding.  The paper notes that such layers need no change of algorithm,
// only loops that match the layout (Section 4.3); here the convolution degenerates to
//   out[n][k][m] = sum over c of w[k][c] * in[n][c][m],   m = p*W + q,
// a dense contraction with no halo, so nothing is gained by staging the input in LDS:
// every wave reads its B operands (32 consecutive pixels of one channel per k-lane
// half: one 128-byte line) straight from global memory into registers, D reduction
// steps ahead of the MFMAs that use them, and its filter values as consecutive floats
// of w[k][.].  There is no LDS, no barrier and no workspace; the waves of a workgroup
// only share a pixel tile so that their identical input reads meet in the L1 cache.
//
// Same MFMA mapping as the other kernels (rows = output channels, columns = pixels).
// The two k-lanes of v_mfma_f32_32x32x2_f32 take channels s and s + CH, CH = ceil(C/2),
// so that a lane's filter values for consecutive steps are consecutive in memory.
#pragma once
#include "conv_dma_kernel.h"

namespace convd {

//
// BLK = 1: input and weights in the blocked layouts (paper, Section 4): in [N][C/4][H*W][4],
// w [K/32][C/4][4][32].  The reduction then runs block by block, two steps per block: in
// step (cb, cc) the k-lanes take channels 4cb + cc and 4cb + 2 + cc, so that a lane's B
// operands of both steps are 8 adjacent bytes of its pixel's pencil (one load, 512 contiguous
// bytes per half-wave) and a step's filter values are 32 consecutive floats per k-lane half.
//
// FLAT = 1: for images smaller than a tile (7x7, 14x14, 28x28 maps) the pixels of all images
// are numbered through, m = n*H*W + p*W + q, and a tile is TQ consecutive ones.
//
// SL = 1: a tile has one pixel block more than the waves' own WP * PBW (the shared block).  The
// waves are dealt to the four SIMDs in turn, so with WP = 8 each SIMD holds waves wp and wp + 4;
// wave 4 + q takes every fourth reduction step of the shared block (every fourth channel block
// when blocked), the four partial sums meet in LDS at the end and wave 4 stores the block.  Each
// SIMD then carries 2 PBW + 1/4 blocks: tiles of 8 PBW + 1 blocks fit sizes such as the 49 blocks
// of half a 56 x 56 map, which no equal split over eight waves does.
template <int KBW_, int PBW_, int WK_, int WP_, int D_, int OCC_, int BLK_ = 0, int FLAT_ = 0, int SL_ = 0>
struct PwGeom {
    static constexpr int SL = SL_;
    static constexpr int BLK = BLK_;
    static constexpr bool FLAT = FLAT_ != 0;
    static constexpr int R = 1, S = 1, ST = 1;
    static constexpr int KBW = KBW_, PBW = PBW_, WK = WK_, WP = WP_, D = D_, OCC = OCC_;
    static constexpr int PAIR = PAIR_C;
    static constexpr int CB = 2 * D;                     // reported: channels in flight per wave
    static constexpr int NT = 64 * WK * WP;
    static constexpr int WPE = (OCC * WK * WP + 3) / 4;
    static constexpr int KT = 32 * KBW * WK;
    static constexpr int NPB = PBW * WP + (SL ? 1 : 0);
    static constexpr int TP = 1, TQ = 32 * NPB;          // a tile is TQ consecutive pixels of one image
    static_assert(D % 4 == 0, "filter values are fetched four steps at a time");
    static_assert(!SL || (WP == 8 && WK == 1 && KBW == 1 && D % (BLK ? 8 : 4) == 0),
                  "shared block: two waves per SIMD, quarters by step (by channel block) within a group");
};

// One wave's work: NB pixel blocks; SHQ = 0: all of them its own; SHQ = q + 1: the last one is
// the tile's shared block, of which this wave computes quarter q.  red: 3 * 16 * 64 floats of LDS
// (shared-block variants only).
template <class G, bool FUSED, int NB, int SHQ>
__device__ __forceinline__ void pw_body(const KernelArgs &a, float *red)
{
    // does this wave multiply pixel block pb in step d of a group (d < 0: a step after the groups)?
    constexpr auto owns = [](int pb, int d) {
        return SHQ == 0 || pb < NB - 1 || (d < 0 ? SHQ == 1 : ((G::BLK ? d >> 1 : d) & 3) == SHQ - 1);
    };
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    __builtin_assume(wave >= 0 && wave < G::NT / 64);
    const int wk = wave % G::WK, wp = wave / G::WK;
    const int h = lane >> 5, j = lane & 31;

    const int C = a.s.C, K = a.s.K;
    const int HW = a.s.H * a.s.W;             // = P*Q
    const int CH = (C + 1) / 2;               // reduction steps

    unsigned bid = blockIdx.x;
    {
        const unsigned g8 = gridDim.x & ~7u;
        if (bid < g8) bid = (bid & 7u) * (g8 >> 3) + (bid >> 3);
    }
    const int kt = bid % a.ktiles;  bid /= a.ktiles;
    // per-image tiling: image n, tile tm of its H*W pixels.  Flat tiling (images smaller than
    // a tile): tile bid of the N*H*W pixels of all images; n is then the image the tile starts in
    const int tm = G::FLAT ? (int)bid : (int)(bid % a.tilesQ);
    const int n = G::FLAT ? __builtin_amdgcn_readfirstlane((int)(((long long)tm * G::TQ) / HW)) : (int)(bid / a.tilesQ);
    const int k0 = kt * G::KT, mt = tm * G::TQ;                    // mt: in the image, or in all images (flat)
    // first pixel of the wave's block pb
    auto mblk = [&](int pb) { return mt + ((SHQ != 0 && pb == NB - 1) ? G::WP * G::PBW : wp * G::PBW + pb) * 32; };
    const int M = G::FLAT ? a.s.N * HW : HW;                       // pixels of the tile may reach
    // pixel m (past the end: the last one; read, computed, not stored) -> image relative to n, pixel in the image
    auto locate = [&](int m, int &ni, int &ml) {
        m = m < M ? m : M - 1;
        if (G::FLAT) {
            const int nl = m / HW;
            ni = nl - n;
            ml = m - nl * HW;
        } else {
            ni = 0;
            ml = m;
        }
    };

    // B: lane (j, h) reads in[n][s + h*CH][block pb, pixel j]; pixels past the image are
    // clamped (read, computed, not stored).  Buffer loads keep the addressing to one
    // 32-bit register per pixel block: byte offset of the lane's pixel in channel h*CH,
    // plus a scalar offset for the step.
    unsigned boff[NB];
#pragma unroll
    for (int pb = 0; pb < NB; ++pb) {
        int ni, ml;
        locate(mblk(pb) + j, ni, ml);
        boff[pb] = (unsigned)((ni * C + h * CH) * HW + ml) * 4u;
    }
    const unsigned plane = (unsigned)HW * 4u;
    // (flat: the tile's pixels lie in several images, the resource runs on past image n)
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        uniform_ptr(a.in + (size_t)n * C * HW), 0, G::FLAT ? 0x7fffffff : (int)((unsigned)C * plane), 0x00020000);
    auto load_b_full = [&](float (&bv)[NB], int s, int d) {  // a step that exists in both halves; d: its place in the group
        const int soff = __builtin_amdgcn_readfirstlane(s) * (int)plane;
#pragma unroll
        for (int pb = 0; pb < NB; ++pb)
            if (owns(pb, d))
                bv[pb] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)boff[pb], soff, 0));
    };
    // the last step of the second half does not exist when C is odd: both its filter
    // value and its B operand are zero (the load is sent past the resource's end)
    auto load_b = [&](float (&bv)[NB], int s) {       // any step
        const bool ok = s + h * CH < C;
        const int soff = __builtin_amdgcn_readfirstlane(s) * (int)plane;
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            if (!owns(pb, -1)) continue;
            const unsigned off = ok ? boff[pb] : 0x80000000u;
            bv[pb] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)off, soff, 0));
        }
    };

    // A: lane (j, h) of k-block kb reads w[k][h*CH + s], consecutive in s
    const float *w_lane[G::KBW];
#pragma unroll
    for (int kb = 0; kb < G::KBW; ++kb) {
        int krow = k0 + (wk * G::KBW + kb) * 32 + j;
        krow = krow < K ? krow : K - 1;
        w_lane[kb] = a.w + (size_t)krow * C + h * CH;
    }
    auto load_a4 = [&](float (&av)[G::KBW][4], int s) {   // steps s .. s+3, all inside the lane's run
#pragma unroll
        for (int kb = 0; kb < G::KBW; ++kb) {
            const dma_f4u v = *reinterpret_cast<const dma_f4u *>(w_lane[kb] + s);
            av[kb][0] = v[0]; av[kb][1] = v[1]; av[kb][2] = v[2]; av[kb][3] = v[3];
        }
    };

    dma_floatx16 acc[G::KBW][NB];
#pragma unroll
    for (int kb = 0; kb < G::KBW; ++kb)
#pragma unroll
        for (int pb = 0; pb < NB; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[kb][pb][v] = 0.f;

    auto mfma_step = [&](const float (&bv)[NB], float av, int kb, int d) {
#pragma unroll
        for (int pb = 0; pb < NB; ++pb)
            if (owns(pb, d)) acc[kb][pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[pb], acc[kb][pb], 0, 0, 0);
    };

    if constexpr (G::BLK != 0) {
        // ---- blocked layouts ----
        const int C4 = (C + 3) / 4;
        const int nsteps = 2 * C4;                       // all of them exist: pad channels hold zeros
        const int nfullb = nsteps / G::D * G::D;
        unsigned boffb[NB];                          // byte offset of the lane's two channels in block 0
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            int ni, ml;
            locate(mblk(pb) + j, ni, ml);
            boffb[pb] = (unsigned)((ni * C4 * HW + ml) * 4 + 2 * h) * 4u;
        }
        const unsigned bplane = (unsigned)HW * 16u;      // bytes of one channel block of one image
        __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
            uniform_ptr(a.in + (size_t)n * C4 * 4 * HW), 0, G::FLAT ? 0x7fffffff : (int)((unsigned)C4 * bplane), 0x00020000);
        typedef unsigned pw_u2 __attribute__((ext_vector_type(2)));
        // B operands of the two steps of block cb
        auto load_b2 = [&](float (&b0)[NB], float (&b1)[NB], int cb, int d) {
            const int soff = __builtin_amdgcn_readfirstlane(cb) * (int)bplane;
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) {
                if (!owns(pb, d)) continue;
                const pw_u2 v = __builtin_amdgcn_raw_buffer_load_b64(rb, (int)boffb[pb], soff, 0);
                const unsigned u0 = v[0], u1 = v[1];   // (plain scalars: bit_cast of a vector-element expression is not one)
                b0[pb] = __builtin_bit_cast(float, u0);
                b1[pb] = __builtin_bit_cast(float, u1);
            }
        };
        // filter values: block row of the wave's k-block kb (clamped: rows past K are computed and
        // discarded), lane part (2h*32 + j) floats, step part (cb*128 + cc*32) floats
        __amdgpu_buffer_rsrc_t ra[G::KBW];
#pragma unroll
        for (int kb = 0; kb < G::KBW; ++kb) {
            int kblk = (k0 + (wk * G::KBW + kb) * 32) / 32;
            kblk = kblk < (K + 31) / 32 ? kblk : (K + 31) / 32 - 1;
            ra[kb] = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(a.w + (size_t)kblk * C4 * 128), 0, C4 * 128 * 4,
                                                       0x00020000);
        }
        const int aoff = (2 * h * 32 + j) * 4;
        auto load_a4b = [&](float (&av)[G::KBW][4], int s) {   // steps s .. s+3 = blocks s/2, s/2 + 1
            const int soff = __builtin_amdgcn_readfirstlane(s / 2) * 512;
#pragma unroll
            for (int kb = 0; kb < G::KBW; ++kb)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    av[kb][e] = __builtin_bit_cast(
                        float, __builtin_amdgcn_raw_buffer_load_b32(ra[kb], aoff, soff + ((e / 2) * 128 + (e % 2) * 32) * 4, 0));
        };
        float bq[G::D][NB];
        float aq[2][G::D / 4][G::KBW][4];
        if (nfullb > 0) {
#pragma unroll
            for (int u = 0; u < G::D / 4; ++u) load_a4b(aq[0][u], 4 * u);
            __builtin_amdgcn_sched_barrier(0);   // keep the load order the loop's counted waits assume
#pragma unroll
            for (int d = 0; d < G::D; d += 2) {
                load_b2(bq[d], bq[d + 1], d / 2, d);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        auto group = [&](int s0, float (&ac)[G::D / 4][G::KBW][4], float (&an)[G::D / 4][G::KBW][4]) {
            const int sn = s0 + G::D < nfullb ? s0 + G::D : s0;     // next group (clamped: reloads this one)
#pragma unroll
            for (int u = 0; u < G::D / 4; ++u) load_a4b(an[u], sn + 4 * u);
#pragma unroll
            for (int d = 0; d < G::D; d += 2) {
#pragma unroll
                for (int kb = 0; kb < G::KBW; ++kb) mfma_step(bq[d], ac[d / 4][kb][d % 4], kb, d);
#pragma unroll
                for (int kb = 0; kb < G::KBW; ++kb) mfma_step(bq[d + 1], ac[d / 4][kb][d % 4 + 1], kb, d);
                load_b2(bq[d], bq[d + 1], (sn + d) / 2, d);
#pragma unroll
                for (int pb = 0; pb < NB; ++pb) {
                    if (!owns(pb, d)) continue;
                    __builtin_amdgcn_sched_group_barrier(0x008, 2 * G::KBW, 0);   // the MFMAs of two steps
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);            // one load
                }
            }
        };
        for (int s0 = 0; s0 < nfullb; s0 += 2 * G::D) {
            group(s0, aq[0], aq[1]);
            if (s0 + G::D >= nfullb) break;
            group(s0 + G::D, aq[1], aq[0]);
        }
        // remaining blocks, one at a time (fewer than D/2 of them)
        for (int s = nfullb; s < nsteps; s += 2) {
            float b0[NB], b1[NB];
            load_b2(b0, b1, s / 2, -1);
            const int soff = __builtin_amdgcn_readfirstlane(s / 2) * 512;
#pragma unroll
            for (int kb = 0; kb < G::KBW; ++kb) {
                const float a0 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ra[kb], aoff, soff, 0));
                const float a1 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ra[kb], aoff, soff + 128, 0));
                mfma_step(b0, a0, kb, -1);
                mfma_step(b1, a1, kb, -1);
            }
        }
    } else {
        // Main loop: whole groups of D steps whose filter runs lie inside both halves (the
        // second half is one step shorter when C is odd).  B operands are D steps ahead.
        const int nfull = C / 2 / G::D * G::D;    // steps covered by full groups (all valid for both halves)
        float bq[G::D][NB];
        float aq[2][G::D / 4][G::KBW][4];         // filter values of this group and of the next
        if (nfull > 0) {
            // filter loads first, as in the loop: the loop's waits are counted in load order and
            // must find the same order on entry as on every later pass
    #pragma unroll
            for (int u = 0; u < G::D / 4; ++u) load_a4(aq[0][u], 4 * u);
            __builtin_amdgcn_sched_barrier(0);   // the scheduler may not reorder these loads
    #pragma unroll
            for (int d = 0; d < G::D; ++d) {
                load_b_full(bq[d], d, d);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        auto group = [&](int s0, float (&ac)[G::D / 4][G::KBW][4], float (&an)[G::D / 4][G::KBW][4]) {
            const int sn = s0 + G::D < nfull ? s0 + G::D : s0;     // next group (clamped: reloads this one)
    #pragma unroll
            for (int u = 0; u < G::D / 4; ++u) load_a4(an[u], sn + 4 * u);
    #pragma unroll
            for (int d = 0; d < G::D; ++d) {
    #pragma unroll
                for (int kb = 0; kb < G::KBW; ++kb) mfma_step(bq[d], ac[d / 4][kb][d % 4], kb, d);
                load_b_full(bq[d], sn + d, d);
                // keep the reloads of this step's registers right behind the MFMAs that read them
    #pragma unroll
                for (int pb = 0; pb < NB; ++pb) {
                    if (!owns(pb, d)) continue;
                    __builtin_amdgcn_sched_group_barrier(0x008, G::KBW, 0);   // KBW MFMAs
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);        // one load
                }
            }
        };
        for (int s0 = 0; s0 < nfull; s0 += 2 * G::D) {
            group(s0, aq[0], aq[1]);
            if (s0 + G::D >= nfull) break;
            group(s0 + G::D, aq[1], aq[0]);
        }
        // Remaining steps, one at a time (fewer than D + 1 of them)
        for (int s = nfull; s < CH; ++s) {
            float bv[NB];
            load_b(bv, s);
            const bool ok = s + h * CH < C;
    #pragma unroll
            for (int kb = 0; kb < G::KBW; ++kb) {
                const float av = ok ? w_lane[kb][s] : 0.f;
                mfma_step(bv, av, kb, -1);
            }
        }

    }

    // ---- shared block: the quarters meet in LDS, wave 4 (quarter 0) holds the sum ----
    if constexpr (G::SL != 0) {
        if constexpr (SHQ >= 2) {
#pragma unroll
            for (int v = 0; v < 16; ++v) red[((SHQ - 2) * 16 + v) * 64 + lane] = acc[0][NB - 1][v];
        }
        __syncthreads();
        if constexpr (SHQ == 1) {
#pragma unroll
            for (int q = 0; q < 3; ++q)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[0][NB - 1][v] += red[(q * 16 + v) * 64 + lane];
        }
    }
    constexpr int NBS = SHQ >= 2 ? NB - 1 : NB;   // blocks this wave stores

    // ---- epilogue (see write_block) ----
    const int KO = a.out_blocked ? (K + 3) / 4 * 4 : K;
    float *out_n = a.out + (size_t)n * KO * HW;
    __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(out_n), 0, 0x7fffffff, 0x00020000);
    const bool fits = (long long)KO * HW * 4 * (G::FLAT ? G::TQ / HW + 2 : 1) < (1ll << 31);
    const Tail tail{a.bias, a.residual ? a.residual + (size_t)n * KO * HW : nullptr, a.relu};
    if (!FUSED && !a.out_blocked && fits && k0 + G::KT <= K) {
        // Plain output, all channels present: the wave's PBW blocks are consecutive pixels,
        // so storing channel row by channel row (blocks innermost) sends PBW * 128 contiguous
        // bytes of one row to memory back to back instead of 128 bytes per row and block.
        unsigned voff[NBS];
        const unsigned oplane = (unsigned)HW * 4u;
#pragma unroll
        for (int pb = 0; pb < NBS; ++pb) {
            const int m = mblk(pb) + j;
            int ni, ml;
            locate(m, ni, ml);
            const size_t o = (size_t)ni * K * HW + ml;
            voff[pb] = m < M ? (unsigned)o * 4u + (unsigned)(4 * h) * oplane : 0x80000000u;
        }
#pragma unroll
        for (int kb = 0; kb < G::KBW; ++kb) {
            const int kw = k0 + (wk * G::KBW + kb) * 32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int soff = (kw + 8 * (v >> 2) + (v & 3)) * (int)oplane;
#pragma unroll
                for (int pb = 0; pb < NBS; ++pb) {
                    const float f = acc[kb][pb][v];
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, f), orsrc, (int)voff[pb], soff, 0);
                }
            }
        }
        return;
    }
#pragma unroll
    for (int pb = 0; pb < NBS; ++pb) {
        const int m = mblk(pb) + j;
        const bool live = m < M;
        int ni, ml;
        locate(m, ni, ml);
#pragma unroll
        for (int kb = 0; kb < G::KBW; ++kb) {
            const int kw = k0 + (wk * G::KBW + kb) * 32;
            write_block<FUSED>(a.out_blocked != 0, fits & (kw + 32 <= K), orsrc, out_n, K, HW, kw, h, live, ni, ml, acc[kb][pb], tail);
        }
    }
}

template <class G, bool FUSED>
__global__ void __launch_bounds__(G::NT, G::WPE) conv_pw_kernel(const KernelArgs a)
{
    if constexpr (G::SL != 0) {
        __shared__ float red[3 * 16 * 64];
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        switch (wave) {
        case 4: pw_body<G, FUSED, G::PBW + 1, 1>(a, red); break;
        case 5: pw_body<G, FUSED, G::PBW + 1, 2>(a, red); break;
        case 6: pw_body<G, FUSED, G::PBW + 1, 3>(a, red); break;
        case 7: pw_body<G, FUSED, G::PBW + 1, 4>(a, red); break;
        default: pw_body<G, FUSED, G::PBW, 0>(a, red); break;
        }
    } else {
        pw_body<G, FUSED, G::PBW, 0>(a, nullptr);
    }
}

template <class G>
static hipError_t launch_pw(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    if constexpr (G::SL != 0) {
        // (no instantiation with the tail: the seven accumulators, the operands in flight and the tail's values do not
        // fit the 256 registers of a wave)
        if (has_tail(a)) return hipErrorInvalidValue;
        hipLaunchKernelGGL((conv_pw_kernel<G, false>), dim3(grid), dim3(G::NT), 0, stream, a);
    } else {
        if (has_tail(a)) hipLaunchKernelGGL((conv_pw_kernel<G, true>), dim3(grid), dim3(G::NT), 0, stream, a);
        else hipLaunchKernelGGL((conv_pw_kernel<G, false>), dim3(grid), dim3(G::NT), 0, stream, a);
    }
    return hipGetLastError();
}

template <class G>
static size_t lds_pw(const Shape &) { return 0; }

template <class G>
constexpr Variant make_pw_variant(const char *name)
{
    // "window": the TQ pixels of a channel that a workgroup reads (once, through L1)
    return Variant{name, 1, 1, 1, G::TP, G::TQ, G::KT, G::NPB, G::CB, G::PAIR, G::NT, G::OCC,
                   G::TQ, 0, 0, &lds_pw<G>, &launch_pw<G>, G::FLAT ? 2 : 1, G::BLK, 0, 0, G::SL != 0 ? 1 : 0};
}

}  // namespace convd
