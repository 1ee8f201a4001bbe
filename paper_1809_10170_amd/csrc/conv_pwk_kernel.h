// Direct-convolution forward kernel for gfx950 (MI355X), pointwise family, input-stationary form:
// 1x1 filter, stride 1, no padding, FEW input channels and many output channels (64 -> 256).  Such a
// layer writes several times what it reads, and its reduction is so short (C/2 MFMA steps) that an
// output-stationary workgroup spends as long filling and draining its pipeline as computing.  Here
// the loop order of the paper's Algorithm 2 is turned round for that case: a wave loads the B operands
// of its pixel blocks for ALL C channels into registers once (C/2 registers per block) and then walks
// the output channels in blocks of 32, for each one streaming C/2 filter values per lane from memory
// (the whole filter is a few tens of KB and stays in L1 / L2), multiplying, and storing the finished
// 32 x 32 blocks while the next channel block is already in the MFMA pipe.  The input is read once,
// every output element is written once, there is no LDS, no barrier and no workspace.
//
// A tile has WP * PBW + 1 = 25 pixel blocks: wave q owns PBW of them and multiplies the last, shared block
// for the channel blocks kb with kb % WP == q, so that every SIMD carries 6 1/4 blocks (6272 blocks of 64
// maps of 56 x 56 make 251 workgroups for 256 CUs).  Either four waves of six blocks, one per SIMD with
// 512 registers (C/2 * 7 operand registers, one filter slice, 7 accumulators), or eight waves of three
// blocks, two per SIMD with 256 registers.  A wave that has the SIMD to itself does not issue its MFMAs
// quite back to back (about 5/6 of the pipe's rate was measured in the walk), but the eight-wave form
// measured slower all the same (the two waves of a SIMD drift apart and the last one ends late; 64 -> 256
// channels at 56 x 56: 70 against 67 us), so only the four-wave form is in the variant table.  Tiles run
// over the pixels of all images numbered through.
//
// Which pixel an MFMA column stands for is free in a pointwise layer, and chosen here for wide memory
// instructions: the wave's 32 * PBW pixels come as a first part of G1 = 4 (PBW = 6) or 2 (PBW = 3) pixels a
// lane and a second part of G2 = PBW - G1: lane j holds pixels G1*j .. G1*j + G1-1 of the first part as
// column j of blocks 0 .. G1-1, and pixels G2*j .. of the second part as column j of the other blocks.
// One load per part and reduction step then fetches the operands of all the wave's blocks (16 + 8 bytes a
// lane, or 8 + 4, instead of 4-byte loads block by block), and one store per part and channel row writes
// their results (G1 * 128 and G2 * 128 contiguous bytes per half-wave).  The shared block is 32 consecutive
// pixels, one per lane.  This needs H*W to be a multiple of 4 (no group of pixels reaches over two images).
//
// BLK = 1: input and weights in the blocked layouts (paper, Section 4): in [N][C/4][H*W][4], w [K/32][C/4][4][32].
// The reduction then runs block by block, two steps per block as in the other pointwise kernels: in step (cb, cc)
// the k-lanes take channels 4cb + cc and 4cb + 2 + cc, a lane's B operands of both steps are 8 adjacent bytes of its
// pixel's pencil (one load; the two halves of the wave take the two halves of the same pencils), and a step's filter
// values are 32 consecutive floats per k-lane half.  Here every block keeps its own 32 consecutive pixels, one per
// lane (wide pixel groups would scatter a load over 64-byte strides), and the plain-output stores are 4 bytes a lane.
//
// Same MFMA mapping as the other kernels otherwise (rows = output channels, columns = pixels); the two
// k-lanes of v_mfma_f32_32x32x2_f32 take channels s and s + C/2.
#pragma once
#include "conv_dma_kernel.h"

namespace convd {

// CH: reduction steps = C/2 (the variant serves exactly C = 2 * CH channels); PBW own blocks per wave, WP waves
template <int CH_, int PBW_, int WP_, int BLK_ = 0>
struct PwkGeom {
    static constexpr int R = 1, S = 1, ST = 1;
    static constexpr int PBW = PBW_, CH = CH_, WP = WP_, BLK = BLK_;
    static constexpr int G1 = PBW == 6 ? 4 : 2, G2 = PBW - G1;     // pixels a lane holds in the two parts (plain input)
    // The wave's blocks come in parts: a part is GS blocks whose column j are GS adjacent pixels of lane j.
    static constexpr int NPART = BLK ? PBW + 1 : 3;               // (the last part is the shared block)
    static constexpr int part_size(int p) { return BLK ? 1 : p == 0 ? G1 : p == 1 ? G2 : 1; }
    static constexpr int part_first(int p) { return BLK ? p : p == 0 ? 0 : p == 1 ? G1 : PBW; }   // its first block
    static constexpr int part_of(int pb) { return BLK ? pb : pb < G1 ? 0 : pb < PBW ? 1 : 2; }
    static constexpr int PAIR = PAIR_C;
    static constexpr int CB = 2 * CH;                    // reported: the channel count the variant takes
    static constexpr int NT = 64 * WP, OCC = 1;
    static constexpr int KT = 32;                        // granule of the walk over output channels
    static constexpr int NPB = PBW * WP + 1;
    static constexpr int TP = 1, TQ = 32 * NPB;          // a tile is TQ consecutive pixels of all images
    static_assert(CH % 4 == 0, "filter values are fetched four steps at a time");
    static_assert((PBW == 6 && WP == 4) || (PBW == 3 && WP == 8), "four waves of six blocks or eight of three");
    static_assert(CH * (PBW + 1) + CH + 16 * (PBW + 1) <= (WP == 4 ? 440 : 230), "operands, a filter slice and accumulators in the wave's registers");
};

// do the byte offsets of a tile's outputs (KO channels of HW pixels an image), counted from the tile's first image, fit 31 bits?
template <class G>
__host__ __device__ inline bool pwk_offsets_fit(int KO, int HW) { return (long long)KO * HW * 4 * (G::TQ / HW + 2) < (1ll << 31); }

// K is a multiple of 32 and every byte offset fits 31 bits (the planner's and the launcher's conditions).  MODE (chosen
// by the launcher): 0: plain output, no tail: bare wide buffer stores; 1: either output layout (see write_block); 2: the
// same with the fused point-wise tail.
// All waves run the same instructions (the wave's number only enters addresses and one uniform branch per channel
// block), so that the unrolled channel block is in the instruction cache once.
template <class G, int MODE>
__global__ void __launch_bounds__(G::NT, 1) conv_pwk_kernel(const KernelArgs a)
{
    constexpr int NB = G::PBW + 1, CH = G::CH;
    constexpr int G1 = G::G1, G2 = G::G2;
    const int lane = threadIdx.x & 63;
    const int Q = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // the wave's number in the workgroup
    const int h = lane >> 5, j = lane & 31;

    const int C = a.s.C, K = a.s.K;           // C == 2 * CH, H*W % 4 == 0 (the planner's and the launcher's conditions)
    const int HW = a.s.H * a.s.W;             // = P*Q
    const int nkb = (K + 31) / 32;

    unsigned bid = blockIdx.x;
    {
        const unsigned g8 = gridDim.x & ~7u;
        if (bid < g8) bid = (bid & 7u) * (g8 >> 3) + (bid >> 3);
    }
    const int mt = (int)bid * G::TQ;                                  // first pixel of the tile, of all N*H*W
    const int n = __builtin_amdgcn_readfirstlane((int)(((long long)mt) / HW));   // the image the tile starts in
    const int M = a.s.N * HW;                                         // (a multiple of 4)
    const int mw = mt + Q * (G::PBW * 32);                            // first of the wave's own 32 * PBW pixels
    // the lane's pixel in block pb
    auto pixel = [&](int pb) {
        const int p = G::part_of(pb);
        return pb < G::PBW ? mw + 32 * G::part_first(p) + G::part_size(p) * j + (pb - G::part_first(p)) : mt + G::WP * G::PBW * 32 + j;
    };
    // pixel m -> image relative to n, pixel in the image
    auto locate = [&](int m, int &ni, int &ml) {
        const int nl = m / HW;
        ni = nl - n;
        ml = m - nl * HW;
    };

    // A: lane (j, h) of channel block kb reads w[kb*32 + j][h*CH + s], s = 0 .. CH-1 (rows past K: the last row;
    // computed, not stored).  There is one register per step: the values of steps 4u .. 4u+3 for the next channel
    // block are fetched into the registers of this block's as soon as its MFMAs of those steps are issued, a whole
    // channel block ahead of their use.
    // Blocked weights: step s = (cb, cc) of channel block kb is w[kb][cb][cc + 2h][j], 32 consecutive floats per k-lane half.
    float av[CH];
    auto a_row = [&](int kb) {
        if constexpr (G::BLK != 0) return a.w + (size_t)kb * (C / 4 * 128) + 2 * h * 32 + j;
        int krow = kb * 32 + j;
        krow = krow < K ? krow : K - 1;
        return a.w + (size_t)krow * C + h * CH;
    };
    auto load_a4 = [&](const float *p, int u) {
        if constexpr (G::BLK != 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) av[4 * u + e] = p[(2 * u + e / 2) * 128 + (e % 2) * 32];
        } else {
            const dma_f4u v = *reinterpret_cast<const dma_f4u *>(p + 4 * u);
            av[4 * u] = v[0]; av[4 * u + 1] = v[1]; av[4 * u + 2] = v[2]; av[4 * u + 3] = v[3];
        }
    };
    {
        const float *p = a_row(0);
#pragma unroll
        for (int u = 0; u < CH / 4; ++u) load_a4(p, u);
    }

    // B: lane (j, h) holds in[n'][s + h*CH][its pixel of block pb] for every step s.  Groups past the last pixel
    // (the last tile) read the tensor's last group instead (computed, not stored).
    // Blocked input: bytes 8h .. 8h+7 of the pixel's pencil in channel block 0; one load is two steps.
    unsigned boff[G::NPART];   // byte offsets of the lane's first pixel of every part in channel h*CH
#pragma unroll
    for (int g = 0; g < G::NPART; ++g) {
        int m = pixel(G::part_first(g));
        m = m < M ? m : M - 4;
        int ni, ml;
        locate(m, ni, ml);
        boff[g] = G::BLK ? (unsigned)((ni * (C / 4) * HW + ml) * 4 + 2 * h) * 4u : (unsigned)((ni * C + h * CH) * HW + ml) * 4u;
    }
    const unsigned plane = (unsigned)HW * (G::BLK ? 16u : 4u);      // bytes of one channel (blocked: channel block) of one image
    // (the tile's pixels lie in several images: the resource runs on past image n; every pixel read exists)
    __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(a.in + (size_t)n * C * HW), 0, 0x7fffffff, 0x00020000);
    float b[CH][NB];
    typedef unsigned pwk_u4 __attribute__((ext_vector_type(4)));
    typedef unsigned pwk_u2 __attribute__((ext_vector_type(2)));
    // GS floats from byte offset off (+ soff) of resource r
    auto load_part = [&](auto gs_tag, __amdgpu_buffer_rsrc_t r, unsigned off, int soff, float *dst) {
        constexpr int GS = decltype(gs_tag)::value;
        if constexpr (GS == 4) {
            const pwk_u4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, soff, 0);
            const unsigned e0 = v[0], e1 = v[1], e2 = v[2], e3 = v[3];   // (plain scalars: bit_cast of a vector-element expression is not one)
            dst[0] = __builtin_bit_cast(float, e0); dst[1] = __builtin_bit_cast(float, e1);
            dst[2] = __builtin_bit_cast(float, e2); dst[3] = __builtin_bit_cast(float, e3);
        } else if constexpr (GS == 2) {
            const pwk_u2 v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, soff, 0);
            const unsigned e0 = v[0], e1 = v[1];
            dst[0] = __builtin_bit_cast(float, e0); dst[1] = __builtin_bit_cast(float, e1);
        } else {
            dst[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, soff, 0));
        }
    };
    if constexpr (G::BLK != 0) {
#pragma unroll
        for (int cb = 0; cb < CH / 2; ++cb)
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) {
                float two[2];
                load_part(IntTag<2>{}, rsrc, boff[pb], cb * (int)plane, two);
                b[2 * cb][pb] = two[0];
                b[2 * cb + 1][pb] = two[1];
            }
    } else {
#pragma unroll
        for (int s = 0; s < CH; ++s) {
            load_part(IntTag<G1>{}, rsrc, boff[0], s * (int)plane, &b[s][0]);
            load_part(IntTag<G2>{}, rsrc, boff[1], s * (int)plane, &b[s][G1]);
            load_part(IntTag<1>{}, rsrc, boff[2], s * (int)plane, &b[s][G::PBW]);
        }
    }

    // output addressing (see write_block)
    const int KO = a.out_blocked ? (K + 3) / 4 * 4 : K;
    float *out_n = a.out + (size_t)n * KO * HW;
    __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(out_n), 0, 0x7fffffff, 0x00020000);
    const Tail tail{a.bias, a.residual ? a.residual + (size_t)n * KO * HW : nullptr, a.relu};
    const unsigned oplane = (unsigned)HW * 4u;
    unsigned voff[MODE == 0 ? G::NPART : 1];     // bare stores: byte offsets of the lane's first pixel of every part in channel 4h
    if constexpr (MODE == 0) {
#pragma unroll
        for (int g = 0; g < G::NPART; ++g) {
            const int m = pixel(G::part_first(g));
            int ni, ml;
            locate(m < M ? m : M - 4, ni, ml);
            const size_t o = (size_t)ni * K * HW + ml;
            voff[g] = m < M ? (unsigned)o * 4u + (unsigned)(4 * h) * oplane : 0x80000000u;
        }
    }

    // one block of 32 output channels: NBK pixel blocks (the wave's own, and the shared one when it is this wave's turn)
    auto kblock = [&](auto nbk_tag, int kb) {
        constexpr int NBK = decltype(nbk_tag)::value;
        const float *pn = a_row(kb + 1 < nkb ? kb + 1 : kb);     // the next slice (after the last one: fetched again, unused)
        dma_floatx16 acc[NBK];
#pragma unroll
        for (int pb = 0; pb < NBK; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[pb][v] = 0.f;
#pragma unroll
        for (int s = 0; s < CH; ++s) {
#pragma unroll
            for (int pb = 0; pb < NBK; ++pb)
                acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s], b[s][pb], acc[pb], 0, 0, 0);
            if (s % 4 == 3) load_a4(pn, s / 4);
        }
        const int kw = kb * 32;
        if constexpr (MODE == 0) {
            // channel row by channel row: the two parts (and the shared block's 128 bytes)
            auto store_part = [&](auto gs_tag, unsigned off, int soff, int p0, int v) {
                constexpr int GS = decltype(gs_tag)::value;
                const float f0 = acc[p0][v];
                if constexpr (GS == 4) {
                    const float f1 = acc[p0 + 1][v], f2 = acc[p0 + 2][v], f3 = acc[p0 + 3][v];
                    const pwk_u4 d = {__builtin_bit_cast(unsigned, f0), __builtin_bit_cast(unsigned, f1),
                                      __builtin_bit_cast(unsigned, f2), __builtin_bit_cast(unsigned, f3)};
                    __builtin_amdgcn_raw_buffer_store_b128(d, orsrc, (int)off, soff, 0);
                } else if constexpr (GS == 2) {
                    const float f1 = acc[p0 + 1][v];
                    const pwk_u2 d = {__builtin_bit_cast(unsigned, f0), __builtin_bit_cast(unsigned, f1)};
                    __builtin_amdgcn_raw_buffer_store_b64(d, orsrc, (int)off, soff, 0);
                } else {
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, f0), orsrc, (int)off, soff, 0);
                }
            };
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int soff = (kw + 8 * (v >> 2) + (v & 3)) * (int)oplane;
                static_for<0, G::NPART>([&](auto p_tag) {
                    constexpr int p = decltype(p_tag)::value;
                    if constexpr (G::part_first(p) < NBK) store_part(IntTag<G::part_size(p)>{}, voff[p], soff, G::part_first(p), v);
                });
            }
        } else {
#pragma unroll
            for (int pb = 0; pb < NBK; ++pb) {
                const int m = pixel(pb);
                int ni, ml;
                locate(m < M ? m : M - 4, ni, ml);
                write_block<MODE == 2>(a.out_blocked != 0, true, orsrc, out_n, K, HW, kw, h, m < M, ni, ml, acc[pb], tail);
                __builtin_amdgcn_sched_barrier(0);     // (one block's tail at a time: its loads are not gathered ahead)
            }
        }
    };

    for (int kb = 0; kb < nkb; ++kb) {
        if (kb % G::WP == Q) kblock(IntTag<NB>{}, kb);      // (this wave's turn at the shared block)
        else kblock(IntTag<NB - 1>{}, kb);
    }
}

template <class G>
static hipError_t launch_pwk(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    const int HW = a.s.H * a.s.W;
    if (a.s.C != G::CB || HW % 4 != 0 || a.s.K % 32 != 0 || !pwk_offsets_fit<G>(a.s.K, HW)) return hipErrorInvalidValue;
    if (has_tail(a)) hipLaunchKernelGGL((conv_pwk_kernel<G, 2>), dim3(grid), dim3(G::NT), 0, stream, a);
    else if (!a.out_blocked) hipLaunchKernelGGL((conv_pwk_kernel<G, 0>), dim3(grid), dim3(G::NT), 0, stream, a);
    else hipLaunchKernelGGL((conv_pwk_kernel<G, 1>), dim3(grid), dim3(G::NT), 0, stream, a);
    return hipGetLastError();
}

template <class G>
static size_t lds_pwk(const Shape &) { return 0; }

template <class G>
constexpr Variant make_pwk_variant(const char *name)
{
    return Variant{name, 1, 1, 1, G::TP, G::TQ, G::KT, G::NPB, G::CB, G::PAIR, G::NT, G::OCC,
                   G::TQ, 0, 0, &lds_pwk<G>, &launch_pwk<G>, 2, G::BLK, 0, 1};
}

}  // namespace convd
