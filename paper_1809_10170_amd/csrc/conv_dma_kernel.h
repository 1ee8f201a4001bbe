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
// are loaded from global memory directly into registers and never touch LDS.  The
// order of the C*R*S additions is free: every loop order computes the same
// convolution (Section 3).
//
// Input staging uses buffer_load_dword ... lds: 64 lanes write 64 consecutive LDS
// words, out-of-range lanes (zero padding, channels past C) read past the buffer
// resource's end and therefore store zeros.  No registers, address arithmetic or LDS
// store instructions are spent per element.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

#include "variant.h"

namespace convd {

typedef float dma_floatx16 __attribute__((ext_vector_type(16)));
typedef float dma_f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float dma_f2u __attribute__((ext_vector_type(2), aligned(4)));

// Two tilings of the output pixels:
//   rectangular (IMG_ = 0): a workgroup owns TP x TQ pixels of one image;
//   flat (IMG_ > 0): for small square images of IMG_ x IMG_ pixels and padding PADC_
//     (both fixed at compile time) the pixels of ALL images are numbered
//     m = (n*P + p)*Q + q and a workgroup owns 32*PBW*WP consecutive ones, whatever
//     image or row they fall in.  Its LDS window holds every input row those pixels
//     touch, the rows of one image after those of the previous one.  No MFMA column
//     is wasted on tile edges and the grid can be cut to fit the machine.
template <int R_, int S_, int ST_, int TP_, int TQ_, int PBW_, int WK_, int WP_, int CB_, int OCC_, int IMG_ = 0,
          int PADC_ = 0, int PF_ = 1, int SC_ = 1, int PBW2_ = 0, int BLK_ = 0, int SL_ = 0>
struct DmaGeom {
    // SL = 1 (flat tiling, eight pixel groups, one 32-channel block): the tile has 8*PBW + 1 blocks.  Pixel groups 0..3
    // own PBW blocks each; groups 4..7 own PBW blocks each and SHARE the last block of the tile: group 4 + q adds to it
    // only in the reduction steps t of a chunk with t % 4 == q, a quarter of the reduction in EVERY chunk (the waves of a
    // workgroup meet once per chunk, so the extra work has to be even within a chunk), and the four partial sums meet
    // through LDS at the end.  Wave w runs on SIMD w % 4, so every SIMD carries 2*PBW + 1/4 blocks: a layer whose blocks per SIMD
    // are a whole number and a quarter (12.25 for 512 x 28 x 28 at batch 32: 13 with two unequal waves) fills the
    // matrix pipes without idle columns, and its 16 x 16 tiles are exactly 256 workgroups.
    static constexpr int SL = SL_;
    // BLK = 1: input and weights in the paper's blocked layouts (Section 4) with pencils of
    // 4 input channels and weight blocks of 4 input x 32 output channels:
    //   in [N][C/4][H][W][4]      w [K/32][C/4][R][S][4][32]
    // A chunk is then one channel block, its window in LDS a [LH][LW][4] array staged by the
    // same LDS-direct loads (16 window columns per load instead of 64 of one channel); lane
    // (j, h) reads channels 2h, 2h+1 of its pixel's pencil, 8 adjacent bytes, so the 64
    // lanes of an operand fetch cover 1 KB without a gap or a bank conflict; the filter
    // values of a step are 32 consecutive floats per k-lane half (one 128-byte line).
    static constexpr int BLK = BLK_;
    static constexpr int PF = PF_;                       // reduction steps the LDS operand fetch runs ahead
    // Split reduction: SC groups of WK*WP waves share one output tile; group sc reduces
    // the chunks sc, sc+SC, ... with stage buffers and a meeting counter of its own (the
    // groups run as independent pipelines), and the partial tiles are summed through LDS
    // at the end.  This is the paper's input-channel blocking (Section 3.1.2) spread over
    // waves: it multiplies the parallelism of layers that have few outputs (single
    // images, 13x13 / 14x14 maps) without any workspace.
    static constexpr int SC = SC_;
    // Unequal waves (flat tilings, WP = 2): the waves of the second pixel group own PBW2
    // blocks instead of PBW.  A SIMD then runs one wave of each kind, PBW + PBW2 blocks in
    // all, which lets the work per SIMD be an odd number of blocks (13 = 7 + 6 where two
    // equal waves could only offer 12 or 14).
    static constexpr int PBW2 = PBW2_;
    static constexpr int R = R_, S = S_, ST = ST_;
    static constexpr int PBW = PBW_, WK = WK_, WP = WP_, CB = CB_, OCC = OCC_;
    static constexpr int IMG = IMG_, PADC = PADC_;
    static constexpr bool FLAT = IMG_ > 0;
    static constexpr int OQ = FLAT ? (IMG + 2 * PADC - S) / ST + 1 : 0;       // flat: output width
    static constexpr int OP = FLAT ? (IMG + 2 * PADC - R) / ST + 1 : 0;       // flat: output height
    static constexpr int NPB = PBW2_ ? PBW_ + PBW2_ : PBW_ * WP_ + (SL_ ? 1 : 0);   // 32-pixel blocks per workgroup
    static constexpr int NPIXF = 32 * NPB;                                     // flat: pixels per workgroup
    static constexpr int NRMAX = FLAT ? (NPIXF + OQ - 2) / OQ + 1 : 0;         // flat: output rows a tile can touch
    static constexpr int NSI = FLAT ? (NRMAX + OP - 2) / OP + 1 : 1;           // flat: images a tile can touch
    static constexpr int TP = FLAT ? 0 : TP_, TQ = FLAT ? OQ : TQ_;
    static constexpr int PAIR = PAIR_C;
    static constexpr int NWG = WK * WP;                  // waves per split group
    static constexpr int NTG = 64 * NWG;                 // threads per split group
    static constexpr int NT = NTG * SC;                  // threads per workgroup
    static constexpr int WPE = (OCC * NWG * SC + 3) / 4; // waves per SIMD the register budget must allow
    static constexpr int KT = 32 * WK;                   // output channels per workgroup
    static constexpr int NPIX = FLAT ? NPIXF : TP * TQ;  // real pixels in the tile
    static constexpr int RS = R * S;
    // halo window rows; flat: consecutive output rows of one image share input rows as
    // usual, a new image starts R - ST rows further down
    static constexpr int LH = FLAT ? (NRMAX - 1) * ST + R + (NSI - 1) * (R - ST) : (TP - 1) * ST + R;
    static constexpr int LW = (TQ - 1) * ST + S;         // halo window columns = LDS row pitch
    static constexpr int PS = LH * LW;                   // floats of one channel's window
    static constexpr int NSEG = (PS + 63) / 64;          // 64-lane loads per channel
    static constexpr int PSP = NSEG * 64;                // LDS stride between channels
    static constexpr int HC = CB / 2;                    // channels per kk half
    static constexpr int PXF = BLK ? 4 : 1;              // LDS floats from one window position to the next
    static constexpr int CHF = BLK ? (4 * PS + 63) / 64 * 64 : CB * PSP;   // floats of one chunk's window array
    static constexpr int HOFF = BLK ? 2 : HC * PSP + 32; // LDS offset of the second kk half (plain: other banks)
    static constexpr int BUF = CHF + 32;                 // floats per stage buffer
    static constexpr int ITEMS = (CHF + NTG - 1) / NTG;  // 64-lane loads per wave and chunk
    static constexpr int NA = HC * RS;                   // filter values per lane and chunk
    static constexpr int STEPS = HC * RS;                // MFMA k-steps per chunk
    static constexpr int GRP = 3 * BUF + 16;             // floats per split group: three stage buffers, arrival counter
    static constexpr int RED = (SC / 2) * NWG * PBW * 1024;   // floats of the final sum's exchange (a tree: half the groups write)
    static_assert((SC & (SC - 1)) == 0, "the split groups' tiles are summed as a binary tree");
    static constexpr size_t LDS_BYTES = sizeof(float) * (size_t)(SC * GRP > RED ? SC * GRP : RED);
    static_assert(CB % 2 == 0, "channel pairing needs an even chunk");
    static_assert(!BLK || CB == 4, "blocked layout: a chunk is one block of 4 channels");
    static_assert(PBW2 == 0 || (FLAT && WP == 2 && SC == 1 && PBW2 < PBW), "unequal waves: flat tiling, two pixel groups");
    static_assert(!SL || (FLAT && WP == 8 && WK == 1 && SC == 1 && PBW2 == 0), "shared last block: flat tiling, eight pixel groups of one k-block");
    static_assert(!FLAT || R >= ST, "flat tiling stacks image windows R - ST rows apart");
    static_assert(PF >= 1 && 2 * PF < STEPS, "operand fetches for the next chunk must follow the meeting point");
    static_assert(NPB * 32 >= NPIX, "pixel blocks must cover the tile");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
};

template <int V>
struct IntTag { static constexpr int value = V; };

// f(IntTag<T0>{}), f(IntTag<T0 + 1>{}), ... f(IntTag<T1 - 1>{}): a loop whose index is a compile-time constant
template <int T0, int T1, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (T0 < T1) {
        f(IntTag<T0>{});
        static_for<T0 + 1, T1>(f);
    }
}

#define CONVD_LDS(p) ((__attribute__((address_space(3))) void *)(p))

// A pointer that is the same in every lane, moved to scalar registers.
// (readfirstlane returns a signed int: widen through unsigned, or a low half with its
// top bit set would smear ones over the high half)
__device__ __forceinline__ void *uniform_ptr(const void *p)
{
    const uintptr_t pa = (uintptr_t)p;
    return (void *)(((uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(pa >> 32)) << 32) |
                    (uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)pa));
}

// Wait until every vector-memory operation this wave has issued is complete
// (s_waitcnt vmcnt(0); expcnt and lgkmcnt left at their maxima).  LDS-direct loads
// (buffer_load ... lds) are counted by vmcnt, not by lgkmcnt: a wave that hands
// LDS filled by such loads to another wave (through a barrier or a release) states
// this wait itself instead of relying on what the compiler inserts for the fence.
__device__ __forceinline__ void wait_vmem_done() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Epilogue stores of one 32 x 32 accumulator block whose 32 output channels all exist:
// buffer stores with the channel row as a scalar offset and one precomputed 32-bit
// register per lane (byte offset of out[.][4h][p][q] from the resource base, or an
// offset past the resource for lanes without a pixel, which the hardware drops).  No
// vector ALU work per store: a wave in its epilogue shares the SIMD with waves that
// issue MFMAs back to back and gets very few vector issue slots.
__device__ __forceinline__ void store_block(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, int kfirst, unsigned plane,
                                            const dma_floatx16 &acc)
{
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int soff = (kfirst + 8 * (v >> 2) + (v & 3)) * (int)plane;
        const float f = acc[v];   // (a plain float: bit_cast of a vector-element expression is not one)
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, f), rsrc, (int)voff, soff, 0);
    }
}

// The same for an output in the blocked activation layout out[N][K/4][P][Q][4]: the four
// accumulator registers 4g .. 4g+3 of a lane are channels 8g + 4h .. + 3 of its pixel, one
// whole pencil, stored with one 16-byte store; voff is the byte offset of the lane's pencil
// in channel block h, the block pair 2g a scalar offset.  A wave's store covers 512
// contiguous bytes per k-lane half.
typedef float dma_f4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_block_pencils(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, int kfirst,
                                                    unsigned plane16, const dma_floatx16 &acc)
{
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int soff = (kfirst / 4 + 2 * g) * (int)plane16;
        const float f0 = acc[4 * g], f1 = acc[4 * g + 1], f2 = acc[4 * g + 2], f3 = acc[4 * g + 3];
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        const u4 d = {__builtin_bit_cast(unsigned, f0), __builtin_bit_cast(unsigned, f1),
                      __builtin_bit_cast(unsigned, f2), __builtin_bit_cast(unsigned, f3)};
        __builtin_amdgcn_raw_buffer_store_b128(d, rsrc, (int)voff, soff, 0);
    }
}

// Epilogue of one 32 x 32 accumulator block, shared by all kernel families: channels
// kw .. kw+31 of the lane's pixel, which is pixel `pix` of the image `ni` images after the
// one that `orsrc` and `out_n` start at.  The output is plain [N][K][P][Q] or blocked
// [N][K/4][P][Q][4] (the layout a following layer's blocked input has; channels that
// complete the last pencil are written as zeros).  Fast path (uniform test by the caller:
// the 32 channels exist and every byte offset fits 31 bits): buffer stores without vector
// ALU work; otherwise plain guarded stores.  Each output element is written exactly once.
//
// Point-wise layers that follow a convolution (bias, skip connection, activation) fold
// into this store (paper, Section 4.3: such layers need no change of the algorithm):
// with a tail, every value becomes relu?(acc + bias[k] + residual[where it is stored])
// before it is written.  Without one (the uniform test below) nothing changes.
struct Tail {
    const float *bias;     // K floats or NULL
    const float *res_n;    // the residual tensor at the position out_n has in out, or NULL
    int relu;
};

__device__ __forceinline__ void store_tile_block(bool blocked, bool fast, __amdgpu_buffer_rsrc_t orsrc, float *out_n,
                                                 int K, int PQ, int kw, int h, bool live, int ni, int pix,
                                                 const dma_floatx16 &acc)
{
    const unsigned oplane = (unsigned)PQ * 4u;
    if (blocked) {
        const int KO = (K + 3) / 4 * 4;
        const size_t o = (size_t)ni * KO * PQ + (size_t)pix * 4;   // the pixel's pencil of channel block 0
        if (fast) {
            const unsigned voff = live ? (unsigned)o * 4u + (unsigned)h * 4u * oplane : 0x80000000u;
            store_block_pencils(orsrc, voff, kw, 4u * oplane, acc);
        } else if (live) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int k = kw + 8 * g + 4 * h;
                if (k < KO) {
                    float *d = out_n + o + (size_t)(k / 4) * PQ * 4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) d[e] = k + e < K ? acc[4 * g + e] : 0.f;
                }
            }
        }
    } else {
        const size_t o = (size_t)ni * K * PQ + pix;                 // out[n'][0][p][q] from out[n][0][0][0]
        if (fast) {
            const unsigned voff = live ? (unsigned)o * 4u + (unsigned)(4 * h) * oplane : 0x80000000u;
            store_block(orsrc, voff, kw, oplane, acc);
        } else if (live) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kw + 8 * (v >> 2) + 4 * h + (v & 3);
                if (k < K) out_n[o + (size_t)k * PQ] = acc[v];
            }
        }
    }
}

// FUSED is a compile-time switch: kernels are instantiated with and without the tail, so
// that the plain convolution's epilogue carries none of its registers or instructions.
template <bool FUSED>
__device__ __forceinline__ void write_block(bool blocked, bool fast, __amdgpu_buffer_rsrc_t orsrc, float *out_n, int K,
                                            int PQ, int kw, int h, bool live, int ni, int pix, const dma_floatx16 &acc,
                                            const Tail &tail)
{
    if constexpr (!FUSED) {
        store_tile_block(blocked, fast, orsrc, out_n, K, PQ, kw, h, live, ni, pix, acc);
        return;
    }
    const int KO = blocked ? (K + 3) / 4 * 4 : K;
    dma_floatx16 val;
    if (fast) {
        // the wave's 32 channels exist and offsets fit 31 bits: bias and residual come in by buffer
        // loads addressed like the stores (scalar channel offsets, one per-lane register, lanes
        // without a pixel read past the resource and get zeros), no address arithmetic per value
        const unsigned oplane = (unsigned)PQ * 4u;
        __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(tail.bias), 0, tail.bias ? K * 4 : 0, 0x00020000);
        __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(tail.res_n), 0, tail.res_n ? 0x7fffffff : 0, 0x00020000);
        // (an absent bias or residual is a resource of size 0: its loads return zeros)
        const size_t o = blocked ? (size_t)ni * KO * PQ + (size_t)pix * 4 : (size_t)ni * K * PQ + pix;
        const unsigned voff = !live ? 0x80000000u
                              : blocked ? (unsigned)o * 4u + (unsigned)h * 4u * oplane : (unsigned)o * 4u + (unsigned)(4 * h) * oplane;
        typedef unsigned tail_u4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int g = 0; g < 4; ++g) {     // four values at a time keeps the loads in flight, and their registers, few
            float rv[4];
            if (blocked) {
                const tail_u4 d = __builtin_amdgcn_raw_buffer_load_b128(rr, (int)voff, (kw / 4 + 2 * g) * (int)(4u * oplane), 0);
                const unsigned d0 = d[0], d1 = d[1], d2 = d[2], d3 = d[3];
                rv[0] = __builtin_bit_cast(float, d0); rv[1] = __builtin_bit_cast(float, d1);
                rv[2] = __builtin_bit_cast(float, d2); rv[3] = __builtin_bit_cast(float, d3);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    rv[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr, (int)voff, (kw + 8 * g + e) * (int)oplane, 0));
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float bvv = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, 16 * h, (kw + 8 * g + e) * 4, 0));
                float x = acc[4 * g + e] + bvv + rv[e];
                if (tail.relu) x = x > 0.f ? x : 0.f;
                val[4 * g + e] = x;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = kw + 8 * (v >> 2) + 4 * h + (v & 3);
            float x = acc[v];
            if (k < K) {
                if (tail.bias) x += tail.bias[k];
                if (tail.res_n && live) {
                    const size_t idx = blocked ? (size_t)ni * KO * PQ + ((size_t)(k / 4) * PQ + pix) * 4 + (k & 3)
                                               : (size_t)ni * K * PQ + (size_t)k * PQ + pix;
                    x += tail.res_n[idx];
                }
                if (tail.relu) x = x > 0.f ? x : 0.f;
            }
            val[v] = x;
        }
    }
    store_tile_block(blocked, fast, orsrc, out_n, K, PQ, kw, h, live, ni, pix, val);
}

// TAILC: C is not a multiple of CB.  The last chunk then reaches past the input
// channels; its filter values are fetched one by one (never past the tensor) and
// cleared where the channel does not exist.  TAILC = false needs C % CB == 0 and
// keeps the steady state free of branches and of per-value work.
// MODE: 0 plain, 1 with the fused point-wise tail, 2 with the output re-mapping (see KernelArgs); three
// instantiations, so that the plain kernel carries none of the other two's registers or instructions.
template <class G, bool TAILC, int MODE>
__device__ __forceinline__ void conv_dma_body(const KernelArgs &a)
{
    constexpr bool FUSED = MODE == 1, REMAP = MODE == 2;
    extern __shared__ __align__(16) float lds[];

    const int lane = threadIdx.x & 63;
    const int wave_wg = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    __builtin_assume(wave_wg >= 0 && wave_wg < G::NT / 64);
    const int sc = wave_wg / G::NWG;                 // split group of this wave
    const int wave = wave_wg - sc * G::NWG;          // wave, thread within the group
    const int tid = wave * 64 + lane;
    const int wk = wave % G::WK, wp = wave / G::WK;
    const int h = lane >> 5, j = lane & 31;
    const int goffs = sc * G::GRP;                   // LDS offset (floats) of this group's stage buffers and counter

    const int C = a.s.C, H = a.s.H, W = a.s.W, K = a.s.K, P = a.s.P, Q = a.s.Q;
    const int CI = G::BLK ? (C + 3) / 4 * 4 : C;     // channels an image occupies in memory (blocked: whole pencils)

    // Workgroup -> tile.  Consecutive workgroup ids are dealt round-robin to the 8
    // XCDs, each with its own L2; the ids are first regrouped so that one XCD works
    // on neighbouring tiles (all channel tiles of a pixel tile share their input).
    unsigned bid = blockIdx.x;
    {
        const unsigned g8 = gridDim.x & ~7u;
        if (bid < g8) bid = (bid & 7u) * (g8 >> 3) + (bid >> 3);
    }
    // output re-mapping: the phases are one more grid dimension, fastest, so that the workgroups that read the same
    // tile of the input run side by side; phase ph has a filter of its own and its own offsets
    // Merged phases (eight k-waves, stride 2: four phases): a workgroup runs ALL phases of its pixel tile for two blocks
    // of 32 output channels, one (phase, block) per wave, so that the input window is staged once for the four phases
    // (as separate workgroups the phases with one or two taps are bound by their staging).  Waves 0..3 take phases
    // 0..3 of the first block, waves 4..7 phases 3..0 of the second: the SIMD that has the four-tap phase of one block
    // has the one-tap phase of the other.
    constexpr bool MERGED = REMAP && G::WK == 8;
    int ph = 0;
    if constexpr (REMAP && !MERGED) {
        const unsigned nb = (unsigned)a.onb, nph = nb * nb;      // phases per dimension that have a tap at all
        ph = (int)(bid % nph);
        bid /= nph;
    }
    const int kt = bid % a.ktiles;  bid /= a.ktiles;
    const int k0 = kt * G::KT;
    int kwv = k0 + wk * 32;                          // first output channel of this wave
    if constexpr (MERGED) {
        ph = (wk & 4) ? 3 - (wk & 3) : (wk & 3);
        kwv = (2 * kt + (wk >> 2)) * 32;
    }
    // the filter of this wave's phase (blocked weights: whole blocks of 32 output channels and pencils of 4 input channels)
    const float *const wp_ = a.w + (REMAP ? (size_t)ph * (G::BLK ? (size_t)((K + 31) / 32 * 32) * CI : (size_t)K * C) * G::RS : 0);
    // rectangular: image n, tile origin (p0, q0).  flat: first pixel m0 of M, which
    // lies in output row g0 (rows of all images numbered through) of image n
    int n, p0 = 0, q0 = 0, m0 = 0, g0 = 0, M = 0;
    if (G::FLAT) {
        // (the divisions run on the vector unit; the results are the same in every lane
        // and go back to scalar registers, or the buffer resource would not be uniform)
        m0 = (int)bid * G::NPIXF;
        M = a.s.N * G::OP * G::OQ;
        g0 = __builtin_amdgcn_readfirstlane(m0 / G::OQ);
        n = __builtin_amdgcn_readfirstlane(g0 / G::OP);
    } else {
        const int tq = bid % a.tilesQ;  bid /= a.tilesQ;
        const int tp = bid % a.tilesP;
        n = bid / a.tilesP;
        p0 = tp * G::TP;
        q0 = tq * G::TQ;
    }
    const int ih0 = p0 * G::ST - a.s.pad, iw0 = q0 * G::ST - a.s.pad;

    // Input staging plan: thread tid owns positions tid + i*NTG of the chunk's
    // [CB][PSP] window array; its byte offset from the chunk's first channel (of the
    // tile's first image), or an offset no buffer can reach where the window lies
    // outside the image.
    unsigned goff[G::ITEMS];
#pragma unroll
    for (int i = 0; i < G::ITEMS; ++i) {
        const int f = i * G::NTG + tid;
        // plain: [CB][PSP] floats, position pos of channel cc; blocked: [PS][4] floats
        const int cc = G::BLK ? 0 : f / G::PSP;
        const int pos = G::BLK ? f / 4 : f - cc * G::PSP;
        const int ci = G::BLK ? f % 4 : 0;
        const int hh = pos / G::LW, col = pos - hh * G::LW;
        int ih, img = 0;
        if (G::FLAT) {
            // window row hh belongs to the last image whose first row is not below it
            int gs = g0, start = 0;
#pragma unroll
            for (int u = 1; u < G::NSI; ++u) {
                const int gu = (n + u) * G::OP, su = (gu - g0) * G::ST + u * (G::R - G::ST);
                if (hh >= su) { img = u; gs = gu; start = su; }
            }
            ih = hh - start + (gs - (n + img) * G::OP) * G::ST - a.s.pad;
        } else {
            ih = ih0 + hh;
        }
        const int iw = iw0 + col;
        const bool ok = (f < G::CHF) & (pos < G::PS) & (n + img < a.s.N) & ((unsigned)ih < (unsigned)H) &
                        ((unsigned)iw < (unsigned)W);
        const unsigned off = G::BLK ? (unsigned)((((img * (CI / 4)) * H + ih) * W + iw) * 16 + ci * 4)
                                    : (unsigned)((((img * C + cc) * H + ih) * W + iw) * 4);
        goff[i] = ok ? off : 0x80000000u;
    }
    const float *in_n = a.in + (size_t)n * CI * H * W;
    const unsigned chan_bytes = (unsigned)(H * W) * 4u;

    // Stage the input window of channels [c0, c0 + CB) into buf.  Rectangular: the
    // resource ends at the image's last channel, so channels past C read as zeros.
    // Flat: the window spans images, so the resource runs on and the loads of channels
    // past C are given the unreachable offset instead.
    auto stage_b = [&](float *buf, int c0) {
        const unsigned span = G::FLAT ? 0x7fffffffu : (unsigned)(CI - c0) * chan_bytes;
        // the base is the same in every lane; saying so keeps the resource in scalar
        // registers (a resource the compiler takes for divergent is looped over lane by lane)
        __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(in_n + (size_t)c0 * H * W), 0, (int)span, 0x00020000);
#pragma unroll
        for (int i = 0; i < G::ITEMS; ++i) {
            const int f0 = i * G::NTG + wave * 64;          // first position of this wave's 64
            if (f0 < G::CHF) {
                float *dst = buf + goffs + f0 + (!G::BLK && f0 >= G::HC * G::PSP ? 32 : 0);
                unsigned off = goff[i];
                if (G::FLAT && !G::BLK) off = c0 + f0 / G::PSP < C ? off : 0x80000000u;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, CONVD_LDS(dst), 4, off, 0, 0, 0);
            }
        }
    };

    // Filter values of this lane: output channel k0 + wk*32 + j (clamped: rows past K
    // are computed and discarded), input channels c0 + h*HC .. + HC, all taps.
    int krow = kwv + j;
    krow = krow < K ? krow : K - 1;
    const float *w_lane = wp_ + ((size_t)krow * C + h * G::HC) * G::RS;
    const long long w_total = (long long)K * C * G::RS;
    const long long w_lane_idx = ((long long)krow * C + h * G::HC) * G::RS;
    // blocked weights: the 32 output channels of the wave are one block row kb; lane (j, h)
    // reads, for tap rs and channel cc of its half, float ((rs*4 + 2h + cc)*32 + j) of the
    // [R][S][4][32] block of (kb, c0/4): a per-lane constant plus a compile-time offset
    const unsigned wb_lane = (unsigned)((2 * h * 32 + j) * 4);
    // (a wave whose 32 channels all lie past K reads the last block that exists; its results are discarded)
    const int kblk = kwv / 32 < (K + 31) / 32 ? kwv / 32 : (K + 31) / 32 - 1;
    const float *wb_row = wp_ + (size_t)kblk * (CI / 4) * (G::RS * 128);
    auto load_a = [&](float (&dst)[G::NA], int c0) {
        if constexpr (G::BLK != 0) {
            __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(
                uniform_ptr(wb_row + (size_t)(c0 / 4) * (G::RS * 128)), 0, G::RS * 128 * 4, 0x00020000);
#pragma unroll
            for (int e = 0; e < G::NA; ++e)   // e = rs*2 + cc, the order the steps use them in
                dst[e] = __builtin_bit_cast(
                    float, __builtin_amdgcn_raw_buffer_load_b32(wr, (int)wb_lane, ((e / 2) * 128 + (e % 2) * 32) * 4, 0));
        } else if (!TAILC) {
            const float *p = w_lane + (size_t)c0 * G::RS;
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
            // one value at a time, the index clamped into the tensor; values of channels
            // that do not exist are cleared by mask_a when the chunk is used
            const long long base = w_lane_idx + (long long)c0 * G::RS;
#pragma unroll
            for (int e = 0; e < G::NA; ++e) {
                const long long idx = base + e;
                dst[e] = wp_[idx < w_total ? idx : w_total - 1];
            }
        }
    };
    auto mask_a = [&](float (&dst)[G::NA], const float (&src)[G::NA], int c0) {
#pragma unroll
        for (int e = 0; e < G::NA; ++e) dst[e] = (!TAILC || c0 + h * G::HC + e / G::RS < C) ? src[e] : 0.f;
    };

    // Everything below depends on how many pixel blocks the wave owns: PBW, or PBW2 for
    // the second pixel group of a variant with unequal waves (same protocol, same number
    // of chunks and meetings, fewer MFMAs per step).
    auto body = [&](auto pbw_tag, auto sh_tag) __attribute__((always_inline)) {
        constexpr int PBW = decltype(pbw_tag)::value;
        constexpr bool SH = decltype(sh_tag)::value != 0;   // the wave's last block is the tile's shared block (see SL)
        constexpr int shq = SH ? decltype(sh_tag)::value - 1 : 0;   // ... to which it adds in the steps t with t % 4 == shq
        // per-lane LDS read offsets (floats): pixel position plus the kk half
        int bbase[PBW];
    #pragma unroll
        for (int pb = 0; pb < PBW; ++pb) {
            // (the first pixel group always owns G::PBW blocks; a shared block is the tile's last)
            const int t = ((SH && pb == PBW - 1) ? G::WP * G::PBW : wp * G::PBW + pb) * 32 + j;
            int pix;
            if constexpr (G::FLAT) {
                int m = m0 + t;
                m = m < M ? m : M - 1;                       // past the last pixel: any valid position
                const int g = m / G::OQ, q = m - g * G::OQ;
                const int sI = g / G::OP - n;                // which of the tile's images
                pix = ((g - g0) * G::ST + sI * (G::R - G::ST)) * G::LW + q * G::ST;
            } else {
                const int py = t / G::TQ, px = t - py * G::TQ;
                pix = t < G::NPIX ? py * G::ST * G::LW + px * G::ST : 0;
            }
            bbase[pb] = pix * G::PXF + h * G::HOFF + goffs;   // (group offset folded in: buffers are then addressed
                                                     // as constant offsets from lds, as without splitting)
        }

        dma_floatx16 acc[PBW];
    #pragma unroll
        for (int pb = 0; pb < PBW; ++pb)
    #pragma unroll
            for (int v = 0; v < 16; ++v) acc[pb][v] = 0.f;

        // Chunk i lives in stage buffer i % 3 and in filter register set i % 3.
        //
        // The waves of a workgroup meet once per chunk, and the meeting is split in two so
        // that nobody stands still (a wave that has a matrix pipe to itself cannot hide a
        // barrier behind another wave):
        //   * at step TX of chunk i a wave ARRIVES: its own loads of chunk i+1 (LDS-direct
        //     input loads and filter loads, issued during chunk i-1) have landed and it has
        //     left chunk i-1 behind; it adds one to a counter in LDS and carries on;
        //   * at step TY > TX it checks that all waves have arrived, which by then they
        //     have unless one is a third of a chunk late.  Chunk i+1 is then readable and
        //     the buffer and register set of chunk i-1 are free: the loads of chunk i+2 are
        //     issued, and the operand fetch of chunk i+1's first steps follows under the
        //     last MFMAs of chunk i, so the matrix pipe sees no gap at a chunk boundary.
        // Within a chunk the B operands of step t+PF are fetched while step t multiplies.
        constexpr int NW = G::NWG;
        unsigned *meet = reinterpret_cast<unsigned *>(lds + goffs + 3 * G::BUF);  // arrivals so far, all chunks
        auto arrive = [&]() {
            // everything this wave has issued, the LDS-direct loads of the next chunk included, is
            // complete (the only vector-memory operations in flight here are those loads), then release
            wait_vmem_done();
            if (lane == 0) __hip_atomic_fetch_add(meet, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        };
        // The wait is bounded so that no wave can hang the GPU.  In a correct run the bound is never
        // reached: every wave of the group executes the same number of chunks and arrives exactly once
        // per chunk without waiting for anybody, so the count reaches every target after at most one
        // chunk's work of the slowest wave (microseconds; the bound is some 0.1 s).  Should it expire
        // all the same, the wave remembers it and stores NaN instead of sums over data it could not
        // know to be complete: a parity check or the caller sees the failure.
        bool late = false;
        auto all_arrived = [&](unsigned target) {
            bool seen = false;
            for (int spin = 0; spin < (1 << 22); ++spin) {
                if (__hip_atomic_load(meet, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= target) { seen = true; break; }
                __builtin_amdgcn_s_sleep(1);
            }
            late |= !seen;
        };
        auto step_off = [](int t) {   // LDS offset (floats) of reduction step t of a chunk
            if (G::BLK) return ((t / 2 / G::S) * G::LW + (t / 2) % G::S) * 4 + t % 2;   // tap t/2, channel t%2 of the half
            const int cc = t / G::RS, rs = t - cc * G::RS;
            return cc * G::PSP + (rs / G::S) * G::LW + rs % G::S;
        };
        auto fetch = [&](const float *buf, int t, float (&bv)[PBW]) {
    #pragma unroll
            for (int pb = 0; pb < PBW; ++pb) bv[pb] = buf[bbase[pb] + step_off(t)];
        };
        const int nch = (C + G::CB - 1) / G::CB;            // chunks in all
        const int nchl = nch > sc ? (nch - sc + G::SC - 1) / G::SC : 0;   // chunks of this split group
        // first channel of the group's local chunk i (past its last chunk: the layer's last
        // chunk again, staged into buffers nothing reads)
        auto chan0 = [&](int i) {
            const int g = i * G::SC + sc;
            return (g < nch ? g : nch - 1) * G::CB;
        };
        float bq[G::PF][PBW];   // B operands of the next PF steps, oldest first
        float a0[G::NA], a1[G::NA], a2[G::NA];
        float *b0 = lds, *b1 = lds + G::BUF, *b2 = lds + 2 * G::BUF;   // (+ goffs, added where they are used)
        if (tid == 0) *meet = 0u;
        stage_b(b0, chan0(0));
        load_a(a0, chan0(0));
        stage_b(b1, chan0(1));
        load_a(a1, chan0(1));
        wait_vmem_done();   // this wave's part of the first two stage buffers has landed
        __syncthreads();

        // The chunk loop, compiled for the taps that carry weights.  A forward pass uses all R*S of them.  The phases
        // of a strided layer's data gradient (output re-mapping) share one padded RT x RT filter shape, and a phase whose
        // first filter row and/or column is padding (all zeros) leaves those taps out of its reduction: SKIP = 2*row + column.
        auto run = [&](auto skip_tag) __attribute__((always_inline)) {
            constexpr int SKR = decltype(skip_tag)::value / 2, SKC = decltype(skip_tag)::value % 2;
            constexpr int NRV = G::R - SKR, NSV = G::S - SKC;        // filter rows and columns in use
            constexpr int NV = G::BLK ? 2 * NRV * NSV : G::HC * NRV * NSV;   // reduction steps of a chunk
            // i-th step in use -> step of the full filter (which register of the chunk's filter values, which tap offset)
            auto vt = [](int i) {
                if (G::BLK) {   // (a blocked chunk takes tap after tap, two channels of the lane's half per step)
                    const int u = i / 2;
                    return ((u / NSV + SKR) * G::S + u % NSV + SKC) * 2 + i % 2;
                }
                const int cc = i / (NRV * NSV), rem = i - cc * (NRV * NSV);
                return cc * G::RS + (rem / NSV + SKR) * G::S + rem % NSV + SKC;
            };
            constexpr int TY = NV - G::PF - 1 > NV / 2 ? NV - G::PF - 1 : NV / 2;
            constexpr int TX = TY * 3 / 5;
            static_assert(TX < TY && TY + G::PF <= NV && 2 * G::PF < NV, "arrive, check, then fetch the next chunk");
            auto chunk = [&](int i, const float *bufc, const float *bufn, float *bufnn, const float (&acr)[G::NA],
                             float (&ann)[G::NA]) __attribute__((always_inline)) {
                float ac[G::NA];
                mask_a(ac, acr, chan0(i));
    #pragma unroll
                for (int t = 0; t < NV; ++t) {
                    if (t == TX) arrive();
                    if (t == TY) {
                        all_arrived((unsigned)NW * (unsigned)(i + 1));
                        // past the last chunk the last one is staged again, into a buffer and a
                        // register set that nothing reads any more (no special case)
                        const int cn = chan0(i + 2);
                        stage_b(bufnn, cn);
                        load_a(ann, cn);
                    }
                    float bnew[PBW];
                    if (t + G::PF < NV) fetch(bufc, vt(t + G::PF), bnew);
                    else fetch(bufn, vt(t + G::PF - NV), bnew);   // past the last chunk: stale but in-bounds, never used
                    const bool last = !SH || (t & 3) == shq;   // (a shared last block: this wave's quarter of the steps)
    #pragma unroll
                    for (int pb = 0; pb < PBW; ++pb)
                        if (pb < PBW - 1 || last)
                            acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(ac[vt(t)], bq[0][pb], acc[pb], 0, 0, 0);
    #pragma unroll
                    for (int pb = 0; pb < PBW; ++pb)
                        if (pb < PBW - 1 || last) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                        }
    #pragma unroll
                    for (int pb = 0; pb < PBW; ++pb) {
    #pragma unroll
                        for (int d = 0; d + 1 < G::PF; ++d) bq[d][pb] = bq[d + 1][pb];
                        bq[G::PF - 1][pb] = bnew[pb];
                    }
                }
            };
    #pragma unroll
            for (int d = 0; d < G::PF; ++d) fetch(b0, vt(d), bq[d]);
            for (int ci = 0; ci < nchl; ci += 3) {
                chunk(ci, b0, b1, b2, a0, a2);
                if (ci + 1 < nchl) chunk(ci + 1, b1, b2, b0, a1, a0);
                if (ci + 2 < nchl) chunk(ci + 2, b2, b0, b1, a2, a1);
            }
        };
        if constexpr (REMAP && G::R > 1 && G::S > 1) {
            // phase (pa, pb) of the input positions has ceil((ofr - pa) / ost) filter rows; the padded shape has R
            const int nbp = a.onb, pa = ph / nbp, pb_ = ph - pa * nbp;
            const int skr = G::R - (a.ofr - pa + a.ost - 1) / a.ost, skc = G::S - (a.ofr - pb_ + a.ost - 1) / a.ost;
            const int sk = __builtin_amdgcn_readfirstlane((skr > 0 ? 2 : 0) + (skc > 0 ? 1 : 0));
            // (a blocked chunk has two steps per tap: a single tap is too short a chunk for the meeting protocol, so the
            // 2 x 2 filter's one-tap phase leaves out its padded row only and multiplies one padded tap)
            constexpr bool BOTH = !(G::BLK && (G::R - 1) * (G::S - 1) < 2);
            if (sk == 0) run(IntTag<0>{});
            else if (sk == 1) run(IntTag<1>{});
            else if (sk == 2 || !BOTH) run(IntTag<2>{});
            else run(IntTag<(BOTH ? 3 : 2)>{});
        } else {
            run(IntTag<0>{});
        }

        if constexpr (G::SL != 0) {
            // The shared block: pixel groups 5, 6, 7 hand their quarter sums to group 4 through LDS (the stage
            // buffers, free once every wave is here and its re-staged loads have landed), added in a fixed order.
            // Every wave of the workgroup passes both barriers, whichever body it runs.
            wait_vmem_done();
            __syncthreads();
            if constexpr (SH) {
                if (shq > 0) {
    #pragma unroll
                    for (int v = 0; v < 16; ++v) lds[((shq - 1) * 16 + v) * 64 + lane] = acc[PBW - 1][v];
                }
            }
            __syncthreads();
            if constexpr (SH) {
                if (shq == 0) {
    #pragma unroll
                    for (int g = 0; g < 3; ++g)
    #pragma unroll
                        for (int v = 0; v < 16; ++v) acc[PBW - 1][v] += lds[(g * 16 + v) * 64 + lane];
                }
            }
        }
        if (G::SC > 1) {
            // Sum the split groups' partial tiles into group 0, as a tree: at every level the upper half of
            // the groups still in play write their tiles to LDS (the stage buffers are free once every wave
            // is here) and the lower half add them, group g taking group g + half's.  The order of the
            // additions is fixed, so the result does not depend on timing.  Past its last chunk a wave has
            // staged that chunk again into buffers nothing reads: those loads must have landed before the
            // buffers are written as the exchange area.
            wait_vmem_done();
            __syncthreads();
            float *red = lds;
    #pragma unroll
            for (int half = G::SC / 2; half >= 1; half /= 2) {
                if (sc >= half && sc < 2 * half) {
                    float *mine = red + ((sc - half) * G::NWG + wave) * PBW * 1024;
    #pragma unroll
                    for (int pb = 0; pb < PBW; ++pb)
    #pragma unroll
                        for (int v = 0; v < 16; ++v) mine[(pb * 16 + v) * 64 + lane] = acc[pb][v];
                }
                __syncthreads();
                if (sc < half) {
                    const float *theirs = red + (sc * G::NWG + wave) * PBW * 1024;
    #pragma unroll
                    for (int pb = 0; pb < PBW; ++pb) {
    #pragma unroll
                        for (int v = 0; v < 16; ++v) acc[pb][v] += theirs[(pb * 16 + v) * 64 + lane];
                        __builtin_amdgcn_sched_barrier(0);   // one block at a time: 16 loads in flight, not 16*PBW
                    }
                }
                if (half > 1) __syncthreads();   // the next level writes where this one has read
            }
            if (sc > 0) return;
        }

        // ---- epilogue (see write_block) ----
        if (late) {   // a meeting's bounded wait expired (see all_arrived): no sums, NaN
#pragma unroll
            for (int pb = 0; pb < PBW; ++pb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[pb][v] = __builtin_nanf("");
        }
        const int kw = kwv;
        const int KO = a.out_blocked ? (K + 3) / 4 * 4 : K;      // channels an output image occupies
        // output re-mapping, see KernelArgs
        const int ost = REMAP ? a.ost : 0, nb = REMAP ? a.onb : 1, OH = REMAP ? a.OH : 0, OW = REMAP ? a.OW : 0;
        const int ooh = REMAP ? a.ooh + ph / nb : 0, oow = REMAP ? a.oow + ph % nb : 0;   // (ooh, oow: those of phase 0)
        const int OPQ = REMAP ? OH * OW : P * Q;                 // pixels of an output channel plane
        const bool fast = (kw + 32 <= K) & ((long long)KO * OPQ * 4 * G::NSI < (1ll << 31));
        float *out_n = a.out + (size_t)n * KO * OPQ;
        __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(out_n), 0, 0x7fffffff, 0x00020000);
        const Tail tail{a.bias, a.residual ? a.residual + (size_t)n * KO * OPQ : nullptr, a.relu};
#pragma unroll
        for (int pb = 0; pb < PBW; ++pb) {
            if (SH && pb == PBW - 1 && shq != 0) continue;   // (the shared block is stored by the group that summed it)
            const int t = ((SH && pb == PBW - 1) ? G::WP * G::PBW : wp * G::PBW + pb) * 32 + j;
            bool live;
            int ni = 0, pix;      // image of the pixel relative to n, pixel index inside its image
            if constexpr (G::FLAT) {
                const int m = m0 + t, pq = G::OP * G::OQ;
                const int nm = m / pq;
                live = m < M;
                ni = nm - n;
                pix = m - nm * pq;
            } else {
                const int py = t / G::TQ, px = t - py * G::TQ;
                const int p = p0 + py, q = q0 + px;
                live = t < G::NPIX && p < P && q < Q;
                pix = p * Q + q;
            }
            if constexpr (REMAP) {
                const int pp = pix / Q, qq = pix - pp * Q;
                const int oh = pp * ost + ooh, ow = qq * ost + oow;
                live = live && (unsigned)oh < (unsigned)OH && (unsigned)ow < (unsigned)OW;
                pix = live ? oh * OW + ow : 0;
            }
            write_block<FUSED>(a.out_blocked != 0, fast, orsrc, out_n, K, OPQ, kw, h, live, ni, pix, acc[pb], tail);
        }
    };
    if constexpr (G::SL != 0) {
        // (one instantiation of the body per quarter: which steps a wave adds to the shared block is then fixed at compile time)
        if (wp < 4) body(IntTag<G::PBW>{}, IntTag<0>{});
        else if (wp == 4) body(IntTag<G::PBW + 1>{}, IntTag<1>{});
        else if (wp == 5) body(IntTag<G::PBW + 1>{}, IntTag<2>{});
        else if (wp == 6) body(IntTag<G::PBW + 1>{}, IntTag<3>{});
        else body(IntTag<G::PBW + 1>{}, IntTag<4>{});
    } else {
        if (G::PBW2 > 0 && wp == 1) body(IntTag<(G::PBW2 > 0 ? G::PBW2 : G::PBW)>{}, IntTag<0>{});
        else body(IntTag<G::PBW>{}, IntTag<0>{});
    }
}

template <class G, bool TAILC, bool FUSED>
__global__ void __launch_bounds__(G::NT, G::WPE) conv_dma_kernel(const KernelArgs a)
{
    conv_dma_body<G, TAILC, FUSED ? 1 : 0>(a);
}

// the same with the output re-mapping (the phases of a strided layer's data gradient)
template <class G, bool TAILC>
__global__ void __launch_bounds__(G::NT, G::WPE) conv_dma_remap_kernel(const KernelArgs a)
{
    conv_dma_body<G, TAILC, 2>(a);
}

// ---------------------------------------------------------------------------
// Host side: launcher and the table entry of one compiled variant.
// ---------------------------------------------------------------------------
inline bool has_tail(const KernelArgs &a) { return a.bias != nullptr || a.residual != nullptr || a.relu != 0; }

// Workgroups above the 64 KB default need the kernel's dynamic LDS limit raised (no allocation
// involved).  Once per kernel and device is enough: `done` is the calling launcher's own bit mask of
// the devices it has been raised on (devices past 63 are asked every time).
inline hipError_t raise_lds_limit(const void *kernel, size_t bytes, std::atomic<unsigned long long> &done)
{
    if (bytes <= 64 * 1024) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = dev >= 0 && dev < 64 ? 1ull << dev : 0ull;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
}

template <class G, bool TAILC>
static hipError_t launch_dma_remap(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    static std::atomic<unsigned long long> raised{0};
    if (hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(&conv_dma_remap_kernel<G, TAILC>), G::LDS_BYTES, raised);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((conv_dma_remap_kernel<G, TAILC>), dim3(grid), dim3(G::NT), G::LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class G, bool TAILC, bool FUSED>
static hipError_t launch_dma_tf(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    static std::atomic<unsigned long long> raised{0};
    if (hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(&conv_dma_kernel<G, TAILC, FUSED>), G::LDS_BYTES, raised);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((conv_dma_kernel<G, TAILC, FUSED>), dim3(grid), dim3(G::NT), G::LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class G, bool TAILC>
static hipError_t launch_dma_t(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    if (a.ost) {   // output re-mapping: compiled for the stride-1 variants of small filters only
        if constexpr (G::ST == 1 && G::R <= 4 && G::SL == 0) {
            return has_tail(a) ? hipErrorInvalidValue : launch_dma_remap<G, TAILC>(a, grid, stream);
        } else {
            return hipErrorInvalidValue;
        }
    }
    return has_tail(a) ? launch_dma_tf<G, TAILC, true>(a, grid, stream) : launch_dma_tf<G, TAILC, false>(a, grid, stream);
}

template <class G>
static hipError_t launch_dma(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    if constexpr (G::BLK != 0) {
        return launch_dma_t<G, false>(a, grid, stream);   // blocked layouts hold whole pencils: no ragged chunk
    } else {
        return a.s.C % G::CB == 0 ? launch_dma_t<G, false>(a, grid, stream) : launch_dma_t<G, true>(a, grid, stream);
    }
}

template <class G>
static size_t lds_dma(const Shape &) { return G::LDS_BYTES; }

template <class G>
constexpr Variant make_dma_variant(const char *name)
{
    return Variant{name, G::R, G::S, G::ST, G::TP, G::FLAT ? 0 : G::TQ, G::KT, G::NPB, G::CB, G::PAIR, G::NT, G::OCC,
                   G::CHF / G::CB, G::IMG, G::PADC, &lds_dma<G>, &launch_dma<G>, 0, G::BLK, (G::WK == 8 && G::ST == 1 && G::R <= 4) ? 1 : 0};
}

}  // namespace convd
