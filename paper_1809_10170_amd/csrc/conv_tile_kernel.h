// Direct-convolution forward kernels for gfx950 (MI355X): fp32 MFMA, LDS-staged
// halo tiles, no workspace.
//
// The computation is the paper's Algorithm 1 (Section 3): six loops around one
// multiply-accumulate.  The paper blocks the output-channel and output-column loops
// for the register file, the input-channel loop for the cache, and runs output
// channels in parallel (Section 3.1.2, Section 3.2, Algorithm 3).  On this GPU the
// same three decisions become:
//   * register block  -> a (32*KBW) x (32*PBW) accumulator tile per wave, held in
//     VGPRs as 32x32 MFMA results; rows are output channels, columns output pixels;
//   * cache block     -> CB input channels staged per step into LDS: the input
//     halo window of the workgroup's pixel tile and the matching filter slice;
//   * parallel loop   -> the grid: every (image, pixel tile, channel tile) is an
//     independent workgroup.
// Because the halo window sits in LDS once and every filter tap reads it at a
// different constant offset, nothing like an im2col matrix ever exists: that is
// the paper's "zero memory overhead" (Sections 1, 2.2) carried over.
//
// v_mfma_f32_32x32x2_f32 operand layout used here: lane l supplies A[i = l%32][kk = l/32]
// and B[kk = l/32][j = l%32]; accumulator register v of lane l holds
// D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].  A = filter slice (i = output channel),
// B = input values (j = output pixel).  The two kk lanes of one instruction take two
// neighbouring input channels at one filter tap (PAIR_C), or, for layers with very
// few input channels, two neighbouring filter columns of one channel (PAIR_S, an odd
// filter width being padded with a zero weight).  Any order of the C*R*S additions
// is a correct convolution (Section 3, "any permutation of the loops").
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "variant.h"

namespace convd {

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int R_, int S_, int ST_, int TP_, int TQ_, int KBW_, int PBW_, int WK_, int WP_, int CB_,
          int PAIR_, int OCC_, int PREF_>
struct Geom {
    static constexpr int PREF = PREF_;                 // 0: load-store-compute; 1: next chunk prefetched into registers;
                                                       // 2: two LDS buffers, staging interleaved with the MFMAs
    static constexpr int R = R_, S = S_, ST = ST_, TP = TP_, TQ = TQ_;
    static constexpr int KBW = KBW_, PBW = PBW_, WK = WK_, WP = WP_, CB = CB_, PAIR = PAIR_, OCC = OCC_;
    static constexpr int NT = 64 * WK * WP;            // threads per workgroup
    static constexpr int WPE = (OCC * WK * WP + 3) / 4; // waves per SIMD the register budget must allow
    // unroll factor of the channel loop inside a chunk (full when staging is interleaved tap by tap)
    static constexpr int UNROLL_OUTER = PREF_ == 2 ? (PAIR_ == PAIR_C ? CB_ / 2 : CB_) : 1;
    static constexpr int SB = 8;                       // staging loads in flight per thread
    static constexpr int KT = 32 * KBW * WK;           // output channels per workgroup
    static constexpr int NPB = PBW * WP;               // 32-pixel blocks per workgroup
    static constexpr int NPIX = TP * TQ;               // real pixels in the tile
    static constexpr int S2 = (S + 1) / 2;
    static constexpr int SPAN = PAIR == PAIR_S ? 2 * S2 : S;
    static constexpr int LH = (TP - 1) * ST + R;       // halo window rows
    static constexpr int LW = (TQ - 1) * ST + SPAN;    // halo window columns
    static constexpr int LWP = LW;                     // LDS row pitch
    static constexpr int PS = LH * LWP;                // LDS channel-plane stride
    static constexpr int RS = R * S;
    static constexpr int STEPS = PAIR == PAIR_C ? (CB / 2) * RS : CB * R * S2;   // MFMA k-steps per chunk
    static constexpr int KP = KT + 1;                  // LDS pitch of one filter k-row (odd: spreads banks)
    static constexpr int LDS_A = STEPS * 2 * KP;       // floats
    static constexpr int LDS_B = CB * PS;              // floats
    static constexpr int NBUF = PREF_ == 2 ? 2 : 1;     // LDS stage buffers
    static constexpr int LDS_DUMP = 64;                // one word per lane: where masked-off lanes store
    static constexpr int LDS_BUF = LDS_A + LDS_B + LDS_DUMP;   // floats per stage buffer: filter, input, dump
    static constexpr size_t LDS_BYTES = sizeof(float) * (size_t)LDS_BUF * NBUF;
    static_assert(NPB * 32 >= NPIX, "pixel blocks must cover the tile");
    static_assert(PAIR == PAIR_S || CB % 2 == 0, "channel pairing needs an even chunk");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
};

typedef float floatx4 __attribute__((ext_vector_type(4)));

// One global load of WV consecutive filter values (WV = 1 or 4).
template <int WV> struct WLoad;
template <> struct WLoad<1> {
    typedef float type;
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ float get(float v, int) { return v; }
};
template <> struct WLoad<4> {
    typedef floatx4 type;
    static __device__ __forceinline__ floatx4 ld(const float *p) { return *reinterpret_cast<const floatx4 *>(p); }
    static __device__ __forceinline__ float get(floatx4 v, int u) { return v[u]; }
};

// G: tile geometry.  WV: filter values per global load; 4 needs a 16-byte aligned
// filter pointer, C*R*S and CB*R*S multiples of 4 and C a multiple of CB (the launcher
// checks), 1 works for anything.
template <class G, int WV>
__global__ void __launch_bounds__(G::NT, G::WPE) conv_tile_kernel(const KernelArgs a)
{
    extern __shared__ __align__(16) float lds[];
    float *ldsA = lds;                 // [STEPS][2][KP]   filter slice, k-lane major
    float *ldsB = lds + G::LDS_A;      // [CB][LH][LWP]    input halo window

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wk = wave % G::WK, wp = wave / G::WK;
    const int h = lane >> 5, j = lane & 31;

    const int C = a.s.C, H = a.s.H, W = a.s.W, K = a.s.K, P = a.s.P, Q = a.s.Q;

    // workgroup -> (channel tile, pixel tile column, pixel tile row, image)
    unsigned bid = blockIdx.x;
    const int kt = bid % a.ktiles;  bid /= a.ktiles;
    const int tq = bid % a.tilesQ;  bid /= a.tilesQ;
    const int tp = bid % a.tilesP;
    const int n = bid / a.tilesP;
    const int p0 = tp * G::TP, q0 = tq * G::TQ, k0 = kt * G::KT;
    const int ih0 = p0 * G::ST - a.s.pad, iw0 = q0 * G::ST - a.s.pad;

    const float *in_n = a.in + (size_t)n * C * H * W;
    const float *w_k = a.w + (size_t)k0 * C * G::RS;

    // per-lane LDS read bases
    int bbase[G::PBW];
#pragma unroll
    for (int pb = 0; pb < G::PBW; ++pb) {
        const int t = (wp * G::PBW + pb) * 32 + j;
        const int py = t / G::TQ, px = t - py * G::TQ;
        const int pix = t < G::NPIX ? py * G::ST * G::LWP + px * G::ST : 0;
        bbase[pb] = pix + h * (G::PAIR == PAIR_C ? G::PS : 1);
    }
    const int abase = h * G::KP + wk * G::KBW * 32 + j;

    floatx16 acc[G::KBW][G::PBW];
#pragma unroll
    for (int kb = 0; kb < G::KBW; ++kb)
#pragma unroll
        for (int pb = 0; pb < G::PBW; ++pb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[kb][pb][v] = 0.f;

    if (G::PAIR == PAIR_S && (G::S & 1)) {
        // the zero weight that pads an odd filter width is written once
        for (int e = tid; e < G::LDS_A; e += G::NT) ldsA[e] = 0.f;
        __syncthreads();   // other threads stage real weights into these rows next
    }

    // ---- staging: global -> registers -> LDS ----
    // Work is dealt to waves by rows, so that everything about an element except its
    // column is wave-uniform (scalar registers) or a compile-time constant: an input
    // row is one (channel, halo row) pair read by consecutive lanes; a filter row is
    // the CB*R*S contiguous values of one output channel.
    constexpr int NW = G::NT / 64;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // Re-read through an opaque scalar wherever elements are enumerated: hoisted out of
    // the chunk loop, the per-element scalars would not fit the scalar register file.
    auto wave_id = [&]() { int t = wave_u; asm volatile("" : "+s"(t)); return t; };

    // input halo window: ROWS rows of LW columns, SEGS lane-segments per row; narrow
    // windows put two channels (sub = 0, 1) side by side in one 64-lane access
    constexpr int SUBS = (G::LW <= 32 && G::CB % 2 == 0) ? 2 : 1;
    constexpr int SEGW = 64 / SUBS;
    constexpr int SEGS = (G::LW + SEGW - 1) / SEGW;
    constexpr int ROWS = (G::CB / SUBS) * G::LH;
    constexpr int ROW_IT = (ROWS + NW - 1) / NW;
    constexpr int NB_IT = ROW_IT * SEGS;
    const int sub = SUBS == 2 ? (lane >> 5) : 0;
    const int lcol = SUBS == 2 ? (lane & 31) : lane;
    const int in_lane_goff = sub * H * W + lcol;
    const int in_lane_loff = sub * G::PS + lcol;

    // Validity and address of input element i of this lane; loads return the raw
    // value (from a safe address when invalid) and the zero fill happens at store
    // time, so that nothing has to touch a prefetched register before its store.
    auto in_addr = [&](int wave_s, int c0, int i, bool &ok) -> unsigned {
        const int ir = i / SEGS, seg = i - ir * SEGS;
        const int rowg = ir * NW + wave_s;
        const int cg = rowg / G::LH, hh = rowg - cg * G::LH;
        const int ih = ih0 + hh;
        const int col = seg * SEGW + lcol;
        const int iw = iw0 + col;
        ok = (rowg < ROWS) & ((unsigned)ih < (unsigned)H) & (c0 + cg * SUBS + sub < C) &
             (col < G::LW) & ((unsigned)iw < (unsigned)W);
        const int off = ((c0 + cg * SUBS) * H + ih) * W + iw0 + seg * SEGW + in_lane_goff;
        return ok ? (unsigned)off : 0u;
    };
    auto in_load = [&](int wave_s, int c0, int i) -> float {
        bool ok;
        return in_n[in_addr(wave_s, c0, i, ok)];
    };
    auto in_store = [&](float *dstB, int wave_s, int c0, int i, float v) {
        bool ok;
        (void)in_addr(wave_s, c0, i, ok);
        const int ir = i / SEGS, seg = i - ir * SEGS;
        const int rowg = ir * NW + wave_s;
        const int cg = rowg / G::LH, hh = rowg - cg * G::LH;
        // masked-off lanes store to their dump word: no branch, the chunk stays one block
        const bool act = (rowg < ROWS) & (seg * SEGW + lcol < G::LW);
        const int idx = cg * SUBS * G::PS + hh * G::LWP + seg * SEGW + in_lane_loff;
        dstB[act ? idx : G::LDS_B + lane] = ok ? v : 0.f;
    };

    // filter slice: KT rows of CRS values, read WV at a time; short rows are packed
    // RPI to a 64-lane access, long rows take WSEGS accesses
    constexpr int CRS = G::CB * G::RS;
    static_assert(CRS % WV == 0, "vector filter loads must not straddle output channels");
    typedef typename WLoad<WV>::type wvec;
    constexpr int V = CRS / WV;
    constexpr int RPI = V <= 64 ? 64 / V : 1;
    constexpr int WSEGS = V <= 64 ? 1 : (V + 63) / 64;
    constexpr int KGRPS = (G::KT + RPI - 1) / RPI;
    constexpr int KG_IT = (KGRPS + NW - 1) / NW;
    constexpr int NA_IT = KG_IT * WSEGS;
    const int ksub = V <= 64 ? lane / V : 0;
    const int jl = V <= 64 ? lane - ksub * V : lane;
    const bool wlane_ok = ksub < RPI;
    const int w_lane_goff = ksub * C * G::RS + jl * WV;
    int aslot[WSEGS][WV];   // LDS position of each value this lane loads, per segment
#pragma unroll
    for (int seg = 0; seg < WSEGS; ++seg)
#pragma unroll
        for (int u = 0; u < WV; ++u) {
            const int jj = (seg * 64 + jl) * WV + u;
            const int cc = jj / G::RS, rs = jj - cc * G::RS;
            int slot;
            if (G::PAIR == PAIR_C) {
                slot = ((cc >> 1) * G::RS + rs) * 2 + (cc & 1);
            } else {
                const int r = rs / G::S, ss = rs - r * G::S;
                slot = ((cc * G::R + r) * G::S2 + (ss >> 1)) * 2 + (ss & 1);
            }
            aslot[seg][u] = jj < CRS ? slot * G::KP + ksub : 0;
        }

    auto w_addr = [&](int wave_s, int c0, int i, bool &ok) -> unsigned {
        const int ik = i / WSEGS, seg = i - ik * WSEGS;
        const int kg = ik * NW + wave_s;
        const int kk = kg * RPI + ksub;
        const int jj = (seg * 64 + jl) * WV;
        // with WV = 4 the launcher guarantees C % CB == 0, so a load never straddles the
        // end of the channels; with WV = 1 the last test cuts the channel tail
        ok = wlane_ok & (kk < G::KT) & (k0 + kk < K) & (jj < CRS) & (jj < (C - c0) * G::RS);
        const int off = (kg * RPI * C + c0) * G::RS + seg * 64 * WV + w_lane_goff;
        return ok ? (unsigned)off : 0u;
    };
    auto w_load = [&](int wave_s, int c0, int i) -> wvec {
        bool ok;
        return WLoad<WV>::ld(w_k + w_addr(wave_s, c0, i, ok));
    };
    auto w_store = [&](float *dstA, int wave_s, int c0, int i, wvec v) {
        bool ok;
        (void)w_addr(wave_s, c0, i, ok);
        const int ik = i / WSEGS, seg = i - ik * WSEGS;
        const int kg = ik * NW + wave_s;
        const int kk = kg * RPI + ksub;
#pragma unroll
        for (int u = 0; u < WV; ++u) {
            const bool act = wlane_ok & (kk < G::KT) & ((seg * 64 + jl) * WV + u < CRS);
            dstA[act ? aslot[seg][u] + kg * RPI : G::LDS_A + G::LDS_B + lane] = ok ? WLoad<WV>::get(v, u) : 0.f;
        }
    };

    // ---- the reduction over one staged chunk: STEPS rank-2 updates of the tile ----
    // Outer loop over channel pairs (PAIR_C) or channels (PAIR_S) is a real loop, the
    // filter taps inside it are unrolled with constant LDS offsets.
    constexpr int OUTER = G::PAIR == PAIR_C ? G::CB / 2 : G::CB;
    constexpr int INNER = G::STEPS / OUTER;                       // taps (PAIR_C) or tap pairs (PAIR_S)
    constexpr int B_OUTER = G::PAIR == PAIR_C ? 2 * G::PS : G::PS; // LDS floats per outer step, input
    constexpr int A_OUTER = INNER * 2 * G::KP;                    // LDS floats per outer step, filter
    // LDS -> register operand fetches for tap t of outer step o
    auto fetch_a = [&](const float *srcA, int o, int t, float (&av)[G::KBW]) {
        const float *pa = srcA + abase + o * A_OUTER;
#pragma unroll
        for (int kb = 0; kb < G::KBW; ++kb) av[kb] = pa[t * 2 * G::KP + kb * 32];
    };
    auto fetch_b = [&](const float *srcB, int o, int t, float (&bv)[G::PBW]) {
        const float *pbase = srcB + o * B_OUTER;
        int boff;
        if (G::PAIR == PAIR_C) {
            const int r = t / G::S, ss = t - r * G::S;
            boff = r * G::LWP + ss;
        } else {
            const int r = t / G::S2, s2 = t - r * G::S2;
            boff = r * G::LWP + 2 * s2;
        }
#pragma unroll
        for (int pb = 0; pb < G::PBW; ++pb) bv[pb] = pbase[bbase[pb] + boff];
    };
    // Software-pipelined: while the MFMAs of one tap issue, the input operands of the
    // next tap and the filter operand of the tap after it are fetched; the scheduling
    // hints pin one LDS read behind each MFMA.  Fetches past the end of the chunk are
    // clamped to its last outer step (their values are never used).
    auto compute = [&](const float *srcA, const float *srcB, auto &&side_work) {
        float a0[G::KBW], a1[G::KBW], b0[G::PBW];
        fetch_a(srcA, 0, 0, a0);
        fetch_b(srcB, 0, 0, b0);
        fetch_a(srcA, (1 / INNER) < OUTER ? 1 / INNER : OUTER - 1, 1 % INNER, a1);
#pragma unroll G::UNROLL_OUTER
        for (int o = 0; o < OUTER; ++o) {
#pragma unroll
            for (int t = 0; t < INNER; ++t) {
                float a2[G::KBW], b1[G::PBW];
                side_work(o, t);
                // taps are numbered o*INNER + t; fetch tap +1 (input) and tap +2 (filter)
                const int o1 = o + (t + 1) / INNER, o2 = o + (t + 2) / INNER;
                fetch_b(srcB, o1 < OUTER ? o1 : OUTER - 1, (t + 1) % INNER, b1);
                fetch_a(srcA, o2 < OUTER ? o2 : OUTER - 1, (t + 2) % INNER, a2);
#pragma unroll
                for (int kb = 0; kb < G::KBW; ++kb)
#pragma unroll
                    for (int pb = 0; pb < G::PBW; ++pb)
                        acc[kb][pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[kb], b0[pb], acc[kb][pb], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < G::KBW * G::PBW; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                    if (G::PREF == 2) {
                        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);   // a little address arithmetic
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one global load
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // one LDS store
                    }
                }
#pragma unroll
                for (int kb = 0; kb < G::KBW; ++kb) { a0[kb] = a1[kb]; a1[kb] = a2[kb]; }
#pragma unroll
                for (int pb = 0; pb < G::PBW; ++pb) b0[pb] = b1[pb];
            }
        }
    };
    auto no_side_work = [](int, int) {};

    if (G::PREF == 2 && WV == 4) {
        // Two LDS stage buffers.  A wave that shares its SIMD with a wave issuing MFMAs
        // back to back gets almost no issue slots, so staging cannot be left to "the
        // other" wave: every wave stages in the shadow of its own MFMAs.  During the
        // taps of chunk i a wave first stores the registers holding chunk i+1 into the
        // other buffer, then reloads them from global memory with chunk i+2.  Past the
        // last chunk the chunk index is clamped: redundant loads of valid memory and
        // stores into a buffer nobody reads again, in exchange for branch-free code.
        constexpr int BUF = G::LDS_BUF;                    // floats per stage buffer
        constexpr int NEL = NB_IT + NA_IT;                 // staged elements per thread
        constexpr int ST_TAPS = G::STEPS / 3 > 0 ? G::STEPS / 3 : 1;   // taps that carry stores
        constexpr int SPT = (NEL + ST_TAPS - 1) / ST_TAPS;             // elements per such tap
        constexpr int LD_TAPS = ST_TAPS;                               // taps that carry loads
        constexpr int LPT = (NEL + LD_TAPS - 1) / LD_TAPS;
        constexpr int LD_T0 = (NEL + SPT - 1) / SPT;                   // first tap with loads
        static_assert(LD_T0 + (NEL + LPT - 1) / LPT <= G::STEPS, "staging does not fit the taps of a chunk");
        const int c_last = ((C - 1) / G::CB) * G::CB;
        float vb[NB_IT];
        wvec va[NA_IT];
        {
            const int ws = wave_id();
#pragma unroll
            for (int i = 0; i < NB_IT; ++i) vb[i] = in_load(ws, 0, i);
#pragma unroll
            for (int i = 0; i < NA_IT; ++i) va[i] = w_load(ws, 0, i);
#pragma unroll
            for (int i = 0; i < NB_IT; ++i) in_store(ldsB, ws, 0, i, vb[i]);
#pragma unroll
            for (int i = 0; i < NA_IT; ++i) w_store(ldsA, ws, 0, i, va[i]);
            const int c1 = G::CB < C ? G::CB : c_last;
#pragma unroll
            for (int i = 0; i < NB_IT; ++i) vb[i] = in_load(ws, c1, i);
#pragma unroll
            for (int i = 0; i < NA_IT; ++i) va[i] = w_load(ws, c1, i);
        }
        __syncthreads();
        int cur = 0;
        for (int c0 = 0; c0 < C; c0 += G::CB, cur ^= 1) {
            const int c1 = c0 + G::CB < C ? c0 + G::CB : c_last;           // chunk held in registers
            const int c2 = c0 + 2 * G::CB < C ? c0 + 2 * G::CB : c_last;   // chunk to load next
            float *curA = ldsA + cur * BUF, *curB = ldsB + cur * BUF;
            float *nxtA = ldsA + (cur ^ 1) * BUF, *nxtB = ldsB + (cur ^ 1) * BUF;
            const int ws = wave_id();
            compute(curA, curB, [&](int o, int t) {
                const int tap = o * INNER + t;   // compile-time when the outer loop is unrolled
#pragma unroll
                for (int e = 0; e < NEL; ++e) {
                    if (e / SPT == tap) {
                        if (e < NB_IT) in_store(nxtB, ws, c1, e, vb[e]);
                        else w_store(nxtA, ws, c1, e - NB_IT, va[e - NB_IT]);
                    }
                    if (e / LPT + LD_T0 == tap) {
                        if (e < NB_IT) vb[e] = in_load(ws, c2, e);
                        else va[e - NB_IT] = w_load(ws, c2, e - NB_IT);
                    }
                }
            });
            __syncthreads();
        }
    } else
    if (G::PREF && WV == 4) {
        // Software pipeline: the next chunk's global loads are in flight while this
        // chunk's MFMAs run; their LDS stores follow the barrier that ends the reads.
        float vb[NB_IT];
        wvec va[NA_IT];
        {
            const int ws = wave_id();
#pragma unroll
            for (int i = 0; i < NB_IT; ++i) vb[i] = in_load(ws, 0, i);
#pragma unroll
            for (int i = 0; i < NA_IT; ++i) va[i] = w_load(ws, 0, i);
        }
        for (int c0 = 0; c0 < C; c0 += G::CB) {
            {
                const int ws = wave_id();
#pragma unroll
                for (int i = 0; i < NB_IT; ++i) in_store(ldsB, ws, c0, i, vb[i]);
#pragma unroll
                for (int i = 0; i < NA_IT; ++i) w_store(ldsA, ws, c0, i, va[i]);
            }
            __syncthreads();
            if (c0 + G::CB < C) {
                const int ws = wave_id();
#pragma unroll
                for (int i = 0; i < NB_IT; ++i) vb[i] = in_load(ws, c0 + G::CB, i);
#pragma unroll
                for (int i = 0; i < NA_IT; ++i) va[i] = w_load(ws, c0 + G::CB, i);
            }
            compute(ldsA, ldsB, no_side_work);
            __syncthreads();
        }
    } else {
        for (int c0 = 0; c0 < C; c0 += G::CB) {
            const int ws = wave_id();
            // a bounded batch of loads at a time (bounds the registers staging needs)
#pragma unroll
            for (int i0 = 0; i0 < NB_IT; i0 += G::SB) {
                float v[G::SB];
#pragma unroll
                for (int b = 0; b < G::SB; ++b)
                    if (i0 + b < NB_IT) v[b] = in_load(ws, c0, i0 + b);
#pragma unroll
                for (int b = 0; b < G::SB; ++b)
                    if (i0 + b < NB_IT) in_store(ldsB, ws, c0, i0 + b, v[b]);
            }
#pragma unroll
            for (int i0 = 0; i0 < NA_IT; i0 += G::SB) {
                wvec v[G::SB];
#pragma unroll
                for (int b = 0; b < G::SB; ++b)
                    if (i0 + b < NA_IT) v[b] = w_load(ws, c0, i0 + b);
#pragma unroll
                for (int b = 0; b < G::SB; ++b)
                    if (i0 + b < NA_IT) w_store(ldsA, ws, c0, i0 + b, v[b]);
            }
            __syncthreads();
            compute(ldsA, ldsB, no_side_work);
            __syncthreads();
        }
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
            for (int kb = 0; kb < G::KBW; ++kb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = k0 + (wk * G::KBW + kb) * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (k < K) out_n[((size_t)k * P + p) * Q + q] = acc[kb][pb][v];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side: launcher and the table entry of one compiled tile variant.
// ---------------------------------------------------------------------------
inline hipError_t allow_lds(const void *fn, size_t bytes)
{
    // Workgroups above the 64 KB default need the limit raised (no allocation involved).
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <class G, int WV>
static hipError_t launch_tile_wv(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    hipError_t e = allow_lds(reinterpret_cast<const void *>(&conv_tile_kernel<G, WV>), G::LDS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((conv_tile_kernel<G, WV>), dim3(grid), dim3(G::NT), G::LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class G>
static hipError_t launch_tile(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    // 16-byte filter loads when every one of them is aligned and stays inside one
    // output channel's row; plain 4-byte loads otherwise (any pointer, any C).
    constexpr bool can4 = G::PAIR == PAIR_C && (G::CB * G::RS) % 4 == 0;
    if (can4) {
        const bool ok4 = ((uintptr_t)a.w & 15u) == 0 && (a.s.C * G::RS) % 4 == 0 && a.s.C % G::CB == 0;
        if (ok4) return launch_tile_wv<G, can4 ? 4 : 1>(a, grid, stream);
    }
    return launch_tile_wv<G, 1>(a, grid, stream);
}

template <class G>
static size_t lds_tile(const Shape &) { return G::LDS_BYTES; }

template <class G>
constexpr Variant make_variant(const char *name)
{
    return Variant{name, G::R, G::S, G::ST, G::TP, G::TQ, G::KT, G::NPB, G::CB, G::PAIR, G::NT, G::OCC,
                   &lds_tile<G>, &launch_tile<G>};
}

}  // namespace convd
