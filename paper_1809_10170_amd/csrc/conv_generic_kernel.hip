// Runtime-shape fallback kernel and the table of all compiled variants.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "variant.h"

namespace convd {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------
// Fallback for any filter size and stride (runtime R, S, stride).  Same operand
// mapping; one chunk is one pair of input channels at one filter row, so the LDS
// need is independent of R.  Tile: 2 output rows x 32 columns x 64 channels,
// four waves each owning one 32x32 accumulator block.  It reads and writes element by
// element, so either layout of each tensor (plain, or the blocked layouts of the
// paper's Section 4) and the fused point-wise tail are index arithmetic here.
//
// It also serves the data gradients the fast path does not (strided layers, unequal
// filter sides, pad > R-1): with a.dil > 1 the "input" is dy read as if zeros stood
// between its elements (position i exists where i % dil == 0 and is element i / dil), and
// the paddings of the two dimensions may differ and be negative (a crop).
// ---------------------------------------------------------------------------
struct GenericGeom {
    static constexpr int TP = 2, TQ = 32, KT = 64, NT = 256, KP = KT + 1;
    static __host__ __device__ int lw(int S, int st) { return (TQ - 1) * st + S; }
    static __host__ __device__ size_t lds_floats(int S, int st) { return (size_t)S * 2 * KP + 2 * TP * lw(S, st); }
};

__global__ void __launch_bounds__(GenericGeom::NT) conv_generic_kernel(const KernelArgs a)
{
    using G = GenericGeom;
    extern __shared__ __align__(16) float lds[];
    const int C = a.s.C, H = a.s.H, W = a.s.W, K = a.s.K, P = a.s.P, Q = a.s.Q;
    const int R = a.s.R, S = a.s.S, st = a.s.stride;
    const int LW = G::lw(S, st);
    float *ldsA = lds;                       // [S][2][KP]
    float *ldsB = lds + S * 2 * G::KP;       // [2][TP][LW]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave & 1, wp = wave >> 1;   // wp = output row of the tile
    const int h = lane >> 5, j = lane & 31;

    unsigned bid = blockIdx.x;
    const int kt = bid % a.ktiles;  bid /= a.ktiles;
    const int tq = bid % a.tilesQ;  bid /= a.tilesQ;
    const int tp = bid % a.tilesP;
    const int n = bid / a.tilesP;
    const int p0 = tp * G::TP, q0 = tq * G::TQ, k0 = kt * G::KT;
    const int dil = a.dil > 1 ? a.dil : 1;
    const int pad_h = a.dil ? a.pad_h : a.s.pad, pad_w = a.dil ? a.pad_w : a.s.pad;
    const int iw0 = q0 * st - pad_w;
    const int C4 = (C + 3) / 4, KO = a.out_blocked ? (K + 3) / 4 * 4 : K;
    const float *in_n = a.in + (size_t)n * (a.in_blocked ? C4 * 4 : C) * H * W;

    const int bbase = (h * G::TP + wp) * LW + j * st;
    const int abase = h * G::KP + wk * 32 + j;

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    const int nB = 2 * G::TP * LW, nA = G::KT * 2 * S;
    for (int c0 = 0; c0 < C; c0 += 2) {
        for (int r = 0; r < R; ++r) {
            for (int e = tid; e < nB; e += G::NT) {
                const int cc = e / (G::TP * LW), rem = e - cc * (G::TP * LW);
                const int py = rem / LW, ww = rem - py * LW;
                int ih = (p0 + py) * st + r - pad_h, iw = iw0 + ww;
                const int c = c0 + cc;
                bool ok = c < C && ih >= 0 && iw >= 0;
                if (dil > 1) {   // dilated input: only every dil-th position holds an element
                    ok = ok && ih % dil == 0 && iw % dil == 0;
                    ih /= dil;
                    iw /= dil;
                }
                float v = 0.f;
                if (ok && ih < H && iw < W)
                    v = a.in_blocked ? in_n[((((size_t)(c >> 2)) * H + ih) * W + iw) * 4 + (c & 3)]
                                     : in_n[((size_t)c * H + ih) * W + iw];
                ldsB[e] = v;
            }
            for (int e = tid; e < nA; e += G::NT) {
                const int kk = e / (2 * S), rem = e - kk * (2 * S);
                const int cc = rem / S, s = rem - cc * S;
                float v = 0.f;
                if (k0 + kk < K && c0 + cc < C) {
                    const int k = k0 + kk, c = c0 + cc;
                    v = a.in_blocked ? a.w[(((((size_t)(k >> 5)) * C4 + (c >> 2)) * R + r) * S + s) * 128 + (c & 3) * 32 + (k & 31)]
                                     : a.w[(((size_t)k * C + c) * R + r) * S + s];
                }
                ldsA[(s * 2 + cc) * G::KP + kk] = v;
            }
            __syncthreads();
            for (int s = 0; s < S; ++s) {
                const float av = ldsA[abase + s * 2 * G::KP];
                const float bv = ldsB[bbase + s];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
            }
            __syncthreads();
        }
    }

    const int p = p0 + wp, q = q0 + j;
    if (p < P && q < Q) {
        const size_t img = (size_t)n * KO * P * Q;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + wk * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (k >= KO) continue;
            const size_t idx = img + (a.out_blocked ? (((size_t)(k >> 2)) * P * Q + (size_t)p * Q + q) * 4 + (k & 3)
                                                    : ((size_t)k * P + p) * Q + q);
            float x = 0.f;                       // (blocked: channels completing the last pencil are zeros)
            if (k < K) {
                x = acc[v];
                if (a.bias) x += a.bias[k];
                if (a.residual) x += a.residual[idx];
                if (a.relu) x = x > 0.f ? x : 0.f;
            }
            a.out[idx] = x;
        }
    }
}

// ---------------------------------------------------------------------------
// Host side: launcher of the fallback and the variant table.
// ---------------------------------------------------------------------------
static size_t lds_generic(const Shape &s)
{
    return sizeof(float) * GenericGeom::lds_floats(s.S, s.stride);
}

static hipError_t launch_generic(const KernelArgs &a, unsigned grid, hipStream_t stream)
{
    const size_t bytes = lds_generic(a.s);
    if (bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_generic_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(conv_generic_kernel, dim3(grid), dim3(GenericGeom::NT), bytes, stream, a);
    return hipGetLastError();
}

static const Variant k_generic = {"generic_2x32_k64", 0, 0, 0, GenericGeom::TP, GenericGeom::TQ, GenericGeom::KT,
                                  2, 2, PAIR_C, GenericGeom::NT, 2, 0, 0, 0, &lds_generic, &launch_generic};

// the compiled variants live in their own translation units (conv_variant.hip)
#ifndef CONVD_VARIANTS_DEF
#define CONVD_VARIANTS_DEF "variants.def"
#endif
#define X(NAME, ...) extern Variant variant_##NAME;
#include CONVD_VARIANTS_DEF
#undef X

static const Variant *const k_variants[] = {
#define X(NAME, ...) &variant_##NAME,
#include CONVD_VARIANTS_DEF
#undef X
    &k_generic,   // any shape; last, so that a compiled variant wins a tie
};

const Variant *const *variant_table(int *count)
{
    *count = (int)(sizeof(k_variants) / sizeof(k_variants[0]));
    return k_variants;
}

}  // namespace convd
