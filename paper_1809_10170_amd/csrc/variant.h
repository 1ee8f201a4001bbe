// Host-side description of the compiled kernel variants, shared by the kernel
// translation unit (which fills the table) and the planner / C ABI (which reads it).
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>

namespace convd {

struct Shape {
    int N, C, H, W, K, R, S, stride, pad, P, Q;
};

// Everything a kernel needs; passed by value as the kernel argument.
struct KernelArgs {
    const float *in;
    const float *w;
    float *out;
    Shape s;
    int tilesP, tilesQ, ktiles;   // grid = ktiles * tilesQ * tilesP * N workgroups
    int dil, pad_h, pad_w;        // runtime-shape fallback as a data gradient: dil >= 1 marks the mode (input dilation,
                                  // separate and possibly negative paddings); dil = 0: an ordinary forward pass
    int in_blocked;               // runtime-shape fallback only (the compiled variants fix it at compile time)
    int out_blocked;              // 0: out[N][K][P][Q]; 1: out[N][ceil(K/4)][P][Q][4] (paper, Section 4.1)
    // fused point-wise tail (all optional): out = relu?(conv + bias[k] + residual[same position as out])
    const float *bias;            // K floats, or NULL
    const float *residual;        // a tensor of out's layout and size, or NULL
    int relu;
    // Output re-mapping (channel-pair kernels, instantiated for it separately; ost = 0: none): result (p, q) is
    // stored at row p*ost + ooh, column q*ost + oow of an OH x OW map if that position exists, and nowhere
    // otherwise.  A strided layer's data gradient is one stride-1 convolution of dy per phase (a, b) of the input
    // positions, a, b < onb = min(stride, R) (further phases have no tap: their positions keep the zeros of the
    // fill), written this way in ONE launch: the grid is onb*onb times the tiles, workgroup id % (onb*onb) is the
    // phase ph = a*onb + b, whose filter is w + ph*K*C*R*S and whose offsets are ooh + a, oow + b.
    int ost, onb, ooh, oow, OH, OW;
    int ofr;                      // ... and the forward layer's (square) filter extent: phase a has ceil((ofr - a) / ost) taps per
                                  // dimension, the first rows / columns of its padded filter are zeros and are skipped
};

// which reduction index the two k-lanes of one MFMA span: two input channels, or
// filter rows r and r + ceil(R/2) of one channel; PAIR_T: none (one tap per MFMA, the two
// halves of the instruction are two blocks of output channels; stages all channels like PAIR_R)
enum Pair { PAIR_C = 0, PAIR_R = 2, PAIR_T = 3 };

struct Variant {
    const char *name;
    int R, S, stride;     // filter and stride the variant is compiled for; 0 = any (runtime)
    int TP, TQ;           // output tile of one workgroup: TP rows x TQ columns of one image
    int KT;               // output channels per workgroup
    int NPB;              // 32-pixel MFMA column blocks per workgroup (NPB*32 >= TP*TQ)
    int CB;               // input channels staged per LDS chunk (PAIR_R: most channels the variant takes)
    int pair;             // which reduction index the two k-lanes of one MFMA span
    int threads;          // workgroup size
    int occupancy;        // workgroups per CU the variant is sized for
    int window;           // floats of LDS window staged per input channel (0: runtime-shape fallback)
    int img, pad;         // flat tiling only (img > 0): the H = W and the pad the variant is compiled for;
                          // a workgroup then owns NPB*32 consecutive pixels of all images (TP = TQ = 0)
    size_t (*lds_bytes)(const Shape &);
    hipError_t (*launch)(const KernelArgs &, unsigned grid, hipStream_t stream);
    int pointwise;        // 1: needs pad 0 (and R = S = stride = 1); a tile is TQ consecutive pixels of
                          // one image taken as a single row of H*W pixels.  2: the same over the pixels of
                          // ALL images numbered through (for images that are not a multiple of the tile)
    int in_blocked;       // 1: input and weights in the blocked layouts (paper, Section 4): in [N][C/4][H][W][4],
                          // w [K/32][C/4][R][S][4][32]
    int merged;           // 1: eight k-waves; serves only the data gradient of a stride-2 layer, all four phases of a
                          // pixel tile in one workgroup (a workgroup then covers 64 output channels, not KT)
    int kloop;            // 1: a workgroup walks ALL output channels of its pixel tile, KT at a time (the grid has no channel
                          // tiles); the variant takes exactly CB input channels, K a multiple of KT, H*W a multiple of 4
    int no_tail;          // 1: the variant has no instantiation with the fused point-wise tail (its registers are spoken
                          // for): a plan that chooses it carries a second choice for calls that bring a tail
};

// The compiled variants (host table of pointers; lives beside the fallback kernel).
const Variant *const *variant_table(int *count);

}  // namespace convd
