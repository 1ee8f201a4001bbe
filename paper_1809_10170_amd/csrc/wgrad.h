// Host-side description of the weight-gradient kernels (conv_wgrad.hip), read by the C ABI.
#pragma once
#include <hip/hip_runtime_api.h>

#include "variant.h"

namespace convd {

struct WgradArgs {
    const float *x;     // [N][C][H][W], or blocked [N][C/4][H][W][4]
    const float *dy;    // [N][K][P][Q], or blocked [N][K/4][P][Q][4]
    float *dw;          // [K][C][R][S], or blocked [K/32][C/4][R][S][4][32]; cleared before the launch and added to atomically
                        // (one split: stored plainly; blocked: still cleared, for the spare channels of its blocks)
    int x_blocked, dy_blocked, dw_blocked;
    Shape s;
    int ktiles, cgroups, splits;   // grid = splits * ktiles * R * cgroups workgroups (all-rows variants: without R)
};

struct WgradVariant {
    const char *name;
    int S, stride;      // filter width and stride the variant is compiled for (any R)
    int CBW, WK, PXC;   // 32-channel input blocks and 32-channel output blocks per workgroup, pixels per chunk
    int pack;           // > 0: columns are (channel, filter column) pairs in `pack` blocks of 32; needs C*S <= 32*pack
    int qw;             // > 0: chunks of PXC / qw whole output rows; needs Q == qw
    int per_cu;         // workgroups whose LDS fits one CU together (1 or 2)
    hipError_t (*launch)(const WgradArgs &, unsigned grid, hipStream_t stream);
    int allr;           // 1: a workgroup owns all filter rows (needs R == S, stride 1); the filter row is no grid dimension
    int WC;             // groups of 32*CBW input channels per workgroup (their waves share the staged dy)
    int WB;             // waves per k-block that share out the column blocks of the same channels
};

const WgradVariant *wgrad_table(int *count);
hipError_t wgrad_clear(float *dw, long long elems, hipStream_t stream);

}  // namespace convd
