// Launchers of the layout re-arrangers (conv_layout_kernels.hip), called by the C ABI.
#pragma once
#include <hip/hip_runtime_api.h>

namespace convd {
hipError_t launch_pack_act(const float *plain, float *blocked, int N, int C, int H, int W, hipStream_t stream);
hipError_t launch_unpack_act(const float *blocked, float *plain, int N, int C, int H, int W, hipStream_t stream);
hipError_t launch_pack_w(const float *plain, float *blocked, int K, int C, int R, int S, hipStream_t stream);
hipError_t launch_dgrad_filter(const float *w, float *wt, int K, int C, int R, int S, hipStream_t stream);
hipError_t launch_dgrad_phase_filter(const float *w, float *wt, int K, int C, int R, int S, int stride, hipStream_t stream);
// ... in the blocked weight layout of the forward problem over dy (stride 1: one phase, the flipped filter)
hipError_t launch_dgrad_filter_blocked(const float *w, float *wt, int K, int C, int R, int S, int stride, hipStream_t stream);
hipError_t launch_fill_zero(float *dst, long long elems, hipStream_t stream);
// Bare MFMA chains on every SIMD (conv_probe.hip): PROBE_BLOCKS workgroups of 256 threads, two per CU; every thread
// writes one float of sums, every workgroup two counters of ticks (shader clock, constant-rate clock).
constexpr int PROBE_BLOCKS = 512;
hipError_t launch_mfma_probe(float *sums, long long *ticks, int iters, hipStream_t stream);
// The library's static device array of STATIC_WT_ELEMS floats on the current device (its address on that
// device, looked up once per device); allocates nothing.
constexpr unsigned STATIC_WT_ELEMS = 4u << 20;
hipError_t static_wt_buffer(float **ptr);
}  // namespace convd
