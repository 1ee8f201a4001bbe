// Re-arrangers between the plain tensors and the paper's blocked layouts (Section 4):
//   activations  plain[n][c][h][w]      <->  blocked[n][c/4][h][w][c%4]
//   weights      plain[k][c][r][s]       ->  blocked[k/32][c/4][r][s][c%4][k%32]
// Positions that complete the last block are written as zeros.  The paper counts the
// weight re-arrangement as a one-time cost for a trained network and keeps the first
// layer's input plain (Section 4.3); the activation re-arrangers exist for callers that
// enter or leave a chain of blocked layers.  Source and destination are both the
// caller's buffers: nothing is allocated here.
#include <hip/hip_runtime.h>

#include <atomic>

#include "layout.h"

namespace convd {

// one thread per destination pencil (4 floats, one 16-byte store)
__global__ void __launch_bounds__(256) pack_act_kernel(const float *__restrict__ src, float *__restrict__ dst, int C,
                                                       long long HW, long long pencils)
{
    const int CB4 = (C + 3) / 4;
    for (long long t = blockIdx.x * 256ll + threadIdx.x; t < pencils; t += gridDim.x * 256ll) {
        const long long pix = t % HW, nb = t / HW;
        const int blk = (int)(nb % CB4);
        const long long n = nb / CB4;
        float4 v;
        float *e = &v.x;
#pragma unroll
        for (int ci = 0; ci < 4; ++ci) {
            const int c = blk * 4 + ci;
            e[ci] = c < C ? src[(n * C + c) * HW + pix] : 0.f;
        }
        *reinterpret_cast<float4 *>(dst + t * 4) = v;
    }
}

// one thread per destination element
__global__ void __launch_bounds__(256) unpack_act_kernel(const float *__restrict__ src, float *__restrict__ dst, int C,
                                                         long long HW, long long elems)
{
    const int CB4 = (C + 3) / 4;
    for (long long t = blockIdx.x * 256ll + threadIdx.x; t < elems; t += gridDim.x * 256ll) {
        const long long pix = t % HW, nc = t / HW;
        const int c = (int)(nc % C);
        const long long n = nc / C;
        dst[t] = src[((n * CB4 + c / 4) * HW + pix) * 4 + c % 4];
    }
}

// one thread per destination element; consecutive threads write consecutive k % 32
__global__ void __launch_bounds__(256) pack_w_kernel(const float *__restrict__ src, float *__restrict__ dst, int K, int C,
                                                     int RS, long long elems)
{
    const int CB4 = (C + 3) / 4;
    for (long long t = blockIdx.x * 256ll + threadIdx.x; t < elems; t += gridDim.x * 256ll) {
        const int ki = (int)(t % 32);
        const int ci = (int)(t / 32 % 4);
        const long long u = t / 128;
        const int rs = (int)(u % RS);
        const int cblk = (int)(u / RS % CB4);
        const int kblk = (int)(u / RS / CB4);
        const int k = kblk * 32 + ki, c = cblk * 4 + ci;
        dst[t] = (k < K && c < C) ? src[((long long)k * C + c) * RS + rs] : 0.f;
    }
}

// Filter of the data gradient for stride 1 (see conv_direct_create_dgrad):
//   wt[c][k][r][s] = w[k][c][R-1-r][S-1-s]
// one thread per destination element
__global__ void __launch_bounds__(256) dgrad_filter_kernel(const float *__restrict__ src, float *__restrict__ dst, int K,
                                                           int C, int R, int S, long long elems)
{
    for (long long t = blockIdx.x * 256ll + threadIdx.x; t < elems; t += gridDim.x * 256ll) {
        const int s = (int)(t % S);
        const int r = (int)(t / S % R);
        const int k = (int)(t / ((long long)R * S) % K);
        const int c = (int)(t / ((long long)R * S * K));
        dst[t] = src[(((long long)k * C + c) * R + (R - 1 - r)) * S + (S - 1 - s)];
    }
}

// Filters of the data gradient of a strided layer with a square filter (see conv_direct_create_dgrad): one
// RT x RT filter (RT = ceil(R / stride)) per phase (a, b) of the input positions that has a tap, a, b < nb = min(stride, R),
//   wt[a*nb + b][c][k][j][l] = w[k][c][a + stride*(RT-1-j)][b + stride*(RT-1-l)]   (0 where that tap does not exist)
// one thread per destination element
__global__ void __launch_bounds__(256) dgrad_phase_filter_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                                 int K, int C, int R, int S, int st, int RT,
                                                                 int nb, long long elems)
{
    for (long long t = blockIdx.x * 256ll + threadIdx.x; t < elems; t += gridDim.x * 256ll) {
        const int l = (int)(t % RT);
        const int j = (int)(t / RT % RT);
        const int k = (int)(t / ((long long)RT * RT) % K);
        const int c = (int)(t / ((long long)RT * RT * K) % C);
        const int ph = (int)(t / ((long long)RT * RT * K * C));
        const int r = ph / nb + st * (RT - 1 - j), s = ph % nb + st * (RT - 1 - l);
        dst[t] = (r < R && s < S) ? src[(((long long)k * C + c) * R + r) * S + s] : 0.f;
    }
}

// The same filters in the blocked weight layout of the forward problem that computes dx (its 32 "output" channels a
// block are the layer's input channels c, its pencils of 4 "input" channels the layer's output channels k):
//   wt[ph][c/32][k/4][j][l][k%4][c%32] = w[k][c][a + stride*(RTR-1-j)][b + stride*(RTS-1-l)]
// (stride 1: one phase, RTR x RTS = R x S, the flipped filter), zeros where the tap or the channel does not exist;
// one thread per destination element
__global__ void __launch_bounds__(256) dgrad_filter_blocked_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                                   int K, int C, int R, int S, int st, int RTR, int RTS,
                                                                   int nb, long long elems)
{
    const int K4 = (K + 3) / 4, C32 = (C + 31) / 32;
    for (long long t = blockIdx.x * 256ll + threadIdx.x; t < elems; t += gridDim.x * 256ll) {
        long long u = t;
        const int ci = (int)(u % 32);  u /= 32;
        const int ki = (int)(u % 4);   u /= 4;
        const int l = (int)(u % RTS);  u /= RTS;
        const int j = (int)(u % RTR);  u /= RTR;
        const int kb = (int)(u % K4);  u /= K4;
        const int cb = (int)(u % C32);
        const int ph = (int)(u / C32);
        const int k = kb * 4 + ki, c = cb * 32 + ci;
        const int r = ph / nb + st * (RTR - 1 - j), s = ph % nb + st * (RTS - 1 - l);
        dst[t] = (k < K && c < C && r < R && s < S) ? src[(((long long)k * C + c) * R + r) * S + s] : 0.f;
    }
}

__global__ void __launch_bounds__(256) fill_zero_kernel(float *dst, long long elems)
{
    for (long long t = blockIdx.x * 256ll + threadIdx.x; t < elems; t += gridDim.x * 256ll) dst[t] = 0.f;
}

static unsigned blocks_for(long long items)
{
    const long long b = (items + 255) / 256;
    return (unsigned)(b < 1 ? 1 : b > 65536 ? 65536 : b);
}

hipError_t launch_pack_act(const float *plain, float *blocked, int N, int C, int H, int W, hipStream_t stream)
{
    const long long HW = (long long)H * W, pencils = (long long)N * ((C + 3) / 4) * HW;
    hipLaunchKernelGGL(pack_act_kernel, dim3(blocks_for(pencils)), dim3(256), 0, stream, plain, blocked, C, HW, pencils);
    return hipGetLastError();
}

hipError_t launch_unpack_act(const float *blocked, float *plain, int N, int C, int H, int W, hipStream_t stream)
{
    const long long HW = (long long)H * W, elems = (long long)N * C * HW;
    hipLaunchKernelGGL(unpack_act_kernel, dim3(blocks_for(elems)), dim3(256), 0, stream, blocked, plain, C, HW, elems);
    return hipGetLastError();
}

hipError_t launch_pack_w(const float *plain, float *blocked, int K, int C, int R, int S, hipStream_t stream)
{
    const long long elems = (long long)((K + 31) / 32) * ((C + 3) / 4) * R * S * 128;
    hipLaunchKernelGGL(pack_w_kernel, dim3(blocks_for(elems)), dim3(256), 0, stream, plain, blocked, K, C, R * S, elems);
    return hipGetLastError();
}

hipError_t launch_dgrad_filter(const float *w, float *wt, int K, int C, int R, int S, hipStream_t stream)
{
    const long long elems = (long long)K * C * R * S;
    hipLaunchKernelGGL(dgrad_filter_kernel, dim3(blocks_for(elems)), dim3(256), 0, stream, w, wt, K, C, R, S, elems);
    return hipGetLastError();
}

hipError_t launch_dgrad_phase_filter(const float *w, float *wt, int K, int C, int R, int S, int stride, hipStream_t stream)
{
    const int RT = (R + stride - 1) / stride;
    const int nb = stride < R ? stride : R;
    const long long elems = (long long)nb * nb * C * K * RT * RT;
    hipLaunchKernelGGL(dgrad_phase_filter_kernel, dim3(blocks_for(elems)), dim3(256), 0, stream, w, wt, K, C, R, S, stride, RT,
                       nb, elems);
    return hipGetLastError();
}

hipError_t launch_dgrad_filter_blocked(const float *w, float *wt, int K, int C, int R, int S, int stride, hipStream_t stream)
{
    const int RTR = (R + stride - 1) / stride, RTS = (S + stride - 1) / stride;
    const int nb = stride < R ? stride : R;
    const long long elems = (long long)nb * nb * ((C + 31) / 32 * 32) * ((K + 3) / 4 * 4) * RTR * RTS;
    hipLaunchKernelGGL(dgrad_filter_blocked_kernel, dim3(blocks_for(elems)), dim3(256), 0, stream, w, wt, K, C, R, S, stride,
                       RTR, RTS, nb, elems);
    return hipGetLastError();
}

// Scratch of the one entry point that may not allocate (conv_direct_run_dgrad_static): the
// transformed filter of a data gradient, which the other entry points take from the caller.
// Every GPU the library runs on holds its own copy of this array, at its own address, until
// the process ends.  In host code the array's name is only a handle for the look-up below:
// host code uses the address that look-up returns, never the name.
static __device__ __align__(256) float scratch[STATIC_WT_ELEMS];

hipError_t static_wt_buffer(float **ptr)
{
    constexpr int kMaxDev = 64;
    static std::atomic<float *> addr[kMaxDev];   // per device, looked up on the first call with that device current
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
    float *p = addr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!sym) return hipErrorInvalidSymbol;
        p = static_cast<float *>(sym);
        addr[dev].store(p, std::memory_order_release);   // (two threads racing here store the same address)
    }
    *ptr = p;
    return hipSuccess;
}

hipError_t launch_fill_zero(float *dst, long long elems, hipStream_t stream)
{
    long long b = (elems + 255) / 256;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)(b < 1 ? 1 : b > 8192 ? 8192 : b)), dim3(256), 0, stream, dst, elems);
    return hipGetLastError();
}

}  // namespace convd
