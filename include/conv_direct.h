/*
 * conv_direct.h -- C ABI of the MI355X (gfx950) zero-workspace direct convolution.
 *
 * The operation (paper: Section 3, Algorithm 1: an input image, filter weights and a
 * stride give the output image), with a batch dimension and symmetric zero padding added:
 *
 *   P = floor((H + 2*pad - R) / stride) + 1,  Q = floor((W + 2*pad - S) / stride) + 1
 *   out[n][k][p][q] = sum over c, r, s of
 *       in[n][c][p*stride + r - pad][q*stride + s - pad] * w[k][c][r][s]
 *
 * Taps outside the image contribute zero; the filter is not flipped; there is no
 * bias, grouping or dilation; stride and pad are the same in both dimensions.
 * The convolution is computed directly from the plain tensors, with no memory beyond
 * them (the paper's central claim, Sections 1 and 4): the library never allocates, frees or copies
 * device memory, makes no packed or lowered copy of the input or the weights, and
 * its kernels use no private scratch.  (The one device array the library itself holds
 * belongs to conv_direct_run_dgrad_static, an entry point for callers that cannot
 * allocate; no other entry point touches it.)  All arithmetic is fp32 (fp32 MFMA
 * accumulation); the order of the C*R*S additions is unspecified.
 *
 * Layouts, row-major with the last index fastest, fp32:
 *   in  [N][C][H][W]    w  [K][C][R][S]    out [N][K][P][Q]
 *
 * Every function returns 0 (CONV_DIRECT_OK) or a negative error code; nothing
 * throws, aborts or sets errno.
 */
#ifndef CONV_DIRECT_H
#define CONV_DIRECT_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CONV_DIRECT_OK            0
#define CONV_DIRECT_EINVAL       (-1) /* a dimension <= 0, stride < 1, pad < 0, filter larger than padded input, NULL argument */
#define CONV_DIRECT_EUNSUPPORTED (-2) /* a tensor has >= 2^31 elements, or no kernel variant can tile the shape */
#define CONV_DIRECT_EALIGN       (-3) /* a device pointer is not 4-byte aligned */
#define CONV_DIRECT_EHIP         (-4) /* the HIP runtime refused the launch; see conv_direct_last_hip_error */
#define CONV_DIRECT_ENOMEM       (-5) /* host allocation of the plan failed */
#define CONV_DIRECT_ETOOBIG      (-6) /* conv_direct_run_dgrad_static: the plan's transformed filter exceeds the static array */

/* Opaque launch plan: host memory only, immutable after creation. */
typedef struct conv_direct_plan conv_direct_plan;

/*
 * Validate a layer shape and choose the kernel variant, tile and grid for it
 * (the per-layer blocking decision of the paper's Section 3.1.2, made for the
 * GPU's register file and LDS instead of a CPU's registers and caches).
 * Host only: touches no device, allocates only the plan.  *plan is set to NULL on
 * error.  The caller releases the plan with conv_direct_destroy.
 */
int conv_direct_create(conv_direct_plan **plan,
                       int N, int C, int H, int W, int K, int R, int S, int stride, int pad);

/*
 * Enqueue the forward convolution on `stream` (a hipStream_t; NULL = the default
 * stream) and return without synchronising.
 *   in  : device pointer, N*C*H*W floats, read only
 *   w   : device pointer, K*C*R*S floats, read only
 *   out : device pointer, N*K*P*Q floats, every element overwritten (beta = 0)
 * The caller owns all three buffers and the stream; the buffers must not overlap
 * and must stay valid until the stream has run the kernel.  Pointers need 4-byte
 * alignment only.  A plan may be run any number of times.
 */
int conv_direct_run(const conv_direct_plan *plan,
                    const float *in, const float *w, float *out, void *stream);

/*
 * conv_direct_run with the point-wise layers that usually follow a convolution folded
 * into the store of the result (paper, Section 4.3: skip and activation layers are
 * point-wise operations that need no change of the algorithm):
 *   out = relu?( conv(in, w) + bias[k] + residual )
 *   bias     : device pointer, K floats, or NULL
 *   residual : device pointer, a tensor of out's layout and size (it may not overlap out), or NULL
 *   relu     : nonzero applies max(., 0) last
 * All NULL / 0 is conv_direct_run.  Still one kernel launch and no workspace.  A few kernel variants have no
 * registers to spare for the tail; a plan that chose one runs calls that bring a tail on its second choice
 * (plan_info: tail_variant), calls without one on its first.
 */
int conv_direct_run_fused(const conv_direct_plan *plan,
                          const float *in, const float *w, const float *bias, const float *residual,
                          int relu, float *out, void *stream);

/* Free the host plan.  conv_direct_destroy(NULL) is a no-op that returns OK. */
int conv_direct_destroy(conv_direct_plan *plan);

/* Output height and width of the planned layer. */
int conv_direct_output_dims(const conv_direct_plan *plan, int *P, int *Q);

/* Device workspace the plan needs: always 0.  Exists so callers can assert it. */
size_t conv_direct_workspace_bytes(const conv_direct_plan *plan);

/*
 * Write a one-line, space-separated key=value description of the plan into buf
 * (variant name, tile, grid, LDS bytes, threads ...; for a data-gradient plan also
 * extra_caller_bytes, the size of the transformed-filter buffer wt the caller provides; tail_variant: the variant
 * that calls with a fused tail run on, "same" unless the plan's variant has no tail; model_clocks: the planner's
 * estimate of the run time in shader clocks, the figure that ranked the variants),
 * NUL-terminated and truncated to n bytes.  Returns the untruncated length, or a negative error code.
 */
int conv_direct_plan_info(const conv_direct_plan *plan, char *buf, size_t n);

/* Static text for an error code. */
const char *conv_direct_strerror(int code);

/* hipError_t value of the most recent failed launch on this thread (0 if none). */
int conv_direct_last_hip_error(void);

/*
 * Testing / tuning aid: like conv_direct_create, but forces the kernel variant
 * whose name is `variant` (as printed by conv_direct_plan_info) instead of asking
 * the planner.  Returns CONV_DIRECT_EUNSUPPORTED if that variant cannot run the
 * shape.  conv_direct_variant_name(i) enumerates the names (NULL past the end).
 */
int conv_direct_create_with_variant(conv_direct_plan **plan, const char *variant,
                                    int N, int C, int H, int W, int K, int R, int S,
                                    int stride, int pad);
const char *conv_direct_variant_name(int index);

/* ------------------------------------------------------------------------
 * Convolution-friendly layouts (paper: Section 4).
 *
 * Activations (Section 4.1): channels in blocks of CONV_DIRECT_ACT_BLOCK = 4; a tensor is
 * a sequence of blocks, each an H x W row-major matrix of pencils of 4 channels:
 *     blocked[n][c / 4][h][w][c % 4]            ceil(C/4) * 4 * N*H*W floats
 * Input and output share this layout, so a layer's output is the next layer's input
 * with no reshape.  Weights (Section 4.2), fastest to slowest: output channel in its
 * block of CONV_DIRECT_W_KBLOCK = 32, input channel in its block of 4, filter column,
 * filter row, input-channel block, output-channel block:
 *     blocked[k / 32][c / 4][r][s][c % 4][k % 32]   ceil(K/32)*32 * ceil(C/4)*4 * R*S floats
 * Positions that complete a last block must hold zeros (the re-arrangers below and the
 * convolution's blocked output write them as zeros).  The paper leaves the block sizes to
 * the implementation; 4 and 32 are what the fp32 MFMA operand shapes of this GPU want.
 * The buffers are the caller's, of the sizes above: still no workspace.
 * ------------------------------------------------------------------------ */
#define CONV_DIRECT_LAYOUT_PLAIN   0
#define CONV_DIRECT_LAYOUT_BLOCKED 1
#define CONV_DIRECT_ACT_BLOCK 4
#define CONV_DIRECT_W_KBLOCK  32

/*
 * Like conv_direct_create, with the layouts of the tensors stated.  in_layout covers
 * `in` and `w` together (blocked input goes with blocked weights; a plain input, as the
 * paper keeps for the first layer of a network, goes with plain KCRS weights); out_layout
 * covers `out`.  (PLAIN, PLAIN) is conv_direct_create.  conv_direct_run then expects
 * buffers of those layouts.  CONV_DIRECT_EINVAL for an unknown layout value.
 */
int conv_direct_create_layout(conv_direct_plan **plan,
                              int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                              int in_layout, int out_layout);

/* conv_direct_create_layout with the kernel variant forced (testing / tuning aid; variant = NULL asks the planner). */
int conv_direct_create_ex(conv_direct_plan **plan, const char *variant,
                          int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                          int in_layout, int out_layout);

/* Number of floats of a blocked activation tensor / blocked weight tensor (0 if a dimension is <= 0). */
size_t conv_direct_blocked_act_elems(int N, int C, int H, int W);
size_t conv_direct_blocked_w_elems(int K, int C, int R, int S);

/*
 * Re-arrangers, enqueued on `stream` (hipStream_t; NULL = default), asynchronous, device
 * pointers, source and destination distinct caller buffers of the plain / blocked sizes,
 * 4-byte aligned (16 for a blocked activation destination).  pack_w is the one-time
 * re-arrangement of a trained network's weights (Section 4.3).
 */
int conv_direct_pack_act(const float *plain, float *blocked, int N, int C, int H, int W, void *stream);
int conv_direct_unpack_act(const float *blocked, float *plain, int N, int C, int H, int W, void *stream);
int conv_direct_pack_w(const float *plain, float *blocked, int K, int C, int R, int S, void *stream);

/* ------------------------------------------------------------------------
 * Data gradient (the backward pass with respect to the input image, which the paper's
 * closing section names as a direction), plain layouts:
 *
 *   dx[n][c][h][w] = sum over k, r, s of dy[n][k][h + pad - r][w + pad - s] * w[k][c][r][s]
 *
 * for stride 1, and in general with dy indices (h + pad - r) / stride, (w + pad - s) / stride
 * where both divide (terms whose dy index falls outside [0,P) x [0,Q) are absent).  For stride 1 this is
 * itself a forward convolution, of dy [N][K][P][Q] with the filter
 *   wt[c][k][r][s] = w[k][c][R-1-r][S-1-s]      (C*K*R*S floats, [C][K][R][S])
 * and padding R-1-pad, and runs on the same zero-workspace kernels:
 *
 *   conv_direct_create_dgrad(&plan, N, C, H, W, K, R, S, stride, pad);   // dims of the FORWARD layer
 *   conv_direct_dgrad_filter(w, wt, K, C, R, S, stream);                 // wt: a caller buffer, once per weight update
 *   conv_direct_run(plan, dy, wt, dx, stream);                           // dx [N][C][H][W], every element written
 *
 * A strided layer with a square filter is stride*stride such convolutions, one per
 * phase (a, b) of the input positions: with h + pad = stride*u + a only the taps
 * r = a + stride*i reach row h, so dx at those rows is the stride-1 convolution of dy with
 * the RT = ceil(R/stride) taps of phase a (zeros where a + stride*i >= R), and likewise
 * along the columns.  The plan then takes nb*nb filters of RT x RT taps, nb = min(stride, R)
 * (phases a >= R have no tap; their positions of dx are zero),
 *   wt[a*nb + b][c][k][j][l] = w[k][c][a + stride*(RT-1-j)][b + stride*(RT-1-l)],
 * and conv_direct_run launches a fill that clears dx and the convolutions of all phases as one
 * grid, each storing to its own positions of dx: no workspace.  Because wt's size and contents depend
 * on the plan, ask the plan:
 *
 *   size_t n = conv_direct_dgrad_wt_elems(plan);                         // floats of wt for this plan
 *   conv_direct_dgrad_prepare(plan, w, wt, stream);                      // w [K][C][R][S] -> wt, any data-gradient plan
 *   conv_direct_run(plan, dy, wt, dx, stream);
 *
 * (for stride 1 conv_direct_dgrad_prepare is conv_direct_dgrad_filter).  Filters with
 * R != S, pad > R-1 and strided shapes no compiled variant serves go to the slow
 * runtime-shape kernel (dy read as if zeros stood between its elements), with the
 * stride-1 form of wt.  conv_direct_output_dims of the plan gives (H, W).  A fused tail
 * is refused for a phase plan (CONV_DIRECT_EINVAL).
 * Blocked layouts (the paper's Section 4): conv_direct_create_dgrad_layout takes the layout of
 * dy ([N][ceil(K/4)][P][Q][4] when blocked) and of dx ([N][ceil(C/4)][H][W][4]; the spare
 * channels of a last pencil are written as zeros) and serves every shape the plain entry point
 * serves, strided layers included.  The weights stay plain [K][C][R][S] (the master copy a
 * weight update writes); conv_direct_dgrad_prepare writes wt in the layout the plan's kernels read
 * -- for a blocked dy the blocked weight layout of the forward problem over dy,
 *   wt[phase][c/32][k/4][j][l][k%4][c%32]  (zeros where the tap or the channel does not exist),
 * conv_direct_dgrad_wt_elems(plan) floats -- so wt is opaque to the caller: always size it with
 * _dgrad_wt_elems and fill it with _dgrad_prepare of the SAME plan.
 *
 * Weight gradient (the backward pass with respect to the filter), any
 * filter, strides up to 4 (compiled variants for the filter widths and strides of the forward
 * variants, a slower run-time-shape variant for the rest):
 *
 *   dw[k][c][r][s] = sum over n, p, q of dy[n][k][p][q] * x[n][c][p*stride + r - pad][q*stride + s - pad]
 *
 *   conv_direct_create_wgrad(&plan, N, C, H, W, K, R, S, stride, pad);   // dims of the FORWARD layer
 *   conv_direct_run_wgrad(plan, x, dy, dw, stream);                      // dw [K][C][R][S], every element written
 *
 * Two launches (a fill that clears dw, then the reduction, whose workgroups add their
 * partial sums into dw with fp32 atomics): no workspace, but the order of the additions
 * is not fixed, so the last bits of dw can differ between runs (see
 * conv_direct_create_wgrad_deterministic for a plan without that).  A wgrad plan can only be
 * passed to conv_direct_run_wgrad, _plan_info, _workspace_bytes and _destroy;
 * CONV_DIRECT_EUNSUPPORTED for strides above 4.
 * ------------------------------------------------------------------------ */
int conv_direct_create_dgrad(conv_direct_plan **plan,
                             int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
int conv_direct_create_dgrad_layout(conv_direct_plan **plan,
                                    int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                    int dy_layout, int dx_layout);   /* CONV_DIRECT_LAYOUT_* */
/* Testing / tuning aid: the same with the kernel variant forced (NULL: the planner's choice); CONV_DIRECT_EUNSUPPORTED
 * if that variant cannot run the data gradient of this layer. */
int conv_direct_create_dgrad_ex(conv_direct_plan **plan, const char *variant,
                                int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                int dy_layout, int dx_layout);
int conv_direct_dgrad_filter(const float *w, float *wt, int K, int C, int R, int S, void *stream);
size_t conv_direct_dgrad_wt_elems(const conv_direct_plan *plan);   /* 0 for a plan that is no data gradient */
int conv_direct_dgrad_prepare(const conv_direct_plan *plan, const float *w, float *wt, void *stream);
int conv_direct_create_wgrad(conv_direct_plan **plan,
                             int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
int conv_direct_run_wgrad(const conv_direct_plan *plan,
                          const float *x, const float *dy, float *dw, void *stream);
/* A weight-gradient plan whose result is the same bit for bit on every run: every tile of dw is reduced by ONE
 * workgroup, which stores it plainly (one launch, no fill, no atomics).  Slower than conv_direct_create_wgrad's plan
 * where the tiles of dw are fewer than the chip's compute units. */
int conv_direct_create_wgrad_deterministic(conv_direct_plan **plan,
                                           int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
/* Testing / tuning aid: conv_direct_create_wgrad with the kernel variant forced (variant = NULL asks the planner;
 * CONV_DIRECT_EUNSUPPORTED if the variant is unknown or cannot run the shape); conv_direct_wgrad_variant_name(i)
 * enumerates the names (NULL past the end). */
int conv_direct_create_wgrad_ex(conv_direct_plan **plan, const char *variant,
                                int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
/* The weight gradient with tensors in the blocked layouts of the paper's Section 4 (each one CONV_DIRECT_LAYOUT_PLAIN
 * or _BLOCKED): x [N][ceil(C/4)][H][W][4], dy [N][ceil(K/4)][P][Q][4] (spare channels of a last pencil must hold
 * zeros or any finite value: they only meet results that are dropped), dw [ceil(K/32)][ceil(C/4)][R][S][4][32] (what
 * conv_direct_pack_w would make of the plain gradient; its spare channels are written as zeros).  variant (NULL: the
 * planner's choice) and deterministic (non-zero: one workgroup per tile of dw, the same bits every run) as in
 * conv_direct_create_wgrad_ex / _deterministic.  Every shape the plain entry points serve. */
int conv_direct_create_wgrad_layout(conv_direct_plan **plan, const char *variant, int deterministic,
                                    int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                    int x_layout, int dy_layout, int dw_layout);
const char *conv_direct_wgrad_variant_name(int index);

/*
 * For callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: the data gradient without the caller's wt
 * buffer.  Same result, bit for bit, as
 *     conv_direct_dgrad_prepare(plan, w, wt, stream);  conv_direct_run(plan, dy, wt, dx, stream);
 * with wt replaced by a file-scope device array inside the library of
 * CONV_DIRECT_STATIC_WT_ELEMS floats (16 MiB; every GPU the library runs on holds its own
 * copy until the process ends).  The call allocates and frees nothing and calls no
 * allocating routine: it enqueues the filter transform into that array, then the kernels of
 * conv_direct_run, on `stream`.
 *   plan : from conv_direct_create_dgrad (any data-gradient plan)
 *   dy   : device, [N][K][P][Q];  w : device, the layer's weights [K][C][R][S], as they are;
 *   dx   : device, [N][C][H][W], every element overwritten
 * CONV_DIRECT_ETOOBIG, before anything is enqueued, if conv_direct_dgrad_wt_elems(plan)
 * exceeds CONV_DIRECT_STATIC_WT_ELEMS; CONV_DIRECT_EINVAL for a plan that is no data
 * gradient or a NULL pointer; CONV_DIRECT_EALIGN; CONV_DIRECT_EHIP.  The first call on a
 * device looks up the array's address on that device (no allocation, but make that call
 * outside a graph capture).  All calls on one GPU share the array, which keeps the last
 * call's contents (every element a call reads it has written first): calls that overlap on
 * one GPU -- two streams, or two threads -- race on it; order them.
 */
#define CONV_DIRECT_STATIC_WT_ELEMS (4u << 20)
int conv_direct_run_dgrad_static(const conv_direct_plan *plan,
                                 const float *dy, const float *w, float *dx, void *stream);

/* ------------------------------------------------------------------------
 * Measured choice of the blocking (the paper's closing section proposes auto-tuning
 * the loops' blocking parameters to close the remaining gap to peak).
 *
 * conv_direct_create_tuned runs every compiled variant that can serve the shape, `reps`
 * times each (after one untimed run), on the caller's own buffers and stream, times
 * them with HIP events and returns a plan for the fastest.  It synchronises the stream,
 * overwrites `out`, allocates no device memory, and records the winner in a per-process
 * table that conv_direct_create / _create_layout consult first from then on (exact match
 * of all dimensions and layouts).  conv_direct_tuning_save / _load write and read that
 * table as text, one line per shape:
 *     N C H W K R S stride pad in_layout out_layout variant
 * A loaded entry that names an unknown variant, or one that cannot run its shape, is
 * ignored (the analytical planner decides).  conv_direct_tuning_clear empties the table.
 * Every create function reads the table; conv_direct_create_tuned, _tuning_load and
 * _tuning_clear write it.  Readers and writers are not synchronised: do not call a writer
 * while another thread is inside any create function.
 * ------------------------------------------------------------------------ */
int conv_direct_create_tuned(conv_direct_plan **plan,
                             int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             int in_layout, int out_layout,
                             const float *in, const float *w, float *out, void *stream, int reps);
int conv_direct_tuning_save(const char *path);   /* CONV_DIRECT_EINVAL if the file cannot be written */
int conv_direct_tuning_load(const char *path);   /* CONV_DIRECT_EINVAL if the file cannot be read or a line is malformed */
int conv_direct_tuning_clear(void);
int conv_direct_tuning_size(void);               /* number of entries */

/* ------------------------------------------------------------------------
 * Measurement aid: the fp32 MFMA rate this chip sustains right now.  The benchmark states
 * each layer as a fraction of the nominal fp32 MFMA peak (256 CUs x 256 flop per clock x
 * 2.4 GHz); under a saturated matrix load the clock is a few per cent lower, and this call
 * measures by how much.  It enqueues, on `stream`, one kernel of independent
 * v_mfma_f32_32x32x2_f32 chains on every SIMD: CONV_DIRECT_PROBE_FLOP_PER_ITER * iters flop
 * in all, to be timed by the caller with events on that stream; rate / 65536 flop per clock
 * is the shader clock under that load.
 *   buf : device, the caller's, CONV_DIRECT_PROBE_BYTES bytes, 8-byte aligned.  On return of
 *         the kernel it holds 512 * 256 floats (sums, of no interest) followed by 512 pairs
 *         of int64: per workgroup the shader-clock counter's and the constant-rate (100 MHz)
 *         counter's advance around its loop.
 * CONV_DIRECT_EINVAL for a NULL buffer or iters < 1, CONV_DIRECT_EALIGN, CONV_DIRECT_EHIP.
 * ------------------------------------------------------------------------ */
#define CONV_DIRECT_PROBE_BYTES (512 * 256 * 4 + 512 * 2 * 8)
#define CONV_DIRECT_PROBE_FLOP_PER_ITER (512.0 * 4 * 8 * 7 * 4096)
int conv_direct_mfma_probe(void *buf, int iters, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CONV_DIRECT_H */
