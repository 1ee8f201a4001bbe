// C ABI and per-layer planner of the direct-convolution library (see
// include/conv_direct.h for the contract).  Host code only: the planner picks, for
// one layer shape, the compiled kernel variant, its tile and the grid -- the GPU
// counterpart of choosing the block sizes C_o,b, W_o,b and C_i,b in the paper's
// Section 3.1.2.  Nothing here allocates, frees or copies device memory.
#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/conv_direct.h"
#include "layout.h"
#include "variant.h"
#include "wgrad.h"

using convd::Shape;
using convd::Variant;

struct conv_direct_plan {
    Shape s;
    const Variant *v;
    int tilesP, tilesQ, ktiles;
    unsigned grid;
    size_t lds_bytes;
    double mfma_efficiency;   // useful / issued multiply-accumulates
    double model_clocks;      // the planner's estimate of the run time in shader clocks (what ranked the variants)
    int in_blocked, out_blocked;   // layouts of in + w, and of out (paper, Section 4)
    int pw_flat;                   // pointwise kernels: tiles run over the pixels of all images
    int dil, pad_h, pad_w;         // data gradients on the runtime-shape kernel (dil >= 1), see variant.h
    int ph_stride, ph_pad, ph_H, ph_W;   // data gradient of a strided layer as ph_stride^2 stride-1 convolutions of dy
                                   // (ph_stride >= 2), one per phase; the forward layer's pad and input size
    int fwd_K, fwd_C, fwd_R, fwd_S;      // data-gradient plans: the forward layer's filter dims (0 otherwise)
    const convd::WgradVariant *wv; // weight-gradient plans only (v is then NULL)
    int wg_cgroups, wg_splits;
    int wg_dy_blocked;             // weight-gradient plans: layout of dy (in_blocked: of x, out_blocked: of dw)
    conv_direct_plan *tail_plan;   // forward plans whose variant cannot fuse a point-wise tail: the plan that calls with a
                                   // tail run on instead (owned; NULL otherwise)
};

namespace {

constexpr int kNumCU = 256;                   // MI355X
constexpr size_t kLdsPerCU = 160 * 1024;
constexpr int64_t kMaxElems = (int64_t)1 << 31;
thread_local int t_last_hip_error = 0;

int launched(hipError_t e)
{
    if (e == hipSuccess) return CONV_DIRECT_OK;
    t_last_hip_error = (int)e;
    return CONV_DIRECT_EHIP;
}

int cdiv(int a, int b) { return (a + b - 1) / b; }
int64_t cdiv64(int64_t a, int64_t b) { return (a + b - 1) / b; }
constexpr int convd_generic_tq = 32;   // pixel columns per workgroup of the runtime-shape fallback

int validate(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, Shape *out)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride < 1 || pad < 0)
        return CONV_DIRECT_EINVAL;
    const int64_t spanH = (int64_t)H + 2 * (int64_t)pad - R, spanW = (int64_t)W + 2 * (int64_t)pad - S;
    if (spanH < 0 || spanW < 0) return CONV_DIRECT_EINVAL;
    const int64_t P = spanH / stride + 1, Q = spanW / stride + 1;
    const int64_t nin = (int64_t)N * C * H * W, nw = (int64_t)K * C * R * S, nout = (int64_t)N * K * P * Q;
    // the kernels index each tensor with 32-bit element offsets inside one image
    if (nin >= kMaxElems || nw >= kMaxElems || nout >= kMaxElems || (int64_t)pad * 2 + H >= kMaxElems / 4)
        return CONV_DIRECT_EUNSUPPORTED;
    *out = Shape{N, C, H, W, K, R, S, stride, pad, (int)P, (int)Q};
    return CONV_DIRECT_OK;
}

// Pointwise kernels cut every image into tiles of TQ pixels; when the image is not a
// multiple of the tile (7x7, 14x14, 28x28 maps against tiles of 224 or 448) the pixels of all
// images are numbered through instead and a tile takes TQ consecutive ones.  A tile then
// reaches over TQ/HW + 2 images at most, all addressed from the first with 31-bit offsets.
bool pointwise_flat(const Variant &v, const Shape &s)
{
    if (v.pointwise != 2) return false;
    const int64_t hw = (int64_t)s.H * s.W;
    const int64_t images = v.TQ / hw + 2;
    const int64_t chans = s.C > s.K ? s.C : s.K;
    return images * (chans + 3) * hw * 4 < ((int64_t)1 << 31);
}

// Can variant v run shape s at all?
bool applicable(const Variant &v, const Shape &s, int in_blocked, int out_blocked)
{
    if (v.R != 0 && (v.in_blocked != 0) != (in_blocked != 0)) return false;   // (the runtime-shape fallback takes either)
    if (v.R != 0 && (v.R != s.R || v.S != s.S || v.stride != s.stride)) return false;
    if ((v.pair == convd::PAIR_R || v.pair == convd::PAIR_T) && s.C > v.CB) return false;   // stages all channels at once
    if (v.img != 0 && (s.H != v.img || s.W != v.img || s.pad != v.pad)) return false;   // flat tiling
    if (v.pointwise && s.pad != 0) return false;
    if (v.pointwise == 2 && (!pointwise_flat(v, s) || (!v.kloop && ((int64_t)s.H * s.W) % v.TQ == 0))) return false;
    // (its lanes take pixels in fours; whole channel blocks only; pointwise_flat() above bounds its byte offsets)
    if (v.kloop && (s.C != v.CB || ((int64_t)s.H * s.W) % 4 != 0 || s.K % v.KT != 0)) return false;
    if (v.lds_bytes(s) > kLdsPerCU) return false;
    if (v.R != 0) {
        // the compiled kernels address the input with 31-bit byte offsets from the first
        // channel they stage: one chunk of channels (flat tiling: of up to 4 images, whole)
        const int64_t plane = (int64_t)s.H * s.W * 4;
        const int64_t reach = v.img != 0 ? 4 * (int64_t)s.C * plane
                              : (v.pair != convd::PAIR_C || v.pointwise) ? (int64_t)s.C * plane : (int64_t)v.CB * plane;
        if (reach >= ((int64_t)1 << 31)) return false;
        // rectangular channel-pair tiles bound their loads by the bytes from the chunk's first channel to the
        // image's end, a 32-bit quantity
        if (v.img == 0 && v.pair == convd::PAIR_C && !v.pointwise && (int64_t)s.C * plane >= ((int64_t)1 << 32)) return false;
    }
    const int64_t grid = v.img != 0
                             ? (int64_t)cdiv(s.K, v.KT) * ((((int64_t)s.N * s.P * s.Q) + v.NPB * 32 - 1) / (v.NPB * 32))
                         : pointwise_flat(v, s) ? (int64_t)(v.kloop ? 1 : cdiv(s.K, v.KT)) * cdiv64((int64_t)s.N * s.P * s.Q, v.TQ)
                         : v.pointwise ? (int64_t)cdiv(s.K, v.KT) * cdiv64((int64_t)s.P * s.Q, v.TQ) * s.N
                                       : (int64_t)cdiv(s.K, v.KT) * cdiv(s.P, v.TP) * cdiv(s.Q, v.TQ) * s.N;
    return grid > 0 && grid < kMaxElems;
}

void fill(conv_direct_plan *p, const Shape &s, const Variant &v)
{
    p->s = s;
    p->v = &v;
    // (merged phases: the eight k-waves of a workgroup are four phases of two 32-channel blocks)
    p->ktiles = v.merged ? cdiv(s.K, 64) : v.kloop ? 1 : cdiv(s.K, v.KT);
    p->pw_flat = pointwise_flat(v, s) ? 1 : 0;
    if (p->pw_flat) {
        p->tilesP = 1;
        p->tilesQ = (int)cdiv64((int64_t)s.N * s.P * s.Q, v.TQ);
        p->grid = (unsigned)((int64_t)p->ktiles * p->tilesQ);
    } else if (v.img != 0) {
        // flat tiling: tilesQ pixel tiles of NPB*32 consecutive pixels over all images
        p->tilesP = 1;
        p->tilesQ = (int)((((int64_t)s.N * s.P * s.Q) + v.NPB * 32 - 1) / (v.NPB * 32));
        p->grid = (unsigned)((int64_t)p->ktiles * p->tilesQ);
    } else if (v.pointwise) {
        // every image is one row of P*Q pixels, cut into tilesQ tiles of TQ
        p->tilesP = 1;
        p->tilesQ = (int)cdiv64((int64_t)s.P * s.Q, v.TQ);
        p->grid = (unsigned)((int64_t)p->ktiles * p->tilesQ * s.N);
    } else {
        p->tilesP = cdiv(s.P, v.TP);
        p->tilesQ = cdiv(s.Q, v.TQ);
        p->grid = (unsigned)((int64_t)p->ktiles * p->tilesP * p->tilesQ * s.N);
    }
    p->lds_bytes = v.lds_bytes(s);
    // issued MACs: every workgroup runs KT x (NPB*32) outputs over the padded reduction
    double red;
    if (v.R == 0) {
        red = 2.0 * cdiv(s.C, 2) * s.R * s.S;
    } else if (v.pointwise) {
        red = 2.0 * cdiv(s.C, 2);
    } else if (v.pair == convd::PAIR_C) {
        red = (double)cdiv(s.C, v.CB) * v.CB * s.R * s.S;
    } else if (v.pair == convd::PAIR_T) {
        red = (double)s.C * s.R * s.S;
    } else {
        red = (double)s.C * (2 * ((s.R + 1) / 2)) * s.S;
    }
    const double issued = (double)p->grid * (v.kloop ? cdiv(s.K, v.KT) * v.KT : v.KT) * (v.NPB * 32.0) * red;
    const double useful = (double)s.N * s.K * s.P * s.Q * ((double)s.C * s.R * s.S);
    p->mfma_efficiency = useful / issued;
}

// Estimated run time of the plan in shader clocks (a model, used only to rank the
// variants that can run a shape).  It is the analytical counterpart, for this GPU, of
// the paper's Section 3.1 reasoning about how many independent FMAs keep the pipes
// busy (Equation 1) within the register file (Equation 2):
//   * a wave needs `mfma_per_wave` 64-clock MFMAs; a SIMD shared by w resident waves
//     finishes them in w times that, at an efficiency that is high when a second wave
//     covers the first one's waits and lower when a wave has the pipe to itself;
//   * workgroups fill the chip's resident slots round after round; the last, partial
//     round runs with fewer waves per SIMD;
//   * every workgroup re-stages its input window: bytes that cross L2 -> LDS, charged
//     at a bandwidth fitted to measurements.  This is what makes compact tiles (small
//     halo) and wide channel tiles (fewer re-reads of the input) win ties.
double cost(const conv_direct_plan &p)
{
    const Variant &v = *p.v;
    const Shape &s = p.s;
    const int wpw = v.threads / 64;                                // waves per workgroup
    // (a data gradient's phases: one launch; at most so many: phases without a tap are not launched; merged: the phases
    // are waves of one workgroup)
    const int64_t grid = (int64_t)p.grid * ((p.ph_stride && !v.merged) ? p.ph_stride * p.ph_stride : 1);
    const double useful = (double)s.N * s.K * s.P * s.Q * ((double)s.C * s.R * s.S);
    const double mfma_per_wave = useful / p.mfma_efficiency / p.grid / wpw / 2048.0;   // 32*32*2 MACs each
    auto round_time = [&](int wgs_per_cu) {
        const int waves_per_simd = cdiv(wgs_per_cu * wpw, 4);      // the busiest SIMD
        const double eff = waves_per_simd >= 2 ? 0.96 : 0.80;
        // (merged phases: the padded count has 4 taps per wave; the busiest SIMD runs a four-tap and a one-tap wave)
        return mfma_per_wave * (v.merged ? 0.625 : 1.0) * 64.0 * waves_per_simd / eff;
    };
    int occ = v.occupancy;
    const int lds_fit = (int)(kLdsPerCU / (p.lds_bytes ? p.lds_bytes : 1));
    if (occ > lds_fit) occ = lds_fit;
    if (occ < 1) occ = 1;
    const int64_t slots = (int64_t)kNumCU * occ;
    const int64_t full = grid / slots, rem = grid % slots;
    double c = full * round_time(occ);
    if (rem) c += round_time((int)cdiv64(rem, kNumCU));
    // prologue and epilogue of each workgroup, mostly hidden behind its CU neighbours
    // (per round every resident workgroup of a CU pays it: small workgroups, many per CU, pay more)
    // (pointwise workgroups have no LDS to fill and no barrier: four of them per CU cost no more than two)
    c += 12000.0 * (v.pointwise ? (occ > 4 ? occ / 4.0 : 1.0) : (occ > 2 ? occ / 2.0 : 1.0)) * (double)cdiv64(grid, slots);
    if (s.R == 1 && s.S == 1) {
        // A 1x1 layer that writes more than it reads is bound by its stores: the results of a workgroup leave as one
        // burst, behind which the operand loads of its CU neighbours wait.  Smaller workgroups, more of them per CU,
        // spread the bursts (measured on 64 -> 256 channels at 56x56: 6 % for 57 KB instead of 115 KB a burst).
        const double in_b = (double)s.N * s.C * s.H * s.W * 4.0, out_b = (double)s.N * s.K * s.P * s.Q * 4.0;
        // (a workgroup that walks all output channels stores block by block along the way)
        if (out_b > in_b && !v.kloop) c += (double)cdiv64(grid, slots) * (out_b / (double)grid) / 4.0 / occ;
    }
    // input staging traffic
    double staged;   // floats one workgroup stages in total
    if (v.R == 0) {
        staged = (double)s.C * s.R * (2.0 * ((convd_generic_tq - 1) * s.stride + s.S)) * 2.0;
    } else if (v.pair != convd::PAIR_C) {
        staged = (double)s.C * v.window;
    } else {
        staged = (double)cdiv(s.C, v.CB) * v.CB * v.window;
    }
    c += staged * 4.0 * grid / 16384.0;   // bytes / (64 B per clock and CU, all CUs at once)
    // filter traffic: every wave fetches the whole filter slice of its 32-channel blocks,
    // however few pixels it owns (what makes very small pixel tiles expensive)
    if (v.R != 0) {
        c += (double)grid * wpw * (v.kloop ? cdiv(s.K, v.KT) : 1) * 32.0 * s.C * s.R * s.S * 4.0 / 16384.0;
    }
    if (v.R == 0) c *= 3.0;   // the runtime-shape fallback synchronises far more often
    return c;
}

// Measured choices (conv_direct_create_tuned, conv_direct_tuning_load): shape and layouts -> variant name.
struct TunedEntry {
    int key[11];   // N C H W K R S stride pad in_layout out_layout
    std::string variant;
};
std::vector<TunedEntry> g_tuned;

const TunedEntry *tuned_lookup(const int (&key)[11])
{
    for (const TunedEntry &e : g_tuned)
        if (std::memcmp(e.key, key, sizeof key) == 0) return &e;
    return nullptr;
}

void tuned_store(const int (&key)[11], const char *variant)
{
    for (TunedEntry &e : g_tuned)
        if (std::memcmp(e.key, key, sizeof key) == 0) {
            e.variant = variant;
            return;
        }
    TunedEntry e;
    std::memcpy(e.key, key, sizeof key);
    e.variant = variant;
    g_tuned.push_back(e);
}

int make_plan(conv_direct_plan **plan, const char *forced, int N, int C, int H, int W, int K, int R,
              int S, int stride, int pad, int in_blocked = 0, int out_blocked = 0, bool pair_family_only = false, int phase_stride = 0,
              bool tail_capable_only = false)
{
    if (!plan) return CONV_DIRECT_EINVAL;
    *plan = nullptr;
    Shape s;
    const int rc = validate(N, C, H, W, K, R, S, stride, pad, &s);
    if (rc != CONV_DIRECT_OK) return rc;
    if (!forced && !pair_family_only) {
        // a measured choice for exactly this problem wins over the model, if it still names a variant that can run it
        const int key[11] = {N, C, H, W, K, R, S, stride, pad, in_blocked, out_blocked};
        if (const TunedEntry *e = tuned_lookup(key)) {
            const std::string name = e->variant;   // (a copy: the recursion below does not touch the table, but be safe)
            // (a second choice for calls with a tail must have one: otherwise the measured name does not count here,
            // and a plan for it would ask for a second choice of its own without end)
            if (make_plan(plan, name.c_str(), N, C, H, W, K, R, S, stride, pad, in_blocked, out_blocked, false, 0, tail_capable_only) ==
                CONV_DIRECT_OK)
                return CONV_DIRECT_OK;
        }
    }

    conv_direct_plan best{};
    bool have = false;
    double best_cost = 0.0;
    int count = 0;
    const Variant *const *table = convd::variant_table(&count);
    for (int i = 0; i < count; ++i) {
        const Variant &v = *table[i];
        if (forced && std::strcmp(forced, v.name) != 0) continue;
        if (!applicable(v, s, in_blocked, out_blocked)) continue;
        if (pair_family_only && (v.pair != convd::PAIR_C || v.pointwise || v.R == 0)) continue;
        if (v.merged && phase_stride != 2) continue;   // (serves only the four phases of a stride-2 layer's data gradient)
        if (tail_capable_only && v.no_tail) continue;
        conv_direct_plan cand{};
        fill(&cand, s, v);
        cand.in_blocked = in_blocked;
        cand.out_blocked = out_blocked;
        cand.ph_stride = phase_stride;
        const double c = cost(cand);
        cand.model_clocks = c;
        if (!have || c < best_cost) {
            best = cand;
            best_cost = c;
            have = true;
        }
    }
    if (!have) return CONV_DIRECT_EUNSUPPORTED;
    conv_direct_plan *p = new (std::nothrow) conv_direct_plan(best);
    if (!p) return CONV_DIRECT_ENOMEM;
    if (best.v->no_tail && !phase_stride) {
        // the second choice, among the variants that can fuse a tail (the runtime-shape kernel is one: there always is one)
        const int rc2 = make_plan(&p->tail_plan, nullptr, N, C, H, W, K, R, S, stride, pad, in_blocked, out_blocked, pair_family_only,
                                  0, true);
        if (rc2 != CONV_DIRECT_OK) {
            delete p;
            return rc2;
        }
    }
    *plan = p;
    return CONV_DIRECT_OK;
}

}  // namespace

extern "C" {

int conv_direct_create(conv_direct_plan **plan, int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad)
{
    return make_plan(plan, nullptr, N, C, H, W, K, R, S, stride, pad);
}

int conv_direct_create_with_variant(conv_direct_plan **plan, const char *variant, int N, int C, int H,
                                    int W, int K, int R, int S, int stride, int pad)
{
    if (!variant) {
        if (plan) *plan = nullptr;
        return CONV_DIRECT_EINVAL;
    }
    return make_plan(plan, variant, N, C, H, W, K, R, S, stride, pad);
}

const char *conv_direct_variant_name(int index)
{
    int count = 0;
    const Variant *const *table = convd::variant_table(&count);
    return (index >= 0 && index < count) ? table[index]->name : nullptr;
}

int conv_direct_run(const conv_direct_plan *plan, const float *in, const float *w, float *out,
                    void *stream)
{
    return conv_direct_run_fused(plan, in, w, nullptr, nullptr, 0, out, stream);
}

int conv_direct_run_fused(const conv_direct_plan *plan, const float *in, const float *w, const float *bias,
                          const float *residual, int relu, float *out, void *stream)
{
    if (!plan || !in || !w || !out || !plan->v) return CONV_DIRECT_EINVAL;
    if (((uintptr_t)in | (uintptr_t)w | (uintptr_t)out | (uintptr_t)bias | (uintptr_t)residual) & 3u)
        return CONV_DIRECT_EALIGN;
    if ((bias || residual || relu) && plan->tail_plan) plan = plan->tail_plan;   // (same problem, a variant that fuses tails)

    convd::KernelArgs a;
    a.in = in;
    a.w = w;
    a.out = out;
    a.s = plan->s;
    a.tilesP = plan->tilesP;
    a.tilesQ = plan->tilesQ;
    a.ktiles = plan->ktiles;
    a.out_blocked = plan->out_blocked;
    a.in_blocked = plan->in_blocked;
    a.dil = plan->dil;
    a.pad_h = plan->pad_h;
    a.pad_w = plan->pad_w;
    a.bias = bias;
    a.residual = residual;
    a.relu = relu ? 1 : 0;
    a.ost = a.onb = a.ooh = a.oow = a.OH = a.OW = a.ofr = 0;
    if (plan->ph_stride) {
        // data gradient of a strided layer: clear dx (positions no window of the forward pass touches stay
        // zero), then one stride-1 convolution of dy per phase, each storing to its own positions of dx
        if (bias || residual || relu) return CONV_DIRECT_EINVAL;
        const int st = plan->ph_stride, RT = plan->s.R;
        const int KO = plan->out_blocked ? (plan->s.K + 3) / 4 * 4 : plan->s.K;   // channels an image of dx occupies
        const int nb = st < plan->fwd_R ? st : plan->fwd_R;   // phases per dimension that have a tap
        // Position h of dx belongs to phase (h + pad) % st, result row (h + pad) / st.  When every phase is launched and
        // the phases' result rows and columns (plan->s.P x plan->s.Q of them) reach the last position, every element of dx
        // is stored by exactly one phase and there is nothing to clear (blocked dx: the spare channels of a last pencil
        // are stored as zeros with their pencil).
        const bool covered = nb == st && (plan->ph_H - 1 + plan->ph_pad) / st <= plan->s.P - 1 &&
                             (plan->ph_W - 1 + plan->ph_pad) / st <= plan->s.Q - 1;
        hipError_t e = covered ? hipSuccess
                               : convd::launch_fill_zero(out, (long long)plan->s.N * KO * plan->ph_H * plan->ph_W, (hipStream_t)stream);
        a.ost = st;                                       // (the channel-pair kernels' output re-mapping, see KernelArgs)
        a.onb = nb;
        a.OH = plan->ph_H;
        a.OW = plan->ph_W;
        a.ooh = a.oow = -plan->ph_pad;
        a.ofr = plan->fwd_R;
        (void)RT;
        if (e == hipSuccess) e = plan->v->launch(a, plan->v->merged ? plan->grid : plan->grid * (unsigned)(nb * nb), (hipStream_t)stream);
        return launched(e);
    }
    const hipError_t e = plan->v->launch(a, plan->grid, (hipStream_t)stream);
    if (e != hipSuccess) {
        t_last_hip_error = (int)e;
        return CONV_DIRECT_EHIP;
    }
    return CONV_DIRECT_OK;
}

int conv_direct_destroy(conv_direct_plan *plan)
{
    if (plan) delete plan->tail_plan;
    delete plan;
    return CONV_DIRECT_OK;
}

int conv_direct_output_dims(const conv_direct_plan *plan, int *P, int *Q)
{
    if (!plan || !P || !Q || !plan->v) return CONV_DIRECT_EINVAL;
    *P = plan->ph_stride ? plan->ph_H : plan->s.P;
    *Q = plan->ph_stride ? plan->ph_W : plan->s.Q;
    return CONV_DIRECT_OK;
}

size_t conv_direct_workspace_bytes(const conv_direct_plan *) { return 0; }

int conv_direct_plan_info(const conv_direct_plan *plan, char *buf, size_t n)
{
    if (!plan || (!buf && n)) return CONV_DIRECT_EINVAL;
    if (plan->wv) {
        const Shape &s = plan->s;
        return std::snprintf(buf, n,
                             "variant=%s kind=wgrad N=%d C=%d H=%d W=%d K=%d R=%d S=%d stride=%d pad=%d P=%d Q=%d "
                             "ktiles=%d cgroups=%d splits=%d grid=%u threads=%d x_layout=%s dy_layout=%s dw_layout=%s workspace_bytes=0",
                             plan->wv->name, s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.P, s.Q, plan->ktiles,
                             plan->wg_cgroups, plan->wg_splits, plan->grid, 64 * plan->wv->WK * plan->wv->WC * plan->wv->WB,
                             plan->in_blocked ? "blocked" : "plain", plan->wg_dy_blocked ? "blocked" : "plain",
                             plan->out_blocked ? "blocked" : "plain");
    }
    const Variant &v = *plan->v;
    const Shape &s = plan->s;
    return std::snprintf(buf, n,
                         "variant=%s N=%d C=%d H=%d W=%d K=%d R=%d S=%d stride=%d pad=%d P=%d Q=%d "
                         "TP=%d TQ=%d KT=%d NPB=%d CB=%d pair=%s tilesP=%d tilesQ=%d ktiles=%d grid=%u "
                         "threads=%d lds_bytes=%zu occupancy=%d flat=%d pointwise=%d mfma_efficiency=%.6g in_layout=%s "
                         "out_layout=%s dgrad_phases=%d extra_caller_bytes=%zu tail_variant=%s model_clocks=%.0f workspace_bytes=0",
                         v.name, s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.P, s.Q, v.TP, v.TQ,
                         v.merged ? 64 : v.kloop ? cdiv(plan->s.K, v.KT) * v.KT : v.KT, v.NPB, v.CB, v.pair == convd::PAIR_C ? "c" : v.pair == convd::PAIR_R ? "r" : "t", plan->tilesP,
                         plan->tilesQ, plan->ktiles, plan->grid, v.threads, plan->lds_bytes, v.occupancy,
                         (v.img != 0 || plan->pw_flat) ? 1 : 0, v.pointwise, plan->mfma_efficiency, plan->in_blocked ? "blocked" : "plain",
                         plan->out_blocked ? "blocked" : "plain",
                         plan->ph_stride ? (plan->ph_stride < plan->fwd_R ? plan->ph_stride : plan->fwd_R) * (plan->ph_stride < plan->fwd_R ? plan->ph_stride : plan->fwd_R) : 0,
                         conv_direct_dgrad_wt_elems(plan) * sizeof(float), plan->tail_plan ? plan->tail_plan->v->name : "same", plan->model_clocks);
}

const char *conv_direct_strerror(int code)
{
    switch (code) {
        case CONV_DIRECT_OK: return "ok";
        case CONV_DIRECT_EINVAL: return "invalid argument (dimension, stride, pad or NULL pointer)";
        case CONV_DIRECT_EUNSUPPORTED: return "shape not supported (tensor too large or no variant fits)";
        case CONV_DIRECT_EALIGN: return "device pointer not 4-byte aligned";
        case CONV_DIRECT_EHIP: return "HIP launch failed (see conv_direct_last_hip_error)";
        case CONV_DIRECT_ENOMEM: return "host allocation failed";
        case CONV_DIRECT_ETOOBIG: return "transformed filter larger than the library's static array (CONV_DIRECT_STATIC_WT_ELEMS floats)";
        default: return "unknown error code";
    }
}

int conv_direct_last_hip_error(void) { return t_last_hip_error; }

int conv_direct_create_ex(conv_direct_plan **plan, const char *variant, int N, int C, int H, int W, int K, int R,
                          int S, int stride, int pad, int in_layout, int out_layout)
{
    if ((in_layout != CONV_DIRECT_LAYOUT_PLAIN && in_layout != CONV_DIRECT_LAYOUT_BLOCKED) ||
        (out_layout != CONV_DIRECT_LAYOUT_PLAIN && out_layout != CONV_DIRECT_LAYOUT_BLOCKED)) {
        if (plan) *plan = nullptr;
        return CONV_DIRECT_EINVAL;
    }
    return make_plan(plan, variant, N, C, H, W, K, R, S, stride, pad, in_layout, out_layout);
}

int conv_direct_create_layout(conv_direct_plan **plan, int N, int C, int H, int W, int K, int R, int S, int stride,
                              int pad, int in_layout, int out_layout)
{
    if ((in_layout != CONV_DIRECT_LAYOUT_PLAIN && in_layout != CONV_DIRECT_LAYOUT_BLOCKED) ||
        (out_layout != CONV_DIRECT_LAYOUT_PLAIN && out_layout != CONV_DIRECT_LAYOUT_BLOCKED)) {
        if (plan) *plan = nullptr;
        return CONV_DIRECT_EINVAL;
    }
    return make_plan(plan, nullptr, N, C, H, W, K, R, S, stride, pad, in_layout, out_layout);
}

int conv_direct_create_tuned(conv_direct_plan **plan, int N, int C, int H, int W, int K, int R, int S, int stride,
                             int pad, int in_layout, int out_layout, const float *in, const float *w, float *out,
                             void *stream, int reps)
{
    if (plan) *plan = nullptr;
    if (!plan || !in || !w || !out || reps < 1) return CONV_DIRECT_EINVAL;
    if ((in_layout != CONV_DIRECT_LAYOUT_PLAIN && in_layout != CONV_DIRECT_LAYOUT_BLOCKED) ||
        (out_layout != CONV_DIRECT_LAYOUT_PLAIN && out_layout != CONV_DIRECT_LAYOUT_BLOCKED))
        return CONV_DIRECT_EINVAL;
    if (((uintptr_t)in | (uintptr_t)w | (uintptr_t)out) & 3u) return CONV_DIRECT_EALIGN;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        t_last_hip_error = (int)hipGetLastError();
        return CONV_DIRECT_EHIP;
    }
    int count = 0, rc = CONV_DIRECT_EUNSUPPORTED;
    const Variant *const *table = convd::variant_table(&count);
    std::string best;
    float best_ms = 0.f;
    for (int i = 0; i < count; ++i) {
        conv_direct_plan *cand = nullptr;
        if (make_plan(&cand, table[i]->name, N, C, H, W, K, R, S, stride, pad, in_layout, out_layout) != CONV_DIRECT_OK)
            continue;
        int r = conv_direct_run(cand, in, w, out, stream);   // untimed: code object load, caches
        if (r == CONV_DIRECT_OK && hipEventRecord(e0, st) != hipSuccess) r = CONV_DIRECT_EHIP;
        for (int k = 0; k < reps && r == CONV_DIRECT_OK; ++k) r = conv_direct_run(cand, in, w, out, stream);
        float ms = 0.f;
        if (r == CONV_DIRECT_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                                    hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
            r = CONV_DIRECT_EHIP;
        conv_direct_destroy(cand);   // (with its second choice, if it has one)
        if (r != CONV_DIRECT_OK) {
            rc = r;
            best.clear();
            break;
        }
        if (best.empty() || ms < best_ms) {
            best = table[i]->name;
            best_ms = ms;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (best.empty()) return rc;
    const int key[11] = {N, C, H, W, K, R, S, stride, pad, in_layout, out_layout};
    tuned_store(key, best.c_str());
    return make_plan(plan, best.c_str(), N, C, H, W, K, R, S, stride, pad, in_layout, out_layout);
}

int conv_direct_tuning_save(const char *path)
{
    if (!path) return CONV_DIRECT_EINVAL;
    FILE *f = std::fopen(path, "w");
    if (!f) return CONV_DIRECT_EINVAL;
    for (const TunedEntry &e : g_tuned) {
        for (int v : e.key) std::fprintf(f, "%d ", v);
        std::fprintf(f, "%s\n", e.variant.c_str());
    }
    return std::fclose(f) == 0 ? CONV_DIRECT_OK : CONV_DIRECT_EINVAL;
}

int conv_direct_tuning_load(const char *path)
{
    if (!path) return CONV_DIRECT_EINVAL;
    FILE *f = std::fopen(path, "r");
    if (!f) return CONV_DIRECT_EINVAL;
    std::vector<TunedEntry> got;
    char line[512];
    int rc = CONV_DIRECT_OK;
    while (std::fgets(line, sizeof line, f)) {
        if (line[0] == '#' || line[0] == '\n') continue;
        TunedEntry e;
        char name[128];
        int *k = e.key;
        if (std::sscanf(line, "%d %d %d %d %d %d %d %d %d %d %d %127s", k, k + 1, k + 2, k + 3, k + 4, k + 5, k + 6, k + 7,
                        k + 8, k + 9, k + 10, name) != 12) {
            rc = CONV_DIRECT_EINVAL;
            break;
        }
        e.variant = name;
        got.push_back(e);
    }
    std::fclose(f);
    if (rc != CONV_DIRECT_OK) return rc;   // nothing taken from a malformed file
    for (const TunedEntry &e : got) tuned_store(e.key, e.variant.c_str());
    return CONV_DIRECT_OK;
}

int conv_direct_tuning_clear(void)
{
    g_tuned.clear();
    return CONV_DIRECT_OK;
}

int conv_direct_tuning_size(void) { return (int)g_tuned.size(); }

int conv_direct_create_wgrad(conv_direct_plan **plan, int N, int C, int H, int W, int K, int R, int S, int stride,
                             int pad)
{
    return conv_direct_create_wgrad_ex(plan, nullptr, N, C, H, W, K, R, S, stride, pad);
}

const char *conv_direct_wgrad_variant_name(int index)
{
    int count = 0;
    const convd::WgradVariant *table = convd::wgrad_table(&count);
    return (index >= 0 && index < count) ? table[index].name : nullptr;
}

static int create_wgrad(conv_direct_plan **plan, const char *variant, bool one_split, int N, int C, int H, int W, int K, int R, int S,
                        int stride, int pad, int xb = 0, int yb = 0, int wb = 0);

int conv_direct_create_wgrad_layout(conv_direct_plan **plan, const char *variant, int deterministic, int N, int C, int H, int W,
                                    int K, int R, int S, int stride, int pad, int x_layout, int dy_layout, int dw_layout)
{
    for (int l : {x_layout, dy_layout, dw_layout})
        if (l != CONV_DIRECT_LAYOUT_PLAIN && l != CONV_DIRECT_LAYOUT_BLOCKED) {
            if (plan) *plan = nullptr;
            return CONV_DIRECT_EINVAL;
        }
    return create_wgrad(plan, variant, deterministic != 0, N, C, H, W, K, R, S, stride, pad, x_layout == CONV_DIRECT_LAYOUT_BLOCKED,
                        dy_layout == CONV_DIRECT_LAYOUT_BLOCKED, dw_layout == CONV_DIRECT_LAYOUT_BLOCKED);
}

int conv_direct_create_wgrad_ex(conv_direct_plan **plan, const char *variant, int N, int C, int H, int W, int K, int R, int S,
                                int stride, int pad)
{
    return create_wgrad(plan, variant, false, N, C, H, W, K, R, S, stride, pad);
}

int conv_direct_create_wgrad_deterministic(conv_direct_plan **plan, int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    return create_wgrad(plan, nullptr, true, N, C, H, W, K, R, S, stride, pad);
}

static int create_wgrad(conv_direct_plan **plan, const char *variant, bool one_split, int N, int C, int H, int W, int K, int R, int S,
                        int stride, int pad, int xb, int yb, int wb)
{
    if (!plan) return CONV_DIRECT_EINVAL;
    *plan = nullptr;
    Shape s;
    const int rc = validate(N, C, H, W, K, R, S, stride, pad, &s);
    if (rc != CONV_DIRECT_OK) return rc;
    // offsets inside one image and one chunk's channel range are 32-bit
    // (blocked activations: whole pencils of 4 channels; a blocked dw: whole blocks of 32 x 4 channels)
    if ((int64_t)(K + 3) * s.P * s.Q * 4 >= ((int64_t)1 << 31) || (int64_t)(C + 3) * H * W * 4 >= ((int64_t)1 << 31) ||
        (int64_t)(K + 31) * (C + 3) * R * S >= kMaxElems)
        return CONV_DIRECT_EUNSUPPORTED;
    int count = 0;
    const convd::WgradVariant *table = convd::wgrad_table(&count);
    const convd::WgradVariant *best = nullptr;
    double best_score = 0.0;
    for (int i = 0; i < count; ++i) {
        const convd::WgradVariant &v = table[i];
        if (variant && std::strcmp(variant, v.name) != 0) continue;
        if (v.S == 0 ? stride > v.stride : (v.S != S || v.stride != stride)) continue;   // S = 0: the fallback
        if (v.pack && !v.allr && (C * S > 32 * v.pack || C > 32 * v.CBW)) continue;
        if (v.pack && v.allr && (C * R * S > 32 * v.pack || C > 4)) continue;
        if (v.qw && v.qw != s.Q) continue;
        if (v.allr && R != S) continue;
        // used fraction of the MFMA work: pixels of a row over whole chunks, output and input channels over whole tiles
        const double cols = v.pack ? (double)C * S * (v.allr ? R : 1) / (32.0 * v.pack) : (double)C / ((double)cdiv(C, 32 * v.CBW * v.WC) * 32 * v.CBW * v.WC);
        const double pix = v.qw ? (double)s.P * s.Q / ((double)cdiv(s.P, v.PXC / v.qw) * v.PXC) : (double)s.Q / ((double)cdiv(s.Q, v.PXC) * v.PXC);
        // (eight waves per CU keep the matrix pipes busier than four: a wave's waits are covered; as one
        // workgroup they also stage dy once for twice the channels: measured 1.04)
        const int nwaves = v.WK * v.WC * v.WB;
        const double score = pix * (v.per_cu * nwaves >= 8 ? 1.12 : 1.0) * (nwaves >= 8 ? 1.03 : 1.0) *
                             ((double)K / ((double)cdiv(K, 32 * v.WK) * 32 * v.WK)) * cols * (v.WK * v.WC * v.WB >= 4 ? 1.0 : 0.98) * (v.S == 0 ? 0.5 : 1.0) * (v.allr ? 1.25 * (v.WB > 1 ? 1.2 * (double)(v.CBW * S * R) / ((double)cdiv(v.CBW * S * R, v.WB) * v.WB) : 1.0) : 1.0);   // (coalesced atomic additions, dy staged once for all filter rows: measured 1.2 to 1.3)
        if (!best || score > best_score) {
            best = &v;
            best_score = score;
        }
    }
    if (!best) return CONV_DIRECT_EUNSUPPORTED;
    conv_direct_plan *p = new (std::nothrow) conv_direct_plan();
    if (!p) return CONV_DIRECT_ENOMEM;
    p->s = s;
    p->v = nullptr;
    p->wv = best;
    p->ktiles = cdiv(K, 32 * best->WK);
    p->wg_cgroups = cdiv(C, 32 * best->CBW * best->WC);
    const int64_t tiles = (int64_t)p->ktiles * p->wg_cgroups * (best->allr ? 1 : R) * (best->S == 0 ? S : 1);   // (fallback: one tap each)
    // How many workgroups share the pixels of one result tile: more of them fill the chip more
    // evenly, but every one adds a full set of atomic additions into dw.  One or two workgroups run
    // per CU at a time (their LDS).  Estimated clocks: rounds * (chunks of a workgroup * MFMA clocks of a
    // chunk + the atomics of its accumulators), the constants fitted to measurements.
    const int nblk = cdiv(best->pack ? best->pack : best->CBW * (best->S == 0 ? 1 : S) * (best->allr ? R : 1), best->WB);
    const int npx = best->qw ? (best->PXC / best->qw) * best->qw : best->PXC;
    const int64_t units = best->qw ? (int64_t)N * cdiv(s.P, best->PXC / best->qw) : (int64_t)N * s.P;
    const int64_t chunks_per_unit = best->qw ? 1 : cdiv(s.Q, best->PXC);
    const double chunk_clk = (npx / 2.0) * nblk * 64.0 / 0.65 * (best->per_cu == 2 ? 1.6 : 1.0);   // (two share a SIMD)
    const double atomics_clk = nblk * 16.0 * 2000.0;
    const int64_t slots = (int64_t)kNumCU * best->per_cu;
    int64_t splits = 1;
    double best_clk = 0.0;
    for (int64_t sp = 1; sp <= units && sp <= (one_split ? 1 : 4096); ++sp) {
        const double clk = (double)cdiv64(tiles * sp, slots) * ((double)cdiv64(units, sp) * chunks_per_unit * chunk_clk + atomics_clk);
        if (sp == 1 || clk < best_clk) {
            best_clk = clk;
            splits = sp;
        }
    }
    p->wg_splits = (int)splits;
    p->in_blocked = xb;
    p->wg_dy_blocked = yb;
    p->out_blocked = wb;
    p->grid = (unsigned)(tiles * splits);
    *plan = p;
    return CONV_DIRECT_OK;
}

int conv_direct_run_wgrad(const conv_direct_plan *plan, const float *x, const float *dy, float *dw, void *stream)
{
    if (!plan || !plan->wv || !x || !dy || !dw) return CONV_DIRECT_EINVAL;
    if (((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dw) & 3u) return CONV_DIRECT_EALIGN;
    const Shape &s = plan->s;
    // (one workgroup per result tile stores its sums plainly: nothing to clear, except the spare channels that complete
    // the blocks of a blocked dw)
    const long long dw_elems = plan->out_blocked ? (long long)conv_direct_blocked_w_elems(s.K, s.C, s.R, s.S) : (long long)s.K * s.C * s.R * s.S;
    const bool clear = plan->wg_splits != 1 || (plan->out_blocked && (s.K % 32 != 0 || s.C % 4 != 0));
    hipError_t e = clear ? convd::wgrad_clear(dw, dw_elems, (hipStream_t)stream) : hipSuccess;
    if (e == hipSuccess) {
        convd::WgradArgs a;
        a.x = x;
        a.dy = dy;
        a.dw = dw;
        a.x_blocked = plan->in_blocked;
        a.dy_blocked = plan->wg_dy_blocked;
        a.dw_blocked = plan->out_blocked;
        a.s = s;
        a.ktiles = plan->ktiles;
        a.cgroups = plan->wg_cgroups;
        a.splits = plan->wg_splits;
        e = plan->wv->launch(a, plan->grid, (hipStream_t)stream);
    }
    return launched(e);
}

int conv_direct_create_dgrad(conv_direct_plan **plan, int N, int C, int H, int W, int K, int R, int S, int stride,
                             int pad)
{
    return conv_direct_create_dgrad_layout(plan, N, C, H, W, K, R, S, stride, pad, CONV_DIRECT_LAYOUT_PLAIN,
                                           CONV_DIRECT_LAYOUT_PLAIN);
}

int conv_direct_create_dgrad_layout(conv_direct_plan **plan, int N, int C, int H, int W, int K, int R, int S, int stride,
                                    int pad, int dy_layout, int dx_layout)
{
    return conv_direct_create_dgrad_ex(plan, nullptr, N, C, H, W, K, R, S, stride, pad, dy_layout, dx_layout);
}

int conv_direct_create_dgrad_ex(conv_direct_plan **plan, const char *variant, int N, int C, int H, int W, int K, int R, int S,
                                int stride, int pad, int dy_layout, int dx_layout)
{
    if (!plan) return CONV_DIRECT_EINVAL;
    *plan = nullptr;
    if ((dy_layout != CONV_DIRECT_LAYOUT_PLAIN && dy_layout != CONV_DIRECT_LAYOUT_BLOCKED) ||
        (dx_layout != CONV_DIRECT_LAYOUT_PLAIN && dx_layout != CONV_DIRECT_LAYOUT_BLOCKED))
        return CONV_DIRECT_EINVAL;
    const int dyb = dy_layout == CONV_DIRECT_LAYOUT_BLOCKED, dxb = dx_layout == CONV_DIRECT_LAYOUT_BLOCKED;
    Shape fwd;
    const int rc = validate(N, C, H, W, K, R, S, stride, pad, &fwd);
    if (rc != CONV_DIRECT_OK) return rc;
    if (stride == 1 && R == S && pad <= R - 1) {
        // the forward problem that computes dx: input dy [N][K][P][Q], C output channels
        const int rc1 = make_plan(plan, variant, N, K, fwd.P, fwd.Q, C, R, S, 1, R - 1 - pad, dyb, dxb);
        if (rc1 == CONV_DIRECT_OK) {
            (*plan)->fwd_K = K;  (*plan)->fwd_C = C;  (*plan)->fwd_R = R;  (*plan)->fwd_S = S;
            return rc1;
        }
        if (rc1 != CONV_DIRECT_EUNSUPPORTED) return rc1;
        // (no variant serves that forward problem: the runtime-shape path below)
    }
    // (the kernels' output re-mapping is compiled for filters of up to 4x4 taps a phase)
    if (stride > 1 && R == S && (R + stride - 1) / stride <= 4 && (int64_t)N * ((C + 3) / 4 * 4) * H * W < kMaxElems) {
        // Strided layer, square filter.  With t = h + pad = stride*u + a, only the taps r = a + stride*i reach
        // row h: dx[h] = sum_i dy[u - i] * w[a + stride*i], a stride-1 convolution of dy with the RT = ceil(R/stride)
        // taps of phase a (zeros where a + stride*i >= R), padding RT - 1, whose result u belongs at
        // h = stride*u + a - pad.  So stride^2 convolutions, one per phase (a, b), on the channel-pair kernels,
        // which store with that re-mapping; no workspace.
        const int RT = cdiv(R, stride);
        conv_direct_plan *sub = nullptr;
        if (make_plan(&sub, variant, N, K, fwd.P, fwd.Q, C, RT, RT, 1, RT - 1, dyb, dxb, true, stride) == CONV_DIRECT_OK) {
            sub->ph_stride = stride;
            sub->ph_pad = pad;
            sub->ph_H = H;
            sub->ph_W = W;
            sub->fwd_K = K;  sub->fwd_C = C;  sub->fwd_R = R;  sub->fwd_S = S;
            *plan = sub;
            return CONV_DIRECT_OK;
        }
    }
    // Otherwise (strided layer, unequal filter sides, pad > R-1): the same forward problem over dy
    // with zeros between its elements and paddings R-1-pad, S-1-pad (negative: a crop), on the
    // runtime-shape kernel, whose output size is the layer's input size.
    int count = 0;
    const Variant *const *table = convd::variant_table(&count);
    const Variant *generic = nullptr;
    for (int i = 0; i < count; ++i)
        if (table[i]->R == 0) generic = table[i];
    if (!generic || (variant && std::strcmp(variant, generic->name) != 0)) return CONV_DIRECT_EUNSUPPORTED;
    if ((int64_t)N * K * fwd.P * fwd.Q >= kMaxElems) return CONV_DIRECT_EUNSUPPORTED;
    Shape s{N, K, fwd.P, fwd.Q, C, R, S, 1, 0, H, W};   // in = dy, K' = C, P' x Q' = H x W
    if (generic->lds_bytes(s) > kLdsPerCU) return CONV_DIRECT_EUNSUPPORTED;
    conv_direct_plan *p = new (std::nothrow) conv_direct_plan();
    if (!p) return CONV_DIRECT_ENOMEM;
    fill(p, s, *generic);
    p->in_blocked = dyb;
    p->out_blocked = dxb;
    p->dil = stride;
    p->pad_h = R - 1 - pad;
    p->pad_w = S - 1 - pad;
    p->fwd_K = K;  p->fwd_C = C;  p->fwd_R = R;  p->fwd_S = S;
    *plan = p;
    return CONV_DIRECT_OK;
}

size_t conv_direct_dgrad_wt_elems(const conv_direct_plan *plan)
{
    if (!plan || !plan->v || !plan->fwd_K) return 0;
    // (blocked: whole blocks of 32 layer-input channels and pencils of 4 layer-output channels, see conv_direct_pack_w)
    const size_t kc = plan->in_blocked ? (size_t)((plan->fwd_C + 31) / 32 * 32) * (size_t)((plan->fwd_K + 3) / 4 * 4)
                                       : (size_t)plan->fwd_C * plan->fwd_K;
    if (plan->ph_stride) {
        const int nb = plan->ph_stride < plan->fwd_R ? plan->ph_stride : plan->fwd_R;
        return (size_t)nb * nb * kc * plan->s.R * plan->s.S;
    }
    return kc * plan->fwd_R * plan->fwd_S;
}

int conv_direct_dgrad_prepare(const conv_direct_plan *plan, const float *w, float *wt, void *stream)
{
    if (!plan || !plan->v || !plan->fwd_K || !w || !wt) return CONV_DIRECT_EINVAL;
    if (((uintptr_t)w | (uintptr_t)wt) & 3u) return CONV_DIRECT_EALIGN;
    if (plan->in_blocked)   // the kernels of this plan read blocked weights
        return launched(convd::launch_dgrad_filter_blocked(w, wt, plan->fwd_K, plan->fwd_C, plan->fwd_R, plan->fwd_S,
                                                           plan->ph_stride ? plan->ph_stride : 1, (hipStream_t)stream));
    if (plan->ph_stride)
        return launched(convd::launch_dgrad_phase_filter(w, wt, plan->fwd_K, plan->fwd_C, plan->fwd_R, plan->fwd_S,
                                                         plan->ph_stride, (hipStream_t)stream));
    return launched(convd::launch_dgrad_filter(w, wt, plan->fwd_K, plan->fwd_C, plan->fwd_R, plan->fwd_S, (hipStream_t)stream));
}

int conv_direct_run_dgrad_static(const conv_direct_plan *plan, const float *dy, const float *w, float *dx, void *stream)
{
    if (!plan || !plan->v || !plan->fwd_K || !dy || !w || !dx) return CONV_DIRECT_EINVAL;
    if (((uintptr_t)dy | (uintptr_t)w | (uintptr_t)dx) & 3u) return CONV_DIRECT_EALIGN;
    static_assert(CONV_DIRECT_STATIC_WT_ELEMS == convd::STATIC_WT_ELEMS, "the header states the array's size");
    if (conv_direct_dgrad_wt_elems(plan) > (size_t)CONV_DIRECT_STATIC_WT_ELEMS) return CONV_DIRECT_ETOOBIG;
    float *wt = nullptr;   // the static array's address on the current device
    const hipError_t e = convd::static_wt_buffer(&wt);
    if (e != hipSuccess) return launched(e);
    const int rc = conv_direct_dgrad_prepare(plan, w, wt, stream);
    if (rc != CONV_DIRECT_OK) return rc;
    return conv_direct_run(plan, dy, wt, dx, stream);
}

int conv_direct_mfma_probe(void *buf, int iters, void *stream)
{
    if (!buf || iters < 1) return CONV_DIRECT_EINVAL;
    if ((uintptr_t)buf & 7u) return CONV_DIRECT_EALIGN;
    static_assert(CONV_DIRECT_PROBE_BYTES == convd::PROBE_BLOCKS * (256 * 4 + 2 * 8), "the header states the buffer's size");
    float *sums = static_cast<float *>(buf);
    long long *ticks = reinterpret_cast<long long *>(sums + convd::PROBE_BLOCKS * 256);
    return launched(convd::launch_mfma_probe(sums, ticks, iters, (hipStream_t)stream));
}

size_t conv_direct_blocked_act_elems(int N, int C, int H, int W)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return 0;
    return (size_t)N * (size_t)((C + 3) / 4) * 4 * (size_t)H * (size_t)W;
}

size_t conv_direct_blocked_w_elems(int K, int C, int R, int S)
{
    if (K <= 0 || C <= 0 || R <= 0 || S <= 0) return 0;
    return (size_t)((K + 31) / 32) * 32 * (size_t)((C + 3) / 4) * 4 * (size_t)R * (size_t)S;
}

static int rearrange_check(const void *src, const void *dst, unsigned dst_align, int64_t a, int64_t b, int64_t c, int64_t d)
{
    if (!src || !dst || a <= 0 || b <= 0 || c <= 0 || d <= 0) return CONV_DIRECT_EINVAL;
    if (((uintptr_t)src & 3u) || ((uintptr_t)dst & (dst_align - 1))) return CONV_DIRECT_EALIGN;
    return CONV_DIRECT_OK;
}


int conv_direct_pack_act(const float *plain, float *blocked, int N, int C, int H, int W, void *stream)
{
    const int rc = rearrange_check(plain, blocked, 16, N, C, H, W);
    if (rc != CONV_DIRECT_OK) return rc;
    return launched(convd::launch_pack_act(plain, blocked, N, C, H, W, (hipStream_t)stream));
}

int conv_direct_unpack_act(const float *blocked, float *plain, int N, int C, int H, int W, void *stream)
{
    const int rc = rearrange_check(blocked, plain, 4, N, C, H, W);
    if (rc != CONV_DIRECT_OK) return rc;
    return launched(convd::launch_unpack_act(blocked, plain, N, C, H, W, (hipStream_t)stream));
}

int conv_direct_dgrad_filter(const float *w, float *wt, int K, int C, int R, int S, void *stream)
{
    const int rc = rearrange_check(w, wt, 4, K, C, R, S);
    if (rc != CONV_DIRECT_OK) return rc;
    return launched(convd::launch_dgrad_filter(w, wt, K, C, R, S, (hipStream_t)stream));
}

int conv_direct_pack_w(const float *plain, float *blocked, int K, int C, int R, int S, void *stream)
{
    const int rc = rearrange_check(plain, blocked, 4, K, C, R, S);
    if (rc != CONV_DIRECT_OK) return rc;
    return launched(convd::launch_pack_w(plain, blocked, K, C, R, S, (hipStream_t)stream));
}

}  // extern "C"
