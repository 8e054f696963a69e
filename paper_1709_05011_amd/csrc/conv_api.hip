// C-ABI entry points of the convolution passes: validation, workspace planning and dispatch to
// the implicit-GEMM kernels.  Everything that can fail is checked before the first launch, so the
// error paths behave the same on a machine without a GPU.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdio.h>
#include <stdint.h>
#include <stdlib.h>

#include "internal.h"

namespace {

struct Regions {
    size_t off = 0;
    size_t take(size_t bytes) {
        const size_t at = off;
        off += (bytes + 255) & ~(size_t)255;
        return at;
    }
};

struct Plan {
    int P = 0, Q = 0, esize = 4;
    bool nchw = false, bf16 = false;
    int cpad = 0;                    // channel count the kernels see for x / w (c rounded up to 4, to 8 for bf16)
    size_t a_nhwc = 0, b_nhwc = 0, out_nhwc = 0;   // NCHW staging: first operand, second operand, result
    size_t xpad = 0, wpad = 0;       // channel-padded copies
    size_t wt = 0;                   // re-ordered filter for backward-data
    size_t part = 0;                 // split partials of backward-weight
    size_t sk = 0, sk_bytes = 0;     // partial tiles of the stream-K blocks (forward, backward-data)
    int splits = 1, m_per_split = 0;
    bool wgrad_direct = true;
    bool stem_wgrad = false;         // ResNet's first layer: the filter-gradient kernels of conv_stem.hip
    bool wgrad_slab = false;         // bf16 3x3 stride-1 pad-1 layer: the kernel that stages the activations once for all taps
    // bf16 problems the bf16 MFMA kernel does not take (backward-data with k not a multiple of 8, or a strided
    // window other than 1x1): operands are widened to fp32 copies, the fp32 pass runs on them, the result is
    // rounded back to bf16.  Same arithmetic class: exact products of bf16 values, fp32 sums.
    bool via_f32 = false;
    bool phases = false;             // strided window other than 1x1: backward-data as one GEMM per stride phase
    size_t f_a = 0, f_b = 0, f_out = 0, f_ws = 0, f_ws_bytes = 0;
    // few-channel stride-2 layer (a network's first convolution) run as a stride-1 convolution over 2x2 pixel
    // blocks: the unfolded input, the filter (or its gradient) in block form, the inner call's workspace
    bool blocks = false;
    int eh = 0, ew = 0, eph = 0, epw = 0, RB = 0, SB = 0, CU = 0, HB = 0;
    lc_conv_desc inner = {};
    size_t s_u = 0, s_w = 0, s_ws = 0, s_ws_bytes = 0;
    size_t total = 0;
};

lc_status check_desc(const lc_conv_desc* d, int* P, int* Q) {
    if (!d) return LC_ERR_NULL;
    if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->r <= 0 || d->s <= 0 ||
        d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
        return LC_ERR_SHAPE;
    if ((long long)d->h + 2LL * d->pad_h < d->r || (long long)d->w + 2LL * d->pad_w < d->s) return LC_ERR_SHAPE;
    if (d->groups < 0 || (d->groups > 1 && (d->c % d->groups != 0 || d->k % d->groups != 0))) return LC_ERR_SHAPE;
    if (d->dtype != LC_F32 && d->dtype != LC_BF16) return LC_ERR_UNSUPPORTED;
    if (d->layout != LC_NCHW && d->layout != LC_NHWC) return LC_ERR_UNSUPPORTED;
    *P = (d->h + 2 * d->pad_h - d->r) / d->stride_h + 1;
    *Q = (d->w + 2 * d->pad_w - d->s) / d->stride_w + 1;
    // index ranges the kernels hold in 32-bit integers
    const long long lim = INT_MAX;
    const long long cp = (d->c + 7) & ~7, kp = (d->k + 7) & ~7;
    if ((long long)d->n * *P * *Q > lim || (long long)d->n * d->h * d->w > lim) return LC_ERR_UNSUPPORTED;
    if ((long long)d->r * d->s * cp > lim || (long long)d->r * d->s * kp > lim) return LC_ERR_UNSUPPORTED;
    if ((long long)d->h * d->w * cp > lim || (long long)*P * *Q * kp > lim) return LC_ERR_UNSUPPORTED;
    if ((long long)d->k * d->r * d->s * cp > lim) return LC_ERR_UNSUPPORTED;
    return LC_OK;
}

// The implicit-GEMM view of the forward pass (pointers left empty).
GemmConv gemm_fwd(const lc_conv_desc* d, int P, int Q, int cpad) {
    GemmConv g = {};
    g.M = d->n * P * Q;
    g.N = d->k;
    g.Kg = d->r * d->s * cpad;
    g.Hi = d->h;
    g.Wi = d->w;
    g.Ci = cpad;
    g.Po = P;
    g.Qo = Q;
    g.R = d->r;
    g.S = d->s;
    g.sh = d->stride_h;
    g.sw = d->stride_w;
    g.ph = d->pad_h;
    g.pw = d->pad_w;
    g.dh = g.dw = 1;
    g.ldd = d->k;
    g.bf16 = d->dtype == LC_BF16;
    return g;
}

// ... and of the backward-data pass: dy is the gathered tensor, the re-ordered filter [c][R-1-r][S-1-s][k] is B.
GemmConv gemm_bwd_data(const lc_conv_desc* d, int P, int Q) {
    GemmConv g = {};
    g.N = d->c;
    g.Kg = d->r * d->s * d->k;
    g.Hi = P;
    g.Wi = Q;
    g.Ci = d->k;
    g.R = d->r;
    g.S = d->s;
    g.ldd = d->c;
    g.dh = g.dw = 1;
    g.sh = g.sw = 1;
    g.bf16 = d->dtype == LC_BF16;
    if (d->r == 1 && d->s == 1 && d->pad_h == 0 && d->pad_w == 0) {
        // 1x1 window: one GEMM row per dy pixel; with a stride the result lands on the stride grid
        // of dx and the rest of each stride cell is zero.
        g.M = d->n * P * Q;
        g.Po = P;
        g.Qo = Q;
        g.ph = g.pw = 0;
        if (d->stride_h > 1 || d->stride_w > 1) {
            g.scatter = 1;
            g.Ho = d->h;
            g.Wo = d->w;
            g.esh = d->stride_h;
            g.esw = d->stride_w;
        }
    } else {
        // one GEMM row per dx pixel, reading dy as if zeros were inserted between its pixels
        g.M = d->n * d->h * d->w;
        g.Po = d->h;
        g.Qo = d->w;
        g.ph = d->r - 1 - d->pad_h;
        g.pw = d->s - 1 - d->pad_w;
        g.dh = d->stride_h;
        g.dw = d->stride_w;
    }
    return g;
}

// Backward-data through a strided window other than 1x1, phase by phase.  dx pixel (h, w) only receives the taps
// with r = (h + pad_h) mod stride_h (mod stride_h) and s likewise, so the pixels of one phase (a, b) -- h = h0 + stride_h*po,
// w = w0 + stride_w*qo -- are a stride-1 backward-data problem over dy with the Ra x Sb sub-filter r = a + stride_h*i,
// s = b + stride_w*j:  dx[h0 + sh*po] = sum_i dy[po + base - i] * w[a + sh*i], base = (h0 + pad_h - a) / sh.  Its GEMM
// has one row per dx pixel of the phase and scatters to the stride grid of dx, offset by (h0, w0).  No multiplication
// is spent on the zeros a "dilated" read of dy would insert; the phases together do the forward pass's work.
struct Phase {
    GemmConv g;
    int a, b, Ra, Sb;
    size_t w_off;        // elements into the re-ordered filter region
    long long d_off;     // elements into dx: (h0 * W + w0) * C
};
constexpr int kMaxPhases = 16;

int plan_phases(const lc_conv_desc* d, int P, int Q, Phase* out, bool* all_covered) {
    const int sh = d->stride_h, sw = d->stride_w;
    int n = 0;
    size_t w_off = 0;
    *all_covered = true;
    for (int a = 0; a < sh; ++a)
        for (int b = 0; b < sw; ++b) {
            const int Ra = a < d->r ? (d->r - 1 - a) / sh + 1 : 0, Sb = b < d->s ? (d->s - 1 - b) / sw + 1 : 0;
            const int h0 = (((a - d->pad_h) % sh) + sh) % sh, w0 = (((b - d->pad_w) % sw) + sw) % sw;
            const int Ha = h0 < d->h ? (d->h - h0 + sh - 1) / sh : 0, Wb = w0 < d->w ? (d->w - w0 + sw - 1) / sw : 0;
            if (Ha == 0 || Wb == 0) continue;                 // no dx pixel has this phase
            if (Ra == 0 || Sb == 0) {                         // pixels no tap reaches: they stay zero
                *all_covered = false;
                continue;
            }
            Phase& ph = out[n++];
            ph.a = a;
            ph.b = b;
            ph.Ra = Ra;
            ph.Sb = Sb;
            ph.w_off = w_off;
            w_off += (size_t)d->k * d->c * Ra * Sb;
            ph.d_off = ((long long)h0 * d->w + w0) * d->c;
            GemmConv g = {};
            g.M = d->n * Ha * Wb;
            g.N = d->c;
            g.Kg = Ra * Sb * d->k;
            g.Hi = P;
            g.Wi = Q;
            g.Ci = d->k;
            g.Po = Ha;
            g.Qo = Wb;
            g.R = Ra;
            g.S = Sb;
            g.sh = g.sw = 1;
            g.ph = Ra - 1 - (h0 + d->pad_h - a) / sh;
            g.pw = Sb - 1 - (w0 + d->pad_w - b) / sw;
            g.dh = g.dw = 1;
            g.ldd = d->c;
            g.scatter = 1;
            g.Ho = d->h;
            g.Wo = d->w;
            g.esh = sh;
            g.esw = sw;
            g.bf16 = d->dtype == LC_BF16;
            ph.g = g;
        }
    return n;
}

// Whether the phase form applies (shape only): a strided window that is not the 1x1 case, at most 4 x 4 phases, and
// every phase a problem the main kernel's scatter epilogue takes.
bool phases_ok(const lc_conv_desc* d, int P, int Q) {
    static const bool off = getenv("LARSCONV_NO_STRIDE_PHASES") != nullptr;       // comparison runs
    if (off || (d->stride_h == 1 && d->stride_w == 1) || d->stride_h > 4 || d->stride_w > 4) return false;
    if (d->r == 1 && d->s == 1 && d->pad_h == 0 && d->pad_w == 0) return false;
    if ((long long)d->n * d->h * d->w > INT_MAX) return false;
    Phase ph[kMaxPhases];
    bool covered;
    const int n = plan_phases(d, P, Q, ph, &covered);
    if (n == 0) return false;
    for (int i = 0; i < n; ++i)
        if (!lc_conv_gemm_scatter_ok(ph[i].g)) return false;
    return true;
}

lc_conv_desc as_f32(const lc_conv_desc* d) {
    lc_conv_desc f = *d;
    f.dtype = LC_F32;
    return f;
}

// A window that covers the whole (unpadded) input -- a fully connected layer written as a convolution -- is
// the same sums as a 1x1 convolution over one pixel with c*h*w channels: the (c, window) index of the filter
// and the (c, pixel) index of the input run in the same order in either layout.  Rewriting it so matters for
// backward-data, where the general formulation would visit every (pixel, tap) pair and find all but one
// empty.  Returns d itself when the rewrite does not apply (or d is not a valid descriptor to begin with).
const lc_conv_desc* whole_window_as_1x1(const lc_conv_desc* d, lc_conv_desc* store) {
    if (!d || d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->stride_h <= 0 || d->stride_w <= 0) return d;
    if (d->pad_h != 0 || d->pad_w != 0 || d->r != d->h || d->s != d->w || (d->h == 1 && d->w == 1)) return d;
    if (d->layout != LC_NCHW && d->layout != LC_NHWC) return d;
    if (d->groups > 1) return d;
    const long long cc = (long long)d->c * d->h * d->w;
    if (cc > 0x7fffffffLL) return d;
    *store = *d;
    store->c = (int)cc;
    store->h = store->w = store->r = store->s = 1;
    store->stride_h = store->stride_w = 1;
    store->layout = LC_NHWC;              // with one pixel the two layouts coincide
    return store;
}

// A stride-2 window over an image with fewer channels than a 16-byte chunk holds (a network's first layer: 7x7
// over RGB) wastes most of every chunk on padding and runs through the few-channels addressing of the matrix
// kernels.  Over 2x2 pixel blocks it is a stride-1 convolution with 4*C channels per block; with the block
// columns of a window laid side by side (see layout.hip) it becomes RB x 1 over CU channels, which the uniform-tap
// kernels take.  Used for forward and backward-weight of bf16 problems in NHWC when it does not cost more
// multiplications than the padded original (measured on the 7x7 first layer of ResNet-50 at batch 512: forward
// 1.32 -> 0.95 ms, backward-weight 1.51 -> 0.92 ms including the unfolding; in fp32, where padding to four channels
// wastes less, the two forms take the same time and the original is kept).  The layer's backward-data (never
// needed for a first layer) keeps the general path.  ResNet's own first layer (stem_shape below) goes to the kernels of
// conv_stem.hip instead, in both types.
bool plan_blocks(const lc_conv_desc* d, int P, int Q, Plan* pl) {
    static const bool off = getenv("LARSCONV_NO_STEM_BLOCKS") != nullptr;       // comparison runs
    const bool bf16 = d->dtype == LC_BF16;
    if (off || !bf16 || d->layout != LC_NHWC || d->stride_h != 2 || d->stride_w != 2 || d->c > 4 || d->r < 3 || d->s < 3) return false;
    pl->eph = (d->pad_h + 1) & ~1;
    pl->epw = (d->pad_w + 1) & ~1;
    pl->eh = pl->eph - d->pad_h;
    pl->ew = pl->epw - d->pad_w;
    pl->RB = (d->r - 1 + pl->eh) / 2 + 1;
    pl->SB = (d->s - 1 + pl->ew) / 2 + 1;
    const int step = bf16 ? 32 : 16;
    pl->CU = (pl->SB * 4 * d->c + step - 1) / step * step;
    pl->HB = P - 1 + pl->RB;
    const int cpad = bf16 ? (d->c + 7) & ~7 : (d->c + 3) & ~3;
    if ((long long)pl->RB * pl->CU > (long long)d->r * d->s * cpad) return false;
    if ((long long)d->n * pl->HB * Q > INT_MAX || (long long)pl->HB * Q * pl->CU > INT_MAX) return false;
    pl->inner = *d;
    pl->inner.c = pl->CU;
    pl->inner.h = pl->HB;
    pl->inner.w = Q;
    pl->inner.r = pl->RB;
    pl->inner.s = 1;
    pl->inner.stride_h = pl->inner.stride_w = 1;
    pl->inner.pad_h = pl->inner.pad_w = 0;
    return true;
}

// ResNet's first layer in NHWC: the kernels of conv_stem.hip take its forward pass and its filter gradient, fp32 and bf16.
bool stem_shape(const lc_conv_desc* d, int P, int Q) {
    return d->layout == LC_NHWC && d->groups <= 1 &&
           lc_conv_stem_f32_ok(d->n, d->c, d->h, d->w, d->k, d->r, d->s, d->stride_h, d->stride_w, d->pad_h, d->pad_w, P, Q);
}
bool stem_direct(const lc_conv_desc* d, const Plan& pl, lc_pass pass) {
    if (pl.blocks || pl.nchw || !stem_shape(d, pl.P, pl.Q)) return false;
    return pass == LC_PASS_FWD || pass == LC_PASS_BWD_WEIGHT;
}

lc_status make_plan(const lc_conv_desc* d, lc_pass pass, Plan* pl) {
    const lc_status st = check_desc(d, &pl->P, &pl->Q);
    if (st != LC_OK) return st;
    if (pass != LC_PASS_FWD && pass != LC_PASS_BWD_DATA && pass != LC_PASS_BWD_WEIGHT) return LC_ERR_UNSUPPORTED;
    if (pass != LC_PASS_BWD_DATA && !stem_shape(d, pl->P, pl->Q) && plan_blocks(d, pl->P, pl->Q, pl)) {
        pl->blocks = true;
        pl->bf16 = d->dtype == LC_BF16;
        pl->esize = pl->bf16 ? 2 : 4;
        Regions rg;
        pl->s_u = rg.take((size_t)d->n * pl->HB * pl->Q * pl->CU * pl->esize);
        pl->s_w = rg.take((size_t)d->k * pl->RB * pl->CU * (pass == LC_PASS_FWD ? (size_t)pl->esize : sizeof(float)));
        pl->s_ws_bytes = conv2d_workspace_bytes(&pl->inner, pass);
        if (pl->s_ws_bytes) pl->s_ws = rg.take(pl->s_ws_bytes);
        pl->total = rg.off;
        return LC_OK;
    }
    pl->bf16 = d->dtype == LC_BF16;
    pl->esize = pl->bf16 ? 2 : 4;
    pl->nchw = d->layout == LC_NCHW;
    const size_t es = (size_t)pl->esize;
    const size_t nx = (size_t)d->n * d->h * d->w * d->c, ny = (size_t)d->n * pl->P * pl->Q * d->k;
    const size_t nw = (size_t)d->k * d->r * d->s * d->c;
    pl->cpad = pl->bf16 ? (d->c + 7) & ~7 : (d->c + 3) & ~3;
    if (pass == LC_PASS_FWD && stem_direct(d, *pl, pass)) {
        pl->total = 0;                           // the kernel reads x and w and writes y: no workspace
        return LC_OK;
    }
    if (stem_direct(d, *pl, pass) && pass == LC_PASS_BWD_WEIGHT) {
        pl->stem_wgrad = true;
        pl->cpad = d->c;                         // its kernel reads the three channels as they are
    }
    const bool pad = pl->cpad != d->c;
    Regions rg;
    pl->phases = pass == LC_PASS_BWD_DATA && phases_ok(d, pl->P, pl->Q);
    if (pass == LC_PASS_BWD_DATA && pl->bf16 && !pl->phases) {
        const GemmConv g = gemm_bwd_data(d, pl->P, pl->Q);
        if (!lc_conv_gemm_bf16_native(g)) {        // pointers are empty here: a question of shape only
            pl->via_f32 = true;
            const lc_conv_desc f = as_f32(d);
            pl->f_a = rg.take(ny * 4);
            pl->f_b = rg.take(nw * 4);
            pl->f_out = rg.take(nx * 4);
            pl->f_ws_bytes = conv2d_workspace_bytes(&f, pass);
            pl->f_ws = rg.take(pl->f_ws_bytes);
            pl->total = rg.off;
            return LC_OK;
        }
    }
    if (pass == LC_PASS_FWD) {
        if (pl->nchw) {
            pl->a_nhwc = rg.take(nx * es);
            pl->b_nhwc = rg.take(nw * es);
            pl->out_nhwc = rg.take(ny * es);
        }
        if (pad) {
            pl->xpad = rg.take((size_t)d->n * d->h * d->w * pl->cpad * es);
            pl->wpad = rg.take((size_t)d->k * d->r * d->s * pl->cpad * es);
        }
        pl->sk_bytes = lc_conv_gemm_workspace(gemm_fwd(d, pl->P, pl->Q, pl->cpad));
        if (pl->sk_bytes) pl->sk = rg.take(pl->sk_bytes);
    } else if (pass == LC_PASS_BWD_DATA) {
        if (pl->nchw) {
            pl->a_nhwc = rg.take(ny * es);
            pl->b_nhwc = rg.take(nw * es);
            pl->out_nhwc = rg.take(nx * es);
        }
        pl->wt = rg.take(nw * es);
        if (pl->phases) {                                // the phases run one after the other and share the region
            Phase ph[kMaxPhases];
            bool covered;
            const int n = plan_phases(d, pl->P, pl->Q, ph, &covered);
            for (int i = 0; i < n; ++i) {
                const size_t b = lc_conv_gemm_workspace(ph[i].g);
                if (b > pl->sk_bytes) pl->sk_bytes = b;
            }
        } else {
            pl->sk_bytes = lc_conv_gemm_workspace(gemm_bwd_data(d, pl->P, pl->Q));
        }
        if (pl->sk_bytes) pl->sk = rg.take(pl->sk_bytes);
    } else {
        if (pl->nchw) {
            pl->a_nhwc = rg.take(nx * es);
            pl->b_nhwc = rg.take(ny * es);
            pl->out_nhwc = rg.take(nw * sizeof(float));
        }
        if (pad) pl->xpad = rg.take((size_t)d->n * d->h * d->w * pl->cpad * es);
        const int M = d->n * pl->P * pl->Q, J = d->r * d->s * pl->cpad;
        pl->wgrad_slab = lc_wgrad_slab_ok(d->n, d->h, d->w, pl->cpad, d->k, d->r, d->s, d->stride_h, d->stride_w, d->pad_h, d->pad_w,
                                          pl->P, pl->Q, pl->bf16);
        if (pl->stem_wgrad) {
            pl->splits = lc_conv_stem_blocks(d->n, pl->P, pl->Q);      // one partial per resident block
            pl->m_per_split = 0;
        } else if (pl->wgrad_slab) {
            pl->splits = lc_wgrad_slab_splits(d->n, d->h, d->w, pl->cpad, d->k, &pl->m_per_split);
        } else {
            pl->splits = lc_wgrad_splits(M, d->k, J, pl->bf16);
            pl->m_per_split = (M + pl->splits - 1) / pl->splits;
        }
        pl->wgrad_direct = pl->splits == 1 && !pad && !pl->stem_wgrad;
        if (!pl->wgrad_direct) pl->part = rg.take((size_t)pl->splits * d->k * J * sizeof(float));
    }
    pl->total = rg.off;
    return LC_OK;
}

// a, b: the two operand tensors (of the descriptor's dtype); c: the result
lc_status check_buffers(const Plan& pl, const void* a, const void* b, const void* c, size_t c_align,
                        const void* ws, size_t ws_bytes) {
    if (!a || !b || !c) return LC_ERR_NULL;
    // fp32 tensors need their natural alignment (16 bytes take the vector path); bf16 tensors 16 bytes
    const uintptr_t mask = pl.bf16 ? 15 : 3;
    if (((uintptr_t)a | (uintptr_t)b) & mask) return LC_ERR_ALIGN;
    if ((uintptr_t)c & (c_align - 1)) return LC_ERR_ALIGN;
    if (pl.total) {
        if (!ws || ((uintptr_t)ws & 255) || ws_bytes < pl.total) return LC_ERR_WORKSPACE;
    }
    return LC_OK;
}

inline char* at(void* ws, size_t off) { return static_cast<char*>(ws) + off; }

thread_local char g_detail[256] = "";

}  // namespace

void lc_begin_call() { (void)hipGetLastError(); }

lc_status lc_end_call() {
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return LC_OK;
    snprintf(g_detail, sizeof(g_detail), "%s: %s", hipGetErrorName(e), hipGetErrorString(e));
    return LC_ERR_LAUNCH;
}

lc_status lc_fail_call(hipError_t e, const char* what) {
    snprintf(g_detail, sizeof(g_detail), "%s: %s: %s", what, hipGetErrorName(e), hipGetErrorString(e));
    (void)hipGetLastError();
    return LC_ERR_LAUNCH;
}

extern "C" const char* lc_last_error_detail(void) { return g_detail; }

extern "C" lc_status conv2d_out_shape(const lc_conv_desc* desc, int* p, int* q) {
    if (!desc || !p || !q) return LC_ERR_NULL;
    int P, Q;
    const lc_status st = check_desc(desc, &P, &Q);
    if (st != LC_OK) return st;
    *p = P;
    *q = Q;
    return LC_OK;
}

namespace {

// A grouped layer runs group by group: the group's channel slice of each activation operand is copied to a dense
// tensor in the workspace, the one-group convolution runs on it, and an activation result is copied back into its
// slice.  The filter (and its gradient) of a group is a contiguous run of k/groups filters and is used in place,
// unless a bf16 slice would start off a 16-byte boundary; then it goes through the workspace too.
struct GroupPlan {
    lc_conv_desc inner = {};
    int G = 1, cg = 0, kg = 0, P = 0, Q = 0;
    size_t es = 4;
    size_t x_rows = 0, x_pitch = 0, x_width = 0;      // 2-D view of x (and dx): rows, pitch and slice width in bytes
    size_t y_rows = 0, y_pitch = 0, y_width = 0;      // ... of y (and dy)
    size_t w_bytes = 0;                               // one group's filter in the operand type
    bool w_copy = false;
    size_t xs = 0, ys = 0, wsl = 0, ws = 0, ws_bytes = 0, total = 0;
};

lc_status plan_groups(const lc_conv_desc* d, lc_pass pass, GroupPlan* gp) {
    const lc_status st = check_desc(d, &gp->P, &gp->Q);
    if (st != LC_OK) return st;
    if (pass != LC_PASS_FWD && pass != LC_PASS_BWD_DATA && pass != LC_PASS_BWD_WEIGHT) return LC_ERR_UNSUPPORTED;
    gp->G = d->groups;
    gp->cg = d->c / gp->G;
    gp->kg = d->k / gp->G;
    gp->es = d->dtype == LC_BF16 ? 2 : 4;
    gp->inner = *d;
    gp->inner.c = gp->cg;
    gp->inner.k = gp->kg;
    gp->inner.groups = 1;
    const size_t hw = (size_t)d->h * d->w, pq = (size_t)gp->P * gp->Q;
    if (d->layout == LC_NHWC) {
        gp->x_rows = (size_t)d->n * hw;
        gp->x_pitch = (size_t)d->c * gp->es;
        gp->x_width = (size_t)gp->cg * gp->es;
        gp->y_rows = (size_t)d->n * pq;
        gp->y_pitch = (size_t)d->k * gp->es;
        gp->y_width = (size_t)gp->kg * gp->es;
    } else {
        gp->x_rows = gp->y_rows = (size_t)d->n;
        gp->x_pitch = (size_t)d->c * hw * gp->es;
        gp->x_width = (size_t)gp->cg * hw * gp->es;
        gp->y_pitch = (size_t)d->k * pq * gp->es;
        gp->y_width = (size_t)gp->kg * pq * gp->es;
    }
    gp->w_bytes = (size_t)gp->kg * gp->cg * d->r * d->s * gp->es;
    gp->w_copy = pass != LC_PASS_BWD_WEIGHT && gp->es == 2 && (gp->w_bytes & 15) != 0;
    Regions rg;
    gp->xs = rg.take(gp->x_rows * gp->x_width);
    gp->ys = rg.take(gp->y_rows * gp->y_width);
    if (gp->w_copy) gp->wsl = rg.take(gp->w_bytes);
    gp->ws_bytes = conv2d_workspace_bytes(&gp->inner, pass);
    if (gp->ws_bytes) gp->ws = rg.take(gp->ws_bytes);
    gp->total = rg.off;
    return LC_OK;
}

// a, b: the pass's two operands, c: its result, as in the entry points.
lc_status run_groups(const lc_conv_desc* d, lc_pass pass, const void* a, const void* b, void* c, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
    GroupPlan gp;
    lc_status st = plan_groups(d, pass, &gp);
    if (st != LC_OK) return st;
    if (!a || !b || !c) return LC_ERR_NULL;
    const uintptr_t mask = gp.es == 2 ? 15 : 3;
    if ((((uintptr_t)a | (uintptr_t)b) & mask) || ((uintptr_t)c & (pass == LC_PASS_BWD_WEIGHT ? 3 : mask))) return LC_ERR_ALIGN;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < gp.total) return LC_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char* xs = at(workspace, gp.xs);
    char* ys = at(workspace, gp.ys);
    void* iws = gp.ws_bytes ? at(workspace, gp.ws) : nullptr;
    for (int g = 0; g < gp.G; ++g) {
        const size_t xo = (size_t)g * gp.x_width, yo = (size_t)g * gp.y_width;
        lc_begin_call();
        if (pass == LC_PASS_FWD) {                      // a = x, b = w, c = y
            const char* wg = static_cast<const char*>(b) + (size_t)g * gp.w_bytes;
            lc_copy2d(static_cast<const char*>(a) + xo, gp.x_pitch, xs, gp.x_width, gp.x_width, gp.x_rows, stream);
            if (gp.w_copy) lc_copy2d(wg, gp.w_bytes, at(workspace, gp.wsl), gp.w_bytes, gp.w_bytes, 1, stream);
            if ((st = lc_end_call()) != LC_OK) return st;
            st = conv2d_fwd(&gp.inner, xs, gp.w_copy ? at(workspace, gp.wsl) : wg, ys, iws, gp.ws_bytes, hip_stream);
            if (st != LC_OK) return st;
            lc_begin_call();
            lc_copy2d(ys, gp.y_width, static_cast<char*>(c) + yo, gp.y_pitch, gp.y_width, gp.y_rows, stream);
        } else if (pass == LC_PASS_BWD_DATA) {          // a = dy, b = w, c = dx
            const char* wg = static_cast<const char*>(b) + (size_t)g * gp.w_bytes;
            lc_copy2d(static_cast<const char*>(a) + yo, gp.y_pitch, ys, gp.y_width, gp.y_width, gp.y_rows, stream);
            if (gp.w_copy) lc_copy2d(wg, gp.w_bytes, at(workspace, gp.wsl), gp.w_bytes, gp.w_bytes, 1, stream);
            if ((st = lc_end_call()) != LC_OK) return st;
            st = conv2d_bwd_data(&gp.inner, ys, gp.w_copy ? at(workspace, gp.wsl) : wg, xs, iws, gp.ws_bytes, hip_stream);
            if (st != LC_OK) return st;
            lc_begin_call();
            lc_copy2d(xs, gp.x_width, static_cast<char*>(c) + xo, gp.x_pitch, gp.x_width, gp.x_rows, stream);
        } else {                                        // a = x, b = dy, c = dw (fp32)
            lc_copy2d(static_cast<const char*>(a) + xo, gp.x_pitch, xs, gp.x_width, gp.x_width, gp.x_rows, stream);
            lc_copy2d(static_cast<const char*>(b) + yo, gp.y_pitch, ys, gp.y_width, gp.y_width, gp.y_rows, stream);
            if ((st = lc_end_call()) != LC_OK) return st;
            float* dwg = static_cast<float*>(c) + (size_t)g * gp.kg * gp.cg * d->r * d->s;
            st = conv2d_bwd_weight(&gp.inner, xs, ys, dwg, iws, gp.ws_bytes, hip_stream);
            if (st != LC_OK) return st;
            lc_begin_call();
        }
        if ((st = lc_end_call()) != LC_OK) return st;
    }
    return LC_OK;
}

}  // namespace

extern "C" size_t conv2d_workspace_bytes(const lc_conv_desc* desc, lc_pass pass) {
    if (desc && desc->groups > 1) {
        GroupPlan gp;
        return plan_groups(desc, pass, &gp) == LC_OK ? gp.total : 0;
    }
    lc_conv_desc canon;
    desc = whole_window_as_1x1(desc, &canon);
    Plan pl;
    if (make_plan(desc, pass, &pl) != LC_OK) return 0;
    return pl.total;
}

namespace {

// The forward pass; `stats` (may be null) receives the column sums of the result from the GEMM's epilogue (see
// conv2d_fwd_stats) -- only for plans whose GEMM writes y itself, which fwd_stats_tiles() reports.
lc_status fwd_impl(const lc_conv_desc* d, const void* x, const void* w, void* y, float* stats, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
    lc_conv_desc canon;
    d = whole_window_as_1x1(d, &canon);
    Plan pl;
    lc_status st = make_plan(d, LC_PASS_FWD, &pl);
    if (st != LC_OK) return st;
    st = check_buffers(pl, x, w, y, pl.bf16 ? 16 : 4, workspace, workspace_bytes);
    if (st != LC_OK) return st;
    if (stats && pl.nchw) return LC_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lc_begin_call();

    if (pl.blocks) {
        void* u = at(workspace, pl.s_u);
        void* wu = at(workspace, pl.s_w);
        lc_stem_unfold(x, u, d->n, d->c, d->h, d->w, pl.Q, pl.HB, pl.SB, pl.CU, pl.eph, pl.epw, pl.esize, stream);
        lc_stem_filter(w, wu, d->k, d->r, d->s, d->c, pl.RB, pl.SB, pl.CU, pl.eh, pl.ew, pl.esize, stream);
        st = lc_end_call();
        if (st != LC_OK) return st;
        return fwd_impl(&pl.inner, u, wu, y, stats, pl.s_ws_bytes ? at(workspace, pl.s_ws) : nullptr, pl.s_ws_bytes, hip_stream);
    }

    if (stem_direct(d, pl, LC_PASS_FWD)) {
        if (pl.bf16) {
            const StemConvBf16 sb = {static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w), static_cast<uint16_t*>(y), stats,
                                     d->n, d->h, d->w, pl.P, pl.Q};
            return lc_launch_conv_stem_bf16(sb, stream);
        }
        const StemConv sc = {static_cast<const float*>(x), static_cast<const float*>(w), static_cast<float*>(y), stats,
                             d->n, d->h, d->w, pl.P, pl.Q};
        return lc_launch_conv_stem_f32(sc, stream);
    }

    const void* xs = x;
    const void* wsrc = w;
    void* ydst = y;
    if (pl.nchw) {
        lc_nchw_to_nhwc(x, at(workspace, pl.a_nhwc), d->n, d->c, d->h * d->w, pl.esize, stream);
        lc_nchw_to_nhwc(w, at(workspace, pl.b_nhwc), d->k, d->c, d->r * d->s, pl.esize, stream);
        xs = at(workspace, pl.a_nhwc);
        wsrc = at(workspace, pl.b_nhwc);
        ydst = at(workspace, pl.out_nhwc);
    }
    if (pl.cpad != d->c) {
        lc_pad_channels(xs, at(workspace, pl.xpad), (size_t)d->n * d->h * d->w, d->c, pl.cpad, pl.esize, stream);
        lc_pad_channels(wsrc, at(workspace, pl.wpad), (size_t)d->k * d->r * d->s, d->c, pl.cpad, pl.esize, stream);
        xs = at(workspace, pl.xpad);
        wsrc = at(workspace, pl.wpad);
    }
    GemmConv g = gemm_fwd(d, pl.P, pl.Q, pl.cpad);
    g.a = xs;
    g.b = wsrc;
    g.d = ydst;
    g.partial = pl.sk_bytes ? reinterpret_cast<float*>(at(workspace, pl.sk)) : nullptr;
    g.stats = stats;
    st = lc_launch_conv_gemm(g, stream);
    if (st != LC_OK) return st;
    if (pl.nchw) lc_nhwc_to_nchw(ydst, y, d->n, d->k, pl.P * pl.Q, pl.esize, stream);
    return lc_end_call();
}

// Row pieces of the statistics conv2d_fwd_stats hands over for this layer; 0 when its plan has no such epilogue
// (NCHW, groups, operands the main kernel does not take).  Needs the operand pointers' alignment only through
// the plan, which assumes what check_buffers() enforces.
size_t fwd_stats_tiles(const lc_conv_desc* d) {
    lc_conv_desc canon;
    int P, Q;
    if (check_desc(d, &P, &Q) != LC_OK || d->groups > 1) return 0;
    d = whole_window_as_1x1(d, &canon);
    Plan pl;
    if (make_plan(d, LC_PASS_FWD, &pl) != LC_OK || pl.nchw) return 0;
    if (pl.blocks) return fwd_stats_tiles(&pl.inner);
    if (stem_direct(d, pl, LC_PASS_FWD)) return lc_conv_stem_f32_stats_pieces(d->n, pl.P, pl.Q);
    GemmConv g = gemm_fwd(d, pl.P, pl.Q, pl.cpad);
    return lc_conv_gemm_stats_tiles(g);
}

}  // namespace

extern "C" lc_status conv2d_fwd(const lc_conv_desc* d, const void* x, const void* w, void* y,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (d && d->groups > 1) return run_groups(d, LC_PASS_FWD, x, w, y, workspace, workspace_bytes, hip_stream);
    return fwd_impl(d, x, w, y, nullptr, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t conv2d_fwd_stats_count(const lc_conv_desc* d) { return d ? fwd_stats_tiles(d) : 0; }

extern "C" lc_status conv2d_fwd_stats(const lc_conv_desc* d, const void* x, const void* w, void* y, float* stats, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
    if (!d) return LC_ERR_NULL;
    int P, Q;
    const lc_status st = check_desc(d, &P, &Q);
    if (st != LC_OK) return st;
    if (fwd_stats_tiles(d) == 0) return LC_ERR_UNSUPPORTED;
    if (!stats) return LC_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(stats) & 7) return LC_ERR_ALIGN;
    return fwd_impl(d, x, w, y, stats, workspace, workspace_bytes, hip_stream);
}

extern "C" lc_status conv2d_bwd_data(const lc_conv_desc* d, const void* dy, const void* w, void* dx,
                                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (d && d->groups > 1) return run_groups(d, LC_PASS_BWD_DATA, dy, w, dx, workspace, workspace_bytes, hip_stream);
    lc_conv_desc canon;
    d = whole_window_as_1x1(d, &canon);
    Plan pl;
    lc_status st = make_plan(d, LC_PASS_BWD_DATA, &pl);
    if (st != LC_OK) return st;
    st = check_buffers(pl, dy, w, dx, pl.bf16 ? 16 : 4, workspace, workspace_bytes);
    if (st != LC_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lc_begin_call();

    if (pl.via_f32) {
        const size_t nx = (size_t)d->n * d->h * d->w * d->c, ny = (size_t)d->n * pl.P * pl.Q * d->k;
        const size_t nw = (size_t)d->k * d->r * d->s * d->c;
        float* fdy = reinterpret_cast<float*>(at(workspace, pl.f_a));
        float* fw = reinterpret_cast<float*>(at(workspace, pl.f_b));
        float* fdx = reinterpret_cast<float*>(at(workspace, pl.f_out));
        lc_bf16_to_f32(dy, fdy, ny, stream);
        lc_bf16_to_f32(w, fw, nw, stream);
        const lc_conv_desc f = as_f32(d);
        st = conv2d_bwd_data(&f, fdy, fw, fdx, pl.f_ws_bytes ? at(workspace, pl.f_ws) : nullptr, pl.f_ws_bytes, hip_stream);
        if (st != LC_OK) return st;
        lc_f32_to_bf16(fdx, dx, nx, stream);
        return lc_end_call();
    }

    const void* dys = dy;
    const void* wsrc = w;
    void* dxdst = dx;
    if (pl.nchw) {
        lc_nchw_to_nhwc(dy, at(workspace, pl.a_nhwc), d->n, d->k, pl.P * pl.Q, pl.esize, stream);
        lc_nchw_to_nhwc(w, at(workspace, pl.b_nhwc), d->k, d->c, d->r * d->s, pl.esize, stream);
        dys = at(workspace, pl.a_nhwc);
        wsrc = at(workspace, pl.b_nhwc);
        dxdst = at(workspace, pl.out_nhwc);
    }
    void* wt = at(workspace, pl.wt);
    if (pl.phases) {
        Phase ph[kMaxPhases];
        bool covered;
        const int n = plan_phases(d, pl.P, pl.Q, ph, &covered);
        if (!covered) lc_zero_bytes(dxdst, (size_t)d->n * d->h * d->w * d->c * pl.esize, stream);
        for (int i = 0; i < n; ++i) {
            void* wp = static_cast<char*>(wt) + ph[i].w_off * pl.esize;
            lc_filter_for_bwd_data_phase(wsrc, wp, d->k, d->c, d->r, d->s, ph[i].a, ph[i].b, d->stride_h, d->stride_w, ph[i].Ra,
                                         ph[i].Sb, pl.esize, stream);
            GemmConv g = ph[i].g;
            g.a = dys;
            g.b = wp;
            g.d = static_cast<char*>(dxdst) + ph[i].d_off * pl.esize;
            g.partial = pl.sk_bytes ? reinterpret_cast<float*>(at(workspace, pl.sk)) : nullptr;
            st = lc_launch_conv_gemm(g, stream);
            if (st != LC_OK) return st;
        }
        if (pl.nchw) lc_nhwc_to_nchw(dxdst, dx, d->n, d->c, d->h * d->w, pl.esize, stream);
        return lc_end_call();
    }
    // filter of the backward convolution: [c][R-1-r][S-1-s][k]
    lc_filter_for_bwd_data(wsrc, wt, d->k, d->c, d->r, d->s, pl.esize, stream);

    GemmConv g = gemm_bwd_data(d, pl.P, pl.Q);
    g.a = dys;
    g.b = wt;
    g.d = dxdst;
    // a strided 1x1 window touches only the stride grid of dx: clear it first, the kernels write the grid
    if (g.scatter) lc_zero_bytes(dxdst, (size_t)d->n * d->h * d->w * d->c * pl.esize, stream);
    g.partial = pl.sk_bytes ? reinterpret_cast<float*>(at(workspace, pl.sk)) : nullptr;
    st = lc_launch_conv_gemm(g, stream);
    if (st != LC_OK) return st;
    if (pl.nchw) lc_nhwc_to_nchw(dxdst, dx, d->n, d->c, d->h * d->w, pl.esize, stream);
    return lc_end_call();
}

namespace {

// Whether the pass ends in the split reduction writing dw itself (the only place the squared norm comes for free).
bool wgrad_sq_fused(const lc_conv_desc* d, const Plan& pl) { return d->groups <= 1 && !pl.blocks && !pl.nchw && !pl.wgrad_direct; }

// conv2d_bwd_weight; sq (may be null) receives the pieces of dw's squared norm.
lc_status bwd_weight_impl(const lc_conv_desc* d, const void* x, const void* dy, float* dw, double* sq, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    if (d && d->groups > 1) {
        const lc_status gs = run_groups(d, LC_PASS_BWD_WEIGHT, x, dy, dw, workspace, workspace_bytes, hip_stream);
        if (gs != LC_OK || !sq) return gs;
        lc_begin_call();
        lc_sq_partials(dw, (size_t)d->k * (d->c / d->groups) * d->r * d->s, sq, static_cast<hipStream_t>(hip_stream));
        return lc_end_call();
    }
    const size_t dw_numel = d ? (size_t)d->k * d->c * d->r * d->s : 0;      // (before the descriptor is canonicalised)
    lc_conv_desc canon;
    d = whole_window_as_1x1(d, &canon);
    Plan pl;
    lc_status st = make_plan(d, LC_PASS_BWD_WEIGHT, &pl);
    if (st != LC_OK) return st;
    st = check_buffers(pl, x, dy, dw, 4, workspace, workspace_bytes);
    if (st != LC_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lc_begin_call();

    if (pl.blocks) {
        void* u = at(workspace, pl.s_u);
        float* dwu = reinterpret_cast<float*>(at(workspace, pl.s_w));
        lc_stem_unfold(x, u, d->n, d->c, d->h, d->w, pl.Q, pl.HB, pl.SB, pl.CU, pl.eph, pl.epw, pl.esize, stream);
        st = lc_end_call();
        if (st != LC_OK) return st;
        st = bwd_weight_impl(&pl.inner, u, dy, dwu, nullptr, pl.s_ws_bytes ? at(workspace, pl.s_ws) : nullptr, pl.s_ws_bytes, hip_stream);
        if (st != LC_OK) return st;
        lc_stem_filter_grad(dwu, dw, d->k, d->r, d->s, d->c, pl.RB, pl.CU, pl.eh, pl.ew, stream);
        if (sq) lc_sq_partials(dw, dw_numel, sq, stream);
        return lc_end_call();
    }

    if (pl.stem_wgrad) {
        float* part = reinterpret_cast<float*>(at(workspace, pl.part));
        if (pl.bf16) {
            const StemWgradBf16 sb = {static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(dy), part, d->n, d->h, d->w, pl.P, pl.Q};
            st = lc_launch_conv_stem_wgrad_bf16(sb, pl.splits, stream);
        } else {
            const StemWgrad sw = {static_cast<const float*>(x), static_cast<const float*>(dy), part, d->n, d->h, d->w, pl.P, pl.Q};
            st = lc_launch_conv_stem_wgrad_f32(sw, pl.splits, stream);
        }
        if (st != LC_OK) return st;
        const bool fused_sq = sq && wgrad_sq_fused(d, pl);
        lc_reduce_splits(part, dw, pl.splits, (size_t)d->k * d->r * d->s * d->c, d->c, d->c, fused_sq ? sq : nullptr, stream);
        if (sq && !fused_sq) lc_sq_partials(dw, dw_numel, sq, stream);
        return lc_end_call();
    }

    const void* xs = x;
    const void* dys = dy;
    float* dwdst = dw;
    if (pl.nchw) {
        lc_nchw_to_nhwc(x, at(workspace, pl.a_nhwc), d->n, d->c, d->h * d->w, pl.esize, stream);
        lc_nchw_to_nhwc(dy, at(workspace, pl.b_nhwc), d->n, d->k, pl.P * pl.Q, pl.esize, stream);
        xs = at(workspace, pl.a_nhwc);
        dys = at(workspace, pl.b_nhwc);
        dwdst = reinterpret_cast<float*>(at(workspace, pl.out_nhwc));
    }
    if (pl.cpad != d->c) {
        lc_pad_channels(xs, at(workspace, pl.xpad), (size_t)d->n * d->h * d->w, d->c, pl.cpad, pl.esize, stream);
        xs = at(workspace, pl.xpad);
    }
    GemmWgrad g = {};
    g.dy = dys;
    g.x = xs;
    g.M = d->n * pl.P * pl.Q;
    g.K = d->k;
    g.J = d->r * d->s * pl.cpad;
    g.H = d->h;
    g.W = d->w;
    g.C = pl.cpad;
    g.P = pl.P;
    g.Q = pl.Q;
    g.R = d->r;
    g.S = d->s;
    g.sh = d->stride_h;
    g.sw = d->stride_w;
    g.ph = d->pad_h;
    g.pw = d->pad_w;
    g.splits = pl.splits;
    g.m_per_split = pl.m_per_split;
    g.bf16 = pl.bf16;
    g.slab = pl.wgrad_slab;
    g.d = pl.wgrad_direct ? dwdst : reinterpret_cast<float*>(at(workspace, pl.part));
    st = lc_launch_wgrad_f32(g, stream);
    if (st != LC_OK) return st;
    const bool fused = sq && wgrad_sq_fused(d, pl);
    if (!pl.wgrad_direct)
        lc_reduce_splits(g.d, dwdst, pl.splits, (size_t)d->k * g.J, pl.cpad, d->c, fused ? sq : nullptr, stream);
    if (pl.nchw) lc_nhwc_to_nchw(dwdst, dw, d->k, d->c, d->r * d->s, 4, stream);
    if (sq && !fused) lc_sq_partials(dw, dw_numel, sq, stream);
    return lc_end_call();
}

}  // namespace

extern "C" lc_status conv2d_bwd_weight(const lc_conv_desc* d, const void* x, const void* dy, float* dw,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    return bwd_weight_impl(d, x, dy, dw, nullptr, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t conv2d_bwd_weight_sq_count(const lc_conv_desc* d) {
    if (!d) return 0;
    int P, Q;
    if (check_desc(d, &P, &Q) != LC_OK) return 0;
    const size_t numel = (size_t)d->k * (d->groups > 1 ? d->c / d->groups : d->c) * d->r * d->s;
    if (d->groups > 1) return lc_sq_partials_blocks(numel);
    lc_conv_desc canon;
    const lc_conv_desc* dc = whole_window_as_1x1(d, &canon);
    Plan pl;
    if (make_plan(dc, LC_PASS_BWD_WEIGHT, &pl) != LC_OK) return 0;
    if (wgrad_sq_fused(dc, pl)) return lc_reduce_splits_blocks((size_t)dc->k * dc->r * dc->s * pl.cpad);
    return lc_sq_partials_blocks(numel);
}

extern "C" lc_status conv2d_bwd_weight_sq(const lc_conv_desc* d, const void* x, const void* dy, float* dw, double* dw_sq_pieces,
                                          void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!dw_sq_pieces) return LC_ERR_NULL;
    if ((uintptr_t)dw_sq_pieces & 7) return LC_ERR_ALIGN;
    return bwd_weight_impl(d, x, dy, dw, dw_sq_pieces, workspace, workspace_bytes, hip_stream);
}


extern "C" const char* lc_status_string(lc_status status) {
    switch (status) {
        case LC_OK: return "ok";
        case LC_ERR_NULL: return "null pointer";
        case LC_ERR_SHAPE: return "invalid shape";
        case LC_ERR_UNSUPPORTED: return "unsupported configuration";
        case LC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LC_ERR_LAUNCH: return "HIP launch error";
        case LC_ERR_ALIGN: return "misaligned tensor pointer";
    }
    return "unknown status";
}
