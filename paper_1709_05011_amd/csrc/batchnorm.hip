// Batch normalisation in training mode (batch statistics, biased variance, no running averages) -- the layer
// the paper adds after each convolution of AlexNet ("Scaling up Batch Size") and that ResNet-50 has throughout.
// Memory-bound: every pass is "reduce per channel, then stream".
//
//   forward:   stats kernel (sum, sum of squares per channel, partial per block)  -> finalize (mean, 1/std,
//              scale = gamma/std, shift = beta - mean*scale)                       -> y = x*scale + shift
//   backward:  sums kernel (sum dy, sum dy*xhat per channel, partial per block)    -> finalize (dgamma, dbeta,
//              a, b, c with dx = a*dy + b*x + c)                                   -> dx
//
// Algorithmic bytes per element: forward 12 (x twice, y once), backward 20 (x and dy twice, dx once).
// The forward sums are those of x - pivot and (x - pivot)^2 with the channel's first value as pivot, so that the
// variance E[d^2] - E[d]^2 does not cancel when the mean is large against the spread (a constant channel gives 0).
// Threads accumulate in fp32 over a few hundred values each, in a fixed order; blocks and the partials of all
// blocks are combined in fp64 in index order: results are bit-identical from run to run.
// Fused variants (the *_ex entry points): the forward pass can add a second tensor (a residual shortcut) and
// clamp at zero; the backward pass can take the gradient of the clamped output and rebuild the mask y > 0 from x
// -- forward and backward derive y's scale and shift from the stored float statistics with the same code, so the
// rebuilt y has the forward's bits.
// NHWC: the tensor is a matrix [pixels][channels]; a block owns a slab of pixels, a thread a group of four
// channels (16-byte accesses).  NCHW: a block owns one channel and a range of images and runs along the
// contiguous pixels of each plane.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/larsconv.h"
#include "internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxSlabs = 1024;       // blocks along the pixels (NHWC) or the images (NCHW)

struct BnGeom {
    int N, C, HW;
    long long M;          // N * HW
    int tx, ty;           // NHWC: threads along channel quads / along rows
    int cblocks;          // NHWC: blocks along the channels
    int slabs;            // blocks along pixels (NHWC) or images (NCHW)
    long long rows_per_slab;
    int vec;              // NHWC: 4 = float4 path (C % 4 == 0 and aligned), 1 = scalar
};

struct BnWorkspace {
    double* partial;      // [slabs][C][2]
    float* coef;          // [5][C]: p, q, r of out = p*A + q*B + r, then scale and shift of y = scale*x + shift
};

enum { kStats = 0, kSums = 1, kMaskedSums = 2 };

// y = scale*x + shift from the stored statistics; both passes call this and get the same bits
__device__ __forceinline__ void scale_shift(float gamma, float beta, float mean, float inv_std, float* scale, float* shift) {
    const double sc = (double)gamma * (double)inv_std;
    *scale = (float)sc;
    *shift = (float)fma(-(double)mean, sc, (double)beta);
}

// ---------------- NHWC ----------------
// MODE kStats: sums of x and x^2.  kSums: sums of dy and dy * (x - mean) * inv_std.  kMaskedSums: the same with
// dy taken as zero where scale*x + shift <= 0.
template <int VEC, int MODE>
__global__ void __launch_bounds__(kThreads) bn_reduce_nhwc_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                                  const float* __restrict__ mean, const float* __restrict__ inv_std,
                                                                  const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                  BnGeom g, BnWorkspace ws) {
    constexpr bool STATS = MODE == kStats;
    __shared__ double red[kThreads][2 * VEC];
    const int tx = threadIdx.x % g.tx, ty = threadIdx.x / g.tx;
    const int c0 = (blockIdx.y * g.tx + tx) * VEC;
    const bool live = c0 < g.C;
    const long long r0 = (long long)blockIdx.x * g.rows_per_slab;
    const long long r1 = r0 + g.rows_per_slab < g.M ? r0 + g.rows_per_slab : g.M;
    float s0[VEC], s1[VEC], mu[VEC], is[VEC], sc[VEC], sh[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        s0[e] = s1[e] = 0.f;
        mu[e] = (!STATS && live) ? mean[c0 + e] : 0.f;
        is[e] = (!STATS && live) ? inv_std[c0 + e] : 0.f;
        sc[e] = sh[e] = 0.f;
        if (MODE == kMaskedSums && live) scale_shift(gamma[c0 + e], beta[c0 + e], mu[e], is[e], &sc[e], &sh[e]);
        if (STATS && live) mu[e] = x[c0 + e];          // the channel's pivot: its value at the first pixel
    }
    if (live) {
        for (long long r = r0 + ty; r < r1; r += g.ty) {
            float a[VEC], b[VEC];
            if constexpr (VEC == 4) {
                const float4 va = *reinterpret_cast<const float4*>(x + r * g.C + c0);
                a[0] = va.x; a[1] = va.y; a[2] = va.z; a[3] = va.w;
                if constexpr (!STATS) {
                    const float4 vb = *reinterpret_cast<const float4*>(dy + r * g.C + c0);
                    b[0] = vb.x; b[1] = vb.y; b[2] = vb.z; b[3] = vb.w;
                }
            } else {
                a[0] = x[r * g.C + c0];
                if constexpr (!STATS) b[0] = dy[r * g.C + c0];
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                if constexpr (STATS) {
                    const float d = a[e] - mu[e];
                    s0[e] += d;
                    s1[e] += d * d;
                } else {
                    const float d = (MODE == kMaskedSums && !(fmaf(sc[e], a[e], sh[e]) > 0.f)) ? 0.f : b[e];
                    s0[e] += d;
                    s1[e] += d * ((a[e] - mu[e]) * is[e]);
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        red[threadIdx.x][2 * e] = (double)s0[e];
        red[threadIdx.x][2 * e + 1] = (double)s1[e];
    }
    __syncthreads();
    if (ty == 0 && live) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            double t0 = 0.0, t1 = 0.0;
            for (int k = 0; k < g.ty; ++k) {              // rows of the block in order
                t0 += red[k * g.tx + tx][2 * e];
                t1 += red[k * g.tx + tx][2 * e + 1];
            }
            double* out = ws.partial + ((size_t)blockIdx.x * g.C + c0 + e) * 2;
            out[0] = t0;
            out[1] = t1;
        }
    }
}

// out = p*A + q*B + r per channel (TWO false: out = p*A + r).  RELU: clamp the result at zero.  MASK: B counts as
// zero where scale*A + shift <= 0.
template <int VEC, bool TWO, bool RELU, bool MASK>
__global__ void __launch_bounds__(kThreads) bn_apply_nhwc_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                                 float* __restrict__ out, const float* __restrict__ coef, BnGeom g) {
    const size_t total = (size_t)g.M * g.C / VEC;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int c0 = (int)((i * VEC) % g.C);
        if constexpr (VEC == 4) {
            const float4 va = reinterpret_cast<const float4*>(a)[i];
            const float4 p = *reinterpret_cast<const float4*>(coef + c0);
            const float4 r = *reinterpret_cast<const float4*>(coef + 2 * g.C + c0);
            float4 o = make_float4(fmaf(p.x, va.x, r.x), fmaf(p.y, va.y, r.y), fmaf(p.z, va.z, r.z), fmaf(p.w, va.w, r.w));
            if constexpr (TWO) {
                float4 vb = reinterpret_cast<const float4*>(b)[i];
                const float4 q = *reinterpret_cast<const float4*>(coef + g.C + c0);
                if constexpr (MASK) {
                    const float4 sc = *reinterpret_cast<const float4*>(coef + 3 * g.C + c0);
                    const float4 sh = *reinterpret_cast<const float4*>(coef + 4 * g.C + c0);
                    if (!(fmaf(sc.x, va.x, sh.x) > 0.f)) vb.x = 0.f;
                    if (!(fmaf(sc.y, va.y, sh.y) > 0.f)) vb.y = 0.f;
                    if (!(fmaf(sc.z, va.z, sh.z) > 0.f)) vb.z = 0.f;
                    if (!(fmaf(sc.w, va.w, sh.w) > 0.f)) vb.w = 0.f;
                }
                o.x = fmaf(q.x, vb.x, o.x); o.y = fmaf(q.y, vb.y, o.y); o.z = fmaf(q.z, vb.z, o.z); o.w = fmaf(q.w, vb.w, o.w);
            }
            if constexpr (RELU) { o.x = fmaxf(o.x, 0.f); o.y = fmaxf(o.y, 0.f); o.z = fmaxf(o.z, 0.f); o.w = fmaxf(o.w, 0.f); }
            reinterpret_cast<float4*>(out)[i] = o;
        } else {
            float o = fmaf(coef[c0], a[i], coef[2 * g.C + c0]);
            if constexpr (TWO) {
                float vb = b[i];
                if constexpr (MASK) if (!(fmaf(coef[3 * g.C + c0], a[i], coef[4 * g.C + c0]) > 0.f)) vb = 0.f;
                o = fmaf(coef[g.C + c0], vb, o);
            }
            if constexpr (RELU) o = fmaxf(o, 0.f);
            out[i] = o;
        }
    }
}

// ---------------- NCHW ----------------
template <int MODE>
__global__ void __launch_bounds__(kThreads) bn_reduce_nchw_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                                  const float* __restrict__ mean, const float* __restrict__ inv_std,
                                                                  const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                  BnGeom g, BnWorkspace ws) {
    constexpr bool STATS = MODE == kStats;
    __shared__ double red[kThreads][2];
    const int ch = blockIdx.y;
    const long long n0 = (long long)blockIdx.x * g.rows_per_slab;
    const long long n1 = n0 + g.rows_per_slab < g.N ? n0 + g.rows_per_slab : g.N;
    const float mu = STATS ? x[(size_t)ch * g.HW] : mean[ch], is = STATS ? 0.f : inv_std[ch];   // STATS: the pivot
    float sc = 0.f, sh = 0.f;
    if (MODE == kMaskedSums) scale_shift(gamma[ch], beta[ch], mu, is, &sc, &sh);
    float s0 = 0.f, s1 = 0.f;
    for (long long n = n0; n < n1; ++n) {
        const size_t base = ((size_t)n * g.C + ch) * g.HW;
        for (int i = threadIdx.x; i < g.HW; i += kThreads) {
            const float a = x[base + i];
            if constexpr (STATS) {
                const float d = a - mu;
                s0 += d;
                s1 += d * d;
            } else {
                const float b = (MODE == kMaskedSums && !(fmaf(sc, a, sh) > 0.f)) ? 0.f : dy[base + i];
                s0 += b;
                s1 += b * ((a - mu) * is);
            }
        }
    }
    red[threadIdx.x][0] = (double)s0;
    red[threadIdx.x][1] = (double)s1;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t0 = 0.0, t1 = 0.0;
        for (int k = 0; k < kThreads; ++k) {
            t0 += red[k][0];
            t1 += red[k][1];
        }
        double* out = ws.partial + ((size_t)blockIdx.x * g.C + ch) * 2;
        out[0] = t0;
        out[1] = t1;
    }
}

template <bool TWO, bool RELU, bool MASK>
__global__ void __launch_bounds__(kThreads) bn_apply_nchw_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                                 float* __restrict__ out, const float* __restrict__ coef, BnGeom g) {
    const size_t total = (size_t)g.M * g.C;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int ch = (int)((i / g.HW) % g.C);
        float o = fmaf(coef[ch], a[i], coef[2 * g.C + ch]);
        if constexpr (TWO) {
            float vb = b[i];
            if constexpr (MASK) if (!(fmaf(coef[3 * g.C + ch], a[i], coef[4 * g.C + ch]) > 0.f)) vb = 0.f;
            o = fmaf(coef[g.C + ch], vb, o);
        }
        if constexpr (RELU) o = fmaxf(o, 0.f);
        out[i] = o;
    }
}

// ---------------- per-channel finalize ----------------
// A block of 256 threads finishes 16 channels: 16 lanes per channel add every 16th slab's partial, then the first
// lane adds the 16 lane sums in lane order.  Returns true in the thread that holds the channel's totals.
constexpr int kFinChannels = 16, kFinLanes = 16;
__device__ __forceinline__ bool channel_totals(const BnWorkspace& ws, const BnGeom& g, int* ch_out, double* t0, double* t1) {
    __shared__ double red[kFinLanes][kFinChannels][2];
    const int cl = threadIdx.x % kFinChannels, sl = threadIdx.x / kFinChannels;
    const int ch = blockIdx.x * kFinChannels + cl;
    double s0 = 0.0, s1 = 0.0;
    if (ch < g.C)
        for (int k = sl; k < g.slabs; k += kFinLanes) {
            s0 += ws.partial[((size_t)k * g.C + ch) * 2];
            s1 += ws.partial[((size_t)k * g.C + ch) * 2 + 1];
        }
    red[sl][cl][0] = s0;
    red[sl][cl][1] = s1;
    __syncthreads();
    if (sl != 0 || ch >= g.C) return false;
    s0 = s1 = 0.0;
    for (int k = 0; k < kFinLanes; ++k) {
        s0 += red[k][cl][0];
        s1 += red[k][cl][1];
    }
    *ch_out = ch;
    *t0 = s0;
    *t1 = s1;
    return true;
}

// forward: mean, 1/std, and y = scale*x + shift (+ residual)
__global__ void __launch_bounds__(kFinChannels* kFinLanes)
bn_finalize_fwd_kernel(BnWorkspace ws, const float* __restrict__ x, size_t pivot_stride, const float* __restrict__ gamma,
                       const float* __restrict__ beta, float* __restrict__ save_mean, float* __restrict__ save_invstd, BnGeom g, float eps) {
    int ch;
    double s0, s1;
    if (!channel_totals(ws, g, &ch, &s0, &s1)) return;
    const double m = (double)g.M;
    const double off = s0 / m;                                  // mean of x - pivot
    const double mean = (double)x[ch * pivot_stride] + off;
    double var = s1 / m - off * off;
    if (var < 0.0) var = 0.0;
    const double inv_std = 1.0 / sqrt(var + (double)eps);
    const float mean_f = (float)mean, inv_std_f = (float)inv_std;
    save_mean[ch] = mean_f;
    save_invstd[ch] = inv_std_f;
    float scale, shift;
    scale_shift(gamma[ch], beta[ch], mean_f, inv_std_f, &scale, &shift);
    ws.coef[ch] = scale;
    ws.coef[g.C + ch] = 1.f;               // the residual, when there is one, is added as it is
    ws.coef[2 * g.C + ch] = shift;
}

// backward: dgamma, dbeta, and dx = a*x + b*dy + c  (coefficient order matches the apply kernels: first tensor x)
__global__ void __launch_bounds__(kFinChannels* kFinLanes)
bn_finalize_bwd_kernel(BnWorkspace ws, const float* __restrict__ gamma, const float* __restrict__ beta, const float* __restrict__ mean,
                       const float* __restrict__ inv_std, float* __restrict__ dgamma, float* __restrict__ dbeta, BnGeom g) {
    int ch;
    double s0, s1;
    if (!channel_totals(ws, g, &ch, &s0, &s1)) return;
    dbeta[ch] = (float)s0;
    dgamma[ch] = (float)s1;
    const double m = (double)g.M, is = (double)inv_std[ch], mu = (double)mean[ch];
    const double a = (double)gamma[ch] * is;                 // coefficient of dy
    const double bx = -a * is * s1 / m;                      // coefficient of x
    ws.coef[ch] = (float)bx;
    ws.coef[g.C + ch] = (float)a;
    ws.coef[2 * g.C + ch] = (float)(-a * s0 / m - bx * mu);
    if (beta) {                            // the apply pass rebuilds the mask y > 0
        float scale, shift;
        scale_shift(gamma[ch], beta[ch], mean[ch], inv_std[ch], &scale, &shift);
        ws.coef[3 * g.C + ch] = scale;
        ws.coef[4 * g.C + ch] = shift;
    }
}

bool geometry(int n, int c, int h, int w, lc_layout layout, bool aligned16, BnGeom* g) {
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return false;
    const long long hw = (long long)h * w;
    if (hw > 0x7fffffffLL) return false;
    g->N = n;
    g->C = c;
    g->HW = (int)hw;
    g->M = (long long)n * hw;
    if (layout == LC_NHWC) {
        g->vec = (c % 4 == 0 && aligned16) ? 4 : 1;
        const int groups = c / g->vec;
        int tx = 1;
        while (tx < groups && tx < 64) tx <<= 1;
        g->tx = tx;
        g->ty = kThreads / tx;
        g->cblocks = (groups + tx - 1) / tx;
        long long slabs = (g->M + g->ty * 8 - 1) / (g->ty * 8);          // at least 8 rows per thread
        if (slabs > kMaxSlabs) slabs = kMaxSlabs;
        if (slabs < 1) slabs = 1;
        g->rows_per_slab = (g->M + slabs - 1) / slabs;
        g->slabs = (int)((g->M + g->rows_per_slab - 1) / g->rows_per_slab);
    } else {
        g->vec = 1;
        g->tx = g->ty = g->cblocks = 0;
        long long slabs = n < 64 ? n : 64;
        g->rows_per_slab = (n + slabs - 1) / slabs;
        g->slabs = (int)((n + g->rows_per_slab - 1) / g->rows_per_slab);
    }
    return true;
}

size_t ws_layout(const BnGeom& g, size_t* coef_off) {
    size_t off = (size_t)g.slabs * g.C * 2 * sizeof(double);
    off = (off + 255) & ~(size_t)255;
    *coef_off = off;
    off += (size_t)5 * g.C * sizeof(float);
    return (off + 255) & ~(size_t)255;
}

inline unsigned stream_blocks(size_t items) {
    size_t b = (items + kThreads - 1) / kThreads;
    if (b > 256u * 64u) b = 256u * 64u;
    return (unsigned)(b ? b : 1);
}

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool al4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; }

}  // namespace

extern "C" size_t batchnorm_workspace_bytes(int n, int c, int h, int w, lc_layout layout) {
    BnGeom g;
    if ((layout != LC_NCHW && layout != LC_NHWC) || !geometry(n, c, h, w, layout, true, &g)) return 0;
    // the scalar path (unaligned tensors) uses more thread columns and never more slabs: size for the larger of the two
    BnGeom g1;
    geometry(n, c, h, w, layout, false, &g1);
    size_t o;
    const size_t a = ws_layout(g, &o), b = ws_layout(g1, &o);
    return a > b ? a : b;
}

extern "C" lc_status batchnorm_fwd_ex(const float* x, const float* gamma, const float* beta, const float* residual, float* y,
                                      float* save_mean, float* save_invstd, int n, int c, int h, int w, float eps, int relu,
                                      lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!x || !gamma || !beta || !y || !save_mean || !save_invstd) return LC_ERR_NULL;
    if (layout != LC_NCHW && layout != LC_NHWC) return LC_ERR_UNSUPPORTED;
    if (!(eps >= 0.f)) return LC_ERR_SHAPE;
    BnGeom g;
    if (!geometry(n, c, h, w, layout, al16(x) && al16(y) && al16(residual), &g)) return LC_ERR_SHAPE;
    if (!al4(x) || !al4(y) || !al4(residual) || !al4(gamma) || !al4(beta) || !al4(save_mean) || !al4(save_invstd)) return LC_ERR_ALIGN;
    size_t coef_off;
    const size_t need = ws_layout(g, &coef_off);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < need) return LC_ERR_WORKSPACE;
    BnWorkspace ws;
    ws.partial = static_cast<double*>(workspace);
    ws.coef = reinterpret_cast<float*>(static_cast<char*>(workspace) + coef_off);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lc_begin_call();
    const size_t total = (size_t)g.M * g.C;
    const dim3 fin_grid((c + kFinChannels - 1) / kFinChannels), fin_block(kFinChannels * kFinLanes);
    const float* none = nullptr;
    const bool two = residual != nullptr, clamp = relu != 0;
    const size_t pivot_stride = layout == LC_NHWC ? 1 : (size_t)g.HW;       // the first pixel's value of channel ch sits at x[ch * stride]
    if (layout == LC_NHWC) {
        const dim3 grid((unsigned)g.slabs, (unsigned)g.cblocks);
        if (g.vec == 4)
            hipLaunchKernelGGL((bn_reduce_nhwc_kernel<4, kStats>), grid, dim3(kThreads), 0, stream, x, none, none, none, none, none, g, ws);
        else
            hipLaunchKernelGGL((bn_reduce_nhwc_kernel<1, kStats>), grid, dim3(kThreads), 0, stream, x, none, none, none, none, none, g, ws);
        hipLaunchKernelGGL(bn_finalize_fwd_kernel, fin_grid, fin_block, 0, stream, ws, x, pivot_stride, gamma, beta, save_mean, save_invstd, g, eps);
        const dim3 agrid(stream_blocks(total / g.vec));
#define LC_BN_APPLY(VEC, TWO, RELU) \
    hipLaunchKernelGGL((bn_apply_nhwc_kernel<VEC, TWO, RELU, false>), agrid, dim3(kThreads), 0, stream, x, residual, y, ws.coef, g)
        if (g.vec == 4) {
            if (two) { if (clamp) LC_BN_APPLY(4, true, true); else LC_BN_APPLY(4, true, false); }
            else { if (clamp) LC_BN_APPLY(4, false, true); else LC_BN_APPLY(4, false, false); }
        } else {
            if (two) { if (clamp) LC_BN_APPLY(1, true, true); else LC_BN_APPLY(1, true, false); }
            else { if (clamp) LC_BN_APPLY(1, false, true); else LC_BN_APPLY(1, false, false); }
        }
#undef LC_BN_APPLY
    } else {
        hipLaunchKernelGGL((bn_reduce_nchw_kernel<kStats>), dim3((unsigned)g.slabs, (unsigned)c), dim3(kThreads), 0, stream, x, none, none, none,
                           none, none, g, ws);
        hipLaunchKernelGGL(bn_finalize_fwd_kernel, fin_grid, fin_block, 0, stream, ws, x, pivot_stride, gamma, beta, save_mean, save_invstd, g, eps);
        const dim3 agrid(stream_blocks(total));
#define LC_BN_APPLY(TWO, RELU) \
    hipLaunchKernelGGL((bn_apply_nchw_kernel<TWO, RELU, false>), agrid, dim3(kThreads), 0, stream, x, residual, y, ws.coef, g)
        if (two) { if (clamp) LC_BN_APPLY(true, true); else LC_BN_APPLY(true, false); }
        else { if (clamp) LC_BN_APPLY(false, true); else LC_BN_APPLY(false, false); }
#undef LC_BN_APPLY
    }
    return lc_end_call();
}

extern "C" lc_status batchnorm_fwd(const float* x, const float* gamma, const float* beta, float* y, float* save_mean,
                                   float* save_invstd, int n, int c, int h, int w, float eps, lc_layout layout, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
    return batchnorm_fwd_ex(x, gamma, beta, nullptr, y, save_mean, save_invstd, n, c, h, w, eps, 0, layout, workspace, workspace_bytes,
                            hip_stream);
}

extern "C" lc_status batchnorm_bwd_ex(const float* x, const float* dy, const float* gamma, const float* beta, const float* save_mean,
                                      const float* save_invstd, float* dx, float* dgamma, float* dbeta, int n, int c, int h, int w,
                                      int relu, lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!x || !dy || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta || (relu && !beta)) return LC_ERR_NULL;
    if (layout != LC_NCHW && layout != LC_NHWC) return LC_ERR_UNSUPPORTED;
    BnGeom g;
    if (!geometry(n, c, h, w, layout, al16(x) && al16(dy) && al16(dx), &g)) return LC_ERR_SHAPE;
    if (!al4(x) || !al4(dy) || !al4(dx) || !al4(gamma) || !al4(beta) || !al4(save_mean) || !al4(save_invstd) || !al4(dgamma) || !al4(dbeta))
        return LC_ERR_ALIGN;
    size_t coef_off;
    const size_t need = ws_layout(g, &coef_off);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < need) return LC_ERR_WORKSPACE;
    BnWorkspace ws;
    ws.partial = static_cast<double*>(workspace);
    ws.coef = reinterpret_cast<float*>(static_cast<char*>(workspace) + coef_off);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lc_begin_call();
    const size_t total = (size_t)g.M * g.C;
    const dim3 fin_grid((c + kFinChannels - 1) / kFinChannels), fin_block(kFinChannels * kFinLanes);
    const bool mask = relu != 0;
    const float* mask_beta = mask ? beta : nullptr;
    if (layout == LC_NHWC) {
        const dim3 grid((unsigned)g.slabs, (unsigned)g.cblocks);
#define LC_BN_REDUCE(VEC, MODE) \
    hipLaunchKernelGGL((bn_reduce_nhwc_kernel<VEC, MODE>), grid, dim3(kThreads), 0, stream, x, dy, save_mean, save_invstd, gamma, mask_beta, g, ws)
        if (g.vec == 4) { if (mask) LC_BN_REDUCE(4, kMaskedSums); else LC_BN_REDUCE(4, kSums); }
        else { if (mask) LC_BN_REDUCE(1, kMaskedSums); else LC_BN_REDUCE(1, kSums); }
#undef LC_BN_REDUCE
        hipLaunchKernelGGL(bn_finalize_bwd_kernel, fin_grid, fin_block, 0, stream, ws, gamma, mask_beta, save_mean, save_invstd, dgamma, dbeta, g);
        const dim3 agrid(stream_blocks(total / g.vec));
#define LC_BN_APPLY(VEC, MASK) \
    hipLaunchKernelGGL((bn_apply_nhwc_kernel<VEC, true, false, MASK>), agrid, dim3(kThreads), 0, stream, x, dy, dx, ws.coef, g)
        if (g.vec == 4) { if (mask) LC_BN_APPLY(4, true); else LC_BN_APPLY(4, false); }
        else { if (mask) LC_BN_APPLY(1, true); else LC_BN_APPLY(1, false); }
#undef LC_BN_APPLY
    } else {
        const dim3 grid((unsigned)g.slabs, (unsigned)c);
        if (mask)
            hipLaunchKernelGGL((bn_reduce_nchw_kernel<kMaskedSums>), grid, dim3(kThreads), 0, stream, x, dy, save_mean, save_invstd, gamma, mask_beta, g, ws);
        else
            hipLaunchKernelGGL((bn_reduce_nchw_kernel<kSums>), grid, dim3(kThreads), 0, stream, x, dy, save_mean, save_invstd, gamma, mask_beta, g, ws);
        hipLaunchKernelGGL(bn_finalize_bwd_kernel, fin_grid, fin_block, 0, stream, ws, gamma, mask_beta, save_mean, save_invstd, dgamma, dbeta, g);
        const dim3 agrid(stream_blocks(total));
        if (mask)
            hipLaunchKernelGGL((bn_apply_nchw_kernel<true, false, true>), agrid, dim3(kThreads), 0, stream, x, dy, dx, ws.coef, g);
        else
            hipLaunchKernelGGL((bn_apply_nchw_kernel<true, false, false>), agrid, dim3(kThreads), 0, stream, x, dy, dx, ws.coef, g);
    }
    return lc_end_call();
}

extern "C" lc_status batchnorm_bwd(const float* x, const float* dy, const float* gamma, const float* save_mean,
                                   const float* save_invstd, float* dx, float* dgamma, float* dbeta, int n, int c, int h, int w,
                                   lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return batchnorm_bwd_ex(x, dy, gamma, nullptr, save_mean, save_invstd, dx, dgamma, dbeta, n, c, h, w, 0, layout, workspace,
                            workspace_bytes, hip_stream);
}
