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

// VEC consecutive elements of a tensor of fp32 values (T = float) or bf16 bit patterns (T = uint16_t) as floats and back
// (bf16 -> fp32 is exact; fp32 -> bf16 rounds to nearest even).  One 16-byte access where VEC elements fill it.
template <typename T, int VEC>
struct Pack;
template <>
struct Pack<float, 4> {
    typedef float4 raw;
    static __device__ __forceinline__ raw fetch(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ __forceinline__ void unpack(const raw& u, float (&v)[4]) { v[0] = u.x; v[1] = u.y; v[2] = u.z; v[3] = u.w; }
    static __device__ __forceinline__ void load(const float* p, float (&v)[4]) { unpack(fetch(p), v); }
    static __device__ __forceinline__ raw pack(const float (&v)[4]) { return make_float4(v[0], v[1], v[2], v[3]); }
    static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <>
struct Pack<float, 1> {
    typedef float raw;
    static __device__ __forceinline__ raw fetch(const float* p) { return *p; }
    static __device__ __forceinline__ void unpack(const raw& u, float (&v)[1]) { v[0] = u; }
    static __device__ __forceinline__ void load(const float* p, float (&v)[1]) { v[0] = *p; }
    static __device__ __forceinline__ raw pack(const float (&v)[1]) { return v[0]; }
    static __device__ __forceinline__ void store(float* p, const float (&v)[1]) { *p = v[0]; }
};
template <>
struct Pack<uint16_t, 8> {
    typedef uint4 raw;
    static __device__ __forceinline__ raw fetch(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }
    static __device__ __forceinline__ void unpack(const raw& u, float (&v)[8]) {
        const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void load(const uint16_t* p, float (&v)[8]) { unpack(fetch(p), v); }
    static __device__ __forceinline__ raw pack(const float (&v)[8]) {
        unsigned w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = lc_bf16x2_rne(v[2 * i], v[2 * i + 1]);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
    static __device__ __forceinline__ void store(uint16_t* p, const float (&v)[8]) {
        unsigned w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = lc_bf16x2_rne(v[2 * i], v[2 * i + 1]);
        *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <typename T>
__device__ __forceinline__ float widen(T v);
template <>
__device__ __forceinline__ float widen<float>(float v) { return v; }
template <>
__device__ __forceinline__ float widen<uint16_t>(uint16_t v) { return __uint_as_float((unsigned)v << 16); }

// ---------------- NHWC ----------------
// MODE kStats: sums of x and x^2.  kSums: sums of dy and dy * (x - mean) * inv_std.  kMaskedSums: the same with
// dy taken as zero where scale*x + shift <= 0.
// JOIN 1 / 2 (with kSums): dy does not exist yet -- it is the gradient that meets at a residual block's output,
// dy = (y > 0 ? da [+ db] : 0), and this pass makes it on the way: computed from y, da (and db), rounded to the storage
// type, written to join.out and summed as stored.  One pass over x saved against making dy first and summing it after.
template <typename T>
struct BnJoin {
    const T* y;
    const T* da;
    const T* db;
    T* out;
    // stride > 1: da and db hold the gradient only at the pixels (i * stride, j * stride) of every image, as
    // [n][hq][wq][c] tensors; it is zero everywhere else (what backward-data of a strided 1x1 convolution produces)
    int stride = 1, w = 0, hw = 0, wq = 0, hwq = 0;
    // row of da / db for pixel row `row` of the full tensor, or -1 off the grid (rows < 2^31: checked on the host)
    __device__ __forceinline__ long long grid_row(long long row) const {
        const unsigned r = (unsigned)row, img = r / (unsigned)hw, rem = r - img * (unsigned)hw;
        const unsigned hh = rem / (unsigned)w, ww = rem - hh * (unsigned)w;
        const unsigned hs = hh / (unsigned)stride, wss = ww / (unsigned)stride;
        if (hs * (unsigned)stride != hh || wss * (unsigned)stride != ww) return -1;
        return (long long)img * hwq + (long long)hs * wq + wss;
    }
};

template <typename T, int VEC, int MODE, int JOIN = 0>
__global__ void __launch_bounds__(kThreads) bn_reduce_nhwc_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                                  const float* __restrict__ mean, const float* __restrict__ inv_std,
                                                                  const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                  BnGeom g, BnWorkspace ws, BnJoin<T> join = BnJoin<T>{}) {
    constexpr bool STATS = MODE == kStats;
    constexpr int TU = 4;                                 // a tile is TU rows of the block's threads (the same for every form: equal sums)
    constexpr int U = JOIN ? 2 : 4;                       // rows a thread has in flight
    static_assert(JOIN == 0 || MODE == kSums, "the joined form makes an unmasked dy");
    __shared__ float red[kThreads * 2 * VEC];
    const int tx = threadIdx.x % g.tx, ty = threadIdx.x / g.tx;
    const int c0 = (blockIdx.y * g.tx + tx) * VEC;
    const bool live = c0 < g.C;
    float s0[VEC], s1[VEC], mu[VEC], is[VEC], sc[VEC], sh[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        s0[e] = s1[e] = 0.f;
        mu[e] = (!STATS && live) ? mean[c0 + e] : 0.f;
        is[e] = (!STATS && live) ? inv_std[c0 + e] : 0.f;
        sc[e] = sh[e] = 0.f;
        if (MODE == kMaskedSums && live) scale_shift(gamma[c0 + e], beta[c0 + e], mu[e], is[e], &sc[e], &sh[e]);
        if (STATS && live) mu[e] = widen<T>(x[c0 + e]);   // the channel's pivot: its value at the first pixel
    }
    auto add_row = [&](const float (&a)[VEC], const float (&b)[VEC]) {
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
    };
    // Tiles of ty * U rows go round the blocks of the grid, so that at any moment the grid reads one contiguous
    // stretch of the tensor (a block that kept to a region of its own would make as many scattered streams as blocks).
    if (live) {
        const long long tile = (long long)g.ty * TU;
        for (long long base = (long long)blockIdx.x * tile; base < g.M; base += (long long)gridDim.x * tile) {
            if (base + tile <= g.M) {                                             // U loads per tensor, then U rows in order
              for (int part = 0; part < TU; part += U) {
                const long long r = base + ty + (long long)part * g.ty;
                typename Pack<T, VEC>::raw ra[U], rb[U], ry[JOIN ? U : 1], rc[JOIN == 2 ? U : 1];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const long long at = (r + (long long)u * g.ty) * g.C + c0;
                    ra[u] = Pack<T, VEC>::fetch(x + at);
                    if constexpr (JOIN) {
                        ry[u] = Pack<T, VEC>::fetch(join.y + at);
                        long long gat = at;
                        if (join.stride > 1) {
                            const long long gr = join.grid_row(r + (long long)u * g.ty);
                            gat = gr < 0 ? -1 : gr * g.C + c0;
                        }
                        rb[u] = typename Pack<T, VEC>::raw{};
                        if (gat >= 0) rb[u] = Pack<T, VEC>::fetch(join.da + gat);
                        if constexpr (JOIN == 2) {
                            rc[u] = typename Pack<T, VEC>::raw{};
                            if (gat >= 0) rc[u] = Pack<T, VEC>::fetch(join.db + gat);
                        }
                    } else if constexpr (!STATS) {
                        rb[u] = Pack<T, VEC>::fetch(dy + at);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);        // all loads are issued before the first is waited for
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float a[VEC], b[VEC];
                    Pack<T, VEC>::unpack(ra[u], a);
                    if constexpr (JOIN) {
                        float yv[VEC], h2[VEC];
                        Pack<T, VEC>::unpack(ry[u], yv);
                        Pack<T, VEC>::unpack(rb[u], b);
                        if constexpr (JOIN == 2) Pack<T, VEC>::unpack(rc[u], h2);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            if constexpr (JOIN == 2) b[e] += h2[e];
                            if (!(yv[e] > 0.f)) b[e] = 0.f;
                        }
                        const typename Pack<T, VEC>::raw stored = Pack<T, VEC>::pack(b);
                        *reinterpret_cast<typename Pack<T, VEC>::raw*>(join.out + (r + (long long)u * g.ty) * g.C + c0) = stored;
                        Pack<T, VEC>::unpack(stored, b);                           // the sums are those of the stored values
                    } else if constexpr (!STATS) {
                        Pack<T, VEC>::unpack(rb[u], b);
                    }
                    add_row(a, b);
                }
              }
            } else {                                                              // the tensor's last, partial tile
                for (long long q = base + ty; q < g.M; q += g.ty) {
                    float a[VEC], b[VEC];
                    Pack<T, VEC>::load(x + q * g.C + c0, a);
                    if constexpr (JOIN) {
                        float yv[VEC], h2[VEC];
                        Pack<T, VEC>::load(join.y + q * g.C + c0, yv);
                        long long gat = q * g.C + c0;
                        if (join.stride > 1) {
                            const long long gr = join.grid_row(q);
                            gat = gr < 0 ? -1 : gr * g.C + c0;
                        }
#pragma unroll
                        for (int e = 0; e < VEC; ++e) b[e] = h2[e] = 0.f;
                        if (gat >= 0) {
                            Pack<T, VEC>::load(join.da + gat, b);
                            if constexpr (JOIN == 2) Pack<T, VEC>::load(join.db + gat, h2);
                        }
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            if constexpr (JOIN == 2) b[e] += h2[e];
                            if (!(yv[e] > 0.f)) b[e] = 0.f;
                        }
                        const typename Pack<T, VEC>::raw stored = Pack<T, VEC>::pack(b);
                        *reinterpret_cast<typename Pack<T, VEC>::raw*>(join.out + q * g.C + c0) = stored;
                        Pack<T, VEC>::unpack(stored, b);
                    } else if constexpr (!STATS) {
                        Pack<T, VEC>::load(dy + q * g.C + c0, b);
                    }
                    add_row(a, b);
                }
            }
        }
    }
    // red[ty][tx][2 * VEC]: a row of the block's threads is one contiguous run of columns
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        red[threadIdx.x * 2 * VEC + 2 * e] = s0[e];
        red[threadIdx.x * 2 * VEC + 2 * e + 1] = s1[e];
    }
    __syncthreads();
    // one thread per column adds the block's rows in order (double); columns of the channels beyond c are left out
    const int ncols = g.tx * 2 * VEC;
    for (int j = threadIdx.x; j < ncols; j += kThreads) {
        const int ch2 = blockIdx.y * ncols + j;           // 2 * channel + which sum
        if (ch2 >= 2 * g.C) continue;
        double t = 0.0;
        for (int k = 0; k < g.ty; ++k) t += (double)red[k * ncols + j];
        ws.partial[(size_t)blockIdx.x * g.C * 2 + ch2] = t;
    }
}

// out = p*A + q*B + r per channel (TWO false: out = p*A + r).  RELU: clamp the result at zero.  MASK: B counts as
// zero where scale*A + shift <= 0.
// VEC consecutive per-channel coefficients (16-byte loads where VEC allows: the arrays start 16-byte aligned and the
// vector paths have c a multiple of VEC)
template <int VEC>
__device__ __forceinline__ void load_coef(const float* __restrict__ p, float (&v)[VEC]) {
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
            const float4 u = reinterpret_cast<const float4*>(p)[q];
            v[4 * q] = u.x; v[4 * q + 1] = u.y; v[4 * q + 2] = u.z; v[4 * q + 3] = u.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = p[e];
    }
}

// INV: the launch makes (threads in the grid) * VEC a multiple of c, so a thread meets the same channels on every
// trip of its loop and keeps their coefficients in registers.
template <typename T, int VEC, bool TWO, bool RELU, bool MASK, bool INV>
__global__ void __launch_bounds__(kThreads) bn_apply_nhwc_kernel(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ out,
                                                                 const float* __restrict__ coef, BnGeom g) {
    const size_t total = (size_t)g.M * g.C / VEC;
    const size_t first = blockIdx.x * (size_t)blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    float p[VEC], r[VEC], q[TWO ? VEC : 1], ms[MASK ? VEC : 1], mh[MASK ? VEC : 1];
    auto coefficients = [&](int c0) {
        load_coef<VEC>(coef + c0, p);
        load_coef<VEC>(coef + 2 * g.C + c0, r);
        if constexpr (TWO) load_coef<VEC>(coef + g.C + c0, q);
        if constexpr (MASK) {
            load_coef<VEC>(coef + 3 * g.C + c0, ms);
            load_coef<VEC>(coef + 4 * g.C + c0, mh);
        }
    };
    if constexpr (INV) coefficients((int)((first * VEC) % g.C));
    for (size_t i = first; i < total; i += stride) {
        if constexpr (!INV) coefficients((int)((i * VEC) % g.C));
        float va[VEC], vb[VEC], o[VEC];
        Pack<T, VEC>::load(a + i * VEC, va);
        if constexpr (TWO) Pack<T, VEC>::load(b + i * VEC, vb);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            o[e] = fmaf(p[e], va[e], r[e]);
            if constexpr (TWO) {
                float t = vb[e];
                if constexpr (MASK)
                    if (!(fmaf(ms[e], va[e], mh[e]) > 0.f)) t = 0.f;
                o[e] = fmaf(q[e], t, o[e]);
            }
            if constexpr (RELU) o[e] = fmaxf(o[e], 0.f);
        }
        Pack<T, VEC>::store(out + i * VEC, o);
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

// Statistics that arrive as fp32 pieces [pieces][cols] (cols = 2 * channels: sum and sum of squares side by side) are
// folded into the slab partials the finalize kernel adds: slab s takes pieces s, s + slabs, ... in that order, in double.
__global__ void __launch_bounds__(kThreads) bn_fold_pieces_kernel(const float* __restrict__ pieces, int n_pieces, double* __restrict__ partial,
                                                                  int slabs, int cols) {
    const int j = blockIdx.y * kThreads + threadIdx.x;
    if (j >= cols) return;
    double t0 = 0.0, t1 = 0.0;
    int t = blockIdx.x;
    for (; t + slabs < n_pieces; t += 2 * slabs) {
        t0 += (double)pieces[(size_t)t * cols + j];
        t1 += (double)pieces[(size_t)(t + slabs) * cols + j];
    }
    if (t < n_pieces) t0 += (double)pieces[(size_t)t * cols + j];
    partial[(size_t)blockIdx.x * cols + j] = t0 + t1;
}

// ---------------- per-channel finalize ----------------
// A block of 256 threads finishes 4 channels: 64 lanes per channel add every 64th slab's partial (two running sums
// each, so that loads overlap), then the first lane adds the 64 lane sums in lane order.  Returns true in the thread
// that holds the channel's totals.  Few channels per block: the layers with 64 channels still start 16 blocks.
constexpr int kFinChannels = 4, kFinLanes = 64;
__device__ __forceinline__ bool channel_totals(const BnWorkspace& ws, const BnGeom& g, int* ch_out, double* t0, double* t1) {
    __shared__ double red[kFinLanes][kFinChannels][2];
    const int cl = threadIdx.x % kFinChannels, sl = threadIdx.x / kFinChannels;
    const int ch = blockIdx.x * kFinChannels + cl;
    double s0 = 0.0, s1 = 0.0, u0 = 0.0, u1 = 0.0;
    if (ch < g.C) {
        const double2* part = reinterpret_cast<const double2*>(ws.partial);
        int k = sl;
        for (; k + kFinLanes < g.slabs; k += 2 * kFinLanes) {
            const double2 a = part[(size_t)k * g.C + ch], b = part[(size_t)(k + kFinLanes) * g.C + ch];
            s0 += a.x; s1 += a.y;
            u0 += b.x; u1 += b.y;
        }
        if (k < g.slabs) {
            const double2 a = part[(size_t)k * g.C + ch];
            s0 += a.x; s1 += a.y;
        }
    }
    red[sl][cl][0] = s0 + u0;
    red[sl][cl][1] = s1 + u1;
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
// A second batch norm whose output is the residual of the first (its statistics already final): see batchnorm_fwd_pair_t.
struct BnSecond {
    const float* gamma = nullptr;
    const float* beta = nullptr;
    const float* mean = nullptr;
    const float* inv_std = nullptr;
};

template <typename T>
__global__ void __launch_bounds__(kFinChannels* kFinLanes)
bn_finalize_fwd_kernel(BnWorkspace ws, const T* __restrict__ x, size_t pivot_stride, const float* __restrict__ gamma,
                       const float* __restrict__ beta, float* __restrict__ save_mean, float* __restrict__ save_invstd, BnGeom g, float eps,
                       BnSecond second) {
    int ch;
    double s0, s1;
    if (!channel_totals(ws, g, &ch, &s0, &s1)) return;
    const double m = (double)g.M;
    const double off = s0 / m;                                  // mean of x - pivot
    const double mean = (x ? (double)widen<T>(x[ch * pivot_stride]) : 0.0) + off;      // x null: plain sums, no pivot
    double var = s1 / m - off * off;
    if (var < 0.0) var = 0.0;
    const double inv_std = 1.0 / sqrt(var + (double)eps);
    const float mean_f = (float)mean, inv_std_f = (float)inv_std;
    save_mean[ch] = mean_f;
    save_invstd[ch] = inv_std_f;
    float scale, shift;
    scale_shift(gamma[ch], beta[ch], mean_f, inv_std_f, &scale, &shift);
    float scale2 = 1.f;                    // the residual, when there is one, is added as it is ...
    if (second.gamma) {                    // ... unless it is the input of a second batch norm, normalised on the way
        float shift2;
        scale_shift(second.gamma[ch], second.beta[ch], second.mean[ch], second.inv_std[ch], &scale2, &shift2);
        shift += shift2;
    }
    ws.coef[ch] = scale;
    ws.coef[g.C + ch] = scale2;
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

bool geometry(int n, int c, int h, int w, lc_layout layout, bool aligned16, BnGeom* g, int wide = 4) {
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return false;
    const long long hw = (long long)h * w;
    if (hw > 0x7fffffffLL) return false;
    g->N = n;
    g->C = c;
    g->HW = (int)hw;
    g->M = (long long)n * hw;
    if (layout == LC_NHWC) {
        g->vec = (c % wide == 0 && aligned16) ? wide : 1;     // wide: elements in 16 bytes
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

// grid of the NHWC apply pass over `items` threads' worth of work; *inv: the grid was sized so that every thread stays on
// one group of channels (grid * kThreads * vec is a multiple of c)
inline unsigned apply_blocks(size_t items, int c, int vec, bool* inv) {
    unsigned b = stream_blocks(items);
    long long x = (long long)kThreads * vec, y = c;
    while (y) { const long long t = x % y; x = y; y = t; }            // x = gcd(kThreads * vec, c)
    const long long m = c / x;
    *inv = m <= 64;
    if (*inv) b = (unsigned)((b + m - 1) / m * m);
    return b;
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

namespace {

// bf16 tensors are taken in NHWC with whole 16-byte groups of channels only (what the bf16 convolutions produce)
template <typename T>
constexpr int kWide = 16 / (int)sizeof(T);

template <typename T>
lc_status bn_fwd_impl(const T* x, const float* gamma, const float* beta, const T* residual, T* y, float* save_mean, float* save_invstd,
                      int n, int c, int h, int w, float eps, int relu, lc_layout layout, void* workspace, size_t workspace_bytes,
                      void* hip_stream, const float* stats = nullptr, size_t stats_tiles = 0, bool stats_only = false,
                      BnSecond second = BnSecond{}, bool check_only = false) {
    constexpr bool kF32 = sizeof(T) == 4;
    if (!x || !gamma || !beta || (!y && !stats_only) || !save_mean || !save_invstd) return LC_ERR_NULL;
    if (second.gamma && !residual) return LC_ERR_NULL;
    if (layout != LC_NCHW && layout != LC_NHWC) return LC_ERR_UNSUPPORTED;
    if (!(eps >= 0.f)) return LC_ERR_SHAPE;
    BnGeom g;
    if (!geometry(n, c, h, w, layout, al16(x) && al16(y) && al16(residual), &g, kWide<T>)) return LC_ERR_SHAPE;
    if (!al4(x) || !al4(y) || !al4(residual) || !al4(gamma) || !al4(beta) || !al4(save_mean) || !al4(save_invstd)) return LC_ERR_ALIGN;
    if (!al4(second.gamma) || !al4(second.beta) || !al4(second.mean) || !al4(second.inv_std)) return LC_ERR_ALIGN;
    if (!kF32 && layout != LC_NHWC) return LC_ERR_UNSUPPORTED;
    if (!kF32 && g.vec != kWide<T>) return c % kWide<T> ? LC_ERR_UNSUPPORTED : LC_ERR_ALIGN;
    if (stats && (layout != LC_NHWC || stats_tiles == 0 || stats_tiles > 0x7fffffffull)) return LC_ERR_UNSUPPORTED;
    if (stats && (reinterpret_cast<uintptr_t>(stats) & 7)) return LC_ERR_ALIGN;
    size_t coef_off;
    const size_t need = ws_layout(g, &coef_off);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < need) return LC_ERR_WORKSPACE;
    if (check_only) return LC_OK;          // (a caller that launches something else first wants every argument checked before)
    BnWorkspace ws;
    ws.partial = static_cast<double*>(workspace);
    ws.coef = reinterpret_cast<float*>(static_cast<char*>(workspace) + coef_off);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lc_begin_call();
    const size_t total = (size_t)g.M * g.C;
    const dim3 fin_grid((c + kFinChannels - 1) / kFinChannels), fin_block(kFinChannels * kFinLanes);
    const T* none = nullptr;
    const float* nonef = nullptr;
    const bool two = residual != nullptr, clamp = relu != 0;
    // sums handed over by the producer of x (plain sums of x and x^2, fp32 pieces in [stats_tiles][c][2]): no pass over x of
    // our own; the pieces are first folded into this pass's slab partials, piece t into slab t mod slabs, in order
    const size_t pivot_stride = layout == LC_NHWC ? 1 : (size_t)g.HW;       // the first pixel's value of channel ch sits at x[ch * stride]
    if (layout == LC_NHWC) {
        const dim3 grid((unsigned)g.slabs, (unsigned)g.cblocks);
        bool inv;
        const dim3 agrid(apply_blocks(total / g.vec, c, g.vec, &inv));
#define LC_BN_APPLY(VEC, TWO, RELU)                                                                                                   \
    do {                                                                                                                              \
        if (inv)                                                                                                                      \
            hipLaunchKernelGGL((bn_apply_nhwc_kernel<T, VEC, TWO, RELU, false, true>), agrid, dim3(kThreads), 0, stream, x, residual, y, \
                               ws.coef, g);                                                                                           \
        else                                                                                                                          \
            hipLaunchKernelGGL((bn_apply_nhwc_kernel<T, VEC, TWO, RELU, false, false>), agrid, dim3(kThreads), 0, stream, x, residual, y, \
                               ws.coef, g);                                                                                           \
    } while (0)
#define LC_BN_FWD(VEC)                                                                                                                  \
    do {                                                                                                                                \
        if (stats) {                                                                                                                    \
            hipLaunchKernelGGL(bn_fold_pieces_kernel, dim3((unsigned)g.slabs, (unsigned)((2 * c + kThreads - 1) / kThreads)),           \
                               dim3(kThreads), 0, stream, stats, (int)stats_tiles, ws.partial, g.slabs, 2 * c);                         \
            hipLaunchKernelGGL(bn_finalize_fwd_kernel<T>, fin_grid, fin_block, 0, stream, ws, none, pivot_stride, gamma, beta,          \
                               save_mean, save_invstd, g, eps, second);                                                                 \
        } else {                                                                                                                        \
            hipLaunchKernelGGL((bn_reduce_nhwc_kernel<T, VEC, kStats>), grid, dim3(kThreads), 0, stream, x, none, nonef, nonef, nonef,  \
                               nonef, g, ws);                                                                                           \
            hipLaunchKernelGGL(bn_finalize_fwd_kernel<T>, fin_grid, fin_block, 0, stream, ws, x, pivot_stride, gamma, beta, save_mean,  \
                               save_invstd, g, eps, second);                                                                            \
        }                                                                                                                               \
        if (stats_only) break;                                                                                                          \
        if (two) { if (clamp) LC_BN_APPLY(VEC, true, true); else LC_BN_APPLY(VEC, true, false); }                                       \
        else { if (clamp) LC_BN_APPLY(VEC, false, true); else LC_BN_APPLY(VEC, false, false); }                                         \
    } while (0)
        if constexpr (kF32) {
            if (g.vec == 4) LC_BN_FWD(4); else LC_BN_FWD(1);
        } else {
            LC_BN_FWD(8);
        }
#undef LC_BN_FWD
#undef LC_BN_APPLY
    } else {
        if constexpr (kF32) {
            hipLaunchKernelGGL((bn_reduce_nchw_kernel<kStats>), dim3((unsigned)g.slabs, (unsigned)c), dim3(kThreads), 0, stream, x, none, nonef,
                               nonef, nonef, nonef, g, ws);
            hipLaunchKernelGGL(bn_finalize_fwd_kernel<T>, fin_grid, fin_block, 0, stream, ws, x, pivot_stride, gamma, beta, save_mean,
                               save_invstd, g, eps, second);
            const dim3 agrid(stream_blocks(total));
#define LC_BN_APPLY(TWO, RELU) \
    hipLaunchKernelGGL((bn_apply_nchw_kernel<TWO, RELU, false>), agrid, dim3(kThreads), 0, stream, x, residual, y, ws.coef, g)
            if (stats_only) return lc_end_call();
            if (two) { if (clamp) LC_BN_APPLY(true, true); else LC_BN_APPLY(true, false); }
            else { if (clamp) LC_BN_APPLY(false, true); else LC_BN_APPLY(false, false); }
#undef LC_BN_APPLY
        }
    }
    return lc_end_call();
}

// y = relu?(bn(x) + bn2(x2)): the statistics of the second batch norm first (no stream pass), then the first with the
// second's scale and shift folded into its residual coefficients, one stream pass over x and x2.
template <typename T>
lc_status bn_fwd_pair_impl(const T* x, const float* gamma, const float* beta, const float* stats, size_t stats_tiles, const T* x2,
                           const float* gamma2, const float* beta2, const float* stats2, size_t stats_tiles2, T* y, float* save_mean,
                           float* save_invstd, float* save_mean2, float* save_invstd2, int n, int c, int h, int w, float eps, int relu,
                           lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!x2 || !y) return LC_ERR_NULL;
    BnSecond second;
    second.gamma = gamma2;
    second.beta = beta2;
    second.mean = save_mean2;
    second.inv_std = save_invstd2;
    // both calls' arguments are checked before the first launches anything
    lc_status st = bn_fwd_impl<T>(x, gamma, beta, x2, y, save_mean, save_invstd, n, c, h, w, eps, relu, layout, workspace, workspace_bytes,
                                  hip_stream, stats, stats_tiles, false, second, true);
    if (st != LC_OK) return st;
    st = bn_fwd_impl<T>(x2, gamma2, beta2, nullptr, nullptr, save_mean2, save_invstd2, n, c, h, w, eps, 0, layout, workspace,
                        workspace_bytes, hip_stream, stats2, stats_tiles2, true);
    if (st != LC_OK) return st;
    return bn_fwd_impl<T>(x, gamma, beta, x2, y, save_mean, save_invstd, n, c, h, w, eps, relu, layout, workspace, workspace_bytes,
                          hip_stream, stats, stats_tiles, false, second);
}

template <typename T>
lc_status bn_bwd_impl(const T* x, const T* dy, const float* gamma, const float* beta, const float* save_mean, const float* save_invstd,
                      T* dx, float* dgamma, float* dbeta, int n, int c, int h, int w, int relu, lc_layout layout, void* workspace,
                      size_t workspace_bytes, void* hip_stream, bool presummed = false) {
    constexpr bool kF32 = sizeof(T) == 4;
    if (!x || !dy || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta || (relu && !beta)) return LC_ERR_NULL;
    if (layout != LC_NCHW && layout != LC_NHWC) return LC_ERR_UNSUPPORTED;
    BnGeom g;
    if (!geometry(n, c, h, w, layout, al16(x) && al16(dy) && al16(dx), &g, kWide<T>)) return LC_ERR_SHAPE;
    if (!al4(x) || !al4(dy) || !al4(dx) || !al4(gamma) || !al4(beta) || !al4(save_mean) || !al4(save_invstd) || !al4(dgamma) || !al4(dbeta))
        return LC_ERR_ALIGN;
    if (!kF32 && layout != LC_NHWC) return LC_ERR_UNSUPPORTED;
    if (!kF32 && g.vec != kWide<T>) return c % kWide<T> ? LC_ERR_UNSUPPORTED : LC_ERR_ALIGN;
    // sums left in the workspace by relu_add_bwd_bnsums_t: only the geometry of the vector path is shared by the two calls
    if (presummed && (layout != LC_NHWC || relu || g.vec != kWide<T>)) return LC_ERR_UNSUPPORTED;
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
        bool inv;
        const dim3 agrid(apply_blocks(total / g.vec, c, g.vec, &inv));
#define LC_BN_BWD(VEC, MODE, MASK)                                                                                                       \
    do {                                                                                                                                \
        if (!presummed)                                                                                                                 \
            hipLaunchKernelGGL((bn_reduce_nhwc_kernel<T, VEC, MODE>), grid, dim3(kThreads), 0, stream, x, dy, save_mean, save_invstd,    \
                               gamma, mask_beta, g, ws, BnJoin<T>{});                                                                   \
        hipLaunchKernelGGL(bn_finalize_bwd_kernel, fin_grid, fin_block, 0, stream, ws, gamma, mask_beta, save_mean, save_invstd, dgamma, \
                           dbeta, g);                                                                                                   \
        if (inv)                                                                                                                        \
            hipLaunchKernelGGL((bn_apply_nhwc_kernel<T, VEC, true, false, MASK, true>), agrid, dim3(kThreads), 0, stream, x, dy, dx,     \
                               ws.coef, g);                                                                                             \
        else                                                                                                                            \
            hipLaunchKernelGGL((bn_apply_nhwc_kernel<T, VEC, true, false, MASK, false>), agrid, dim3(kThreads), 0, stream, x, dy, dx,    \
                               ws.coef, g);                                                                                             \
    } while (0)
        if constexpr (kF32) {
            if (g.vec == 4) { if (mask) LC_BN_BWD(4, kMaskedSums, true); else LC_BN_BWD(4, kSums, false); }
            else { if (mask) LC_BN_BWD(1, kMaskedSums, true); else LC_BN_BWD(1, kSums, false); }
        } else {
            if (mask) LC_BN_BWD(8, kMaskedSums, true); else LC_BN_BWD(8, kSums, false);
        }
#undef LC_BN_BWD
    } else {
        if constexpr (kF32) {
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
    }
    return lc_end_call();
}

// dx = (y > 0 ? da [+ db] : 0) and, in the workspace, the sums batch-norm backward needs of that dx against x_bn
template <typename T>
lc_status bn_join_impl(const T* y, const T* da, const T* db, T* dx, const T* x_bn, const float* save_mean, const float* save_invstd, int n,
                       int c, int h, int w, lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream, int stride = 1) {
    if (!y || !da || !dx || !x_bn || !save_mean || !save_invstd) return LC_ERR_NULL;
    if (layout != LC_NHWC) return LC_ERR_UNSUPPORTED;
    if (stride < 1) return LC_ERR_SHAPE;
    BnGeom g;
    if (!geometry(n, c, h, w, layout, al16(y) && al16(da) && al16(db) && al16(dx) && al16(x_bn), &g, kWide<T>)) return LC_ERR_SHAPE;
    if (!al4(y) || !al4(da) || !al4(db) || !al4(dx) || !al4(x_bn) || !al4(save_mean) || !al4(save_invstd)) return LC_ERR_ALIGN;
    if (g.vec != kWide<T>) return c % kWide<T> ? LC_ERR_UNSUPPORTED : LC_ERR_ALIGN;
    if (stride > 1 && g.M > 0x7fffffffLL) return LC_ERR_SHAPE;          // the grid index arithmetic is 32-bit
    size_t coef_off;
    const size_t need = ws_layout(g, &coef_off);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < need) return LC_ERR_WORKSPACE;
    BnWorkspace ws;
    ws.partial = static_cast<double*>(workspace);
    ws.coef = reinterpret_cast<float*>(static_cast<char*>(workspace) + coef_off);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lc_begin_call();
    const dim3 grid((unsigned)g.slabs, (unsigned)g.cblocks);
    const float* nonef = nullptr;
    const T* none = nullptr;
    BnJoin<T> join{y, da, db, dx};
    if (stride > 1) {
        join.stride = stride;
        join.w = w;
        join.hw = g.HW;
        join.wq = (w + stride - 1) / stride;
        join.hwq = ((h + stride - 1) / stride) * join.wq;
    }
    if (db)
        hipLaunchKernelGGL((bn_reduce_nhwc_kernel<T, kWide<T>, kSums, 2>), grid, dim3(kThreads), 0, stream, x_bn, none, save_mean, save_invstd,
                           nonef, nonef, g, ws, join);
    else
        hipLaunchKernelGGL((bn_reduce_nhwc_kernel<T, kWide<T>, kSums, 1>), grid, dim3(kThreads), 0, stream, x_bn, none, save_mean, save_invstd,
                           nonef, nonef, g, ws, join);
    return lc_end_call();
}

}  // namespace

extern "C" lc_status relu_add_bwd_bnsums_t(lc_dtype dtype, const void* y, const void* da, const void* db, void* dx, const void* x_bn,
                                           const float* save_mean, const float* save_invstd, int n, int c, int h, int w, lc_layout layout,
                                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (dtype == LC_F32)
        return bn_join_impl<float>(static_cast<const float*>(y), static_cast<const float*>(da), static_cast<const float*>(db),
                                   static_cast<float*>(dx), static_cast<const float*>(x_bn), save_mean, save_invstd, n, c, h, w, layout,
                                   workspace, workspace_bytes, hip_stream);
    if (dtype == LC_BF16)
        return bn_join_impl<uint16_t>(static_cast<const uint16_t*>(y), static_cast<const uint16_t*>(da), static_cast<const uint16_t*>(db),
                                      static_cast<uint16_t*>(dx), static_cast<const uint16_t*>(x_bn), save_mean, save_invstd, n, c, h, w,
                                      layout, workspace, workspace_bytes, hip_stream);
    return LC_ERR_UNSUPPORTED;
}

extern "C" lc_status relu_add_bwd_bnsums_grid_t(lc_dtype dtype, const void* y, const void* da, const void* db, void* dx, const void* x_bn,
                                                const float* save_mean, const float* save_invstd, int n, int c, int h, int w,
                                                int grad_stride, lc_layout layout, void* workspace, size_t workspace_bytes,
                                                void* hip_stream) {
    if (dtype == LC_F32)
        return bn_join_impl<float>(static_cast<const float*>(y), static_cast<const float*>(da), static_cast<const float*>(db),
                                   static_cast<float*>(dx), static_cast<const float*>(x_bn), save_mean, save_invstd, n, c, h, w, layout,
                                   workspace, workspace_bytes, hip_stream, grad_stride);
    if (dtype == LC_BF16)
        return bn_join_impl<uint16_t>(static_cast<const uint16_t*>(y), static_cast<const uint16_t*>(da), static_cast<const uint16_t*>(db),
                                      static_cast<uint16_t*>(dx), static_cast<const uint16_t*>(x_bn), save_mean, save_invstd, n, c, h, w,
                                      layout, workspace, workspace_bytes, hip_stream, grad_stride);
    return LC_ERR_UNSUPPORTED;
}

extern "C" lc_status batchnorm_bwd_presummed_t(lc_dtype dtype, const void* x, const void* dy, const float* gamma, const float* save_mean,
                                               const float* save_invstd, void* dx, float* dgamma, float* dbeta, int n, int c, int h, int w,
                                               lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (dtype == LC_F32)
        return bn_bwd_impl<float>(static_cast<const float*>(x), static_cast<const float*>(dy), gamma, nullptr, save_mean, save_invstd,
                                  static_cast<float*>(dx), dgamma, dbeta, n, c, h, w, 0, layout, workspace, workspace_bytes, hip_stream, true);
    if (dtype == LC_BF16)
        return bn_bwd_impl<uint16_t>(static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(dy), gamma, nullptr, save_mean,
                                     save_invstd, static_cast<uint16_t*>(dx), dgamma, dbeta, n, c, h, w, 0, layout, workspace,
                                     workspace_bytes, hip_stream, true);
    return LC_ERR_UNSUPPORTED;
}

extern "C" lc_status batchnorm_fwd_ex(const float* x, const float* gamma, const float* beta, const float* residual, float* y,
                                      float* save_mean, float* save_invstd, int n, int c, int h, int w, float eps, int relu,
                                      lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return bn_fwd_impl<float>(x, gamma, beta, residual, y, save_mean, save_invstd, n, c, h, w, eps, relu, layout, workspace, workspace_bytes,
                              hip_stream);
}

extern "C" lc_status batchnorm_fwd_t(lc_dtype dtype, const void* x, const float* gamma, const float* beta, const void* residual, void* y,
                                     float* save_mean, float* save_invstd, int n, int c, int h, int w, float eps, int relu,
                                     lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (dtype == LC_F32)
        return bn_fwd_impl<float>(static_cast<const float*>(x), gamma, beta, static_cast<const float*>(residual), static_cast<float*>(y),
                                  save_mean, save_invstd, n, c, h, w, eps, relu, layout, workspace, workspace_bytes, hip_stream);
    if (dtype == LC_BF16)
        return bn_fwd_impl<uint16_t>(static_cast<const uint16_t*>(x), gamma, beta, static_cast<const uint16_t*>(residual),
                                     static_cast<uint16_t*>(y), save_mean, save_invstd, n, c, h, w, eps, relu, layout, workspace,
                                     workspace_bytes, hip_stream);
    return LC_ERR_UNSUPPORTED;
}

extern "C" lc_status batchnorm_fwd_pre(lc_dtype dtype, const void* x, const float* gamma, const float* beta, const void* residual, void* y,
                                       float* save_mean, float* save_invstd, int n, int c, int h, int w, float eps, int relu,
                                       lc_layout layout, const float* stats, size_t stats_tiles, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
    if (!stats) return LC_ERR_NULL;
    if (dtype == LC_F32)
        return bn_fwd_impl<float>(static_cast<const float*>(x), gamma, beta, static_cast<const float*>(residual), static_cast<float*>(y),
                                  save_mean, save_invstd, n, c, h, w, eps, relu, layout, workspace, workspace_bytes, hip_stream, stats,
                                  stats_tiles);
    if (dtype == LC_BF16)
        return bn_fwd_impl<uint16_t>(static_cast<const uint16_t*>(x), gamma, beta, static_cast<const uint16_t*>(residual),
                                     static_cast<uint16_t*>(y), save_mean, save_invstd, n, c, h, w, eps, relu, layout, workspace,
                                     workspace_bytes, hip_stream, stats, stats_tiles);
    return LC_ERR_UNSUPPORTED;
}

extern "C" lc_status batchnorm_fwd_pair_t(lc_dtype dtype, const void* x, const float* gamma, const float* beta, const float* stats,
                                          size_t stats_tiles, const void* x2, const float* gamma2, const float* beta2, const float* stats2,
                                          size_t stats_tiles2, void* y, float* save_mean, float* save_invstd, float* save_mean2,
                                          float* save_invstd2, int n, int c, int h, int w, float eps, int relu, lc_layout layout,
                                          void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (dtype == LC_F32)
        return bn_fwd_pair_impl<float>(static_cast<const float*>(x), gamma, beta, stats, stats_tiles, static_cast<const float*>(x2), gamma2,
                                       beta2, stats2, stats_tiles2, static_cast<float*>(y), save_mean, save_invstd, save_mean2, save_invstd2,
                                       n, c, h, w, eps, relu, layout, workspace, workspace_bytes, hip_stream);
    if (dtype == LC_BF16)
        return bn_fwd_pair_impl<uint16_t>(static_cast<const uint16_t*>(x), gamma, beta, stats, stats_tiles, static_cast<const uint16_t*>(x2),
                                          gamma2, beta2, stats2, stats_tiles2, static_cast<uint16_t*>(y), save_mean, save_invstd, save_mean2,
                                          save_invstd2, n, c, h, w, eps, relu, layout, workspace, workspace_bytes, hip_stream);
    return LC_ERR_UNSUPPORTED;
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
    return bn_bwd_impl<float>(x, dy, gamma, beta, save_mean, save_invstd, dx, dgamma, dbeta, n, c, h, w, relu, layout, workspace,
                              workspace_bytes, hip_stream);
}

extern "C" lc_status batchnorm_bwd_t(lc_dtype dtype, const void* x, const void* dy, const float* gamma, const float* beta,
                                     const float* save_mean, const float* save_invstd, void* dx, float* dgamma, float* dbeta, int n, int c,
                                     int h, int w, int relu, lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (dtype == LC_F32)
        return bn_bwd_impl<float>(static_cast<const float*>(x), static_cast<const float*>(dy), gamma, beta, save_mean, save_invstd,
                                  static_cast<float*>(dx), dgamma, dbeta, n, c, h, w, relu, layout, workspace, workspace_bytes, hip_stream);
    if (dtype == LC_BF16)
        return bn_bwd_impl<uint16_t>(static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(dy), gamma, beta, save_mean,
                                     save_invstd, static_cast<uint16_t*>(dx), dgamma, dbeta, n, c, h, w, relu, layout, workspace,
                                     workspace_bytes, hip_stream);
    return LC_ERR_UNSUPPORTED;
}

extern "C" lc_status batchnorm_bwd(const float* x, const float* dy, const float* gamma, const float* save_mean,
                                   const float* save_invstd, float* dx, float* dgamma, float* dbeta, int n, int c, int h, int w,
                                   lc_layout layout, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return batchnorm_bwd_ex(x, dy, gamma, nullptr, save_mean, save_invstd, dx, dgamma, dbeta, n, c, h, w, 0, layout, workspace,
                            workspace_bytes, hip_stream);
}
