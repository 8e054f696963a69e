// Glue layers of the networks the paper trains: ReLU, max pooling (2x2, and any window / stride / pad for the
// overlapping pools of ResNet-50 and AlexNet), global average pooling, bias, softmax cross-entropy, and the
// gradient that meets at a residual block's output.  The paper does not discuss them (they are implied by the
// networks, "Experimental Settings"); these are the textbook definitions in fp32, memory-bound streaming kernels.
// Reductions run in a fixed order (bit-identical reruns).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/larsconv.h"
#include "internal.h"
#include "pool_patch.h"

namespace {

constexpr int kThreads = 256;

inline unsigned blocks_for(size_t count) {
    size_t b = (count + kThreads - 1) / kThreads;
    if (b > 65535u * 16u) b = 65535u * 16u;           // grid-stride loops take the rest
    return (unsigned)(b ? b : 1);
}

__global__ void relu_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, size_t count) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        y[i] = x[i] > 0.f ? x[i] : 0.f;
}

__global__ void relu_bwd_kernel(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ dx, size_t count) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        dx[i] = x[i] > 0.f ? dy[i] : 0.f;
}

// dx = (da + db) where y > 0, else 0: the two gradients that arrive at a residual block's output (from the next
// block's first convolution and from its shortcut), taken through the block's last ReLU in one pass.
// MASKED false: dx = da + db everywhere (y is not read).
template <int VEC, bool TWO, bool MASKED>
__global__ void __launch_bounds__(kThreads) relu_add_bwd_kernel(const float* __restrict__ y, const float* __restrict__ da,
                                                                const float* __restrict__ db, float* __restrict__ dx, size_t count) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) {
        if constexpr (VEC == 4) {
            float4 m = make_float4(1.f, 1.f, 1.f, 1.f);
            if constexpr (MASKED) m = reinterpret_cast<const float4*>(y)[i];
            float4 g = reinterpret_cast<const float4*>(da)[i];
            if constexpr (TWO) {
                const float4 h = reinterpret_cast<const float4*>(db)[i];
                g.x += h.x; g.y += h.y; g.z += h.z; g.w += h.w;
            }
            reinterpret_cast<float4*>(dx)[i] = make_float4(m.x > 0.f ? g.x : 0.f, m.y > 0.f ? g.y : 0.f, m.z > 0.f ? g.z : 0.f, m.w > 0.f ? g.w : 0.f);
        } else {
            float g = da[i];
            if constexpr (TWO) g += db[i];
            dx[i] = (!MASKED || y[i] > 0.f) ? g : 0.f;
        }
    }
}

// element (n, c, h, w) of a tensor in either layout
__device__ __forceinline__ size_t at(bool nhwc, int C, int H, int W, int n, int c, int h, int w) {
    return nhwc ? (((size_t)n * H + h) * W + w) * C + c : (((size_t)n * C + c) * H + h) * W + w;
}

// One thread per output element; the index of the first maximum in row-major window order goes to idx.
__global__ void maxpool2x2_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, uint8_t* __restrict__ idx, int N, int C,
                                      int H, int W, bool nhwc) {
    const int Ho = H / 2, Wo = W / 2;
    const size_t total = (size_t)N * C * Ho * Wo;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        int n, c, p, q;
        size_t t = o;
        if (nhwc) {
            c = (int)(t % C); t /= C;
            q = (int)(t % Wo); t /= Wo;
            p = (int)(t % Ho); n = (int)(t / Ho);
        } else {
            q = (int)(t % Wo); t /= Wo;
            p = (int)(t % Ho); t /= Ho;
            c = (int)(t % C); n = (int)(t / C);
        }
        float best = x[at(nhwc, C, H, W, n, c, 2 * p, 2 * q)];
        int bi = 0;
#pragma unroll
        for (int k = 1; k < 4; ++k) {
            const float v = x[at(nhwc, C, H, W, n, c, 2 * p + (k >> 1), 2 * q + (k & 1))];
            if (v > best) {                             // strictly greater: the first maximum wins ties
                best = v;
                bi = k;
            }
        }
        y[o] = best;
        idx[o] = (uint8_t)bi;
    }
}

__global__ void maxpool2x2_bwd_kernel(const float* __restrict__ dy, const uint8_t* __restrict__ idx, float* __restrict__ dx, int N,
                                      int C, int H, int W, bool nhwc) {
    const int Ho = H / 2, Wo = W / 2;
    const size_t total = (size_t)N * C * Ho * Wo;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        int n, c, p, q;
        size_t t = o;
        if (nhwc) {
            c = (int)(t % C); t /= C;
            q = (int)(t % Wo); t /= Wo;
            p = (int)(t % Ho); n = (int)(t / Ho);
        } else {
            q = (int)(t % Wo); t /= Wo;
            p = (int)(t % Ho); t /= Ho;
            c = (int)(t % C); n = (int)(t / C);
        }
        const int bi = idx[o];
        const float g = dy[o];
#pragma unroll
        for (int k = 0; k < 4; ++k) dx[at(nhwc, C, H, W, n, c, 2 * p + (k >> 1), 2 * q + (k & 1))] = k == bi ? g : 0.f;
    }
}

// One wave per (n, c): pixels summed in strides of 64, lanes combined by a fixed shuffle tree.
// Max pool, window K x K, any stride and pad (pad < K): one thread per output element; padding taps never win;
// idx is the tap (row * K + column) of the first maximum in row-major window order.
__global__ void __launch_bounds__(kThreads) maxpool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, uint8_t* __restrict__ idx,
                                                               int N, int C, int H, int W, int K, int stride, int pad, int Ho, int Wo, bool nhwc) {
    const size_t total = (size_t)N * C * Ho * Wo;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        int n, c, p, q;
        size_t t = o;
        if (nhwc) {
            c = (int)(t % C); t /= C;
            q = (int)(t % Wo); t /= Wo;
            p = (int)(t % Ho); n = (int)(t / Ho);
        } else {
            q = (int)(t % Wo); t /= Wo;
            p = (int)(t % Ho); t /= Ho;
            c = (int)(t % C); n = (int)(t / C);
        }
        float best = 0.f;
        int bi = -1;
        for (int r = 0; r < K; ++r) {
            const int ih = p * stride - pad + r;
            if (ih < 0 || ih >= H) continue;
            for (int s2 = 0; s2 < K; ++s2) {
                const int iw = q * stride - pad + s2;
                if (iw < 0 || iw >= W) continue;
                const float v = x[at(nhwc, C, H, W, n, c, ih, iw)];
                if (bi < 0 || v > best) {               // strictly greater: the first maximum wins ties
                    best = v;
                    bi = r * K + s2;
                }
            }
        }
        y[o] = best;
        idx[o] = (uint8_t)bi;
    }
}

// One thread per input element gathers from the (at most ceil(K/stride)^2) windows that contain it, in output
// order: no atomics, the sum order is fixed.
__global__ void __launch_bounds__(kThreads) maxpool_bwd_kernel(const float* __restrict__ dy, const uint8_t* __restrict__ idx, float* __restrict__ dx,
                                                               int N, int C, int H, int W, int K, int stride, int pad, int Ho, int Wo, bool nhwc) {
    const size_t total = (size_t)N * C * H * W;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        int n, c, h, w;
        size_t t = o;
        if (nhwc) {
            c = (int)(t % C); t /= C;
            w = (int)(t % W); t /= W;
            h = (int)(t % H); n = (int)(t / H);
        } else {
            w = (int)(t % W); t /= W;
            h = (int)(t % H); t /= H;
            c = (int)(t % C); n = (int)(t / C);
        }
        // outputs p with p*stride - pad <= h <= p*stride - pad + K - 1
        const int hp = h + pad, wp = w + pad;
        int p0 = hp - K + 1 <= 0 ? 0 : (hp - K + stride) / stride;
        int q0 = wp - K + 1 <= 0 ? 0 : (wp - K + stride) / stride;
        int p1 = hp / stride, q1 = wp / stride;
        if (p1 > Ho - 1) p1 = Ho - 1;
        if (q1 > Wo - 1) q1 = Wo - 1;
        float acc = 0.f;
        for (int p = p0; p <= p1; ++p)
            for (int q = q0; q <= q1; ++q) {
                const int tap = (hp - p * stride) * K + (wp - q * stride);
                const size_t oo = at(nhwc, C, Ho, Wo, n, c, p, q);
                if (idx[oo] == (uint8_t)tap) acc += dy[oo];
            }
        dx[o] = acc;
    }
}

// The same two kernels for NHWC with the channel count a multiple of four: a thread owns four neighbouring
// channels of one pixel (16-byte accesses, four index bytes as one word).
__global__ void __launch_bounds__(kThreads) maxpool_fwd_nhwc4_kernel(const float* __restrict__ x, float* __restrict__ y, uint8_t* __restrict__ idx,
                                                                     int N, int C4, int H, int W, int K, int stride, int pad, int Ho, int Wo) {
    const size_t total = (size_t)N * Ho * Wo * C4;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        size_t t = o;
        const int c4 = (int)(t % C4); t /= C4;
        const int q = (int)(t % Wo); t /= Wo;
        const int p = (int)(t % Ho);
        const int n = (int)(t / Ho);
        float best[4] = {0.f, 0.f, 0.f, 0.f};
        int bi[4] = {-1, -1, -1, -1};
        for (int r = 0; r < K; ++r) {
            const int ih = p * stride - pad + r;
            if (ih < 0 || ih >= H) continue;
            for (int s2 = 0; s2 < K; ++s2) {
                const int iw = q * stride - pad + s2;
                if (iw < 0 || iw >= W) continue;
                const float4 v4 = reinterpret_cast<const float4*>(x)[(((size_t)n * H + ih) * W + iw) * C4 + c4];
                const float v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (bi[e] < 0 || v[e] > best[e]) {
                        best[e] = v[e];
                        bi[e] = r * K + s2;
                    }
            }
        }
        reinterpret_cast<float4*>(y)[o] = make_float4(best[0], best[1], best[2], best[3]);
        reinterpret_cast<uchar4*>(idx)[o] = make_uchar4((uint8_t)bi[0], (uint8_t)bi[1], (uint8_t)bi[2], (uint8_t)bi[3]);
    }
}

__global__ void __launch_bounds__(kThreads) maxpool_bwd_nhwc4_kernel(const float* __restrict__ dy, const uint8_t* __restrict__ idx, float* __restrict__ dx,
                                                                     int N, int C4, int H, int W, int K, int stride, int pad, int Ho, int Wo) {
    const size_t total = (size_t)N * H * W * C4;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        size_t t = o;
        const int c4 = (int)(t % C4); t /= C4;
        const int w = (int)(t % W); t /= W;
        const int h = (int)(t % H);
        const int n = (int)(t / H);
        const int hp = h + pad, wp = w + pad;
        const int p0 = hp - K + 1 <= 0 ? 0 : (hp - K + stride) / stride;
        const int q0 = wp - K + 1 <= 0 ? 0 : (wp - K + stride) / stride;
        int p1 = hp / stride, q1 = wp / stride;
        if (p1 > Ho - 1) p1 = Ho - 1;
        if (q1 > Wo - 1) q1 = Wo - 1;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int p = p0; p <= p1; ++p)
            for (int q = q0; q <= q1; ++q) {
                const uint8_t tap = (uint8_t)((hp - p * stride) * K + (wp - q * stride));
                const size_t oo = (((size_t)n * Ho + p) * Wo + q) * C4 + c4;
                const uchar4 i4 = reinterpret_cast<const uchar4*>(idx)[oo];
                const float4 g = reinterpret_cast<const float4*>(dy)[oo];
                if (i4.x == tap) acc[0] += g.x;
                if (i4.y == tap) acc[1] += g.y;
                if (i4.z == tap) acc[2] += g.z;
                if (i4.w == tap) acc[3] += g.w;
            }
        reinterpret_cast<float4*>(dx)[o] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    }
}

__global__ void global_avgpool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int N, int C, int H, int W, bool nhwc) {
    const int lane = threadIdx.x & 63;
    const size_t pair = (size_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (pair >= (size_t)N * C) return;
    const int n = (int)(pair / C), c = (int)(pair % C);
    const int hw = H * W;
    float s = 0.f;
    for (int i = lane; i < hw; i += 64) s += x[at(nhwc, C, H, W, n, c, i / W, i % W)];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) y[pair] = s / (float)hw;
}

// NHWC with the channel count a multiple of four: a thread owns four neighbouring channels of one image and adds its pixels
// in order (16-byte loads, neighbouring threads on neighbouring channels).
__global__ void __launch_bounds__(kThreads) global_avgpool_fwd_nhwc4_kernel(const float4* __restrict__ x, float4* __restrict__ y, int N,
                                                                            int C4, int HW) {
    const size_t total = (size_t)N * C4;
    const float inv = 1.f / (float)HW;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const size_t n = o / C4;
        const int c4 = (int)(o % C4);
        const float4* src = x + n * HW * C4 + c4;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 7
        for (int i = 0; i < HW; ++i) {
            const float4 v = src[(size_t)i * C4];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        y[o] = make_float4(s.x * inv, s.y * inv, s.z * inv, s.w * inv);
    }
}

__global__ void global_avgpool_bwd_kernel(const float* __restrict__ dy, float* __restrict__ dx, int N, int C, int H, int W, bool nhwc) {
    const size_t total = (size_t)N * C * H * W;
    const float inv = 1.f / (float)(H * W);
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        size_t nc;
        if (nhwc) {
            const int c = (int)(i % C);
            nc = (i / ((size_t)C * H * W)) * C + c;
        } else {
            nc = i / ((size_t)H * W);
        }
        dx[i] = dy[nc] * inv;
    }
}

__global__ void bias_add_kernel(float* __restrict__ y, const float* __restrict__ b, size_t rows, int K) {
    const size_t total = rows * K;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) y[i] += b[i % K];
}

// A block owns 64 columns; its four waves take every fourth row each, four rows in flight per wave, and the sixteen running
// sums of a column are combined in a fixed order.
__global__ void __launch_bounds__(kThreads) bias_grad_kernel(const float* __restrict__ dy, float* __restrict__ db, size_t rows, int K) {
    constexpr int kWaves = kThreads / 64;
    __shared__ float part[kWaves][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + lane;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    if (k < K) {
        size_t r = wave;
        for (; r + 3 * kWaves < rows; r += 4 * kWaves) {
#pragma unroll
            for (int u = 0; u < 4; ++u) s[u] += dy[(r + (size_t)u * kWaves) * K + k];
        }
        for (; r < rows; r += kWaves) s[0] += dy[r * K + k];
    }
    part[wave][lane] = (s[0] + s[1]) + (s[2] + s[3]);
    __syncthreads();
    if (wave == 0 && k < K) db[k] = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
}

// One wave per row: softmax, the row's -log p[label], and (softmax - onehot) / N.  row_loss[n] is reduced by
// the second kernel in index order.
__global__ void softmax_xent_rows_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels, float* __restrict__ row_loss,
                                         float* __restrict__ dlogits, int N, int K) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (n >= N) return;
    const float* z = logits + (size_t)n * K;
    float m = -3.402823466e38f;
    for (int k = lane; k < K; k += 64) m = fmaxf(m, z[k]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    float s = 0.f;
    for (int k = lane; k < K; k += 64) s += expf(z[k] - m);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    const int lab = min(max(labels[n], 0), K - 1);   // (a label outside [0, K) is the caller's error; stay inside the row)
    const float inv_n = 1.f / (float)N;
    for (int k = lane; k < K; k += 64) {
        const float p = expf(z[k] - m) / s;
        dlogits[(size_t)n * K + k] = (p - (k == lab ? 1.f : 0.f)) * inv_n;
    }
    if (lane == 0) row_loss[n] = -(z[lab] - m - logf(s));
}

__global__ void mean_kernel(const float* __restrict__ v, float* __restrict__ out, int N) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    double s = 0.0;
    for (int i = 0; i < N; ++i) s += (double)v[i];
    out[0] = (float)(s / (double)N);
}

inline bool bad_layout(lc_layout l) { return l != LC_NCHW && l != LC_NHWC; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3) != 0; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

extern "C" lc_status relu_fwd(const float* x, float* y, size_t count, void* hip_stream) {
    if (!x || !y) return LC_ERR_NULL;
    if (misaligned(x) || misaligned(y)) return LC_ERR_ALIGN;
    if (count == 0) return LC_OK;
    lc_begin_call();
    hipLaunchKernelGGL(relu_fwd_kernel, dim3(blocks_for(count)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), x, y, count);
    return lc_end_call();
}

extern "C" lc_status relu_bwd(const float* x, const float* dy, float* dx, size_t count, void* hip_stream) {
    if (!x || !dy || !dx) return LC_ERR_NULL;
    if (misaligned(x) || misaligned(dy) || misaligned(dx)) return LC_ERR_ALIGN;
    if (count == 0) return LC_OK;
    lc_begin_call();
    hipLaunchKernelGGL(relu_bwd_kernel, dim3(blocks_for(count)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), x, dy, dx,
                       count);
    return lc_end_call();
}

extern "C" lc_status maxpool2x2_fwd(const float* x, float* y, uint8_t* idx, int n, int c, int h, int w, lc_layout layout,
                                    void* hip_stream) {
    if (!x || !y || !idx) return LC_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || (h & 1) || (w & 1)) return LC_ERR_SHAPE;
    if (bad_layout(layout)) return LC_ERR_UNSUPPORTED;
    if (misaligned(x) || misaligned(y)) return LC_ERR_ALIGN;
    lc_begin_call();
    const size_t total = (size_t)n * c * (h / 2) * (w / 2);
    hipLaunchKernelGGL(maxpool2x2_fwd_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), x, y,
                       idx, n, c, h, w, layout == LC_NHWC);
    return lc_end_call();
}

extern "C" lc_status maxpool2x2_bwd(const float* dy, const uint8_t* idx, float* dx, int n, int c, int h, int w, lc_layout layout,
                                    void* hip_stream) {
    if (!dy || !idx || !dx) return LC_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || (h & 1) || (w & 1)) return LC_ERR_SHAPE;
    if (bad_layout(layout)) return LC_ERR_UNSUPPORTED;
    if (misaligned(dy) || misaligned(dx)) return LC_ERR_ALIGN;
    lc_begin_call();
    const size_t total = (size_t)n * c * (h / 2) * (w / 2);
    hipLaunchKernelGGL(maxpool2x2_bwd_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), dy,
                       idx, dx, n, c, h, w, layout == LC_NHWC);
    return lc_end_call();
}

extern "C" lc_status relu_add_bwd(const float* y, const float* da, const float* db, float* dx, size_t count, void* hip_stream) {
    if (!da || !dx || (!y && !db)) return LC_ERR_NULL;
    if (count == 0) return LC_OK;
    if (misaligned(y) || misaligned(da) || misaligned(db) || misaligned(dx)) return LC_ERR_ALIGN;
    lc_begin_call();
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    const bool vec = count % 4 == 0 && al16(y) && al16(da) && al16(db) && al16(dx);
    const size_t items = vec ? count / 4 : count;
    const dim3 grid(blocks_for(items));
#define LC_RAB(VEC, TWO, MASKED) \
    hipLaunchKernelGGL((relu_add_bwd_kernel<VEC, TWO, MASKED>), grid, dim3(kThreads), 0, stream, y, da, db, dx, items)
    if (vec) {
        if (!y) LC_RAB(4, true, false);
        else if (db) LC_RAB(4, true, true);
        else LC_RAB(4, false, true);
    } else {
        if (!y) LC_RAB(1, true, false);
        else if (db) LC_RAB(1, true, true);
        else LC_RAB(1, false, true);
    }
#undef LC_RAB
    return lc_end_call();
}

namespace {
struct PoolF32 {                                // four fp32 channels per thread
    using T = float;
    static constexpr int VEC = 4;
    static __device__ void load(const float* p, float (&v)[4]) {
        const float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    static __device__ void store(float* p, const float (&v)[4]) { *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]); }
};

// output size of a pool; false when the arguments make no sense
bool pool_shape(int n, int c, int h, int w, int window, int stride, int pad, int* ho, int* wo) {
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || window < 1 || window > 15 || stride < 1 || pad < 0 || pad >= window) return false;
    if (h + 2 * pad < window || w + 2 * pad < window) return false;
    *ho = (h + 2 * pad - window) / stride + 1;
    *wo = (w + 2 * pad - window) / stride + 1;
    // the last window must start inside the image, or it would see padding only
    return (*ho - 1) * stride - pad < h && (*wo - 1) * stride - pad < w;
}
}  // namespace

extern "C" lc_status maxpool_fwd(const float* x, float* y, uint8_t* idx, int n, int c, int h, int w, int window, int stride, int pad,
                                 lc_layout layout, void* hip_stream) {
    if (!x || !y || !idx) return LC_ERR_NULL;
    int ho, wo;
    if (!pool_shape(n, c, h, w, window, stride, pad, &ho, &wo)) return LC_ERR_SHAPE;
    if (bad_layout(layout)) return LC_ERR_UNSUPPORTED;
    if (misaligned(x) || misaligned(y)) return LC_ERR_ALIGN;
    lc_begin_call();
    const size_t total = (size_t)n * c * ho * wo;
    if (layout == LC_NHWC && c % 4 == 0 && aligned16(x) && aligned16(y) && (reinterpret_cast<uintptr_t>(idx) & 3) == 0)
        hipLaunchKernelGGL(maxpool_fwd_nhwc4_kernel, dim3(blocks_for(total / 4)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                           x, y, idx, n, c / 4, h, w, window, stride, pad, ho, wo);
    else
        hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), x, y, idx,
                           n, c, h, w, window, stride, pad, ho, wo, layout == LC_NHWC);
    return lc_end_call();
}

extern "C" lc_status maxpool_bwd(const float* dy, const uint8_t* idx, float* dx, int n, int c, int h, int w, int window, int stride,
                                 int pad, lc_layout layout, void* hip_stream) {
    if (!dy || !idx || !dx) return LC_ERR_NULL;
    int ho, wo;
    if (!pool_shape(n, c, h, w, window, stride, pad, &ho, &wo)) return LC_ERR_SHAPE;
    if (bad_layout(layout)) return LC_ERR_UNSUPPORTED;
    if (misaligned(dy) || misaligned(dx)) return LC_ERR_ALIGN;
    lc_begin_call();
    const size_t total = (size_t)n * c * h * w;
    const bool vec4 = layout == LC_NHWC && c % 4 == 0 && aligned16(dy) && aligned16(dx) && (reinterpret_cast<uintptr_t>(idx) & 3) == 0;
    if (vec4 && window == 3 && stride == 2 && pad == 1)
        hipLaunchKernelGGL(maxpool_bwd_3x3s2_kernel<PoolF32>, dim3(blocks_for((size_t)n * ((h + 1) / 2) * ((w + 1) / 2) * (c / 4))),
                           dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), dy, idx, dx, n, c / 4, h, w, ho, wo);
    else if (vec4)
        hipLaunchKernelGGL(maxpool_bwd_nhwc4_kernel, dim3(blocks_for(total / 4)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                           dy, idx, dx, n, c / 4, h, w, window, stride, pad, ho, wo);
    else
        hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), dy, idx,
                           dx, n, c, h, w, window, stride, pad, ho, wo, layout == LC_NHWC);
    return lc_end_call();
}

extern "C" lc_status global_avgpool_fwd(const float* x, float* y, int n, int c, int h, int w, lc_layout layout, void* hip_stream) {
    if (!x || !y) return LC_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return LC_ERR_SHAPE;
    if (bad_layout(layout)) return LC_ERR_UNSUPPORTED;
    if (misaligned(x) || misaligned(y)) return LC_ERR_ALIGN;
    lc_begin_call();
    const size_t pairs = (size_t)n * c;
    if (layout == LC_NHWC && c % 4 == 0 && aligned16(x) && aligned16(y) && (long long)h * w <= 0x7fffffffLL) {
        hipLaunchKernelGGL(global_avgpool_fwd_nhwc4_kernel, dim3(blocks_for(pairs / 4)), dim3(kThreads), 0,
                           static_cast<hipStream_t>(hip_stream), reinterpret_cast<const float4*>(x), reinterpret_cast<float4*>(y), n, c / 4,
                           h * w);
        return lc_end_call();
    }
    const size_t blocks = (pairs + kThreads / 64 - 1) / (kThreads / 64);
    if (blocks > 0x7fffffffull) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(global_avgpool_fwd_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), x, y,
                       n, c, h, w, layout == LC_NHWC);
    return lc_end_call();
}

extern "C" lc_status global_avgpool_bwd(const float* dy, float* dx, int n, int c, int h, int w, lc_layout layout, void* hip_stream) {
    if (!dy || !dx) return LC_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return LC_ERR_SHAPE;
    if (bad_layout(layout)) return LC_ERR_UNSUPPORTED;
    if (misaligned(dy) || misaligned(dx)) return LC_ERR_ALIGN;
    lc_begin_call();
    hipLaunchKernelGGL(global_avgpool_bwd_kernel, dim3(blocks_for((size_t)n * c * h * w)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), dy, dx, n, c, h, w, layout == LC_NHWC);
    return lc_end_call();
}

extern "C" lc_status bias_add(float* y, const float* b, size_t rows, int k, void* hip_stream) {
    if (!y || !b) return LC_ERR_NULL;
    if (k <= 0) return LC_ERR_SHAPE;
    if (misaligned(y) || misaligned(b)) return LC_ERR_ALIGN;
    if (rows == 0) return LC_OK;
    lc_begin_call();
    hipLaunchKernelGGL(bias_add_kernel, dim3(blocks_for(rows * k)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), y, b, rows, k);
    return lc_end_call();
}

extern "C" lc_status bias_grad(const float* dy, float* db, size_t rows, int k, void* hip_stream) {
    if (!dy || !db) return LC_ERR_NULL;
    if (k <= 0) return LC_ERR_SHAPE;
    if (misaligned(dy) || misaligned(db)) return LC_ERR_ALIGN;
    lc_begin_call();
    hipLaunchKernelGGL(bias_grad_kernel, dim3((unsigned)((k + 63) / 64)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), dy, db, rows, k);
    return lc_end_call();
}

extern "C" lc_status softmax_xent(const float* logits, const int32_t* labels, float* loss, float* dlogits, float* row_scratch, int n,
                                  int k, void* hip_stream) {
    if (!logits || !labels || !loss || !dlogits || !row_scratch) return LC_ERR_NULL;
    if (n <= 0 || k <= 0) return LC_ERR_SHAPE;
    if (misaligned(logits) || misaligned(labels) || misaligned(loss) || misaligned(dlogits) || misaligned(row_scratch)) return LC_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lc_begin_call();
    hipLaunchKernelGGL(softmax_xent_rows_kernel, dim3((unsigned)((n + kThreads / 64 - 1) / (kThreads / 64))), dim3(kThreads), 0, stream,
                       logits, labels, row_scratch, dlogits, n, k);
    hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(64), 0, stream, row_scratch, loss, n);
    return lc_end_call();
}
