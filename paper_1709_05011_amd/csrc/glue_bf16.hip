// The glue layers a bf16 training step needs between its convolutions (mixed-precision training as the paper's
// fastest runs use it, "State-of-the-art results"): overlapping max pooling, the gradient that meets at a residual
// block's output, and global average pooling, on activations stored as bf16 in NHWC with the channel count a
// multiple of eight.  Arithmetic is fp32; a result that is stored as bf16 is rounded once, to nearest even.
// A thread owns eight neighbouring channels of one pixel: one 16-byte access per tensor.
// The `_t` entry points take the storage type as an argument and hand fp32 to the fp32 kernels of glue.hip.
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

__device__ __forceinline__ void load8(const uint16_t* p, float (&v)[8]) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

__device__ __forceinline__ void store8(uint16_t* p, const float (&v)[8]) {
    unsigned w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = lc_bf16x2_rne(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}

struct PoolBF16 {                               // eight bf16 channels per thread
    using T = uint16_t;
    static constexpr int VEC = 8;
    static __device__ void load(const uint16_t* p, float (&v)[8]) { load8(p, v); }
    static __device__ void store(uint16_t* p, const float (&v)[8]) { store8(p, v); }
};

// dx = round(da + db) where y > 0, else 0 (MASKED false: everywhere; TWO false: da alone)
template <bool TWO, bool MASKED>
__global__ void __launch_bounds__(kThreads) relu_add_bwd_bf16_kernel(const uint16_t* __restrict__ y, const uint16_t* __restrict__ da,
                                                                     const uint16_t* __restrict__ db, uint16_t* __restrict__ dx,
                                                                     size_t groups) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < groups; i += (size_t)gridDim.x * blockDim.x) {
        float g[8], h[8], m[8];
        load8(da + i * 8, g);
        if constexpr (TWO) {
            load8(db + i * 8, h);
#pragma unroll
            for (int e = 0; e < 8; ++e) g[e] += h[e];
        }
        if constexpr (MASKED) {
            load8(y + i * 8, m);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (!(m[e] > 0.f)) g[e] = 0.f;
        }
        store8(dx + i * 8, g);
    }
}

// the first maximum in row-major window order; its index within the window goes to idx (one byte per element)
__global__ void __launch_bounds__(kThreads) maxpool_fwd_bf16_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ y,
                                                                    uint8_t* __restrict__ idx, int N, int C8, int H, int W, int K,
                                                                    int stride, int pad, int Ho, int Wo) {
    const size_t total = (size_t)N * Ho * Wo * C8;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        size_t t = o;
        const int c8 = (int)(t % C8); t /= C8;
        const int q = (int)(t % Wo); t /= Wo;
        const int p = (int)(t % Ho);
        const int n = (int)(t / Ho);
        float best[8];
        int bi[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            best[e] = 0.f;
            bi[e] = -1;
        }
        for (int r = 0; r < K; ++r) {
            const int ih = p * stride - pad + r;
            if (ih < 0 || ih >= H) continue;
            for (int s2 = 0; s2 < K; ++s2) {
                const int iw = q * stride - pad + s2;
                if (iw < 0 || iw >= W) continue;
                float v[8];
                load8(x + ((((size_t)n * H + ih) * W + iw) * C8 + c8) * 8, v);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (bi[e] < 0 || v[e] > best[e]) {
                        best[e] = v[e];
                        bi[e] = r * K + s2;
                    }
            }
        }
        store8(y + o * 8, best);              // exact: the values are bf16 already
        unsigned lo = 0, hi = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            lo |= (unsigned)(uint8_t)bi[e] << (8 * e);
            hi |= (unsigned)(uint8_t)bi[4 + e] << (8 * e);
        }
        reinterpret_cast<uint2*>(idx)[o] = make_uint2(lo, hi);
    }
}

// dx(pixel) = round(sum of dy over the windows whose recorded maximum is that pixel), in window order
__global__ void __launch_bounds__(kThreads) maxpool_bwd_bf16_kernel(const uint16_t* __restrict__ dy, const uint8_t* __restrict__ idx,
                                                                    uint16_t* __restrict__ dx, int N, int C8, int H, int W, int K,
                                                                    int stride, int pad, int Ho, int Wo) {
    const size_t total = (size_t)N * H * W * C8;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        size_t t = o;
        const int c8 = (int)(t % C8); t /= C8;
        const int w = (int)(t % W); t /= W;
        const int h = (int)(t % H);
        const int n = (int)(t / H);
        const int hp = h + pad, wp = w + pad;
        const int p0 = hp - K + 1 <= 0 ? 0 : (hp - K + stride) / stride;
        const int q0 = wp - K + 1 <= 0 ? 0 : (wp - K + stride) / stride;
        int p1 = hp / stride, q1 = wp / stride;
        if (p1 > Ho - 1) p1 = Ho - 1;
        if (q1 > Wo - 1) q1 = Wo - 1;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        for (int p = p0; p <= p1; ++p)
            for (int q = q0; q <= q1; ++q) {
                const unsigned tap = (unsigned)((hp - p * stride) * K + (wp - q * stride));
                const size_t oo = (((size_t)n * Ho + p) * Wo + q) * C8 + c8;
                const uint2 i8 = reinterpret_cast<const uint2*>(idx)[oo];
                float g[8];
                load8(dy + oo * 8, g);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const unsigned which = ((e < 4 ? i8.x : i8.y) >> (8 * (e & 3))) & 0xffu;
                    if (which == tap) acc[e] += g[e];
                }
            }
        store8(dx + o * 8, acc);
    }
}

// y[n][c] (fp32) = mean over the pixels of x[n][.][c] (bf16), summed in pixel order
__global__ void __launch_bounds__(kThreads) global_avgpool_fwd_bf16_kernel(const uint16_t* __restrict__ x, float* __restrict__ y, int N,
                                                                          int C8, int HW) {
    const size_t total = (size_t)N * C8;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const size_t n = o / C8;
        const int c8 = (int)(o % C8);
        float s[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] = 0.f;
        for (int i = 0; i < HW; ++i) {
            float v[8];
            load8(x + ((n * HW + i) * C8 + c8) * 8, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] += v[e];
        }
        const float hw = (float)HW;
        reinterpret_cast<float4*>(y)[o * 2] = make_float4(s[0] / hw, s[1] / hw, s[2] / hw, s[3] / hw);
        reinterpret_cast<float4*>(y)[o * 2 + 1] = make_float4(s[4] / hw, s[5] / hw, s[6] / hw, s[7] / hw);
    }
}

// dx[n][.][c] (bf16) = round(dy[n][c] / pixels) (dy fp32)
__global__ void __launch_bounds__(kThreads) global_avgpool_bwd_bf16_kernel(const float* __restrict__ dy, uint16_t* __restrict__ dx, int N,
                                                                          int C8, int HW) {
    const size_t total = (size_t)N * HW * C8;
    const float inv = 1.f / (float)HW;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const int c8 = (int)(o % C8);
        const size_t n = o / ((size_t)HW * C8);
        const float4 a = reinterpret_cast<const float4*>(dy)[(n * C8 + c8) * 2], b = reinterpret_cast<const float4*>(dy)[(n * C8 + c8) * 2 + 1];
        const float v[8] = {a.x * inv, a.y * inv, a.z * inv, a.w * inv, b.x * inv, b.y * inv, b.z * inv, b.w * inv};
        store8(dx + o * 8, v);
    }
}

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool al8(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 7) == 0; }

// output size of a pool; false when the arguments make no sense (the rule maxpool_fwd applies)
bool pool_shape(int n, int c, int h, int w, int window, int stride, int pad, int* ho, int* wo) {
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || window < 1 || window > 15 || stride < 1 || pad < 0 || pad >= window) return false;
    if (h + 2 * pad < window || w + 2 * pad < window) return false;
    *ho = (h + 2 * pad - window) / stride + 1;
    *wo = (w + 2 * pad - window) / stride + 1;
    return (*ho - 1) * stride - pad < h && (*wo - 1) * stride - pad < w;
}

}  // namespace

extern "C" lc_status relu_add_bwd_t(lc_dtype dtype, const void* y, const void* da, const void* db, void* dx, size_t count,
                                    void* hip_stream) {
    if (dtype == LC_F32)
        return relu_add_bwd(static_cast<const float*>(y), static_cast<const float*>(da), static_cast<const float*>(db),
                            static_cast<float*>(dx), count, hip_stream);
    if (dtype != LC_BF16) return LC_ERR_UNSUPPORTED;
    if (!da || !dx || (!y && !db)) return LC_ERR_NULL;
    if (count == 0) return LC_OK;
    if (count % 8) return LC_ERR_UNSUPPORTED;
    if (!al16(y) || !al16(da) || !al16(db) || !al16(dx)) return LC_ERR_ALIGN;
    lc_begin_call();
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t groups = count / 8;
    const dim3 grid(blocks_for(groups));
    const uint16_t *yy = static_cast<const uint16_t*>(y), *a = static_cast<const uint16_t*>(da), *b = static_cast<const uint16_t*>(db);
    uint16_t* out = static_cast<uint16_t*>(dx);
    if (!y)
        hipLaunchKernelGGL((relu_add_bwd_bf16_kernel<true, false>), grid, dim3(kThreads), 0, stream, yy, a, b, out, groups);
    else if (db)
        hipLaunchKernelGGL((relu_add_bwd_bf16_kernel<true, true>), grid, dim3(kThreads), 0, stream, yy, a, b, out, groups);
    else
        hipLaunchKernelGGL((relu_add_bwd_bf16_kernel<false, true>), grid, dim3(kThreads), 0, stream, yy, a, b, out, groups);
    return lc_end_call();
}

extern "C" lc_status maxpool_fwd_t(lc_dtype dtype, const void* x, void* y, uint8_t* idx, int n, int c, int h, int w, int window,
                                   int stride, int pad, lc_layout layout, void* hip_stream) {
    if (dtype == LC_F32)
        return maxpool_fwd(static_cast<const float*>(x), static_cast<float*>(y), idx, n, c, h, w, window, stride, pad, layout, hip_stream);
    if (dtype != LC_BF16) return LC_ERR_UNSUPPORTED;
    if (!x || !y || !idx) return LC_ERR_NULL;
    int ho, wo;
    if (!pool_shape(n, c, h, w, window, stride, pad, &ho, &wo)) return LC_ERR_SHAPE;
    if (layout != LC_NHWC || c % 8) return LC_ERR_UNSUPPORTED;
    if (!al16(x) || !al16(y) || !al8(idx)) return LC_ERR_ALIGN;
    lc_begin_call();
    const size_t total = (size_t)n * ho * wo * (c / 8);
    hipLaunchKernelGGL(maxpool_fwd_bf16_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint16_t*>(x), static_cast<uint16_t*>(y), idx, n, c / 8, h, w, window, stride, pad, ho, wo);
    return lc_end_call();
}

extern "C" lc_status maxpool_bwd_t(lc_dtype dtype, const void* dy, const uint8_t* idx, void* dx, int n, int c, int h, int w, int window,
                                   int stride, int pad, lc_layout layout, void* hip_stream) {
    if (dtype == LC_F32)
        return maxpool_bwd(static_cast<const float*>(dy), idx, static_cast<float*>(dx), n, c, h, w, window, stride, pad, layout, hip_stream);
    if (dtype != LC_BF16) return LC_ERR_UNSUPPORTED;
    if (!dy || !idx || !dx) return LC_ERR_NULL;
    int ho, wo;
    if (!pool_shape(n, c, h, w, window, stride, pad, &ho, &wo)) return LC_ERR_SHAPE;
    if (layout != LC_NHWC || c % 8) return LC_ERR_UNSUPPORTED;
    if (!al16(dy) || !al16(dx) || !al8(idx)) return LC_ERR_ALIGN;
    lc_begin_call();
    const size_t total = (size_t)n * h * w * (c / 8);
    if (window == 3 && stride == 2 && pad == 1)
        hipLaunchKernelGGL(maxpool_bwd_3x3s2_kernel<PoolBF16>, dim3(blocks_for((size_t)n * ((h + 1) / 2) * ((w + 1) / 2) * (c / 8))),
                           dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), static_cast<const uint16_t*>(dy), idx,
                           static_cast<uint16_t*>(dx), n, c / 8, h, w, ho, wo);
    else
        hipLaunchKernelGGL(maxpool_bwd_bf16_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                           static_cast<const uint16_t*>(dy), idx, static_cast<uint16_t*>(dx), n, c / 8, h, w, window, stride, pad, ho, wo);
    return lc_end_call();
}

extern "C" lc_status global_avgpool_fwd_t(lc_dtype dtype, const void* x, float* y, int n, int c, int h, int w, lc_layout layout,
                                          void* hip_stream) {
    if (dtype == LC_F32) return global_avgpool_fwd(static_cast<const float*>(x), y, n, c, h, w, layout, hip_stream);
    if (dtype != LC_BF16) return LC_ERR_UNSUPPORTED;
    if (!x || !y) return LC_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || (long long)h * w > 0x7fffffffLL) return LC_ERR_SHAPE;
    if (layout != LC_NHWC || c % 8) return LC_ERR_UNSUPPORTED;
    if (!al16(x) || !al16(y)) return LC_ERR_ALIGN;
    lc_begin_call();
    hipLaunchKernelGGL(global_avgpool_fwd_bf16_kernel, dim3(blocks_for((size_t)n * (c / 8))), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const uint16_t*>(x), y, n, c / 8, h * w);
    return lc_end_call();
}

extern "C" lc_status global_avgpool_bwd_t(lc_dtype dtype, const float* dy, void* dx, int n, int c, int h, int w, lc_layout layout,
                                          void* hip_stream) {
    if (dtype == LC_F32) return global_avgpool_bwd(dy, static_cast<float*>(dx), n, c, h, w, layout, hip_stream);
    if (dtype != LC_BF16) return LC_ERR_UNSUPPORTED;
    if (!dy || !dx) return LC_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || (long long)h * w > 0x7fffffffLL) return LC_ERR_SHAPE;
    if (layout != LC_NHWC || c % 8) return LC_ERR_UNSUPPORTED;
    if (!al16(dy) || !al16(dx)) return LC_ERR_ALIGN;
    lc_begin_call();
    hipLaunchKernelGGL(global_avgpool_bwd_bf16_kernel, dim3(blocks_for((size_t)n * h * w * (c / 8))), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), dy, static_cast<uint16_t*>(dx), n, c / 8, h * w);
    return lc_end_call();
}
