// Data-movement helpers around the convolution kernels: fills, NCHW <-> NHWC transposes, filter
// re-ordering for backward-data, channel padding and the fixed-order sum of split partials.
// All of them are plain bandwidth-bound kernels; none is on the NHWC fast path except the filter
// re-ordering (a few MB) and the split reduction.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.h"

namespace {

__global__ void fill_f32_kernel(float* __restrict__ dst, float value, size_t count) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = value;
}

__global__ void zero16_kernel(uint4* __restrict__ dst, size_t count) {
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = z;
}

inline unsigned grid_for(size_t count, int threads) {
    size_t g = (count + threads - 1) / threads;
    if (g > 65535 * 16) g = 65535 * 16;
    return (unsigned)(g ? g : 1);
}

// dst[n][x][y] = src[n][y][x] for a batch of (rows x cols) matrices, through a 32x33 LDS tile.
template <typename T>
__global__ void __launch_bounds__(256) transpose_kernel(const T* __restrict__ src, T* __restrict__ dst, int rows, int cols) {
    __shared__ T tile[32][33];
    const size_t img = (size_t)blockIdx.z * rows * cols;
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8) {
        const int r = r0 + i, c = c0 + tx;
        if (r < rows && c < cols) tile[i][tx] = src[img + (size_t)r * cols + c];
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int c = c0 + i, r = r0 + tx;
        if (r < rows && c < cols) dst[img + (size_t)c * rows + r] = tile[tx][i];
    }
}

template <typename T>
void transpose_batched(const void* src, void* dst, int batch, int rows, int cols, hipStream_t stream) {
    // grid.z is limited to 65535: walk larger batches in slabs
    for (int b0 = 0; b0 < batch; b0 += 65535) {
        const int nb = (batch - b0) < 65535 ? (batch - b0) : 65535;
        const size_t off = (size_t)b0 * rows * cols;
        hipLaunchKernelGGL(transpose_kernel<T>, dim3((cols + 31) / 32, (rows + 31) / 32, nb), dim3(256), 0, stream,
                           static_cast<const T*>(src) + off, static_cast<T*>(dst) + off, rows, cols);
    }
}

// out[c][R-1-r][S-1-s][k] = in[k][r][s][c]
template <typename T>
__global__ void filter_bwd_data_kernel(const T* __restrict__ in, T* __restrict__ out, int K, int C, int R, int S) {
    const size_t total = (size_t)K * C * R * S;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const int k = (int)(o % K);
        size_t t = o / K;
        const int s2 = (int)(t % S);
        t /= S;
        const int r2 = (int)(t % R);
        const int c = (int)(t / R);
        out[o] = in[(((size_t)k * R + (R - 1 - r2)) * S + (S - 1 - s2)) * C + c];
    }
}

template <typename T>
__global__ void pad_channels_kernel(const T* __restrict__ src, T* __restrict__ dst, size_t rows, int c, int cpad) {
    const size_t total = rows * (size_t)cpad;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const int ch = (int)(o % cpad);
        const size_t row = o / cpad;
        dst[o] = ch < c ? src[row * c + ch] : T(0);
    }
}

// dw[i] = sum_z part[z][i].  SL lanes of the block share one output: lane j adds the j-th run of
// consecutive splits (four interleaved partial sums, combined in a fixed tree), then the SL lane sums are
// added in lane order.  The order depends on (splits, SL) only, never on timing: bit-identical reruns.
template <int SL>
__global__ void __launch_bounds__(256) reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ dw, int splits,
                                                            size_t count, int cpad, int c) {
    constexpr int OUT = 256 / SL;
    __shared__ float sm[SL][OUT];
    const int o = threadIdx.x % OUT, lane = threadIdx.x / OUT;
    const size_t i = (size_t)blockIdx.x * OUT + o;
    float acc = 0.f;
    if (i < count) {
        const int per = (splits + SL - 1) / SL;
        const int z0 = lane * per, z1 = min(splits, z0 + per);
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        int z = z0;
        for (; z + 4 <= z1; z += 4) {
            a0 += part[(size_t)z * count + i];
            a1 += part[(size_t)(z + 1) * count + i];
            a2 += part[(size_t)(z + 2) * count + i];
            a3 += part[(size_t)(z + 3) * count + i];
        }
        for (; z < z1; ++z) a0 += part[(size_t)z * count + i];
        acc = (a0 + a1) + (a2 + a3);
    }
    if (SL > 1) {
        sm[lane][o] = acc;
        __syncthreads();
        if (lane != 0) return;
        acc = sm[0][o];
#pragma unroll
        for (int j = 1; j < SL; ++j) acc += sm[j][o];
    }
    if (i >= count) return;
    if (cpad == c) {
        dw[i] = acc;
    } else {
        const int ch = (int)(i % cpad);
        if (ch < c) dw[(i / cpad) * c + ch] = acc;
    }
}

__global__ void bf16_to_f32_kernel(const uint16_t* __restrict__ src, float* __restrict__ dst, size_t count) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = __uint_as_float((uint32_t)src[i] << 16);
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst, size_t count) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = lc_bf16_rne(src[i]);
}

}  // namespace

void lc_bf16_to_f32(const void* src, float* dst, size_t count, hipStream_t stream) {
    if (!count) return;
    hipLaunchKernelGGL(bf16_to_f32_kernel, dim3(grid_for(count, 256)), dim3(256), 0, stream, static_cast<const uint16_t*>(src), dst,
                       count);
}

void lc_f32_to_bf16(const float* src, void* dst, size_t count, hipStream_t stream) {
    if (!count) return;
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(grid_for(count, 256)), dim3(256), 0, stream, src, static_cast<uint16_t*>(dst), count);
}

void lc_fill_f32(float* dst, float value, size_t count, hipStream_t stream) {
    if (!count) return;
    hipLaunchKernelGGL(fill_f32_kernel, dim3(grid_for(count, 256)), dim3(256), 0, stream, dst, value, count);
}

void lc_fill_u32x4(void* dst, size_t count16, hipStream_t stream) {
    if (!count16) return;
    hipLaunchKernelGGL(zero16_kernel, dim3(grid_for(count16, 256)), dim3(256), 0, stream, static_cast<uint4*>(dst), count16);
}

void lc_nchw_to_nhwc(const void* src, void* dst, int n, int c, int hw, int esize, hipStream_t stream) {
    if (esize == 4) transpose_batched<float>(src, dst, n, c, hw, stream);
    else transpose_batched<uint16_t>(src, dst, n, c, hw, stream);
}

void lc_nhwc_to_nchw(const void* src, void* dst, int n, int c, int hw, int esize, hipStream_t stream) {
    if (esize == 4) transpose_batched<float>(src, dst, n, hw, c, stream);
    else transpose_batched<uint16_t>(src, dst, n, hw, c, stream);
}

void lc_filter_for_bwd_data(const void* w_krsc, void* out, int k, int c, int r, int s, int esize, hipStream_t stream) {
    const size_t total = (size_t)k * c * r * s;
    if (esize == 4)
        hipLaunchKernelGGL(filter_bwd_data_kernel<float>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const float*>(w_krsc), static_cast<float*>(out), k, c, r, s);
    else
        hipLaunchKernelGGL(filter_bwd_data_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const uint16_t*>(w_krsc), static_cast<uint16_t*>(out), k, c, r, s);
}

void lc_pad_channels(const void* src, void* dst, size_t rows, int c, int cpad, int esize, hipStream_t stream) {
    const size_t total = rows * (size_t)cpad;
    if (!total) return;
    if (esize == 4)
        hipLaunchKernelGGL(pad_channels_kernel<float>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const float*>(src), static_cast<float*>(dst), rows, c, cpad);
    else
        hipLaunchKernelGGL(pad_channels_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), rows, c, cpad);
}

void lc_reduce_splits(const float* part, float* dw, int splits, size_t count, int cpad, int c, hipStream_t stream) {
    if (!count) return;
    // few outputs: spread each output's splits over more lanes so that the chip still fills
    if (count >= (size_t)1 << 18)
        hipLaunchKernelGGL(reduce_splits_kernel<1>, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, part, dw, splits,
                           count, cpad, c);
    else if (count >= (size_t)1 << 15)
        hipLaunchKernelGGL(reduce_splits_kernel<4>, dim3((unsigned)((count + 63) / 64)), dim3(256), 0, stream, part, dw, splits,
                           count, cpad, c);
    else
        hipLaunchKernelGGL(reduce_splits_kernel<16>, dim3((unsigned)((count + 15) / 16)), dim3(256), 0, stream, part, dw, splits,
                           count, cpad, c);
}
