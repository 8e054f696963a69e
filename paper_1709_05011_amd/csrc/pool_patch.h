// Gradient of the 3x3 / stride 2 / padding 1 max pool (ResNet-50's only pool) for NHWC tensors, shared by the fp32 and the
// bf16 glue: one thread per 2x2 patch of input pixels and IO::VEC neighbouring channels.
//
// Window p covers the input rows 2p-1 .. 2p+1, so an even row 2i lies in window i only (as its middle row) and an odd row
// 2i+1 in windows i (last row) and i+1 (first row); the same holds for columns.  The four pixels of patch (i, j) therefore
// need exactly the four windows (i..i+1) x (j..j+1): each window's gradient vector and index bytes are loaded once per
// patch, where a thread per pixel loads 2.25 windows per pixel on average.  Every pixel still adds its windows in window
// order (row-major), so the result is the per-pixel kernel's bit for bit.
//
// IO supplies the element type and its conversions: IO::T, IO::VEC (4 or 8), IO::load(const T*, float*), IO::store(T*,
// const float*).  idx holds one byte per output element (the tap, row * 3 + column, of the window's first maximum) and
// must be 4-byte aligned; dy and dx 16-byte aligned.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

template <typename IO>
__global__ void __launch_bounds__(256) maxpool_bwd_3x3s2_kernel(const typename IO::T* __restrict__ dy, const uint8_t* __restrict__ idx,
                                                                typename IO::T* __restrict__ dx, int N, int CV, int H, int W, int Ho,
                                                                int Wo) {
    constexpr int VEC = IO::VEC;
    const int Hp = (H + 1) / 2, Wp = (W + 1) / 2;
    const size_t total = (size_t)N * Hp * Wp * CV;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        size_t t = o;
        const int cv = (int)(t % CV); t /= CV;
        const int j = (int)(t % Wp); t /= Wp;
        const int i = (int)(t % Hp);
        const int n = (int)(t / Hp);
        float acc[2][2][VEC];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[a][b][e] = 0.f;
#pragma unroll
        for (int dp = 0; dp < 2; ++dp)
#pragma unroll
            for (int dq = 0; dq < 2; ++dq) {
                const int p = i + dp, q = j + dq;
                if (p >= Ho || q >= Wo) continue;
                const size_t oo = (((size_t)n * Ho + p) * Wo + q) * CV + cv;
                uint32_t taps[VEC / 4];
#pragma unroll
                for (int k = 0; k < VEC / 4; ++k) taps[k] = reinterpret_cast<const uint32_t*>(idx)[oo * (VEC / 4) + k];
                float g[VEC];
                IO::load(dy + oo * VEC, g);
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        const int r = a + 1 - 2 * dp, s = b + 1 - 2 * dq;   // the patch pixel's place in this window
                        if (r < 0 || s < 0) continue;
                        const unsigned tap = (unsigned)(r * 3 + s);
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            if (((taps[e / 4] >> (8 * (e & 3))) & 0xffu) == tap) acc[a][b][e] += g[e];
                    }
            }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int h = 2 * i + a, w = 2 * j + b;
                if (h < H && w < W) IO::store(dx + ((((size_t)n * H + h) * W + w) * CV + cv) * VEC, acc[a][b]);
            }
    }
}
