// Data-movement helpers around the convolution kernels: fills, NCHW <-> NHWC transposes, filter
// re-ordering for backward-data, channel padding and the fixed-order sum of split partials.
// All of them are plain bandwidth-bound kernels; none is on the NHWC fast path except the filter
// re-ordering (a few MB) and the split reduction.
#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>

#include "internal.h"

namespace {

__global__ void fill_f32_kernel(float* __restrict__ dst, float value, size_t count) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = value;
}

__global__ void zero2_kernel(uint16_t* __restrict__ dst, size_t count) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) dst[i] = 0;
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

// out[c][R-1-r][S-1-s][k] = in[k][r][s][c] as one 32x32 LDS-tiled transpose per window tap (blockIdx.z): rows of
// 32 channels are read, rows of 32 filters written, both contiguous.
template <typename T>
__global__ void __launch_bounds__(256) filter_bwd_data_tiled_kernel(const T* __restrict__ in, T* __restrict__ out, int K, int C, int RS) {
    __shared__ T tile[32][33];
    const int tap = blockIdx.z, c0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const T* src = in + (size_t)tap * C;                     // in[k][tap][c]:  k * RS*C + tap*C + c
    T* dst = out + (size_t)(RS - 1 - tap) * K;               // out[c][RS-1-tap][k]: c * RS*K + (RS-1-tap)*K + k
    for (int i = ty; i < 32; i += 8) {
        const int k = k0 + i, c = c0 + tx;
        if (k < K && c < C) tile[i][tx] = src[(size_t)k * RS * C + c];
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int c = c0 + i, k = k0 + tx;
        if (k < K && c < C) dst[(size_t)c * RS * K + k] = tile[tx][i];
    }
}

// the same, one thread per element (window counts beyond the grid's z range)
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

// Sub-filter of one stride phase of a strided backward-data pass, re-ordered like the whole filter above:
// out[c][Ra-1-i][Sb-1-j][k] = in[k][a + sh*i][b + sw*j][c]  (the taps r = a, a + sh, ... and s = b, b + sw, ...).
template <typename T>
__global__ void filter_bwd_data_phase_kernel(const T* __restrict__ in, T* __restrict__ out, int K, int C, int R, int S, int a, int b,
                                             int sh, int sw, int Ra, int Sb) {
    const size_t total = (size_t)K * C * Ra * Sb;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const int k = (int)(o % K);
        size_t t = o / K;
        const int j2 = (int)(t % Sb);
        t /= Sb;
        const int i2 = (int)(t % Ra);
        const int c = (int)(t / Ra);
        const int r = a + sh * (Ra - 1 - i2), s2 = b + sw * (Sb - 1 - j2);
        out[o] = in[(((size_t)k * R + r) * S + s2) * C + c];
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

// ---- few-channel stride-2 convolutions as a stride-1 convolution over 2x2 pixel blocks ----
// With hb = (h + eph) / 2 and i = (h + eph) % 2 (eph = the padding rounded up to even), output row p reads the
// block rows p .. p + RB - 1, and likewise along the width.  The unfolded tensor U[n][hb][q][cu] holds, for output
// column q, the SB block columns q .. q + SB - 1 side by side: cu = ((bs*2 + i)*2 + j)*C + c is the input value at
// h = 2*hb + i - eph, w = 2*(q + bs) + j - epw (zero outside the image and for cu >= SB*4*C).  The convolution is
// then RB x 1, stride 1, no padding, over CU channels: every k-step of the matrix kernels lies in one tap.
struct StemGeom {
    int C, H, W, Q, HB, SB, CU, eph, epw;
};

template <typename T>
__global__ void stem_unfold_kernel(const T* __restrict__ x, T* __restrict__ u, size_t total, StemGeom g) {
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const int cu = (int)(o % g.CU);
        size_t t = o / g.CU;
        const int q = (int)(t % g.Q); t /= g.Q;
        const int hb = (int)(t % g.HB);
        const size_t n = t / g.HB;
        T v = T(0);
        if (cu < g.SB * 4 * g.C) {
            const int c = cu % g.C, ij = (cu / g.C) & 3, bs = cu / (4 * g.C);
            const int h = 2 * hb + (ij >> 1) - g.eph, w = 2 * (q + bs) + (ij & 1) - g.epw;
            if (h >= 0 && h < g.H && w >= 0 && w < g.W) v = x[((n * g.H + h) * g.W + w) * g.C + c];
        }
        u[o] = v;
    }
}

// The same through LDS: a block builds one row (n, hb) of U.  It first copies the two input rows the block row is
// made of into LDS, shifted by the left padding and surrounded by zeros; there, for each row parity i, the values
// of output column q and block column bs are the 2*C consecutive elements from (2*q + 2*bs)*C on.  Each thread
// then assembles 16-byte chunks of U and stores them side by side.
template <typename T, int C>
__global__ void __launch_bounds__(256) stem_unfold_row_kernel(const T* __restrict__ x, T* __restrict__ u, StemGeom g, int wl) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    T* rows = reinterpret_cast<T*>(smem_raw);                 // [2][wl * C]
    constexpr int EPC = 16 / (int)sizeof(T);
    const int hb = blockIdx.x % g.HB;
    const size_t n = blockIdx.x / g.HB;
    const int row_len = wl * C;
    for (int e = threadIdx.x; e < 2 * row_len; e += 256) {
        const int i = e >= row_len, pos = e - i * row_len;
        const int h = 2 * hb + i - g.eph;
        const int w = pos / C - g.epw, c = pos % C;
        T v = T(0);
        if (h >= 0 && h < g.H && w >= 0 && w < g.W) v = x[((n * g.H + h) * g.W + w) * C + c];
        rows[e] = v;
    }
    __syncthreads();
    // Work in pairs of elements: the runs of 2*C elements start at even positions on both sides, so a pair never
    // straddles two runs and sits at an even position in LDS (the row length is even as well).
    using Pair = typename std::conditional<sizeof(T) == 4, uint2, unsigned>::type;
    constexpr int PPC = EPC / 2;                              // pairs per 16-byte chunk
    const Pair* prow = reinterpret_cast<const Pair*>(rows);
    const int row_pairs = row_len / 2;
    const int chunks_per_q = g.CU / EPC, chunks = g.Q * chunks_per_q;
    T* out = u + ((n * g.HB + hb) * (size_t)g.Q) * g.CU;
    for (int ch = threadIdx.x; ch < chunks; ch += 256) {
        const int q = ch / chunks_per_q, pu0 = (ch % chunks_per_q) * PPC;
        __attribute__((aligned(16))) Pair v[PPC];
#pragma unroll
        for (int e = 0; e < PPC; ++e) {
            const int pu = pu0 + e;
            const int bs = pu / (2 * C), rem = pu % (2 * C), i = rem / C, jp = rem % C;
            v[e] = bs < g.SB ? prow[i * row_pairs + (q + bs) * C + jp] : Pair{};
        }
        *reinterpret_cast<uint4*>(out + (size_t)ch * EPC) = *reinterpret_cast<const uint4*>(v);
    }
}

// filter [K][R][S][C] -> [K][RB][CU] in the order of U (taps that the blocks add beyond the window are zero),
// and the gradient of that filter back to [K][R][S][C] (each window tap has exactly one place in the block form)
template <typename T>
__global__ void stem_filter_kernel(const T* __restrict__ w, T* __restrict__ wu, int K, int R, int S, int C, int RB, int SB, int CU,
                                   int eh, int ew) {
    const size_t total = (size_t)K * RB * CU;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const int cu = (int)(o % CU);
        const int br = (int)((o / CU) % RB);
        const size_t k = o / ((size_t)CU * RB);
        T v = T(0);
        if (cu < SB * 4 * C) {
            const int c = cu % C, ij = (cu / C) & 3, bs = cu / (4 * C);
            const int r = 2 * br + (ij >> 1) - eh, s2 = 2 * bs + (ij & 1) - ew;
            if (r >= 0 && r < R && s2 >= 0 && s2 < S) v = w[((k * R + r) * S + s2) * C + c];
        }
        wu[o] = v;
    }
}

__global__ void stem_filter_grad_kernel(const float* __restrict__ dwu, float* __restrict__ dw, int K, int R, int S, int C, int RB, int CU,
                                        int eh, int ew) {
    const size_t total = (size_t)K * R * S * C;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(o % C);
        size_t t = o / C;
        const int s2 = (int)(t % S); t /= S;
        const int r = (int)(t % R);
        const size_t k = t / R;
        const int rr = r + eh, ss = s2 + ew;
        const int cu = (((ss >> 1) * 2 + (rr & 1)) * 2 + (ss & 1)) * C + c;
        dw[o] = dwu[(k * RB + (rr >> 1)) * CU + cu];
    }
}

// Sum over the block of one double per thread, in a fixed order (lanes by butterfly, then the four waves in order);
// thread 0 holds the result.
__device__ __forceinline__ double block_sum_double(double x, double* red /* 4 doubles of LDS */) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// dw[i] = sum_z part[z][i].  SL lanes of the block share one output: lane j adds the j-th run of
// consecutive splits (four interleaved partial sums, combined in a fixed tree), then the SL lane sums are
// added in lane order.  The order depends on (splits, SL) only, never on timing: bit-identical reruns.
// sq (may be null) receives, per block, the sum of the squares of the values the block wrote to dw (in double): the
// filter gradient's squared norm in pieces, for the layer-wise update that follows.
template <int SL>
__global__ void __launch_bounds__(256) reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ dw, int splits,
                                                            size_t count, int cpad, int c, double* __restrict__ sq) {
    constexpr int OUT = 256 / SL;
    __shared__ float sm[SL][OUT];
    __shared__ double red[4];
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
        if (lane == 0) {
            acc = sm[0][o];
#pragma unroll
            for (int j = 1; j < SL; ++j) acc += sm[j][o];
        }
    }
    bool wrote = false;
    if (lane == 0 && i < count) {
        if (cpad == c) {
            dw[i] = acc;
            wrote = true;
        } else {
            const int ch = (int)(i % cpad);
            if (ch < c) {
                dw[(i / cpad) * c + ch] = acc;
                wrote = true;
            }
        }
    }
    if (sq) {
        const double total = block_sum_double(wrote ? (double)acc * (double)acc : 0.0, red);
        if (threadIdx.x == 0) sq[blockIdx.x] = total;
    }
}

// sq[b] = sum of x[i]^2 over block b's 4096 elements (in double, fixed order): the squared norm of a tensor in pieces.
__global__ void __launch_bounds__(256) sq_partials_kernel(const float* __restrict__ x, size_t count, double* __restrict__ sq) {
    __shared__ double red[4];
    const size_t base = (size_t)blockIdx.x * 4096;
    double s = 0.0;
#pragma unroll 4
    for (int j = 0; j < 16; ++j) {
        const size_t i = base + threadIdx.x + (size_t)j * 256;
        if (i < count) {
            const float v = x[i];
            s += (double)v * (double)v;
        }
    }
    const double total = block_sum_double(s, red);
    if (threadIdx.x == 0) sq[blockIdx.x] = total;
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

// Zero `bytes` bytes (an even number) at a 2-byte aligned address: 16-byte stores where the alignment allows.
void lc_zero_bytes(void* dst, size_t bytes, hipStream_t stream) {
    if (!bytes) return;
    char* p = static_cast<char*>(dst);
    if ((reinterpret_cast<uintptr_t>(p) & 15) == 0) {
        const size_t body = bytes / 16;
        lc_fill_u32x4(p, body, stream);
        p += body * 16;
        bytes -= body * 16;
    } else if ((reinterpret_cast<uintptr_t>(p) & 3) == 0) {
        const size_t body = bytes / 4;
        lc_fill_f32(reinterpret_cast<float*>(p), 0.f, body, stream);
        p += body * 4;
        bytes -= body * 4;
    }
    if (bytes) hipLaunchKernelGGL(zero2_kernel, dim3(grid_for(bytes / 2, 256)), dim3(256), 0, stream, reinterpret_cast<uint16_t*>(p), bytes / 2);
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
    if ((long long)r * s <= 65535 && (k + 31) / 32 <= 65535) {
        const dim3 grid((c + 31) / 32, (k + 31) / 32, r * s);
        if (esize == 4)
            hipLaunchKernelGGL(filter_bwd_data_tiled_kernel<float>, grid, dim3(256), 0, stream, static_cast<const float*>(w_krsc),
                               static_cast<float*>(out), k, c, r * s);
        else
            hipLaunchKernelGGL(filter_bwd_data_tiled_kernel<uint16_t>, grid, dim3(256), 0, stream, static_cast<const uint16_t*>(w_krsc),
                               static_cast<uint16_t*>(out), k, c, r * s);
        return;
    }
    if (esize == 4)
        hipLaunchKernelGGL(filter_bwd_data_kernel<float>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const float*>(w_krsc), static_cast<float*>(out), k, c, r, s);
    else
        hipLaunchKernelGGL(filter_bwd_data_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const uint16_t*>(w_krsc), static_cast<uint16_t*>(out), k, c, r, s);
}

void lc_filter_for_bwd_data_phase(const void* w_krsc, void* out, int k, int c, int r, int s, int a, int b, int sh, int sw, int ra,
                                  int sb, int esize, hipStream_t stream) {
    const size_t total = (size_t)k * c * ra * sb;
    if (!total) return;
    if (esize == 4)
        hipLaunchKernelGGL(filter_bwd_data_phase_kernel<float>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const float*>(w_krsc), static_cast<float*>(out), k, c, r, s, a, b, sh, sw, ra, sb);
    else
        hipLaunchKernelGGL(filter_bwd_data_phase_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const uint16_t*>(w_krsc), static_cast<uint16_t*>(out), k, c, r, s, a, b, sh, sw, ra, sb);
}

// Strided 2-D copy (a channel slice of an activation tensor to or from a dense one): element (row, i) of width-V vectors.
template <typename V>
__global__ void __launch_bounds__(256) copy2d_kernel(const char* __restrict__ src, size_t src_pitch, char* __restrict__ dst,
                                                     size_t dst_pitch, size_t wvec, size_t total) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t row = i / wvec, col = i - row * wvec;
        *reinterpret_cast<V*>(dst + row * dst_pitch + col * sizeof(V)) = *reinterpret_cast<const V*>(src + row * src_pitch + col * sizeof(V));
    }
}

void lc_copy2d(const void* src, size_t src_pitch, void* dst, size_t dst_pitch, size_t width_bytes, size_t rows, hipStream_t stream) {
    if (!width_bytes || !rows) return;
    const uintptr_t all = (uintptr_t)src | (uintptr_t)dst | src_pitch | dst_pitch | width_bytes;
    const char* s = static_cast<const char*>(src);
    char* d = static_cast<char*>(dst);
    if ((all & 15) == 0) {
        const size_t wv = width_bytes / 16, total = wv * rows;
        hipLaunchKernelGGL(copy2d_kernel<uint4>, dim3(grid_for(total, 256)), dim3(256), 0, stream, s, src_pitch, d, dst_pitch, wv, total);
    } else if ((all & 3) == 0) {
        const size_t wv = width_bytes / 4, total = wv * rows;
        hipLaunchKernelGGL(copy2d_kernel<uint32_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream, s, src_pitch, d, dst_pitch, wv, total);
    } else {
        const size_t wv = width_bytes / 2, total = wv * rows;
        hipLaunchKernelGGL(copy2d_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream, s, src_pitch, d, dst_pitch, wv, total);
    }
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

void lc_stem_unfold(const void* x, void* u, int n, int c, int h, int w, int q, int hb, int sb, int cu, int eph, int epw, int esize,
                    hipStream_t stream) {
    const size_t total = (size_t)n * hb * q * cu;
    if (!total) return;
    const StemGeom g = {c, h, w, q, hb, sb, cu, eph, epw};
    // the LDS row holds every pixel column a block row can touch: 2 * (q + sb - 1) of them, each c wide
    const int wl = 2 * (q + sb - 1);
    const size_t lds = (size_t)2 * wl * c * esize;
    const bool by_rows = lds <= 48 * 1024 && (long long)n * hb <= 0x7fffffffLL && (reinterpret_cast<uintptr_t>(u) & 15) == 0 &&
                         (cu * esize) % 16 == 0;
    if (by_rows) {
        const dim3 grid((unsigned)((size_t)n * hb));
#define LC_UNFOLD(T, CC) \
    hipLaunchKernelGGL((stem_unfold_row_kernel<T, CC>), grid, dim3(256), lds, stream, static_cast<const T*>(x), static_cast<T*>(u), g, wl)
        if (esize == 4) {
            switch (c) {
                case 1: LC_UNFOLD(float, 1); return;
                case 2: LC_UNFOLD(float, 2); return;
                case 3: LC_UNFOLD(float, 3); return;
                case 4: LC_UNFOLD(float, 4); return;
            }
        } else {
            switch (c) {
                case 1: LC_UNFOLD(uint16_t, 1); return;
                case 2: LC_UNFOLD(uint16_t, 2); return;
                case 3: LC_UNFOLD(uint16_t, 3); return;
                case 4: LC_UNFOLD(uint16_t, 4); return;
            }
        }
#undef LC_UNFOLD
    }
    if (esize == 4)
        hipLaunchKernelGGL(stem_unfold_kernel<float>, dim3(grid_for(total, 256)), dim3(256), 0, stream, static_cast<const float*>(x),
                           static_cast<float*>(u), total, g);
    else
        hipLaunchKernelGGL(stem_unfold_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const uint16_t*>(x), static_cast<uint16_t*>(u), total, g);
}

void lc_stem_filter(const void* w, void* wu, int k, int r, int s, int c, int rb, int sb, int cu, int eh, int ew, int esize,
                    hipStream_t stream) {
    const size_t total = (size_t)k * rb * cu;
    if (esize == 4)
        hipLaunchKernelGGL(stem_filter_kernel<float>, dim3(grid_for(total, 256)), dim3(256), 0, stream, static_cast<const float*>(w),
                           static_cast<float*>(wu), k, r, s, c, rb, sb, cu, eh, ew);
    else
        hipLaunchKernelGGL(stem_filter_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream,
                           static_cast<const uint16_t*>(w), static_cast<uint16_t*>(wu), k, r, s, c, rb, sb, cu, eh, ew);
}

void lc_stem_filter_grad(const float* dwu, float* dw, int k, int r, int s, int c, int rb, int cu, int eh, int ew, hipStream_t stream) {
    const size_t total = (size_t)k * r * s * c;
    hipLaunchKernelGGL(stem_filter_grad_kernel, dim3(grid_for(total, 256)), dim3(256), 0, stream, dwu, dw, k, r, s, c, rb, cu, eh, ew);
}

// Grid of the split reduction for `count` outputs: few outputs spread each output's splits over more lanes so that the
// chip still fills.  A fixed function of count (it is also the number of squared-norm pieces the reduction emits).
static int reduce_splits_lanes(size_t count) { return count >= (size_t)1 << 18 ? 1 : count >= (size_t)1 << 15 ? 4 : 16; }

size_t lc_reduce_splits_blocks(size_t count) {
    const size_t out = 256 / reduce_splits_lanes(count);
    return (count + out - 1) / out;
}

void lc_reduce_splits(const float* part, float* dw, int splits, size_t count, int cpad, int c, double* sq, hipStream_t stream) {
    if (!count) return;
    const unsigned grid = (unsigned)lc_reduce_splits_blocks(count);
    switch (reduce_splits_lanes(count)) {
        case 1: hipLaunchKernelGGL(reduce_splits_kernel<1>, dim3(grid), dim3(256), 0, stream, part, dw, splits, count, cpad, c, sq); break;
        case 4: hipLaunchKernelGGL(reduce_splits_kernel<4>, dim3(grid), dim3(256), 0, stream, part, dw, splits, count, cpad, c, sq); break;
        default: hipLaunchKernelGGL(reduce_splits_kernel<16>, dim3(grid), dim3(256), 0, stream, part, dw, splits, count, cpad, c, sq);
    }
}

size_t lc_sq_partials_blocks(size_t count) { return (count + 4095) / 4096; }

void lc_sq_partials(const float* x, size_t count, double* sq, hipStream_t stream) {
    if (!count) return;
    hipLaunchKernelGGL(sq_partials_kernel, dim3((unsigned)lc_sq_partials_blocks(count)), dim3(256), 0, stream, x, count, sq);
}
