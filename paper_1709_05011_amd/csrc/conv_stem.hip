// ResNet's first layer (7x7 window, stride 2, padding 3, 3 -> 64 channels, NHWC, output height and width multiples of 16):
// forward pass and filter gradient, each in fp32 and in bf16, from an input slab in LDS.  The layer is the first of the
// paper's ResNet-50 ("ImageNet training with ResNet-50"): 2 % of the network's multiplications, 4 % of the step's time on
// the general kernels.  Four kernels: conv_stem_f32_kernel (described first), conv_stem_wgrad_f32_kernel,
// conv_stem_bf16_kernel, conv_stem_wgrad_bf16_kernel; lc_conv_stem_f32_ok() is the shape test for all of them.
//
// The general kernel pads the three channels to four (a pass over the input and 25 % more multiplications) and gathers every
// window element with per-lane address arithmetic.  Here a block owns 16 x 16 output pixels: their 37 x 37 input pixels
// (37 rows of 111 contiguous floats in NHWC) go to LDS once, the whole filter sits in LDS for the life of the block, and an
// MFMA operand is read at `lane's pixel + (r, s, c)` where the second term is a compile-time constant: no address
// arithmetic in the loop at all.  A filter row's 21 values are padded to 22 so that the two k of an MFMA (32x32x2) never
// straddle rows: 154 k instead of 147 (the general kernel ran 196).  The slab pitch of 112 floats makes the A reads of a wave
// (32 pixels: 2 rows x 16 columns, 6 floats apart, two k) fall on 64 distinct banks; the filter is stored [k][64] with the
// two 32-column halves of odd rows swapped, for the same reason.  Blocks are persistent (filter loaded once), the next
// tile's slab is fetched into registers under the MFMAs, operands are read one k pair ahead.  A wave owns 4 rows x 16 columns
// of pixels x 64 filters; the batch-norm statistics of conv2d_fwd_stats come out of its accumulators, one piece per wave.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>

#include "../../include/larsconv.h"
#include "internal.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory"); }

namespace stem {
constexpr int R = 7, S = 7, C = 3, N = 64, ST = 2, PAD = 3;
constexpr int TH = 16, TW = 16;                    // output pixels per tile
constexpr int SR = (TH - 1) * ST + R;              // 37 slab rows
constexpr int SWF = ((TW - 1) * ST + S) * C;       // 111 floats of a slab row
constexpr int SP = 112;                            // slab pitch in floats (element 111 stays zero: the 22nd tap of a window's last pixel)
constexpr int T2 = (S * C + 1) / 2 * 2;            // 22: a filter row's 21 values and a zero, so that a k pair never straddles rows
constexpr int KP = R * T2;                         // 154
constexpr int SLAB = SR * SP;                      // 4144 floats
constexpr int LD = (SLAB + 255) / 256;             // 17 loads per thread
}  // namespace stem

__global__ void __launch_bounds__(256, 2) conv_stem_f32_kernel(const StemConv p) {
    using namespace stem;
    extern __shared__ __attribute__((aligned(16))) float st_smem[];
    float* Bs = st_smem;                 // [KP][64], the two 32-column halves of odd rows swapped
    float* slab = st_smem + KP * N;      // [2][SLAB]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, m = lane & 31;
    const int tiles_x = p.Q / TW, tiles_y = p.P / TH, tiles = p.imgs * tiles_y * tiles_x;

    for (int idx = tid; idx < N * R * S * C; idx += 256) {          // coalesced reads of the filter, scattered into [k][n]
        const int n = idx / (R * S * C), rem = idx - n * (R * S * C), r = rem / (S * C), t = rem - r * (S * C);
        const int k = r * T2 + t;
        Bs[k * N + (n ^ ((k & 1) << 5))] = p.w[idx];
    }
    if (T2 > S * C)
        for (int idx = tid; idx < R * N; idx += 256) {              // the zero that completes each filter row's last k pair
            const int r = idx / N, n = idx - r * N, k = r * T2 + T2 - 1;
            Bs[k * N + (n ^ ((k & 1) << 5))] = 0.f;
        }
    const int a_lane = ((4 * wave + (m >> 4)) * ST) * SP + (m & 15) * ST * C + half;
    int b_lane[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) b_lane[j] = half * N + ((m + 32 * j) ^ (half << 5));

    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, (int)((long long)p.imgs * p.H * p.W * C * 4), 0x00020000);
    float g[LD];
    auto gload = [&](int tile) {
        const int tx = tile % tiles_x, t2 = tile / tiles_x, ty = t2 % tiles_y, img = t2 / tiles_y;
        const int h0 = ty * TH * ST - PAD, w0f = (tx * TW * ST - PAD) * C;
        const int base = (img * p.H + h0) * p.W * C + w0f;              // floats; may be negative: only valid lanes use it
#pragma unroll
        for (int l = 0; l < LD; ++l) {
            const int e = tid + 256 * l, i = e / SP, f = e - i * SP;
            const bool ok = (e < SLAB) & (f < SWF) & ((unsigned)(h0 + i) < (unsigned)p.H) & ((unsigned)(w0f + f) < (unsigned)(p.W * C));
            const unsigned off = ok ? (unsigned)(base + i * p.W * C + f) * 4u : 0x80000000u;
            g[l] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(x_rsrc, off, 0, 0));
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int l = 0; l < LD; ++l) {
            const int e = tid + 256 * l;
            if (e < SLAB) slab[buf * SLAB + e] = g[l];
        }
    };

    int tile = blockIdx.x;
    if (tile < tiles) gload(tile);
    int buf = 0;
    for (; tile < tiles; tile += gridDim.x) {
        sstore(buf);
        lds_barrier();
        if (tile + (int)gridDim.x < tiles) gload(tile + gridDim.x);
        f32x16 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        const float* sa = slab + buf * SLAB + a_lane;
        float a[2][2], b[2][2];                                        // [slot][tile]: operands of k pair kp in slot kp & 1
        auto read_pair = [&](int kp, int slot) __attribute__((always_inline)) {
            const int r = kp / (T2 / 2), t = 2 * (kp % (T2 / 2));
#pragma unroll
            for (int i = 0; i < 2; ++i) a[slot][i] = sa[(2 * i * ST + r) * SP + t];
#pragma unroll
            for (int j = 0; j < 2; ++j) b[slot][j] = Bs[kp * 2 * N + b_lane[j]];
        };
        read_pair(0, 0);
#pragma unroll
        for (int kp = 0; kp < KP / 2; ++kp) {
            if (kp + 1 < KP / 2) read_pair(kp + 1, (kp + 1) & 1);     // one pair (four MFMAs) ahead
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kp & 1][i], b[kp & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the wave's 4 rows x 16 columns of output pixels, 64 channels
        const int tx = tile % tiles_x, t2 = tile / tiles_x, ty = t2 % tiles_y, img = t2 / tiles_y;
        float* yo = p.y + (((long long)img * p.P + ty * TH + 4 * wave) * p.Q + tx * TW) * N + 4 * half * N + m;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 2 * i + (v >> 3), col = 8 * ((v >> 2) & 1) + (v & 3);
#pragma unroll
                for (int j = 0; j < 2; ++j) yo[(row * p.Q + col) * N + 32 * j] = acc[i][j][v];
            }
        if (p.stats) {
            typedef float flt2 __attribute__((ext_vector_type(2)));
            flt2* st = reinterpret_cast<flt2*>(p.stats) + ((size_t)tile * 4 + wave) * N;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float sum = 0.f, sq = 0.f;
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        sum += acc[i][j][v];
                        sq = fmaf(acc[i][j][v], acc[i][j][v], sq);
                    }
                sum += __shfl_xor(sum, 32);
                sq += __shfl_xor(sq, 32);
                if (half == 0) st[32 * j + m] = flt2{sum, sq};
            }
        }
        buf ^= 1;
    }
}

// The same layer's filter gradient, dW[k][r][s][c] = sum over output pixels of dY[pixel][k] * X[window of the pixel][r][s][c]
// (the general kernel: channels padded to four, per-lane gathers, 1.09 ms + a padding pass at batch 256).  Same tiles, same
// slab.  A wave owns 32 of the 64 filters and 8 of the tile's 16 pixel rows and keeps all 5 x 32 columns of its part of dW
// (147 of them used) in registers for the whole life of the block; per pixel pair it reads dY straight from memory (one
// value per lane, a row of pairs ahead) and the five X operands from the slab at `lane's (r, s, c) + pixel`, the pixel being
// a compile-time constant.  When its tiles are done the block adds the two waves of each filter half through LDS and writes
// one partial [64][147]; the fixed-order sum over the blocks is reduce_splits_kernel's, as for every filter gradient.
__global__ void __launch_bounds__(256, 2) conv_stem_wgrad_f32_kernel(const StemWgrad p) {
    using namespace stem;
    constexpr int J = R * S * C, JT = (J + 31) / 32;          // 147 columns in 5 tiles of 32 (the last 13 columns are not stored)
    extern __shared__ __attribute__((aligned(16))) float sw_smem[];
    float* slab = sw_smem;               // [2][SLAB]; the block's final sum over its waves reuses it
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l = lane & 31;
    const int kt = wave >> 1, rh = wave & 1;            // the wave's 32 filters and its 8 of the tile's 16 pixel rows
    const int tiles_x = p.Q / TW, tiles_y = p.P / TH, tiles = p.imgs * tiles_y * tiles_x;

    int b_lane[JT];                      // slab offset of this lane's (r, s, c) for each column tile, plus the wave's rows and the pixel of its half
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
        const int j = 32 * jt + l;
        b_lane[jt] = (j < J ? (j / (S * C)) * SP + j % (S * C) : 0) + ST * C * half + ST * 8 * rh * SP;
    }
    const unsigned a_lane = (unsigned)(half * N + 32 * kt + l) * 4u;

    const long long x_img = (long long)p.H * p.W * C, y_img = (long long)p.P * p.Q * N;
    float g[LD];
    auto gload = [&](int tile) {
        const int tx = tile % tiles_x, t2 = tile / tiles_x, ty = t2 % tiles_y, img = t2 / tiles_y;
        const int h0 = ty * TH * ST - PAD, w0f = (tx * TW * ST - PAD) * C;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(p.x + img * x_img), 0, (int)(x_img * 4), 0x00020000);
        const int base = h0 * p.W * C + w0f;                            // floats within the image; may be negative: only valid lanes use it
#pragma unroll
        for (int i2 = 0; i2 < LD; ++i2) {
            const int e = tid + 256 * i2, i = e / SP, f = e - i * SP;
            const bool ok = (e < SLAB) & (f < SWF) & ((unsigned)(h0 + i) < (unsigned)p.H) & ((unsigned)(w0f + f) < (unsigned)(p.W * C));
            const unsigned off = ok ? (unsigned)(base + i * p.W * C + f) * 4u : 0x80000000u;
            g[i2] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, 0));
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i2 = 0; i2 < LD; ++i2) {
            const int e = tid + 256 * i2;
            if (e < SLAB) slab[buf * SLAB + e] = g[i2];
        }
    };
    // dY of one row of the wave's pixels: 8 pixel pairs, one value per lane each
    float a[2][8];
    auto yload = [&](int tile, int row, int set) __attribute__((always_inline)) {
        const int tx = tile % tiles_x, t2 = tile / tiles_x, ty = t2 % tiles_y, img = t2 / tiles_y;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(p.dy + img * y_img), 0, (int)(y_img * 4), 0x00020000);
        const int soff = (((ty * TH + 8 * rh + row) * p.Q + tx * TW) * N) * 4;
#pragma unroll
        for (int c2 = 0; c2 < 8; ++c2)
            a[set][c2] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, a_lane, soff + 2 * c2 * N * 4, 0));
    };

    f32x16 acc[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[jt][v] = 0.f;

    int tile = blockIdx.x;
    if (tile < tiles) {
        gload(tile);
        yload(tile, 0, 0);
    }
    int buf = 0;
    for (; tile < tiles; tile += gridDim.x) {
        sstore(buf);
        lds_barrier();
        const int next = tile + (int)gridDim.x;
        if (next < tiles) gload(next);
        const float* sb = slab + buf * SLAB;
#pragma unroll
        for (int row = 0; row < 8; ++row) {
            if (row < 7) yload(tile, row + 1, (row + 1) & 1);
            else if (next < tiles) yload(next, 0, 0);
            float b[2][JT];
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) b[0][jt] = sb[b_lane[jt] + ST * row * SP];
#pragma unroll
            for (int c2 = 0; c2 < 8; ++c2) {
                if (c2 + 1 < 8) {
#pragma unroll
                    for (int jt = 0; jt < JT; ++jt) b[(c2 + 1) & 1][jt] = sb[b_lane[jt] + ST * row * SP + ST * C * 2 * (c2 + 1)];
                }
#pragma unroll
                for (int jt = 0; jt < JT; ++jt)
                    acc[jt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[row & 1][c2], b[c2 & 1][jt], acc[jt], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        buf ^= 1;
    }

    // the block's sum over the two waves that share a filter half, one column tile of dw at a time, written as this block's partial
    float* part = p.part + (size_t)blockIdx.x * N * J;
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
        lds_barrier();                                                    // the slab (or the last round) is no longer read
#pragma unroll
        for (int v = 0; v < 16; ++v) slab[(wave * 16 + v) * 64 + lane] = acc[jt][v];
        lds_barrier();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int e = tid + 256 * i, k2 = e >> 10, v = (e >> 6) & 15, ln = e & 63;
            const float s2 = slab[((2 * k2) * 16 + v) * 64 + ln] + slab[((2 * k2 + 1) * 16 + v) * 64 + ln];
            const int rowk = k2 * 32 + 8 * (v >> 2) + 4 * (ln >> 5) + (v & 3), col = jt * 32 + (ln & 31);
            if (col < J) part[rowk * J + col] = s2;
        }
    }
}

// The forward pass in bf16 (bf16 x, w and y, fp32 sums, y rounded once).  Same tiles and slab (as bf16, fetched element by
// element: a slab row starts on a 2-byte boundary).  An MFMA (32x32x16) takes 8 consecutive k from a lane, so a filter row's
// 21 values are padded to 32: two MFMA steps per row, a lane's 8 values never straddle rows and start on a 4-byte boundary of
// the slab (four 4-byte LDS reads); 224 k in 14 steps -- 56 MFMAs per wave and tile, a tenth of the fp32 kernel's matrix
// time: the kernel is bound by its memory traffic (y is 5/6 of it).  The filter sits in LDS as [64][224 + 8].  Two
// neighbouring pixels of a channel are rounded together and swapped with the neighbouring lane, so that every lane stores two
// channels of one pixel as a dword; the statistics are those of the rounded values.
namespace stemb {
constexpr int R = 7, S = 7, C = 3, N = 64, ST = 2, PAD = 3;
constexpr int TH = 16, TW = 16;
constexpr int SR = (TH - 1) * ST + R;              // 37 slab rows
constexpr int SWF = ((TW - 1) * ST + S) * C;       // 111 elements of a slab row
constexpr int KR = 32;                             // k per filter row: its 21 values and 11 zeros (two MFMA steps of 16, a lane's 8 k never straddle rows)
constexpr int KP = R * KR;                         // 224
constexpr int SP = 124;                            // slab pitch in elements: a window's last pixel reads up to element 90 + 31
constexpr int SLAB = SR * SP;                      // 4588
constexpr int LD = (SLAB + 255) / 256;             // 18
constexpr int BP = KP + 8;                         // filter pitch in elements (16-byte aligned rows, 8 banks apart)
}  // namespace stemb

__global__ void __launch_bounds__(256, 2) conv_stem_bf16_kernel(const StemConvBf16 p) {
    using namespace stemb;
    extern __shared__ __attribute__((aligned(16))) uint16_t sb_smem[];
    uint16_t* Bs = sb_smem;                  // [64][BP]
    uint16_t* slab = sb_smem + N * BP;       // [2][SLAB]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb = lane >> 5, m = lane & 31;
    const int tiles_x = p.Q / TW, tiles_y = p.P / TH, tiles = p.imgs * tiles_y * tiles_x;

    for (int idx = tid; idx < N * BP / 2; idx += 256) reinterpret_cast<unsigned*>(Bs)[idx] = 0u;
    __syncthreads();
    for (int idx = tid; idx < N * R * S * C; idx += 256) {
        const int n = idx / (R * S * C), rem = idx - n * (R * S * C), r = rem / (S * C), t = rem - r * (S * C);
        Bs[n * BP + r * KR + t] = p.w[idx];
    }
    const int a_lane = ((4 * wave + (m >> 4)) * ST) * SP + (m & 15) * ST * C + 8 * kb;     // elements (even: 4-byte aligned)
    int b_lane[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) b_lane[j] = (m + 32 * j) * BP + 8 * kb;

    const long long x_img = (long long)p.H * p.W * C;
    unsigned g[LD];
    auto gload = [&](int tile) {
        const int tx = tile % tiles_x, t2 = tile / tiles_x, ty = t2 % tiles_y, img = t2 / tiles_y;
        const int h0 = ty * TH * ST - PAD, w0f = (tx * TW * ST - PAD) * C;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(p.x + img * x_img), 0, (int)(x_img * 2), 0x00020000);
        const int base = h0 * p.W * C + w0f;
#pragma unroll
        for (int l = 0; l < LD; ++l) {
            const int e = tid + 256 * l, i = e / SP, f = e - i * SP;
            const bool ok = (e < SLAB) & (f < SWF) & ((unsigned)(h0 + i) < (unsigned)p.H) & ((unsigned)(w0f + f) < (unsigned)(p.W * C));
            const unsigned off = ok ? (unsigned)(base + i * p.W * C + f) * 2u : 0x80000000u;
            g[l] = __builtin_amdgcn_raw_buffer_load_b16(rsrc, off, 0, 0);
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int l = 0; l < LD; ++l) {
            const int e = tid + 256 * l;
            if (e < SLAB) slab[buf * SLAB + e] = (uint16_t)g[l];
        }
    };

    int tile = blockIdx.x;
    if (tile < tiles) gload(tile);
    int buf = 0;
    for (; tile < tiles; tile += gridDim.x) {
        sstore(buf);
        lds_barrier();
        if (tile + (int)gridDim.x < tiles) gload(tile + gridDim.x);
        f32x16 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        const uint16_t* sa = slab + buf * SLAB + a_lane;
#pragma unroll
        for (int s = 0; s < KP / 16; ++s) {
            const int r = s / 2, t0 = 16 * (s % 2);
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const unsigned* q = reinterpret_cast<const unsigned*>(sa + (2 * i * ST + r) * SP + t0);
                const u32x4 v = {q[0], q[1], q[2], q[3]};
                a[i] = __builtin_bit_cast(bf16x8, v);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Bs + b_lane[j] + 16 * s));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        const int tx = tile % tiles_x, t2 = tile / tiles_x, ty = t2 % tiles_y, img = t2 / tiles_y;
        // Registers v and v + 1 hold two neighbouring pixels of the lane's channel: the pair is rounded together, swapped with
        // the neighbouring lane, and every lane stores two channels of one pixel as a dword (even lanes the first pixel, odd
        // lanes the second).
        const int odd = lane & 1;
        uint16_t* yo = p.y + (((long long)img * p.P + ty * TH + 4 * wave) * p.Q + tx * TW) * N + (4 * kb + odd) * N + (m & ~1);
        const unsigned perm_sel = odd ? 0x03020706u : 0x05040100u;
        float sum[2] = {0.f, 0.f}, sq[2] = {0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                const int row = 2 * i + (v >> 3), col = 8 * ((v >> 2) & 1) + (v & 3);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                    typedef float f32x2 __attribute__((ext_vector_type(2)));
                    const f32x2 pr = {acc[i][j][v], acc[i][j][v + 1]};
                    const unsigned u = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, bf16x2));
                    const unsigned got = (unsigned)__builtin_amdgcn_mov_dpp((int)u, 0xB1 /* quad_perm 1,0,3,2 */, 0xF, 0xF, true);
                    *reinterpret_cast<unsigned*>(yo + (row * p.Q + col) * N + 32 * j) = __builtin_amdgcn_perm(got, u, perm_sel);
                    const float f0 = __uint_as_float(u << 16), f1 = __uint_as_float(u & 0xffff0000u);
                    sum[j] += f0;
                    sq[j] = fmaf(f0, f0, sq[j]);
                    sum[j] += f1;
                    sq[j] = fmaf(f1, f1, sq[j]);
                }
            }
        if (p.stats) {
            typedef float flt2 __attribute__((ext_vector_type(2)));
            flt2* st = reinterpret_cast<flt2*>(p.stats) + ((size_t)tile * 4 + wave) * N;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float s1 = sum[j] + __shfl_xor(sum[j], 32), s2 = sq[j] + __shfl_xor(sq[j], 32);
                if (kb == 0) st[32 * j + m] = flt2{s1, s2};
            }
        }
        buf ^= 1;
    }
}

// The filter gradient in bf16 (bf16 x and dY, fp32 sums and dW).  The reduction runs over pixels, and a `32x32x16` MFMA takes
// 8 consecutive reduction values from a lane: both operands come from LDS through the transposing read (see
// wgrad_bf16_kernel), which lets every lane point anywhere.  dY of the tile sits in LDS as [pixel][64].  The slab keeps four
// channels per pixel (the fourth zero), so that a pixel is 8 bytes and the 16 pixels of an output row, two input pixels
// apart, are "rows" 16 bytes apart that overlap: row i of the operand matrix of filter row r is the 32 elements (s, c) from
// pixel 2 i on -- 7 x 4 window elements and a zero tail.  One MFMA step is one output row of the tile (16 pixels); the columns
// of dW come out as (r, s * 4 + c), 7 tiles of 32.  A wave owns 32 filters and the filter rows 0-3 or 4-6 for the life of the
// block and writes its part of the block's partial itself (no sum across waves).  0.92 ms (unfolding pass + gathering
// kernel) -> 0.33 ms at batch 512.
namespace stemwb {
constexpr int R = 7, S = 7, C = 3, N = 64, ST = 2, PAD = 3;
constexpr int TH = 16, TW = 16;
constexpr int SR = (TH - 1) * ST + R;              // 37 slab rows
constexpr int SPX = (TW - 1) * ST + S;             // 37 slab pixels per row
constexpr int CP = 4;                              // channels per slab pixel (the fourth stays zero): a pixel is 8 bytes
constexpr int SPB = 152;                           // slab pitch in elements: the last pixel's 32 window elements end at 15 * 8 + 32
constexpr int SLAB = SR * SPB;                     // 5624 elements
constexpr int SLD = (SR * SPX * C + 255) / 256;    // 17 element loads per thread
constexpr int PA = 96;                             // dY pitch in elements ([pixel][64] + 32: rows 64 bytes apart modulo 256)
constexpr int J = R * S * C;                       // 147
}  // namespace stemwb

__global__ void __launch_bounds__(256, 2) conv_stem_wgrad_bf16_kernel(const StemWgradBf16 p) {
    using namespace stemwb;
    __shared__ __attribute__((aligned(16))) uint16_t slab[SLAB];
    __shared__ __attribute__((aligned(16))) uint16_t dys[TH * TW * PA];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kt = wave >> 1, r0 = (wave & 1) * 4, nr = (wave & 1) ? 3 : 4;   // the wave's 32 filters and its filter rows r0 .. r0 + nr - 1
    const int tiles_x = p.Q / TW, tiles_y = p.P / TH, tiles = p.imgs * tiles_y * tiles_x;

    for (int i = tid; i < SLAB / 2; i += 256) reinterpret_cast<unsigned*>(slab)[i] = 0u;    // fourth channels and row tails stay zero

    const long long x_img = (long long)p.H * p.W * C;
    unsigned gx[SLD];
    u32x4 gy[8];
    auto gload = [&](int tile) {
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));                                 // recompute the per-element indices every tile: hoisted, they cost 70 registers
        const int tx = tile % tiles_x, t2 = tile / tiles_x, ty = t2 % tiles_y, img = t2 / tiles_y;
        const int h0 = ty * TH * ST - PAD, w0 = tx * TW * ST - PAD;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(p.x + img * x_img), 0, (int)(x_img * 2), 0x00020000);
#pragma unroll
        for (int l = 0; l < SLD; ++l) {
            const int e = tid + 256 * l, i = e / (SPX * C), f = e - i * (SPX * C);
            const bool ok = (e < SR * SPX * C) & ((unsigned)(h0 + i) < (unsigned)p.H) & ((unsigned)(w0 * C + f) < (unsigned)(p.W * C));
            const unsigned off = ok ? (unsigned)(((h0 + i) * p.W + w0) * C + f) * 2u : 0x80000000u;
            gx[l] = __builtin_amdgcn_raw_buffer_load_b16(rsrc, off, 0, 0);
        }
        const uint16_t* yb = p.dy + (((long long)img * p.P + ty * TH) * p.Q + tx * TW) * N;
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            const int id = tid + 256 * l, px = id >> 3, cq = id & 7;
            gy[l] = *reinterpret_cast<const u32x4*>(yb + ((long long)(px >> 4) * p.Q + (px & 15)) * N + cq * 8);
        }
    };
    auto sstore = [&]() {
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
#pragma unroll
        for (int l = 0; l < SLD; ++l) {
            const int e = tid + 256 * l, i = e / (SPX * C), f = e - i * (SPX * C), px = f / C, c = f - px * C;
            if (e < SR * SPX * C) slab[i * SPB + px * CP + c] = (uint16_t)gx[l];
        }
#pragma unroll
        for (int l = 0; l < 8; ++l) {
            const int id = tid + 256 * l, px = id >> 3, cq = id & 7;
            *reinterpret_cast<u32x4*>(&dys[px * PA + cq * 8]) = gy[l];
        }
    };

    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    // transposing read: within 16 lanes, lane i points at 4 consecutive elements of reduction row i / 4 (columns 4 * (i % 4) ..)
    // and receives column i of those 4 rows; lanes 16..31 the next 16 columns, lanes 32..63 the rows 8 further down
    const int tr_row = 8 * (lane >> 5) + ((lane & 15) >> 2), tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    auto tr4 = [&](const uint16_t* q) __attribute__((always_inline)) {
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)q);
    };
    const int a_lane = tr_row * PA + kt * 32 + tr_col;               // dY: reduction rows are the 16 pixels of an output row
    const int b_lane = tr_row * (ST * CP) + tr_col;                  // X: pixel i of the row sits 8 elements after pixel i - 1

    f32x16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    int tile = blockIdx.x;
    if (tile < tiles) gload(tile);
    for (; tile < tiles; tile += gridDim.x) {
        lds_barrier();                                                // everyone is done with the previous tile (and the clearing)
        sstore();
        lds_barrier();
        if (tile + (int)gridDim.x < tiles) gload(tile + gridDim.x);
#pragma unroll
        for (int py = 0; py < TH; ++py) {
            const uint16_t* qa = dys + py * TW * PA + a_lane;
            const s16x4 alo = tr4(qa), ahi = tr4(qa + 4 * PA);
            const s16x8 av = {alo[0], alo[1], alo[2], alo[3], ahi[0], ahi[1], ahi[2], ahi[3]};
            const bf16x8 a = __builtin_bit_cast(bf16x8, av);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (t < nr) {
                    const uint16_t* qb = slab + (ST * py + r0 + t) * SPB + b_lane;
                    const s16x4 blo = tr4(qb), bhi = tr4(qb + 4 * ST * CP);
                    const s16x8 bv = {blo[0], blo[1], blo[2], blo[3], bhi[0], bhi[1], bhi[2], bhi[3]};
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bv), acc[t], 0, 0, 0);
                }
            }
            if (py & 1) __builtin_amdgcn_sched_barrier(0);           // keep the reads of at most two rows in flight (registers)
        }
    }

    // each wave owns its (filters, filter rows) part of dW: column t' = s * 4 + c of filter row r -> element (r, s, c)
    float* part = p.part + (size_t)blockIdx.x * N * J;
    const int tq = lane & 31, s = tq >> 2, c = tq & 3;
#pragma unroll
    for (int t = 0; t < 4; ++t)
        if (t < nr && s < S && c < C) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kt * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                part[k * J + ((r0 + t) * S + s) * C + c] = acc[t][v];
            }
        }
}

}  // namespace

bool lc_conv_stem_f32_ok(int imgs, int c, int h, int w, int k, int r, int s, int sh, int sw, int ph, int pw, int P, int Q) {
    using namespace stem;
    if (getenv("LARSCONV_NO_STEM_DIRECT")) return false;                   // comparison runs
    if (c != C || k != N || r != R || s != S || sh != ST || sw != ST || ph != PAD || pw != PAD) return false;
    if (P % TH != 0 || Q % TW != 0) return false;
    // (buffer descriptors are per image for the filter gradient and over the whole input for the forward pass)
    return (long long)imgs * h * w * C * 4 < 0x7fff0000LL && (long long)P * Q * N * 4 < 0x7fff0000LL &&
           (long long)imgs * (P / TH) * (Q / TW) < 0x7fffffffLL / 4;
}

size_t lc_conv_stem_f32_stats_pieces(int imgs, int P, int Q) { return (size_t)imgs * (P / stem::TH) * (Q / stem::TW) * 4; }

// Resident blocks of both kernels: two per compute unit, each walks its tiles (a fixed function of the shape and the device:
// the plan sizes the partials of the filter gradient with it).
int lc_conv_stem_blocks(int imgs, int P, int Q) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    const long long tiles = (long long)imgs * (P / stem::TH) * (Q / stem::TW);
    return (int)(tiles < 2LL * cus ? tiles : 2LL * cus);
}

lc_status lc_launch_conv_stem_wgrad_f32(const StemWgrad& p, int blocks, hipStream_t stream) {
    using namespace stem;
    if (p.P % TH != 0 || p.Q % TW != 0 || blocks != lc_conv_stem_blocks(p.imgs, p.P, p.Q)) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(conv_stem_wgrad_f32_kernel, dim3((unsigned)blocks), dim3(256), (size_t)(2 * SLAB) * 4, stream, p);
    return lc_end_call();
}

lc_status lc_launch_conv_stem_wgrad_bf16(const StemWgradBf16& p, int blocks, hipStream_t stream) {
    using namespace stemwb;
    if (p.P % TH != 0 || p.Q % TW != 0 || blocks != lc_conv_stem_blocks(p.imgs, p.P, p.Q)) return LC_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(p.dy) & 15) || (reinterpret_cast<uintptr_t>(p.x) & 1)) return LC_ERR_ALIGN;
    hipLaunchKernelGGL(conv_stem_wgrad_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p);
    return lc_end_call();
}

lc_status lc_launch_conv_stem_bf16(const StemConvBf16& p, hipStream_t stream) {
    using namespace stemb;
    constexpr size_t lds = (size_t)(N * BP + 2 * SLAB) * 2;
    if (p.P % TH != 0 || p.Q % TW != 0) return LC_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.w)) & 1 || reinterpret_cast<uintptr_t>(p.y) & 3) return LC_ERR_ALIGN;
    const int blocks = lc_conv_stem_blocks(p.imgs, p.P, p.Q);
    hipLaunchKernelGGL(conv_stem_bf16_kernel, dim3((unsigned)blocks), dim3(256), lds, stream, p);
    return lc_end_call();
}

lc_status lc_launch_conv_stem_f32(const StemConv& p, hipStream_t stream) {
    using namespace stem;
    constexpr size_t lds = (size_t)(KP * N + 2 * SLAB) * 4;
    static bool once = [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(conv_stem_f32_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) ==
               hipSuccess;
    }();
    if (!once) return LC_ERR_LAUNCH;
    if (p.P % TH != 0 || p.Q % TW != 0) return LC_ERR_UNSUPPORTED;
    const int blocks = lc_conv_stem_blocks(p.imgs, p.P, p.Q);
    hipLaunchKernelGGL(conv_stem_f32_kernel, dim3((unsigned)blocks), dim3(256), lds, stream, p);
    return lc_end_call();
}
