// Declarations shared by the translation units of liblarsconv (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/larsconv.h"

// Launch bookkeeping (conv_api.hip).  lc_begin_call() drops any stale error another user of the HIP
// runtime left on this thread, so that lc_end_call() reports only what this library's launches caused.
void lc_begin_call();
lc_status lc_end_call();     // LC_OK, or LC_ERR_LAUNCH with the detail text recorded
lc_status lc_fail_call(hipError_t e, const char* what);   // records "what: error" as the detail text, returns LC_ERR_LAUNCH

// fp32 -> bf16, round to nearest even (NaN stays NaN): the conversion instruction of gfx950
__device__ __forceinline__ uint16_t lc_bf16_rne(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }
// two at once: lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t lc_bf16x2_rne(float lo, float hi) {
    typedef float lc_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 lc_bf16x2 __attribute__((ext_vector_type(2)));
    const lc_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, lc_bf16x2));
}

// ---- small device-side utilities (layout.hip) ----
void lc_bf16_to_f32(const void* src, float* dst, size_t count, hipStream_t stream);
void lc_f32_to_bf16(const float* src, void* dst, size_t count, hipStream_t stream);
void lc_fill_f32(float* dst, float value, size_t count, hipStream_t stream);
void lc_fill_u32x4(void* dst, size_t bytes16, hipStream_t stream);   // zero `bytes16` * 16 bytes
void lc_zero_bytes(void* dst, size_t bytes, hipStream_t stream);      // zero an even number of bytes at a 2-byte aligned address

// rows x width_bytes bytes from src (row pitch src_pitch bytes) to dst (row pitch dst_pitch); every size a multiple of 2
void lc_copy2d(const void* src, size_t src_pitch, void* dst, size_t dst_pitch, size_t width_bytes, size_t rows, hipStream_t stream);

// NCHW <-> NHWC for activations ([n][c][hw] <-> [n][hw][c]); esize 4 (fp32) or 2 (bf16).
void lc_nchw_to_nhwc(const void* src, void* dst, int n, int c, int hw, int esize, hipStream_t stream);
void lc_nhwc_to_nchw(const void* src, void* dst, int n, int c, int hw, int esize, hipStream_t stream);

// Filter re-ordering.  All take and give fp32 or bf16 by esize.
//  KRSC -> [c][R-1-r][S-1-s][k]  (the filter of the backward-data convolution)
void lc_filter_for_bwd_data(const void* w_krsc, void* out, int k, int c, int r, int s, int esize, hipStream_t stream);
//  the taps r = a, a + sh, ... / s = b, b + sw, ... of it (ra x sb of them) in the same order: one stride phase
void lc_filter_for_bwd_data_phase(const void* w_krsc, void* out, int k, int c, int r, int s, int a, int b, int sh, int sw, int ra,
                                  int sb, int esize, hipStream_t stream);
//  pad the channel dimension (innermost) of an [rows][c] array with zeros to [rows][cpad]
// few-channel stride-2 convolution as a stride-1 convolution over 2x2 pixel blocks (see layout.hip)
void lc_stem_unfold(const void* x, void* u, int n, int c, int h, int w, int q, int hb, int sb, int cu, int eph, int epw, int esize,
                    hipStream_t stream);
void lc_stem_filter(const void* w, void* wu, int k, int r, int s, int c, int rb, int sb, int cu, int eh, int ew, int esize,
                    hipStream_t stream);
void lc_stem_filter_grad(const float* dwu, float* dw, int k, int r, int s, int c, int rb, int cu, int eh, int ew, hipStream_t stream);
void lc_pad_channels(const void* src, void* dst, size_t rows, int c, int cpad, int esize, hipStream_t stream);

// dw[k][j] (j < cols, c index j % cpad < c kept) = sum over splits of part[z][k][cols] in index order.
// sq (may be null): one double per block of the reduction, lc_reduce_splits_blocks(rows_times_cols) of them, the sum of
// the squares of the values that block wrote to dw.
void lc_reduce_splits(const float* part, float* dw, int splits, size_t rows_times_cols, int cpad, int c, double* sq, hipStream_t stream);
size_t lc_reduce_splits_blocks(size_t rows_times_cols);
// sq[b] = sum of x[i]^2 over elements 4096*b .. 4096*b + 4095: lc_sq_partials_blocks(count) doubles
void lc_sq_partials(const float* x, size_t count, double* sq, hipStream_t stream);
size_t lc_sq_partials_blocks(size_t count);

// ---- implicit-GEMM convolution kernels (conv_igemm.hip) ----
// One problem D[m][n] = sum_kg A(m, kg) * B[n][kg] where A is gathered from an NHWC tensor:
// row m = (img, po, qo), column kg = (r, s, ci).
struct GemmConv {
    const void* a;      // gathered tensor [imgs][Hi][Wi][Ci]
    const void* b;      // [N][Kg], Kg = R*S*Ci contiguous
    void* d;            // output rows of ldd elements
    int M, N, Kg;
    int Hi, Wi, Ci;
    int Po, Qo;         // m -> (img, po, qo)
    int R, S;
    int sh, sw;         // position stride:  h = po*sh - ph + r
    int ph, pw;
    int dh, dw;         // > 1: "dilated" read, valid only where h % dh == 0, then h /= dh
    int ldd;
    // scatter epilogue (0 = off): row (img,po,qo) is pixel (po*esh, qo*esw) of an [imgs][Ho][Wo][ldd] tensor that
    // the caller has cleared; the pixels between the stride grid stay zero.
    int scatter, Ho, Wo, esh, esw;
    // stream-K split, filled in by the launcher: whole-tile blocks, blocks sharing the k-steps of the
    // remaining tiles, their total k-steps, and the workspace for partial tiles (2 slots per such block)
    int dp_tiles, sk_blocks;
    long long sk_iters;
    float* partial;
    // multiply-high division constants for Qo and Po (filled in by the launcher)
    unsigned qo_mul, qo_shift, po_mul, po_shift;
    int bf16;           // operands a, b and result d are bf16 (sums stay fp32)
    // not null (main and slab kernels, no scatter): [lc_conv_gemm_stats_tiles()][N][2] floats -- per half tile of rows and
    // per column, the sum and the sum of squares of the values stored to d (as stored: after rounding to bf16)
    float* stats;
};
lc_status lc_launch_conv_gemm(const GemmConv& p, hipStream_t stream);
size_t lc_conv_gemm_stats_tiles(const GemmConv& p);   // row pieces of `stats` for this problem; 0: the kernel that takes it has none
extern "C" int lc_selftest_division(int max_d);   // host check of the multiply-high division constants (0 = all good)
bool lc_conv_gemm_bf16_native(const GemmConv& p);   // can the bf16 MFMA kernel take this problem (shape and alignment)?
bool lc_conv_gemm_scatter_ok(const GemmConv& p);    // can the main kernel's scatter epilogue take this problem?
size_t lc_conv_gemm_workspace(const GemmConv& p);   // bytes `partial` must hold for this problem (0 = none)

// ResNet's first layer in fp32 (conv_stem.hip): 7x7, stride 2, padding 3, 3 -> 64 channels, NHWC, P and Q multiples of 16.
struct StemConv {
    const float* x;     // [imgs][H][W][3]
    const float* w;     // [64][7][7][3]
    float* y;           // [imgs][P][Q][64]
    float* stats;       // [pieces][64][2] (sum, sum of squares per piece of 64 pixels) or null
    int imgs, H, W, P, Q;
};
struct StemConvBf16 {
    const uint16_t* x;  // [imgs][H][W][3]
    const uint16_t* w;  // [64][7][7][3]
    uint16_t* y;        // [imgs][P][Q][64]
    float* stats;       // as StemConv
    int imgs, H, W, P, Q;
};
lc_status lc_launch_conv_stem_bf16(const StemConvBf16& p, hipStream_t stream);
struct StemWgrad {
    const float* x;     // [imgs][H][W][3]
    const float* dy;    // [imgs][P][Q][64]
    float* part;        // [blocks][64][147]: one partial filter gradient per block
    int imgs, H, W, P, Q;
};
struct StemWgradBf16 {
    const uint16_t* x;  // [imgs][H][W][3]
    const uint16_t* dy; // [imgs][P][Q][64]
    float* part;        // as StemWgrad
    int imgs, H, W, P, Q;
};
lc_status lc_launch_conv_stem_wgrad_bf16(const StemWgradBf16& p, int blocks, hipStream_t stream);
int lc_conv_stem_blocks(int imgs, int P, int Q);
lc_status lc_launch_conv_stem_wgrad_f32(const StemWgrad& p, int blocks, hipStream_t stream);
bool lc_conv_stem_f32_ok(int imgs, int c, int h, int w, int k, int r, int s, int sh, int sw, int ph, int pw, int P, int Q);
size_t lc_conv_stem_f32_stats_pieces(int imgs, int P, int Q);
lc_status lc_launch_conv_stem_f32(const StemConv& p, hipStream_t stream);

// Filter gradient: D[k][j] = sum_m dY[m][k] * Xg(m, j), m = (img, p, q), j = (r, s, c); the reduction
// over m is cut into `splits` ranges, split z writing to d + z * K * J.
struct GemmWgrad {
    const void* dy;     // [M][K]
    const void* x;      // [imgs][H][W][C]
    float* d;           // [splits][K][J]
    int M, K, J;
    int H, W, C, P, Q, R, S;
    int sh, sw, ph, pw;
    int splits, m_per_split;
    int bf16;           // dy and x are bf16 (widened on the fly; the sums and d stay fp32)
    int slab;           // 3x3 stride-1 pad-1 bf16 layer for wgrad3x3_slab_kernel: m_per_split counts padded positions
};
lc_status lc_launch_wgrad_f32(const GemmWgrad& p, hipStream_t stream);
int lc_wgrad_splits(int M, int K, int J, bool bf16);   // fixed function of the shape (determinism)
bool lc_wgrad_slab_ok(int imgs, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw, int P, int Q, bool bf16);
int lc_wgrad_slab_splits(int imgs, int H, int W, int C, int K, int* pos_per_split);
