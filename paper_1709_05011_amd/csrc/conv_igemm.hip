// Implicit-GEMM convolution kernels for gfx950 (fp32 operands, fp32 MFMA accumulation).
//
// Forward and backward-data run as  D[m][n] = sum_kg A(m,kg) * B[n][kg]  where row m is an output
// pixel (img, po, qo), column kg = (r, s, ci) walks the filter window with the channel innermost,
// and A(m,kg) is read straight from the NHWC activation tensor (zero outside the image): the
// im2col matrix is never written to memory, its tiles exist only in LDS.  Backward-weight runs as
// D[k][j] = sum_m dY[m][k] * X(m, j), a GEMM whose reduction runs over the batch and all output
// pixels, cut into splits that write separate partial tiles (summed afterwards in a fixed order).
//
// Tiling: a block of 4 waves owns a BM x BN tile of D; each wave owns (BM/2) x (BN/2) of it as
// 32x32 MFMA tiles (v_mfma_f32_32x32x2_f32: lane l feeds A[row l%32][k l/32] and B[k l/32][col l%32];
// it returns D[8*(v/4) + 4*(l/32) + v%4][l%32] in accumulator register v).  Operand tiles go
// global -> registers -> LDS with the next tile's global loads in flight while the current tile is
// multiplied (two LDS buffers, one barrier per k-step).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int VEC> struct VecT;
template <> struct VecT<4> {
    using type = float4;
    static __device__ __forceinline__ type zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
};
template <> struct VecT<1> {
    using type = float;
    static __device__ __forceinline__ type zero() { return 0.f; }
};

__device__ __forceinline__ float elem(const float4& v, int e) {
    return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
}

// Blocks are dealt round-robin to the 8 XCDs, each with its own L2.  Re-number them so that every
// XCD works on one contiguous run of tiles (neighbouring tiles share A rows and the whole filter).
__device__ __forceinline__ int xcd_tile(int bid, int total) {
    const int per = (total + 7) >> 3, rem = total & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    if (rem == 0 || xcd < rem) return xcd * per + idx;
    return rem * per + (xcd - rem) * (per - 1) + idx;
}

// ------------------------------------------------------------------------------------------------
// forward / backward-data kernel: both operands contiguous along the reduction index
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int WGM, int WGN, int VEC>
__global__ void __launch_bounds__(WGM* WGN * 64) conv_gemm_f32_kernel(const GemmConv p) {
    constexpr int T = WGM * WGN * 64;
    constexpr int KQ = BK / VEC;          // vectors per tile row
    constexpr int RPP = T / KQ;           // tile rows covered by one pass of the block
    constexpr int LA = BM / RPP, LB = BN / RPP;
    constexpr int PITCH = BK + 4;         // floats; keeps 16-byte alignment and spreads banks
    constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
    static_assert(T % KQ == 0 && BM % RPP == 0 && BN % RPP == 0 && BK % 8 == 0, "tile shape");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
    using V = typename VecT<VEC>::type;

    __shared__ __attribute__((aligned(16))) float As[2][BM * PITCH];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int nbn = (p.N + BN - 1) / BN;
    const int tile = xcd_tile(blockIdx.x, gridDim.x);
    const int m0 = (tile / nbn) * BM, n0 = (tile % nbn) * BN;

    const float* __restrict__ A = static_cast<const float*>(p.a);
    const float* __restrict__ B = static_cast<const float*>(p.b);
    const int kq = tid % KQ, lrow = tid / KQ;

    long long a_base[LA];
    int a_h[LA], a_w[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int m = m0 + lrow + i * RPP;
        if (m < p.M) {
            const int qo = m % p.Qo, t = m / p.Qo;
            const int po = t % p.Po, img = t / p.Po;
            a_h[i] = po * p.sh - p.ph;
            a_w[i] = qo * p.sw - p.pw;
            a_base[i] = (long long)img * p.Hi * p.Wi * p.Ci;
        } else {
            a_h[i] = -(1 << 28);          // every tap fails the bounds test
            a_w[i] = 0;
            a_base[i] = 0;
        }
    }
    long long b_off[LB];
    bool b_ok[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int n = n0 + lrow + i * RPP;
        b_ok[i] = n < p.N;
        b_off[i] = (long long)n * p.Kg;
    }

    // position of this thread's vector inside the filter window
    int kg = kq * VEC;
    int c = kg % p.Ci, r, s;
    {
        const int rs = kg / p.Ci;
        s = rs % p.S;
        r = rs / p.S;
    }
    const bool dilated = (p.dh > 1) | (p.dw > 1);

    V ra[LA], rb[LB];
    auto gload = [&]() {
        const bool kok = r < p.R;         // same as kg < Kg
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            int h = a_h[i] + r, w = a_w[i] + s;
            bool ok = kok && h >= 0 && w >= 0;
            if (dilated) {
                ok = ok && (h % p.dh == 0) && (w % p.dw == 0);
                h /= p.dh;
                w /= p.dw;
            }
            ok = ok && h < p.Hi && w < p.Wi;
            ra[i] = ok ? *reinterpret_cast<const V*>(A + a_base[i] + ((long long)h * p.Wi + w) * p.Ci + c)
                       : VecT<VEC>::zero();
        }
#pragma unroll
        for (int i = 0; i < LB; ++i)
            rb[i] = (b_ok[i] && kok) ? *reinterpret_cast<const V*>(B + b_off[i] + kg) : VecT<VEC>::zero();
    };
    auto advance = [&]() {
        kg += BK;
        c += BK;
        while (c >= p.Ci) {
            c -= p.Ci;
            if (++s == p.S) {
                s = 0;
                ++r;
            }
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<V*>(&As[buf][(lrow + i * RPP) * PITCH + kq * VEC]) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<V*>(&Bs[buf][(lrow + i * RPP) * PITCH + kq * VEC]) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // lanes 0-31 take k = 0..3 of each group of 8, lanes 32-63 take k = 4..7 (same split for A and B)
    const int frag = (lane & 31) * PITCH + 4 * (lane >> 5);
    auto compute = [&](int buf) {
        const float* as = &As[buf][wm * WTM * PITCH + frag];
        const float* bs = &Bs[buf][wn * WTN * PITCH + frag];
#pragma unroll
        for (int k8 = 0; k8 < BK / 8; ++k8) {
            float4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const float4*>(as + i * 32 * PITCH + k8 * 8);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const float4*>(bs + j * 32 * PITCH + k8 * 8);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(elem(a[i], e), elem(b[j], e), acc[i][j], 0, 0, 0);
        }
    };

    const int nkt = (p.Kg + BK - 1) / BK;
    gload();
    sstore(0);
    __syncthreads();
    int cur = 0;
    for (int kt = 0; kt < nkt; ++kt) {
        const bool more = kt + 1 < nkt;
        if (more) {
            advance();
            gload();
        }
        compute(cur);
        if (more) sstore(cur ^ 1);
        __syncthreads();
        cur ^= 1;
    }

    float* __restrict__ D = static_cast<float*>(p.d);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wm * WTM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (row >= p.M) continue;
            if (!p.scatter) {
                float* drow = D + (long long)row * p.ldd;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = n0 + wn * WTN + j * 32 + (lane & 31);
                    if (col < p.N) drow[col] = acc[i][j][v];
                }
            } else {
                const int qo = row % p.Qo, t = row / p.Qo;
                const int po = t % p.Po, img = t / p.Po;
                for (int dy = 0; dy < p.esh; ++dy) {
                    const int h = po * p.esh + dy;
                    if (h >= p.Ho) break;
                    for (int dx = 0; dx < p.esw; ++dx) {
                        const int w = qo * p.esw + dx;
                        if (w >= p.Wo) break;
                        float* drow = D + (((long long)img * p.Ho + h) * p.Wo + w) * p.ldd;
                        const bool corner = (dy | dx) == 0;
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            const int col = n0 + wn * WTN + j * 32 + (lane & 31);
                            if (col < p.N) drow[col] = corner ? acc[i][j][v] : 0.f;
                        }
                    }
                }
            }
        }
}

// ------------------------------------------------------------------------------------------------
// backward-weight kernel: both operands contiguous along their *output* index (k resp. c), the
// reduction index m strides over rows.  LDS holds [reduction][row] so that the row-contiguous
// global vectors are stored as they arrive and MFMA fragments are read with unit lane stride.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int WGM, int WGN, int VEC>
__global__ void __launch_bounds__(WGM* WGN * 64) wgrad_f32_kernel(const GemmWgrad p) {
    constexpr int T = WGM * WGN * 64;
    constexpr int AQ = BM / VEC, BQ = BN / VEC;       // vectors per reduction row
    constexpr int ARPP = T / AQ, BRPP = T / BQ;       // reduction rows per pass
    constexpr int LA = BK / ARPP, LB = BK / BRPP;
    constexpr int PA = BM + 4, PB = BN + 4;
    constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
    static_assert(T % AQ == 0 && T % BQ == 0 && BK % ARPP == 0 && BK % BRPP == 0 && BK % 2 == 0, "tile shape");
    static_assert(LA >= 1 && LB >= 1, "tile shape");
    using V = typename VecT<VEC>::type;

    __shared__ __attribute__((aligned(16))) float As[2][BK * PA];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK * PB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int nbn = (p.J + BN - 1) / BN;
    const int tile = blockIdx.x;
    const int k0 = (tile / nbn) * BM, j0 = (tile % nbn) * BN;
    const int z = blockIdx.y;
    const int m_begin = z * p.m_per_split;
    const int m_end = min(p.M, m_begin + p.m_per_split);

    const float* __restrict__ DY = static_cast<const float*>(p.dy);
    const float* __restrict__ X = static_cast<const float*>(p.x);

    // dY tile: column (output channel) fixed per thread
    const int a_cq = tid % AQ, a_kr = tid / AQ;
    const int a_col = k0 + a_cq * VEC;
    const bool a_ok = a_col < p.K;
    // X tile: column j = (r, s, c) fixed per thread
    const int b_cq = tid % BQ, b_kr = tid / BQ;
    const int b_col = j0 + b_cq * VEC;
    const bool b_ok = b_col < p.J;
    int fr, fs, fc;
    {
        const int rs = b_col / p.C;
        fc = b_col % p.C;
        fs = rs % p.S;
        fr = rs / p.S;
    }
    // (img, po, qo) of each reduction row this thread loads for the X tile
    int b_img[LB], b_p[LB], b_q[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int m = m_begin + b_kr + i * BRPP;
        b_q[i] = m % p.Q;
        const int t = m / p.Q;
        b_p[i] = t % p.P;
        b_img[i] = t / p.P;
    }
    int mt = m_begin;                     // first reduction row of the tile being loaded

    V ra[LA], rb[LB];
    auto gload = [&]() {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int m = mt + a_kr + i * ARPP;
            ra[i] = (a_ok && m < m_end) ? *reinterpret_cast<const V*>(DY + (long long)m * p.K + a_col) : VecT<VEC>::zero();
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int m = mt + b_kr + i * BRPP;
            const int h = b_p[i] * p.sh - p.ph + fr, w = b_q[i] * p.sw - p.pw + fs;
            const bool ok = b_ok && m < m_end && h >= 0 && h < p.H && w >= 0 && w < p.W;
            rb[i] = ok ? *reinterpret_cast<const V*>(X + (((long long)b_img[i] * p.H + h) * p.W + w) * p.C + fc)
                       : VecT<VEC>::zero();
        }
    };
    auto advance = [&]() {
        mt += BK;
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            b_q[i] += BK;
            while (b_q[i] >= p.Q) {
                b_q[i] -= p.Q;
                if (++b_p[i] == p.P) {
                    b_p[i] = 0;
                    ++b_img[i];
                }
            }
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<V*>(&As[buf][(a_kr + i * ARPP) * PA + a_cq * VEC]) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<V*>(&Bs[buf][(b_kr + i * BRPP) * PB + b_cq * VEC]) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    auto compute = [&](int buf) {
        const float* as = &As[buf][(lane >> 5) * PA + wm * WTM + (lane & 31)];
        const float* bs = &Bs[buf][(lane >> 5) * PB + wn * WTN + (lane & 31)];
#pragma unroll
        for (int k2 = 0; k2 < BK / 2; ++k2) {
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = as[2 * k2 * PA + i * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = bs[2 * k2 * PB + j * 32];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };

    const int nkt = (m_end - m_begin + BK - 1) / BK;
    if (nkt > 0) {
        gload();
        sstore(0);
        __syncthreads();
        int cur = 0;
        for (int kt = 0; kt < nkt; ++kt) {
            const bool more = kt + 1 < nkt;
            if (more) {
                advance();
                gload();
            }
            compute(cur);
            if (more) sstore(cur ^ 1);
            __syncthreads();
            cur ^= 1;
        }
    }

    float* __restrict__ D = p.d + (long long)z * p.K * p.J;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = k0 + wm * WTM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (row >= p.K) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = j0 + wn * WTN + j * 32 + (lane & 31);
                if (col < p.J) D[(long long)row * p.J + col] = acc[i][j][v];
            }
        }
}

inline bool aligned16(const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) == 0; }

template <int BM, int BN, int BK, int VEC>
lc_status launch_conv(const GemmConv& p, hipStream_t stream) {
    const long long tiles = (long long)((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffffLL) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((conv_gemm_f32_kernel<BM, BN, BK, 2, 2, VEC>), dim3((unsigned)tiles), dim3(256), 0, stream, p);
    return lc_end_call();
}

template <int BM, int BN, int BK, int VEC>
lc_status launch_wgrad(const GemmWgrad& p, hipStream_t stream) {
    const long long tiles = (long long)((p.K + BM - 1) / BM) * ((p.J + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffffLL || p.splits > 65535) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((wgrad_f32_kernel<BM, BN, BK, 2, 2, VEC>), dim3((unsigned)tiles, (unsigned)p.splits), dim3(256), 0,
                       stream, p);
    return lc_end_call();
}

}  // namespace

lc_status lc_launch_conv_gemm_f32(const GemmConv& p, hipStream_t stream) {
    const bool vec = (p.Ci % 4 == 0) && aligned16(p.a) && aligned16(p.b);
    if (!vec) return launch_conv<64, 64, 16, 1>(p, stream);
    if (p.N > 64) return launch_conv<128, 128, 16, 4>(p, stream);
    return launch_conv<128, 64, 16, 4>(p, stream);
}

// Output tile of the filter-gradient kernel for a shape (also fixes the split count).
static void wgrad_tile(int K, int J, int* bm, int* bn) {
    *bm = K > 64 ? 128 : 64;
    *bn = J > 64 ? 128 : 64;
}

int lc_wgrad_splits(int M, int K, int J) {
    int bm, bn;
    wgrad_tile(K, J, &bm, &bn);
    const long long tiles = (long long)((K + bm - 1) / bm) * ((J + bn - 1) / bn);
    long long want = (1024 + tiles - 1) / tiles;          // about four blocks per compute unit in total
    const long long most = (M + 255) / 256;               // at least 256 reduction rows per split
    if (want > most) want = most;
    if (want < 1) want = 1;
    if (want > 4096) want = 4096;
    return (int)want;
}

lc_status lc_launch_wgrad_f32(const GemmWgrad& p, hipStream_t stream) {
    const bool vec = (p.C % 4 == 0) && (p.K % 4 == 0) && aligned16(p.dy) && aligned16(p.x);
    int bm, bn;
    wgrad_tile(p.K, p.J, &bm, &bn);
    if (!vec) return launch_wgrad<64, 64, 16, 1>(p, stream);
    if (bm == 128 && bn == 128) return launch_wgrad<128, 128, 16, 4>(p, stream);
    if (bm == 128) return launch_wgrad<128, 64, 16, 4>(p, stream);
    if (bn == 128) return launch_wgrad<64, 128, 16, 4>(p, stream);
    return launch_wgrad<64, 64, 16, 4>(p, stream);
}
