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
#include <type_traits>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

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

// Write one wave's accumulators (TM x TN tiles of 32x32) to D: plain rows, or the scatter form used by
// the strided 1x1 backward-data pass.
// D holds fp32, or bf16 (rounded to nearest even) when BF16OUT.
template <bool BF16OUT> struct OutT { using type = float; static __device__ __forceinline__ float cvt(float x) { return x; } };
template <> struct OutT<true> {
    using type = uint16_t;
    static __device__ __forceinline__ uint16_t cvt(float x) { return lc_bf16_rne(x); }
};

template <int TM, int TN, bool BF16OUT = false>
__device__ __forceinline__ void store_tile(const GemmConv& p, const f32x16 (&acc)[TM][TN], int row0, int col0, int lane,
                                           int vsel = -1 /* >= 0: only accumulator register vsel of each tile */) {
    using O = typename OutT<BF16OUT>::type;
    O* __restrict__ D = static_cast<O*>(p.d);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            if (vsel >= 0 && v != vsel) continue;
            const int row = row0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (row >= p.M) continue;
            if (!p.scatter) {
                O* drow = D + (long long)row * p.ldd;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = col0 + j * 32 + (lane & 31);
                    if (col < p.N) drow[col] = OutT<BF16OUT>::cvt(acc[i][j][v]);
                }
            } else {
                // the row's pixel on the stride grid; the pixels between the grid belong to the caller (cleared, or
                // written by the other stride phases)
                const int qo = row % p.Qo, t = row / p.Qo;
                const int po = t % p.Po, img = t / p.Po;
                O* drow = D + (((long long)img * p.Ho + (long long)po * p.esh) * p.Wo + (long long)qo * p.esw) * p.ldd;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = col0 + j * 32 + (lane & 31);
                    if (col < p.N) drow[col] = OutT<BF16OUT>::cvt(acc[i][j][v]);
                }
            }
        }
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

    store_tile<TM, TN>(p, acc, m0 + wm * WTM, n0 + wn * WTN, lane);
}

// ------------------------------------------------------------------------------------------------
// Main forward / backward-data kernel (channel counts that are multiples of 4, no dilated read).
//
// LDS tile: [row][16 floats] unpadded; the four 16-byte chunks of a row are permuted by chunk ^ swz(row)
// so that the b128 fragment reads of 8 or 16 consecutive rows hit distinct banks.  The permutation is
// applied on the global side: the lane that owns LDS slot s of a row fetches chunk s ^ swz(row).
// Positions outside the image, rows past M or N and columns past Kg fetch from a 16-byte block of zeros
// instead, so every lane always loads and the loop has no branch.
//
// Pipeline per 16-wide k-step ("tile"): the tile two steps ahead travels global -> registers, the tile one
// step ahead registers -> LDS (two LDS buffers), fragments are double-buffered in registers so that the LDS
// reads of the next half-step and the global loads are issued in the shadow of the MFMAs.
//
// Work distribution ("stream-K"): the first dp_tiles output tiles are computed one per block.  The k-steps
// of the remaining tiles are laid end to end and cut into sk_blocks equal ranges, one per block, so that the
// last, partially filled round of blocks costs its share of the work instead of a whole round.  A block
// whose range covers only part of a tile's k-steps writes its accumulators to the workspace; a second small
// kernel adds the parts of each such tile in k order (fixed order: bit-identical reruns) and stores it.
// ------------------------------------------------------------------------------------------------
__device__ __attribute__((aligned(16))) const float g_zero_chunk[4] = {0.f, 0.f, 0.f, 0.f};

__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 2)) & 3; }

// ok ? a : b on pointers by bit masking: never a branch, whatever the cost of computing a
__device__ __forceinline__ const void* pick(bool ok, const void* a, const void* b) {
    const uintptr_t m = (uintptr_t)0 - (uintptr_t)ok;
    return reinterpret_cast<const void*>((reinterpret_cast<uintptr_t>(a) & m) | (reinterpret_cast<uintptr_t>(b) & ~m));
}
// 16-byte load through the global (not flat) path: a flat load would also count as an LDS operation
__device__ __forceinline__ float4 load_global16(const void* ptr) {
    typedef float gf4 __attribute__((ext_vector_type(4)));
    const gf4 v = *(const __attribute__((address_space(1))) gf4*)(uintptr_t)ptr;
    return make_float4(v.x, v.y, v.z, v.w);
}
// This wave's LDS writes and reads are complete, then the workgroup barrier.  Global loads stay in flight
// (__syncthreads() would wait for them too).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory"); }

// Accumulators of one wave <-> a partial-tile slot in the workspace, in register order: every store
// instruction writes 64 consecutive floats.
template <int TM, int TN>
__device__ __forceinline__ size_t partial_index(int wave, int i, int j, int v, int lane) {
    return ((((size_t)wave * TM + i) * TN + j) * 16 + v) * 64 + lane;
}

// BF16: operands are bf16 (8 per 16-byte chunk, k-step 32), multiplied with v_mfma_f32_32x32x16_bf16 (lane l
// feeds A[row l%32][k 8*(l/32) .. +7], i.e. exactly one LDS chunk per MFMA); the result is stored as bf16.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// UT ("uniform tap"): the channel count is a multiple of the k-step, so a k-step lies inside one filter tap
// and its (r, s, first channel) are the same for every lane.  They are then tracked in scalar registers, the
// operands are fetched with buffer loads (tile-relative 32-bit byte offset per lane + scalar offset of the
// k-step), and a tap outside the image is a bit in a per-row mask that moves the lane's offset past the end
// of the buffer, where the hardware returns zeros.  That leaves two vector ALU instructions per activation
// load in the main loop; on this chip every vector ALU instruction displaces MFMA issue time.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned kBufferWords3 = 0x00020000u;       // raw buffer, 32-bit data format
constexpr unsigned kBufferBytes = 0x80000000u;        // buffer size given to the hardware; offsets with bit 31 set read zeros

// ------------------------------------------------------------------------------------------------
// Persistent form of the main kernel.  The grid is one round of resident blocks; each block walks its own
// sequence of segments -- whole tiles (one per round of the launch), then its share of the stream-K
// k-steps -- as ONE software pipeline: the loads run two k-steps ahead of the MFMAs straight across tile
// boundaries, so the memory latency at the start of a tile and the stores at its end are covered by MFMAs
// of neighbouring tiles instead of standing alone.  What is paid once per tile is kept off the vector ALU
// (every vector ALU instruction displaces MFMA issue time on this chip, and layers with few k-steps pay it
// often): index arithmetic uses multiply-high division with constants from the host, and the tile is stored with buffer stores
// whose row part of the address is a scalar offset and whose bounds are the buffer's size (rows) and bit 31
// of the lane offset (columns).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int div_by(int n, unsigned mul, unsigned shift) {       // n / d for 0 <= n < 2^31, see magic_for()
    return mul ? (int)(__umulhi((unsigned)n, mul) >> shift) : n;
}

// Blocks per compute unit: 3 for tiles up to 128x128 (64 accumulator registers per lane), 2 for the 128x256 tile, 1 for
// the 256x256 tile (run by eight waves, two per SIMD, each with 128 accumulator registers).
constexpr int pk_blocks_per_cu(int bm, int bn) { return bm * bn >= 256 * 256 ? 1 : bm * bn > 128 * 128 ? 2 : 3; }
// Waves along the columns of the tile: 2 (a 2 x 2 block of waves), or 4 for the 256x256 tile (2 x 4 waves of 128 x 64).
constexpr int pk_waves_n(int bm, int bn) { return bm * bn >= 256 * 256 ? 4 : 2; }

template <int BM, int BN, bool SMALLC, bool BF16, bool UT, bool SCATTER>
__global__ void __launch_bounds__(2 * pk_waves_n(BM, BN) * 64, pk_blocks_per_cu(BM, BN) * pk_waves_n(BM, BN) / 2)
conv_gemm_pk_kernel(const GemmConv p) {
    using E = typename OutT<BF16>::type;
    constexpr int ES = (int)sizeof(E);
    constexpr int EPC = BF16 ? 8 : 4;
    constexpr int BK = 4 * EPC;
    constexpr int WN_ = pk_waves_n(BM, BN), NWV = 2 * WN_;              // waves: 2 along the rows x WN_ along the columns
    constexpr int LA = BM / (16 * NWV), LB = BN / (16 * NWV), LPT = LA + LB;
    constexpr int WTM = BM / 2, WTN = BN / WN_, TM = WTM / 32, TN = WTN / 32;
    constexpr int STAGE = (BM + BN) * 16;
    static_assert(BM % (16 * NWV) == 0 && BN % (16 * NWV) == 0 && WTM % 32 == 0 && WTN % 32 == 0, "tile shape");

    __shared__ __attribute__((aligned(1024))) float lds[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN_, wn = wave % WN_;
    const int nbn = (p.N + BN - 1) / BN;
    const int nkt = (p.Kg + BK - 1) / BK;
    const E* __restrict__ A = static_cast<const E*>(p.a);
    const E* __restrict__ B = static_cast<const E*>(p.b);
    const int lrow = lane >> 2;
    const int kq = (lane & 3) ^ swz(lrow);
    const int Hi_ = p.Hi, Wi_ = p.Wi, Ci_ = p.Ci, R_ = p.R, S_ = p.S, M_ = p.M, N_ = p.N, Kg_ = p.Kg, ldd_ = p.ldd;
    const int sh_ = p.sh, sw_ = p.sw, ph_ = p.ph, pw_ = p.pw, Po_ = p.Po;
    const unsigned qmul = p.qo_mul, qsh = p.qo_shift, pmul = p.po_mul, psh = p.po_shift;
    const int Qo_ = p.Qo;
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = swz(frow);
    const int a_frag = (wm * WTM + frow) * 16, b_frag = BM * 16 + (wn * WTN + frow) * 16;

    // ---- this block's segments: `rounds` whole tiles, then its stream-K range cut at the tile boundaries ----
    const int G = gridDim.x, bid = blockIdx.x;
    const int rounds = p.dp_tiles / G;                     // the launcher makes dp_tiles a multiple of the grid
    int sk_it = 0, sk_len = 0;
    if (bid < p.sk_blocks) {
        sk_it = (int)((long long)bid * p.sk_iters / p.sk_blocks);
        sk_len = (int)((long long)(bid + 1) * p.sk_iters / p.sk_blocks) - sk_it;
    }
    const int sk_tile = sk_it / nkt, sk_k0 = sk_it - sk_tile * nkt;
    const int F = rounds * nkt + sk_len;                   // k-steps this block runs
    if (F == 0) return;
    auto segment = [&](int s, int& tile, int& k0, int& k1) __attribute__((always_inline)) {
        if (s < rounds) {
            tile = xcd_tile(s * G + bid, p.dp_tiles);
            k0 = 0;
            k1 = nkt;
        } else {                                           // piece s - rounds of the stream-K range
            const int t = sk_tile + (s - rounds);
            tile = p.dp_tiles + t;
            k0 = s == rounds ? sk_k0 : 0;
            k1 = min(nkt, sk_it + sk_len - t * nkt);
        }
    };

    // ---------------- load side ----------------
    int l_seg = -1, l_k = 0, l_k1 = 0;                     // segment being loaded, next k-step, end
    // generic addressing (pointer per row, position in the window per lane)
    long long a_base[LA];
    int a_h[LA], a_w[LA];
    long long b_off[LB];
    int kg = 0, c = 0, r = 0, s = 0;
    // uniform-tap addressing
    unsigned a_voff[LA], a_inv[LA], b_voff[LB];
    __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, 0, (int)kBufferWords3);
    __amdgpu_buffer_rsrc_t b_rsrc = a_rsrc;
    int u_kt = 0, u_c = 0, u_s = 0, u_r = 0;

    auto loader_setup = [&](int tile, int k0) __attribute__((always_inline)) {
        const int tm = tile / nbn;
        const int m0 = tm * BM, n0 = (tile - tm * nbn) * BN;
        if constexpr (UT) {
            const int pq = Po_ * Qo_;
            const int img0 = m0 / pq;
            const int phb = max(ph_, 0), pwb = max(pw_, 0);
            const int taps = R_ * S_;
            const unsigned full = taps >= 32 ? ~0u : (1u << taps) - 1u;
            unsigned rep = 0;
            for (int rr = 0; rr < R_; ++rr) rep |= 1u << (rr * S_);
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                const int m = m0 + (i * NWV + wave) * 16 + lrow;
                const int t = div_by(m, qmul, qsh), qo = m - t * Qo_;
                const int img = div_by(t, pmul, psh), po = t - img * Po_;
                const int h0 = po * sh_ - ph_, w0 = qo * sw_ - pw_;
                // taps of this pixel's window inside the image: rows rlo..rhi, columns slo..shi
                int rlo = max(0, -h0), rhi = min(R_ - 1, Hi_ - 1 - h0);
                int slo = max(0, -w0), shi = min(S_ - 1, Wi_ - 1 - w0);
                const bool ok = (m < M_) & (rlo <= rhi) & (slo <= shi);
                rlo = min(rlo, R_ - 1);
                rhi = max(rhi, 0);
                slo = min(slo, S_ - 1);
                const int sspan = max(shi - slo, 0);
                const unsigned hm = (full << (rlo * S_)) & (full >> ((R_ - 1 - rhi) * S_));
                const unsigned wmk = rep * (((2u << sspan) - 1u) << slo);
                a_inv[i] = ok ? ~(hm & wmk) : ~0u;
                a_voff[i] = ok ? (unsigned)(((((img - img0) * Hi_ + h0 + phb) * Wi_) + w0 + pwb) * Ci_ * ES + kq * 16) : 0u;
            }
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                const int nl = (i * NWV + wave) * 16 + lrow;
                b_voff[i] = (n0 + nl < N_) ? (unsigned)(nl * Kg_ * ES + kq * 16) : kBufferBytes;
            }
            const long long a_first = ((long long)img0 * Hi_ * Wi_ - ((long long)phb * Wi_ + pwb)) * Ci_;
            a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(A + a_first), 0, (int)kBufferBytes, (int)kBufferWords3);
            b_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(B + (long long)n0 * Kg_), 0, (int)kBufferBytes, (int)kBufferWords3);
            u_kt = k0;
            const int kg0 = k0 * BK, rs0 = kg0 / Ci_;
            u_c = kg0 - rs0 * Ci_;
            u_r = rs0 / S_;
            u_s = rs0 - u_r * S_;
        } else {
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                const int m = m0 + (i * NWV + wave) * 16 + lrow;
                if (m < M_) {
                    const int t = div_by(m, qmul, qsh), qo = m - t * Qo_;
                    const int img = div_by(t, pmul, psh), po = t - img * Po_;
                    a_h[i] = po * sh_ - ph_;
                    a_w[i] = qo * sw_ - pw_;
                    a_base[i] = (long long)img * Hi_ * Wi_ * Ci_;
                } else {
                    a_h[i] = -(1 << 28);              // every tap fails the bounds test
                    a_w[i] = 0;
                    a_base[i] = 0;
                }
            }
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                const int n = n0 + (i * NWV + wave) * 16 + lrow;
                b_off[i] = n < N_ ? (long long)n * Kg_ : -1;
            }
            kg = k0 * BK + kq * EPC;
            const int rs = kg / Ci_;
            c = kg - rs * Ci_;
            r = rs / S_;
            s = rs - r * S_;
        }
    };

    float4 g[LPT];                                // the k-step in flight between global memory and LDS
    auto gload_tile = [&]() __attribute__((always_inline)) {
        if constexpr (UT) {
            const int tap = u_r * S_ + u_s;
            const unsigned up = 31u - (unsigned)tap;
            const int a_soff = ((u_r * Wi_ + u_s) * Ci_ + u_c) * ES;
            const int b_soff = u_kt * BK * ES;
#pragma unroll
            for (int l = 0; l < LA; ++l) {
                const unsigned vo = ((a_inv[l] << up) & kBufferBytes) | a_voff[l];
                g[l] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)vo, a_soff, 0));
            }
#pragma unroll
            for (int l = 0; l < LB; ++l)
                g[LA + l] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, (int)b_voff[l], b_soff, 0));
            ++u_kt;
            u_c += BK;
            const bool wrap = u_c == Ci_;
            u_c = wrap ? 0 : u_c;
            u_s += wrap ? 1 : 0;
            const bool wrap2 = u_s == S_;
            u_s = wrap2 ? 0 : u_s;
            u_r += wrap2 ? 1 : 0;
        } else {
            const bool kok = r < R_;              // same as kg < Kg
#pragma unroll
            for (int l = 0; l < LA; ++l) {
                const int h = a_h[l] + r, w = a_w[l] + s;
                const bool ok = kok & ((unsigned)h < (unsigned)Hi_) & ((unsigned)w < (unsigned)Wi_);
                g[l] = load_global16(pick(ok, A + a_base[l] + ((long long)h * Wi_ + w) * Ci_ + c, g_zero_chunk));
            }
#pragma unroll
            for (int l = 0; l < LB; ++l)
                g[LA + l] = load_global16(pick(kok & (b_off[l] >= 0), B + b_off[l] + kg, g_zero_chunk));
            kg += BK;
            c += BK;
            if (SMALLC) {
                while (c >= Ci_) {
                    c -= Ci_;
                    if (++s == S_) {
                        s = 0;
                        ++r;
                    }
                }
            } else {
                const bool wrap = c >= Ci_;
                c = wrap ? c - Ci_ : c;
                s += wrap ? 1 : 0;
                const bool wrap2 = s == S_;
                s = wrap2 ? 0 : s;
                r += wrap2 ? 1 : 0;
            }
        }
    };
    // fetch the next k-step of the block's sequence (the caller knows there is one)
    auto load_step = [&]() __attribute__((always_inline)) {
        if (l_k == l_k1) {
            int tile;
            ++l_seg;
            segment(l_seg, tile, l_k, l_k1);
            loader_setup(tile, l_k);
        }
        gload_tile();
        ++l_k;
    };
    auto sstore = [&](int buf) __attribute__((always_inline)) {
        float* base = lds + buf * STAGE + wave * 256 + lane * 4;
#pragma unroll
        for (int l = 0; l < LPT; ++l)
            *reinterpret_cast<float4*>(base + (l < LA ? l * (NWV * 256) : BM * 16 + (l - LA) * (NWV * 256))) = g[l];
    };

    // ---------------- compute side ----------------
    f32x16 acc[TM][TN];
    float4 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int buf, int k8, int slot) __attribute__((always_inline)) {
        const float* base = lds + buf * STAGE;
        const int ch = ((2 * k8 + fhalf) ^ fsw) * 4;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[slot][i] = *reinterpret_cast<const float4*>(base + a_frag + i * 32 * 16 + ch);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[slot][j] = *reinterpret_cast<const float4*>(base + b_frag + j * 32 * 16 + ch);
    };
    // one group of MFMAs: every 32x32 tile of the wave advanced by one k-slice
    auto mfma_group = [&](int slot, int e) __attribute__((always_inline)) {
        if (BF16 && e != 0) return;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (BF16)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[slot][i]),
                                                                        __builtin_bit_cast(bf16x8, fb[slot][j]), acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(elem(fa[slot][i], e), elem(fb[slot][j], e), acc[i][j], 0, 0, 0);
            }
    };
    auto clear_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    };

    int c_seg = 0, c_tile, c_k0, c_k, c_k1;
    segment(0, c_tile, c_k0, c_k1);
    c_k = c_k0;
    // store (or park) the finished segment
    auto epilogue = [&]() __attribute__((always_inline)) {
        const int tm = c_tile / nbn;
        const int m0 = tm * BM, n0 = (c_tile - tm * nbn) * BN;
        if (c_k0 == 0 && c_k1 == nkt) {
            if constexpr (SCATTER) {
                // Row (img, po, qo) of the GEMM is pixel (po*esh, qo*esw) of image img in the [imgs][Ho][Wo][ldd] result;
                // the pixels between the stride grid are zero and were cleared by the caller before the launch.  An
                // accumulator register holds one row in lanes 0..31 and the row four further down in lanes 32..63;
                // rows are wave-uniform, so their pixel offsets (relative to the tile's first pixel) are computed
                // on the scalar unit and each lane picks its own.
                const int Ho_ = p.Ho, Wo_ = p.Wo, esh_ = p.esh, esw_ = p.esw;
                int t0 = div_by(m0, qmul, qsh);
                const int q0 = m0 - t0 * Qo_, i0 = div_by(t0, pmul, psh), p0 = t0 - i0 * Po_;
                const long long first_px = ((long long)i0 * Ho_ + p0 * esh_) * Wo_ + q0 * esw_;
                const __amdgpu_buffer_rsrc_t d_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)(static_cast<E*>(p.d) + first_px * ldd_), 0, (int)kBufferBytes, (int)kBufferWords3);
                auto px_off = [&](int m) __attribute__((always_inline)) {        // scalar: byte offset of row m's pixel
                    const int t = div_by(m, qmul, qsh), qo = m - t * Qo_;
                    const int img = div_by(t, pmul, psh), po = t - img * Po_;
                    const long long px = ((long long)img * Ho_ + po * esh_) * Wo_ + qo * esw_;
                    return (unsigned)((int)(px - first_px) * ldd_ * ES);
                };
                const bool hi = lane >= 32;
                const int odd = lane & 1;
                const bool pairs = BF16 && ((N_ | ldd_) & 1) == 0;
                if (m0 + BM <= M_) {
                    unsigned colpart[TN];                       // bit 31 past N: stays set after a pixel offset is added
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int col = n0 + wn * WTN + j * 32 + (lane & 31);
                        colpart[j] = col < N_ ? (unsigned)((pairs ? (col & ~1) : col) * ES) : kBufferBytes;
                    }
                    const unsigned perm_sel = odd ? 0x03020706u : 0x05040100u;
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int v = 0; v < 16; v += 2) {
                            const int m = m0 + wm * WTM + i * 32 + 8 * (v >> 2) + (v & 3);
                            const unsigned o0 = px_off(m), o1 = px_off(m + 1), o4 = px_off(m + 4), o5 = px_off(m + 5);
                            const unsigned row_a = hi ? o4 : o0, row_b = hi ? o5 : o1;     // rows of registers v and v + 1
#pragma unroll
                            for (int j = 0; j < TN; ++j) {
                                if constexpr (BF16) {
                                    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                                    typedef float f32x2 __attribute__((ext_vector_type(2)));
                                    const f32x2 pr = {acc[i][j][v], acc[i][j][v + 1]};
                                    const unsigned u = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, bf16x2));
                                    if (pairs) {                // as in the plain tile store: a lane stores a column pair of one row
                                        const unsigned got = (unsigned)__builtin_amdgcn_mov_dpp((int)u, 0xB1 /* quad_perm 1,0,3,2 */, 0xF, 0xF, true);
                                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_amdgcn_perm(got, u, perm_sel), d_rsrc,
                                                                              (int)(colpart[j] + (odd ? row_b : row_a)), 0, 0);
                                    } else {
                                        __builtin_amdgcn_raw_buffer_store_b16((short)(u & 0xffffu), d_rsrc, (int)(colpart[j] + row_a), 0, 0);
                                        __builtin_amdgcn_raw_buffer_store_b16((short)(u >> 16), d_rsrc, (int)(colpart[j] + row_b), 0, 0);
                                    }
                                } else {
                                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][v]), d_rsrc, (int)(colpart[j] + row_a), 0, 0);
                                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][v + 1]), d_rsrc, (int)(colpart[j] + row_b), 0, 0);
                                }
                            }
                        }
                } else {
                    // the last tile along M: rows are checked one by one on the scalar unit, each half of the wave is
                    // stored by its own instruction with the other half's lanes parked past the end of the buffer
                    unsigned d_voff[2][TN];
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int col = n0 + wn * WTN + j * 32 + (lane & 31);
                        d_voff[0][j] = (col < N_ && !hi) ? (unsigned)(col * ES) : kBufferBytes;
                        d_voff[1][j] = (col < N_ && hi) ? (unsigned)(col * ES) : kBufferBytes;
                    }
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
#pragma unroll
                            for (int hs = 0; hs < 2; ++hs) {
                                const int m = m0 + wm * WTM + i * 32 + 8 * (v >> 2) + 4 * hs + (v & 3);
                                if (m >= M_) continue;
                                const int soff = (int)px_off(m);
#pragma unroll
                                for (int j = 0; j < TN; ++j) {
                                    if constexpr (BF16)
                                        __builtin_amdgcn_raw_buffer_store_b16((short)lc_bf16_rne(acc[i][j][v]), d_rsrc, (int)d_voff[hs][j], soff, 0);
                                    else
                                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][v]), d_rsrc, (int)d_voff[hs][j], soff, 0);
                                }
                            }
                }
            } else {
                // rows: scalar offset, cut off at M by the size of the buffer; columns: lane offset, bit 31 past N
                const long long rows_left = (long long)(M_ - m0) * ldd_ * ES;
                const __amdgpu_buffer_rsrc_t d_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)(static_cast<E*>(p.d) + (long long)m0 * ldd_), 0, (int)(rows_left > 0x7fffffffLL ? 0x7fffffffLL : rows_left),
                    (int)kBufferWords3);
                // bf16 with an even row length: neighbouring lanes (neighbouring columns) trade values so that every
                // lane stores a pair of columns as one dword -- even lanes for row r0, odd lanes for row r0 + 1.
                const bool pairs = BF16 && ((N_ | ldd_) & 1) == 0;
                const int odd = lane & 1;
                unsigned d_voff[TN];
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = n0 + wn * WTN + j * 32 + (lane & 31);
                    d_voff[j] = col < N_ ? (unsigned)((4 * (lane >> 5) * ldd_ + col) * ES) : kBufferBytes;
                    if (pairs && col < N_) d_voff[j] = (unsigned)(((4 * (lane >> 5) + odd) * ldd_ + (col & ~1)) * ES);
                }
                // byte selectors of v_perm_b32 over {received, own}: even lanes keep their low half and take the
                // neighbour's low half above it; odd lanes take the neighbour's high half below their own high half
                const unsigned perm_sel = odd ? 0x03020706u : 0x05040100u;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int v = 0; v < 16; v += 2) {
                        // accumulator registers v and v + 1 are rows r0 and r0 + 1 of the same column
                        const int r0 = wm * WTM + i * 32 + 8 * (v >> 2) + (v & 3);
                        const int soff = r0 * ldd_ * ES;
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            if constexpr (BF16) {
                                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                                typedef float f32x2 __attribute__((ext_vector_type(2)));
                                const f32x2 pr = {acc[i][j][v], acc[i][j][v + 1]};
                                const unsigned u = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, bf16x2));
                                if (pairs) {
                                    // u = {row r0 | row r0 + 1} of this lane's column; swap with the neighbouring lane
                                    const unsigned got = (unsigned)__builtin_amdgcn_mov_dpp((int)u, 0xB1 /* quad_perm 1,0,3,2 */, 0xF, 0xF, true);
                                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_amdgcn_perm(got, u, perm_sel), d_rsrc, (int)d_voff[j], soff, 0);
                                } else {
                                    __builtin_amdgcn_raw_buffer_store_b16((short)(u & 0xffffu), d_rsrc, (int)d_voff[j], soff, 0);
                                    __builtin_amdgcn_raw_buffer_store_b16((short)(u >> 16), d_rsrc, (int)d_voff[j], soff + ldd_ * ES, 0);
                                }
                            } else {
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][v]), d_rsrc, (int)d_voff[j], soff, 0);
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][v + 1]), d_rsrc, (int)d_voff[j], soff + ldd_ * ES, 0);
                            }
                        }
                    }
            }
            if constexpr (!SCATTER) {
                if (p.stats) {
                    // Per column, the sum and the sum of squares of what this wave has just stored (the values as stored:
                    // rounded where the result is bf16) over its WTM rows; rows past M count as zero.  A lane holds 16 rows
                    // of a column per 32x32 tile, the other half of the wave the other 16.
                    typedef float flt2 __attribute__((ext_vector_type(2)));
                    flt2* st = reinterpret_cast<flt2*>(p.stats) + (size_t)(tm * 2 + wm) * N_;
                    const bool ragged = m0 + BM > M_;
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        float sum = 0.f, sq = 0.f;
#pragma unroll
                        for (int i = 0; i < TM; ++i)
#pragma unroll
                            for (int v = 0; v < 16; v += 2) {
                                float x0 = acc[i][j][v], x1 = acc[i][j][v + 1];
                                if constexpr (BF16) {
                                    const unsigned u = lc_bf16x2_rne(x0, x1);
                                    x0 = __uint_as_float(u << 16);
                                    x1 = __uint_as_float(u & 0xffff0000u);
                                }
                                if (ragged) {
                                    const int row = m0 + wm * WTM + i * 32 + 8 * (v >> 2) + 4 * fhalf + (v & 3);
                                    if (row >= M_) x0 = 0.f;
                                    if (row + 1 >= M_) x1 = 0.f;
                                }
                                sum += x0;
                                sq = fmaf(x0, x0, sq);
                                sum += x1;
                                sq = fmaf(x1, x1, sq);
                            }
                        sum += __shfl_xor(sum, 32);
                        sq += __shfl_xor(sq, 32);
                        const int col = n0 + wn * WTN + j * 32 + frow;
                        if (fhalf == 0 && col < N_) st[col] = flt2{sum, sq};
                    }
                }
            }
        } else {
            // part of a tile: it is the first piece of this block's stream-K range (slot 2*bid) or the last (2*bid + 1)
            float* part = p.partial + ((size_t)2 * bid + (c_seg == rounds ? 0 : 1)) * (BM * BN);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) part[partial_index<TM, TN>(wave, i, j, v, lane)] = acc[i][j][v];
        }
    };

    // ---------------- the pipeline ----------------
    load_step();                                  // k-step 0 of the sequence
    sstore(0);
    if (F > 1) load_step();                       // k-step 1
    clear_acc();
    lds_barrier();
    read_frags(0, 0, 0);
    // One k-step out of LDS buffer `cur` (a literal at both calls)
    auto step = [&](int cur, int f) __attribute__((always_inline)) {
        read_frags(cur, 1, 1);
        mfma_group(0, 0);
        mfma_group(0, 1);
        __builtin_amdgcn_sched_barrier(0);
        sstore(cur ^ 1);                          // k-step f + 1: its buffer was last read one step ago
        mfma_group(0, 2);
        __builtin_amdgcn_sched_barrier(0);
        if (f + 2 < F) load_step();               // k-step f + 2 into the registers just stored
        mfma_group(0, 3);
        __builtin_amdgcn_sched_barrier(0);
        lds_barrier();
        read_frags(cur ^ 1, 0, 0);                // first half of k-step f + 1
#pragma unroll
        for (int e = 0; e < 4; ++e) mfma_group(1, e);
        if (++c_k == c_k1) {                      // the segment is complete: store it, the next step starts a new one
            __builtin_amdgcn_sched_barrier(0);
            epilogue();
            clear_acc();
            ++c_seg;
            segment(c_seg, c_tile, c_k0, c_k1);
            c_k = c_k0;
        }
    };
    // The last step runs through the same code: what it stores to LDS, reads back as "next" fragments and
    // takes as the next segment is never used.
    for (int f = 0; f < F; f += 2) {
        step(0, f);
        if (f + 1 < F) step(1, f + 1);
    }
}

// Adds the parts of every tile that stream-K blocks split between them, in k order, and stores the tile.
// Block (t, v) handles accumulator register v of every 32x32 MFMA tile of stream-K tile t, with the thread
// geometry of the main kernel: 16 blocks per tile keep the whole chip busy on what is a small reduction.
template <int BM, int BN, bool BF16>
__global__ void __launch_bounds__(2 * pk_waves_n(BM, BN) * 64) conv_gemm_fixup_kernel(const GemmConv p) {
    constexpr int WN_ = pk_waves_n(BM, BN);
    constexpr int BK = BF16 ? 32 : 16, TM = BM / 64, TN = BN / (32 * WN_);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WN_, wn = wave % WN_;
    const int v = blockIdx.y;
    const int nbn = (p.N + BN - 1) / BN;
    const int nkt = (p.Kg + BK - 1) / BK;
    const long long tb = (long long)blockIdx.x * nkt, te = tb + nkt;      // this tile's k-steps in stream-K positions
    auto begin_of = [&](long long j) { return j * p.sk_iters / p.sk_blocks; };
    long long j = tb * p.sk_blocks / p.sk_iters;
    while (j > 0 && begin_of(j) > tb) --j;
    while (begin_of(j + 1) <= tb) ++j;
    if (begin_of(j) <= tb && begin_of(j + 1) >= te) return;              // one block did the whole tile and stored it

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jj = 0; jj < TN; ++jj) acc[i][jj][0] = 0.f;
    for (; j < p.sk_blocks && begin_of(j) < te; ++j) {
        const bool first_of_block = begin_of(j) >= tb;                   // the segment starts where the block's range starts
        const float* part = p.partial + ((size_t)2 * j + (first_of_block ? 0 : 1)) * (BM * BN);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int jj = 0; jj < TN; ++jj) acc[i][jj][0] += part[partial_index<TM, TN>(wave, i, jj, v, lane)];
    }
    // move the sums to register position v, where store_tile expects them
    f32x16 out[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jj = 0; jj < TN; ++jj)
#pragma unroll
            for (int u = 0; u < 16; ++u) out[i][jj][u] = acc[i][jj][0];
    const int tile = p.dp_tiles + blockIdx.x;
    const int m0 = (tile / nbn) * BM, n0 = (tile % nbn) * BN;
    store_tile<TM, TN, BF16>(p, out, m0 + wm * (BM / 2), n0 + wn * (BN / WN_), lane, v);
}

// The column sums of the tiles that stream-K blocks shared (the main kernel sums the tiles it stores whole): block
// (t, h) reads the rows of half h of tile first_tile + t back from d.  VEC4: a thread owns four neighbouring columns and
// every (256 / (bn / 4))-th row (one 16- or 8-byte load each, all independent), the rows of a column group are then
// added in order through LDS; otherwise one thread per column walks the rows.
template <bool BF16, bool VEC4>
__global__ void __launch_bounds__(256) tile_stats_kernel(const GemmConv p, int bm, int bn, int first_tile) {
    using E = typename OutT<BF16>::type;
    typedef float flt2 __attribute__((ext_vector_type(2)));
    const int nbn = (p.N + bn - 1) / bn;
    const int tile = first_tile + blockIdx.x, tm = tile / nbn;
    const int m0 = tm * bm + (int)blockIdx.y * (bm / 2), n0 = (tile - tm * nbn) * bn;
    const E* __restrict__ D = static_cast<const E*>(p.d);
    const int m1 = min(m0 + bm / 2, p.M);
    flt2* out = reinterpret_cast<flt2*>(p.stats) + (size_t)(tm * 2 + (int)blockIdx.y) * p.N;
    if constexpr (VEC4) {
        __shared__ double red[256][8];
        const int groups = bn / 4, lanes = 256 / groups;          // bn 64, 128, 256: 16, 8, 4 row lanes per column group
        const int cg = threadIdx.x % groups, rl = threadIdx.x / groups;
        const int col = n0 + cg * 4;
        double sum[4] = {0.0, 0.0, 0.0, 0.0}, sq[4] = {0.0, 0.0, 0.0, 0.0};
        if (col < p.N)
            for (int r = m0 + rl; r < m1; r += lanes) {
                float x[4];
                if constexpr (BF16) {
                    const uint2 u = *reinterpret_cast<const uint2*>(D + (long long)r * p.ldd + col);
                    x[0] = __uint_as_float(u.x << 16); x[1] = __uint_as_float(u.x & 0xffff0000u);
                    x[2] = __uint_as_float(u.y << 16); x[3] = __uint_as_float(u.y & 0xffff0000u);
                } else {
                    const float4 u = *reinterpret_cast<const float4*>(D + (long long)r * p.ldd + col);
                    x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sum[e] += (double)x[e];
                    sq[e] += (double)x[e] * (double)x[e];
                }
            }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            red[threadIdx.x][e] = sum[e];
            red[threadIdx.x][4 + e] = sq[e];
        }
        __syncthreads();
        if (rl == 0 && col < p.N) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double s1 = 0.0, s2 = 0.0;
                for (int k = 0; k < lanes; ++k) {
                    s1 += red[k * groups + cg][e];
                    s2 += red[k * groups + cg][4 + e];
                }
                out[col + e] = flt2{(float)s1, (float)s2};
            }
        }
    } else {
        const int col = n0 + (int)threadIdx.x;
        if ((int)threadIdx.x >= bn || col >= p.N) return;
        double sum = 0.0, sq = 0.0;
        for (int r = m0; r < m1; ++r) {
            float x;
            if constexpr (BF16) x = __uint_as_float((unsigned)D[(long long)r * p.ldd + col] << 16);
            else x = D[(long long)r * p.ldd + col];
            sum += (double)x;
            sq += (double)x * (double)x;
        }
        out[col] = flt2{(float)sum, (float)sq};
    }
}

// ------------------------------------------------------------------------------------------------
// bf16 3x3 window, stride 1, padding 1 (forward, and backward-data, which is the same convolution of dy with the
// re-ordered filter): the activation slab of a tile is staged ONCE per 32-channel chunk and all nine taps read it.
// The main kernel fetches a tile's activation rows again for every tap; its bf16 loop is bound by exactly that operand
// path (global -> LDS), and here the activation share of it falls to about a ninth (the slab with its halo is 1.6 to 3.2
// times the tile's pixels).
// Tile: 128 consecutive output pixels x BN filters, four waves (2 x 2).  Pixels are numbered over "virtual rows"
// image * (H + 1) + row: the one empty row between two images is the lower halo of one and the upper halo of the next.
// The slab holds the virtual rows of the tile's pixels plus one above and one below, each W + 2 pixels wide (the halo
// columns), 80 bytes per pixel: 64 of data (32 channels) and 16 of padding, so that the 16-byte fragment reads of 16
// consecutive pixels fall on distinct LDS banks without a per-tap swizzle.  Halo pixels are loaded as zeros (lane offset
// past the end of the buffer).  A tap (r, s) then is a wave-uniform displacement ((r - 1) * (W + 2) + (s - 1)) * 80 bytes
// of every lane's fragment address.  The filter tile of the next step is double-buffered as in the main kernel.
// ------------------------------------------------------------------------------------------------
constexpr int kSlabPitch = 80;         // bytes between slab pixels
constexpr int kSlabMaxVec = 8;         // 16-byte slab vectors per thread: slabs of up to 512 pixels

template <int BN>
__global__ void __launch_bounds__(256, 2) conv3x3_slab_kernel(const GemmConv p) {
    constexpr int BM = 128, WTM = 64, WTN = BN / 2, TM = 2, TN = WTN / 32, LB = BN * 4 / 256;
    extern __shared__ __attribute__((aligned(1024))) unsigned char slab_smem[];
    float* bl = reinterpret_cast<float*>(slab_smem);                 // filter tile, two stages of BN rows x 64 bytes
    unsigned char* slab = slab_smem + 2 * BN * 64;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int nbn = (p.N + BN - 1) / BN;
    const int tile = xcd_tile(blockIdx.x, gridDim.x);
    const int m0 = (tile / nbn) * BM, n0 = (tile % nbn) * BN;
    const int H = p.Hi, W = p.Wi, C = p.Ci, W2 = W + 2, HW = H * W, M_ = p.M, N_ = p.N, ldd_ = p.ldd;
    const int imgs = M_ / HW;
    const int ncc = C / 32, steps = ncc * 9;
    const int lrow = lane >> 2, kq = (lane & 3) ^ swz(lrow);
    const int frow = lane & 31, fhalf = lane >> 5, fsw = swz(frow);

    const int img0 = m0 / HW, p0 = (m0 - img0 * HW) / W;
    const int vr0 = img0 * (H + 1) + p0 - 1;                        // virtual row of slab row 0 (the upper halo)
    const int m_last = min(m0 + BM, M_) - 1;
    const int img1 = m_last / HW, p1 = (m_last - img1 * HW) / W;
    const int slab_px = (img1 * (H + 1) + p1 + 2 - vr0) * W2;       // at most what the launcher sized the LDS for

    // slab vector e = tid + i * 256 is chunk e % 4 of slab pixel e / 4
    const __amdgpu_buffer_rsrc_t a_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)p.a, 0, (int)((long long)M_ * C * 2), (int)kBufferWords3);
    unsigned a_voff[kSlabMaxVec];
#pragma unroll
    for (int i = 0; i < kSlabMaxVec; ++i) {
        const int e = tid + i * 256, sp = e >> 2, ch = e & 3;
        const int srow = sp / W2, col = sp - srow * W2;
        const int vr = vr0 + srow;
        const int img = vr >= 0 ? vr / (H + 1) : 0, h = vr - img * (H + 1);
        const bool ok = sp < slab_px && col >= 1 && col <= W && vr >= 0 && h < H && img < imgs;
        a_voff[i] = ok ? (unsigned)((((long long)img * H + h) * W + (col - 1)) * C * 2 + ch * 16) : kBufferBytes;
    }
    const __amdgpu_buffer_rsrc_t b_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)p.b, 0, (int)((long long)N_ * 9 * C * 2), (int)kBufferWords3);
    unsigned b_voff[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int n = n0 + (i * 4 + wave) * 16 + lrow;
        b_voff[i] = n < N_ ? (unsigned)((long long)n * 9 * C * 2 + kq * 16) : kBufferBytes;
    }
    unsigned a_frag[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int m = m0 + wm * WTM + i * 32 + frow;
        if (m >= M_) m = m0;                                         // rows past the end read some valid pixel; never stored
        const int img = m / HW, r = m - img * HW, pp = r / W, q = r - pp * W;
        a_frag[i] = (unsigned)(((img * (H + 1) + pp - vr0) * W2 + q + 1) * kSlabPitch + fhalf * 16);
    }
    const int b_frag = (wn * WTN + frow) * 16;

    u32x4 ga[kSlabMaxVec], gb[LB];
    auto gload_slab = [&](int cc) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kSlabMaxVec; ++i)
            if (i * 256 < slab_px * 4) ga[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, a_voff[i], cc * 64, 0);
    };
    auto sstore_slab = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kSlabMaxVec; ++i) {
            const int e = tid + i * 256;
            if (e < slab_px * 4) *reinterpret_cast<u32x4*>(slab + (e >> 2) * kSlabPitch + (e & 3) * 16) = ga[i];
        }
    };
    auto gload_b = [&](int t) __attribute__((always_inline)) {
        const int cc = t / 9, tap = t - cc * 9;
        const int soff = (tap * C + cc * 32) * 2;
#pragma unroll
        for (int i = 0; i < LB; ++i) gb[i] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, b_voff[i], soff, 0);
    };
    auto sstore_b = [&](int buf) __attribute__((always_inline)) {
        float* base = bl + buf * (BN * 16) + wave * 256 + lane * 4;
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<u32x4*>(base + i * 1024) = gb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    float4 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int buf, int tap, int k8, int slot) __attribute__((always_inline)) {
        const int r = tap / 3, s = tap - r * 3;
        const int delta = ((r - 1) * W2 + (s - 1)) * kSlabPitch + k8 * 32;        // wave-uniform
        const float* bb = bl + buf * (BN * 16);
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[slot][i] = *reinterpret_cast<const float4*>(slab + (int)a_frag[i] + delta);
        const int ch = ((2 * k8 + fhalf) ^ fsw) * 4;
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[slot][j] = *reinterpret_cast<const float4*>(bb + b_frag + j * 32 * 16 + ch);
    };
    auto mfma = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[slot][i]),
                                                                    __builtin_bit_cast(bf16x8, fb[slot][j]), acc[i][j], 0, 0, 0);
    };

    gload_slab(0);
    gload_b(0);
    sstore_slab();
    sstore_b(0);
    if (steps > 1) gload_b(1);
    lds_barrier();
    read_frags(0, 0, 0, 0);
    int cur = 0;
    for (int cc = 0; cc < ncc; ++cc) {
        const bool more_cc = cc + 1 < ncc;
        if (more_cc) gload_slab(cc + 1);                     // held in registers until this chunk's last tap is done
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            const int t = cc * 9 + tap;
            read_frags(cur, tap, 1, 1);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 1 < steps) sstore_b(cur ^ 1);            // the filter tile of step t + 1, loaded a step ago
            mfma(0);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 2 < steps) gload_b(t + 2);
            if (tap == 8 && more_cc) {
                lds_barrier();                               // every wave has read its last fragments of this chunk's slab
                sstore_slab();
            }
            lds_barrier();
            if (t + 1 < steps) read_frags(cur ^ 1, tap == 8 ? 0 : tap + 1, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            mfma(1);
            cur ^= 1;
        }
    }

    // tile store as in the main kernel: rows by scalar offset and cut off at M by the size of the buffer, columns by lane
    // offset with bit 31 past N; with an even row length neighbouring lanes trade halves and store column pairs
    {
        const long long rows_left = (long long)(M_ - m0) * ldd_ * 2;
        const __amdgpu_buffer_rsrc_t d_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(static_cast<uint16_t*>(p.d) + (long long)m0 * ldd_), 0, (int)(rows_left > 0x7fffffffLL ? 0x7fffffffLL : rows_left),
            (int)kBufferWords3);
        const bool pairs = ((N_ | ldd_) & 1) == 0;
        const int odd = lane & 1;
        unsigned d_voff[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * WTN + j * 32 + frow;
            d_voff[j] = col < N_ ? (unsigned)((4 * fhalf * ldd_ + col) * 2) : kBufferBytes;
            if (pairs && col < N_) d_voff[j] = (unsigned)(((4 * fhalf + odd) * ldd_ + (col & ~1)) * 2);
        }
        const unsigned perm_sel = odd ? 0x03020706u : 0x05040100u;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                const int r0 = wm * WTM + i * 32 + 8 * (v >> 2) + (v & 3);       // registers v and v + 1: rows r0 and r0 + 1
                const int soff = r0 * ldd_ * 2;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const unsigned u = lc_bf16x2_rne(acc[i][j][v], acc[i][j][v + 1]);
                    if (pairs) {
                        const unsigned got = (unsigned)__builtin_amdgcn_mov_dpp((int)u, 0xB1 /* quad_perm 1,0,3,2 */, 0xF, 0xF, true);
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_amdgcn_perm(got, u, perm_sel), d_rsrc, (int)d_voff[j], soff, 0);
                    } else {
                        __builtin_amdgcn_raw_buffer_store_b16((short)(u & 0xffffu), d_rsrc, (int)d_voff[j], soff, 0);
                        __builtin_amdgcn_raw_buffer_store_b16((short)(u >> 16), d_rsrc, (int)d_voff[j], soff + ldd_ * 2, 0);
                    }
                }
            }
    }
    if (p.stats) {
        // per column, the sum and the sum of squares of the stored (rounded) values over this wave's 64 rows, as in the main kernel
        typedef float flt2 __attribute__((ext_vector_type(2)));
        flt2* st = reinterpret_cast<flt2*>(p.stats) + (size_t)((m0 / BM) * 2 + wm) * N_;
        const bool ragged = m0 + BM > M_;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            float sum = 0.f, sq = 0.f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    const unsigned u = lc_bf16x2_rne(acc[i][j][v], acc[i][j][v + 1]);
                    float x0 = __uint_as_float(u << 16), x1 = __uint_as_float(u & 0xffff0000u);
                    if (ragged) {
                        const int row = m0 + wm * WTM + i * 32 + 8 * (v >> 2) + 4 * fhalf + (v & 3);
                        if (row >= M_) x0 = 0.f;
                        if (row + 1 >= M_) x1 = 0.f;
                    }
                    sum += x0;
                    sq = fmaf(x0, x0, sq);
                    sum += x1;
                    sq = fmaf(x1, x1, sq);
                }
            sum += __shfl_xor(sum, 32);
            sq += __shfl_xor(sq, 32);
            const int col = n0 + wn * WTN + j * 32 + frow;
            if (fhalf == 0 && col < N_) st[col] = flt2{sum, sq};
        }
    }
}

// ------------------------------------------------------------------------------------------------
// backward-weight kernel: both operands contiguous along their *output* index (k resp. c), the
// reduction index m strides over rows.  LDS holds [reduction][row] so that the row-contiguous
// global vectors are stored as they arrive and MFMA fragments are read with unit lane stride.
// ------------------------------------------------------------------------------------------------
// VEC operand elements from global memory as fp32 (bf16 is widened exactly); loads through the global path
#define LC_GLOBAL __attribute__((address_space(1)))
template <int VEC, bool BF16>
__device__ __forceinline__ typename VecT<VEC>::type load_widen(const void* ptr) {
    const uintptr_t addr = reinterpret_cast<uintptr_t>(ptr);
    if constexpr (!BF16 && VEC == 4) {
        return load_global16(ptr);
    } else if constexpr (!BF16) {
        return *(const LC_GLOBAL float*)addr;
    } else if constexpr (VEC == 4) {
        typedef unsigned int gu2 __attribute__((ext_vector_type(2)));
        const gu2 u = *(const LC_GLOBAL gu2*)addr;
        return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                           __uint_as_float(u.y & 0xffff0000u));
    } else {
        return __uint_as_float((uint32_t)(*(const LC_GLOBAL unsigned short*)addr) << 16);
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, int VEC, bool BF16>
__global__ void __launch_bounds__(WGM* WGN * 64) wgrad_f32_kernel(const GemmWgrad p) {
    using E = typename OutT<BF16>::type;              // operand element type
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
    // Work items are numbered split-major (all tiles of a split next to each other) and dealt to the XCDs in
    // contiguous runs: the tiles of a split, which read the same rows of dY and X, then share one L2.
    const int tiles_ = ((p.K + BM - 1) / BM) * nbn;
    const int work = xcd_tile(blockIdx.x, tiles_ * p.splits);
    const int z = work / tiles_;
    const int tile = work - z * tiles_;
    const int k0 = (tile / nbn) * BM, j0 = (tile % nbn) * BN;
    const int m_begin = z * p.m_per_split;
    const int m_end = min(p.M, m_begin + p.m_per_split);

    const E* __restrict__ DY = static_cast<const E*>(p.dy);
    const E* __restrict__ X = static_cast<const E*>(p.x);

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
            ra[i] = load_widen<VEC, BF16>(pick(a_ok & (m < m_end), DY + (long long)m * p.K + a_col, g_zero_chunk));
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int m = mt + b_kr + i * BRPP;
            const int h = b_p[i] * p.sh - p.ph + fr, w = b_q[i] * p.sw - p.pw + fs;
            const bool ok = b_ok & (m < m_end) & ((unsigned)h < (unsigned)p.H) & ((unsigned)w < (unsigned)p.W);
            rb[i] = load_widen<VEC, BF16>(pick(ok, X + (((long long)b_img[i] * p.H + h) * p.W + w) * p.C + fc, g_zero_chunk));
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

    // fragments of the next pair of reduction rows are read while the current pair is multiplied
    auto compute = [&](int buf) {
        const float* as = &As[buf][(lane >> 5) * PA + wm * WTM + (lane & 31)];
        const float* bs = &Bs[buf][(lane >> 5) * PB + wn * WTN + (lane & 31)];
        float a[2][TM], b[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[0][i] = as[i * 32];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[0][j] = bs[j * 32];
#pragma unroll
        for (int k2 = 0; k2 < BK / 2; ++k2) {
            const int cs = k2 & 1, ns = cs ^ 1;
            if (k2 + 1 < BK / 2) {
#pragma unroll
                for (int i = 0; i < TM; ++i) a[ns][i] = as[2 * (k2 + 1) * PA + i * 32];
#pragma unroll
                for (int j = 0; j < TN; ++j) b[ns][j] = bs[2 * (k2 + 1) * PB + j * 32];
                __builtin_amdgcn_sched_barrier(0);      // keep these reads in front of the MFMAs below
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cs][i], b[cs][j], acc[i][j], 0, 0, 0);
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

// ------------------------------------------------------------------------------------------------
// backward-weight kernel with scalar addressing (fp32 operands, channel counts multiples of 4, filter
// windows of at most 32 taps).  Same GEMM, LDS layout, split and fragment reads as wgrad_f32_kernel; the
// difference is where the address arithmetic runs.  A wave fetches whole reduction rows: one load
// instruction covers the BN columns of ONE output pixel m, so the pixel's (image, p, q), its byte offset and
// the set of filter taps that fall inside the image are wave-uniform and are kept in scalar registers
// (advanced by 16 rows per step with precomputed digits of 16 in the (Q, P) number system).  A lane only
// holds what depends on its column: the tap's byte offset and the tap's bit position.  A lane whose tap is
// outside the image for this pixel gets bit 31 of its buffer offset set and the hardware returns zeros.
// dY rows past the end of the split are cut off by the size of the dY buffer descriptor.
// ------------------------------------------------------------------------------------------------
// BF16: operands are bf16 (reduction step 32, LDS holds bf16, MFMA operands come from the transposing LDS read as
// in wgrad_bf16_kernel); everything about the addressing is the same with 2-byte elements.
// PLAIN: a 1x1 window with stride 1 and no padding.  Output pixel m then reads input pixel m, X is a plain
// [M][C] matrix like dY, and both operands are fetched with 16-byte loads at a lane-constant offset plus the
// step's scalar offset: no per-pixel work at all.
template <int BM, int BN, bool BF16, bool PLAIN>
__global__ void __launch_bounds__(256, 4) wgrad_ut_kernel(const GemmWgrad p) {   // 4 blocks per compute unit: lc_wgrad_splits()
    using E = typename OutT<BF16>::type;                          // operand element type (float, or the bits of a bf16)
    constexpr int ES = (int)sizeof(E);
    constexpr int EPC = 16 / ES;                                  // elements per 16-byte vector
    constexpr int BK = BF16 ? 32 : 16;
    constexpr int AQ = BM / EPC, ARPP = 256 / AQ, LA = BK / ARPP; // dY: 16-byte vectors, ARPP rows per pass
    constexpr int BV = BN / 64;                                   // X: elements per lane and row (one row per wave and load)
    constexpr int RW = BK / 4;                                    // X rows per wave and step
    constexpr int BQ = BN / EPC, BRPP = 256 / BQ, LB = BK / BRPP; // PLAIN: X in 16-byte vectors like dY
    constexpr int PA = BM + (BF16 ? 32 : 4), PB = BN + (BF16 ? 32 : 4);
    constexpr int WTM = BM / 2, WTN = BN / 2, TM = WTM / 32, TN = WTN / 32;
    static_assert(PLAIN || BV == 2 || (BV == 1 && !BF16), "tile shape");
    static_assert(256 % AQ == 0 && BK % ARPP == 0 && LA >= 1, "tile shape");
    using BVt = typename std::conditional<BF16, unsigned, typename std::conditional<BV == 2, float2, float>::type>::type;

    __shared__ __attribute__((aligned(16))) E As[2][BK * PA];
    __shared__ __attribute__((aligned(16))) E Bs[2][BK * PB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int nbn = (p.J + BN - 1) / BN;
    // Work items are numbered split-major (all tiles of a split next to each other) and dealt to the XCDs in
    // contiguous runs: the tiles of a split, which read the same rows of dY and X, then share one L2.
    const int tiles_ = ((p.K + BM - 1) / BM) * nbn;
    const int work = xcd_tile(blockIdx.x, tiles_ * p.splits);
    const int z = work / tiles_;
    const int tile = work - z * tiles_;
    const int k0 = (tile / nbn) * BM, j0 = (tile % nbn) * BN;
    const int m_begin = z * p.m_per_split;
    const int m_end = min(p.M, m_begin + p.m_per_split);
    const int H_ = p.H, W_ = p.W, C_ = p.C, P_ = p.P, Q_ = p.Q, R_ = p.R, S_ = p.S, K_ = p.K;
    const int sh_ = p.sh, sw_ = p.sw, ph_ = p.ph, pw_ = p.pw;

    // dY: lane-constant offset inside a 16-row step; the step's first row is the scalar offset
    const int a_cq = tid % AQ, a_kr = tid / AQ;
    const int a_col = k0 + a_cq * EPC;
    unsigned a_voff[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) a_voff[i] = a_col < K_ ? (unsigned)(((a_kr + i * ARPP) * K_ + a_col) * ES) : kBufferBytes;
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(static_cast<const E*>(p.dy) + (long long)m_begin * K_), 0, (int)((unsigned)(m_end - m_begin) * K_ * (unsigned)ES),
        (int)kBufferWords3);

    // PLAIN: X addressed like dY
    const int pb_cq = tid % BQ, pb_kr = tid / BQ;
    unsigned pb_voff[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i)
        pb_voff[i] = j0 + pb_cq * EPC < p.J ? (unsigned)(((pb_kr + i * BRPP) * C_ + j0 + pb_cq * EPC) * ES) : kBufferBytes;
    const __amdgpu_buffer_rsrc_t pb_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(static_cast<const E*>(p.x) + (long long)m_begin * C_), 0, (int)((unsigned)(m_end - m_begin) * C_ * (unsigned)ES),
        (int)kBufferWords3);
    // X: the lane's column j = (r, s, c): byte offset of the tap relative to the pixel's window origin, bit position
    const int b_col = j0 + lane * BV;
    unsigned b_voff = kBufferBytes, b_up = 0;
    if (b_col < p.J) {
        const int rs = b_col / C_, fc = b_col - rs * C_;
        const int fr = rs / S_, fs = rs - fr * S_;
        b_voff = (unsigned)(((fr * W_ + fs) * C_ + fc) * ES);
        b_up = 31u - (unsigned)rs;
    }
    const int pq = P_ * Q_;
    const int img_first = m_begin / pq;
    const int phb = max(ph_, 0), pwb = max(pw_, 0);
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(static_cast<const E*>(p.x) + ((long long)img_first * H_ * W_ - ((long long)phb * W_ + pwb)) * C_), 0,
        (int)kBufferBytes, (int)kBufferWords3);
    // scalar state of this wave's RW rows: (image - img_first, p, q) of row m_begin + step * 16 + wave * RW + i
    int s_img[RW], s_p[RW], s_q[RW];
#pragma unroll
    for (int i = 0; i < RW; ++i) {
        const int m = m_begin + wave * RW + i;
        const int t = m / Q_;
        s_q[i] = m - t * Q_;
        const int im = t / P_;
        s_p[i] = t - im * P_;
        s_img[i] = im - img_first;
    }
    // 16 rows further: 16 = (d_img * P + d_p) * Q + d_q
    const int d_q = BK % Q_, d_t = BK / Q_, d_p = d_t % P_, d_img = d_t / P_;
    const int taps = R_ * S_;
    const unsigned full = taps >= 32 ? ~0u : (1u << taps) - 1u;
    unsigned rep = 0;                                             // bit r*S for every r: spreads a mask over s to all rows of the window
    for (int r = 0; r < R_; ++r) rep |= 1u << (r * S_);
    int mt = m_begin;                                             // first reduction row of the step being loaded

    float4 ra[LA];
    BVt rb[RW];
    float4 prb[LB];
    auto gload = [&]() __attribute__((always_inline)) {
        const int a_soff = (mt - m_begin) * K_ * ES;
#pragma unroll
        for (int i = 0; i < LA; ++i)
            ra[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)a_voff[i], a_soff, 0));
        if constexpr (PLAIN) {
            const int b_soff = (mt - m_begin) * C_ * ES;
#pragma unroll
            for (int i = 0; i < LB; ++i)
                prb[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(pb_rsrc, (int)pb_voff[i], b_soff, 0));
            return;
        }
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            const int h0 = s_p[i] * sh_ - ph_, w0 = s_q[i] * sw_ - pw_;
            int rlo = max(0, -h0), rhi = min(R_ - 1, H_ - 1 - h0);
            int slo = max(0, -w0), shi = min(S_ - 1, W_ - 1 - w0);
            const bool ok = (rlo <= rhi) & (slo <= shi) & (mt + wave * RW + i < m_end);
            rlo = min(rlo, R_ - 1);                              // keep the shifts below in range when the row is dead
            rhi = max(rhi, 0);
            slo = min(slo, S_ - 1);
            const int sspan = max(shi - slo, 0);
            const unsigned hm = (full << (rlo * S_)) & (full >> ((R_ - 1 - rhi) * S_));
            const unsigned wmask = rep * (((2u << sspan) - 1u) << slo);
            const unsigned inv = ok ? ~(hm & wmask) : ~0u;        // taps outside the image for this pixel
            const int soff = ok ? (((s_img[i] * H_ + s_p[i] * sh_ + phb - ph_) * W_ + s_q[i] * sw_ + pwb - pw_) * C_) * ES : 0;
            const unsigned vo = ((inv << b_up) & kBufferBytes) | b_voff;
            if constexpr (BF16)
                rb[i] = __builtin_amdgcn_raw_buffer_load_b32(b_rsrc, (int)vo, soff, 0);
            else if constexpr (BV == 2)
                rb[i] = __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(b_rsrc, (int)vo, soff, 0));
            else
                rb[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(b_rsrc, (int)vo, soff, 0));
        }
    };
    auto advance = [&]() __attribute__((always_inline)) {
        mt += BK;
        if constexpr (PLAIN) return;
#pragma unroll
        for (int i = 0; i < RW; ++i) {
            int q = s_q[i] + d_q;
            const bool cq = q >= Q_;
            q -= cq ? Q_ : 0;
            int pp = s_p[i] + d_p + (cq ? 1 : 0);
            const bool cp = pp >= P_;
            pp -= cp ? P_ : 0;
            s_q[i] = q;
            s_p[i] = pp;
            s_img[i] += d_img + (cp ? 1 : 0);
        }
    };
    auto sstore = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<float4*>(&As[buf][(a_kr + i * ARPP) * PA + a_cq * EPC]) = ra[i];
        if constexpr (PLAIN) {
#pragma unroll
            for (int i = 0; i < LB; ++i) *reinterpret_cast<float4*>(&Bs[buf][(pb_kr + i * BRPP) * PB + pb_cq * EPC]) = prb[i];
            return;
        }
#pragma unroll
        for (int i = 0; i < RW; ++i) *reinterpret_cast<BVt*>(&Bs[buf][(wave * RW + i) * PB + lane * BV]) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Fragments of one group of reduction rows (fp32: 2 rows, one MFMA of k = 2 per tile; bf16: 16 rows, one MFMA of
    // k = 16 per tile), double-buffered: slot g & 1 holds group g of the step.
    constexpr int NG = BF16 ? BK / 16 : BK / 2;
    using Frag = typename std::conditional<BF16, bf16x8, float>::type;
    Frag fa[2][TM], fb[2][TN];
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    // bf16: the transposing LDS read (see wgrad_bf16_kernel): this lane's row and column inside a 16-row group
    const int tr_row = 8 * (lane >> 5) + ((lane & 15) >> 2), tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    auto read_frags = [&](int buf, int g, int slot) __attribute__((always_inline)) {
        if constexpr (BF16) {
            auto one = [&](const E* base, int pitch) __attribute__((always_inline)) {
                const E* q = base + (16 * g + tr_row) * pitch + tr_col;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)q);
                const s16x4 hi =
                    __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)(q + 4 * pitch));
                const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                return __builtin_bit_cast(bf16x8, v);
            };
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[slot][i] = one(&As[buf][wm * WTM + i * 32], PA);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[slot][j] = one(&Bs[buf][wn * WTN + j * 32], PB);
        } else {
            const E* as = &As[buf][(2 * g + (lane >> 5)) * PA + wm * WTM + (lane & 31)];
            const E* bs = &Bs[buf][(2 * g + (lane >> 5)) * PB + wn * WTN + (lane & 31)];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[slot][i] = as[i * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[slot][j] = bs[j * 32];
        }
    };
    auto mfma_group = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (BF16)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
            }
    };

    // One step out of LDS buffer `cur` (a literal at each call).  On entry slot 0 holds the step's first group of
    // rows and the registers hold the next step's rows.  Those go to the other LDS buffer early in the step, the
    // loads of the step after next follow into the same registers, and behind the barrier before the last group
    // the first fragments of the next step are read while the last MFMAs run.  Steps past the end of the split
    // are fetched and stored like the others: all of their rows are past m_end, so nothing is read from memory
    // and zeros are stored.
    constexpr int G_STORE = NG > 2 ? 1 : 0, G_LOAD = NG > 2 ? 3 : 0;
    auto step = [&](int cur) __attribute__((always_inline)) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            if (g + 1 < NG) {
                read_frags(cur, g + 1, (g + 1) & 1);
            } else {
                lds_barrier();
                read_frags(cur ^ 1, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_group(g & 1);
            __builtin_amdgcn_sched_barrier(0);
            if (g == G_STORE) sstore(cur ^ 1);
            if (g == G_LOAD) {
                advance();
                gload();
            }
        }
    };
    const int nkt = (m_end - m_begin + BK - 1) / BK;
    if (nkt > 0) {
        gload();
        sstore(0);
        advance();
        gload();
        lds_barrier();
        read_frags(0, 0, 0);
        int kt = 0;
        for (; kt + 2 <= nkt; kt += 2) {
            step(0);
            step(1);
        }
        if (kt < nkt) step(0);
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

// ------------------------------------------------------------------------------------------------
// backward-weight kernel for bf16 operands on the bf16 matrix pipe (channel counts multiples of 8).
// Same GEMM and split as wgrad_f32_kernel, reduction step 32.  LDS holds [reduction row][output index]
// in bf16 as the 16-byte global vectors arrive; an MFMA operand (8 consecutive reduction rows of one
// output index) is gathered with eight 16-bit LDS reads, consecutive lanes reading consecutive elements.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN>
__global__ void __launch_bounds__(256) wgrad_bf16_kernel(const GemmWgrad p) {
    constexpr int BK = 32;                            // reduction rows per step: two k-16 MFMA steps
    constexpr int AQ = BM / 8, BQ = BN / 8;           // 16-byte vectors per reduction row
    constexpr int ARPP = 256 / AQ, BRPP = 256 / BQ;   // reduction rows per pass of the block
    constexpr int LA = BK / ARPP, LB = BK / BRPP;
    constexpr int PA = BM + 32, PB = BN + 32;         // elements: four consecutive rows start 64 bytes apart modulo 256
    constexpr int WTM = BM / 2, WTN = BN / 2, TM = WTM / 32, TN = WTN / 32;
    static_assert(256 % AQ == 0 && 256 % BQ == 0 && BK % ARPP == 0 && BK % BRPP == 0 && LA >= 1 && LB >= 1, "tile shape");

    __shared__ __attribute__((aligned(16))) uint16_t As[2][BK * PA];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BK * PB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int nbn = (p.J + BN - 1) / BN;
    // Work items are numbered split-major (all tiles of a split next to each other) and dealt to the XCDs in
    // contiguous runs: the tiles of a split, which read the same rows of dY and X, then share one L2.
    const int tiles_ = ((p.K + BM - 1) / BM) * nbn;
    const int work = xcd_tile(blockIdx.x, tiles_ * p.splits);
    const int z = work / tiles_;
    const int tile = work - z * tiles_;
    const int k0 = (tile / nbn) * BM, j0 = (tile % nbn) * BN;
    const int m_begin = z * p.m_per_split;
    const int m_end = min(p.M, m_begin + p.m_per_split);

    const uint16_t* __restrict__ DY = static_cast<const uint16_t*>(p.dy);
    const uint16_t* __restrict__ X = static_cast<const uint16_t*>(p.x);

    const int a_cq = tid % AQ, a_kr = tid / AQ;
    const int a_col = k0 + a_cq * 8;
    const bool a_ok = a_col < p.K;
    const int b_cq = tid % BQ, b_kr = tid / BQ;
    const int b_col = j0 + b_cq * 8;
    const bool b_ok = b_col < p.J;
    int fr, fs, fc;
    {
        const int rs = b_col / p.C;
        fc = b_col % p.C;
        fs = rs % p.S;
        fr = rs / p.S;
    }
    int b_img[LB], b_p[LB], b_q[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int m = m_begin + b_kr + i * BRPP;
        b_q[i] = m % p.Q;
        const int t = m / p.Q;
        b_p[i] = t % p.P;
        b_img[i] = t / p.P;
    }
    int mt = m_begin;

    float4 ra[LA], rb[LB];                            // raw 16-byte vectors (8 bf16 each)
    auto gload = [&]() {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int m = mt + a_kr + i * ARPP;
            ra[i] = load_global16(pick(a_ok & (m < m_end), DY + (long long)m * p.K + a_col, g_zero_chunk));
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int m = mt + b_kr + i * BRPP;
            const int h = b_p[i] * p.sh - p.ph + fr, w = b_q[i] * p.sw - p.pw + fs;
            const bool ok = b_ok & (m < m_end) & ((unsigned)h < (unsigned)p.H) & ((unsigned)w < (unsigned)p.W);
            rb[i] = load_global16(pick(ok, X + (((long long)b_img[i] * p.H + h) * p.W + w) * p.C + fc, g_zero_chunk));
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
        for (int i = 0; i < LA; ++i) *reinterpret_cast<float4*>(&As[buf][(a_kr + i * ARPP) * PA + a_cq * 8]) = ra[i];
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<float4*>(&Bs[buf][(b_kr + i * BRPP) * PB + b_cq * 8]) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Operand of one MFMA: reduction rows 16*t + 8*(lane>>5) + 0..7 of output index (lane & 31), fetched with
    // the transposing LDS read.  Within 16 lanes, lane i points at 4 consecutive elements of row i/4 (columns
    // 4*(i%4)..) and receives column i of those 4 rows: 4 consecutive reduction rows of one output index.  Lanes
    // 16..31 take the next 16 columns, lanes 32..63 the rows 8 further down; a second read 4 rows down
    // completes the 8 values.
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    const int tr_row = 8 * (lane >> 5) + ((lane & 15) >> 2), tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    auto frag = [&](const uint16_t* base, int pitch, int t) __attribute__((always_inline)) {
        const uint16_t* q = base + (16 * t + tr_row) * pitch + tr_col;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)q);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)(q + 4 * pitch));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, v);
    };
    auto compute = [&](int buf) {
#pragma unroll
        for (int t = 0; t < BK / 16; ++t) {
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = frag(&As[buf][wm * WTM + i * 32], PA, t);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = frag(&Bs[buf][wn * WTN + j * 32], PB, t);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
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

// ------------------------------------------------------------------------------------------------
// backward-weight of a 3x3 / stride 1 / padding 1 layer in bf16 with the activations staged once for all nine taps.
// wgrad_bf16_kernel gathers the im2col matrix: every activation pixel is fetched nine times, once per tap, and the 64-wide
// tiles of the layers with 64 filters feed few MFMAs per byte.  Here a block owns 64 filters x 64 channels x all nine taps.
//
// Pixels are numbered as positions of a padded image: virtual row v = image * (H + 1) + h (row H of every image is an empty
// row: the lower halo of one image and the upper halo of the next), W + 2 columns (column 0 and W + 1 are halo), position
// = v * (W + 2) + column.  With dY and X both zero on the halo,
//     dW[k][r][s][c] = sum over positions of dY[position][k] * X[position + (r - 1) * (W + 2) + (s - 1)][c],
// so a tap is a displacement of the X operand by a fixed number of positions.  The reduction runs over all positions (the
// 2 / (W + 2) of them that are halo cost MFMAs on zeros), cut into `splits` ranges of m_per_split positions.
//
// LDS: dY of the current 32 positions (two buffers) and a ring of X positions reaching 32 * L >= W + 3 positions behind
// and ahead of them, (2 L + 2) chunks of 32; both as [position][64 channels] with the pitch of wgrad_bf16_kernel, read with
// the transposing LDS read.  A fragment's 16 positions start at any ring row, so rows 0..15 are mirrored behind the last
// row and a read never wraps inside a fragment: its start row is scalar arithmetic.  Halo positions are loaded as zeros
// (buffer loads, the offset of an invalid lane points past the buffer).  Positions are tracked on the scalar unit: a wave
// loads eight consecutive positions, so column, image row and image of the first are wave-uniform and a lane that runs past
// the end of the row (at most once: W + 2 >= 8) takes the next row's values.
//
// Pipeline: a step is 18 items (two halves of 16 positions x nine taps), one MFMA each; the X fragment of item g + 5 is
// read before the MFMA of item g (six register sets; 18 % 6 == 0); the LDS stores of the next step and the barrier sit five
// items before the end of the step, so the first reads of the next step run under the last MFMAs of this one; global loads
// are two steps ahead and the barrier waits for LDS only.
// ------------------------------------------------------------------------------------------------
constexpr int kWsPitch = 96;          // elements between positions in LDS: 128 bytes of data, 64 of padding
constexpr int kWsMaxL = 3;            // W + 3 <= 96

__global__ void __launch_bounds__(256, 2) wgrad3x3_slab_kernel(const GemmWgrad p) {
    extern __shared__ __attribute__((aligned(16))) uint16_t ws_smem[];
    const int H = p.H, W = p.W, Wp = W + 2, H1 = H + 1;
    const int L = (W + 3 + 31) / 32, RING = (2 * L + 2) * 32;
    uint16_t* dys = ws_smem;                           // [2][32][kWsPitch]
    uint16_t* xs = ws_smem + 2 * 32 * kWsPitch;        // [RING + 16][kWsPitch]: rows RING.. mirror rows 0..15

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = wave >> 1, ch = wave & 1;
    const int tiles_c = p.C / 64, tiles_ = (p.K / 64) * tiles_c;
    const int work = xcd_tile(blockIdx.x, gridDim.x);  // split-major: the tiles of a split share its rows of dY and X in one L2
    const int z = work / tiles_, tile = work - z * tiles_;
    const int k0 = (tile / tiles_c) * 64, c0 = (tile % tiles_c) * 64;
    const int imgs = p.M / (H * W);
    const long long total = (long long)imgs * H1 * Wp;
    const long long pos_begin = (long long)z * p.m_per_split;
    int nsteps = 0;
    if (pos_begin < total) {
        const long long left = total - pos_begin;
        nsteps = (int)((left < p.m_per_split ? left : (long long)p.m_per_split) + 31) / 32;
    }

    const int po = tid >> 3, cq = tid & 7, j8 = lane >> 3;
    struct Track { int col, h, img, rowbase; };       // of a wave's first position; rowbase: first pixel of the (most recent) image row
    const int per_img = H1 * Wp;
    const int eimg = (32 * L + per_img - 1) / per_img;            // whole virtual images that make every position non-negative
    auto init = [&](long long pos) {
        const long long q = pos + (long long)eimg * per_img;
        const long long v = q / Wp;
        Track t;
        t.col = (int)(q - v * Wp);
        const long long im = v / H1;
        t.h = (int)(v - im * H1);
        t.img = (int)im - eimg;
        t.rowbase = (t.img * H + (t.h < H ? t.h : H - 1)) * W;
        return t;
    };
    auto advance = [&](Track& t) {
        t.col += 32;
        while (t.col >= Wp) {
            t.col -= Wp;
            if (++t.h == H1) {
                t.h = 0;
                ++t.img;
            }
            if (t.h != H) t.rowbase += W;
        }
    };
    auto offset_of = [&](const Track& t, int pixel_bytes) {
        int h2 = t.h + 1, img2 = t.img, rb2 = t.rowbase;          // the row after
        if (h2 == H1) {
            h2 = 0;
            ++img2;
        }
        if (h2 != H) rb2 += W;
        const bool v1 = ((unsigned)t.img < (unsigned)imgs) & (t.h < H), v2 = ((unsigned)img2 < (unsigned)imgs) & (h2 < H);
        int c = t.col + j8;
        const bool wr = c >= Wp;
        c = wr ? c - Wp : c;
        const bool ok = (wr ? v2 : v1) & (c >= 1) & (c <= W);
        const int pix = (wr ? rb2 : t.rowbase) + c - 1;
        return ok ? (unsigned)pix * (unsigned)pixel_bytes + (unsigned)cq * 16u : 0x80000000u;
    };
    Track ta = init(pos_begin + 8 * wave), tb = init(pos_begin - 32 * L + 8 * wave);
    const uint16_t* DY = static_cast<const uint16_t*>(p.dy) + k0;
    const uint16_t* X = static_cast<const uint16_t*>(p.x) + c0;
    const __amdgpu_buffer_rsrc_t y_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)DY, 0, (int)((long long)p.M * p.K * 2 - k0 * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t x_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, (int)((long long)p.M * p.C * 2 - c0 * 2), 0x00020000);
    auto load_y = [&]() {
        const unsigned off = offset_of(ta, p.K * 2);
        advance(ta);
        return __builtin_amdgcn_raw_buffer_load_b128(y_rsrc, off, 0, 0);
    };
    auto load_x = [&]() {
        const unsigned off = offset_of(tb, p.C * 2);
        advance(tb);
        return __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, off, 0, 0);
    };
    int xslot = 0;                                                  // ring row of the next chunk of X (uniform)
    auto store_x = [&](const u32x4& v) {
        *reinterpret_cast<u32x4*>(&xs[(xslot + po) * kWsPitch + cq * 8]) = v;
        if (xslot == 0 && po < 16) *reinterpret_cast<u32x4*>(&xs[(RING + po) * kWsPitch + cq * 8]) = v;
        xslot += 32;
        if (xslot == RING) xslot = 0;
    };
    auto store_y = [&](int buf, const u32x4& v) { *reinterpret_cast<u32x4*>(&dys[(buf * 32 + po) * kWsPitch + cq * 8]) = v; };

    f32x16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const int tr_row = 8 * (lane >> 5) + ((lane & 15) >> 2), tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const int lane_a = tr_row * kWsPitch + kh * 32 + tr_col, lane_b = tr_row * kWsPitch + ch * 32 + tr_col;
    auto frag = [&](const uint16_t* q) __attribute__((always_inline)) {     // see wgrad_bf16_kernel
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)q);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)(q + 4 * kWsPitch));
        const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, v);
    };

    constexpr int PD = 5, NB = 6;
    if (nsteps > 0) {
        for (int j = 0; j < 2 * L + 1; ++j) store_x(load_x());
        store_y(0, load_y());
        u32x4 ra[2], rb[2];                                         // slot s % 2: operands of step s, loaded two steps before
#pragma unroll
        for (int d = 1; d <= 2; ++d)
            if (d < nsteps) {
                ra[d % 2] = load_y();
                rb[d % 2] = load_x();
            }
        lds_barrier();
        int base = 32 * L;                                          // ring row of the current step's first position
        bf16x8 a0, a1, bq[NB];
        auto read_item = [&](int i, int rbase, int buf) __attribute__((always_inline)) {   // item i: half i / 9, tap i % 9
            const int t16 = i / 9, tap = i % 9;
            if (tap == 0) {
                const bf16x8 a = frag(dys + buf * 32 * kWsPitch + 16 * t16 * kWsPitch + lane_a);
                if (t16 == 0) a0 = a; else a1 = a;
            }
            int u = rbase + 16 * t16 + (tap / 3 - 1) * Wp + (tap % 3 - 1);
            u = u < 0 ? u + RING : (u >= RING ? u - RING : u);
            bq[i % NB] = frag(xs + u * kWsPitch + lane_b);
        };
#pragma unroll
        for (int i = 0; i < PD; ++i) read_item(i, base, 0);
        auto step_fn = [&](int step, int par) __attribute__((always_inline)) {   // par = step & 1 (compile time)
            int nbase = base + 32;
            if (nbase == RING) nbase = 0;
#pragma unroll
            for (int i = 0; i < 18; ++i) {
                if (i == 18 - PD) {
                    if (step + 1 < nsteps) {
                        store_y(par ^ 1, ra[par ^ 1]);
                        store_x(rb[par ^ 1]);
                        if (step + 3 < nsteps) {
                            ra[par ^ 1] = load_y();
                            rb[par ^ 1] = load_x();
                        }
                    }
                    lds_barrier();
                }
                if (i + PD < 18) read_item(i + PD, base, par);
                else read_item(i + PD - 18, nbase, par ^ 1);       // the next step's first items (in bounds; unused after the last step)
                acc[i % 9] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(i < 9 ? a0 : a1, bq[i % NB], acc[i % 9], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            base = nbase;
        };
        int step = 0;
        for (; step + 2 <= nsteps; step += 2) {
            step_fn(step, 0);
            step_fn(step + 1, 1);
        }
        if (step < nsteps) step_fn(step, 0);
    }

    float* __restrict__ D = p.d + (long long)z * p.K * p.J;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = k0 + kh * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            const int col = tap * p.C + c0 + ch * 32 + (lane & 31);
            D[(long long)row * p.J + col] = acc[tap][v];
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

template <int BM, int BN, int BK, int VEC, bool BF16>
lc_status launch_wgrad(const GemmWgrad& p, hipStream_t stream) {
    const long long tiles = (long long)((p.K + BM - 1) / BM) * ((p.J + BN - 1) / BN);
    if (tiles <= 0 || tiles * p.splits > 0x7fffffffLL) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((wgrad_f32_kernel<BM, BN, BK, 2, 2, VEC, BF16>), dim3((unsigned)(tiles * p.splits)), dim3(256), 0,
                       stream, p);
    return lc_end_call();
}

// Split of the output tiles into whole-tile blocks and stream-K blocks for a BM x BN tiling.
struct SkPlan {
    int dp_tiles, sk_blocks;
    long long sk_iters;
};

int device_cu_count() {
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0)
            cus = 256;
        (void)hipGetLastError();
        return cus;
    }();
    return n;
}

SkPlan sk_plan(long long tiles, int nkt, int resident_blocks, bool allow_split = true) {
    SkPlan pl;
    const long long rounds = tiles / resident_blocks;
    long long dp = rounds * resident_blocks;
    long long rest = tiles - dp;
    pl.dp_tiles = (int)dp;
    pl.sk_blocks = 0;
    pl.sk_iters = 0;
    if (rest == 0 || !allow_split || getenv("LARSCONV_NO_STREAMK")) {   // every round is full, or splitting tiles is not wanted
        pl.dp_tiles = (int)tiles;
        return pl;
    }
    pl.sk_iters = rest * nkt;
    long long blocks = pl.sk_iters / 8;                      // at least 8 k-steps per stream-K block
    if (blocks > resident_blocks) blocks = resident_blocks;
    if (blocks < 1) blocks = 1;
    pl.sk_blocks = (int)blocks;
    return pl;
}

// Blocks of the main kernel that fit on the chip at once (the kernel's launch bounds hold it to this).
inline int resident_blocks(int bm, int bn) { return pk_blocks_per_cu(bm, bn) * device_cu_count(); }

// Tile of the main kernel for a problem.  fp32: 128 rows, 64 columns for narrow results, otherwise 128.  bf16
// adds larger tiles, because its loop is bound by what moves through LDS per MFMA, and both the staging writes and
// the fragment reads per MFMA fall with the tile's sides:
//   128x256 for results at least 256 wide with at least three rounds of such tiles (a quarter fewer LDS and load
//           instructions per MFMA than 128x128: 5 to 20 % on such layers; with fewer rounds the coarser tiles
//           leave compute units idle at the end);
//   256x256 (eight waves) for results at least 256 wide whose tiles fill whole rounds of the chip well enough;
//   256x64  for results at most 64 wide with at least three rounds of such tiles: a wave then owns 128 x 32 and
//           issues as many MFMAs per load as in the 128x128 tile (4 to 7 % on the 56x56 layers with 64 filters
//           or channels).
// The few-channels and scatter variants are built for 128 rows and 64 or 128 columns only.
struct MainTile {
    int bm, bn;
};
inline MainTile main_tile(const GemmConv& p) {
    static const bool no_wide = getenv("LARSCONV_NO_WIDE_TILE") != nullptr;    // comparison runs
    static const bool no_tall = getenv("LARSCONV_NO_TALL_TILE") != nullptr;
    static const bool no_big = getenv("LARSCONV_NO_BIG_TILE") != nullptr;
    MainTile t{128, p.N <= 64 ? 64 : 128};
    if (!p.bf16 || p.Ci < 32 || p.scatter) return t;
    if (p.N <= 64) {
        if (!no_tall && (p.M + 255) / 256 >= 3LL * resident_blocks(256, 64)) t.bm = 256;
        return t;
    }
    if (p.N >= 256 && !no_big) {
        // 256x256, eight waves: half the operand bytes per MFMA through the vector-memory path and LDS of the 128x128 tile.
        // Taken when its tiles fill the chip at least once and the last, partly filled round wastes less than the tile
        // gains (measured over ResNet-50's layers at batch 512: results up to 512 wide gain 5 to 20 % from 70 % fill on;
        // wider results only with at least 16 k-steps per tile and 85 % fill, otherwise the 128x256 tile is faster).
        const long long tiles = (long long)((p.M + 255) / 256) * ((p.N + 255) / 256);
        const long long res = resident_blocks(256, 256);
        const long long rounds = (tiles + res - 1) / res;
        const int nkt = (p.Kg + 31) / 32;
        static const int fill_env = [] {
            const char* e = getenv("LARSCONV_BIG_TILE_FILL");                  // comparison runs: another threshold
            return e ? atoi(e) : 0;
        }();
        const int fill = fill_env ? fill_env : (p.N <= 512 ? 70 : 85);
        if (tiles >= res && tiles * 100 >= rounds * res * fill && (fill_env || p.N <= 512 || nkt >= 16)) return MainTile{256, 256};
    }
    if (p.N >= 256 && !no_wide) {
        const long long tiles = (long long)((p.M + 127) / 128) * ((p.N + 255) / 256);
        if (tiles >= 3LL * resident_blocks(128, 256)) t.bn = 256;
    }
    return t;
}

template <int BM, int BN>
bool sk_geometry(const GemmConv& p, long long* tiles, int* nkt) {
    const int bk = p.bf16 ? 32 : 16;
    *tiles = (long long)((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
    *nkt = (p.Kg + bk - 1) / bk;
    return *tiles > 0 && *tiles * *nkt < 0x7fffffffLL;
}

// Whether the uniform-tap variant of the main kernel takes this problem: k-steps that do not straddle taps,
// a tap mask that fits 32 bits, and tile-relative byte offsets (the images a tile can touch plus one filter
// window, and BN filter rows) that stay below 2^31.
template <int BM, int BN>
bool uniform_tap_ok(const GemmConv& p) {
    static const bool off = getenv("LARSCONV_NO_UNIFORM_TAP") != nullptr;     // comparison runs
    const int bk = p.bf16 ? 32 : 16, es = p.bf16 ? 2 : 4;
    if (off || p.Ci % bk != 0 || (long long)p.R * p.S > 32) return false;
    const long long pq = (long long)p.Po * p.Qo;
    const long long images = BM / pq + 2;
    const long long a_span = ((images * p.Hi + (p.ph > 0 ? p.ph : 0) + p.R + 1) * p.Wi + p.S + 1) * p.Ci * es;
    const long long b_span = (long long)(BN + 1) * p.Kg * es;
    return a_span < 0x7fff0000LL && b_span < 0x7fff0000LL;
}

// Constants for div_by(): n / d == umulhi(n, mul) >> shift for 0 <= n < 2^31 (mul == 0 stands for d == 1).
// With L = ceil(log2 d) and mul = ceil(2^(31+L) / d) the error term n * (mul*d - 2^(31+L)) stays below 2^(31+L).
void magic_for(int d, unsigned* mul, unsigned* shift) {
    if (d <= 1) {
        *mul = 0;
        *shift = 0;
        return;
    }
    int L = 0;
    while ((1ll << L) < d) ++L;
    *mul = (unsigned)((((unsigned long long)1 << (31 + L)) + (unsigned)d - 1) / (unsigned)d);
    *shift = (unsigned)(L - 1);
}

}  // namespace

// Host-side check of the division constants against plain division (the device evaluates the same two
// operations with __umulhi): 0 if n / d is reproduced for every divisor up to max_d at the edges of each
// quotient step and at the top of the 31-bit range, otherwise the first failing divisor.
extern "C" int lc_selftest_division(int max_d) {
    for (int d = 1; d <= max_d; ++d) {
        unsigned mul, shift;
        magic_for(d, &mul, &shift);
        auto q = [&](unsigned n) { return mul ? (unsigned)(((unsigned long long)n * mul) >> 32) >> shift : n; };
        const unsigned top = 0x7fffffffu;
        const unsigned probes[] = {0u, 1u, (unsigned)d - 1, (unsigned)d, (unsigned)d + 1, 2u * d - 1, 2u * d, 1000003u, top - 1, top,
                                   top / d * d, top / d * d - 1};
        for (unsigned n : probes)
            if (n <= top && q(n) != n / (unsigned)d) return d;
        for (unsigned k = 1; k < 4096; ++k) {                   // quotient steps spread over the range
            const unsigned long long n = (unsigned long long)k * 524287ull % (top / d + 1) * d;
            if (n >= 1 && (q((unsigned)n) != n / d || q((unsigned)n - 1) != (n - 1) / d)) return d;
        }
    }
    return 0;
}

namespace {

template <int BM, int BN, bool SMALLC, bool BF16>
lc_status launch_conv_sk(GemmConv p, hipStream_t stream) {
    long long tiles;
    int nkt;
    if (!sk_geometry<BM, BN>(p, &tiles, &nkt)) return LC_ERR_UNSUPPORTED;
    const int resident = resident_blocks(BM, BN);
    // (a 256x256 tile's partial sums are 256 KB per block and piece: writing and re-reading them costs more than the idle
    // end of the last round, which main_tile() has already bounded)
    SkPlan pl = sk_plan(tiles, nkt, resident, BM * BN < 256 * 256);
    // persistent kernel: one round of resident blocks, each taking dp_tiles / grid whole tiles and then its
    // stream-K range; without a workspace for partial tiles the ranges are whole tiles
    if (pl.sk_blocks > 0 && !p.partial) pl.sk_blocks = 0;
    if (pl.sk_blocks == 0) {
        const long long rest = tiles % resident;
        pl.dp_tiles = (int)(tiles - rest);
        pl.sk_blocks = (int)rest;
        pl.sk_iters = rest * nkt;
    }
    p.dp_tiles = pl.dp_tiles;
    p.sk_blocks = pl.sk_blocks;
    p.sk_iters = pl.sk_iters;
    magic_for(p.Qo, &p.qo_mul, &p.qo_shift);
    magic_for(p.Po, &p.po_mul, &p.po_shift);
    const unsigned grid = pl.dp_tiles > 0 ? (unsigned)resident : (unsigned)pl.sk_blocks;
    const dim3 threads(2 * pk_waves_n(BM, BN) * 64);
    const bool whole = pl.sk_blocks == 0 || pl.sk_iters == (long long)pl.sk_blocks * nkt;
    const bool ut = !SMALLC && uniform_tap_ok<BM, BN>(p);
    if (p.scatter && p.stats) return LC_ERR_UNSUPPORTED;
    if (p.scatter) {                          // the scatter epilogue addresses the result relative to the tile's first pixel
        const long long span = ((long long)BM / ((long long)p.Po * p.Qo) + 2) * p.Ho * p.Wo * p.ldd * (p.bf16 ? 2 : 4);
        if (span >= 0x7fff0000LL || SMALLC || BN > 128 || BM > 128) return LC_ERR_UNSUPPORTED;   // (1x1 windows never have fewer channels than a k-step)
        if constexpr (BN <= 128 && BM <= 128) {
            if (ut)
                hipLaunchKernelGGL((conv_gemm_pk_kernel<BM, BN, false, BF16, true, true>), dim3(grid), threads, 0, stream, p);
            else
                hipLaunchKernelGGL((conv_gemm_pk_kernel<BM, BN, false, BF16, false, true>), dim3(grid), threads, 0, stream, p);
        }
    } else if (ut) {
        hipLaunchKernelGGL((conv_gemm_pk_kernel<BM, BN, false, BF16, true, false>), dim3(grid), threads, 0, stream, p);
    } else {
        hipLaunchKernelGGL((conv_gemm_pk_kernel<BM, BN, SMALLC, BF16, false, false>), dim3(grid), threads, 0, stream, p);
    }
    if (!whole) {
        hipLaunchKernelGGL((conv_gemm_fixup_kernel<BM, BN, BF16>), dim3((unsigned)(tiles - pl.dp_tiles), 16), threads, 0, stream, p);
        if (p.stats) {
            const dim3 sgrid((unsigned)(tiles - pl.dp_tiles), 2);
            const bool vec4 = p.N % 4 == 0 && p.ldd % 4 == 0 && (reinterpret_cast<uintptr_t>(p.d) & 15) == 0;
            if (vec4)
                hipLaunchKernelGGL((tile_stats_kernel<BF16, true>), sgrid, dim3(256), 0, stream, p, BM, BN, pl.dp_tiles);
            else
                hipLaunchKernelGGL((tile_stats_kernel<BF16, false>), sgrid, dim3(256), 0, stream, p, BM, BN, pl.dp_tiles);
        }
    }
    return lc_end_call();
}

inline bool use_main_kernel(const GemmConv& p) {
    static const bool classic = [] {
        const char* e = getenv("LARSCONV_KERNEL");          // LARSCONV_KERNEL=classic: comparison runs
        return e && strcmp(e, "classic") == 0;
    }();
    const bool vec = (p.Ci % (p.bf16 ? 8 : 4) == 0) && aligned16(p.a) && aligned16(p.b);
    // (the scatter epilogue of the main kernel is not built for its few-channels variant)
    const bool few_scatter = p.scatter && p.Ci < (p.bf16 ? 32 : 16);
    // (its tile store addresses a tile's rows with 32-bit byte offsets)
    const bool wide_rows = (long long)288 * p.ldd * (p.bf16 ? 2 : 4) >= 0x7fff0000LL;
    return vec && !(p.dh > 1 || p.dw > 1) && !(classic && !p.bf16) && !few_scatter && !wide_rows;
}

}  // namespace

// Calls f.template operator()<BM, BN>() for the tile main_tile() picks.
template <typename F>
auto with_main_tile(const GemmConv& p, F&& f) {
    const MainTile t = main_tile(p);
    if (t.bm == 256 && t.bn == 256) return f.template operator()<256, 256>();
    if (t.bm == 256) return f.template operator()<256, 64>();
    if (t.bn == 256) return f.template operator()<128, 256>();
    if (t.bn == 128) return f.template operator()<128, 128>();
    return f.template operator()<128, 64>();
}

size_t lc_conv_gemm_workspace(const GemmConv& p) {
    if (!use_main_kernel(p)) return 0;
    return with_main_tile(p, [&]<int BM, int BN>() -> size_t {
        long long tiles;
        int nkt;
        if (!sk_geometry<BM, BN>(p, &tiles, &nkt)) return 0;
        const SkPlan pl = sk_plan(tiles, nkt, resident_blocks(BM, BN), BM * BN < 256 * 256);
        return (size_t)2 * pl.sk_blocks * BM * BN * sizeof(float);
    });
}

bool lc_conv_gemm_bf16_native(const GemmConv& p) { return p.bf16 && use_main_kernel(p); }

bool lc_conv_gemm_scatter_ok(const GemmConv& p) {
    if (!p.scatter || !use_main_kernel(p) || p.Ci < (p.bf16 ? 32 : 16)) return false;
    // (the scatter epilogue addresses the result relative to the tile's first pixel with 32-bit byte offsets)
    const long long span = (128LL / ((long long)p.Po * p.Qo) + 2) * p.Ho * p.Wo * p.ldd * (p.bf16 ? 2 : 4);
    return span < 0x7fff0000LL;
}

// The slab kernel's conditions: bf16, 3x3 window with stride 1 and padding 1 (so the output has the input's size),
// whole 32-channel chunks, byte offsets that fit 31 bits, a slab of at most 512 pixels, and enough tiles to fill the chip
// (below that the main kernel's stream-K split is worth more).  Returns the LDS bytes of the launch in *lds.
static bool slab_kernel_ok(const GemmConv& p, int bn, size_t* lds) {
    static const bool off = getenv("LARSCONV_NO_SLAB") != nullptr;       // comparison runs
    if (off || !p.bf16 || p.scatter || p.R != 3 || p.S != 3 || p.sh != 1 || p.sw != 1 || p.ph != 1 || p.pw != 1 || p.dh > 1 || p.dw > 1)
        return false;
    if (p.Po != p.Hi || p.Qo != p.Wi || p.Ci % 32 != 0 || p.Kg != 9 * p.Ci) return false;
    if (!aligned16(p.a) || !aligned16(p.b) || (reinterpret_cast<uintptr_t>(p.d) & 3)) return false;
    const long long hw = (long long)p.Hi * p.Wi;
    if (p.M % hw != 0) return false;
    if ((long long)p.M * p.Ci * 2 >= 0x7fff0000LL || (long long)p.N * 9 * p.Ci * 2 >= 0x7fff0000LL || (long long)288 * p.ldd * 2 >= 0x7fff0000LL)
        return false;
    // rows a tile's 128 consecutive pixels can span, the empty rows between the images it can touch, and the two halo rows
    const long long rows = (128 + p.Wi - 2) / p.Wi + (128 + hw - 2) / hw + 3;
    const long long px = rows * (p.Wi + 2);
    if (px > (long long)kSlabMaxVec * 64) return false;
    *lds = (size_t)2 * bn * 64 + (size_t)px * kSlabPitch;
    const char* e = getenv("LARSCONV_SLAB_MIN_TILES");                      // tests lower it to send small shapes here
    const long long min_tiles = e ? atoll(e) : device_cu_count();
    const long long tiles = (long long)((p.M + 127) / 128) * ((p.N + bn - 1) / bn);
    if (tiles < min_tiles) return false;
    // where the main kernel runs its 256x256 tile (half the filter bytes per MFMA as well) it measures 4-6 % faster
    const MainTile t = main_tile(p);
    return e != nullptr || !(t.bm == 256 && t.bn == 256);
}

template <int BN>
static lc_status launch_slab(const GemmConv& p, size_t lds, hipStream_t stream) {
    static bool once = [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(conv3x3_slab_kernel<BN>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   2 * BN * 64 + kSlabMaxVec * 64 * kSlabPitch) == hipSuccess;
    }();
    if (!once) return LC_ERR_LAUNCH;
    const long long tiles = (long long)((p.M + 127) / 128) * ((p.N + BN - 1) / BN);
    hipLaunchKernelGGL((conv3x3_slab_kernel<BN>), dim3((unsigned)tiles), dim3(256), lds, stream, p);
    return lc_end_call();
}

// The tile the main kernel runs a problem with (0 x 0: another kernel takes it); mirrors lc_launch_conv_gemm.
static void main_kernel_tile(const GemmConv& p, int* bm, int* bn) {
    *bm = *bn = 0;
    size_t lds;
    if (p.bf16 && slab_kernel_ok(p, p.N > 64 ? 128 : 64, &lds)) {       // the slab kernel: 128 rows
        *bm = 128;
        *bn = p.N > 64 ? 128 : 64;
        return;
    }
    if (!use_main_kernel(p) || p.scatter) return;
    if (p.bf16) {
        if (p.Ci < 32) {
            *bm = 128;
            *bn = p.N > 64 ? 128 : 64;
        } else {
            const MainTile t = main_tile(p);
            *bm = t.bm;
            *bn = t.bn;
        }
        return;
    }
    *bm = 128;
    *bn = p.N > 64 ? 128 : 64;
}

size_t lc_conv_gemm_stats_tiles(const GemmConv& p) {
    int bm, bn;
    main_kernel_tile(p, &bm, &bn);
    return bm ? (size_t)2 * ((p.M + bm - 1) / bm) : 0;
}

lc_status lc_launch_conv_gemm(const GemmConv& p, hipStream_t stream) {
    if (p.stats && lc_conv_gemm_stats_tiles(p) == 0) return LC_ERR_UNSUPPORTED;
    if (p.bf16) {
        size_t lds;
        const int bn = p.N > 64 ? 128 : 64;
        if (slab_kernel_ok(p, bn, &lds)) return bn == 128 ? launch_slab<128>(p, lds, stream) : launch_slab<64>(p, lds, stream);
    }
    if (p.bf16) {
        if (!use_main_kernel(p)) return LC_ERR_UNSUPPORTED;       // the caller converts to fp32 instead
        if (p.Ci < 32) return p.N > 64 ? launch_conv_sk<128, 128, true, true>(p, stream) : launch_conv_sk<128, 64, true, true>(p, stream);
        return with_main_tile(p, [&]<int BM, int BN>() { return launch_conv_sk<BM, BN, false, true>(p, stream); });
    }
    const bool vec = (p.Ci % 4 == 0) && aligned16(p.a) && aligned16(p.b);
    if (!vec) return launch_conv<64, 64, 16, 1>(p, stream);
    if (use_main_kernel(p)) {
        if (p.Ci < 16) return p.N > 64 ? launch_conv_sk<128, 128, true, false>(p, stream) : launch_conv_sk<128, 64, true, false>(p, stream);
        return p.N > 64 ? launch_conv_sk<128, 128, false, false>(p, stream) : launch_conv_sk<128, 64, false, false>(p, stream);
    }
    if (p.N > 64) return launch_conv<128, 128, 16, 4>(p, stream);
    return launch_conv<128, 64, 16, 4>(p, stream);
}

// Output tile of the filter-gradient kernel for a shape (also fixes the split count).
static void wgrad_tile(int K, int J, int* bm, int* bn) {
    *bm = K > 64 ? 128 : 64;
    *bn = J > 64 ? 128 : 64;
}

int lc_wgrad_splits(int M, int K, int J, bool bf16) {
    int bm, bn;
    wgrad_tile(K, J, &bm, &bn);
    const long long tiles = (long long)((K + bm - 1) / bm) * ((J + bn - 1) / bn);
    // blocks of this tiling that fit on the chip at once (registers and LDS of the kernel instances below):
    // the split count fills exactly one such round, never spills a few blocks into a second one
    const int per_cu = (bm == 128 && bn == 128) ? 4 : (bm == 64 && bn == 64) ? 8 : (bf16 ? 5 : 6);
    const long long round = (long long)per_cu * device_cu_count();
    long long want = round / tiles;
    const long long most = (M + 255) / 256;               // at least 256 reduction rows per split
    if (want > most) want = most;
    if (want < 1) want = 1;
    if (want > 8192) want = 8192;
    return (int)want;
}

// Whether wgrad3x3_slab_kernel takes a layer (a fixed function of the shape: the plan's workspace depends on it).
bool lc_wgrad_slab_ok(int imgs, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw, int P, int Q, bool bf16) {
    if (getenv("LARSCONV_NO_WGRAD_SLAB")) return false;                    // comparison runs
    if (!bf16 || R != 3 || S != 3 || sh != 1 || sw != 1 || ph != 1 || pw != 1 || P != H || Q != W) return false;
    if (C % 64 != 0 || K % 64 != 0 || W < 6 || (W + 3 + 31) / 32 > kWsMaxL) return false;
    // narrow images spend too many MFMAs on halo positions (2 of every W + 2) and the 128-wide tiles of
    // wgrad_bf16_kernel are as fast from 14 x 14 down; tests lower the threshold to send small shapes here
    const char* e = getenv("LARSCONV_WGRAD_SLAB_MIN_W");
    if (W < (e ? atoi(e) : 24)) return false;
    const long long pixels = (long long)imgs * H * W, positions = (long long)imgs * (H + 1) * (W + 2);
    return pixels * (C > K ? C : K) * 2 < 0x7fff0000LL && positions < 0x7ff00000LL;
}

// Splits of its reduction: two blocks per compute unit in one round, at least 256 positions each.
int lc_wgrad_slab_splits(int imgs, int H, int W, int C, int K, int* pos_per_split) {
    const long long tiles = (long long)(K / 64) * (C / 64), positions = (long long)imgs * (H + 1) * (W + 2);
    long long want = 2LL * device_cu_count() / tiles;
    const long long most = (positions + 255) / 256;
    if (want > most) want = most;
    if (want < 1) want = 1;
    if (want > 8192) want = 8192;
    *pos_per_split = (int)(((positions + want - 1) / want + 31) / 32 * 32);
    return (int)want;
}

static lc_status launch_wgrad_slab(const GemmWgrad& p, hipStream_t stream) {
    constexpr size_t most = (size_t)(2 * 32 + (2 * kWsMaxL + 2) * 32 + 16) * kWsPitch * 2;
    static bool once = [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad3x3_slab_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)most) ==
               hipSuccess;
    }();
    if (!once) return LC_ERR_LAUNCH;
    if (!aligned16(p.dy) || !aligned16(p.x) || p.m_per_split % 32 != 0) return LC_ERR_ALIGN;
    const int L = (p.W + 3 + 31) / 32;
    const size_t lds = (size_t)(2 * 32 + (2 * L + 2) * 32 + 16) * kWsPitch * 2;
    const long long tiles = (long long)(p.K / 64) * (p.C / 64);
    if (L > kWsMaxL || tiles * p.splits > 0x7fffffffLL) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(wgrad3x3_slab_kernel, dim3((unsigned)(tiles * p.splits)), dim3(256), lds, stream, p);
    return lc_end_call();
}

template <int BM, int BN>
static lc_status launch_wgrad_bf16(const GemmWgrad& p, hipStream_t stream) {
    const long long tiles = (long long)((p.K + BM - 1) / BM) * ((p.J + BN - 1) / BN);
    if (tiles <= 0 || tiles * p.splits > 0x7fffffffLL) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((wgrad_bf16_kernel<BM, BN>), dim3((unsigned)(tiles * p.splits)), dim3(256), 0, stream, p);
    return lc_end_call();
}

// Whether wgrad_ut_kernel takes this problem: 16-byte vectors (channel counts multiples of 4, of 8 for bf16), a
// window of at most 32 taps, and buffer offsets (a split's rows of dY; the images a split touches plus one
// window of X) below 2^31 bytes.
static bool wgrad_ut_ok(const GemmWgrad& p) {
    static const bool off = getenv("LARSCONV_NO_UNIFORM_TAP") != nullptr;     // comparison runs
    const int epc = p.bf16 ? 8 : 4, es = p.bf16 ? 2 : 4;
    if (off || p.C % epc != 0 || p.K % epc != 0 || (long long)p.R * p.S > 32) return false;
    if ((((uintptr_t)p.dy | (uintptr_t)p.x) & 15) != 0) return false;
    const long long rows = (long long)p.m_per_split + 64;
    const long long a_span = rows * p.K * es;
    const long long images = rows / ((long long)p.P * p.Q) + 2;
    const long long b_span = ((images * p.H + (p.ph > 0 ? p.ph : 0) + p.R + 1) * p.W + p.S + 1) * p.C * es;
    return a_span < 0x7fff0000LL && b_span < 0x7fff0000LL;
}

template <int BM, int BN, bool BF16, bool PLAIN>
static lc_status launch_wgrad_ut(const GemmWgrad& p, hipStream_t stream) {
    const long long tiles = (long long)((p.K + BM - 1) / BM) * ((p.J + BN - 1) / BN);
    if (tiles <= 0 || tiles * p.splits > 0x7fffffffLL) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((wgrad_ut_kernel<BM, BN, BF16, PLAIN>), dim3((unsigned)(tiles * p.splits)), dim3(256), 0, stream, p);
    return lc_end_call();
}

template <bool BF16>
static lc_status dispatch_wgrad(const GemmWgrad& p, hipStream_t stream) {
    if (p.slab) return BF16 ? launch_wgrad_slab(p, stream) : LC_ERR_UNSUPPORTED;   // (m_per_split counts positions: no other kernel can take it)
    if (wgrad_ut_ok(p) && !(BF16 && getenv("LARSCONV_WGRAD_WIDEN"))) {
        // only the 128 x 128 tiling: with narrower tiles a step has too few MFMAs to hide the scalar work and the
        // narrower loads, and the kernels below measure faster
        int bm, bn;
        wgrad_tile(p.K, p.J, &bm, &bn);
        // (bf16: only the plain 1x1 case -- with eight pixels per wave and step and an eighth of the MFMA time the
        // per-pixel scalar work of the general case does not hide)
        const bool plain = p.R == 1 && p.S == 1 && p.sh == 1 && p.sw == 1 && p.ph == 0 && p.pw == 0 && p.H == p.P && p.W == p.Q;
        if (bm == 128 && bn == 128 && plain) return launch_wgrad_ut<128, 128, BF16, true>(p, stream);
        if (plain) {                                  // (no per-pixel work: pays with every tile shape)
            if (bm == 128) return launch_wgrad_ut<128, 64, BF16, true>(p, stream);
            if (bn == 128) return launch_wgrad_ut<64, 128, BF16, true>(p, stream);
            return launch_wgrad_ut<64, 64, BF16, true>(p, stream);
        }
        if (bm == 128 && bn == 128 && !BF16) return launch_wgrad_ut<128, 128, false, false>(p, stream);
    }
    if (BF16 && p.C % 8 == 0 && p.K % 8 == 0 && aligned16(p.dy) && aligned16(p.x) && !getenv("LARSCONV_WGRAD_WIDEN")) {
        int bm, bn;                                   // the bf16 matrix pipe; LARSCONV_WGRAD_WIDEN=1: comparison runs
        wgrad_tile(p.K, p.J, &bm, &bn);
        if (bm == 128 && bn == 128) return launch_wgrad_bf16<128, 128>(p, stream);
        if (bm == 128) return launch_wgrad_bf16<128, 64>(p, stream);
        if (bn == 128) return launch_wgrad_bf16<64, 128>(p, stream);
        return launch_wgrad_bf16<64, 64>(p, stream);
    }
    // vector path: 4 elements per load (16 bytes fp32, 8 bytes bf16)
    const uintptr_t amask = BF16 ? 7 : 15;
    const bool vec = (p.C % 4 == 0) && (p.K % 4 == 0) && !(((uintptr_t)p.dy | (uintptr_t)p.x) & amask);
    int bm, bn;
    wgrad_tile(p.K, p.J, &bm, &bn);
    if (!vec) return launch_wgrad<64, 64, 16, 1, BF16>(p, stream);
    if (bm == 128 && bn == 128) return launch_wgrad<128, 128, 16, 4, BF16>(p, stream);
    if (bm == 128) return launch_wgrad<128, 64, 16, 4, BF16>(p, stream);
    if (bn == 128) return launch_wgrad<64, 128, 16, 4, BF16>(p, stream);
    return launch_wgrad<64, 64, 16, 4, BF16>(p, stream);
}

lc_status lc_launch_wgrad_f32(const GemmWgrad& p, hipStream_t stream) {
    return p.bf16 ? dispatch_wgrad<true>(p, stream) : dispatch_wgrad<false>(p, stream);
}
