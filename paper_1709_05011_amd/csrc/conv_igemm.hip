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
template <int TM, int TN>
__device__ __forceinline__ void store_tile(const GemmConv& p, const f32x16 (&acc)[TM][TN], int row0, int col0, int lane) {
    float* __restrict__ D = static_cast<float*>(p.d);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (row >= p.M) continue;
            if (!p.scatter) {
                float* drow = D + (long long)row * p.ldd;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = col0 + j * 32 + (lane & 31);
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
                            const int col = col0 + j * 32 + (lane & 31);
                            if (col < p.N) drow[col] = corner ? acc[i][j][v] : 0.f;
                        }
                    }
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
// forward / backward-data kernel, pipelined: global -> LDS without passing through registers
// (global_load_lds_dwordx4), STAGES tiles in flight, fragments of the next k-step read while the
// current one is multiplied.  Requires channel counts that are multiples of 4 and no dilated read.
//
// LDS tile: [row][16 floats] unpadded (a wave-wide direct load fills 16 rows x 64 B contiguously); the
// four 16-byte chunks of a row are permuted by chunk ^ swz(row) so that the b128 fragment reads of 8 or
// 16 consecutive rows hit distinct banks.  The permutation is applied on the global side: the lane that
// owns LDS slot s of a row fetches chunk s ^ swz(row).  Positions outside the image, rows past M or N
// and columns past Kg fetch from a 16-byte block of zeros instead, so every lane always loads.
// ------------------------------------------------------------------------------------------------
__device__ __attribute__((aligned(16))) const float g_zero_chunk[4] = {0.f, 0.f, 0.f, 0.f};

__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 2)) & 3; }

// The direct loads and the waits on them are written as inline assembly: the compiler then keeps no
// score of them and does not add a wait for *all* loads in flight in front of every LDS read (it cannot
// tell the stages apart); the kernel counts them itself.  Each is a compiler barrier for memory accesses.
// m0 holds the wave-uniform LDS byte address of the 1 KB run the 64 lanes fill (16 B per lane, lane order).
__device__ __forceinline__ void lds_dma16(const void* gptr, unsigned lds_byte_addr) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_byte_addr) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
// ok ? a : b on pointers by bit masking: never a branch, whatever the cost of computing a
__device__ __forceinline__ const float* pick(bool ok, const float* a, const float* b) {
    const uintptr_t m = (uintptr_t)0 - (uintptr_t)ok;
    return reinterpret_cast<const float*>((reinterpret_cast<uintptr_t>(a) & m) | (reinterpret_cast<uintptr_t>(b) & ~m));
}
// 16-byte load through the global (not flat) path: a flat load would also count as an LDS operation
__device__ __forceinline__ float4 load_global16(const float* ptr) {
    typedef float gf4 __attribute__((ext_vector_type(4)));
    const gf4 v = *(const __attribute__((address_space(1))) gf4*)(uintptr_t)ptr;
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" : : : "memory"); }

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Three LDS stages hold tiles kt-1 (being vacated), kt (being multiplied) and kt+1 (landing).  Per tile:
//   read the k = 8..15 fragments of tile kt; first 4 MFMAs of its k = 0..7 half
//   wait for this thread's loads of tile kt+1, barrier          (everybody's loads have landed)
//   issue the loads of tile kt+2 into the stage of tile kt-1, one load per group of 4 MFMAs, so that the
//   address arithmetic runs in the shadow of the matrix pipe
//   read the k = 0..7 fragments of tile kt+1; the 16 MFMAs of the k = 8..15 half of tile kt
// A stage is overwritten only one full iteration after its last fragment read was consumed by an MFMA,
// so no wait on LDS reads is needed in front of the barrier.
// SMALLC: the gathered tensor has fewer than 16 channels, one 16-wide k-step then spans several filter taps.
template <int BM, int BN, bool SMALLC, bool DIST2>
__global__ void __launch_bounds__(256) conv_gemm_f32_pipe_kernel(const GemmConv p) {
    constexpr int BK = 16, STAGES = 3;
    constexpr int LA = BM / 64, LB = BN / 64;     // 16-row blocks per wave and tile
    constexpr int LPT = LA + LB;                  // direct loads per thread and tile
    constexpr int WTM = BM / 2, WTN = BN / 2, TM = WTM / 32, TN = WTN / 32;
    constexpr int STAGE = (BM + BN) * BK;         // floats per stage: A rows then B rows
    static_assert(BM % 64 == 0 && BN % 64 == 0, "tile shape");

    __shared__ __attribute__((aligned(1024))) float lds[STAGES * STAGE];
    const unsigned lds_addr = (unsigned)(uintptr_t)(lds_ptr_t)lds;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform, lives in an SGPR
    const int wm = wave >> 1, wn = wave & 1;
    const int nbn = (p.N + BN - 1) / BN;
    const int tile = xcd_tile(blockIdx.x, gridDim.x);
    const int m0 = (tile / nbn) * BM, n0 = (tile % nbn) * BN;

    const float* __restrict__ A = static_cast<const float*>(p.a);
    const float* __restrict__ B = static_cast<const float*>(p.b);

    // this lane's place in a 16-row block: row lane/4, LDS slot lane%4, global chunk slot ^ swz(row)
    const int lrow = lane >> 2;
    const int kq = (lane & 3) ^ swz(lrow);

    long long a_base[LA];
    int a_h[LA], a_w[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int m = m0 + (i * 4 + wave) * 16 + lrow;
        if (m < p.M) {
            const int qo = m % p.Qo, t = m / p.Qo;
            const int po = t % p.Po, img = t / p.Po;
            a_h[i] = po * p.sh - p.ph;
            a_w[i] = qo * p.sw - p.pw;
            a_base[i] = (long long)img * p.Hi * p.Wi * p.Ci;
        } else {
            a_h[i] = -(1 << 28);
            a_w[i] = 0;
            a_base[i] = 0;
        }
    }
    long long b_off[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int n = n0 + (i * 4 + wave) * 16 + lrow;
        b_off[i] = n < p.N ? (long long)n * p.Kg : -1;
    }

    int kg = kq * 4;
    // copies of the descriptor fields used inside the main loop (the inline-assembly memory clobbers would
    // otherwise make the compiler re-read them from the kernel arguments every iteration)
    const int Hi_ = p.Hi, Wi_ = p.Wi, Ci_ = p.Ci, R_ = p.R, S_ = p.S;
    int c = kg % p.Ci, r, s;
    {
        const int rs = kg / p.Ci;
        s = rs % p.S;
        r = rs / p.S;
    }

    // direct load number l (A blocks first, then B blocks) of the tile at (r, s, c) into stage st
    auto issue_one = [&](int st, int l) {
        const unsigned base = lds_addr + (unsigned)(st * STAGE + wave * 256) * 4u;
        const bool kok = r < R_;
        if (l < LA) {
            const int h = a_h[l] + r, w = a_w[l] + s;
            const bool ok = kok & ((unsigned)h < (unsigned)Hi_) & ((unsigned)w < (unsigned)Wi_);   // no short-circuit branches
            lds_dma16(pick(ok, A + a_base[l] + ((long long)h * Wi_ + w) * Ci_ + c, g_zero_chunk), base + l * 4096u);
        } else {
            const int i = l - LA;
            lds_dma16(pick(kok & (b_off[i] >= 0), B + b_off[i] + kg, g_zero_chunk), base + (unsigned)(BM * BK) * 4u + i * 4096u);
        }
    };
    // step (r, s, c) to the next tile
    auto advance = [&]() {
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
        } else {                                  // at most one wrap: written without branches
            const bool wrap = c >= Ci_;
            c = wrap ? c - Ci_ : c;
            s += wrap ? 1 : 0;
            const bool wrap2 = s == S_;
            s = wrap2 ? 0 : s;
            r += wrap2 ? 1 : 0;
        }
    };
    auto issue_tile = [&](int st) {
#pragma unroll
        for (int l = 0; l < LPT; ++l) issue_one(st, l);
        advance();
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment addressing: lane reads row (lane & 31) of a 32-row MFMA tile, chunk 2*k8 + (lane >> 5)
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = swz(frow);
    const int a_frag = (wm * WTM + frow) * BK, b_frag = BM * BK + (wn * WTN + frow) * BK;
    float4 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int st, int k8, int slot) {
        const float* base = lds + st * STAGE;
        const int ch = ((2 * k8 + fhalf) ^ fsw) * 4;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[slot][i] = *reinterpret_cast<const float4*>(base + a_frag + i * 32 * BK + ch);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[slot][j] = *reinterpret_cast<const float4*>(base + b_frag + j * 32 * BK + ch);
    };
    auto mfma_e = [&](int slot, int e) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(elem(fa[slot][i], e), elem(fb[slot][j], e), acc[i][j], 0, 0, 0);
    };

    const int nkt = (p.Kg + BK - 1) / BK;
    issue_tile(0);
    issue_tile(1);
    wait_vmcnt<LPT>();                            // tile 0 has landed (this thread's part)
    block_barrier();
    if (DIST2) issue_tile(2);
    read_frags(0, 0, 0);
    int st = 0;                                   // stage of tile kt
    // The last tile is peeled off so that the loop body has no branch between the fragment reads and the
    // MFMAs that follow them (a join there makes the compiler wait for the reads just issued).
    for (int kt = 0; kt + 1 < nkt; ++kt) {
        const int nx = st == 2 ? 0 : st + 1;      // stage of tile kt+1
        const int fr = nx == 2 ? 0 : nx + 1;      // stage of tile kt-1 = stage of tile kt+2
        read_frags(st, 1, 1);
        mfma_e(0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (DIST2) {
            wait_vmcnt<LPT>();                    // tile kt+1 landed; tile kt+2 may still be in flight
            asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");   // the k = 8..15 reads of tile kt are in registers
        } else {
            wait_vmcnt<0>();
        }
        block_barrier();
#pragma unroll
        for (int e = 1; e < 4; ++e) {             // loads spread over the three remaining MFMA groups
#pragma unroll
            for (int l = 0; l < LPT; ++l)
                if (l * 3 / LPT == e - 1) issue_one(DIST2 ? st : fr, l);
            if (e == 3) advance();
            mfma_e(0, e);
            __builtin_amdgcn_sched_barrier(0);
        }
        read_frags(nx, 0, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) mfma_e(1, e);
        st = nx;
    }
    read_frags(st, 1, 1);
#pragma unroll
    for (int e = 0; e < 4; ++e) mfma_e(0, e);
#pragma unroll
    for (int e = 0; e < 4; ++e) mfma_e(1, e);
    // the loads of the tile past the end (zeros) may still be in flight into LDS: let them land before exit
    wait_vmcnt<0>();

    store_tile<TM, TN>(p, acc, m0 + wm * WTM, n0 + wn * WTN, lane);
}

// ------------------------------------------------------------------------------------------------
// forward / backward-data kernel, register-staged variant of the pipelined kernel: same LDS layout and
// MFMA schedule, but a tile travels global -> registers (one iteration in flight) -> LDS (two buffers).
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, bool SMALLC>
__global__ void __launch_bounds__(256) conv_gemm_f32_stage_kernel(const GemmConv p) {
    constexpr int BK = 16;
    constexpr int LA = BM / 64, LB = BN / 64, LPT = LA + LB;
    constexpr int WTM = BM / 2, WTN = BN / 2, TM = WTM / 32, TN = WTN / 32;
    constexpr int STAGE = (BM + BN) * BK;
    static_assert(BM % 64 == 0 && BN % 64 == 0, "tile shape");

    __shared__ __attribute__((aligned(1024))) float lds[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int nbn = (p.N + BN - 1) / BN;
    const int tile = xcd_tile(blockIdx.x, gridDim.x);
    const int m0 = (tile / nbn) * BM, n0 = (tile % nbn) * BN;

    const float* __restrict__ A = static_cast<const float*>(p.a);
    const float* __restrict__ B = static_cast<const float*>(p.b);
    const int lrow = lane >> 2;
    const int kq = (lane & 3) ^ swz(lrow);

    long long a_base[LA];
    int a_h[LA], a_w[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int m = m0 + (i * 4 + wave) * 16 + lrow;
        if (m < p.M) {
            const int qo = m % p.Qo, t = m / p.Qo;
            const int po = t % p.Po, img = t / p.Po;
            a_h[i] = po * p.sh - p.ph;
            a_w[i] = qo * p.sw - p.pw;
            a_base[i] = (long long)img * p.Hi * p.Wi * p.Ci;
        } else {
            a_h[i] = -(1 << 28);
            a_w[i] = 0;
            a_base[i] = 0;
        }
    }
    long long b_off[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int n = n0 + (i * 4 + wave) * 16 + lrow;
        b_off[i] = n < p.N ? (long long)n * p.Kg : -1;
    }
    int kg = kq * 4;
    const int Hi_ = p.Hi, Wi_ = p.Wi, Ci_ = p.Ci, R_ = p.R, S_ = p.S;
    int c = kg % p.Ci, r, s;
    {
        const int rs = kg / p.Ci;
        s = rs % p.S;
        r = rs / p.S;
    }

    float4 g[LPT];                                // the tile in flight
    auto gload_one = [&](int l) {
        const bool kok = r < R_;
        float4 v;
        if (l < LA) {
            const int h = a_h[l] + r, w = a_w[l] + s;
            const bool ok = kok & ((unsigned)h < (unsigned)Hi_) & ((unsigned)w < (unsigned)Wi_);   // no short-circuit branches
            v = load_global16(pick(ok, A + a_base[l] + ((long long)h * Wi_ + w) * Ci_ + c, g_zero_chunk));
        } else {
            v = load_global16(pick(kok & (b_off[l - LA] >= 0), B + b_off[l - LA] + kg, g_zero_chunk));
        }
        g[l] = v;
    };
    auto advance = [&]() {
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
    };
    // registers -> LDS: lane (row lane/4, slot lane%4) of 16-row block (l*4 + wave); 16 B per lane, lane order
    auto sstore = [&](int buf) {
        float* base = lds + buf * STAGE + wave * 256 + lane * 4;
#pragma unroll
        for (int l = 0; l < LPT; ++l)
            *reinterpret_cast<float4*>(base + (l < LA ? l * 1024 : BM * BK + (l - LA) * 1024)) = g[l];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int frow = lane & 31, fhalf = lane >> 5;
    const int fsw = swz(frow);
    const int a_frag = (wm * WTM + frow) * BK, b_frag = BM * BK + (wn * WTN + frow) * BK;
    float4 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int buf, int k8, int slot) {
        const float* base = lds + buf * STAGE;
        const int ch = ((2 * k8 + fhalf) ^ fsw) * 4;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[slot][i] = *reinterpret_cast<const float4*>(base + a_frag + i * 32 * BK + ch);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[slot][j] = *reinterpret_cast<const float4*>(base + b_frag + j * 32 * BK + ch);
    };
    auto mfma_e = [&](int slot, int e) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(elem(fa[slot][i], e), elem(fb[slot][j], e), acc[i][j], 0, 0, 0);
    };
    // LDS writes and reads of this wave are complete, then the barrier; global loads stay in flight
    auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory"); };

    const int nkt = (p.Kg + BK - 1) / BK;
#pragma unroll
    for (int l = 0; l < LPT; ++l) gload_one(l);   // tile 0
    advance();
    sstore(0);
#pragma unroll
    for (int l = 0; l < LPT; ++l) gload_one(l);   // tile 1 (zeros if there is none)
    advance();
    lds_barrier();
    read_frags(0, 0, 0);
    int cur = 0;
    for (int kt = 0; kt + 1 < nkt; ++kt) {
        read_frags(cur, 1, 1);                    // k = 8..15 of tile kt
        mfma_e(0, 0);
        mfma_e(0, 1);
        __builtin_amdgcn_sched_barrier(0);
        sstore(cur ^ 1);                          // tile kt+1: its buffer was last read one iteration ago
        mfma_e(0, 2);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int l = 0; l < LPT; ++l) gload_one(l);   // tile kt+2 into the registers just stored
        advance();
        mfma_e(0, 3);
        __builtin_amdgcn_sched_barrier(0);
        lds_barrier();
        read_frags(cur ^ 1, 0, 0);                // k = 0..7 of tile kt+1
#pragma unroll
        for (int e = 0; e < 4; ++e) mfma_e(1, e);
        cur ^= 1;
    }
    read_frags(cur, 1, 1);
#pragma unroll
    for (int e = 0; e < 4; ++e) mfma_e(0, e);
#pragma unroll
    for (int e = 0; e < 4; ++e) mfma_e(1, e);

    store_tile<TM, TN>(p, acc, m0 + wm * WTM, n0 + wn * WTN, lane);
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

template <int BM, int BN, bool SMALLC, bool DIST2>
lc_status launch_conv_pipe(const GemmConv& p, hipStream_t stream) {
    const long long tiles = (long long)((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffffLL) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((conv_gemm_f32_pipe_kernel<BM, BN, SMALLC, DIST2>), dim3((unsigned)tiles), dim3(256), 0, stream, p);
    return lc_end_call();
}

template <int BM, int BN, bool SMALLC>
lc_status launch_conv_stage(const GemmConv& p, hipStream_t stream) {
    const long long tiles = (long long)((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
    if (tiles <= 0 || tiles > 0x7fffffffLL) return LC_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((conv_gemm_f32_stage_kernel<BM, BN, SMALLC>), dim3((unsigned)tiles), dim3(256), 0, stream, p);
    return lc_end_call();
}

// LARSCONV_KERNEL=classic selects the register-staged kernels everywhere (for comparison runs).
static bool use_pipe_kernels() {
    static const bool on = [] {
        const char* e = getenv("LARSCONV_KERNEL");
        return !(e && strcmp(e, "classic") == 0);
    }();
    return on;
}

}  // namespace

lc_status lc_launch_conv_gemm_f32(const GemmConv& p, hipStream_t stream) {
    const bool vec = (p.Ci % 4 == 0) && aligned16(p.a) && aligned16(p.b);
    if (!vec) return launch_conv<64, 64, 16, 1>(p, stream);
    const bool dilated = p.dh > 1 || p.dw > 1;
    if (!dilated && use_pipe_kernels()) {
        static const bool stage = [] { const char* e = getenv("LARSCONV_KERNEL"); return e && strcmp(e, "stage") == 0; }();
        if (stage) {
            if (p.Ci < 16) return p.N > 64 ? launch_conv_stage<128, 128, true>(p, stream) : launch_conv_stage<128, 64, true>(p, stream);
            return p.N > 64 ? launch_conv_stage<128, 128, false>(p, stream) : launch_conv_stage<128, 64, false>(p, stream);
        }
        static const bool d2 = [] { const char* e = getenv("LARSCONV_DIST"); return !(e && atoi(e) == 1); }();
        if (p.Ci < 16) return p.N > 64 ? launch_conv_pipe<128, 128, true, true>(p, stream) : launch_conv_pipe<128, 64, true, true>(p, stream);
        if (d2) return p.N > 64 ? launch_conv_pipe<128, 128, false, true>(p, stream) : launch_conv_pipe<128, 64, false, true>(p, stream);
        return p.N > 64 ? launch_conv_pipe<128, 128, false, false>(p, stream) : launch_conv_pipe<128, 64, false, false>(p, stream);
    }
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
