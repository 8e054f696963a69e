// Layer-wise LARS update for gfx950: segmented per-tensor norm reduction, then one streaming
// update pass.  Both kernels are bound by HBM bandwidth: 8 B/param for the norms (read w, g) and
// 20 B/param for the update (read w, g, v; write w, v), 22 with the bf16 weight copy.
//
// The parameter list is cut into fixed-size chunks of one tensor each, so that 161 tensors of
// 64 .. 2.4 M elements (ResNet-50) load the chip evenly and no launch is made per tensor.
//   1. lars_norm_kernel      two chunks per block: sum w^2 and sum g^2 of each (fp32 per thread over 16
//                            elements, then fp64 across lanes with wavefront shuffles and across waves
//                            through LDS) -> one fp64 partial per chunk.  The per-tensor descriptors
//                            travel as kernel arguments (192 per launch: no host staging buffer, no
//                            copy engine, nothing to keep alive after the call returns); the blocks
//                            copy them into the workspace and fill the chunk -> tensor map on the way.
//   2. lars_finalize_kernel  one block per tensor adds its partials in index order and writes
//                            lr * trust ratio: bit-identical from run to run.
//   3. lars_update_kernel    one block per chunk, chunks taken in reverse so that the tail of the
//                            norm pass, still resident in L2 / Infinity Cache, is re-read first.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kVecPerThread = 4;                            // float4 loads per thread per array
constexpr int kChunk = kThreads * kVecPerThread * 4;        // 4096 elements
constexpr int kTablePerLaunch = 192;                        // descriptors per table launch (13.5 KB of kernel arguments)

struct LarsTensor {
    float* w;
    const float* g;
    float* v;
    uint16_t* w_lowp;      // bf16 copy of the new weights or null
    long long numel;
    const double* g_sq;    // pieces of sum g^2 computed elsewhere (their sum in index order), or null: the norm pass reads g
    int chunk_start;       // first chunk of this tensor
    int n_chunks;
    float eta;             // trust coefficient of this tensor
    float weight_decay;
    int skip;              // != 0: trust ratio 1 (no layer-wise scaling)
    int g_sq_count;
};
static_assert(sizeof(LarsTensor) == 72, "descriptor layout");
static_assert(kTablePerLaunch <= kThreads, "the norm kernel probes the table with one thread per descriptor");

struct LarsGroupArgs {
    LarsTensor t[kTablePerLaunch];
    int first;             // index of t[0] in the full list
    int count;
    int chunk_begin;       // first chunk of the group
    int chunk_count;
};

struct LarsWorkspace {      // device pointers carved out of the caller's workspace
    LarsTensor* table;
    int* chunk_tensor;
    double* partial;        // [n_chunks][2]
    float* step_scale;      // [n_tensors]  lr * trust
};

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// Sum over the block in a fixed tree; every thread returns the total.
__device__ __forceinline__ double2 block_sum2(double a, double b, double* lds /* 2*4 doubles */) {
    a = wave_sum(a);
    b = wave_sum(b);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        lds[wave] = a;
        lds[4 + wave] = b;
    }
    __syncthreads();
    return make_double2((lds[0] + lds[1]) + (lds[2] + lds[3]), (lds[4] + lds[5]) + (lds[6] + lds[7]));
}

constexpr int kNormChunks = 2;                              // chunks per block of the norm pass

// A block takes kNormChunks neighbouring chunks.  It finds the tensor of each with one parallel probe of the
// descriptor table (a thread per tensor; the table sits in the kernel-argument segment), issues the loads of all its
// chunks before it adds anything up, and writes one fp64 partial pair per chunk, as if each chunk had its own block.
__global__ void __launch_bounds__(kThreads) lars_norm_kernel(const LarsGroupArgs args, LarsWorkspace ws) {
    __shared__ double red[8];
    __shared__ int owner[kNormChunks];
    if (blockIdx.x == 0 && threadIdx.x < args.count) ws.table[args.first + threadIdx.x] = args.t[threadIdx.x];
    const int c0 = (int)blockIdx.x * kNormChunks;          // first chunk of the block, relative to the group
    if (c0 >= args.chunk_count) return;                    // a group of empty tensors still gets its table written
    const int nc = args.chunk_count - c0 < kNormChunks ? args.chunk_count - c0 : kNormChunks;
    if ((int)threadIdx.x < args.count) {                   // kTablePerLaunch <= kThreads: one probe covers the table
        const int start = args.t[threadIdx.x].chunk_start, n = args.t[threadIdx.x].n_chunks;
#pragma unroll
        for (int k = 0; k < kNormChunks; ++k) {
            const int chunk = args.chunk_begin + c0 + k;
            if (k < nc && chunk >= start && chunk < start + n) owner[k] = (int)threadIdx.x;   // exactly one tensor owns a chunk
        }
    }
    __syncthreads();

    float4 a[kNormChunks][kVecPerThread], b[kNormChunks][kVecPerThread];
    const float* wp[kNormChunks];
    const float* gp[kNormChunks];
    int len[kNormChunks];
    bool full[kNormChunks], have_g[kNormChunks];
#pragma unroll
    for (int k = 0; k < kNormChunks; ++k) {
        full[k] = false;
        have_g[k] = false;
        len[k] = 0;
        wp[k] = gp[k] = nullptr;
        if (k >= nc) continue;
        const int chunk = args.chunk_begin + c0 + k;
        const int idx = owner[k];
        if (threadIdx.x == 0) ws.chunk_tensor[chunk] = args.first + idx;
        const long long off = (long long)(chunk - args.t[idx].chunk_start) * kChunk;
        const long long rem = args.t[idx].numel - off;
        len[k] = rem < kChunk ? (int)rem : kChunk;
        wp[k] = args.t[idx].w + off;
        // a tensor whose sum g^2 arrives from elsewhere: g is not read (w stands in for the address, its squares are dropped)
        have_g[k] = args.t[idx].g_sq != nullptr;
        gp[k] = have_g[k] ? wp[k] : args.t[idx].g + off;
        full[k] = len[k] == kChunk && ((((uintptr_t)wp[k]) | ((uintptr_t)gp[k])) & 15) == 0;
        if (full[k]) {
#pragma unroll
            for (int i = 0; i < kVecPerThread; ++i) {
                a[k][i] = reinterpret_cast<const float4*>(wp[k])[threadIdx.x + i * kThreads];
                if (!have_g[k]) b[k][i] = reinterpret_cast<const float4*>(gp[k])[threadIdx.x + i * kThreads];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < kNormChunks; ++k) {
        if (k >= nc) continue;
        float sw = 0.f, sg = 0.f;
        if (full[k]) {
#pragma unroll
            for (int i = 0; i < kVecPerThread; ++i) {
                sw += a[k][i].x * a[k][i].x + a[k][i].y * a[k][i].y + a[k][i].z * a[k][i].z + a[k][i].w * a[k][i].w;
                if (!have_g[k])
                    sg += b[k][i].x * b[k][i].x + b[k][i].y * b[k][i].y + b[k][i].z * b[k][i].z + b[k][i].w * b[k][i].w;
            }
        } else {
            for (int i = threadIdx.x; i < len[k]; i += kThreads) {
                const float x = wp[k][i];
                sw += x * x;
                if (!have_g[k]) {
                    const float y = gp[k][i];
                    sg += y * y;
                }
            }
        }
        const double2 s = block_sum2((double)sw, (double)sg, red);
        if (threadIdx.x == 0) {
            const int chunk = args.chunk_begin + c0 + k;
            ws.partial[2 * chunk] = s.x;
            ws.partial[2 * chunk + 1] = s.y;
        }
    }
}

__global__ void __launch_bounds__(kThreads)
lars_finalize_kernel(LarsWorkspace ws, float lr, float* __restrict__ trust_out) {
    __shared__ double red[8];
    const int l = blockIdx.x;
    const int chunk_start = ws.table[l].chunk_start, n_chunks = ws.table[l].n_chunks;
    const float eta = ws.table[l].eta, weight_decay = ws.table[l].weight_decay;
    const bool skip = ws.table[l].skip != 0;
    double pw = 0.0, pg = 0.0;
    // thread-strided, four independent running sums per thread so that the loads of a long tensor overlap; the
    // order of every addition is fixed
    const double2* __restrict__ part = reinterpret_cast<const double2*>(ws.partial) + chunk_start;
    double qw[4] = {0.0, 0.0, 0.0, 0.0}, qg[4] = {0.0, 0.0, 0.0, 0.0};
    int c = threadIdx.x;
    for (; c + 3 * kThreads < n_chunks; c += 4 * kThreads) {
        double2 p[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) p[j] = part[c + j * kThreads];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            qw[j] += p[j].x;
            qg[j] += p[j].y;
        }
    }
    for (; c < n_chunks; c += kThreads) {
        const double2 p = part[c];
        qw[0] += p.x;
        qg[0] += p.y;
    }
    pw = (qw[0] + qw[1]) + (qw[2] + qw[3]);
    pg = (qg[0] + qg[1]) + (qg[2] + qg[3]);
    const double* __restrict__ pieces = ws.table[l].g_sq;
    if (pieces) {                          // sum g^2 was computed where g was written: add its pieces the same way
        const int n_pieces = ws.table[l].g_sq_count;
        double r[4] = {0.0, 0.0, 0.0, 0.0};
        int j = threadIdx.x;
        for (; j + 3 * kThreads < n_pieces; j += 4 * kThreads) {
            double q[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) q[u] = pieces[j + u * kThreads];
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] += q[u];
        }
        for (; j < n_pieces; j += kThreads) r[0] += pieces[j];
        pg = (r[0] + r[1]) + (r[2] + r[3]);
    }
    const double2 tot = block_sum2(pw, pg, red);
    if (threadIdx.x == 0) {
        const double nw = sqrt(tot.x), ng = sqrt(tot.y);
        const double den = ng + (double)weight_decay * nw;
        const double trust = (!skip && nw > 0.0 && den > 0.0) ? (double)eta * nw / den : 1.0;
        ws.step_scale[l] = (float)((double)lr * trust);
        if (trust_out) trust_out[l] = (float)trust;
    }
}

__global__ void __launch_bounds__(kThreads)
lars_update_kernel(LarsWorkspace ws, int n_chunks, float momentum) {
    const int chunk = n_chunks - 1 - (int)blockIdx.x;
    const int l = ws.chunk_tensor[chunk];
    const LarsTensor t = ws.table[l];
    const float weight_decay = t.weight_decay;
    const float scale = ws.step_scale[l];
    const long long off = (long long)(chunk - t.chunk_start) * kChunk;
    const long long rem = t.numel - off;
    const int len = rem < kChunk ? (int)rem : kChunk;
    float* __restrict__ w = t.w + off;
    const float* __restrict__ g = t.g + off;
    float* __restrict__ v = t.v + off;
    uint16_t* __restrict__ lp = t.w_lowp ? t.w_lowp + off : nullptr;

    const bool vec = ((((uintptr_t)w) | ((uintptr_t)g) | ((uintptr_t)v)) & 15) == 0 && (((uintptr_t)lp) & 7) == 0;
    if (vec && len == kChunk) {
        float4 a[kVecPerThread], b[kVecPerThread], m[kVecPerThread];
#pragma unroll
        for (int i = 0; i < kVecPerThread; ++i) {
            a[i] = reinterpret_cast<const float4*>(w)[threadIdx.x + i * kThreads];
            b[i] = reinterpret_cast<const float4*>(g)[threadIdx.x + i * kThreads];
            m[i] = reinterpret_cast<const float4*>(v)[threadIdx.x + i * kThreads];
        }
#pragma unroll
        for (int i = 0; i < kVecPerThread; ++i) {
            float4 nv, nw;
            nv.x = fmaf(momentum, m[i].x, scale * fmaf(weight_decay, a[i].x, b[i].x));
            nv.y = fmaf(momentum, m[i].y, scale * fmaf(weight_decay, a[i].y, b[i].y));
            nv.z = fmaf(momentum, m[i].z, scale * fmaf(weight_decay, a[i].z, b[i].z));
            nv.w = fmaf(momentum, m[i].w, scale * fmaf(weight_decay, a[i].w, b[i].w));
            nw.x = a[i].x - nv.x;
            nw.y = a[i].y - nv.y;
            nw.z = a[i].z - nv.z;
            nw.w = a[i].w - nv.w;
            reinterpret_cast<float4*>(v)[threadIdx.x + i * kThreads] = nv;
            reinterpret_cast<float4*>(w)[threadIdx.x + i * kThreads] = nw;
            if (lp) {
                ushort4 h;
                h.x = lc_bf16_rne(nw.x);
                h.y = lc_bf16_rne(nw.y);
                h.z = lc_bf16_rne(nw.z);
                h.w = lc_bf16_rne(nw.w);
                reinterpret_cast<ushort4*>(lp)[threadIdx.x + i * kThreads] = h;
            }
        }
    } else {
        for (int i = threadIdx.x; i < len; i += kThreads) {
            const float x = w[i];
            const float nv = fmaf(momentum, v[i], scale * fmaf(weight_decay, x, g[i]));
            const float nw = x - nv;
            v[i] = nv;
            w[i] = nw;
            if (lp) lp[i] = lc_bf16_rne(nw);
        }
    }
}

// Workspace carving shared by the size query and the call.
struct LarsLayout {
    size_t table, chunk_tensor, partial, step_scale, total;
    long long n_chunks;
};

bool lars_layout(int n_tensors, const int64_t* numel, LarsLayout* out) {
    long long chunks = 0;
    for (int l = 0; l < n_tensors; ++l) {
        if (numel[l] < 0) return false;
        chunks += (numel[l] + kChunk - 1) / kChunk;
    }
    if (chunks > 0x7fffffffLL) return false;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += (bytes + 255) & ~(size_t)255;
        return at;
    };
    out->table = take(sizeof(LarsTensor) * (size_t)n_tensors);
    out->chunk_tensor = take(sizeof(int) * (size_t)chunks);
    out->partial = take(sizeof(double) * 2 * (size_t)chunks);
    out->step_scale = take(sizeof(float) * (size_t)n_tensors);
    out->total = off;
    out->n_chunks = chunks;
    return true;
}

}  // namespace

extern "C" size_t lars_workspace_bytes(int n_tensors, const int64_t* numel) {
    LarsLayout lay;
    if (n_tensors <= 0 || !numel || !lars_layout(n_tensors, numel, &lay)) return 0;
    return lay.total;
}

namespace {

// Argument checks shared by the entry points (everything but the workspace), then the layout of the scratch memory.
lc_status lars_check(int n_tensors, float* const* w, const float* const* g, float* const* v, const int64_t* numel,
                     void* const* w_lowp_out, LarsLayout* lay) {
    if (n_tensors < 0) return LC_ERR_SHAPE;
    if (!w || !g || !v || !numel) return LC_ERR_NULL;
    if (!lars_layout(n_tensors, numel, lay)) return LC_ERR_SHAPE;
    for (int l = 0; l < n_tensors; ++l) {
        if (numel[l] == 0) continue;
        if (!w[l] || !g[l] || !v[l]) return LC_ERR_NULL;
        if ((((uintptr_t)w[l]) | ((uintptr_t)g[l]) | ((uintptr_t)v[l])) & 3) return LC_ERR_ALIGN;
        if (w_lowp_out && (((uintptr_t)w_lowp_out[l]) & 1)) return LC_ERR_ALIGN;
    }
    return LC_OK;
}

// The launches of one step on scratch memory at `base` (device, 256-byte aligned, lay.total bytes).
lc_status lars_run(int n_tensors, float* const* w, const float* const* g, float* const* v, const int64_t* numel, float eta,
                   float momentum, float weight_decay, float lr, const float* eta_per_tensor,
                   const float* weight_decay_per_tensor, const uint8_t* skip, const double* const* g_sq_pieces,
                   const int64_t* g_sq_counts, float* trust_out, void* const* w_lowp_out, const LarsLayout& lay, char* base,
                   hipStream_t stream) {
    LarsWorkspace ws;
    ws.table = reinterpret_cast<LarsTensor*>(base + lay.table);
    ws.chunk_tensor = reinterpret_cast<int*>(base + lay.chunk_tensor);
    ws.partial = reinterpret_cast<double*>(base + lay.partial);
    ws.step_scale = reinterpret_cast<float*>(base + lay.step_scale);
    lc_begin_call();

    LarsGroupArgs args;
    int chunk_cursor = 0;
    for (int first = 0; first < n_tensors; first += kTablePerLaunch) {
        const int count = (n_tensors - first) < kTablePerLaunch ? (n_tensors - first) : kTablePerLaunch;
        args.chunk_begin = chunk_cursor;
        for (int i = 0; i < count; ++i) {
            const int l = first + i;
            LarsTensor& t = args.t[i];
            t.w = w[l];
            t.g = g[l];
            t.v = v[l];
            t.w_lowp = w_lowp_out ? static_cast<uint16_t*>(w_lowp_out[l]) : nullptr;
            t.numel = numel[l];
            t.eta = eta_per_tensor ? eta_per_tensor[l] : eta;
            t.weight_decay = weight_decay_per_tensor ? weight_decay_per_tensor[l] : weight_decay;
            t.skip = skip ? (int)skip[l] : 0;
            const bool pre = g_sq_pieces && g_sq_counts && g_sq_pieces[l] && g_sq_counts[l] > 0;
            t.g_sq = pre ? g_sq_pieces[l] : nullptr;
            t.g_sq_count = pre ? (int)g_sq_counts[l] : 0;
            t.chunk_start = chunk_cursor;
            t.n_chunks = (int)((numel[l] + kChunk - 1) / kChunk);
            chunk_cursor += t.n_chunks;
        }
        args.first = first;
        args.count = count;
        args.chunk_count = chunk_cursor - args.chunk_begin;
        const int grid = args.chunk_count > 0 ? (args.chunk_count + kNormChunks - 1) / kNormChunks : 1;
        hipLaunchKernelGGL(lars_norm_kernel, dim3(grid), dim3(kThreads), 0, stream, args, ws);
    }
    hipLaunchKernelGGL(lars_finalize_kernel, dim3(n_tensors), dim3(kThreads), 0, stream, ws, lr, trust_out);
    if (lay.n_chunks > 0)
        hipLaunchKernelGGL(lars_update_kernel, dim3((unsigned)lay.n_chunks), dim3(kThreads), 0, stream, ws, (int)lay.n_chunks,
                           momentum);
    return lc_end_call();
}

}  // namespace

extern "C" lc_status lars_step_ex(int n_tensors, float* const* w, const float* const* g, float* const* v,
                                  const int64_t* numel, float eta, float momentum, float weight_decay, float lr,
                                  const float* eta_per_tensor, const float* weight_decay_per_tensor, const uint8_t* skip,
                                  float* trust_out, void* const* w_lowp_out,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (n_tensors == 0) return LC_OK;
    LarsLayout lay;
    const lc_status st = lars_check(n_tensors, w, g, v, numel, w_lowp_out, &lay);
    if (st != LC_OK) return st;
    if (!workspace || (((uintptr_t)workspace) & 255) || workspace_bytes < lay.total) return LC_ERR_WORKSPACE;
    return lars_run(n_tensors, w, g, v, numel, eta, momentum, weight_decay, lr, eta_per_tensor, weight_decay_per_tensor, skip,
                    nullptr, nullptr, trust_out, w_lowp_out, lay, static_cast<char*>(workspace), static_cast<hipStream_t>(hip_stream));
}

extern "C" lc_status lars_step_pre(int n_tensors, float* const* w, const float* const* g, float* const* v,
                                   const int64_t* numel, float eta, float momentum, float weight_decay, float lr,
                                   const float* eta_per_tensor, const float* weight_decay_per_tensor, const uint8_t* skip,
                                   const double* const* g_sq_pieces, const int64_t* g_sq_counts,
                                   float* trust_out, void* const* w_lowp_out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (n_tensors == 0) return LC_OK;
    LarsLayout lay;
    const lc_status st = lars_check(n_tensors, w, g, v, numel, w_lowp_out, &lay);
    if (st != LC_OK) return st;
    if ((g_sq_pieces == nullptr) != (g_sq_counts == nullptr)) return LC_ERR_NULL;
    if (g_sq_pieces)
        for (int l = 0; l < n_tensors; ++l) {
            if (g_sq_counts[l] < 0 || g_sq_counts[l] > 0x7fffffffLL) return LC_ERR_SHAPE;
            if (g_sq_pieces[l] && (((uintptr_t)g_sq_pieces[l]) & 7)) return LC_ERR_ALIGN;
        }
    if (!workspace || (((uintptr_t)workspace) & 255) || workspace_bytes < lay.total) return LC_ERR_WORKSPACE;
    return lars_run(n_tensors, w, g, v, numel, eta, momentum, weight_decay, lr, eta_per_tensor, weight_decay_per_tensor, skip,
                    g_sq_pieces, g_sq_counts, trust_out, w_lowp_out, lay, static_cast<char*>(workspace),
                    static_cast<hipStream_t>(hip_stream));
}

// ---- the same step on scratch memory that the library holds itself, for callers that cannot allocate ----
// A fixed array in device memory; every GPU the library runs on holds its own copy at its own address until the
// process ends.  Host code never uses the array's name as an address: the address on the current device is asked
// for once per device and kept.
constexpr size_t kStaticScratchBytes = LARS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each device, null until asked for

lc_status scratch_of_current_device(char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return lc_fail_call(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return LC_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return lc_fail_call(e, "hipGetSymbolAddress");
        if (!p || (((uintptr_t)p) & 255)) return lc_fail_call(hipErrorInvalidSymbol, "hipGetSymbolAddress (null or misaligned)");
        g_scratch_ptr[dev] = static_cast<char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return LC_OK;
}

}  // namespace

extern "C" lc_status lars_step_ex_static(int n_tensors, float* const* w, const float* const* g, float* const* v,
                                         const int64_t* numel, float eta, float momentum, float weight_decay, float lr,
                                         const float* eta_per_tensor, const float* weight_decay_per_tensor,
                                         const uint8_t* skip, float* trust_out, void* const* w_lowp_out, void* hip_stream) {
    if (n_tensors == 0) return LC_OK;
    LarsLayout lay;
    const lc_status st = lars_check(n_tensors, w, g, v, numel, w_lowp_out, &lay);
    if (st != LC_OK) return st;
    if (lay.total > kStaticScratchBytes) return LC_ERR_WORKSPACE;     // the list needs more than the fixed array holds
    char* base = nullptr;
    const lc_status sp = scratch_of_current_device(&base);
    if (sp != LC_OK) return sp;
    // Nothing in the array has to start at zero: the norm pass writes the table, the chunk map and every partial
    // sum of this list before the later kernels read them, and the finalize kernel writes every step scale.
    return lars_run(n_tensors, w, g, v, numel, eta, momentum, weight_decay, lr, eta_per_tensor, weight_decay_per_tensor, skip,
                    nullptr, nullptr, trust_out, w_lowp_out, lay, base, static_cast<hipStream_t>(hip_stream));
}

extern "C" lc_status lars_step(int n_tensors, float* const* w, const float* const* g, float* const* v,
                               const int64_t* numel, float eta, float momentum, float weight_decay, float lr,
                               float* trust_out, void* const* w_lowp_out,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    return lars_step_ex(n_tensors, w, g, v, numel, eta, momentum, weight_decay, lr, nullptr, nullptr, nullptr, trust_out,
                        w_lowp_out, workspace, workspace_bytes, hip_stream);
}

extern "C" float lars_warmup_poly_lr(float base_lr, float start_lr, int64_t iter, int64_t warmup_iters, int64_t max_iter,
                                     float power) {
    if (warmup_iters > 0 && iter < warmup_iters)
        return (float)((double)start_lr + ((double)base_lr - (double)start_lr) * (double)iter / (double)warmup_iters);
    const int64_t w = warmup_iters > 0 ? warmup_iters : 0;
    if (max_iter <= w) return base_lr;
    double frac = 1.0 - (double)(iter - w) / (double)(max_iter - w);
    if (frac < 0.0) frac = 0.0;
    return (float)((double)base_lr * pow(frac, (double)power));
}

extern "C" float lars_poly_lr(float base_lr, int64_t iter, int64_t max_iter, float power) {
    if (max_iter <= 0) return base_lr;
    double frac = 1.0 - (double)iter / (double)max_iter;
    if (frac < 0.0) frac = 0.0;
    return (float)((double)base_lr * pow(frac, (double)power));
}
