// Latent change reduction (Section 3.2 HLC, Eq. (5)): sum|cur - prev| and sum|prev| in one
// pass over both tensors, deterministic result.
//
// HBM-bound (8 bytes read per element, 12 bytes written in total).  The grid is at most one
// block of 1024 threads per CU; a lane has four 16 B loads per tensor in flight (128 KiB per
// CU), sums four terms in binary32 and carries the running sums in binary64.  Wavefronts
// combine with DPP moves (no LDS round trips) and every block leaves one partial pair.  A
// second, single-block launch adds the partial pairs in index order, so the bits do not depend
// on scheduling.  Single-launch forms were measured and are not faster: the block that arrives
// last has to see the others' partial sums, and on this chip (one L2 per XCD) that costs either
// a release fence per block, which writes the L2 back (35 us for 1024 blocks), or stores and
// arrival counters that go to memory and are waited for one after the other (2.3 us, what the
// second launch costs).
#include <atomic>

#include "qc_internal.h"

namespace qc {
namespace {

constexpr int kThreads = 256;       // combine kernels, variation pass
constexpr int kWideThreads = 1024;  // streaming passes: 16 wavefronts per CU
constexpr int kMaxBlocks = 256;     // one block per CU
constexpr int kUnroll = 4;          // float4 loads in flight per tensor per lane

// one DPP move of a binary64 value (two 32-bit halves); CTRL as in the ISA's dpp_ctrl field
template <int CTRL>
__device__ inline double dpp_move(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes, the same bits in every lane: butterflies inside a row of 16 lanes
// (quad_perm [1,0,3,2], [2,3,0,1], row_half_mirror, row_mirror), then the four row sums in
// index order.
__device__ inline double wave_sum(double v) {
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    double r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        r[i] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 16 * i),
                                __builtin_amdgcn_readlane(__double2loint(v), 16 * i));
    return (r[0] + r[1]) + (r[2] + r[3]);
}

// A reduction reads its tensors once, so it loads them non-temporally: measured against ordinary
// loads this is 6 % faster on the 33.5 MB latent pair (cold 9.7 -> 9.1 us) and 10-13 % faster from
// 0.5 GB on (2.1 GB: 5.8 -> 6.6 TB/s), provided every load instruction of a wavefront covers whole
// lines (a lane stride of 16 B); the exception is the frame gradient, whose second read of every
// element is meant to hit in the caches.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline float4 stream4f(const float4 *p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ inline uint4 stream4u(const void *p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ inline float abs4(const float4 &a, const float4 &b) {
    return (fabsf(a.x - b.x) + fabsf(a.y - b.y)) + (fabsf(a.z - b.z) + fabsf(a.w - b.w));
}
__device__ inline float abs4(const float4 &b) {
    return (fabsf(b.x) + fabsf(b.y)) + (fabsf(b.z) + fabsf(b.w));
}

// block-wide sums of COUNT values in wavefront order; result valid in thread 0.
// sh holds COUNT * (THREADS / 64) doubles and may be reused after the call.
template <int THREADS, int COUNT>
__device__ inline void block_sum(double (&v)[COUNT], double *sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int c = 0; c < COUNT; ++c) {
        v[c] = wave_sum(v[c]);
        if (lane == 0) sh[COUNT * wave + c] = v[c];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int c = 0; c < COUNT; ++c) {
            double t = sh[c];
            for (int w = 1; w < THREADS / 64; ++w) t += sh[COUNT * w + c];
            v[c] = t;
        }
    }
    __syncthreads();
}

// A block takes contiguous chunks of kWideThreads * kUnroll float4 (64 KiB per tensor) and
// strides over the tensor by the grid; all of a chunk's loads are issued before the first use.
__global__ __launch_bounds__(kWideThreads) void latent_delta_partial_kernel(
    const float *__restrict__ cur, const float *__restrict__ prev, int64_t n,
    double *__restrict__ partials) {
    __shared__ double sh[2 * (kWideThreads / 64)];
    const int64_t n4 = n / 4;
    const float4 *c4 = reinterpret_cast<const float4 *>(cur);
    const float4 *p4 = reinterpret_cast<const float4 *>(prev);
    constexpr int64_t kChunk = (int64_t)kWideThreads * kUnroll;
    double s[2] = {0.0, 0.0};
    for (int64_t base = (int64_t)blockIdx.x * kChunk; base < n4; base += (int64_t)gridDim.x * kChunk) {
        float4 a[kUnroll], b[kUnroll];
        bool ok[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t i = base + u * kWideThreads + threadIdx.x;
            ok[u] = i < n4;
            const int64_t j = ok[u] ? i : 0;   // a valid index either way
            a[u] = stream4f(c4 + j);
            b[u] = stream4f(p4 + j);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            if (ok[u]) { s[0] += (double)abs4(a[u], b[u]); s[1] += (double)abs4(b[u]); }
    }
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - n4 * 4)) {  // up to 3 trailing elements
        const int64_t j = n4 * 4 + threadIdx.x;
        s[0] += (double)fabsf(cur[j] - prev[j]);
        s[1] += (double)fabsf(prev[j]);
    }
    block_sum<kWideThreads, 2>(s, sh);
    if (threadIdx.x == 0) {
        partials[2 * blockIdx.x] = s[0];
        partials[2 * blockIdx.x + 1] = s[1];
    }
}

// one block: fixed-order combine of the partial pairs, then the ratio
__global__ __launch_bounds__(kThreads) void latent_delta_final_kernel(
    const double *__restrict__ partials, int count, float *__restrict__ out3) {
    __shared__ double sh[2 * (kThreads / 64)];
    double s[2] = {0.0, 0.0};
    for (int b = threadIdx.x; b < count; b += kThreads) {
        s[0] += partials[2 * b];
        s[1] += partials[2 * b + 1];
    }
    block_sum<kThreads, 2>(s, sh);
    if (threadIdx.x == 0) {
        const double num = s[0], den = s[1];
        float rel;
        if (den > 0.0) rel = (float)(num / den);
        else rel = num > 0.0 ? __builtin_inff() : 0.0f;
        out3[0] = (float)num;
        out3[1] = (float)den;
        out3[2] = rel;
    }
}

// ---- cosine similarity of two feature tensors (Section 3.3 SRAP, Eq. (9)) -------------------
// Same scheme with three running sums: <a, b>, <a, a>, <b, b>.

// One 16 B load of a float or bf16 tensor (4 or 8 consecutive elements), widened to float.
template <typename T>
struct Pack;
template <>
struct Pack<float> {
    static constexpr int kElems = 4;
    float4 v;
    __device__ void stream(const float *p) { v = stream4f(reinterpret_cast<const float4 *>(p)); }
    __device__ float get(int i) const {
        switch (i) { case 0: return v.x; case 1: return v.y; case 2: return v.z; default: return v.w; }
    }
};
template <>
struct Pack<uint16_t> {  // bf16 bit patterns
    static constexpr int kElems = 8;
    uint4 v;
    __device__ void stream(const uint16_t *p) { v = stream4u(p); }
    __device__ float get(int i) const {
        uint32_t w;
        switch (i >> 1) { case 0: w = v.x; break; case 1: w = v.y; break; case 2: w = v.z; break; default: w = v.w; }
        return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
    }
};

// A block takes contiguous chunks of kWideThreads * kUnroll packs per tensor; consecutive lanes
// take consecutive packs.  Every four consecutive elements are summed in binary32, the sums
// carried in binary64.
template <typename T>
__global__ __launch_bounds__(kWideThreads) void similarity_partial_kernel(
    const T *__restrict__ a, const T *__restrict__ b, int64_t n, double *__restrict__ partials) {
    __shared__ double sh[3 * (kWideThreads / 64)];
    constexpr int E = Pack<T>::kElems;
    const int64_t packs = n / E;
    constexpr int64_t kChunk = (int64_t)kWideThreads * kUnroll;
    double s[3] = {0.0, 0.0, 0.0};  // <a,b>, <a,a>, <b,b>
    for (int64_t base = (int64_t)blockIdx.x * kChunk; base < packs; base += (int64_t)gridDim.x * kChunk) {
        Pack<T> x[kUnroll], y[kUnroll];
        bool ok[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t i = base + u * kWideThreads + threadIdx.x;
            ok[u] = i < packs;
            const int64_t j = ok[u] ? i : 0;   // a valid index either way
            x[u].stream(a + E * j);
            y[u].stream(b + E * j);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (!ok[u]) continue;
#pragma unroll
            for (int g = 0; g < E / 4; ++g) {
                float pab = 0.f, paa = 0.f, pbb = 0.f;
#pragma unroll
                for (int e = 4 * g; e < 4 * g + 4; ++e) {
                    const float xv = x[u].get(e), yv = y[u].get(e);
                    pab += xv * yv;
                    paa += xv * xv;
                    pbb += yv * yv;
                }
                s[0] += (double)pab;
                s[1] += (double)paa;
                s[2] += (double)pbb;
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - packs * E)) {  // up to E - 1 trailing elements
        const int64_t j = packs * E + threadIdx.x;
        float xv, yv;
        if constexpr (sizeof(T) == 2) {
            xv = __uint_as_float((uint32_t)a[j] << 16);
            yv = __uint_as_float((uint32_t)b[j] << 16);
        } else {
            xv = a[j];
            yv = b[j];
        }
        s[0] += (double)(xv * yv);
        s[1] += (double)(xv * xv);
        s[2] += (double)(yv * yv);
    }
    block_sum<kWideThreads, 3>(s, sh);
    if (threadIdx.x == 0) {
        partials[3 * blockIdx.x] = s[0];
        partials[3 * blockIdx.x + 1] = s[1];
        partials[3 * blockIdx.x + 2] = s[2];
    }
}

__global__ __launch_bounds__(kThreads) void similarity_final_kernel(
    const double *__restrict__ partials, int count, float *__restrict__ out4) {
    __shared__ double sh[3 * (kThreads / 64)];
    double s[3] = {0.0, 0.0, 0.0};
    for (int b = threadIdx.x; b < count; b += kThreads) {
        s[0] += partials[3 * b]; s[1] += partials[3 * b + 1]; s[2] += partials[3 * b + 2];
    }
    block_sum<kThreads, 3>(s, sh);
    if (threadIdx.x == 0) {
        const double denom = sqrt(s[1]) * sqrt(s[2]);
        out4[0] = (float)s[0];
        out4[1] = (float)s[1];
        out4[2] = (float)s[2];
        out4[3] = denom > 0.0 ? (float)(s[0] / denom) : 0.0f;
    }
}

// ---- inter-frame gradient norm (Section 3.2 HLC, second factor of Eq. (5)) -----------------
// The feature map is [frames, inner]; the gradient is the forward difference along the frame
// axis and the norm is Euclidean.  As a reduction it is a pass over the pair (m, m + inner):
// every element is read twice, the second time one frame (inner elements) later, which the
// caches absorb for the frame sizes of a latent.

// 8 consecutive elements of a float or bf16 tensor, widened to float
template <typename T>
struct Oct;
template <>
struct Oct<float> {
    float4 lo, hi;
    __device__ void load(const float *p) {
        lo = reinterpret_cast<const float4 *>(p)[0];
        hi = reinterpret_cast<const float4 *>(p)[1];
    }
    __device__ float get(int i) const {
        const float4 &f = i < 4 ? lo : hi;
        switch (i & 3) { case 0: return f.x; case 1: return f.y; case 2: return f.z; default: return f.w; }
    }
};
template <>
struct Oct<uint16_t> {  // bf16 bit patterns
    uint4 v;
    __device__ void load(const uint16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ float get(int i) const {
        uint32_t w;
        switch (i >> 1) { case 0: w = v.x; break; case 1: w = v.y; break; case 2: w = v.z; break; default: w = v.w; }
        return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
    }
};

__device__ inline float widen(float v) { return v; }
__device__ inline float widen(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// VEC: inner is a multiple of 8, so both streams can be read 8 elements at a time.
template <typename T, bool VEC>
__global__ __launch_bounds__(kWideThreads) void gradient_partial_kernel(
    const T *__restrict__ m, int64_t inner, int64_t n, double *__restrict__ partials) {
    __shared__ double sh[kWideThreads / 64];
    const T *lo = m, *hi = m + inner;
    double s[1] = {0.0};
    int64_t done = 0;
    if constexpr (VEC) {
        const int64_t n8 = n / 8;
        constexpr int64_t kChunk = (int64_t)kWideThreads * 2;
        for (int64_t base = (int64_t)blockIdx.x * kChunk; base < n8; base += (int64_t)gridDim.x * kChunk) {
            Oct<T> x[2], y[2];
            const int64_t i0 = base + threadIdx.x, i1 = i0 + kWideThreads;
            const bool ok[2] = {i0 < n8, i1 < n8};
            x[0].load(lo + 8 * (ok[0] ? i0 : 0));
            y[0].load(hi + 8 * (ok[0] ? i0 : 0));
            x[1].load(lo + 8 * (ok[1] ? i1 : 0));
            y[1].load(hi + 8 * (ok[1] ? i1 : 0));
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (!ok[u]) continue;
                float p[2] = {0.f, 0.f};
#pragma unroll
                for (int e = 0; e < 8; ++e) {  // two 4-term binary32 sums
                    const float d = y[u].get(e) - x[u].get(e);
                    p[e >> 2] += d * d;
                }
                s[0] += (double)p[0] + (double)p[1];
            }
        }
        done = n8 * 8;
    }
    const int64_t stride = (int64_t)gridDim.x * kWideThreads;
    for (int64_t j = done + (int64_t)blockIdx.x * kWideThreads + threadIdx.x; j < n; j += stride) {
        const float d = widen(hi[j]) - widen(lo[j]);
        s[0] += (double)(d * d);
    }
    block_sum<kWideThreads, 1>(s, sh);
    if (threadIdx.x == 0) partials[blockIdx.x] = s[0];
}

__global__ __launch_bounds__(kThreads) void gradient_final_kernel(
    const double *__restrict__ partials, int count, float *__restrict__ out2) {
    __shared__ double sh[kThreads / 64];
    double s[1] = {0.0};
    for (int b = threadIdx.x; b < count; b += kThreads) s[0] += partials[b];
    block_sum<kThreads, 1>(s, sh);
    if (threadIdx.x == 0) {
        out2[0] = (float)s[0];
        out2[1] = (float)sqrt(s[0]);
    }
}

// ---- cumulative variation over the previous steps (Section 3.3 SRAP, Eq. (11)) --------------
// L1 distance of the current tensor to each of COUNT earlier ones in one pass: the current
// tensor is read once, not once per distance.

struct PrevList { const float *p[QC_MAX_PREV]; };
constexpr int kVarThreads = 512;   // two wavefronts per SIMD: room for 2 (COUNT + 1) float4 per lane

template <int COUNT>
__global__ __launch_bounds__(kVarThreads) void variation_partial_kernel(
    const float *__restrict__ cur, PrevList prevs, int64_t n, double *__restrict__ partials) {
    __shared__ double sh[COUNT * (kVarThreads / 64)];
    const int64_t n4 = n / 4;
    const float4 *c4 = reinterpret_cast<const float4 *>(cur);
    constexpr int64_t kChunk = (int64_t)kVarThreads * 2;
    double d[COUNT];
#pragma unroll
    for (int c = 0; c < COUNT; ++c) d[c] = 0.0;
    for (int64_t base = (int64_t)blockIdx.x * kChunk; base < n4; base += (int64_t)gridDim.x * kChunk) {
        const int64_t i = base + threadIdx.x;
        const bool first = i < n4, second = i + kVarThreads < n4;
        const int64_t i0 = first ? i : 0, i1 = second ? i + kVarThreads : 0;  // valid either way
        const float4 a0 = stream4f(c4 + i0), a1 = stream4f(c4 + i1);
        float4 b0[COUNT], b1[COUNT];
#pragma unroll
        for (int c = 0; c < COUNT; ++c) {
            const float4 *p4 = reinterpret_cast<const float4 *>(prevs.p[c]);
            b0[c] = stream4f(p4 + i0);
            b1[c] = stream4f(p4 + i1);
        }
#pragma unroll
        for (int c = 0; c < COUNT; ++c) {
            if (first) d[c] += (double)abs4(a0, b0[c]);
            if (second) d[c] += (double)abs4(a1, b1[c]);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - n4 * 4)) {  // up to 3 trailing elements
        const int64_t j = n4 * 4 + threadIdx.x;
#pragma unroll
        for (int c = 0; c < COUNT; ++c) d[c] += (double)fabsf(cur[j] - prevs.p[c][j]);
    }
    block_sum<kVarThreads, COUNT>(d, sh);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int c = 0; c < COUNT; ++c) partials[(int64_t)blockIdx.x * QC_MAX_PREV + c] = d[c];
    }
}

__global__ __launch_bounds__(kThreads) void variation_final_kernel(
    const double *__restrict__ partials, int blocks, int count, float *__restrict__ out) {
    __shared__ double sh[kThreads / 64];
    double total = 0.0;
    for (int c = 0; c < count; ++c) {
        double v[1] = {0.0};
        for (int b = threadIdx.x; b < blocks; b += kThreads) v[0] += partials[(int64_t)b * QC_MAX_PREV + c];
        block_sum<kThreads, 1>(v, sh);
        if (threadIdx.x == 0) {
            out[c] = (float)v[0];
            total += v[0];
        }
    }
    if (threadIdx.x == 0) out[count] = (float)total;
}

template <int COUNT>
void launch_variation(const float *cur, const PrevList &prevs, int64_t n, double *partials,
                      unsigned blocks, hipStream_t stream) {
    variation_partial_kernel<COUNT><<<dim3(blocks), dim3(kVarThreads), 0, stream>>>(cur, prevs, n, partials);
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace
}  // namespace qc

using namespace qc;

extern "C" size_t qc_latent_delta_workspace_bytes(int64_t n) {
    if (n < 1) return 0;
    return (size_t)kMaxBlocks * 2 * sizeof(double);
}

extern "C" qc_status qc_latent_delta(const float *cur, const float *prev, int64_t n, float *out3,
                                     void *workspace, size_t workspace_bytes, void *stream) {
    if (!cur || !prev || !out3 || !workspace || n < 1) return QC_ERR_INVALID_ARG;
    if (!aligned(cur, 16) || !aligned(prev, 16) || !aligned(out3, 4) || !aligned(workspace, 256))
        return QC_ERR_INVALID_ARG;
    if (workspace_bytes < qc_latent_delta_workspace_bytes(n)) return QC_ERR_WORKSPACE;
    // one chunk of kWideThreads * kUnroll float4 per block and pass; at most one block per CU
    int64_t blocks = (n / 4 + (int64_t)kWideThreads * kUnroll - 1) / ((int64_t)kWideThreads * kUnroll);
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    double *partials = (double *)workspace;
    latent_delta_partial_kernel<<<dim3((unsigned)blocks), dim3(kWideThreads), 0, (hipStream_t)stream>>>(
        cur, prev, n, partials);
    if (hipGetLastError() != hipSuccess) return QC_ERR_DEVICE;
    latent_delta_final_kernel<<<dim3(1), dim3(kThreads), 0, (hipStream_t)stream>>>(
        partials, (int)blocks, out3);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

// ---- qc_latent_delta for callers that cannot allocate ---------------------------------------
// The per-block partial sums live in a file-scope device array instead of a caller's workspace.
// `scratch` below is the host-side handle of that array, not a device address: host code asks
// the runtime once per device for the address of that device's copy and uses only that.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)kMaxBlocks * 2 * sizeof(double);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// device address of the current device's copy of `scratch`, resolved on first use
qc_status static_scratch(void **out) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0) return QC_ERR_DEVICE;
    if (device >= kMaxDevices) return QC_ERR_UNSUPPORTED;
    void *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QC_ERR_DEVICE;
        g_scratch_ptr[device].store(p, std::memory_order_release);  // racing threads store the same value
    }
    *out = p;
    return QC_OK;
}
}  // namespace

extern "C" qc_status qc_latent_delta_static(const float *cur, const float *prev, int64_t n,
                                            float *out3, void *stream) {
    if (!cur || !prev || !out3 || n < 1) return QC_ERR_INVALID_ARG;
    if (n > QC_LATENT_DELTA_STATIC_MAX_N) return QC_ERR_UNSUPPORTED;
    void *ws = nullptr;
    if (qc_status st = static_scratch(&ws); st != QC_OK) return st;
    // every partial pair the second launch reads is written by the first: nothing to clear
    return qc_latent_delta(cur, prev, n, out3, ws, kStaticScratchBytes, stream);
}

extern "C" size_t qc_layer_similarity_workspace_bytes(int64_t n) {
    if (n < 1) return 0;
    return (size_t)kMaxBlocks * 3 * sizeof(double);
}

extern "C" qc_status qc_layer_similarity(const void *a, const void *b, qc_dtype dt, int64_t n,
                                         float *out4, void *workspace, size_t workspace_bytes,
                                         void *stream) {
    if (!a || !b || !out4 || !workspace || n < 1) return QC_ERR_INVALID_ARG;
    if (dt != QC_F32 && dt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (!aligned(a, 16) || !aligned(b, 16) || !aligned(out4, 4) || !aligned(workspace, 256))
        return QC_ERR_INVALID_ARG;
    if (workspace_bytes < qc_layer_similarity_workspace_bytes(n)) return QC_ERR_WORKSPACE;
    const int64_t packs = n / (dt == QC_BF16 ? 8 : 4);
    int64_t blocks = (packs + (int64_t)kWideThreads * kUnroll - 1) / ((int64_t)kWideThreads * kUnroll);
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    double *partials = (double *)workspace;
    const dim3 grid((unsigned)blocks), block(kWideThreads);
    hipStream_t st = (hipStream_t)stream;
    if (dt == QC_BF16)
        similarity_partial_kernel<uint16_t><<<grid, block, 0, st>>>((const uint16_t *)a, (const uint16_t *)b, n, partials);
    else
        similarity_partial_kernel<float><<<grid, block, 0, st>>>((const float *)a, (const float *)b, n, partials);
    if (hipGetLastError() != hipSuccess) return QC_ERR_DEVICE;
    similarity_final_kernel<<<dim3(1), dim3(kThreads), 0, (hipStream_t)stream>>>(partials, (int)blocks, out4);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" size_t qc_frame_gradient_norm_workspace_bytes(int64_t frames, int64_t inner) {
    if (frames < 1 || inner < 1) return 0;
    return (size_t)kMaxBlocks * sizeof(double);
}

extern "C" qc_status qc_frame_gradient_norm(const void *m, qc_dtype dt, int64_t frames,
                                            int64_t inner, float *out2, void *workspace,
                                            size_t workspace_bytes, void *stream) {
    if (!m || !out2 || !workspace || frames < 1 || inner < 1) return QC_ERR_INVALID_ARG;
    if (dt != QC_F32 && dt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (!aligned(m, 16) || !aligned(out2, 4) || !aligned(workspace, 256)) return QC_ERR_INVALID_ARG;
    if (frames > INT64_MAX / inner) return QC_ERR_INVALID_ARG;
    if (workspace_bytes < qc_frame_gradient_norm_workspace_bytes(frames, inner)) return QC_ERR_WORKSPACE;
    const int64_t n = (frames - 1) * inner;  // number of differences
    const bool vec = inner % 8 == 0;
    const int64_t per_block = (int64_t)kWideThreads * (vec ? 16 : 4);
    int64_t blocks = (n + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    double *partials = (double *)workspace;
    const dim3 grid((unsigned)blocks), block(kWideThreads);
    hipStream_t st = (hipStream_t)stream;
    if (dt == QC_BF16) {
        if (vec) gradient_partial_kernel<uint16_t, true><<<grid, block, 0, st>>>((const uint16_t *)m, inner, n, partials);
        else gradient_partial_kernel<uint16_t, false><<<grid, block, 0, st>>>((const uint16_t *)m, inner, n, partials);
    } else {
        if (vec) gradient_partial_kernel<float, true><<<grid, block, 0, st>>>((const float *)m, inner, n, partials);
        else gradient_partial_kernel<float, false><<<grid, block, 0, st>>>((const float *)m, inner, n, partials);
    }
    if (hipGetLastError() != hipSuccess) return QC_ERR_DEVICE;
    gradient_final_kernel<<<dim3(1), dim3(kThreads), 0, st>>>(partials, (int)blocks, out2);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" size_t qc_cumulative_variation_workspace_bytes(int64_t n, int count) {
    if (n < 1 || count < 1 || count > QC_MAX_PREV) return 0;
    return (size_t)kMaxBlocks * QC_MAX_PREV * sizeof(double);
}

extern "C" qc_status qc_cumulative_variation(const float *cur, const float *const *prevs, int count,
                                             int64_t n, float *out, void *workspace,
                                             size_t workspace_bytes, void *stream) {
    if (!cur || !prevs || !out || !workspace || n < 1 || count < 1) return QC_ERR_INVALID_ARG;
    if (count > QC_MAX_PREV) return QC_ERR_UNSUPPORTED;
    if (!aligned(cur, 16) || !aligned(out, 4) || !aligned(workspace, 256)) return QC_ERR_INVALID_ARG;
    PrevList list;
    for (int c = 0; c < QC_MAX_PREV; ++c) {
        list.p[c] = c < count ? prevs[c] : nullptr;
        if (c < count && (!prevs[c] || !aligned(prevs[c], 16))) return QC_ERR_INVALID_ARG;
    }
    if (workspace_bytes < qc_cumulative_variation_workspace_bytes(n, count)) return QC_ERR_WORKSPACE;
    int64_t blocks = (n / 4 + (int64_t)kVarThreads * 2 - 1) / ((int64_t)kVarThreads * 2);
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    double *partials = (double *)workspace;
    hipStream_t st = (hipStream_t)stream;
    const unsigned g = (unsigned)blocks;
    switch (count) {
        case 1: launch_variation<1>(cur, list, n, partials, g, st); break;
        case 2: launch_variation<2>(cur, list, n, partials, g, st); break;
        case 3: launch_variation<3>(cur, list, n, partials, g, st); break;
        case 4: launch_variation<4>(cur, list, n, partials, g, st); break;
        case 5: launch_variation<5>(cur, list, n, partials, g, st); break;
        case 6: launch_variation<6>(cur, list, n, partials, g, st); break;
        case 7: launch_variation<7>(cur, list, n, partials, g, st); break;
        default: launch_variation<8>(cur, list, n, partials, g, st); break;
    }
    if (hipGetLastError() != hipSuccess) return QC_ERR_DEVICE;
    variation_final_kernel<<<dim3(1), dim3(kThreads), 0, st>>>(partials, (int)blocks, count, out);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}
