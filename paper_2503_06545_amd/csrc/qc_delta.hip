// Latent change reduction (Section 3.2 HLC, Eq. (5)): sum|cur - prev| and sum|prev| in one
// pass over both tensors, deterministic result.
//
// HBM-bound (8 bytes read per element, 12 bytes written in total).  Each lane reads 16 B per
// load, sums four terms in binary32 and carries the running sums in binary64; wavefronts
// combine by shuffles and every block leaves one partial pair.  A second, single-block launch
// adds the partial pairs in index order, so the bits do not depend on scheduling.  (A single
// launch that lets the last block to arrive do the combine was measured slower: the device-scope
// arrival counter costs about 15 ns per block, more than the second launch.)
#include "qc_internal.h"

namespace qc {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 256;     // one block per CU
constexpr int kUnroll = 4;          // float4 loads in flight per tensor per lane

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    return v;
}

__device__ inline float abs4(const float4 &a, const float4 &b) {
    return (fabsf(a.x - b.x) + fabsf(a.y - b.y)) + (fabsf(a.z - b.z) + fabsf(a.w - b.w));
}
__device__ inline float abs4(const float4 &b) {
    return (fabsf(b.x) + fabsf(b.y)) + (fabsf(b.z) + fabsf(b.w));
}

// block-wide sum of (num, den); result valid in thread 0
__device__ inline void block_sum(double &num, double &den, double *sh) {
    num = wave_sum(num);
    den = wave_sum(den);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sh[2 * wave] = num; sh[2 * wave + 1] = den; }
    __syncthreads();
    if (threadIdx.x == 0) {
        num = sh[0]; den = sh[1];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) { num += sh[2 * w]; den += sh[2 * w + 1]; }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kThreads) void latent_delta_partial_kernel(
    const float *__restrict__ cur, const float *__restrict__ prev, int64_t n,
    double *__restrict__ partials) {
    __shared__ double sh[2 * (kThreads / 64)];
    const int64_t n4 = n / 4;
    const float4 *c4 = reinterpret_cast<const float4 *>(cur);
    const float4 *p4 = reinterpret_cast<const float4 *>(prev);
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    double num = 0.0, den = 0.0;

    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    for (; i + (kUnroll - 1) * stride < n4; i += kUnroll * stride) {
        float4 a[kUnroll], b[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) { a[u] = c4[i + u * stride]; b[u] = p4[i + u * stride]; }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) { num += (double)abs4(a[u], b[u]); den += (double)abs4(b[u]); }
    }
    for (; i < n4; i += stride) {
        const float4 a = c4[i], b = p4[i];
        num += (double)abs4(a, b);
        den += (double)abs4(b);
    }
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - n4 * 4)) {  // up to 3 trailing elements
        const int64_t j = n4 * 4 + threadIdx.x;
        num += (double)fabsf(cur[j] - prev[j]);
        den += (double)fabsf(prev[j]);
    }
    block_sum(num, den, sh);
    if (threadIdx.x == 0) {
        partials[2 * blockIdx.x] = num;
        partials[2 * blockIdx.x + 1] = den;
    }
}

// one block: fixed-order combine of the partial pairs, then the ratio
__global__ __launch_bounds__(kThreads) void latent_delta_final_kernel(
    const double *__restrict__ partials, int count, float *__restrict__ out3) {
    __shared__ double sh[2 * (kThreads / 64)];
    double num = 0.0, den = 0.0;
    for (int b = threadIdx.x; b < count; b += kThreads) {
        num += partials[2 * b];
        den += partials[2 * b + 1];
    }
    block_sum(num, den, sh);
    if (threadIdx.x == 0) {
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

template <typename T>
__global__ __launch_bounds__(kThreads) void similarity_partial_kernel(
    const T *__restrict__ a, const T *__restrict__ b, int64_t n, double *__restrict__ partials) {
    __shared__ double sh[3 * (kThreads / 64)];
    const int64_t n8 = n / 8;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n8; i += 2 * stride) {
        Oct<T> x[2], y[2];
        const bool second = i + stride < n8;
        x[0].load(a + 8 * i);
        y[0].load(b + 8 * i);
        if (second) { x[1].load(a + 8 * (i + stride)); y[1].load(b + 8 * (i + stride)); }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u == 1 && !second) break;
            float pab[2] = {0.f, 0.f}, paa[2] = {0.f, 0.f}, pbb[2] = {0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 8; ++e) {  // two 4-term binary32 sums each
                const float xv = x[u].get(e), yv = y[u].get(e);
                pab[e >> 2] += xv * yv;
                paa[e >> 2] += xv * xv;
                pbb[e >> 2] += yv * yv;
            }
            ab += (double)pab[0] + (double)pab[1];
            aa += (double)paa[0] + (double)paa[1];
            bb += (double)pbb[0] + (double)pbb[1];
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - n8 * 8)) {  // up to 7 trailing elements
        const int64_t j = n8 * 8 + threadIdx.x;
        float xv, yv;
        if constexpr (sizeof(T) == 2) {
            xv = __uint_as_float((uint32_t)a[j] << 16);
            yv = __uint_as_float((uint32_t)b[j] << 16);
        } else {
            xv = a[j];
            yv = b[j];
        }
        ab += (double)(xv * yv);
        aa += (double)(xv * xv);
        bb += (double)(yv * yv);
    }
    ab = wave_sum(ab); aa = wave_sum(aa); bb = wave_sum(bb);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sh[3 * wave] = ab; sh[3 * wave + 1] = aa; sh[3 * wave + 2] = bb; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) { sh[0] += sh[3 * w]; sh[1] += sh[3 * w + 1]; sh[2] += sh[3 * w + 2]; }
        partials[3 * blockIdx.x] = sh[0];
        partials[3 * blockIdx.x + 1] = sh[1];
        partials[3 * blockIdx.x + 2] = sh[2];
    }
}

__global__ __launch_bounds__(kThreads) void similarity_final_kernel(
    const double *__restrict__ partials, int count, float *__restrict__ out4) {
    __shared__ double sh[3 * (kThreads / 64)];
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int b = threadIdx.x; b < count; b += kThreads) {
        ab += partials[3 * b]; aa += partials[3 * b + 1]; bb += partials[3 * b + 2];
    }
    ab = wave_sum(ab); aa = wave_sum(aa); bb = wave_sum(bb);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sh[3 * wave] = ab; sh[3 * wave + 1] = aa; sh[3 * wave + 2] = bb; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) { sh[0] += sh[3 * w]; sh[1] += sh[3 * w + 1]; sh[2] += sh[3 * w + 2]; }
        const double denom = sqrt(sh[1]) * sqrt(sh[2]);
        out4[0] = (float)sh[0];
        out4[1] = (float)sh[1];
        out4[2] = (float)sh[2];
        out4[3] = denom > 0.0 ? (float)(sh[0] / denom) : 0.0f;
    }
}

// block-wide sum of one value; result valid in thread 0.  sh holds kThreads / 64 doubles.
__device__ inline double block_sum1(double v, double *sh) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        v = sh[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) v += sh[w];
    }
    return v;
}

// ---- inter-frame gradient norm (Section 3.2 HLC, second factor of Eq. (5)) -----------------
// The feature map is [frames, inner]; the gradient is the forward difference along the frame
// axis and the norm is Euclidean.  As a reduction it is a pass over the pair (m, m + inner):
// every element is read twice, the second time one frame (inner elements) later, which the
// caches absorb for the frame sizes of a latent.

__device__ inline float widen(float v) { return v; }
__device__ inline float widen(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// VEC: inner is a multiple of 8, so both streams can be read 8 elements at a time.
template <typename T, bool VEC>
__global__ __launch_bounds__(kThreads) void gradient_partial_kernel(
    const T *__restrict__ m, int64_t inner, int64_t n, double *__restrict__ partials) {
    __shared__ double sh[kThreads / 64];
    const T *lo = m, *hi = m + inner;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t first = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    double ss = 0.0;
    int64_t done = 0;
    if constexpr (VEC) {
        const int64_t n8 = n / 8;
        for (int64_t i = first; i < n8; i += 2 * stride) {
            Oct<T> x[2], y[2];
            const bool second = i + stride < n8;
            x[0].load(lo + 8 * i);
            y[0].load(hi + 8 * i);
            if (second) { x[1].load(lo + 8 * (i + stride)); y[1].load(hi + 8 * (i + stride)); }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (u == 1 && !second) break;
                float p[2] = {0.f, 0.f};
#pragma unroll
                for (int e = 0; e < 8; ++e) {  // two 4-term binary32 sums
                    const float d = y[u].get(e) - x[u].get(e);
                    p[e >> 2] += d * d;
                }
                ss += (double)p[0] + (double)p[1];
            }
        }
        done = n8 * 8;
    }
    for (int64_t j = done + first; j < n; j += stride) {
        const float d = widen(hi[j]) - widen(lo[j]);
        ss += (double)(d * d);
    }
    ss = block_sum1(ss, sh);
    if (threadIdx.x == 0) partials[blockIdx.x] = ss;
}

__global__ __launch_bounds__(kThreads) void gradient_final_kernel(
    const double *__restrict__ partials, int count, float *__restrict__ out2) {
    __shared__ double sh[kThreads / 64];
    double ss = 0.0;
    for (int b = threadIdx.x; b < count; b += kThreads) ss += partials[b];
    ss = block_sum1(ss, sh);
    if (threadIdx.x == 0) {
        out2[0] = (float)ss;
        out2[1] = (float)sqrt(ss);
    }
}

// ---- cumulative variation over the previous steps (Section 3.3 SRAP, Eq. (11)) --------------
// L1 distance of the current tensor to each of COUNT earlier ones in one pass: the current
// tensor is read once, not once per distance.

struct PrevList { const float *p[QC_MAX_PREV]; };

template <int COUNT>
__global__ __launch_bounds__(kThreads) void variation_partial_kernel(
    const float *__restrict__ cur, PrevList prevs, int64_t n, double *__restrict__ partials) {
    __shared__ double sh[kThreads / 64];
    const int64_t n4 = n / 4;
    const float4 *c4 = reinterpret_cast<const float4 *>(cur);
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    double d[COUNT];
#pragma unroll
    for (int c = 0; c < COUNT; ++c) d[c] = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += 2 * stride) {
        const bool second = i + stride < n4;
        const int64_t i1 = second ? i + stride : i;  // a valid index either way
        const float4 a0 = c4[i], a1 = c4[i1];
        float4 b0[COUNT], b1[COUNT];
#pragma unroll
        for (int c = 0; c < COUNT; ++c) {
            const float4 *p4 = reinterpret_cast<const float4 *>(prevs.p[c]);
            b0[c] = p4[i];
            b1[c] = p4[i1];
        }
#pragma unroll
        for (int c = 0; c < COUNT; ++c) {
            d[c] += (double)abs4(a0, b0[c]);
            if (second) d[c] += (double)abs4(a1, b1[c]);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - n4 * 4)) {  // up to 3 trailing elements
        const int64_t j = n4 * 4 + threadIdx.x;
#pragma unroll
        for (int c = 0; c < COUNT; ++c) d[c] += (double)fabsf(cur[j] - prevs.p[c][j]);
    }
#pragma unroll
    for (int c = 0; c < COUNT; ++c) {
        const double t = block_sum1(d[c], sh);
        if (threadIdx.x == 0) partials[(int64_t)blockIdx.x * QC_MAX_PREV + c] = t;
    }
}

__global__ __launch_bounds__(kThreads) void variation_final_kernel(
    const double *__restrict__ partials, int blocks, int count, float *__restrict__ out) {
    __shared__ double sh[kThreads / 64];
    double total = 0.0;
    for (int c = 0; c < count; ++c) {
        double v = 0.0;
        for (int b = threadIdx.x; b < blocks; b += kThreads) v += partials[(int64_t)b * QC_MAX_PREV + c];
        v = block_sum1(v, sh);
        if (threadIdx.x == 0) {
            out[c] = (float)v;
            total += v;
        }
    }
    if (threadIdx.x == 0) out[count] = (float)total;
}

template <int COUNT>
void launch_variation(const float *cur, const PrevList &prevs, int64_t n, double *partials,
                      unsigned blocks, hipStream_t stream) {
    variation_partial_kernel<COUNT><<<dim3(blocks), dim3(kThreads), 0, stream>>>(cur, prevs, n, partials);
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
    // one float4 per tensor per lane per unrolled step; at most one block per CU
    int64_t blocks = (n / 4 + (int64_t)kThreads * kUnroll - 1) / ((int64_t)kThreads * kUnroll);
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    double *partials = (double *)workspace;
    latent_delta_partial_kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
        cur, prev, n, partials);
    if (hipGetLastError() != hipSuccess) return QC_ERR_DEVICE;
    latent_delta_final_kernel<<<dim3(1), dim3(kThreads), 0, (hipStream_t)stream>>>(
        partials, (int)blocks, out3);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
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
    int64_t blocks = (n / 8 + (int64_t)kThreads * 2 - 1) / ((int64_t)kThreads * 2);
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    double *partials = (double *)workspace;
    if (dt == QC_BF16)
        similarity_partial_kernel<uint16_t><<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
            (const uint16_t *)a, (const uint16_t *)b, n, partials);
    else
        similarity_partial_kernel<float><<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
            (const float *)a, (const float *)b, n, partials);
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
    const int64_t per_block = (int64_t)kThreads * (vec ? 16 : 4);
    int64_t blocks = (n + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    double *partials = (double *)workspace;
    const dim3 grid((unsigned)blocks), block(kThreads);
    hipStream_t st = (hipStream_t)stream;
    if (dt == QC_BF16) {
        if (vec) gradient_partial_kernel<uint16_t, true><<<grid, block, 0, st>>>((const uint16_t *)m, inner, n, partials);
        else gradient_partial_kernel<uint16_t, false><<<grid, block, 0, st>>>((const uint16_t *)m, inner, n, partials);
    } else {
        if (vec) gradient_partial_kernel<float, true><<<grid, block, 0, st>>>((const float *)m, inner, n, partials);
        else gradient_partial_kernel<float, false><<<grid, block, 0, st>>>((const float *)m, inner, n, partials);
    }
    if (hipGetLastError() != hipSuccess) return QC_ERR_DEVICE;
    gradient_final_kernel<<<dim3(1), block, 0, st>>>(partials, (int)blocks, out2);
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
    int64_t blocks = (n / 4 + (int64_t)kThreads * 2 - 1) / ((int64_t)kThreads * 2);
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
