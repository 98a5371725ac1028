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
