// Latent change reduction (Section 3.2 HLC, Eq. (5)): sum|cur - prev| and sum|prev| in one
// pass over both tensors, one launch, deterministic result.
//
// HBM-bound (8 bytes read per element, 12 bytes written in total).  Each lane reads 16 B per
// load, sums four terms in binary32 and carries the running sums in binary64; wavefronts
// combine by shuffles, blocks leave one partial pair each, and the block that finishes last
// adds the partials in index order, so the bits do not depend on scheduling.
#include "qc_internal.h"

namespace qc {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 2048;
constexpr int kControlBytes = 256;  // [0] = arrival counter, rest padding
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

__global__ __launch_bounds__(kThreads) void latent_delta_kernel(const float *__restrict__ cur,
                                                                const float *__restrict__ prev,
                                                                int64_t n, float *__restrict__ out3,
                                                                unsigned int *counter,
                                                                double *partials) {
    __shared__ double sh[2 * (kThreads / 64)];
    __shared__ bool is_last;
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
        __hip_atomic_store(&partials[2 * blockIdx.x], num, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&partials[2 * blockIdx.x + 1], den, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        const unsigned int ticket = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        is_last = ticket == gridDim.x - 1;
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();

    // last block: fixed-order combine of all partial pairs
    num = 0.0; den = 0.0;
    for (int b = threadIdx.x; b < (int)gridDim.x; b += kThreads) {
        num += __hip_atomic_load(&partials[2 * b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        den += __hip_atomic_load(&partials[2 * b + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    block_sum(num, den, sh);
    if (threadIdx.x == 0) {
        float rel;
        if (den > 0.0) rel = (float)(num / den);
        else rel = num > 0.0 ? __builtin_inff() : 0.0f;
        out3[0] = (float)num;
        out3[1] = (float)den;
        out3[2] = rel;
        __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ void zero_control_kernel(unsigned int *control) {
    if (threadIdx.x < kControlBytes / 4) control[threadIdx.x] = 0u;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace
}  // namespace qc

using namespace qc;

extern "C" size_t qc_latent_delta_workspace_bytes(int64_t n) {
    if (n < 1) return 0;
    return (size_t)kControlBytes + (size_t)kMaxBlocks * 2 * sizeof(double);
}

extern "C" qc_status qc_latent_delta_workspace_init(void *workspace, size_t workspace_bytes,
                                                    void *stream) {
    if (!workspace || !aligned(workspace, 256)) return QC_ERR_INVALID_ARG;
    if (workspace_bytes < (size_t)kControlBytes) return QC_ERR_WORKSPACE;
    zero_control_kernel<<<dim3(1), dim3(64), 0, (hipStream_t)stream>>>((unsigned int *)workspace);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" qc_status qc_latent_delta(const float *cur, const float *prev, int64_t n, float *out3,
                                     void *workspace, size_t workspace_bytes, void *stream) {
    if (!cur || !prev || !out3 || !workspace || n < 1) return QC_ERR_INVALID_ARG;
    if (!aligned(cur, 16) || !aligned(prev, 16) || !aligned(out3, 4) || !aligned(workspace, 256))
        return QC_ERR_INVALID_ARG;
    if (workspace_bytes < qc_latent_delta_workspace_bytes(n)) return QC_ERR_WORKSPACE;
    // one float4 per tensor per lane per unrolled step; cap the grid at the partial buffer
    int64_t blocks = (n / 4 + (int64_t)kThreads * kUnroll - 1) / ((int64_t)kThreads * kUnroll);
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    uint8_t *base = (uint8_t *)workspace;
    latent_delta_kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
        cur, prev, n, out3, (unsigned int *)base, (double *)(base + kControlBytes));
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}
