// qc_roofs: measures the roofs this GPU actually sustains, next to which the kernels of
// libqc are judged: streaming HBM bandwidth, the int8 MFMA issue rate with all-zero and with
// random operands (the chip is power limited: the clock it holds depends on how many bits
// toggle), the same MFMA loop fed with operand traffic in the proportions of the GEMM kernel,
// and LDS / L2 delivery rates per CU.  Stand-alone program, not part of libqc; prints one line
// per measurement, each followed by a machine-readable "@key value" line that bench.py reads.
// `--quick` runs only the measurements bench.py puts beside its own numbers (HBM streams, the
// cold 32 MiB read, the 16x16x64 MFMA loop).  Each measurement runs for several tens of
// milliseconds so that the clocks have settled.
#include <hip/hip_runtime.h>
#include <initializer_list>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <type_traits>
#include <vector>

#define CK(x)                                                                     \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// ---- HBM ---------------------------------------------------------------------------------
// POLICY bit 0: non-temporal loads, bit 1: non-temporal stores.  For buffers far larger than the
// caches, as here, what a pass leaves in them only costs; every roof below is the best over the
// launch shapes and these policies.
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int POLICY>
__device__ inline float4 ld16(const float4 *p) {
    if constexpr (POLICY & 1) {
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
        return make_float4(v.x, v.y, v.z, v.w);
    } else {
        return *p;
    }
}

template <int POLICY>
__device__ inline void st16(float4 *p, const float4 &v) {
    if constexpr (POLICY & 2) __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4 *>(p));
    else *p = v;
}

// Copy: like the read stream below, U loads of a lane in flight, then its U stores.
template <int THREADS, int U, int POLICY = 0>
__global__ __launch_bounds__(THREADS) void copy_kernel(const float4 *__restrict__ a,
                                                       float4 *__restrict__ b, int64_t n4) {
    constexpr int64_t kChunk = (int64_t)THREADS * U;
    for (int64_t base = (int64_t)blockIdx.x * kChunk; base < n4; base += (int64_t)gridDim.x * kChunk) {
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * THREADS + threadIdx.x;
            v[u] = ld16<POLICY>(a + (i < n4 ? i : 0));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * THREADS + threadIdx.x;
            if (i < n4) st16<POLICY>(b + i, v[u]);
        }
    }
}

// Two bytes read for every byte written (the proportions of the activation quantization:
// bf16 in, int8 out): two float4 loads feed one float4 store.
template <int THREADS, int U, int POLICY = 0>
__global__ __launch_bounds__(THREADS) void read2_write1_kernel(const float4 *__restrict__ a,
                                                               float4 *__restrict__ b, int64_t n4_out) {
    constexpr int64_t kChunk = (int64_t)THREADS * U;
    for (int64_t base = (int64_t)blockIdx.x * kChunk; base < n4_out; base += (int64_t)gridDim.x * kChunk) {
        float4 v[U], w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * THREADS + threadIdx.x;
            const int64_t j = i < n4_out ? i : 0;
            v[u] = ld16<POLICY>(a + 2 * j);
            w[u] = ld16<POLICY>(a + 2 * j + 1);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * THREADS + threadIdx.x;
            if (i < n4_out)
                st16<POLICY>(b + i, make_float4(v[u].x + w[u].x, v[u].y + w[u].y, v[u].z + w[u].z, v[u].w + w[u].w));
        }
    }
}

// Read-only stream: a block takes contiguous chunks of THREADS * U float4 and strides over the
// buffer by the grid; the U loads of a lane are all in flight before the first use.
template <int THREADS, int U, int POLICY = 0>
__global__ __launch_bounds__(THREADS) void read_kernel(const float4 *__restrict__ a, float *out,
                                                       int64_t n4) {
    float s = 0;
    constexpr int64_t kChunk = (int64_t)THREADS * U;
    for (int64_t base = (int64_t)blockIdx.x * kChunk; base < n4; base += (int64_t)gridDim.x * kChunk) {
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * THREADS + threadIdx.x;
            v[u] = ld16<POLICY>(a + (i < n4 ? i : 0));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) s += v[u].x + v[u].w;
    }
    if (s == 12345.678f) out[0] = s;
}

// The same over two buffers at once (the access pattern of the latent-change reduction).
template <int THREADS, int U, int POLICY = 0>
__global__ __launch_bounds__(THREADS) void read2_kernel(const float4 *__restrict__ a,
                                                        const float4 *__restrict__ b, float *out,
                                                        int64_t n4) {
    float s = 0;
    constexpr int64_t kChunk = (int64_t)THREADS * U;
    for (int64_t base = (int64_t)blockIdx.x * kChunk; base < n4; base += (int64_t)gridDim.x * kChunk) {
        float4 v[U], w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * THREADS + threadIdx.x;
            v[u] = ld16<POLICY>(a + (i < n4 ? i : 0));
            w[u] = ld16<POLICY>(b + (i < n4 ? i : 0));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) s += v[u].x + w[u].w;
    }
    if (s == 12345.678f) out[0] = s;
}

// ---- MFMA with optional operand traffic -----------------------------------------------------
// per iteration: 16 MFMAs (2 x 8 tiles); LDSR ds_read_b128 per wavefront from LDS; GLD 16 B/lane
// global loads per wavefront from an L2-resident buffer.  VIA_LDS: those GLD loads are
// direct-to-LDS copies into a ring private to the wavefront, each followed by a ds_read_b128 of
// the same size (the reads race with the copies on purpose: only the traffic matters here).
template <int LDSR, int GLD, bool VIA_LDS = false, bool M16 = false>
__global__ __launch_bounds__(256, 2) void mfma_kernel(const v4i *__restrict__ data,
                                                      const uint8_t *__restrict__ gsrc, int iters,
                                                      int *out) {
    __shared__ __attribute__((aligned(1024))) uint8_t lds[16384 + 32768];
    for (int i = threadIdx.x; i < 16384 / 16; i += 256) ((v4i *)lds)[i] = data[i];
    for (int i = threadIdx.x; i < 32768 / 16; i += 256) ((v4i *)(lds + 16384))[i] = data[i & 1023];
    __syncthreads();
    uint8_t *ring = lds + 16384 + (threadIdx.x >> 6) * 8192;  // 8 slots of 1 KiB per wavefront
    const uint32_t ring_lane = (uint32_t)(uintptr_t)ring + (threadIdx.x & 63) * 16;
    v16i acc[8];   // as 16x16 tiles: acc[t] holds four of them
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v4i a[2], b[8];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = data[(threadIdx.x * 4 + i) & 1023];
#pragma unroll
    for (int i = 0; i < 8; ++i) b[i] = data[(threadIdx.x * 8 + i) & 1023];
    const uint8_t *g = gsrc + ((size_t)(blockIdx.x & 63) * 65536) + wave * 16384 + lane * 16;
    v4i gx = {0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
        v4i gl[GLD > 0 ? GLD : 1];
#pragma unroll
        for (int j = 0; j < GLD; ++j) {
            const uint8_t *src = g + ((it * GLD + j) & 15) * 1024;
            if (VIA_LDS) {
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void *)src,
                    (__attribute__((address_space(3))) void *)(ring + ((it * GLD + j) & 7) * 1024), 16, 0, 0);
                asm volatile("ds_read_b128 %0, %1" : "=v"(gl[j])
                             : "v"(ring_lane + (uint32_t)(((it * GLD + j + 4) & 7) * 1024)));
            } else {
                gl[j] = *(const v4i *)src;
            }
        }
#pragma unroll
        for (int j = 0; j < LDSR; ++j) {
            const v4i v = *(const v4i *)(lds + ((j + it) & 15) * 1024 + lane * 16);
            if (j < 8) b[j] = v;
            else a[j & 1] = v;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (M16) {  // the same multiply count as two 16x16x64 operations
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int q = 2 * i + h;
                        v4i c = {acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]};
                        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[t], c, 0, 0, 0);
                        acc[t][4 * q] = c[0]; acc[t][4 * q + 1] = c[1]; acc[t][4 * q + 2] = c[2]; acc[t][4 * q + 3] = c[3];
                    }
                } else {
                    acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[t], acc[t], 0, 0, 0);
                }
            }
        if (VIA_LDS) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < GLD; ++j) gx ^= gl[j];
    }
    if (VIA_LDS) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int s = gx[0] ^ gx[1] ^ gx[2] ^ gx[3];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
    if (s == 0x7fffffff) out[0] = s;
}

// ---- LDS -------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void lds_read_kernel(int iters, int *out) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[16384];
    for (int i = threadIdx.x; i < 16384 / 4; i += 1024) ((int *)lds)[i] = i;
    __syncthreads();
    const unsigned addr = (threadIdx.x & 63) * 16 + ((threadIdx.x >> 6) & 7) * 1024;
    v4i a, b, c, d, e, f, g, h;
    for (int it = 0; it < iters; ++it) {
        asm volatile(
            "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:1024\n"
            "ds_read_b128 %2, %8 offset:2048\n ds_read_b128 %3, %8 offset:3072\n"
            "ds_read_b128 %4, %8 offset:4096\n ds_read_b128 %5, %8 offset:5120\n"
            "ds_read_b128 %6, %8 offset:6144\n ds_read_b128 %7, %8 offset:7168\n"
            "s_waitcnt lgkmcnt(0)\n"
            : "=v"(a), "=v"(b), "=v"(c), "=v"(d), "=v"(e), "=v"(f), "=v"(g), "=v"(h)
            : "v"(addr)
            : "memory");
    }
    if (a[0] + b[0] + c[0] + d[0] + e[0] + f[0] + g[0] + h[0] == 0x7fffffff) out[0] = 1;
}

__global__ __launch_bounds__(512) void lds_write_kernel(int iters, int *out) {
    extern __shared__ __attribute__((aligned(16))) uint8_t dyn_lds[];
    const unsigned addr = (threadIdx.x & 63) * 16 + ((threadIdx.x >> 6) & 7) * 8192;
    const v4i v = {(int)threadIdx.x, 1, 2, 3};
    for (int it = 0; it < iters; ++it) {
        asm volatile(
            "ds_write_b128 %0, %1\n ds_write_b128 %0, %1 offset:1024\n"
            "ds_write_b128 %0, %1 offset:2048\n ds_write_b128 %0, %1 offset:3072\n"
            "ds_write_b128 %0, %1 offset:4096\n ds_write_b128 %0, %1 offset:5120\n"
            "ds_write_b128 %0, %1 offset:6144\n ds_write_b128 %0, %1 offset:7168\n"
            "s_waitcnt lgkmcnt(0)\n" ::"v"(addr), "v"(v)
            : "memory");
    }
    __syncthreads();
    if (dyn_lds[threadIdx.x] == 77 && iters < 0) out[0] = 1;
}

// ---- L2 -> CU ---------------------------------------------------------------------------------
template <int THREADS>
__global__ __launch_bounds__(THREADS) void l2_load_kernel(const uint8_t *src, int iters, int *out) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint8_t *base = src + (size_t)(blockIdx.x % 16) * 65536;  // 1 MiB hot set
    v4i acc = {0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
        v4i v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int chunk = (it * 8 + j) * (THREADS / 64) + wave;
            v[j] = *(const v4i *)(base + ((size_t)chunk * 1024) % 65536 + lane * 16);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j];
    }
    if (acc[0] + acc[1] + acc[2] + acc[3] == 0x12345) out[0] = 1;
}

template <typename F>
static float settled_ms(F launch) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float ms = 0, total = 0;
    while (total < 80.f) {  // let the clocks settle
        CK(hipEventRecord(e0));
        launch();
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        total += ms;
    }
    float sum = 0;
    for (int i = 0; i < 3; ++i) {
        CK(hipEventRecord(e0));
        launch();
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        CK(hipEventElapsedTime(&ms, e0, e1));
        sum += ms;
    }
    return sum / 3;
}

int main(int argc, char **argv) {
    const bool quick = argc > 1 && strcmp(argv[1], "--quick") == 0;
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int CU = prop.multiProcessorCount;
    const double ghz = 2.4;
    printf("device %s, %d CUs; per-CU rates below are quoted per clock of a nominal %.1f GHz\n",
           prop.gcnArchName, CU, ghz);
    int *dout;
    CK(hipMalloc(&dout, 64));

    {  // HBM
        const int64_t n = (int64_t)1 << 30;
        float4 *a, *b;
        CK(hipMalloc(&a, n));
        CK(hipMalloc(&b, n));
        CK(hipMemset(a, 1, n));
        CK(hipMemset(b, 2, n));
        auto best_of = [](std::initializer_list<float> ms) {
            float b = 1e30f;
            for (float m : ms) b = m < b ? m : b;
            return b;
        };
        float *fout = (float *)dout;
        const int64_t n4 = n / 16;
        float ms = settled_ms([&] { read_kernel<256, 4><<<16384, 256>>>(a, fout, n4); });
        float ms2 = settled_ms([&] { read_kernel<1024, 4><<<CU, 1024>>>(a, fout, n4); });
        float ms3 = settled_ms([&] { read_kernel<256, 8><<<8 * CU, 256>>>(a, fout, n4); });
        float ms4 = settled_ms([&] { read_kernel<1024, 4, 1><<<CU, 1024>>>(a, fout, n4); });
        float ms5 = settled_ms([&] { read_kernel<256, 8, 1><<<8 * CU, 256>>>(a, fout, n4); });
        const float best = best_of({ms, ms2, ms3, ms4, ms5});
        printf("hbm  read-only stream, 1 GiB (three launch shapes: %.0f / %.0f / %.0f; the last two with "
               "non-temporal loads: %.0f / %.0f): %7.0f GB/s\n",
               n / ms * 1e-6, n / ms2 * 1e-6, n / ms3 * 1e-6, n / ms4 * 1e-6, n / ms5 * 1e-6, n / best * 1e-6);
        printf("@hbm_read_gbs %.0f\n", n / best * 1e-6);
        ms = settled_ms([&] { copy_kernel<256, 1><<<65536, 256>>>(a, b, n4); });
        ms2 = settled_ms([&] { copy_kernel<256, 4><<<8 * CU, 256>>>(a, b, n4); });
        ms3 = settled_ms([&] { copy_kernel<1024, 4><<<CU, 1024>>>(a, b, n4); });
        ms4 = settled_ms([&] { copy_kernel<256, 4, 1><<<8 * CU, 256>>>(a, b, n4); });
        ms5 = settled_ms([&] { copy_kernel<256, 4, 2><<<8 * CU, 256>>>(a, b, n4); });
        float ms6 = settled_ms([&] { copy_kernel<256, 4, 3><<<8 * CU, 256>>>(a, b, n4); });
        const float cbest = best_of({ms, ms2, ms3, ms4, ms5, ms6});
        printf("hbm  copy, 1 GiB read + 1 GiB written (three launch shapes: %.0f / %.0f / %.0f; the second "
               "with non-temporal loads / stores / both: %.0f / %.0f / %.0f): %7.0f GB/s\n",
               2.0 * n / ms * 1e-6, 2.0 * n / ms2 * 1e-6, 2.0 * n / ms3 * 1e-6, 2.0 * n / ms4 * 1e-6,
               2.0 * n / ms5 * 1e-6, 2.0 * n / ms6 * 1e-6, 2.0 * n / cbest * 1e-6);
        printf("@hbm_copy_gbs %.0f\n", 2.0 * n / cbest * 1e-6);
        {   // 1 GiB read, 512 MiB written
            const int64_t n4o = n / 32;
            ms = settled_ms([&] { read2_write1_kernel<256, 2><<<8 * CU, 256>>>(a, b, n4o); });
            ms2 = settled_ms([&] { read2_write1_kernel<256, 4><<<8 * CU, 256>>>(a, b, n4o); });
            ms3 = settled_ms([&] { read2_write1_kernel<1024, 2><<<CU, 1024>>>(a, b, n4o); });
            ms4 = settled_ms([&] { read2_write1_kernel<256, 4, 1><<<8 * CU, 256>>>(a, b, n4o); });
            ms5 = settled_ms([&] { read2_write1_kernel<256, 4, 2><<<8 * CU, 256>>>(a, b, n4o); });
            ms6 = settled_ms([&] { read2_write1_kernel<256, 4, 3><<<8 * CU, 256>>>(a, b, n4o); });
            const float mbest = best_of({ms, ms2, ms3, ms4, ms5, ms6});
            printf("hbm  1 GiB read + 512 MiB written, the quantizer's proportions (three launch shapes: "
                   "%.0f / %.0f / %.0f; the second with non-temporal loads / stores / both: %.0f / %.0f / %.0f): "
                   "%7.0f GB/s\n",
                   1.5 * n / ms * 1e-6, 1.5 * n / ms2 * 1e-6, 1.5 * n / ms3 * 1e-6, 1.5 * n / ms4 * 1e-6,
                   1.5 * n / ms5 * 1e-6, 1.5 * n / ms6 * 1e-6, 1.5 * n / mbest * 1e-6);
            printf("@hbm_read2_write1_gbs %.0f\n", 1.5 * n / mbest * 1e-6);
        }
        // Two 16 MiB buffers per launch (the size of the latent pair), each launch on the next
        // of 12 distinct pairs so that nothing is left in the caches from the launch before, and
        // the same on one pair that stays in the Infinity Cache.  Timed as bench.py times its
        // kernels: events around a batch of back-to-back launches, so the figure includes what
        // a launch boundary costs.
        const int64_t m = (int64_t)16 << 20;   // bytes per buffer
        hipEvent_t e0, e1;
        CK(hipEventCreate(&e0));
        CK(hipEventCreate(&e1));
        for (int cold = 1; cold >= 0; --cold) {
            double us_of[2];
            for (int nt = 0; nt < 2; ++nt) {   // ordinary loads, then non-temporal ones
                float sum = 0;
                const int rounds = 10, batch = 24;
                for (int r = -300; r < rounds; ++r) {   // about 50 ms of the same launches first
                    CK(hipEventRecord(e0));
                    for (int i = 0; i < batch; ++i) {
                        const int64_t off = cold ? (int64_t)(i % 12) * 2 * m : 0;
                        const float4 *p = (const float4 *)((const char *)a + off), *q = (const float4 *)((const char *)a + off + m);
                        if (nt) read2_kernel<1024, 4, 1><<<CU, 1024>>>(p, q, (float *)dout, m / 16);
                        else read2_kernel<1024, 4, 0><<<CU, 1024>>>(p, q, (float *)dout, m / 16);
                    }
                    CK(hipEventRecord(e1));
                    CK(hipEventSynchronize(e1));
                    float t;
                    CK(hipEventElapsedTime(&t, e0, e1));
                    if (r >= 0) sum += t / batch;
                }
                us_of[nt] = sum / rounds * 1e3;
            }
            const double us = us_of[0] < us_of[1] ? us_of[0] : us_of[1];
            printf("hbm  read-only, 2 x 16 MiB per launch, %s (ordinary / non-temporal loads: %.2f / %.2f): "
                   "%6.2f us per launch, %7.0f GB/s\n",
                   cold ? "cold (12 pairs in turn)" : "warm (one pair again and again)", us_of[0], us_of[1], us,
                   2.0 * m / us * 1e-3);
            printf("@read_32mib_%s_us %.2f\n", cold ? "cold" : "warm", us);
        }
        CK(hipFree(a));
        CK(hipFree(b));
    }

    v4i *d_zero, *d_rand;
    uint8_t *gsrc;
    {
        std::vector<int> h(16384), z(16384, 0);
        srand(3);
        for (auto &v : h) {
            uint32_t w = 0;
            for (int b = 0; b < 4; ++b) {
                const int g = (rand() % 41) - 20 + (rand() % 41) - 20;  // spread like weight codes
                w |= (uint32_t)(uint8_t)(int8_t)g << (8 * b);
            }
            v = (int)w;
        }
        CK(hipMalloc(&d_zero, 65536));
        CK(hipMalloc(&d_rand, 65536));
        CK(hipMemcpy(d_zero, z.data(), 65536, hipMemcpyHostToDevice));
        CK(hipMemcpy(d_rand, h.data(), 65536, hipMemcpyHostToDevice));
        std::vector<uint8_t> hg(64 * 65536);
        for (auto &v : hg) v = rand() & 255;
        CK(hipMalloc(&gsrc, hg.size()));
        CK(hipMemcpy(gsrc, hg.data(), hg.size(), hipMemcpyHostToDevice));
    }
    const int iters = 20000, blocks = 2 * CU;
    const double ops = (double)blocks * 4 * iters * 16 * 65536.0;
    auto tops = [&](float ms) { return ops / ms * 1e-9; };
    // Operand traffic is quoted per 32 K multiply-adds: one 32x32x32 or two 16x16x64 operations.
    auto mfma_lines = [&](auto m16_tag, const char *form, const char *key) {
        constexpr bool M16 = decltype(m16_tag)::value;
        double v;
        v = tops(settled_ms([&] { mfma_kernel<0, 0, false, M16><<<blocks, 256>>>(d_zero, gsrc, iters, dout); }));
        printf("mfma %s, 2 wavefronts/SIMD, registers only, zero operands:  %5.0f TOPS\n", form, v);
        printf("@mfma_%s_zero_tops %.0f\n", key, v);
        v = tops(settled_ms([&] { mfma_kernel<0, 0, false, M16><<<blocks, 256>>>(d_rand, gsrc, iters, dout); }));
        printf("  random int8 operands:                                                 %5.0f TOPS\n", v);
        printf("@mfma_%s_random_tops %.0f\n", key, v);
        if (!quick) {
            printf("  random + 0.5 ds_read_b128 per 32 K multiply-adds:                     %5.0f TOPS\n",
                   tops(settled_ms([&] { mfma_kernel<8, 0, false, M16><<<blocks, 256>>>(d_rand, gsrc, iters, dout); })));
            printf("  random + 256 B loaded from L2:                                        %5.0f TOPS\n",
                   tops(settled_ms([&] { mfma_kernel<0, 4, false, M16><<<blocks, 256>>>(d_rand, gsrc, iters, dout); })));
            printf("  random + 256 B copied L2 -> LDS and read back from LDS:               %5.0f TOPS\n",
                   tops(settled_ms([&] { mfma_kernel<0, 4, true, M16><<<blocks, 256>>>(d_rand, gsrc, iters, dout); })));
        }
        v = tops(settled_ms([&] { mfma_kernel<8, 6, false, M16><<<blocks, 256>>>(d_rand, gsrc, iters, dout); }));
        printf("  random + 0.5 ds_read_b128 and 384 B from L2 (the GEMM's proportions): %5.0f TOPS\n", v);
        printf("@mfma_%s_gemm_traffic_tops %.0f\n", key, v);
        if (!quick)
            printf("  random + 0.5 ds_read_b128 and 128 B from L2:                          %5.0f TOPS\n",
                   tops(settled_ms([&] { mfma_kernel<8, 2, false, M16><<<blocks, 256>>>(d_rand, gsrc, iters, dout); })));
    };
    if (!quick) mfma_lines(std::false_type{}, "v_mfma_i32_32x32x32_i8", "32x32x32");
    mfma_lines(std::true_type{}, "v_mfma_i32_16x16x64_i8", "16x16x64");
    if (quick) return 0;

    {
        const int li = 20000;
        float ms = settled_ms([&] { lds_read_kernel<<<CU, 1024>>>(li, dout); });
        printf("lds  ds_read_b128, 16 wavefronts/CU:   %6.1f B/clk/CU\n",
               (double)1024 * li * 8 * 16 / (ms * 1e-3) / (ghz * 1e9));
        ms = settled_ms([&] { lds_write_kernel<<<CU, 512, 65536>>>(li, dout); });
        printf("lds  ds_write_b128, 8 wavefronts/CU:   %6.1f B/clk/CU\n",
               (double)512 * li * 8 * 16 / (ms * 1e-3) / (ghz * 1e9));
        const int di = 4000;
        ms = settled_ms([&] { l2_load_kernel<256><<<2 * CU, 256>>>(gsrc, di, dout); });
        printf("l2   global_load_dwordx4, 8 wavefronts/CU:  %6.1f B/clk/CU\n",
               (double)2 * 256 * di * 8 * 16 / (ms * 1e-3) / (ghz * 1e9));
        ms = settled_ms([&] { l2_load_kernel<1024><<<CU, 1024>>>(gsrc, di, dout); });
        printf("l2   global_load_dwordx4, 16 wavefronts/CU: %6.1f B/clk/CU\n",
               (double)1024 * di * 8 * 16 / (ms * 1e-3) / (ghz * 1e9));
    }
    return 0;
}
