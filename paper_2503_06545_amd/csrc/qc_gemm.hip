// Integer GEMM with fused dequantize / bias / GELU epilogue (Section 4.1 "Hardware
// Implementation": the DiT linears as low-bit GEMMs with quantization fused around them).
//
//   acc[m, n] = sum_k qx[m, k] * qw[n, k]          exact, int32, v_mfma_i32_32x32x32_i8
//   Y[m, n]   = act(acc * sx[m] * sw[n] + bias[n])
//
// Block tile 256 tokens x 128 channels, 4 wavefronts as 2 (tokens) x 2 (channels), each
// 128 x 64 = 4 x 2 MFMA tiles (128 accumulator registers), two blocks per CU so that one
// block's epilogue overlaps the other's MFMA loop.  Operands arrive pre-arranged as 1 KiB
// MFMA fragments (see qc_internal.h), so HBM -> LDS is a linear direct-to-LDS copy and
// LDS -> register reads are linear 16 B/lane and conflict free.  K advances 64 per stage
// through a 3-deep ring of LDS buffers.  The weight is the MFMA "A" operand (rows of the
// result tile = channels) and the tokens the "B" operand, so a lane owns one token and runs
// of consecutive channels, which the weight row permutation widens to 8.
#include "qc_internal.h"

namespace qc {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kStages = 3;
constexpr int kXFrags = (kTileM / kFragRows) * 2;  // 16 fragments of X per 64-k stage

template <int BITS>
struct StageLayout {
    // fragments (1 KiB each) of W per stage: 8-bit 4 row blocks x 2 k fragments; 4-bit one
    // 64-k unit per row block
    static constexpr int kWFrags = BITS == 8 ? (kTileN / kFragRows) * 2 : (kTileN / kFragRows);
    static constexpr int kFrags = kWFrags + kXFrags;
    static constexpr int kBytes = kFrags * kFragBytes;
    static constexpr int kFragsPerWave = kFrags / 4;
    static_assert(kFrags % 4 == 0, "fragments must split evenly over 4 wavefronts");
};

struct GemmArgs {
    const uint8_t *x_tiled;
    const float *x_scale;
    const uint8_t *w_codes;
    const float *w_scale;
    const float *bias;
    void *Y;
    int64_t M, N;
    int KF;         // 32-k fragments per row (Kp / 32)
    int m_tiles, n_tiles;
};

__device__ inline void lds_dma_16(const uint8_t *gsrc, uint8_t *lds_dst) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void *)gsrc,
        (__attribute__((address_space(3))) void *)lds_dst, 16, 0, 0);
}

__device__ inline float gelu_tanh_f(float y) {
    // 0.5 y (1 + tanh(u)) = y / (1 + exp(-2u)),  u = sqrt(2/pi) (y + 0.044715 y^3)
    const float c1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;  // -2 sqrt(2/pi) log2(e)
    const float c2 = c1 * 0.044715f;
    const float t = y * (c1 + c2 * (y * y));
    return y * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}

__device__ inline float gelu_erf_f(float y) { return 0.5f * y * (1.0f + erff(y * 0.70710678118654752f)); }

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    // round to nearest even on the dropped 16 bits
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

// Map the launch's block index to a tile so that the blocks resident on one XCD at a time
// (block b runs on XCD b % 8) work on a compact 8 x 8 patch of tiles and share its operand
// panels through that XCD's L2.
__device__ inline void tile_of_block(int b, int nblocks, int m_tiles, int n_tiles, int &mt, int &nt) {
    const int xcd = b % 8, slot = b / 8;
    const int per = nblocks / 8, extra = nblocks % 8;
    const int v = xcd * per + (xcd < extra ? xcd : extra) + slot;  // blocks of one XCD are consecutive
    constexpr int kGroupM = 8;
    const int per_group = kGroupM * n_tiles;
    const int g = v / per_group, r = v % per_group;
    const int m0 = g * kGroupM;
    const int gm = (m_tiles - m0) < kGroupM ? (m_tiles - m0) : kGroupM;
    mt = m0 + r % gm;
    nt = r / gm;
}

template <int BITS, int OUT, int EPI>
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmArgs a) {
    using L = StageLayout<BITS>;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wn = wave & 1, wm = wave >> 1;
    int mt, nt;
    tile_of_block(blockIdx.x, gridDim.x, a.m_tiles, a.n_tiles, mt, nt);

    const int stages = a.KF / 2;
    // global source of each fragment this wavefront copies, at stage 0
    const uint8_t *src[L::kFragsPerWave];
    int src_step[L::kFragsPerWave];
#pragma unroll
    for (int j = 0; j < L::kFragsPerWave; ++j) {
        const int f = wave * L::kFragsPerWave + j;
        if (f < L::kWFrags) {
            if (BITS == 8) {
                const int rb = f >> 1, kf = f & 1;
                src[j] = a.w_codes + ((int64_t)(nt * 4 + rb) * a.KF + kf) * kFragBytes;
                src_step[j] = 2 * kFragBytes;
            } else {
                src[j] = a.w_codes + ((int64_t)(nt * 4 + f) * (a.KF / 2)) * kFragBytes;
                src_step[j] = kFragBytes;
            }
        } else {
            const int fx = f - L::kWFrags;
            const int rb = fx >> 1, kf = fx & 1;
            src[j] = a.x_tiled + ((int64_t)(mt * 8 + rb) * a.KF + kf) * kFragBytes;
            src_step[j] = 2 * kFragBytes;
        }
        src[j] += lane * 16;
    }

    auto issue = [&](int stage) {
        uint8_t *buf = lds + (stage % kStages) * L::kBytes;
#pragma unroll
        for (int j = 0; j < L::kFragsPerWave; ++j) {
            const int f = wave * L::kFragsPerWave + j;
            lds_dma_16(src[j] + (int64_t)stage * src_step[j], buf + f * kFragBytes);
        }
    };

    v16i acc[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][j][r] = 0;

    issue(0);
    if (stages > 1) issue(1);

    for (int s = 0; s < stages; ++s) {
        if (s + 1 < stages) __builtin_amdgcn_s_waitcnt(0x0F70 | L::kFragsPerWave);  // vmcnt <= one stage
        else __builtin_amdgcn_s_waitcnt(0x0F70);                                     // vmcnt == 0
        __builtin_amdgcn_s_barrier();
        if (s + 2 < stages) issue(s + 2);

        const uint8_t *buf = lds + (s % kStages) * L::kBytes;
        const uint8_t *xb = buf + L::kWFrags * kFragBytes + lane * 16;
        if (BITS == 8) {
#pragma unroll
            for (int kf = 0; kf < 2; ++kf) {
                v4i wa[2], xbv[4];
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    wa[t] = *reinterpret_cast<const v4i *>(buf + ((wn * 2 + t) * 2 + kf) * kFragBytes + lane * 16);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    xbv[j] = *reinterpret_cast<const v4i *>(xb + ((wm * 4 + j) * 2 + kf) * kFragBytes);
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[t][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wa[t], xbv[j], acc[t][j], 0, 0, 0);
            }
        } else {
            v4i packed[2];
#pragma unroll
            for (int t = 0; t < 2; ++t)
                packed[t] = *reinterpret_cast<const v4i *>(buf + (wn * 2 + t) * kFragBytes + lane * 16);
#pragma unroll
            for (int kf = 0; kf < 2; ++kf) {
                v4i wa[2], xbv[4];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const uint32_t v0 = (uint32_t)packed[t][2 * kf], v1 = (uint32_t)packed[t][2 * kf + 1];
                    wa[t][0] = (int)((v0 << 4) & 0xF0F0F0F0u);
                    wa[t][1] = (int)(v0 & 0xF0F0F0F0u);
                    wa[t][2] = (int)((v1 << 4) & 0xF0F0F0F0u);
                    wa[t][3] = (int)(v1 & 0xF0F0F0F0u);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    xbv[j] = *reinterpret_cast<const v4i *>(xb + ((wm * 4 + j) * 2 + kf) * kFragBytes);
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[t][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wa[t], xbv[j], acc[t][j], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: registers -> Y --------------------------------------------------------
    // Lane (c = lane % 32, h = lane / 32) of MFMA tile (t, j) holds, in register r, token
    // m0 + 32 j + c and channel n0 + 16 (r / 4) + 8 h + 4 t + r % 4.
    const int c = lane & 31, h = lane >> 5;
    const int64_t m_base = (int64_t)mt * kTileM + wm * 128 + c;
    const int64_t n_base = (int64_t)nt * kTileN + wn * 64 + 8 * h;
    const bool vec_ok = (a.N % 8) == 0;

    float sx[4];
    if (OUT != QC_OUT_I32_ACC) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t m = m_base + 32 * j;
            sx[j] = m < a.M ? a.x_scale[m] : 0.0f;
        }
    }

#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int64_t n0 = n_base + 16 * g;
        if (n0 >= a.N) continue;
        const bool full = vec_ok && n0 + 8 <= a.N;
        float sw[8], bs[8];
        if (OUT != QC_OUT_I32_ACC) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool in = n0 + e < a.N;
                sw[e] = in ? a.w_scale[n0 + e] : 0.0f;
                if (BITS == 4) sw[e] *= 0.0625f;  // operands carried codes times 16
                bs[e] = (in && a.bias) ? a.bias[n0 + e] : 0.0f;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t m = m_base + 32 * j;
            if (m >= a.M) continue;
            int raw[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) raw[e] = acc[e >> 2][j][4 * g + (e & 3)];
            if (OUT == QC_OUT_I32_ACC) {
                int32_t *y = reinterpret_cast<int32_t *>(a.Y) + m * a.N + n0;
#pragma unroll
                for (int e = 0; e < 8; ++e) if (BITS == 4) raw[e] >>= 4;  // exact: multiples of 16
                if (full) {
                    reinterpret_cast<int4 *>(y)[0] = make_int4(raw[0], raw[1], raw[2], raw[3]);
                    reinterpret_cast<int4 *>(y)[1] = make_int4(raw[4], raw[5], raw[6], raw[7]);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) if (n0 + e < a.N) y[e] = raw[e];
                }
            } else {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float y = fmaf((float)raw[e] * sx[j], sw[e], bs[e]);
                    if (EPI == QC_EPI_GELU_TANH) y = gelu_tanh_f(y);
                    else if (EPI == QC_EPI_GELU_ERF) y = gelu_erf_f(y);
                    v[e] = y;
                }
                if (OUT == QC_OUT_F32) {
                    float *y = reinterpret_cast<float *>(a.Y) + m * a.N + n0;
                    if (full) {
                        reinterpret_cast<float4 *>(y)[0] = make_float4(v[0], v[1], v[2], v[3]);
                        reinterpret_cast<float4 *>(y)[1] = make_float4(v[4], v[5], v[6], v[7]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) if (n0 + e < a.N) y[e] = v[e];
                    }
                } else {
                    uint16_t *y = reinterpret_cast<uint16_t *>(a.Y) + m * a.N + n0;
                    if (full) {
                        *reinterpret_cast<uint4 *>(y) =
                            make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                       pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (n0 + e < a.N) y[e] = (uint16_t)(pack_bf16x2(v[e], 0.0f) & 0xffffu);
                    }
                }
            }
        }
    }
}

template <int BITS, int OUT, int EPI>
hipError_t launch_variant(const GemmArgs &args, hipStream_t stream) {
    using L = StageLayout<BITS>;
    constexpr int kLds = kStages * L::kBytes;
    static bool configured = false;  // a per-function attribute; setting it twice is harmless
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<BITS, OUT, EPI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int blocks = args.m_tiles * args.n_tiles;
    gemm_kernel<BITS, OUT, EPI><<<dim3((unsigned)blocks), dim3(kThreads), kLds, stream>>>(args);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_bits(const GemmArgs &args, qc_epilogue epi, qc_out ydt, hipStream_t stream) {
    if (ydt == QC_OUT_I32_ACC) return launch_variant<BITS, QC_OUT_I32_ACC, QC_EPI_NONE>(args, stream);
#define QC_EPI_CASE(O)                                                                        \
    switch (epi) {                                                                            \
        case QC_EPI_NONE: return launch_variant<BITS, O, QC_EPI_NONE>(args, stream);          \
        case QC_EPI_GELU_TANH: return launch_variant<BITS, O, QC_EPI_GELU_TANH>(args, stream);\
        default: return launch_variant<BITS, O, QC_EPI_GELU_ERF>(args, stream);               \
    }
    if (ydt == QC_OUT_F32) { QC_EPI_CASE(QC_OUT_F32) }
    QC_EPI_CASE(QC_OUT_BF16)
#undef QC_EPI_CASE
}

}  // namespace

hipError_t launch_gemm(const uint8_t *x_tiled, const float *x_scale, const uint8_t *w_packed,
                       const float *w_scale, const float *bias, void *Y, int64_t M, int64_t N,
                       int64_t K, int bits, qc_epilogue epi, qc_out ydt, hipStream_t stream) {
    GemmArgs args;
    args.x_tiled = x_tiled;
    args.x_scale = x_scale;
    args.w_codes = w_packed + kPackedHeaderBytes;
    args.w_scale = w_scale;
    args.bias = bias;
    args.Y = Y;
    args.M = M;
    args.N = N;
    args.KF = (int)(round_up(K, kKAlign) / kFragK);
    args.m_tiles = (int)(round_up(M, kTileM) / kTileM);
    args.n_tiles = (int)(round_up(N, kTileN) / kTileN);
    return bits == 8 ? launch_bits<8>(args, epi, ydt, stream) : launch_bits<4>(args, epi, ydt, stream);
}

}  // namespace qc
