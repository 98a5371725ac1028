// Integer GEMM with fused dequantize / bias / GELU epilogue (Section 4.1 "Hardware
// Implementation": the DiT linears as low-bit GEMMs with quantization fused around them).
//
//   acc[m, n] = sum_k qx[m, k] * qw[n, k]          exact, int32, v_mfma_i32_16x16x64_i8
//   Y[m, n]   = act(acc * sx[m] * sw[n] + bias[n])
//
// Two kernels share the wavefront tile, the operand formats and the epilogue: gemm_kernel
// streams its weight tile through a ring in LDS and takes any K; gemm_resident_kernel (further
// down) keeps a whole weight tile in LDS and is taken for short reductions on large problems.
//
// gemm_kernel: block tile 256 tokens x 128 channels, 4 wavefronts stacked along the tokens, each
// 64 x 128 = 4 x 8 MFMA tiles (128 accumulator registers), two blocks per CU so that one
// block's epilogue overlaps the other's MFMA loop.  Operands arrive pre-arranged as 1 KiB
// MFMA fragments (see qc_internal.h).  The weight tile, which all four wavefronts use, goes
// HBM -> LDS by linear direct-to-LDS copies through a 3-deep ring of 64-k stages and is read
// back 16 B/lane, conflict free; the activation fragments are private to a wavefront and go
// HBM -> registers directly (LDS writes are the scarce resource: about 64 B/clk/CU against
// 256 B/clk/CU for reads).  Inside a stage the weight reads of the second half of the channels
// are in flight under the MFMAs of the first half.  Tokens are the MFMA "A" operand (rows of the
// result tile, four per lane) and channels the "B" operand (columns = lanes); the weight row
// permutation makes a lane's eight tiles eight consecutive channels, so 16 lanes store 128
// consecutive channels of one token at a time.  The 16x16x64 form of the MFMA is used because
// the chip holds a higher clock on it than on the 32x32x32 form under its power cap (measured:
// 4.1 against 3.4 POP/s on random operands, registers only).  The output is written with
// non-temporal stores: it is not read again by this kernel and would otherwise push the operand
// panels out of the L2.
#include <type_traits>

#include "qc_internal.h"

namespace qc {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kStages = 3;   // LDS ring of weight stages (4 and 6 were measured: 1.5 % and 3 % slower)
constexpr int kXSlots = 3;   // register ring of activation stages

template <int BITS>
struct StageLayout {
    // Only the weight tile goes through LDS (all four wavefronts use all of it).  1 KiB pieces
    // per 64-k stage: 8 bit one fragment per block of 16 channels; 4 bit one nibble unit per
    // two such blocks.
    static constexpr int kWFrags = BITS == 8 ? kTileN / kFragRows : kTileN / kFragRows / 2;
    static constexpr int kBytes = kWFrags * kFragBytes;
    static constexpr int kFragsPerWave = kWFrags / 4;
    static_assert(kWFrags % 4 == 0, "fragments must split evenly over 4 wavefronts");
};

struct GemmArgs {
    const uint8_t *x_tiled;
    const float *x_scale;   // Mp entries (padded), 16 B aligned
    const float *x_corr;    // asymmetric activations only: per token code shift - zero point, Mp entries
    const int32_t *w_rowsum;  // asymmetric activations only: per channel sum of the weight codes
    const uint8_t *w_codes;
    const float *w_scale;
    const float *bias;
    void *Y;
    int64_t M, N;
    int KF;         // 64-k stages (Kp / 64)
    int m_tiles, n_tiles;
    int group_m;    // token tiles per patch of the block -> tile map (ring kernel)
    bool resident;  // run the kernel that keeps the weight tile in LDS
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
    const float t = y * fmaf(c2, y * y, c1);
    return y * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}

// 0.5 y (1 + erf(y / sqrt 2)) with erfc(x) = t (a1 + t (a2 + .. a5 t)) exp(-x^2), t = 1 / (1 + p x)
// for x >= 0 (Abramowitz and Stegun 7.1.26, absolute error below 1.5e-7) and erf odd.  For
// negative y the product form keeps the small result's relative accuracy.  Far fewer registers
// than the math library's erff, which matters next to 128 live accumulators.
__device__ inline float gelu_erf_f(float y) {
    const float x = fabsf(y) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float q = p * t * __builtin_amdgcn_exp2f(x * x * -1.4426950408889634f);  // erfc(x)
    const float gate = y >= 0.0f ? 2.0f - q : q;
    return 0.5f * y * gate;
}

// two floats -> two bf16 (round to nearest even), one v_cvt_pk_bf16_f32
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    const f2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf2));
}

// Map the launch's block index to a tile so that the blocks resident on one XCD at a time
// (block b runs on XCD b % 8) work on a compact 8 x 8 patch of tiles and share its operand
// panels through that XCD's L2.
__device__ inline void tile_of_block(int b, int nblocks, int m_tiles, int n_tiles, int group_m,
                                     int &mt, int &nt) {
    const int xcd = b % 8, slot = b / 8;
    const int per = nblocks / 8, extra = nblocks % 8;
    const int v = xcd * per + (xcd < extra ? xcd : extra) + slot;  // blocks of one XCD are consecutive
    const int kGroupM = group_m;
    const int per_group = kGroupM * n_tiles;
    const int g = v / per_group, r = v % per_group;
    const int m0 = g * kGroupM;
    const int gm = (m_tiles - m0) < kGroupM ? (m_tiles - m0) : kGroupM;
    mt = m0 + r % gm;
    nt = r / gm;
}

// vmcnt(n) with the other counters left unconstrained (gfx9 encoding: bits 3:0 and 15:14, n < 64)
#define QC_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// Epilogue of one wavefront's 64 x 128 tile: registers -> Y.  Lane (c = lane % 16, h = lane / 16)
// of MFMA tile (i, t) holds, in register r, token m_wave + 16 i + 4 h + r and channel
// 128 nt + 8 c + t.  sx64 / cx64: the tile's 64 token scales / corrections, lds_sw / lds_bs /
// lds_rs: the channel tile's 128 scales, biases and code sums, all in LDS.
template <int BITS, int OUT, int EPI, bool ASYM>
__device__ __forceinline__ void store_wave_tile(v4i (&acc)[4][8], const GemmArgs &a, int64_t m_wave, int nt,
                                                int lane, const float *sx64, const float *cx64,
                                                const float *lds_sw, const float *lds_bs, const float *lds_rs) {
    const int c = lane & 15, h = lane >> 4;
    const int64_t n0 = (int64_t)nt * kTileN + 8 * c;
    const int64_t m0 = m_wave + 4 * h;
    constexpr int kOutBytes = OUT == QC_OUT_BF16 ? 2 : 4;
    constexpr int kVecChannels = 16 / kOutBytes;  // channels in one 16 B store
    const bool interior = m_wave + kWaveM <= a.M && (int64_t)(nt + 1) * kTileN <= a.N &&
                          (a.N % kVecChannels) == 0;  // uniform over the wavefront
    char *const y_wave = reinterpret_cast<char *>(a.Y) + (m_wave * a.N + (int64_t)nt * kTileN) * kOutBytes;
    const uint32_t lane_off = (uint32_t)((4 * h * a.N + 8 * c) * kOutBytes);  // N <= 2^26

    auto write_tile = [&](auto checked_tag) {
        constexpr bool CHECKED = decltype(checked_tag)::value;
        if (CHECKED && n0 >= a.N) return;
        bool vec[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) vec[j] = !CHECKED || ((a.N % 4) == 0 && n0 + 4 * j + 4 <= a.N);
        const bool vec8 = !CHECKED || (vec[1] && (a.N % 8) == 0);

        float sw[8], bs[8], rs[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) sw[t] = bs[t] = rs[t] = 0.0f;
        if (OUT != QC_OUT_I32_ACC) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float4 s4 = *reinterpret_cast<const float4 *>(lds_sw + 8 * c + 4 * j);
                const float4 b4 = *reinterpret_cast<const float4 *>(lds_bs + 8 * c + 4 * j);
                sw[4 * j + 0] = s4.x; sw[4 * j + 1] = s4.y; sw[4 * j + 2] = s4.z; sw[4 * j + 3] = s4.w;
                bs[4 * j + 0] = b4.x; bs[4 * j + 1] = b4.y; bs[4 * j + 2] = b4.z; bs[4 * j + 3] = b4.w;
                if (ASYM) {
                    const float4 r4 = *reinterpret_cast<const float4 *>(lds_rs + 8 * c + 4 * j);
                    rs[4 * j + 0] = r4.x; rs[4 * j + 1] = r4.y; rs[4 * j + 2] = r4.z; rs[4 * j + 3] = r4.w;
                }
            }
        }

#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t m4 = m0 + 16 * i;
            if (CHECKED && m4 >= a.M) continue;
            float sx[4] = {0.f, 0.f, 0.f, 0.f}, cx[4] = {0.f, 0.f, 0.f, 0.f};
            if (OUT != QC_OUT_I32_ACC) {
                const float4 x4 = *reinterpret_cast<const float4 *>(sx64 + 16 * i + 4 * h);
                sx[0] = x4.x; sx[1] = x4.y; sx[2] = x4.z; sx[3] = x4.w;
                if (ASYM) {
                    const float4 c4 = *reinterpret_cast<const float4 *>(cx64 + 16 * i + 4 * h);
                    cx[0] = c4.x; cx[1] = c4.y; cx[2] = c4.z; cx[3] = c4.w;
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (CHECKED && m4 + q >= a.M) continue;
                int raw[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) raw[t] = acc[i][t][q];
                char *const y_row = y_wave + (int64_t)(16 * i + q) * a.N * kOutBytes + lane_off;
                if (OUT == QC_OUT_I32_ACC) {
                    int32_t *y = reinterpret_cast<int32_t *>(y_row);
                    if (BITS == 4) {
#pragma unroll
                        for (int t = 0; t < 8; ++t) raw[t] >>= 4;  // exact: multiples of 16
                    }
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (vec[j]) {
                            __builtin_nontemporal_store(v4i{raw[4 * j], raw[4 * j + 1], raw[4 * j + 2], raw[4 * j + 3]},
                                                        reinterpret_cast<v4i *>(y + 4 * j));
                        } else {
#pragma unroll
                            for (int t = 4 * j; t < 4 * j + 4; ++t) if (n0 + t < a.N) y[t] = raw[t];
                        }
                    }
                } else {
                    float v[8];
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        float af = (float)raw[t];
                        if (ASYM) af = fmaf(cx[q], rs[t], af);
                        float y = fmaf(af * sx[q], sw[t], bs[t]);
                        if (EPI == QC_EPI_GELU_TANH) y = gelu_tanh_f(y);
                        else if (EPI == QC_EPI_GELU_ERF) y = gelu_erf_f(y);
                        v[t] = y;
                    }
                    if (OUT == QC_OUT_F32) {
                        float *y = reinterpret_cast<float *>(y_row);
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            if (vec[j]) {
                                __builtin_nontemporal_store(f4{v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]},
                                                            reinterpret_cast<f4 *>(y + 4 * j));
                            } else {
#pragma unroll
                                for (int t = 4 * j; t < 4 * j + 4; ++t) if (n0 + t < a.N) y[t] = v[t];
                            }
                        }
                    } else {
                        uint16_t *y = reinterpret_cast<uint16_t *>(y_row);
                        uint32_t pk[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) pk[j] = pack_bf16x2(v[2 * j], v[2 * j + 1]);
                        if (vec8) {
                            __builtin_nontemporal_store(u4{pk[0], pk[1], pk[2], pk[3]}, reinterpret_cast<u4 *>(y));
                        } else {
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                if (vec[j]) {
                                    __builtin_nontemporal_store(u2{pk[2 * j], pk[2 * j + 1]},
                                                                reinterpret_cast<u2 *>(y + 4 * j));
                                } else {
#pragma unroll
                                    for (int t = 4 * j; t < 4 * j + 4; ++t)
                                        if (n0 + t < a.N)
                                            y[t] = (uint16_t)(t % 2 ? pk[t / 2] >> 16 : pk[t / 2] & 0xffffu);
                                }
                            }
                        }
                    }
                }
            }
        }
    };
    if (interior) write_tile(std::false_type{});
    else write_tile(std::true_type{});
}

// ASYM: the activation codes are the unsigned codes of the asymmetric quantizer minus a shift h
// (128 for 8-bit codes, else 0; Section 3.1 Eq. (3)-(4) as printed).  With c[m] = h - z[m] the dequantized activation
// is sx (code + c), so the epilogue adds c[m] * sum_k qw[n, k] to the accumulator.
template <int BITS, int OUT, int EPI, bool ASYM>
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmArgs a) {
    using L = StageLayout<BITS>;
    constexpr int FPW = L::kFragsPerWave;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int mt, nt;
    tile_of_block(blockIdx.x, gridDim.x, a.m_tiles, a.n_tiles, a.group_m, mt, nt);

    const int stages = a.KF;
    // The epilogue's scales and bias are fetched now (one value per thread) and handed round
    // through LDS after the main loop, so that the epilogue does not start with a chain of L2
    // round trips.
    float *lds_sx = reinterpret_cast<float *>(lds + kStages * L::kBytes);  // 256 token scales
    float *lds_sw = lds_sx + kTileM;                                       // 128 channel scales
    float *lds_bs = lds_sw + kTileN;                                       // 128 biases
    float *lds_cx = lds_bs + kTileN;                                       // ASYM: 256 corrections
    float *lds_rs = lds_cx + kTileM;                                       // ASYM: 128 code sums
    float my_sx = 0.0f, my_sw = 0.0f, my_bs = 0.0f, my_cx = 0.0f, my_rs = 0.0f;
    if (OUT != QC_OUT_I32_ACC) {
        my_sx = a.x_scale[(int64_t)mt * kTileM + threadIdx.x];  // x_scale is padded to Mp
        if (ASYM) my_cx = a.x_corr[(int64_t)mt * kTileM + threadIdx.x];
        const int64_t n = (int64_t)nt * kTileN + threadIdx.x;
        if (threadIdx.x < kTileN && n < a.N) {
            my_sw = a.w_scale[n];
            if (BITS == 4) my_sw *= 0.0625f;  // operands carry codes times 16
            if (a.bias) my_bs = a.bias[n];
            if (ASYM) {
                my_rs = (float)a.w_rowsum[n];  // |sum| <= 127 K < 2^24: exact
                if (BITS == 4) my_rs *= 16.0f;
            }
        }
    }
    // The pieces of the weight stage tile this wavefront copies HBM -> LDS, at stage 0 (a
    // stage tile is contiguous in memory).
    const uint8_t *const wsrc = a.w_codes + (int64_t)nt * a.KF * L::kBytes + wave * FPW * kFragBytes + lane * 16;
    // copy the weight pieces of K stage `stage` into ring buffer `ring % 3`
    auto issue_w = [&](int stage, int ring) {
        uint8_t *buf = lds + (ring % kStages) * L::kBytes;
#pragma unroll
        for (int j = 0; j < FPW; ++j)
            lds_dma_16(wsrc + (int64_t)stage * L::kBytes + j * kFragBytes, buf + (wave * FPW + j) * kFragBytes);
    };

    // Activation fragments are private to a wavefront (its 64 tokens), so they skip LDS:
    // HBM -> registers, 16 B per lane, two stages ahead.  xq[slot][i]: tokens 16 i .. of the
    // stage held in `slot`.  Loads and LDS reads are asm so that they stay
    // in flight across loop iterations under explicit s_waitcnt counts; each wait names the
    // registers it makes valid, which orders the MFMAs that consume them behind it.
    v4i xq[kXSlots][4];
    const uint8_t *const xsrc = a.x_tiled + ((int64_t)(mt * (kTileM / kWaveM) + wave) * a.KF) * (4 * kFragBytes) + lane * 16;

#define QC_GLOBAL_LOAD(dst, ptr, imm) \
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(dst) : "v"(ptr), "n"(imm) : "memory")
#define QC_ISSUE_X(stage, SLOT)                                              \
    do {                                                                     \
        const uint8_t *p_ = xsrc + (int64_t)(stage) * (4 * kFragBytes);      \
        QC_GLOBAL_LOAD(xq[SLOT][0], p_, 0);                                  \
        QC_GLOBAL_LOAD(xq[SLOT][1], p_, kFragBytes);                         \
        QC_GLOBAL_LOAD(xq[SLOT][2], p_, 2 * kFragBytes);                     \
        QC_GLOBAL_LOAD(xq[SLOT][3], p_, 3 * kFragBytes);                     \
    } while (0)
#define QC_WAIT_X(n, SLOT)                                                                    \
    asm volatile("s_waitcnt vmcnt(" #n ")" : "+v"(xq[SLOT][0]), "+v"(xq[SLOT][1]),            \
                 "+v"(xq[SLOT][2]), "+v"(xq[SLOT][3]))

    // LDS -> registers for the weight fragments.
    //   wr[h][t]: 16-channel block 4 h + t (8 bit);  wr[0][u]: nibble unit of blocks 2 u, 2 u + 1 (4 bit)
    v4i wr[2][4];
    const uint32_t lds_lane = (uint32_t)(uintptr_t)lds + lane * 16;  // LDS byte address of this lane
#define QC_DS_READ(dst, addr, imm) \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(imm))
#define QC_READ_W(stage, H)                                                          \
    do {                                                                             \
        const uint32_t base_ = lds_lane + ((stage) % kStages) * L::kBytes;           \
        if (BITS == 8) {                                                             \
            QC_DS_READ(wr[H][0], base_, (4 * H + 0) * kFragBytes);                   \
            QC_DS_READ(wr[H][1], base_, (4 * H + 1) * kFragBytes);                   \
            QC_DS_READ(wr[H][2], base_, (4 * H + 2) * kFragBytes);                   \
            QC_DS_READ(wr[H][3], base_, (4 * H + 3) * kFragBytes);                   \
        } else if (H == 0) {                                                        \
            QC_DS_READ(wr[0][0], base_, 0 * kFragBytes);                             \
            QC_DS_READ(wr[0][1], base_, 1 * kFragBytes);                             \
            QC_DS_READ(wr[0][2], base_, 2 * kFragBytes);                             \
            QC_DS_READ(wr[0][3], base_, 3 * kFragBytes);                             \
        }                                                                            \
    } while (0)
#define QC_WAIT_W(n, H) \
    asm volatile("s_waitcnt lgkmcnt(" #n ")" : "+v"(wr[H][0]), "+v"(wr[H][1]), "+v"(wr[H][2]), "+v"(wr[H][3]))

    v4i acc[4][8];   // [16-token block][16-channel block]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[i][t] = v4i{0, 0, 0, 0};

    // 4 bit: nibbles -> int8 operand dwords holding 16 * code, channel blocks 4 h .. 4 h + 3
    auto unpack = [&](v4i (&w)[4], int h) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const v4i unit = wr[0][2 * h + t / 2];
            const uint32_t v0 = (uint32_t)unit[2 * (t % 2)], v1 = (uint32_t)unit[2 * (t % 2) + 1];
            w[t][0] = (int)((v0 << 4) & 0xF0F0F0F0u);
            w[t][1] = (int)(v0 & 0xF0F0F0F0u);
            w[t][2] = (int)((v1 << 4) & 0xF0F0F0F0u);
            w[t][3] = (int)(v1 & 0xF0F0F0F0u);
        }
    };

    // One 64-k stage.  SLOT = stage % 3 and NEXT2 = (stage + 2) % 3 are literal constants (the
    // loop is unrolled by three) so the activation ring stays in fixed registers.
    // VMEM operations complete in issue order; with D = kStages the issue order per wavefront is
    //   W(0) .. W(D-3) X(0) W(D-2) X(1) W(D-1), then in stage s: X(s+2), W(s+D)
    // i.e. from X(0) on an X and a W alternate.  X(s+2) goes out after the wait for X(s), among
    // the first MFMAs of the stage, so at that wait W X(s+1) W are behind X(s) (2 FPW + 4
    // operations).  At the wait for W(s+1) in the middle of the stage, D - 1 activation stages
    // and D - 2 weight stages are behind it, once the stage is past the first D - 3, whose
    // weights are waited for before the loop.  (A deeper weight ring buys nothing: the loop is
    // not waiting for the weights.)  Past the end
    // of K the stage index is clamped to the last stage: those copies repeat data that is not
    // used again (they hit in cache), which keeps the instruction stream and the wait counts
    // uniform.
    constexpr int kWBehind = 4 * (kStages - 1) + FPW * (kStages - 2);
    static_assert(kStages >= 3 && kWBehind < 64, "vmcnt is a 6-bit counter");
    const int last = stages - 1;
#define QC_CLAMP(st) ((st) < last ? (st) : last)
    // The sixteen MFMAs of a half stage (4 token blocks x 4 channel blocks) are independent, so
    // their order is free.  8 bit: token block outer.  4 bit: channel block outer, so that the
    // MFMAs that share an unpacked weight fragment follow each other.
#define QC_MFMA_LOOPS                                                                           \
    _Pragma("unroll") for (int o_ = 0; o_ < 16; ++o_)                                           \
        for (int i = BITS == 8 ? o_ / 4 : o_ % 4, t = BITS == 8 ? o_ % 4 : o_ / 4, once_ = 1; once_; once_ = 0)
#define QC_STAGE(s, SLOT, NEXT2)                                                               \
    do {                                                                                       \
        QC_WAIT_W(0, 0);                                  /* channel half 0 of W(s) is here */ \
        if (BITS == 8) QC_WAIT_X(8, SLOT); else QC_WAIT_X(6, SLOT);        /* X(s) is here */  \
        v4i w4a[4], w4b[4];                                                                    \
        if (BITS == 4) unpack(w4a, 0);                                                         \
        /* issued here, not before the waits, so that the loads go out under the MFMAs */      \
        QC_ISSUE_X(QC_CLAMP((s) + 2), NEXT2);                                                  \
        QC_READ_W((s), 1);        /* channel half 1: lands under the MFMAs of channel half 0 */ \
        QC_MFMA_LOOPS                                                                          \
                acc[i][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(                             \
                    xq[SLOT][i], BITS == 8 ? wr[0][t] : w4a[t], acc[i][t], 0, 0, 0);           \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        QC_WAIT_VMCNT(kWBehind);                                        /* W(s+1) has landed */\
        /* this wavefront's reads of W(s) are done ... */                                      \
        if (BITS == 8) QC_WAIT_W(0, 1);                                                        \
        __builtin_amdgcn_s_barrier(); /* ... and everybody else's: ring buffer s % 3 is free */\
        asm volatile("" ::: "memory");                                                         \
        if (BITS == 4) unpack(w4b, 1);   /* before the reads below overwrite the nibbles */     \
        issue_w(QC_CLAMP((s) + kStages), (s) + kStages);                                       \
        /* after the last stage this reads data that is not used */                            \
        QC_READ_W((s) + 1, 0);                                                                 \
        QC_MFMA_LOOPS                                                                          \
                acc[i][4 + t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(                         \
                    xq[SLOT][i], BITS == 8 ? wr[1][t] : w4b[t], acc[i][4 + t], 0, 0, 0);       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
    } while (0)

    // ---- main loop -------------------------------------------------------------------
#pragma unroll
    for (int j = 0; j < kStages - 2; ++j) issue_w(QC_CLAMP(j), j);
    QC_ISSUE_X(0, 0);
    issue_w(QC_CLAMP(kStages - 2), kStages - 2);
    QC_ISSUE_X(QC_CLAMP(1), 1);
    issue_w(QC_CLAMP(kStages - 1), kStages - 1);
    // W(0) .. W(kStages - 3) have landed: behind them are X(0) W X(1) W
    QC_WAIT_VMCNT(8 + 2 * FPW);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    QC_READ_W(0, 0);

    for (int s = 0; s < stages; s += 3) {
        QC_STAGE(s, 0, 2);
        QC_STAGE(s + 1, 1, 0);
        QC_STAGE(s + 2, 2, 1);
    }
    // drain everything still in flight before the registers are reused
    QC_WAIT_W(0, 0);
    QC_WAIT_X(0, 0);
    QC_WAIT_X(0, 1);
    QC_WAIT_X(0, 2);
#undef QC_MFMA_LOOPS
#undef QC_CLAMP
#undef QC_STAGE
#undef QC_WAIT_W
#undef QC_READ_W
#undef QC_DS_READ
#undef QC_WAIT_X
#undef QC_ISSUE_X
#undef QC_GLOBAL_LOAD

    // park the scales (fetched at kernel start, long since arrived) where every lane can pick
    // the ones of its tokens and channels
    if (OUT != QC_OUT_I32_ACC) {
        lds_sx[threadIdx.x] = my_sx;
        if (threadIdx.x < kTileN) { lds_sw[threadIdx.x] = my_sw; lds_bs[threadIdx.x] = my_bs; }
        if (ASYM) {
            lds_cx[threadIdx.x] = my_cx;
            if (threadIdx.x < kTileN) lds_rs[threadIdx.x] = my_rs;
        }
        __syncthreads();
    }

    // ---- epilogue: registers -> Y --------------------------------------------------------
    store_wave_tile<BITS, OUT, EPI, ASYM>(acc, a, (int64_t)mt * kTileM + wave * kWaveM, nt, lane,
                                           lds_sx + wave * kWaveM, lds_cx + wave * kWaveM, lds_sw, lds_bs, lds_rs);
}

// ---- the same GEMM with the weight tile resident in LDS (short reductions) ---------------------
// When a whole channel tile of the weights (128 channels x Kp) fits in LDS beside the scales, a
// block of eight wavefronts, one per CU, loads it once and then every wavefront walks token tiles
// of 64 on its own: no weight copies and no block barriers inside the reduction, which is what
// the ring version above spends 5-9 % of its time on when K is 1152.  Work is cut into rounds of
// (channel tile, 512 tokens = one 64-token tile per wavefront) and dealt to the blocks by the
// static schedule of resident_rounds() (qc_internal.h): a block changes its weight tile once or
// twice per launch, and the blocks of an XCD read the same few token chunks at the same time.
constexpr int kResThreads = 512;
constexpr int kResWaves = kResThreads / 64;
static_assert(kRoundTokens == kResWaves * kWaveM, "a round is one 64-token tile per wavefront");

// LDS of the resident kernel, a fixed layout whatever K is (one block per CU has the CU's 160 KiB
// to itself, and a static size needs no launch attribute): the weight tile, 128 channel scales,
// biases and code sums, 64 token scales and corrections per wavefront.
constexpr int kResWeightBytes = 18 * 8192;   // 128 channels x 1152 k of 8-bit codes, x 2304 k of 4-bit ones
constexpr int kResLdsBytes = kResWeightBytes + 3 * kTileN * (int)sizeof(float) + 2 * kResWaves * kWaveM * (int)sizeof(float);
static_assert(kResLdsBytes <= 160 * 1024, "more than the LDS of a CU");

template <int BITS, int OUT, int EPI, bool ASYM>
__global__ __launch_bounds__(kResThreads, 1) void gemm_resident_kernel(GemmArgs a) {
    using L = StageLayout<BITS>;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[kResLdsBytes];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int stages = a.KF;

    float *lds_sw = reinterpret_cast<float *>(lds + kResWeightBytes);      // 128 channel scales
    float *lds_bs = lds_sw + kTileN;                                       // 128 biases
    float *lds_rs = lds_bs + kTileN;                                       // ASYM: 128 code sums
    float *lds_sx = lds_rs + kTileN + wave * kWaveM;                       // this wavefront's 64 token scales
    float *lds_cx = lds_sx + kResWaves * kWaveM;                           // ASYM: its 64 corrections

    // this block's XCD (block b runs on XCD b % 8), its place there and the XCD's token chunks
    const ResidentXcd xs = resident_xcd((int)blockIdx.x, (int)gridDim.x, resident_chunks(a.m_tiles));
    const int slot = xs.slot, nbx = xs.blocks, c_lo = xs.c_lo, c_hi = xs.c_hi;
    const int wave_tiles = a.m_tiles * (kTileM / kWaveM);          // 64-token tiles inside Mp

    v4i xq[kXSlots][4];
    v4i wr[2][4];
    const uint32_t lds_lane = (uint32_t)(uintptr_t)lds + lane * 16;

#define QC_GLOBAL_LOAD(dst, ptr, imm) \
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(dst) : "v"(ptr), "n"(imm) : "memory")
#define QC_ISSUE_X(ptr, SLOT)                                                \
    do {                                                                     \
        const uint8_t *p_ = (ptr);                                           \
        QC_GLOBAL_LOAD(xq[SLOT][0], p_, 0);                                  \
        QC_GLOBAL_LOAD(xq[SLOT][1], p_, kFragBytes);                         \
        QC_GLOBAL_LOAD(xq[SLOT][2], p_, 2 * kFragBytes);                     \
        QC_GLOBAL_LOAD(xq[SLOT][3], p_, 3 * kFragBytes);                     \
    } while (0)
#define QC_WAIT_X(n, SLOT)                                                                    \
    asm volatile("s_waitcnt vmcnt(" #n ")" : "+v"(xq[SLOT][0]), "+v"(xq[SLOT][1]),            \
                 "+v"(xq[SLOT][2]), "+v"(xq[SLOT][3]))
#define QC_DS_READ(dst, addr, imm) \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(imm))
#define QC_READ_W(stage, H)                                                          \
    do {                                                                             \
        const uint32_t base_ = lds_lane + (uint32_t)(stage) * L::kBytes;             \
        if (BITS == 8) {                                                             \
            QC_DS_READ(wr[H][0], base_, (4 * H + 0) * kFragBytes);                   \
            QC_DS_READ(wr[H][1], base_, (4 * H + 1) * kFragBytes);                   \
            QC_DS_READ(wr[H][2], base_, (4 * H + 2) * kFragBytes);                   \
            QC_DS_READ(wr[H][3], base_, (4 * H + 3) * kFragBytes);                   \
        } else if (H == 0) {                                                        \
            QC_DS_READ(wr[0][0], base_, 0 * kFragBytes);                             \
            QC_DS_READ(wr[0][1], base_, 1 * kFragBytes);                             \
            QC_DS_READ(wr[0][2], base_, 2 * kFragBytes);                             \
            QC_DS_READ(wr[0][3], base_, 3 * kFragBytes);                             \
        }                                                                            \
    } while (0)
#define QC_WAIT_W(n, H) \
    asm volatile("s_waitcnt lgkmcnt(" #n ")" : "+v"(wr[H][0]), "+v"(wr[H][1]), "+v"(wr[H][2]), "+v"(wr[H][3]))
#define QC_MFMA_LOOPS                                                                           \
    _Pragma("unroll") for (int o_ = 0; o_ < 16; ++o_)                                           \
        for (int i = BITS == 8 ? o_ / 4 : o_ % 4, t = BITS == 8 ? o_ % 4 : o_ / 4, once_ = 1; once_; once_ = 0)
    const int last = stages - 1;
#define QC_CLAMP(st) ((st) < last ? (st) : last)
    // One 64-k stage.  The only vector memory operations of the loop are the activation loads,
    // which complete in issue order: at the wait for X(s), X(s+1) (four loads) is behind it.
    // Past the end of K the stage index is clamped (a repeat that hits in cache), which keeps
    // the instruction stream and the counts uniform.
#define QC_RES_STAGE(s, SLOT, NEXT2)                                                           \
    do {                                                                                       \
        QC_WAIT_W(0, 0);                                  /* channel half 0 of W(s) is here */ \
        QC_WAIT_X(4, SLOT);                                                /* X(s) is here */  \
        v4i w4a[4], w4b[4];                                                                    \
        if (BITS == 4) unpack(w4a, 0);                                                         \
        QC_ISSUE_X(xsrc + (int64_t)QC_CLAMP((s) + 2) * (4 * kFragBytes), NEXT2);               \
        QC_READ_W((s), 1);        /* channel half 1: lands under the MFMAs of channel half 0 */ \
        QC_MFMA_LOOPS                                                                          \
                acc[i][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(                             \
                    xq[SLOT][i], BITS == 8 ? wr[0][t] : w4a[t], acc[i][t], 0, 0, 0);           \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        if (BITS == 8) QC_WAIT_W(0, 1);                                                        \
        if (BITS == 4) unpack(w4b, 1);   /* before the reads below overwrite the nibbles */     \
        QC_READ_W(QC_CLAMP((s) + 1), 0);                                                       \
        QC_MFMA_LOOPS                                                                          \
                acc[i][4 + t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(                         \
                    xq[SLOT][i], BITS == 8 ? wr[1][t] : w4b[t], acc[i][4 + t], 0, 0, 0);       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
    } while (0)

    // the rounds of this block, one after the other
    int pass = 0;
    RoundRange rr = resident_rounds(0, slot, nbx, a.n_tiles, c_hi - c_lo);
    int id = rr.id0 - 1;
    auto advance = [&]() -> bool {   // to the block's next round; false when there is none
        ++id;
        while (id >= rr.id1) {
            ++pass;
            if (pass * nbx >= a.n_tiles) return false;
            rr = resident_rounds(pass, slot, nbx, a.n_tiles, c_hi - c_lo);
            id = rr.id0;
        }
        return true;
    };
    auto x_of_tile = [&](int wt) { return a.x_tiled + ((int64_t)wt * stages) * (4 * kFragBytes) + lane * 16; };

    // Every wavefront runs every round of its block, so that no branch goes round the in-flight
    // loads: a wavefront whose tile lies past the end of the (padded) tokens, which only happens
    // in the last chunk, computes on the last tile instead and stores nothing.
    if (!advance()) return;   // the whole block: no round at all
    int nt = rr.nt_off + id / rr.w;
    int wt = (c_lo + rr.c_off + id % rr.w) * kResWaves + wave;
    int cur_nt = -1;
    bool have;
    do {
        const int wt_ld = wt < wave_tiles ? wt : wave_tiles - 1;   // where this tile's inputs are read
        const uint8_t *const xsrc = x_of_tile(wt_ld);
        if (nt != cur_nt) {   // uniform over the block
            cur_nt = nt;
            __syncthreads();  // every wavefront is done with the previous tile and its scales
            const uint8_t *wsrc = a.w_codes + (int64_t)nt * stages * L::kBytes + lane * 16;
            for (int st = wave; st < stages; st += kResWaves) {
#pragma unroll
                for (int j = 0; j < L::kWFrags; ++j)
                    lds_dma_16(wsrc + (int64_t)st * L::kBytes + j * kFragBytes, lds + st * L::kBytes + j * kFragBytes);
            }
            if (OUT != QC_OUT_I32_ACC && threadIdx.x < kTileN) {
                const int64_t n = (int64_t)nt * kTileN + threadIdx.x;
                float sw = 0.0f, bs = 0.0f, rs = 0.0f;
                if (n < a.N) {
                    sw = a.w_scale[n];
                    if (BITS == 4) sw *= 0.0625f;  // operands carry codes times 16
                    if (a.bias) bs = a.bias[n];
                    if (ASYM) {
                        rs = (float)a.w_rowsum[n];
                        if (BITS == 4) rs *= 16.0f;
                    }
                }
                lds_sw[threadIdx.x] = sw;
                lds_bs[threadIdx.x] = bs;
                if (ASYM) lds_rs[threadIdx.x] = rs;
            }
            QC_WAIT_VMCNT(0);
            __syncthreads();
        }
        const int nt_now = nt, wt_now = wt;
        have = advance();
        if (have) {
            nt = rr.nt_off + id / rr.w;
            wt = (c_lo + rr.c_off + id % rr.w) * kResWaves + wave;
        }

        float my_sx = 0.0f, my_cx = 0.0f;
        if (OUT != QC_OUT_I32_ACC) {
            my_sx = a.x_scale[(int64_t)wt_ld * kWaveM + lane];  // x_scale is padded to Mp
            if (ASYM) my_cx = a.x_corr[(int64_t)wt_ld * kWaveM + lane];
        }
        v4i acc[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int t = 0; t < 8; ++t) acc[i][t] = v4i{0, 0, 0, 0};
        auto unpack = [&](v4i (&w)[4], int h) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const v4i unit = wr[0][2 * h + t / 2];
                const uint32_t v0 = (uint32_t)unit[2 * (t % 2)], v1 = (uint32_t)unit[2 * (t % 2) + 1];
                w[t][0] = (int)((v0 << 4) & 0xF0F0F0F0u);
                w[t][1] = (int)(v0 & 0xF0F0F0F0u);
                w[t][2] = (int)((v1 << 4) & 0xF0F0F0F0u);
                w[t][3] = (int)(v1 & 0xF0F0F0F0u);
            }
        };

        // Nothing of this wavefront is in flight here but the scale loads above and the stores of
        // its previous tile, all older than these loads.
        QC_ISSUE_X(xsrc, 0);
        QC_ISSUE_X(xsrc + (int64_t)QC_CLAMP(1) * (4 * kFragBytes), 1);
        QC_READ_W(0, 0);
        for (int s = 0; s < stages; s += 3) {
            QC_RES_STAGE(s, 0, 2);
            QC_RES_STAGE(s + 1, 1, 0);
            QC_RES_STAGE(s + 2, 2, 1);
        }
        // everything in flight has landed before the registers are used for anything else
        QC_WAIT_W(0, 0);
        QC_WAIT_X(0, 0);
        QC_WAIT_X(0, 1);
        QC_WAIT_X(0, 2);

        if (OUT != QC_OUT_I32_ACC) {   // hand the token scales round inside the wavefront
            lds_sx[lane] = my_sx;
            if (ASYM) lds_cx[lane] = my_cx;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        store_wave_tile<BITS, OUT, EPI, ASYM>(acc, a, (int64_t)wt_now * kWaveM, nt_now, lane, lds_sx, lds_cx,
                                               lds_sw, lds_bs, lds_rs);
    } while (have);
#undef QC_RES_STAGE
#undef QC_CLAMP
#undef QC_MFMA_LOOPS
#undef QC_WAIT_W
#undef QC_READ_W
#undef QC_DS_READ
#undef QC_WAIT_X
#undef QC_ISSUE_X
#undef QC_GLOBAL_LOAD
}

constexpr int kResBlocks = 256;   // one block per CU

template <int BITS, int OUT, int EPI, bool ASYM>
hipError_t launch_variant(const GemmArgs &args, hipStream_t stream) {
    if (args.resident) {
        gemm_resident_kernel<BITS, OUT, EPI, ASYM><<<dim3(kResBlocks), dim3(kResThreads), 0, stream>>>(args);
        return hipGetLastError();
    }
    using L = StageLayout<BITS>;
    constexpr int kLds = kStages * L::kBytes +
                         (kTileM + 2 * kTileN + (ASYM ? kTileM + kTileN : 0)) * (int)sizeof(float);
    // far below the 64 KiB a kernel may use without an attribute, so the first launch of a
    // variant needs no set-up call and can be captured into a graph like any other
    static_assert(kLds <= 64 * 1024, "dynamic LDS beyond the default limit needs an attribute");
    const int blocks = args.m_tiles * args.n_tiles;
    gemm_kernel<BITS, OUT, EPI, ASYM><<<dim3((unsigned)blocks), dim3(kThreads), kLds, stream>>>(args);
    return hipGetLastError();
}

template <int BITS, bool ASYM>
hipError_t launch_bits(const GemmArgs &args, qc_epilogue epi, qc_out ydt, hipStream_t stream) {
    // the raw accumulators are the same kernel with or without a zero point
    if (ydt == QC_OUT_I32_ACC) return launch_variant<BITS, QC_OUT_I32_ACC, QC_EPI_NONE, false>(args, stream);
#define QC_EPI_CASE(O)                                                                        \
    switch (epi) {                                                                            \
        case QC_EPI_NONE: return launch_variant<BITS, O, QC_EPI_NONE, ASYM>(args, stream);         \
        case QC_EPI_GELU_TANH: return launch_variant<BITS, O, QC_EPI_GELU_TANH, ASYM>(args, stream);\
        default: return launch_variant<BITS, O, QC_EPI_GELU_ERF, ASYM>(args, stream);             \
    }
    if (ydt == QC_OUT_F32) { QC_EPI_CASE(QC_OUT_F32) }
    QC_EPI_CASE(QC_OUT_BF16)
#undef QC_EPI_CASE
}

}  // namespace

bool gemm_resident_fits(int64_t K, int bits) {
    const int64_t KF = round_up(K, kKAlign) / kFragK;
    return KF * (bits == 8 ? StageLayout<8>::kBytes : StageLayout<4>::kBytes) <= kResWeightBytes;
}

// The resident kernel is taken when the weight tile fits, the blocks get 6 rounds or more on
// average and the static schedule is within 4 % of an even split.  Measured against the ring
// kernel at K = 1152 (rounds per block: gain): 3.4: -9 %, 4.5: -6 % (the weight tile a block loads
// first and its last, partly idle rounds weigh too much), 6.8: +3.5 %, 9: 0 to +2.5 %, 13.5: +4 %,
// 18: +2 to +9 %, 27 (QKV at M = 131072): 434 -> 420 us, 36 (fc1 + GELU): 650 -> 625 us; K = 384,
// 36 rounds: +10 %.
bool gemm_resident_chosen(int64_t M, int64_t N, int64_t K, int bits) {
    if (!gemm_resident_fits(K, bits)) return false;
    const int m_tiles = (int)(round_up(M, kTileM) / kTileM), n_tiles = (int)(round_up(N, kTileN) / kTileN);
    const int64_t total = (int64_t)n_tiles * resident_chunks(m_tiles);
    if (total < 6 * kResBlocks) return false;
    int most = 0, seen[2] = {-1, -1};   // the XCDs' chunk counts differ by one at most
    for (int xcd = 0; xcd < 8; ++xcd) {
        const ResidentXcd x = resident_xcd(xcd, kResBlocks, resident_chunks(m_tiles));
        const int cx = x.c_hi - x.c_lo;
        if (cx == seen[0] || cx == seen[1]) continue;
        seen[seen[0] < 0 ? 0 : 1] = cx;
        for (int slot = 0; slot < x.blocks; ++slot) {
            const int r = resident_block_rounds(xcd + 8 * slot, kResBlocks, n_tiles, m_tiles, nullptr, 0);
            most = r > most ? r : most;
        }
    }
    return (int64_t)most * kResBlocks * 100 <= total * 104;
}

int gemm_resident_blocks() { return kResBlocks; }

hipError_t launch_gemm(const uint8_t *x_tiled, const float *x_scale, const uint8_t *w_packed,
                       const float *w_scale, const float *bias, void *Y, int64_t M, int64_t N,
                       int64_t K, int bits, qc_epilogue epi, qc_out ydt, const float *x_corr,
                       const int32_t *w_rowsum, GemmKernel which, hipStream_t stream) {
    if (which == kGemmResident && !gemm_resident_fits(K, bits)) return hipErrorInvalidValue;
    GemmArgs args;
    args.resident = which == kGemmResident || (which == kGemmAuto && gemm_resident_chosen(M, N, K, bits));
    args.x_tiled = x_tiled;
    args.x_scale = x_scale;
    args.x_corr = x_corr;
    args.w_rowsum = w_rowsum;
    args.w_codes = w_packed + kPackedHeaderBytes;
    args.w_scale = w_scale;
    args.bias = bias;
    args.Y = Y;
    args.M = M;
    args.N = N;
    args.KF = (int)(round_up(K, kKAlign) / kFragK);
    args.m_tiles = (int)(round_up(M, kTileM) / kTileM);
    args.n_tiles = (int)(round_up(N, kTileN) / kTileN);
    // The blocks resident on one XCD at a time cover a patch of group_m token tiles by as many
    // channel tiles as fit.  With many channel tiles an 8 x 8 patch keeps both operand panels of
    // the patch in that XCD's L2; with few (all of them resident at once anyway) a narrow patch
    // launches the blocks that share a token panel next to each other, so that they read it at
    // the same time (fc2, 9 channel tiles, K = 4608: 870 MB instead of 1370 MB fetched by the L2s).
    // Measured at M = 131072: 8 is the best of 4 .. 32 for the wide layers; for the narrow ones
    // 2 is the best of 1 .. 8 at K = 1152 and 3 the best of 2 .. 6 at K = 4608 (545 against
    // 557 us with 8-bit weights, no difference at M = 65536 or with 4-bit weights).
    args.group_m = args.n_tiles > 16 ? 8 : (args.KF >= 36 ? 3 : 2);
    if (x_corr && w_rowsum)
        return bits == 8 ? launch_bits<8, true>(args, epi, ydt, stream)
                         : launch_bits<4, true>(args, epi, ydt, stream);
    return bits == 8 ? launch_bits<8, false>(args, epi, ydt, stream)
                     : launch_bits<4, false>(args, epi, ydt, stream);
}

}  // namespace qc
