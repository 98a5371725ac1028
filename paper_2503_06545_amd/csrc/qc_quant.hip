// Per-token dynamic activation quantization (Section 4.1 "Quantization Scheme": activation
// parameters computed online; Section 3.1 Eq. (3)-(4) in symmetric signed form).
//
// HBM-bound: every element of X is read once and one int8 code is written.  A row is held in
// registers between the absmax pass and the cast, so there is no second read.  Blocks are
// small (one wavefront per 1152 columns of 8 rows) and many per CU, so that the load,
// arithmetic and store phases of different blocks overlap.
//
// The quotient x / s is the correctly rounded IEEE one, computed without a division per
// element: with r = RN(1 / s) (one true division per row) and q0 = RN(x * r), the residual
// e = x - s * q0 is exact in one fma and q = RN(q0 + e * r) is RN(x / s) for every |x / s| that
// can round to a non-zero code (Markstein's correction step: one suffices when the reciprocal
// is correctly rounded; checked against true division on the CPU over all bf16 inputs, random
// binary32 ones, constructed near-ties and the scales whose significand is all ones).
#include <type_traits>

#include "qc_internal.h"

namespace qc {
namespace {

constexpr int kGenericThreads = 256;
constexpr int kUnit = 16;          // elements handled as one unit: 16 codes = one 16 B store
constexpr int kUnitsPerThread = 9; // units held by one lane

// How a kernel treats the caches on its one pass (picked per call by cache_policy()): the chip's
// last-level cache in front of HBM holds 256 MiB, and what the pass leaves in it decides whether
// the GEMM that follows finds the codes there.
enum CachePolicy {
    kCachePlain = 0,    // input and codes both fit: ordinary loads and stores
    kStreamLoads = 1,   // the codes fit, not the input beside them: non-temporal loads of X
    kStreamStores = 2,  // the codes do not fit either: non-temporal stores of the codes
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ inline uint4 load16(const void *p) {
    if constexpr (NT) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    } else {
        return *reinterpret_cast<const uint4 *>(p);
    }
}

template <bool NT>
__device__ inline void store16(void *p, const uint4 &v) {
    if constexpr (NT) __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(p));
    else *reinterpret_cast<uint4 *>(p) = v;
}

__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// 16 elements of one row, widened to float.
template <typename XT>
struct Unit;

template <>
struct Unit<float> {
    float4 v[4];
    template <bool NT>
    __device__ void load(const float *p) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 w = load16<NT>(p + 4 * i);
            v[i] = make_float4(__uint_as_float(w.x), __uint_as_float(w.y), __uint_as_float(w.z), __uint_as_float(w.w));
        }
    }
    __device__ void zero() {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __device__ float get(int i) const {
        const float4 &f = v[i >> 2];
        switch (i & 3) { case 0: return f.x; case 1: return f.y; case 2: return f.z; default: return f.w; }
    }
};

template <>
struct Unit<uint16_t> {  // bf16 bit patterns
    uint4 v[2];
    template <bool NT>
    __device__ void load(const uint16_t *p) {
        v[0] = load16<NT>(p);
        v[1] = load16<NT>(p + 8);
    }
    __device__ void zero() { v[0] = v[1] = make_uint4(0, 0, 0, 0); }
    __device__ float get(int i) const {
        const uint4 &u = v[i >> 3];
        uint32_t w;
        switch ((i >> 1) & 3) { case 0: w = u.x; break; case 1: w = u.y; break; case 2: w = u.z; break; default: w = u.w; }
        return (i & 1) ? bf16_hi(w) : bf16_lo(w);
    }
};

// code = clamp(rne(x / s), -qmax, qmax): true IEEE division, then round half to even.
__device__ inline int quant_code(float x, float s, float qmax) {
    float r = rintf(x / s);
    r = fminf(fmaxf(r, -qmax), qmax);
    return (int)r;
}

// RN(x / s) from r = RN(1 / s): product, exact residual, one correction.
__device__ inline float quotient(float x, float s, float r) {
    const float q = x * r;
    return fmaf(fmaf(-s, q, x), r, q);
}

// Four quotients -> four int8 codes in one dword.  Clamping to [-qmax, qmax] before rounding
// equals rounding then clamping; adding 1.5 * 2^23 rounds to an integer (ties to even) and
// leaves its two's complement low byte in the low byte of the float.
__device__ inline uint32_t codes4(float q0, float q1, float q2, float q3, float qmax) {
    const float magic = 12582912.0f;
    const uint32_t y0 = __float_as_uint(__builtin_amdgcn_fmed3f(q0, -qmax, qmax) + magic);
    const uint32_t y1 = __float_as_uint(__builtin_amdgcn_fmed3f(q1, -qmax, qmax) + magic);
    const uint32_t y2 = __float_as_uint(__builtin_amdgcn_fmed3f(q2, -qmax, qmax) + magic);
    const uint32_t y3 = __float_as_uint(__builtin_amdgcn_fmed3f(q3, -qmax, qmax) + magic);
    const uint32_t lo = __builtin_amdgcn_perm(y1, y0, 0x0c0c0400u);  // [y0.b0, y1.b0, 0, 0]
    const uint32_t hi = __builtin_amdgcn_perm(y3, y2, 0x04000c0cu);  // [0, 0, y2.b0, y3.b0]
    return lo | hi;
}

__device__ inline float scale_of(float absmax, float qmax) { return fmaxf(absmax, kAbsmaxFloor) / qmax; }

// One scale for a whole activation tensor (Section 4.1 "Quantization Scheme": activation
// quantization per layer, parameters computed online): a first launch leaves the absmax of up to
// 256 slabs of the tensor in `partials`; every wavefront of the quantization kernel combines
// them itself (max is exact in any order), which needs neither atomics nor a third launch.
struct TensorMax {
    const float *partials;  // nullptr: one scale per row
    int count;
    bool single_scale;      // write x_scale[0] only, not one (equal) value per row
};

__device__ inline float tensor_absmax(const TensorMax &t, int lane) {
    float a = 0.0f;
    for (int j = lane; j < t.count; j += 64) a = fmaxf(a, t.partials[j]);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) a = fmaxf(a, __shfl_xor(a, d));
    return a;
}

constexpr int kSlabThreads = 256;
constexpr int kMaxSlabs = 256;

template <typename XT>
__global__ __launch_bounds__(kSlabThreads) void tensor_absmax_kernel(const XT *__restrict__ X, int64_t n,
                                                                    float *__restrict__ partials) {
    __shared__ float wave_max[kSlabThreads / 64];
    constexpr int kPer = 16 / (int)sizeof(XT);  // elements per 16 B load
    const int64_t nv = n / kPer;
    const int64_t stride = (int64_t)gridDim.x * kSlabThreads;
    float a = 0.0f;
    for (int64_t i = (int64_t)blockIdx.x * kSlabThreads + threadIdx.x; i < nv; i += stride) {
        const uint4 v = reinterpret_cast<const uint4 *>(X)[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (sizeof(XT) == 2) {
                a = fmaxf(a, fabsf(bf16_lo(w[j])));
                a = fmaxf(a, fabsf(bf16_hi(w[j])));
            } else {
                a = fmaxf(a, fabsf(__uint_as_float(w[j])));
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - nv * kPer)) {  // trailing elements
        const XT t = X[nv * kPer + threadIdx.x];
        if constexpr (sizeof(XT) == 2) a = fmaxf(a, fabsf(__uint_as_float((uint32_t)t << 16)));
        else a = fmaxf(a, fabsf(t));
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) a = fmaxf(a, __shfl_xor(a, d));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kSlabThreads / 64; ++w) a = fmaxf(a, wave_max[w]);
        partials[blockIdx.x] = a;
    }
}

// 8 lanes share a row and a wavefront holds 8 rows x 1152 columns (72 units of 16, 9 per lane)
// in registers, so that every 16 B store of the fragment layout completes a 128 B line (8 rows
// x 16 B) within one instruction.  Longer rows are cut into column slices of 1152, one
// wavefront of the block per slice; the slices agree on the row absmax through LDS.  Needs
// K % 16 == 0 and K <= 8 slices.
constexpr int kLanesPerRow = 8;
constexpr int kRowsPerBlock = 64 / kLanesPerRow;
constexpr int kUnitsPerSlice = kLanesPerRow * kUnitsPerThread;  // 72 units = 1152 columns
constexpr int kMaxSlices = 8;

// TENSOR: the absmax comes from `tmax` (one scale for the whole tensor).  A template parameter
// rather than a test of tmax.partials, so that the per-token kernel is compiled exactly as if
// the other did not exist.
template <typename XT, bool TENSOR, int POLICY>
__global__ __launch_bounds__(64 * kMaxSlices) void quant_rows_kernel(
    const XT *__restrict__ X, int64_t M, int64_t K, int8_t *__restrict__ qx,
    uint8_t *__restrict__ qx_tiled, int64_t KF, float *__restrict__ x_scale, float qmax,
    TensorMax tmax) {
    __shared__ float slice_max[kMaxSlices][kRowsPerBlock];
    const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6, slices = blockDim.x >> 6;
    const int sub = lane % kLanesPerRow, row_in_block = lane / kLanesPerRow;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + row_in_block;
    const int units = (int)(K / kUnit);
    const bool live = row < M;
    const XT *xrow = X + (live ? row : 0) * K;

    Unit<XT> u[kUnitsPerThread];
#pragma unroll
    for (int i = 0; i < kUnitsPerThread; ++i) {
        const int ui = slice * kUnitsPerSlice + i * kLanesPerRow + sub;
        if (live && ui < units) u[i].template load<POLICY == kStreamLoads>(xrow + (int64_t)ui * kUnit);
        else u[i].zero();
    }

    float a = 0.0f;
    if (TENSOR) {  // one scale for the whole tensor: its absmax was reduced beforehand
        a = tensor_absmax(tmax, lane);
    } else {
#pragma unroll
        for (int i = 0; i < kUnitsPerThread; ++i)
#pragma unroll
            for (int e = 0; e < kUnit; ++e) a = fmaxf(a, fabsf(u[i].get(e)));
#pragma unroll
        for (int d = 1; d < kLanesPerRow; d <<= 1) a = fmaxf(a, __shfl_xor(a, d));
        if (slices > 1) {  // uniform over the block
            if (sub == 0) slice_max[slice][row_in_block] = a;
            __syncthreads();
            for (int sl = 0; sl < slices; ++sl) a = fmaxf(a, slice_max[sl][row_in_block]);
        }
    }

    const float s = scale_of(a, qmax);
    const float r = 1.0f / s;  // correctly rounded
    if (TENSOR && tmax.single_scale) {
        if (blockIdx.x == 0 && threadIdx.x == 0) x_scale[0] = s;
    } else if (live && sub == 0 && slice == 0) {
        x_scale[row] = s;
    }
    if (!live) return;

    int8_t *out_rows = qx ? qx + row * K : nullptr;
    uint8_t *out_tiled = qx_tiled ? qx_tiled + act_frag_offset(row, 0, KF) : nullptr;
#pragma unroll
    for (int i = 0; i < kUnitsPerThread; ++i) {
        const int ui = slice * kUnitsPerSlice + i * kLanesPerRow + sub;
        if (ui >= units) continue;
        uint32_t w[4];
#pragma unroll
        for (int d = 0; d < 4; ++d)
            w[d] = codes4(quotient(u[i].get(4 * d + 0), s, r), quotient(u[i].get(4 * d + 1), s, r),
                          quotient(u[i].get(4 * d + 2), s, r), quotient(u[i].get(4 * d + 3), s, r), qmax);
        const uint4 out = make_uint4(w[0], w[1], w[2], w[3]);
        if (out_rows) store16<POLICY == kStreamStores>(out_rows + (int64_t)ui * kUnit, out);
        // unit ui covers k = 16 ui ..: 64-k stage ui / 4, k quarter ui % 4 (see act_frag_offset)
        if (out_tiled)
            store16<POLICY == kStreamStores>(out_tiled + (int64_t)(ui >> 2) * (4 * kFragBytes) + (ui & 3) * 256, out);
    }
}

// ---- rotation fused into the quantization (Section 3.2 AIGQ (1); Section 4.1 "Hardware
// Implementation") -----------------------------------------------------------------------------
// Each block of `rot` consecutive columns (16, 32, 64 or 128) is multiplied by the Walsh-Hadamard
// matrix of that size before the absmax and the cast, as a butterfly network in binary32 with
// the strides in ascending order: one rounding per output and stage, so the bits do not depend
// on which lane does which butterfly.  With the lane layout above, the 8 lanes of a row hold one
// aligned run of 128 columns per register unit: strides 1..8 are butterflies inside a lane's 16
// values, strides 16, 32, 64 pair lanes sub ^ 1, sub ^ 2, sub ^ 4 (DPP moves, no LDS).

__device__ inline float dpp_quad_xor1(float v) {  // lane ^ 1: quad_perm [1, 0, 3, 2]
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false));
}
__device__ inline float dpp_quad_xor2(float v) {  // lane ^ 2: quad_perm [2, 3, 0, 1]
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false));
}
__device__ inline float dpp_xor4(float v) {
    // lanes 0-3 and 8-11 of a row of 16 take lane + 4 (row_shl:4, banks 0 and 2), the others
    // lane - 4 (row_shr:4, banks 1 and 3)
    int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x104, 0xF, 0x5, false);
    t = __builtin_amdgcn_update_dpp(t, __float_as_int(v), 0x114, 0xF, 0xA, false);
    return __int_as_float(t);
}

template <typename XT, int POLICY>
__global__ __launch_bounds__(64 * kMaxSlices) void quant_rows_rot_kernel(
    const XT *__restrict__ X, int64_t M, int64_t K, int8_t *__restrict__ qx,
    uint8_t *__restrict__ qx_tiled, int64_t KF, float *__restrict__ x_scale, float qmax, int rot) {
    __shared__ float slice_max[kMaxSlices][kRowsPerBlock];
    const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6, slices = blockDim.x >> 6;
    const int sub = lane % kLanesPerRow, row_in_block = lane / kLanesPerRow;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + row_in_block;
    const int units = (int)(K / kUnit);
    const bool live = row < M;
    const XT *xrow = X + (live ? row : 0) * K;

    Unit<XT> u[kUnitsPerThread];
#pragma unroll
    for (int i = 0; i < kUnitsPerThread; ++i) {
        const int ui = slice * kUnitsPerSlice + i * kLanesPerRow + sub;
        if (live && ui < units) u[i].template load<POLICY == kStreamLoads>(xrow + (int64_t)ui * kUnit);
        else u[i].zero();
    }

    // +1 for the lane that holds the lower half of a cross-lane pair, -1 for the upper one:
    // fma(sign, own, other) is own + other below and other - own above, one rounding either way
    const float sg1 = (sub & 1) ? -1.0f : 1.0f, sg2 = (sub & 2) ? -1.0f : 1.0f,
                sg4 = (sub & 4) ? -1.0f : 1.0f;
    float f[kUnitsPerThread][kUnit];
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < kUnitsPerThread; ++i) {
#pragma unroll
        for (int e = 0; e < kUnit; ++e) f[i][e] = u[i].get(e);
#pragma unroll
        for (int h = 1; h < kUnit; h <<= 1)
#pragma unroll
            for (int j = 0; j < kUnit; ++j)
                if ((j & h) == 0) {
                    const float lo = f[i][j], hi = f[i][j + h];
                    f[i][j] = lo + hi;
                    f[i][j + h] = lo - hi;
                }
        if (rot >= 32) {
#pragma unroll
            for (int e = 0; e < kUnit; ++e) f[i][e] = fmaf(sg1, f[i][e], dpp_quad_xor1(f[i][e]));
        }
        if (rot >= 64) {
#pragma unroll
            for (int e = 0; e < kUnit; ++e) f[i][e] = fmaf(sg2, f[i][e], dpp_quad_xor2(f[i][e]));
        }
        if (rot >= 128) {
#pragma unroll
            for (int e = 0; e < kUnit; ++e) f[i][e] = fmaf(sg4, f[i][e], dpp_xor4(f[i][e]));
        }
#pragma unroll
        for (int e = 0; e < kUnit; ++e) a = fmaxf(a, fabsf(f[i][e]));
    }
#pragma unroll
    for (int d = 1; d < kLanesPerRow; d <<= 1) a = fmaxf(a, __shfl_xor(a, d));
    if (slices > 1) {  // uniform over the block
        if (sub == 0) slice_max[slice][row_in_block] = a;
        __syncthreads();
        for (int sl = 0; sl < slices; ++sl) a = fmaxf(a, slice_max[sl][row_in_block]);
    }

    const float s = scale_of(a, qmax);
    const float r = 1.0f / s;  // correctly rounded
    if (live && sub == 0 && slice == 0) x_scale[row] = s;
    if (!live) return;

    int8_t *out_rows = qx ? qx + row * K : nullptr;
    uint8_t *out_tiled = qx_tiled ? qx_tiled + act_frag_offset(row, 0, KF) : nullptr;
#pragma unroll
    for (int i = 0; i < kUnitsPerThread; ++i) {
        const int ui = slice * kUnitsPerSlice + i * kLanesPerRow + sub;
        if (ui >= units) continue;
        uint32_t w[4];
#pragma unroll
        for (int d = 0; d < 4; ++d)
            w[d] = codes4(quotient(f[i][4 * d + 0], s, r), quotient(f[i][4 * d + 1], s, r),
                          quotient(f[i][4 * d + 2], s, r), quotient(f[i][4 * d + 3], s, r), qmax);
        const uint4 out = make_uint4(w[0], w[1], w[2], w[3]);
        if (out_rows) store16<POLICY == kStreamStores>(out_rows + (int64_t)ui * kUnit, out);
        if (out_tiled)
            store16<POLICY == kStreamStores>(out_tiled + (int64_t)(ui >> 2) * (4 * kFragBytes) + (ui & 3) * 256, out);
    }
}

// ---- the quantizer as printed, asymmetric (Section 3.1 Eq. (3)-(4)) ----------------------------
//   s = max(hi - lo, 2^-64) / levels,  z = -rne(lo / s),  code = clamp(rne(x / s) + z, 0, levels)
// with levels = 2^b - 1.  Same layout and the same division-free quotient as above (it is
// exact for these larger quotients as well, checked on the host).  `shifted` selects what is
// stored: the canonical unsigned code and z, or, for the GEMM, code - shift as a signed byte
// and the correction shift - z (shift = asym_code_shift(act_bits)).
template <typename XT, int POLICY>
__global__ __launch_bounds__(64 * kMaxSlices) void quant_rows_asym_kernel(
    const XT *__restrict__ X, int64_t M, int64_t K, uint8_t *__restrict__ qx,
    uint8_t *__restrict__ qx_tiled, int64_t KF, float *__restrict__ x_scale,
    float *__restrict__ x_aux, float levels, float shift, bool shifted) {
    __shared__ float slice_lo[kMaxSlices][kRowsPerBlock], slice_hi[kMaxSlices][kRowsPerBlock];
    const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6, slices = blockDim.x >> 6;
    const int sub = lane % kLanesPerRow, row_in_block = lane / kLanesPerRow;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + row_in_block;
    const int units = (int)(K / kUnit);
    const bool live = row < M;
    const XT *xrow = X + (live ? row : 0) * K;

    Unit<XT> u[kUnitsPerThread];
#pragma unroll
    for (int i = 0; i < kUnitsPerThread; ++i) {
        const int ui = slice * kUnitsPerSlice + i * kLanesPerRow + sub;
        if (live && ui < units) u[i].template load<POLICY == kStreamLoads>(xrow + (int64_t)ui * kUnit);
        else u[i].zero();
    }

    // units past the end of the row hold zeros, which must not enter the minimum or maximum
    float lo = __builtin_inff(), hi = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < kUnitsPerThread; ++i) {
        const int ui = slice * kUnitsPerSlice + i * kLanesPerRow + sub;
        if (ui < units) {
#pragma unroll
            for (int e = 0; e < kUnit; ++e) {
                lo = fminf(lo, u[i].get(e));
                hi = fmaxf(hi, u[i].get(e));
            }
        }
    }
#pragma unroll
    for (int d = 1; d < kLanesPerRow; d <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, d));
        hi = fmaxf(hi, __shfl_xor(hi, d));
    }
    if (slices > 1) {  // uniform over the block
        if (sub == 0) { slice_lo[slice][row_in_block] = lo; slice_hi[slice][row_in_block] = hi; }
        __syncthreads();
        for (int sl = 0; sl < slices; ++sl) {
            lo = fminf(lo, slice_lo[sl][row_in_block]);
            hi = fmaxf(hi, slice_hi[sl][row_in_block]);
        }
    }
    if (!live) return;

    const float s = fmaxf(hi - lo, kAbsmaxFloor) / levels;
    const float r = 1.0f / s;  // correctly rounded
    const float z = -rintf(quotient(lo, s, r));
    if (sub == 0 && slice == 0) {
        x_scale[row] = s;
        x_aux[row] = shifted ? shift - z : z;
    }
    // clamp(rne(q) + z, 0, levels) - shift = clamp(rne(q) + (z - shift), -shift, levels - shift)
    const float off = shifted ? z - shift : z;
    const float cmin = shifted ? -shift : 0.0f, cmax = shifted ? levels - shift : levels;
    const float magic = 12582912.0f;  // 1.5 * 2^23: the sum's low byte is the integer's low byte

    uint8_t *out_rows = qx ? qx + row * K : nullptr;
    uint8_t *out_tiled = qx_tiled ? qx_tiled + act_frag_offset(row, 0, KF) : nullptr;
#pragma unroll
    for (int i = 0; i < kUnitsPerThread; ++i) {
        const int ui = slice * kUnitsPerSlice + i * kLanesPerRow + sub;
        if (ui >= units) continue;
        uint32_t w[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = rintf(quotient(u[i].get(4 * d + e), s, r)) + off;
                y[e] = __float_as_uint(__builtin_amdgcn_fmed3f(v, cmin, cmax) + magic);
            }
            w[d] = __builtin_amdgcn_perm(y[1], y[0], 0x0c0c0400u) | __builtin_amdgcn_perm(y[3], y[2], 0x04000c0cu);
        }
        const uint4 out = make_uint4(w[0], w[1], w[2], w[3]);
        if (out_rows) store16<POLICY == kStreamStores>(out_rows + (int64_t)ui * kUnit, out);
        if (out_tiled)
            store16<POLICY == kStreamStores>(out_tiled + (int64_t)(ui >> 2) * (4 * kFragBytes) + (ui & 3) * 256, out);
    }
}

// Any K, any alignment: one wavefront per row, two passes over the row (the second one is
// served by the caches).  Slow path for shapes the vector kernel does not take.
template <typename XT>
__global__ __launch_bounds__(kGenericThreads) void quant_rows_generic_kernel(
    const XT *__restrict__ X, int64_t M, int64_t K, int8_t *__restrict__ qx,
    uint8_t *__restrict__ qx_tiled, int64_t KF, float *__restrict__ x_scale, float qmax,
    TensorMax tmax) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * (kGenericThreads / 64) + (threadIdx.x >> 6);
    if (row >= M) return;
    const XT *xrow = X + row * K;
    auto widen = [](XT v) -> float {
        if constexpr (sizeof(XT) == 2) return __uint_as_float((uint32_t)v << 16);
        else return v;
    };
    float a = 0.0f;
    if (tmax.partials) {
        a = tensor_absmax(tmax, lane);
    } else {
        for (int64_t k = lane; k < K; k += 64) a = fmaxf(a, fabsf(widen(xrow[k])));
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) a = fmaxf(a, __shfl_xor(a, d));
    }
    const float s = scale_of(a, qmax);
    if (tmax.single_scale) {
        if (row == 0 && lane == 0) x_scale[0] = s;
    } else if (lane == 0) {
        x_scale[row] = s;
    }
    for (int64_t k = lane; k < K; k += 64) {
        const int8_t c = (int8_t)quant_code(widen(xrow[k]), s, qmax);
        if (qx) qx[row * K + k] = c;
        if (qx_tiled) qx_tiled[act_frag_offset(row, k, KF)] = (uint8_t)c;
    }
}

// Measured with bf16 input at K = 1152 and 4608 (whole qc_qlinear, GEMM included): up to 226 MB
// of input plus codes ordinary accesses are the fastest (non-temporal ones 8 % slower on the
// quantization); from 339 MB on, while the codes alone stay below the cache size, non-temporal
// loads leave the codes in the cache for the GEMM (M = 131072, K = 1152: quantization 83 -> 75 us,
// whole call 545 -> 512 us); with more than 256 MiB of codes non-temporal stores win instead
// (M = 131072, K = 4608: 324 -> 304 us, whole call 848 -> 836 us).
int cache_policy(int64_t M, int64_t K, size_t x_elem_bytes) {
    constexpr int64_t kLastLevelCache = (int64_t)256 << 20;
    const int64_t codes = M * K, input = codes * (int64_t)x_elem_bytes;
    if (codes > kLastLevelCache) return kStreamStores;
    if (input + codes > kLastLevelCache) return kStreamLoads;
    return kCachePlain;
}

// calls f(std::integral_constant<int, policy>) for the policy picked at run time
template <typename F>
hipError_t with_policy(int policy, F &&f) {
    switch (policy) {
        case kStreamLoads: return f(std::integral_constant<int, kStreamLoads>{});
        case kStreamStores: return f(std::integral_constant<int, kStreamStores>{});
        default: return f(std::integral_constant<int, kCachePlain>{});
    }
}

template <typename XT>
hipError_t launch_typed(const XT *X, int64_t M, int64_t K, int8_t *qx, uint8_t *qx_tiled,
                        int64_t KF, float *x_scale, float qmax, int rot, TensorMax tmax,
                        hipStream_t stream) {
    const int64_t units = K / kUnit;
    const int64_t slices = (units + kUnitsPerSlice - 1) / kUnitsPerSlice;
    const bool vec = (K % kUnit == 0) && slices <= kMaxSlices;
    const int policy = cache_policy(M, K, sizeof(XT));
    if (rot) {
        if (!vec || K % rot) return hipErrorInvalidValue;  // the entry points reject these first
        const int64_t blocks = (M + kRowsPerBlock - 1) / kRowsPerBlock;
        return with_policy(policy, [&](auto pol) {
            quant_rows_rot_kernel<XT, decltype(pol)::value>
                <<<dim3((unsigned)blocks), dim3((unsigned)(64 * slices)), 0, stream>>>(
                    X, M, K, qx, qx_tiled, KF, x_scale, qmax, rot);
            return hipGetLastError();
        });
    }
    if (!vec) {
        const int64_t blocks = (M + 3) / 4;
        quant_rows_generic_kernel<XT><<<dim3((unsigned)blocks), dim3(kGenericThreads), 0, stream>>>(
            X, M, K, qx, qx_tiled, KF, x_scale, qmax, tmax);
        return hipGetLastError();
    }
    const int64_t blocks = (M + kRowsPerBlock - 1) / kRowsPerBlock;
    if (tmax.partials) {
        // the tensor was read once already for its absmax: what the caches still hold of it helps
        quant_rows_kernel<XT, true, kCachePlain><<<dim3((unsigned)blocks), dim3((unsigned)(64 * slices)), 0, stream>>>(
            X, M, K, qx, qx_tiled, KF, x_scale, qmax, tmax);
        return hipGetLastError();
    }
    return with_policy(policy, [&](auto pol) {
        quant_rows_kernel<XT, false, decltype(pol)::value>
            <<<dim3((unsigned)blocks), dim3((unsigned)(64 * slices)), 0, stream>>>(
                X, M, K, qx, qx_tiled, KF, x_scale, qmax, tmax);
        return hipGetLastError();
    });
}

}  // namespace

bool quant_vector_path(int64_t K) {
    return K % kUnit == 0 && K / kUnit <= (int64_t)kUnitsPerSlice * kMaxSlices;
}

hipError_t launch_quant_act_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K, uint8_t *qx_rowmajor,
                                 uint8_t *qx_tiled, int64_t KF, float *x_scale, float *x_aux,
                                 int act_bits, bool shifted, hipStream_t stream) {
    if (!quant_vector_path(K)) return hipErrorInvalidValue;  // the entry points reject these first
    const float levels = (float)((1 << act_bits) - 1), shift = (float)asym_code_shift(act_bits);
    const int64_t slices = (K / kUnit + kUnitsPerSlice - 1) / kUnitsPerSlice;
    const dim3 grid((unsigned)((M + kRowsPerBlock - 1) / kRowsPerBlock)), block((unsigned)(64 * slices));
    if (xdt == QC_BF16)
        return with_policy(cache_policy(M, K, 2), [&](auto pol) {
            quant_rows_asym_kernel<uint16_t, decltype(pol)::value><<<grid, block, 0, stream>>>(
                (const uint16_t *)X, M, K, qx_rowmajor, qx_tiled, KF, x_scale, x_aux, levels, shift, shifted);
            return hipGetLastError();
        });
    return with_policy(cache_policy(M, K, 4), [&](auto pol) {
        quant_rows_asym_kernel<float, decltype(pol)::value><<<grid, block, 0, stream>>>(
            (const float *)X, M, K, qx_rowmajor, qx_tiled, KF, x_scale, x_aux, levels, shift, shifted);
        return hipGetLastError();
    });
}

bool quant_rotation_supported(int64_t K, int rot_block) {
    if (rot_block != 16 && rot_block != 32 && rot_block != 64 && rot_block != 128) return false;
    return K % rot_block == 0 && K / kUnit <= (int64_t)kUnitsPerSlice * kMaxSlices;
}

hipError_t launch_quant_act(const void *X, qc_dtype xdt, int64_t M, int64_t K, int8_t *qx_rowmajor,
                            uint8_t *qx_tiled, int64_t KF, float *x_scale, int act_bits,
                            int rot_block, hipStream_t stream) {
    const float qmax = (float)((1 << (act_bits - 1)) - 1);  // 127, 31 or 7 in an int8 container
    const TensorMax per_row = {nullptr, 0, false};
    if (xdt == QC_BF16)
        return launch_typed<uint16_t>((const uint16_t *)X, M, K, qx_rowmajor, qx_tiled, KF, x_scale,
                                      qmax, rot_block, per_row, stream);
    return launch_typed<float>((const float *)X, M, K, qx_rowmajor, qx_tiled, KF, x_scale, qmax,
                               rot_block, per_row, stream);
}

size_t tensor_partials_bytes() { return (size_t)kMaxSlabs * sizeof(float); }

hipError_t launch_quant_act_tensor(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                   int8_t *qx_rowmajor, uint8_t *qx_tiled, int64_t KF,
                                   float *x_scale, bool single_scale, float *partials, int act_bits,
                                   hipStream_t stream) {
    const float qmax = (float)((1 << (act_bits - 1)) - 1);
    const int64_t n = M * K;
    const int per = xdt == QC_BF16 ? 8 : 4;
    int64_t slabs = (n / per + (int64_t)kSlabThreads * 8 - 1) / ((int64_t)kSlabThreads * 8);
    if (slabs < 1) slabs = 1;
    if (slabs > kMaxSlabs) slabs = kMaxSlabs;
    if (xdt == QC_BF16)
        tensor_absmax_kernel<uint16_t><<<dim3((unsigned)slabs), dim3(kSlabThreads), 0, stream>>>(
            (const uint16_t *)X, n, partials);
    else
        tensor_absmax_kernel<float><<<dim3((unsigned)slabs), dim3(kSlabThreads), 0, stream>>>(
            (const float *)X, n, partials);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    const TensorMax tmax = {partials, (int)slabs, single_scale};
    if (xdt == QC_BF16)
        return launch_typed<uint16_t>((const uint16_t *)X, M, K, qx_rowmajor, qx_tiled, KF, x_scale,
                                      qmax, 0, tmax, stream);
    return launch_typed<float>((const float *)X, M, K, qx_rowmajor, qx_tiled, KF, x_scale, qmax, 0,
                               tmax, stream);
}

}  // namespace qc
