// Offline weight quantization and packing (Section 4.1 "Quantization Scheme": per-channel
// weights; Section 3.2 AIGQ (1): bit-width chosen per layer), plus the test hooks that turn
// the library's internal orders back into canonical row-major codes.
#include "qc_internal.h"

namespace qc {
namespace {

constexpr int kThreads = 256;

__device__ inline int weight_code(float w, float s, float qmax) {
    float r = rintf(w / s);  // IEEE division, ties to even
    r = fminf(fmaxf(r, -qmax), qmax);
    return (int)r;
}

// Eight consecutive weights of a row, k = k8 .. k8 + 7 (zeros past K or for a padding row),
// after the counter-rotation that matches rotated activations (Section 3.2 AIGQ (1), Section
// 4.1): each block of `rot` columns times the Walsh-Hadamard matrix, then times 1 / rot.  Same
// butterfly network as the activation side, binary32, strides ascending: 1, 2, 4 inside the
// lane's eight values, 8 .. rot / 2 between lanes lane ^ 1 .. lane ^ (rot / 16).  Every lane of
// the wavefront must call it (the exchanges are wavefront-wide); rot = 0 returns the weights.
__device__ inline void load8_rotated(const float *wrow, int64_t k8, int64_t K, bool live, int rot,
                                     int lane, float (&v)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (live && k8 + e < K) ? wrow[k8 + e] : 0.0f;
    if (rot == 0) return;
#pragma unroll
    for (int h = 1; h < 8; h <<= 1)
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if ((j & h) == 0) {
                const float lo = v[j], hi = v[j + h];
                v[j] = lo + hi;
                v[j + h] = lo - hi;
            }
    for (int h = 8; h < rot; h <<= 1) {
        const int partner = h >> 3;
        const float sign = (lane & partner) ? -1.0f : 1.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = fmaf(sign, v[e], __shfl_xor(v[e], partner));
    }
    const float inv = 1.0f / (float)rot;  // a power of two: exact
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= inv;
}

// One wavefront per (padded) output channel.
__global__ __launch_bounds__(kThreads) void pack_weight_kernel(const float *__restrict__ W,
                                                               int64_t N, int64_t K, int bits,
                                                               int rot,
                                                               uint8_t *__restrict__ blob,
                                                               float *__restrict__ w_scale,
                                                               int64_t Np, int64_t Kp) {
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        uint32_t *h32 = reinterpret_cast<uint32_t *>(blob);
        h32[0] = kPackedTag;
        h32[1] = (uint32_t)bits;
        int64_t *h64 = reinterpret_cast<int64_t *>(blob + 8);
        h64[0] = N; h64[1] = K; h64[2] = Np; h64[3] = Kp;
        h32[10] = (uint32_t)rot;
    }
    if (n >= Np) return;
    const bool live = n < N;
    const float *wrow = W + (live ? n : 0) * K;
    const float qmax = bits == 8 ? 127.0f : 7.0f;

    // the same trip count for every lane: the rotation exchanges values across the wavefront
    const int64_t trips = (Kp + 64 * 8 - 1) / (64 * 8);
    float a = 0.0f;
    for (int64_t t = 0; t < trips; ++t) {
        float v[8];
        load8_rotated(wrow, (t * 64 + lane) * 8, K, live, rot, lane, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf(v[e]));
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) a = fmaxf(a, __shfl_xor(a, d));
    const float s = fmaxf(a, kAbsmaxFloor) / qmax;
    if (live && lane == 0) w_scale[n] = s;

    uint8_t *codes = blob + kPackedHeaderBytes;
    const int64_t KF = Kp / kFragK;
    for (int64_t t = 0; t < trips; ++t) {
        const int64_t k8 = (t * 64 + lane) * 8;
        float v[8];
        load8_rotated(wrow, k8, K, live, rot, lane, v);
        if (k8 >= Kp) continue;
        int c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            c[e] = (live && k8 + e < K) ? weight_code(v[e], s, qmax) : 0;
        if (bits == 8) {
            uint2 out;
            out.x = (c[0] & 0xff) | ((c[1] & 0xff) << 8) | ((c[2] & 0xff) << 16) | ((uint32_t)(c[3] & 0xff) << 24);
            out.y = (c[4] & 0xff) | ((c[5] & 0xff) << 8) | ((c[6] & 0xff) << 16) | ((uint32_t)(c[7] & 0xff) << 24);
            *reinterpret_cast<uint2 *>(codes + weight_frag_offset(n, k8, KF)) = out;
        } else {
            uint32_t out = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) out |= (uint32_t)(c[e] & 0xf) << (4 * w4_nibble_of(e));
            *reinterpret_cast<uint32_t *>(codes + w4_dword_offset(n, k8, KF)) = out;
        }
    }
}

__global__ __launch_bounds__(kThreads) void unpack_weight_kernel(const uint8_t *__restrict__ blob,
                                                                 int64_t N, int64_t K, int bits,
                                                                 int64_t Kp,
                                                                 int8_t *__restrict__ out) {
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= N * K) return;
    const int64_t n = idx / K, k = idx % K;
    const uint8_t *codes = blob + kPackedHeaderBytes;
    const int64_t KF = Kp / kFragK;
    if (bits == 8) {
        out[idx] = (int8_t)codes[weight_frag_offset(n, k, KF)];
    } else {
        const int64_t k8 = k - k % 8;
        const uint32_t v = *reinterpret_cast<const uint32_t *>(codes + w4_dword_offset(n, k8, KF));
        const int nib = (int)((v >> (4 * w4_nibble_of((int)(k % 8)))) & 0xf);
        out[idx] = (int8_t)(nib >= 8 ? nib - 16 : nib);
    }
}

// Sum of the codes of each output channel, read back from the packed blob (one wavefront per
// channel).  The epilogue of the asymmetric-activation linear multiplies it by the token's
// zero-point correction.
__global__ __launch_bounds__(kThreads) void weight_row_sums_kernel(const uint8_t *__restrict__ blob,
                                                                   int64_t N, int64_t K, int bits,
                                                                   int64_t Kp,
                                                                   int32_t *__restrict__ sums) {
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (n >= N) return;
    const uint8_t *codes = blob + kPackedHeaderBytes;
    const int64_t KF = Kp / kFragK;
    int32_t acc = 0;
    for (int64_t k8 = (int64_t)lane * 8; k8 < K; k8 += 64 * 8) {
        if (bits == 8) {
            const uint2 v = *reinterpret_cast<const uint2 *>(codes + weight_frag_offset(n, k8, KF));
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t w = e < 4 ? v.x : v.y;
                if (k8 + e < K) acc += (int32_t)(int8_t)((w >> (8 * (e & 3))) & 0xff);
            }
        } else {
            const uint32_t v = *reinterpret_cast<const uint32_t *>(codes + w4_dword_offset(n, k8, KF));
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int nib = (int)((v >> (4 * w4_nibble_of(e))) & 0xf);
                if (k8 + e < K) acc += nib >= 8 ? nib - 16 : nib;
            }
        }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) acc += __shfl_xor(acc, d);
    if (lane == 0) sums[n] = acc;
}

// The same for the workspace of the asymmetric linear: unsigned codes back from the stored
// signed bytes (code - shift), zero point back from the stored correction shift - z.
__global__ __launch_bounds__(kThreads) void untile_act_asym_kernel(const uint8_t *__restrict__ tiled,
                                                                   const float *__restrict__ scales,
                                                                   const float *__restrict__ corr,
                                                                   int64_t M, int64_t K, int64_t KF,
                                                                   int shift, uint8_t *__restrict__ qx,
                                                                   float *__restrict__ x_scale,
                                                                   float *__restrict__ x_zero) {
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx < M) {
        x_scale[idx] = scales[idx];
        x_zero[idx] = (float)shift - corr[idx];
    }
    if (idx >= M * K) return;
    const int64_t m = idx / K, k = idx % K;
    qx[idx] = (uint8_t)((int)(int8_t)tiled[act_frag_offset(m, k, KF)] + shift);
}

__global__ __launch_bounds__(kThreads) void untile_act_kernel(const uint8_t *__restrict__ tiled,
                                                              const float *__restrict__ scales,
                                                              int64_t M, int64_t K, int64_t KF,
                                                              int8_t *__restrict__ qx,
                                                              float *__restrict__ x_scale) {
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx < M) x_scale[idx] = scales[idx];
    if (idx >= M * K) return;
    const int64_t m = idx / K, k = idx % K;
    qx[idx] = (int8_t)tiled[act_frag_offset(m, k, KF)];
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace
}  // namespace qc

using namespace qc;

extern "C" size_t qc_packed_weight_bytes(int64_t N, int64_t K, int bits) {
    if ((bits != 4 && bits != 8) || N < 1 || K < 1 || K > QC_MAX_K || N > QC_MAX_N) return 0;
    if (bits == 4 && (K % 2)) return 0;
    const int64_t Np = round_up(N, kTileN), Kp = round_up(K, kKAlign);
    return (size_t)kPackedHeaderBytes + (size_t)(Np * Kp * bits / 8);
}

namespace {
qc_status pack_weight_any(const float *W, int64_t N, int64_t K, int bits, int rot, void *packed,
                          float *w_scale, void *stream) {
    if (!W || !packed || !w_scale || N < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (!aligned(W, 16) || !aligned(packed, 256) || !aligned(w_scale, 16)) return QC_ERR_INVALID_ARG;
    if (qc_packed_weight_bytes(N, K, bits) == 0) return QC_ERR_UNSUPPORTED;
    if (rot && !quant_rotation_supported(K, rot)) return QC_ERR_UNSUPPORTED;
    const int64_t Np = round_up(N, kTileN), Kp = round_up(K, kKAlign);
    const int64_t blocks = Np / (kThreads / 64);
    pack_weight_kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
        W, N, K, bits, rot, (uint8_t *)packed, w_scale, Np, Kp);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}
}  // namespace

extern "C" qc_status qc_pack_weight(const float *W, int64_t N, int64_t K, int bits, void *packed,
                                    float *w_scale, void *stream) {
    return pack_weight_any(W, N, K, bits, 0, packed, w_scale, stream);
}

extern "C" qc_status qc_pack_weight_rot(const float *W, int64_t N, int64_t K, int bits,
                                        int rot_block, void *packed, float *w_scale, void *stream) {
    if (rot_block == 0) return QC_ERR_UNSUPPORTED;
    return pack_weight_any(W, N, K, bits, rot_block, packed, w_scale, stream);
}

extern "C" qc_status qc_unpack_weight_codes(const void *packed, int64_t N, int64_t K, int bits,
                                            int8_t *codes, void *stream) {
    if (!packed || !codes || N < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (!aligned(packed, 256)) return QC_ERR_INVALID_ARG;
    if (qc_packed_weight_bytes(N, K, bits) == 0) return QC_ERR_UNSUPPORTED;
    const int64_t Kp = round_up(K, kKAlign);
    const int64_t blocks = (N * K + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    unpack_weight_kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
        (const uint8_t *)packed, N, K, bits, Kp, codes);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" qc_status qc_debug_workspace_act(const void *workspace, int64_t M, int64_t K,
                                            int8_t *qx, float *x_scale, void *stream) {
    if (!workspace || !qx || !x_scale || M < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (K > QC_MAX_K) return QC_ERR_UNSUPPORTED;
    if (!aligned(workspace, 256)) return QC_ERR_INVALID_ARG;
    const ActWorkspace ws = act_workspace(M, K);
    const uint8_t *base = (const uint8_t *)workspace;
    const int64_t blocks = (M * K + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    untile_act_kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
        base + ws.scale_bytes, (const float *)base, M, K, ws.KF, qx, x_scale);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" qc_status qc_weight_row_sums(const void *packed, int64_t N, int64_t K, int bits,
                                        int32_t *row_sums, void *stream) {
    if (!packed || !row_sums || N < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (!aligned(packed, 256) || !aligned(row_sums, 16)) return QC_ERR_INVALID_ARG;
    if (qc_packed_weight_bytes(N, K, bits) == 0) return QC_ERR_UNSUPPORTED;
    const int64_t Kp = round_up(K, kKAlign);
    const int64_t blocks = (N + kThreads / 64 - 1) / (kThreads / 64);
    weight_row_sums_kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
        (const uint8_t *)packed, N, K, bits, Kp, row_sums);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" qc_status qc_debug_workspace_act_asym(const void *workspace, int64_t M, int64_t K,
                                                 int act_bits, uint8_t *qx, float *x_scale,
                                                 float *x_zero, void *stream) {
    if (!workspace || !qx || !x_scale || !x_zero || M < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (act_bits != 8 && act_bits != 6 && act_bits != 4) return QC_ERR_UNSUPPORTED;
    if (K > QC_MAX_K) return QC_ERR_UNSUPPORTED;
    if (!aligned(workspace, 256)) return QC_ERR_INVALID_ARG;
    const ActWorkspaceAsym ws = act_workspace_asym(M, K);
    const uint8_t *base = (const uint8_t *)workspace;
    const int64_t blocks = (M * K + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    untile_act_asym_kernel<<<dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(
        base + ws.codes_offset, (const float *)base, (const float *)(base + ws.corr_offset), M, K,
        ws.sym.KF, asym_code_shift(act_bits), qx, x_scale, x_zero);
    return hipGetLastError() == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}
