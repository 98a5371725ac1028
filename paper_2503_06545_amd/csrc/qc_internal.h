// Internal declarations shared by the libqc translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qc.h"

namespace qc {

// ---- data layout of the GEMM operands in HBM -------------------------------------------
//
// Both GEMM operands are stored as "fragments": the 1 KiB a 64-lane wavefront hands to one
// v_mfma_i32_32x32x32_i8 as its A or B operand, lane after lane (lane l supplies 16
// consecutive k of row l % 32, k half l / 32).  A fragment therefore covers 32 rows x 32 k,
// and a wavefront moves it HBM -> LDS -> registers with fully linear 16 B/lane accesses.
//
//   fragment index   = (row / 32) * KF + k / 32          KF = Kp / 32, Kp = K rounded up to 192
//   byte in fragment = (((k % 32) / 16) * 32 + row % 32) * 16 + k % 16
//
// Activations use their token index as `row`.  Weights use a permuted row index p so that a
// lane of the GEMM ends up holding 4 consecutive output channels of one token (one 8 B bf16
// or 16 B float store, 32 lanes covering 128 consecutive channels): inside each group of
// 128 channels, channel n = 128 G + r sits at p = 128 G + 32 * (r % 4) + r / 4.
// 4-bit weights keep the same (p, k) -> lane mapping but one 1 KiB unit spans 64 k: lane l
// holds 8 bytes of nibbles for the even 32-k fragment and 8 bytes for the odd one.  Inside a
// dword of 8 nibbles, k offset e (0..7) sits in nibble (e < 4 ? 2 e : 2 (e - 4) + 1), so that
// (v << 4) & 0xF0F0F0F0 and v & 0xF0F0F0F0 are the int8 operand dwords (codes times 16).

constexpr int kFragRows = 32;
constexpr int kFragK = 32;
constexpr int kFragBytes = 1024;
constexpr int kKAlign = 192;       // K is padded to this: three 64-k pipeline stages of the GEMM
constexpr int kTileM = 256;        // GEMM block tile, tokens
constexpr int kTileN = 128;        // GEMM block tile, output channels
constexpr int kPackedHeaderBytes = 256;
constexpr uint32_t kPackedTag = 0x51433031u;  // "QC01"
constexpr float kAbsmaxFloor = 0x1p-64f;

__host__ __device__ inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

__host__ __device__ inline int64_t frag_offset(int64_t row, int64_t k, int64_t KF) {
    return ((row / kFragRows) * KF + k / kFragK) * kFragBytes +
           (((k % kFragK) / 16) * 32 + row % kFragRows) * 16 + k % 16;
}

__host__ __device__ inline int64_t weight_row_of_channel(int64_t n) {
    const int64_t r = n % 128;
    return (n - r) + 32 * (r % 4) + r / 4;
}

// workspace of qc_qlinear: [ x_scale: Mp floats ][ tiled codes: Mp * Kp bytes ]
struct ActWorkspace {
    int64_t Mp, Kp, KF;
    size_t scale_bytes, total_bytes;
};

__host__ inline ActWorkspace act_workspace(int64_t M, int64_t K) {
    ActWorkspace w;
    w.Mp = round_up(M, kTileM);
    w.Kp = round_up(K, kKAlign);
    w.KF = w.Kp / kFragK;
    w.scale_bytes = (size_t)round_up(w.Mp * 4, 256);
    w.total_bytes = w.scale_bytes + (size_t)w.Mp * (size_t)w.Kp;
    return w;
}

// ---- launchers (each returns hipGetLastError() of its launch) --------------------------

// rot_block: 0 for no rotation, else the Walsh-Hadamard block size (quant_rotation_supported)
hipError_t launch_quant_act(const void *X, qc_dtype xdt, int64_t M, int64_t K, int8_t *qx_rowmajor,
                            uint8_t *qx_tiled, int64_t KF, float *x_scale, int act_bits,
                            int rot_block, hipStream_t stream);
bool quant_rotation_supported(int64_t K, int rot_block);
// One scale for the whole tensor: a slab-wise absmax launch into `partials`
// (tensor_partials_bytes() bytes), then the row kernels with that absmax.  single_scale: write
// x_scale[0] only; otherwise x_scale[m] gets the same value for every row (what the GEMM reads).
size_t tensor_partials_bytes();
hipError_t launch_quant_act_tensor(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                   int8_t *qx_rowmajor, uint8_t *qx_tiled, int64_t KF,
                                   float *x_scale, bool single_scale, float *partials, int act_bits,
                                   hipStream_t stream);
// K the vector quantization kernels take: a multiple of 16, at most 9216
bool quant_vector_path(int64_t K);
// Asymmetric codes (Section 3.1 Eq. (3)-(4) as printed).  shifted = false: canonical unsigned
// codes and x_aux = zero point; shifted = true: codes minus 2^(b-1) as signed bytes and
// x_aux = 2^(b-1) - zero point, what the GEMM consumes.
hipError_t launch_quant_act_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K, uint8_t *qx_rowmajor,
                                 uint8_t *qx_tiled, int64_t KF, float *x_scale, float *x_aux,
                                 int act_bits, bool shifted, hipStream_t stream);

// workspace of qc_qlinear_asym: [ x_scale: Mp floats ][ x_corr: Mp floats ][ tiled codes ]
struct ActWorkspaceAsym {
    ActWorkspace sym;
    size_t corr_offset, codes_offset, total_bytes;
};

__host__ inline ActWorkspaceAsym act_workspace_asym(int64_t M, int64_t K) {
    ActWorkspaceAsym w;
    w.sym = act_workspace(M, K);
    w.corr_offset = w.sym.scale_bytes;
    w.codes_offset = 2 * w.sym.scale_bytes;
    w.total_bytes = w.sym.total_bytes + w.sym.scale_bytes;
    return w;
}

hipError_t launch_gemm(const uint8_t *x_tiled, const float *x_scale, const uint8_t *w_packed,
                       const float *w_scale, const float *bias, void *Y, int64_t M, int64_t N,
                       int64_t K, int bits, qc_epilogue epi, qc_out ydt, const float *x_corr,
                       const int32_t *w_rowsum, hipStream_t stream);

}  // namespace qc
