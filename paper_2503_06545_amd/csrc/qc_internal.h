// Internal declarations shared by the libqc translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qc.h"

namespace qc {

// ---- data layout of the GEMM operands in HBM -------------------------------------------
//
// Both GEMM operands are stored as "fragments": the 1 KiB a 64-lane wavefront hands to one
// v_mfma_i32_16x16x64_i8 as its A or B operand, lane after lane (lane l supplies the 16
// consecutive k of row l % 16 that start at 16 (l / 16)).  A fragment therefore covers
// 16 rows x 64 k, and a wavefront moves it HBM -> LDS -> registers with fully linear 16 B/lane
// accesses.  (The 16x16x64 form of the instruction is used because under the power cap it runs
// at a higher clock than the 32x32x32 form: it reads more operand but less accumulator data
// per multiply.)  With KF = Kp / 64 and Kp = K rounded up to 192:
//
//   activations, token m:  fragment ((m / 64) * KF + k / 64) * 4 + (m % 64) / 16, row m % 16
//       (the 4 KiB a wavefront of the GEMM needs per 64-k stage are contiguous)
//   weights, channel n = 128 G + 8 c + t:  fragment (G * KF + k / 64) * 8 + t, row c
//       (the 8 KiB stage tile of a block is contiguous; a lane of the GEMM ends up holding 8
//       consecutive output channels of one token, i.e. one 16 B bf16 store, 16 lanes covering
//       128 consecutive channels)
//   byte in fragment = (((k % 64) / 16) * 16 + row) * 16 + k % 16
//
// 4-bit weights keep the same (n, k) -> lane mapping but one 1 KiB unit holds two fragments'
// worth of nibbles: unit (G * KF + k / 64) * 4 + t / 2, where lane l has 8 bytes for fragment
// t even followed by 8 bytes for t odd.  Inside a dword of 8 nibbles, k offset e (0..7) sits in
// nibble (e < 4 ? 2 e : 2 (e - 4) + 1), so that (v << 4) & 0xF0F0F0F0 and v & 0xF0F0F0F0 are
// the int8 operand dwords (codes times 16).

constexpr int kFragRows = 16;
constexpr int kFragK = 64;
constexpr int kFragBytes = 1024;
constexpr int kKAlign = 192;       // K is padded to this: three 64-k pipeline stages of the GEMM
constexpr int kTileM = 256;        // GEMM block tile, tokens
constexpr int kTileN = 128;        // GEMM block tile, output channels
constexpr int kWaveM = 64;         // tokens of one wavefront of the GEMM
constexpr int kPackedHeaderBytes = 256;
constexpr uint32_t kPackedTag = 0x51433032u;  // "QC02"
constexpr float kAbsmaxFloor = 0x1p-64f;

__host__ __device__ inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

__host__ __device__ inline int64_t byte_in_frag(int64_t row16, int64_t k) {
    return (((k % kFragK) / 16) * 16 + row16) * 16 + k % 16;
}

// byte offset of activation code (m, k) from the start of the tiled codes
__host__ __device__ inline int64_t act_frag_offset(int64_t m, int64_t k, int64_t KF) {
    const int64_t frag = ((m / kWaveM) * KF + k / kFragK) * (kWaveM / kFragRows) + (m % kWaveM) / kFragRows;
    return frag * kFragBytes + byte_in_frag(m % kFragRows, k);
}

// byte offset of 8-bit weight code (n, k) from the start of the code area
__host__ __device__ inline int64_t weight_frag_offset(int64_t n, int64_t k, int64_t KF) {
    const int64_t r = n % kTileN;
    const int64_t frag = ((n / kTileN) * KF + k / kFragK) * (kTileN / kFragRows) + r % 8;
    return frag * kFragBytes + byte_in_frag(r / 8, k);
}

// byte offset (from the start of the code area) of the dword that holds the 8 nibbles of
// channel n, k = k8 .. k8 + 7 (k8 a multiple of 8)
__host__ __device__ inline int64_t w4_dword_offset(int64_t n, int64_t k8, int64_t KF) {
    const int64_t r = n % kTileN, t = r % 8;
    const int64_t unit = ((n / kTileN) * KF + k8 / kFragK) * (kTileN / kFragRows / 2) + t / 2;
    const int64_t lane = ((k8 % kFragK) / 16) * 16 + r / 8;
    return unit * kFragBytes + lane * 16 + (t % 2) * 8 + ((k8 % 16) / 8) * 4;
}

__host__ __device__ inline int w4_nibble_of(int e) { return e < 4 ? 2 * e : 2 * (e - 4) + 1; }

// workspace of qc_qlinear: [ x_scale: Mp floats ][ tiled codes: Mp * Kp bytes ]
// The quantization kernels write rows 0 .. M-1 and columns 0 .. K-1 only.  The GEMM reads whole
// fragments, padding included: what it finds in columns K .. Kp-1 is multiplied by the zero codes
// qc_pack_weight stores in the weights' K padding (so any bytes will do), and rows M .. Mp-1 are
// accumulated and never stored.  Packed weights must therefore always carry zeros in their K
// padding.
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
// codes and x_aux = zero point; shifted = true: codes minus asym_code_shift(act_bits) as signed
// bytes and x_aux = that shift - zero point, what the GEMM consumes.
hipError_t launch_quant_act_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K, uint8_t *qx_rowmajor,
                                 uint8_t *qx_tiled, int64_t KF, float *x_scale, float *x_aux,
                                 int act_bits, bool shifted, hipStream_t stream);

// What the asymmetric linear subtracts from the unsigned codes before it stores them as the
// GEMM's signed bytes: 8-bit codes (0..255) must be centred to fit; 6- and 4-bit codes fit as
// they are, and stored unshifted they have no sign bits to toggle, which under the power cap
// makes the GEMM up to 6 % faster than on centred codes.
__host__ __device__ inline int asym_code_shift(int act_bits) { return act_bits == 8 ? 128 : 0; }

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

// ---- schedule of the GEMM kernel that keeps its weight tile in LDS ---------------------------
constexpr int kRoundTokens = 512;   // one round: a channel tile x 512 tokens, 64 per wavefront

// rounds of 512 tokens over the padded token count (m_tiles tiles of 256)
__host__ __device__ inline int resident_chunks(int m_tiles) { return m_tiles / 2 + (m_tiles & 1); }

// Block b of a launch of nb blocks runs on XCD b % 8; the XCDs split the token chunks evenly.
struct ResidentXcd {
    int slot, blocks;   // the block's index among the blocks of its XCD, and how many those are
    int c_lo, c_hi;     // the XCD's chunks
};

__host__ __device__ inline ResidentXcd resident_xcd(int b, int nb, int chunks) {
    ResidentXcd x;
    const int xcd = b % 8;
    x.slot = b / 8;
    x.blocks = nb / 8 + (xcd < nb % 8 ? 1 : 0);
    x.c_lo = (int)((int64_t)chunks * xcd / 8);
    x.c_hi = (int)((int64_t)chunks * (xcd + 1) / 8);
    return x;
}

// The static schedule of the resident kernel on one XCD: `blocks` blocks (one per CU) share
// `chunks` rounds of 512 tokens x `n_tiles` channel tiles.  Two things decide it: a block should
// keep its weight tile for many rounds, and the blocks of the XCD should be reading the same few
// token chunks at the same time, because the XCD's L2 (4 MB) can hold the activations of a handful
// of chunks (576 KiB each at K = 1152) and the fabric behind it cannot deliver them once per
// channel tile (measured: with every block on its own chunk the kernel runs at the fabric's
// 5.7 TB/s, 55 % slower).  Channel tiles are taken in passes of at most `blocks`; within a pass of
// t tiles, k = blocks / t groups of t blocks each walk their own run of chunks in step, one
// channel tile per block, and the blocks left over share the remaining chunks x all t tiles in
// tile-major order.  A block's rounds of a pass are ids [id0, id1) with channel tile
// nt_off + id / w and chunk c_off + id % w.
struct RoundRange {
    int id0, id1, w, nt_off, c_off;
};

__host__ __device__ inline RoundRange resident_rounds(int pass, int slot, int blocks, int n_tiles, int chunks) {
    const int t = n_tiles - pass * blocks < blocks ? n_tiles - pass * blocks : blocks;
    const int k = blocks / t, main_n = k * t, side_n = blocks - main_n;
    int cm = 0, side0 = chunks;   // chunks per group, first chunk of the left-over blocks
    if (side_n > 0) {
        // the nearest split to equal rounds for everybody
        const int lo = (int)((int64_t)t * chunks / blocks);
        int best = -1;
        for (int c = lo; c <= lo + 1; ++c) {
            if ((int64_t)k * c > chunks) continue;
            const int side_r = (int)(((int64_t)t * (chunks - k * c) + side_n - 1) / side_n);
            const int cost = c > side_r ? c : side_r;
            if (best < 0 || cost < best) { best = cost; cm = c; }
        }
        side0 = k * cm;
    }
    RoundRange r;
    if (slot < main_n) {
        const int j = slot / t;
        const int g_lo = side_n ? j * cm : (int)((int64_t)chunks * j / k);
        const int g_hi = side_n ? (j + 1) * cm : (int)((int64_t)chunks * (j + 1) / k);
        r.id0 = 0;
        r.id1 = g_hi - g_lo;
        r.w = r.id1 > 0 ? r.id1 : 1;
        r.nt_off = pass * blocks + slot % t;
        r.c_off = g_lo;
    } else {
        const int q = slot - main_n, cs = chunks - side0;
        const int64_t total = (int64_t)t * cs;
        r.id0 = (int)(total * q / side_n);
        r.id1 = (int)(total * (q + 1) / side_n);
        r.w = cs > 0 ? cs : 1;
        r.nt_off = pass * blocks;
        r.c_off = side0;
    }
    return r;
}


// The rounds of block b in the order it runs them, as (channel tile, chunk) pairs; returns their
// number and writes the first `cap` of them to `pairs` (2 ints each) when it is not null.
__host__ __device__ inline int resident_block_rounds(int b, int nb, int n_tiles, int m_tiles, int *pairs, int cap) {
    const ResidentXcd x = resident_xcd(b, nb, resident_chunks(m_tiles));
    int n = 0;
    for (int pass = 0; pass * x.blocks < n_tiles; ++pass) {
        const RoundRange r = resident_rounds(pass, x.slot, x.blocks, n_tiles, x.c_hi - x.c_lo);
        for (int id = r.id0; id < r.id1; ++id, ++n)
            if (pairs && n < cap) {
                pairs[2 * n] = r.nt_off + id / r.w;
                pairs[2 * n + 1] = x.c_lo + r.c_off + id % r.w;
            }
    }
    return n;
}

enum GemmKernel { kGemmAuto = 0, kGemmRing = 1, kGemmResident = 2 };
// whether a 128-channel weight tile of this reduction length fits the resident kernel's LDS
bool gemm_resident_fits(int64_t K, int bits);
// whether launch_gemm picks the resident kernel for this problem by itself
bool gemm_resident_chosen(int64_t M, int64_t N, int64_t K, int bits);
int gemm_resident_blocks();

hipError_t launch_gemm(const uint8_t *x_tiled, const float *x_scale, const uint8_t *w_packed,
                       const float *w_scale, const float *bias, void *Y, int64_t M, int64_t N,
                       int64_t K, int bits, qc_epilogue epi, qc_out ydt, const float *x_corr,
                       const int32_t *w_rowsum, GemmKernel which, hipStream_t stream);

}  // namespace qc
