// C ABI entry points for activation quantization and the fused quantized linear: argument
// checks first, then launches on the caller's stream.  Nothing here allocates or synchronises.
#include "qc_internal.h"

using namespace qc;

namespace {
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
}  // namespace

extern "C" const char *qc_status_string(qc_status status) {
    switch (status) {
        case QC_OK: return "QC_OK";
        case QC_ERR_INVALID_ARG: return "QC_ERR_INVALID_ARG: null or misaligned pointer, bad size or enum";
        case QC_ERR_UNSUPPORTED: return "QC_ERR_UNSUPPORTED: size or combination not implemented";
        case QC_ERR_WORKSPACE: return "QC_ERR_WORKSPACE: workspace too small";
        case QC_ERR_DEVICE: return "QC_ERR_DEVICE: the HIP runtime refused a launch";
    }
    return "unknown qc_status";
}

extern "C" int qc_version(void) { return 1003; }

// ---- decision rules: host arithmetic only ---------------------------------------------------

namespace {
// 0, 1, 2 for value < low, low <= value < high, value >= high; -1 for NaN or low > high
int three_way(float value, float low, float high) {
    if (value != value || low != low || high != high || low > high) return -1;
    if (value < low) return 0;
    return value < high ? 1 : 2;
}
}  // namespace

extern "C" float qc_divergence_score(float l1_change, int k, float grad_norm) {
    if (k < 1) return __builtin_nanf("");
    return (float)((double)l1_change / (double)k * (double)grad_norm);
}

extern "C" int qc_cache_interval(float D, float delta1, float delta2, int tau_max, int tau_mid,
                                 int tau_min) {
    const int which = three_way(D, delta1, delta2);
    return which < 0 ? -1 : which == 0 ? tau_max : which == 1 ? tau_mid : tau_min;
}

extern "C" int qc_activation_bits(float D, float theta1, float theta2, int bit_max, int bit_mid,
                                  int bit_min) {
    const int which = three_way(D, theta1, theta2);
    return which < 0 ? -1 : which == 0 ? bit_max : which == 1 ? bit_mid : bit_min;
}

extern "C" float qc_prune_probability(float S, float tau_low, float tau_high, float p_base) {
    if (S != S || tau_low != tau_low || tau_high != tau_high || p_base != p_base ||
        tau_low > tau_high)
        return __builtin_nanf("");
    if (S > tau_high) return 1.0f;
    if (S < tau_low) return 0.0f;
    return p_base;
}

// ---- shared argument checks -------------------------------------------------------------------
// Every entry point checks in the same order: INVALID_ARG (pointers, sizes, enums, alignment),
// then UNSUPPORTED, then WORKSPACE; nothing is launched before all of them have passed.

namespace {

bool act_bits_ok(int b) { return b == 8 || b == 6 || b == 4; }

// the activation side of a call: X [M, K] of xdt
qc_status check_activation(const void *X, qc_dtype xdt, int64_t M, int64_t K) {
    if (!X || M < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16)) return QC_ERR_INVALID_ARG;
    return QC_OK;
}

// the weight / output side of a linear: packed blob, scales, optional bias, Y [M, N]
qc_status check_linear_side(const void *packed, const float *w_scale, const float *bias,
                            qc_epilogue epi, const void *Y, qc_out ydt, int64_t M, int64_t K,
                            int64_t N) {
    if (!packed || !w_scale || !Y || M < 1 || K < 1 || N < 1) return QC_ERR_INVALID_ARG;
    if (epi != QC_EPI_NONE && epi != QC_EPI_GELU_TANH && epi != QC_EPI_GELU_ERF) return QC_ERR_INVALID_ARG;
    if (ydt != QC_OUT_F32 && ydt != QC_OUT_BF16 && ydt != QC_OUT_I32_ACC) return QC_ERR_INVALID_ARG;
    if (!aligned(packed, 256) || !aligned(w_scale, 16) || !aligned(Y, 16) || (bias && !aligned(bias, 16)))
        return QC_ERR_INVALID_ARG;
    return QC_OK;
}

qc_status check_workspace_pointer(const void *workspace) {
    return workspace && aligned(workspace, 256) ? QC_OK : QC_ERR_INVALID_ARG;
}

// what the quantization kernels take.  vector_only: the variant has no kernel for K that is not
// a multiple of 16 or exceeds 9216; rot_block 0 = no rotation
qc_status check_quant_supported(int64_t M, int64_t K, int act_bits, bool vector_only, int rot_block) {
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (K > QC_MAX_K || (M + 3) / 4 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (vector_only && !quant_vector_path(K)) return QC_ERR_UNSUPPORTED;
    if (rot_block && !quant_rotation_supported(K, rot_block)) return QC_ERR_UNSUPPORTED;
    return QC_OK;
}

// what the GEMM takes
qc_status check_gemm_supported(int64_t M, int64_t K, int64_t N, int bits) {
    if (qc_packed_weight_bytes(N, K, bits) == 0) return QC_ERR_UNSUPPORTED;
    const int64_t tiles = (round_up(M, kTileM) / kTileM) * (round_up(N, kTileN) / kTileN);
    return tiles > 0x7fffffffLL ? QC_ERR_UNSUPPORTED : QC_OK;
}

#define QC_TRY(expr)                          \
    do {                                      \
        const qc_status st_ = (expr);         \
        if (st_ != QC_OK) return st_;         \
    } while (0)

qc_status device_status(hipError_t e) { return e == hipSuccess ? QC_OK : QC_ERR_DEVICE; }

// How the activations of a quantized linear are quantized.
struct ActQuant {
    int act_bits;
    int rot_block;  // 0: no rotation
};

// stand-alone quantizer: codes row major
qc_status quant_act_any(const void *X, qc_dtype xdt, int64_t M, int64_t K, ActQuant how,
                        int8_t *qx, float *x_scale, void *stream) {
    QC_TRY(check_activation(X, xdt, M, K));
    if (!qx || !x_scale || !aligned(qx, 16) || !aligned(x_scale, 4)) return QC_ERR_INVALID_ARG;
    QC_TRY(check_quant_supported(M, K, how.act_bits, false, how.rot_block));
    return device_status(launch_quant_act(X, xdt, M, K, qx, nullptr, 0, x_scale, how.act_bits,
                                          how.rot_block, (hipStream_t)stream));
}

// first half of a linear: codes in the GEMM's order + scales into the workspace
qc_status qlinear_quant_any(const void *X, qc_dtype xdt, int64_t M, int64_t K, ActQuant how,
                            void *workspace, size_t workspace_bytes, void *stream) {
    QC_TRY(check_activation(X, xdt, M, K));
    QC_TRY(check_workspace_pointer(workspace));
    QC_TRY(check_quant_supported(M, K, how.act_bits, false, how.rot_block));
    const ActWorkspace ws = act_workspace(M, K);
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    uint8_t *base = (uint8_t *)workspace;
    return device_status(launch_quant_act(X, xdt, M, K, nullptr, base + ws.scale_bytes, ws.KF,
                                          (float *)base, how.act_bits, how.rot_block,
                                          (hipStream_t)stream));
}

qc_status qlinear_any(const void *X, qc_dtype xdt, int64_t M, int64_t K, ActQuant how,
                      const void *packed, const float *w_scale, int bits, int64_t N,
                      const float *bias, qc_epilogue epi, void *Y, qc_out ydt, void *workspace,
                      size_t workspace_bytes, void *stream) {
    // both halves' checks up front, so that a failed call has no side effect
    QC_TRY(check_activation(X, xdt, M, K));
    QC_TRY(check_linear_side(packed, w_scale, bias, epi, Y, ydt, M, K, N));
    QC_TRY(check_workspace_pointer(workspace));
    QC_TRY(check_quant_supported(M, K, how.act_bits, false, how.rot_block));
    QC_TRY(check_gemm_supported(M, K, N, bits));
    if (workspace_bytes < act_workspace(M, K).total_bytes) return QC_ERR_WORKSPACE;
    QC_TRY(qlinear_quant_any(X, xdt, M, K, how, workspace, workspace_bytes, stream));
    return qc_qlinear_gemm(workspace, workspace_bytes, M, K, packed, w_scale, bits, N, bias, epi, Y,
                           ydt, stream);
}

}  // namespace

// ---- per-token symmetric quantization (8, 6 or 4 bit codes), optionally rotated ------------------

extern "C" size_t qc_qlinear_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M < 1 || K < 1 || N < 1 || K > QC_MAX_K) return 0;
    return act_workspace(M, K).total_bytes;
}

extern "C" qc_status qc_quant_act_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                       int act_bits, int8_t *qx, float *x_scale, void *stream) {
    return quant_act_any(X, xdt, M, K, {act_bits, 0}, qx, x_scale, stream);
}

extern "C" qc_status qc_quant_act(const void *X, qc_dtype xdt, int64_t M, int64_t K, int8_t *qx,
                                  float *x_scale, void *stream) {
    return quant_act_any(X, xdt, M, K, {8, 0}, qx, x_scale, stream);
}

extern "C" qc_status qc_quant_act_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                      int act_bits, int rot_block, int8_t *qx, float *x_scale,
                                      void *stream) {
    if (rot_block == 0) return QC_ERR_UNSUPPORTED;
    return quant_act_any(X, xdt, M, K, {act_bits, rot_block}, qx, x_scale, stream);
}

extern "C" qc_status qc_qlinear_quant_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                           int act_bits, void *workspace, size_t workspace_bytes,
                                           void *stream) {
    return qlinear_quant_any(X, xdt, M, K, {act_bits, 0}, workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear_quant(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                      void *workspace, size_t workspace_bytes, void *stream) {
    return qlinear_quant_any(X, xdt, M, K, {8, 0}, workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear_quant_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                          int act_bits, int rot_block, void *workspace,
                                          size_t workspace_bytes, void *stream) {
    if (rot_block == 0) return QC_ERR_UNSUPPORTED;
    return qlinear_quant_any(X, xdt, M, K, {act_bits, rot_block}, workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear_gemm(const void *workspace, size_t workspace_bytes, int64_t M,
                                     int64_t K, const void *packed, const float *w_scale, int bits,
                                     int64_t N, const float *bias, qc_epilogue epi, void *Y,
                                     qc_out ydt, void *stream) {
    QC_TRY(check_linear_side(packed, w_scale, bias, epi, Y, ydt, M, K, N));
    QC_TRY(check_workspace_pointer(workspace));
    QC_TRY(check_gemm_supported(M, K, N, bits));
    const ActWorkspace ws = act_workspace(M, K);
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    const uint8_t *base = (const uint8_t *)workspace;
    return device_status(launch_gemm(base + ws.scale_bytes, (const float *)base,
                                     (const uint8_t *)packed, w_scale, bias, Y, M, N, K, bits, epi,
                                     ydt, nullptr, nullptr, kGemmAuto, (hipStream_t)stream));
}

extern "C" qc_status qc_qlinear_act_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                         int act_bits, const void *packed, const float *w_scale,
                                         int bits, int64_t N, const float *bias, qc_epilogue epi,
                                         void *Y, qc_out ydt, void *workspace,
                                         size_t workspace_bytes, void *stream) {
    return qlinear_any(X, xdt, M, K, {act_bits, 0}, packed, w_scale, bits, N, bias, epi, Y, ydt,
                       workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                const void *packed, const float *w_scale, int bits, int64_t N,
                                const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                                void *workspace, size_t workspace_bytes, void *stream) {
    return qlinear_any(X, xdt, M, K, {8, 0}, packed, w_scale, bits, N, bias, epi, Y, ydt, workspace,
                       workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                                    int rot_block, const void *packed, const float *w_scale,
                                    int bits, int64_t N, const float *bias, qc_epilogue epi, void *Y,
                                    qc_out ydt, void *workspace, size_t workspace_bytes,
                                    void *stream) {
    if (rot_block == 0) return QC_ERR_UNSUPPORTED;
    return qlinear_any(X, xdt, M, K, {act_bits, rot_block}, packed, w_scale, bits, N, bias, epi, Y,
                       ydt, workspace, workspace_bytes, stream);
}

// ---- asymmetric activations (Section 3.1 Eq. (3)-(4) as printed) --------------------------------

extern "C" size_t qc_qlinear_asym_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M < 1 || K < 1 || N < 1 || K > QC_MAX_K) return 0;
    return act_workspace_asym(M, K).total_bytes;
}

extern "C" qc_status qc_quant_act_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                       int act_bits, uint8_t *qx, float *x_scale, float *x_zero,
                                       void *stream) {
    QC_TRY(check_activation(X, xdt, M, K));
    if (!qx || !x_scale || !x_zero || !aligned(qx, 16) || !aligned(x_scale, 4) || !aligned(x_zero, 4))
        return QC_ERR_INVALID_ARG;
    QC_TRY(check_quant_supported(M, K, act_bits, true, 0));
    return device_status(launch_quant_act_asym(X, xdt, M, K, qx, nullptr, 0, x_scale, x_zero,
                                               act_bits, false, (hipStream_t)stream));
}

extern "C" qc_status qc_qlinear_asym_quant(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                           int act_bits, void *workspace, size_t workspace_bytes,
                                           void *stream) {
    QC_TRY(check_activation(X, xdt, M, K));
    QC_TRY(check_workspace_pointer(workspace));
    QC_TRY(check_quant_supported(M, K, act_bits, true, 0));
    const ActWorkspaceAsym ws = act_workspace_asym(M, K);
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    uint8_t *base = (uint8_t *)workspace;
    return device_status(launch_quant_act_asym(X, xdt, M, K, nullptr, base + ws.codes_offset,
                                               ws.sym.KF, (float *)base,
                                               (float *)(base + ws.corr_offset), act_bits, true,
                                               (hipStream_t)stream));
}

extern "C" qc_status qc_qlinear_asym_gemm(const void *workspace, size_t workspace_bytes, int64_t M,
                                          int64_t K, const void *packed, const float *w_scale,
                                          const int32_t *w_row_sums, int bits, int64_t N,
                                          const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                                          void *stream) {
    QC_TRY(check_linear_side(packed, w_scale, bias, epi, Y, ydt, M, K, N));
    if (!w_row_sums || !aligned(w_row_sums, 16)) return QC_ERR_INVALID_ARG;
    QC_TRY(check_workspace_pointer(workspace));
    QC_TRY(check_gemm_supported(M, K, N, bits));
    if (!quant_vector_path(K)) return QC_ERR_UNSUPPORTED;
    const ActWorkspaceAsym ws = act_workspace_asym(M, K);
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    const uint8_t *base = (const uint8_t *)workspace;
    return device_status(launch_gemm(base + ws.codes_offset, (const float *)base,
                                     (const uint8_t *)packed, w_scale, bias, Y, M, N, K, bits, epi,
                                     ydt, (const float *)(base + ws.corr_offset), w_row_sums,
                                     kGemmAuto, (hipStream_t)stream));
}

extern "C" qc_status qc_qlinear_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                     int act_bits, const void *packed, const float *w_scale,
                                     const int32_t *w_row_sums, int bits, int64_t N,
                                     const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                                     void *workspace, size_t workspace_bytes, void *stream) {
    QC_TRY(check_activation(X, xdt, M, K));
    QC_TRY(check_linear_side(packed, w_scale, bias, epi, Y, ydt, M, K, N));
    if (!w_row_sums || !aligned(w_row_sums, 16)) return QC_ERR_INVALID_ARG;
    QC_TRY(check_workspace_pointer(workspace));
    QC_TRY(check_quant_supported(M, K, act_bits, true, 0));
    QC_TRY(check_gemm_supported(M, K, N, bits));
    if (workspace_bytes < act_workspace_asym(M, K).total_bytes) return QC_ERR_WORKSPACE;
    QC_TRY(qc_qlinear_asym_quant(X, xdt, M, K, act_bits, workspace, workspace_bytes, stream));
    return qc_qlinear_asym_gemm(workspace, workspace_bytes, M, K, packed, w_scale, w_row_sums, bits,
                                N, bias, epi, Y, ydt, stream);
}

// ---- one activation scale per layer input (Section 4.1 "Quantization Scheme") ------------------

extern "C" size_t qc_quant_act_tensor_workspace_bytes(int64_t M, int64_t K) {
    if (M < 1 || K < 1 || K > QC_MAX_K) return 0;
    return tensor_partials_bytes();
}

extern "C" qc_status qc_quant_act_tensor(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                         int act_bits, int8_t *qx, float *x_scale, void *workspace,
                                         size_t workspace_bytes, void *stream) {
    QC_TRY(check_activation(X, xdt, M, K));
    if (!qx || !x_scale || !aligned(qx, 16) || !aligned(x_scale, 4)) return QC_ERR_INVALID_ARG;
    QC_TRY(check_workspace_pointer(workspace));
    QC_TRY(check_quant_supported(M, K, act_bits, false, 0));
    if (workspace_bytes < tensor_partials_bytes()) return QC_ERR_WORKSPACE;
    return device_status(launch_quant_act_tensor(X, xdt, M, K, qx, nullptr, 0, x_scale, true,
                                                 (float *)workspace, act_bits, (hipStream_t)stream));
}

extern "C" size_t qc_qlinear_tensor_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M < 1 || K < 1 || N < 1 || K > QC_MAX_K) return 0;
    return act_workspace(M, K).total_bytes + tensor_partials_bytes();
}

extern "C" qc_status qc_qlinear_tensor(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                       int act_bits, const void *packed, const float *w_scale,
                                       int bits, int64_t N, const float *bias, qc_epilogue epi,
                                       void *Y, qc_out ydt, void *workspace, size_t workspace_bytes,
                                       void *stream) {
    QC_TRY(check_activation(X, xdt, M, K));
    QC_TRY(check_linear_side(packed, w_scale, bias, epi, Y, ydt, M, K, N));
    QC_TRY(check_workspace_pointer(workspace));
    QC_TRY(check_quant_supported(M, K, act_bits, false, 0));
    QC_TRY(check_gemm_supported(M, K, N, bits));
    const ActWorkspace ws = act_workspace(M, K);
    if (workspace_bytes < ws.total_bytes + tensor_partials_bytes()) return QC_ERR_WORKSPACE;
    // [ the workspace of qc_qlinear ][ slab maxima ]: the first part is what qc_qlinear_gemm and
    // qc_debug_workspace_act read, with the one scale repeated for every token
    uint8_t *base = (uint8_t *)workspace;
    QC_TRY(device_status(launch_quant_act_tensor(X, xdt, M, K, nullptr, base + ws.scale_bytes, ws.KF,
                                                 (float *)base, false,
                                                 (float *)(base + ws.total_bytes), act_bits,
                                                 (hipStream_t)stream)));
    return qc_qlinear_gemm(workspace, workspace_bytes, M, K, packed, w_scale, bits, N, bias, epi, Y,
                           ydt, stream);
}

// ---- test hooks for the GEMM's choice of kernel and its static schedule (host only) -------------

extern "C" int qc_debug_gemm_kernel(int64_t M, int64_t K, int64_t N, int bits) {
    if (M < 1 || K < 1 || N < 1 || check_gemm_supported(M, K, N, bits) != QC_OK) return 0;
    return gemm_resident_chosen(M, N, K, bits) ? 2 : 1;
}

extern "C" int qc_debug_gemm_schedule(int64_t M, int64_t N, int block, int32_t *pairs, int cap) {
    if (M < 1 || N < 1 || block < 0 || block >= gemm_resident_blocks() || cap < 0) return -1;
    const int64_t m_tiles = round_up(M, kTileM) / kTileM, n_tiles = round_up(N, kTileN) / kTileN;
    if (m_tiles * n_tiles > 0x7fffffffLL) return -1;
    return resident_block_rounds(block, gemm_resident_blocks(), (int)n_tiles, (int)m_tiles, pairs, cap);
}
