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

extern "C" int qc_version(void) { return 1002; }

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

extern "C" size_t qc_qlinear_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M < 1 || K < 1 || N < 1 || K > QC_MAX_K) return 0;
    return act_workspace(M, K).total_bytes;
}

namespace {
bool act_bits_ok(int b) { return b == 8 || b == 6 || b == 4; }
}  // namespace

namespace {
// rot_block 0 = no rotation
qc_status quant_act_any(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                        int rot_block, int8_t *qx, float *x_scale, void *stream) {
    if (!X || !qx || !x_scale || M < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16) || !aligned(qx, 16) || !aligned(x_scale, 4)) return QC_ERR_INVALID_ARG;
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (K > QC_MAX_K || (M + 3) / 4 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (rot_block && !quant_rotation_supported(K, rot_block)) return QC_ERR_UNSUPPORTED;
    hipError_t e = launch_quant_act(X, xdt, M, K, qx, nullptr, 0, x_scale, act_bits, rot_block,
                                    (hipStream_t)stream);
    return e == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

qc_status qlinear_quant_any(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                            int rot_block, void *workspace, size_t workspace_bytes, void *stream) {
    if (!X || !workspace || M < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16) || !aligned(workspace, 256)) return QC_ERR_INVALID_ARG;
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (K > QC_MAX_K || (M + 3) / 4 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (rot_block && !quant_rotation_supported(K, rot_block)) return QC_ERR_UNSUPPORTED;
    const ActWorkspace ws = act_workspace(M, K);
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    uint8_t *base = (uint8_t *)workspace;
    hipError_t e = launch_quant_act(X, xdt, M, K, nullptr, base + ws.scale_bytes, ws.KF,
                                    (float *)base, act_bits, rot_block, (hipStream_t)stream);
    return e == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

qc_status qlinear_any(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                      int rot_block, const void *packed, const float *w_scale, int bits, int64_t N,
                      const float *bias, qc_epilogue epi, void *Y, qc_out ydt, void *workspace,
                      size_t workspace_bytes, void *stream) {
    // every argument is checked before the first launch, so a failed call has no side effect
    if (!X || !packed || !w_scale || !Y || !workspace || M < 1 || K < 1 || N < 1)
        return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (epi != QC_EPI_NONE && epi != QC_EPI_GELU_TANH && epi != QC_EPI_GELU_ERF) return QC_ERR_INVALID_ARG;
    if (ydt != QC_OUT_F32 && ydt != QC_OUT_BF16 && ydt != QC_OUT_I32_ACC) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16) || !aligned(packed, 256) || !aligned(w_scale, 16) || !aligned(Y, 16) ||
        !aligned(workspace, 256) || (bias && !aligned(bias, 16)))
        return QC_ERR_INVALID_ARG;
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (qc_packed_weight_bytes(N, K, bits) == 0) return QC_ERR_UNSUPPORTED;
    if (rot_block && !quant_rotation_supported(K, rot_block)) return QC_ERR_UNSUPPORTED;
    if ((M + 3) / 4 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    const ActWorkspace ws = act_workspace(M, K);
    if ((ws.Mp / kTileM) * (round_up(N, kTileN) / kTileN) > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    qc_status st = qlinear_quant_any(X, xdt, M, K, act_bits, rot_block, workspace, workspace_bytes,
                                     stream);
    if (st != QC_OK) return st;
    return qc_qlinear_gemm(workspace, workspace_bytes, M, K, packed, w_scale, bits, N, bias, epi, Y,
                           ydt, stream);
}
}  // namespace

extern "C" qc_status qc_quant_act_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                       int act_bits, int8_t *qx, float *x_scale, void *stream) {
    return quant_act_any(X, xdt, M, K, act_bits, 0, qx, x_scale, stream);
}

extern "C" qc_status qc_quant_act_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                      int act_bits, int rot_block, int8_t *qx, float *x_scale,
                                      void *stream) {
    if (rot_block == 0) return QC_ERR_UNSUPPORTED;
    return quant_act_any(X, xdt, M, K, act_bits, rot_block, qx, x_scale, stream);
}

extern "C" qc_status qc_qlinear_quant_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                          int act_bits, int rot_block, void *workspace,
                                          size_t workspace_bytes, void *stream) {
    if (rot_block == 0) return QC_ERR_UNSUPPORTED;
    return qlinear_quant_any(X, xdt, M, K, act_bits, rot_block, workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                                    int rot_block, const void *packed, const float *w_scale,
                                    int bits, int64_t N, const float *bias, qc_epilogue epi, void *Y,
                                    qc_out ydt, void *workspace, size_t workspace_bytes,
                                    void *stream) {
    if (rot_block == 0) return QC_ERR_UNSUPPORTED;
    return qlinear_any(X, xdt, M, K, act_bits, rot_block, packed, w_scale, bits, N, bias, epi, Y,
                       ydt, workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_quant_act(const void *X, qc_dtype xdt, int64_t M, int64_t K, int8_t *qx,
                                  float *x_scale, void *stream) {
    return qc_quant_act_bits(X, xdt, M, K, 8, qx, x_scale, stream);
}

extern "C" qc_status qc_qlinear_quant_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                           int act_bits, void *workspace, size_t workspace_bytes,
                                           void *stream) {
    return qlinear_quant_any(X, xdt, M, K, act_bits, 0, workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear_quant(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                      void *workspace, size_t workspace_bytes, void *stream) {
    return qc_qlinear_quant_bits(X, xdt, M, K, 8, workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear_gemm(const void *workspace, size_t workspace_bytes, int64_t M,
                                     int64_t K, const void *packed, const float *w_scale, int bits,
                                     int64_t N, const float *bias, qc_epilogue epi, void *Y,
                                     qc_out ydt, void *stream) {
    if (!packed || !w_scale || !Y || !workspace || M < 1 || K < 1 || N < 1)
        return QC_ERR_INVALID_ARG;
    if (epi != QC_EPI_NONE && epi != QC_EPI_GELU_TANH && epi != QC_EPI_GELU_ERF) return QC_ERR_INVALID_ARG;
    if (ydt != QC_OUT_F32 && ydt != QC_OUT_BF16 && ydt != QC_OUT_I32_ACC) return QC_ERR_INVALID_ARG;
    if (!aligned(packed, 256) || !aligned(w_scale, 16) || !aligned(Y, 16) ||
        !aligned(workspace, 256) || (bias && !aligned(bias, 16)))
        return QC_ERR_INVALID_ARG;
    if (qc_packed_weight_bytes(N, K, bits) == 0) return QC_ERR_UNSUPPORTED;
    const ActWorkspace ws = act_workspace(M, K);
    const int64_t tiles = (ws.Mp / kTileM) * (round_up(N, kTileN) / kTileN);
    if (tiles > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    const uint8_t *base = (const uint8_t *)workspace;
    hipError_t e = launch_gemm(base + ws.scale_bytes, (const float *)base, (const uint8_t *)packed,
                               w_scale, bias, Y, M, N, K, bits, epi, ydt, nullptr, nullptr,
                               (hipStream_t)stream);
    return e == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" qc_status qc_qlinear_act_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                         int act_bits, const void *packed, const float *w_scale,
                                         int bits, int64_t N, const float *bias, qc_epilogue epi,
                                         void *Y, qc_out ydt, void *workspace,
                                         size_t workspace_bytes, void *stream) {
    return qlinear_any(X, xdt, M, K, act_bits, 0, packed, w_scale, bits, N, bias, epi, Y, ydt,
                       workspace, workspace_bytes, stream);
}

extern "C" qc_status qc_qlinear(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                const void *packed, const float *w_scale, int bits, int64_t N,
                                const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                                void *workspace, size_t workspace_bytes, void *stream) {
    return qc_qlinear_act_bits(X, xdt, M, K, 8, packed, w_scale, bits, N, bias, epi, Y, ydt,
                               workspace, workspace_bytes, stream);
}

// ---- asymmetric activations (Section 3.1 Eq. (3)-(4) as printed) --------------------------------

extern "C" size_t qc_qlinear_asym_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (M < 1 || K < 1 || N < 1 || K > QC_MAX_K) return 0;
    return act_workspace_asym(M, K).total_bytes;
}

extern "C" qc_status qc_quant_act_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                       int act_bits, uint8_t *qx, float *x_scale, float *x_zero,
                                       void *stream) {
    if (!X || !qx || !x_scale || !x_zero || M < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16) || !aligned(qx, 16) || !aligned(x_scale, 4) || !aligned(x_zero, 4))
        return QC_ERR_INVALID_ARG;
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (!quant_vector_path(K) || (M + 7) / 8 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    hipError_t e = launch_quant_act_asym(X, xdt, M, K, qx, nullptr, 0, x_scale, x_zero, act_bits,
                                         false, (hipStream_t)stream);
    return e == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" qc_status qc_qlinear_asym_quant(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                           int act_bits, void *workspace, size_t workspace_bytes,
                                           void *stream) {
    if (!X || !workspace || M < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16) || !aligned(workspace, 256)) return QC_ERR_INVALID_ARG;
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (!quant_vector_path(K) || (M + 7) / 8 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    const ActWorkspaceAsym ws = act_workspace_asym(M, K);
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    uint8_t *base = (uint8_t *)workspace;
    hipError_t e = launch_quant_act_asym(X, xdt, M, K, nullptr, base + ws.codes_offset, ws.sym.KF,
                                         (float *)base, (float *)(base + ws.corr_offset), act_bits,
                                         true, (hipStream_t)stream);
    return e == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" qc_status qc_qlinear_asym_gemm(const void *workspace, size_t workspace_bytes, int64_t M,
                                          int64_t K, const void *packed, const float *w_scale,
                                          const int32_t *w_row_sums, int bits, int64_t N,
                                          const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                                          void *stream) {
    if (!packed || !w_scale || !w_row_sums || !Y || !workspace || M < 1 || K < 1 || N < 1)
        return QC_ERR_INVALID_ARG;
    if (epi != QC_EPI_NONE && epi != QC_EPI_GELU_TANH && epi != QC_EPI_GELU_ERF) return QC_ERR_INVALID_ARG;
    if (ydt != QC_OUT_F32 && ydt != QC_OUT_BF16 && ydt != QC_OUT_I32_ACC) return QC_ERR_INVALID_ARG;
    if (!aligned(packed, 256) || !aligned(w_scale, 16) || !aligned(w_row_sums, 16) ||
        !aligned(Y, 16) || !aligned(workspace, 256) || (bias && !aligned(bias, 16)))
        return QC_ERR_INVALID_ARG;
    if (qc_packed_weight_bytes(N, K, bits) == 0 || !quant_vector_path(K)) return QC_ERR_UNSUPPORTED;
    const ActWorkspaceAsym ws = act_workspace_asym(M, K);
    if ((ws.sym.Mp / kTileM) * (round_up(N, kTileN) / kTileN) > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    const uint8_t *base = (const uint8_t *)workspace;
    hipError_t e = launch_gemm(base + ws.codes_offset, (const float *)base, (const uint8_t *)packed,
                               w_scale, bias, Y, M, N, K, bits, epi, ydt,
                               (const float *)(base + ws.corr_offset), w_row_sums,
                               (hipStream_t)stream);
    return e == hipSuccess ? QC_OK : QC_ERR_DEVICE;
}

extern "C" qc_status qc_qlinear_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K,
                                     int act_bits, const void *packed, const float *w_scale,
                                     const int32_t *w_row_sums, int bits, int64_t N,
                                     const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                                     void *workspace, size_t workspace_bytes, void *stream) {
    // every argument is checked before the first launch, so a failed call has no side effect
    if (!X || !packed || !w_scale || !w_row_sums || !Y || !workspace || M < 1 || K < 1 || N < 1)
        return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (epi != QC_EPI_NONE && epi != QC_EPI_GELU_TANH && epi != QC_EPI_GELU_ERF) return QC_ERR_INVALID_ARG;
    if (ydt != QC_OUT_F32 && ydt != QC_OUT_BF16 && ydt != QC_OUT_I32_ACC) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16) || !aligned(packed, 256) || !aligned(w_scale, 16) ||
        !aligned(w_row_sums, 16) || !aligned(Y, 16) || !aligned(workspace, 256) ||
        (bias && !aligned(bias, 16)))
        return QC_ERR_INVALID_ARG;
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (qc_packed_weight_bytes(N, K, bits) == 0 || !quant_vector_path(K)) return QC_ERR_UNSUPPORTED;
    if ((M + 7) / 8 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    const ActWorkspaceAsym ws = act_workspace_asym(M, K);
    if ((ws.sym.Mp / kTileM) * (round_up(N, kTileN) / kTileN) > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (workspace_bytes < ws.total_bytes) return QC_ERR_WORKSPACE;
    qc_status st = qc_qlinear_asym_quant(X, xdt, M, K, act_bits, workspace, workspace_bytes, stream);
    if (st != QC_OK) return st;
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
    if (!X || !qx || !x_scale || !workspace || M < 1 || K < 1) return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16) || !aligned(qx, 16) || !aligned(x_scale, 4) || !aligned(workspace, 256))
        return QC_ERR_INVALID_ARG;
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (K > QC_MAX_K || (M + 3) / 4 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (workspace_bytes < tensor_partials_bytes()) return QC_ERR_WORKSPACE;
    hipError_t e = launch_quant_act_tensor(X, xdt, M, K, qx, nullptr, 0, x_scale, true,
                                           (float *)workspace, act_bits, (hipStream_t)stream);
    return e == hipSuccess ? QC_OK : QC_ERR_DEVICE;
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
    if (!X || !packed || !w_scale || !Y || !workspace || M < 1 || K < 1 || N < 1)
        return QC_ERR_INVALID_ARG;
    if (xdt != QC_F32 && xdt != QC_BF16) return QC_ERR_INVALID_ARG;
    if (epi != QC_EPI_NONE && epi != QC_EPI_GELU_TANH && epi != QC_EPI_GELU_ERF) return QC_ERR_INVALID_ARG;
    if (ydt != QC_OUT_F32 && ydt != QC_OUT_BF16 && ydt != QC_OUT_I32_ACC) return QC_ERR_INVALID_ARG;
    if (!aligned(X, 16) || !aligned(packed, 256) || !aligned(w_scale, 16) || !aligned(Y, 16) ||
        !aligned(workspace, 256) || (bias && !aligned(bias, 16)))
        return QC_ERR_INVALID_ARG;
    if (!act_bits_ok(act_bits)) return QC_ERR_UNSUPPORTED;
    if (qc_packed_weight_bytes(N, K, bits) == 0) return QC_ERR_UNSUPPORTED;
    if ((M + 3) / 4 > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    const ActWorkspace ws = act_workspace(M, K);
    if ((ws.Mp / kTileM) * (round_up(N, kTileN) / kTileN) > 0x7fffffffLL) return QC_ERR_UNSUPPORTED;
    if (workspace_bytes < ws.total_bytes + tensor_partials_bytes()) return QC_ERR_WORKSPACE;
    // [ the workspace of qc_qlinear ][ slab maxima ]: the first part is what qc_qlinear_gemm and
    // qc_debug_workspace_act read, with the one scale repeated for every token
    uint8_t *base = (uint8_t *)workspace;
    hipError_t e = launch_quant_act_tensor(X, xdt, M, K, nullptr, base + ws.scale_bytes, ws.KF,
                                           (float *)base, false, (float *)(base + ws.total_bytes),
                                           act_bits, (hipStream_t)stream);
    if (e != hipSuccess) return QC_ERR_DEVICE;
    return qc_qlinear_gemm(workspace, workspace_bytes, M, K, packed, w_scale, bits, N, bias, epi, Y,
                           ydt, stream);
}
