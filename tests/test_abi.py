"""Host-side checks that need no GPU: the library loads, exports what include/qc.h declares,
its size queries are right and argument errors are caught before any launch."""
import ctypes
import os
import re

import pytest

from paper_2503_06545_amd import binding as qc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "qc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(qc.EXPORTS)
    lib = ctypes.CDLL(qc.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_binding_constants_equal_the_header():
    text = open(os.path.join(ROOT, "include", "qc.h")).read()
    for name, value in re.findall(r"#define\s+(QC_MAX_\w+)\s+(\d+)", text):
        assert getattr(qc, name) == int(value), name
    # enumerators: "NAME = value" inside the typedef enums
    enums = dict(re.findall(r"\b(QC_[A-Z0-9_]+)\s*=\s*(\d+)", re.sub(r"/\*.*?\*/", "", text, flags=re.S)))
    assert len(enums) >= 13
    for name, value in enums.items():
        assert getattr(qc, name) == int(value), name


def test_version_and_status_strings():
    assert qc.qc_version() == 1003
    assert qc.status_string(0) == "QC_OK"
    for s in range(1, 5):
        assert qc.status_string(s).startswith("QC_ERR_")


def test_size_queries():
    # int8: padded to 128 channels x 192 k, plus a 256-byte header
    assert qc.qc_packed_weight_bytes(3456, 1152, 8) == 256 + 3456 * 1152
    assert qc.qc_packed_weight_bytes(1152, 4608, 4) == 256 + 1152 * 4608 // 2
    assert qc.qc_packed_weight_bytes(200, 100, 8) == 256 + 256 * 192
    assert qc.qc_packed_weight_bytes(10, 15, 4) == 0          # odd K with 4 bits
    assert qc.qc_packed_weight_bytes(10, 16, 5) == 0
    assert qc.qc_packed_weight_bytes(0, 16, 8) == 0
    assert qc.qc_packed_weight_bytes(10, qc.QC_MAX_K + 1, 8) == 0
    assert qc.qc_packed_weight_bytes((1 << 26) + 1, 16, 8) == 0
    assert qc.qc_qlinear_workspace_bytes(16384, 1152, 3456) == 16384 * 4 + 16384 * 1152
    assert qc.qc_qlinear_workspace_bytes(300, 100, 7) == 512 * 4 + 512 * 192
    assert qc.qc_qlinear_workspace_bytes(0, 100, 7) == 0
    assert qc.qc_latent_delta_workspace_bytes(1 << 22) == 256 * 16
    assert qc.qc_latent_delta_workspace_bytes(0) == 0


def test_argument_errors_come_before_any_launch():
    A = 0x10000  # a fake, aligned, never dereferenced address: every call below must fail first
    assert qc.qc_quant_act(None, qc.QC_BF16, 4, 16, A, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_quant_act(A, qc.QC_BF16, 0, 16, A, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_quant_act(A, 7, 4, 16, A, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_quant_act(A + 2, qc.QC_BF16, 4, 16, A, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_quant_act(A, qc.QC_BF16, 4, qc.QC_MAX_K + 1, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_bits(A, qc.QC_BF16, 4, 16, 5, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_bits(None, qc.QC_BF16, 4, 16, 6, A, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_qlinear_quant_bits(A, qc.QC_BF16, 4, 16, 3, A, 1 << 30) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_qlinear_quant_bits(A, qc.QC_BF16, 4, 16, 6, A, 16) == qc.QC_ERR_WORKSPACE
    assert qc.qc_qlinear_act_bits(A, qc.QC_BF16, 4, 16, 7, A, A, 8, 8, None, qc.QC_EPI_NONE, A,
                                  qc.QC_OUT_BF16, A, 1 << 30) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_pack_weight(A, 8, 15, 4, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_pack_weight(A, 8, 16, 3, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_pack_weight(A, 8, 16, 8, A + 16, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_pack_weight(A, 8, 16, 8, None, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_unpack_weight_codes(A, 8, 15, 4, A) == qc.QC_ERR_UNSUPPORTED
    ok = dict(X=A, xdt=qc.QC_BF16, M=4, K=16, packed=A, w_scale=A, bits=8, N=8, bias=None,
              epi=qc.QC_EPI_NONE, Y=A, ydt=qc.QC_OUT_BF16, workspace=A, workspace_bytes=1 << 30)
    def call(**kw):
        return qc.qc_qlinear(**{**ok, **kw})
    assert call(X=None) == qc.QC_ERR_INVALID_ARG
    assert call(workspace=None) == qc.QC_ERR_INVALID_ARG
    assert call(epi=9) == qc.QC_ERR_INVALID_ARG
    assert call(ydt=9) == qc.QC_ERR_INVALID_ARG
    assert call(bias=A + 4) == qc.QC_ERR_INVALID_ARG
    assert call(bits=4, K=15) == qc.QC_ERR_UNSUPPORTED
    assert call(bits=2) == qc.QC_ERR_UNSUPPORTED
    assert call(workspace_bytes=16) == qc.QC_ERR_WORKSPACE
    assert qc.qc_latent_delta(A, A, 0, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_latent_delta(A, A + 4, 8, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_latent_delta(A, A, 8, A, A, 8) == qc.QC_ERR_WORKSPACE
    assert qc.qc_layer_similarity(A, None, qc.QC_F32, 8, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_layer_similarity(A, A, 5, 8, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_layer_similarity(A, A, qc.QC_BF16, 8, A, A, 8) == qc.QC_ERR_WORKSPACE
    assert qc.qc_layer_similarity_workspace_bytes(100) == 256 * 24
    # asymmetric activations
    assert qc.qc_quant_act_asym(A, qc.QC_BF16, 4, 1152, 8, A, A, None) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_quant_act_asym(A, qc.QC_BF16, 4, 1152, 5, A, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_asym(A, qc.QC_BF16, 4, 1000, 8, A, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_asym(A, qc.QC_BF16, 4, 9216 + 16, 8, A, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_weight_row_sums(A, 8, 15, 4, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_weight_row_sums(A, 8, 16, 8, None) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_qlinear_asym(A, qc.QC_BF16, 4, 1152, 8, A, A, None, 8, 8, None, qc.QC_EPI_NONE, A,
                              qc.QC_OUT_BF16, A, 1 << 30) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_qlinear_asym(A, qc.QC_BF16, 4, 1152, 8, A, A, A, 8, 8, None, qc.QC_EPI_NONE, A,
                              qc.QC_OUT_BF16, A, 64) == qc.QC_ERR_WORKSPACE
    assert qc.qc_qlinear_asym(A, qc.QC_BF16, 4, 1144, 8, A, A, A, 8, 8, None, qc.QC_EPI_NONE, A,
                              qc.QC_OUT_BF16, A, 1 << 30) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_debug_workspace_act_asym(A, 4, 1152, 7, A, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_qlinear_asym_quant(A, qc.QC_BF16, 4, 1152, 8, A, 64) == qc.QC_ERR_WORKSPACE
    assert qc.qc_qlinear_asym_quant(A, qc.QC_BF16, 4, 1152, 3, A, 1 << 30) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_qlinear_asym_gemm(A, 1 << 30, 4, 1152, A, A, None, 8, 8, None, qc.QC_EPI_NONE, A,
                                   qc.QC_OUT_BF16) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_qlinear_asym_gemm(A, 64, 4, 1152, A, A, A, 8, 8, None, qc.QC_EPI_NONE, A,
                                   qc.QC_OUT_BF16) == qc.QC_ERR_WORKSPACE
    assert qc.qc_qlinear_asym_workspace_bytes(300, 100, 7) == 2 * 512 * 4 + 512 * 192
    # one scale per tensor
    assert qc.qc_quant_act_tensor(A, qc.QC_BF16, 4, 16, 8, A, A, None, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_quant_act_tensor(A, qc.QC_BF16, 4, 16, 5, A, A, A, 1 << 20) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_tensor(A, qc.QC_BF16, 4, 16, 8, A, A, A, 16) == qc.QC_ERR_WORKSPACE
    assert qc.qc_quant_act_tensor_workspace_bytes(4, 16) == 1024
    assert qc.qc_qlinear_tensor_workspace_bytes(300, 100, 7) == 512 * 4 + 512 * 192 + 1024
    assert qc.qc_qlinear_tensor(A, qc.QC_BF16, 4, 16, 8, A, A, 8, 8, None, qc.QC_EPI_NONE, A,
                                qc.QC_OUT_BF16, A, qc.qc_qlinear_workspace_bytes(4, 16, 8)) == qc.QC_ERR_WORKSPACE
    assert qc.qc_qlinear_tensor(A, qc.QC_BF16, 4, 16, 8, A, A, 8, 8, None, 7, A,
                                qc.QC_OUT_BF16, A, 1 << 30) == qc.QC_ERR_INVALID_ARG
    # rotation: block sizes, divisibility, the K limit of the vector path
    assert qc.qc_quant_act_rot(A, qc.QC_BF16, 4, 1152, 8, 0, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_rot(A, qc.QC_BF16, 4, 1152, 8, 48, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_rot(A, qc.QC_BF16, 4, 1152, 8, 256, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_rot(A, qc.QC_BF16, 4, 1000, 8, 64, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_rot(A, qc.QC_BF16, 4, 9216 + 128, 8, 128, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_quant_act_rot(None, qc.QC_BF16, 4, 1152, 8, 128, A, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_pack_weight_rot(A, 8, 1152, 8, 100, A, A) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_pack_weight_rot(A, 8, 1152, 8, 128, None, A) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_qlinear_quant_rot(A, qc.QC_BF16, 4, 1152, 8, 128, A, 16) == qc.QC_ERR_WORKSPACE
    assert qc.qc_qlinear_quant_rot(A, qc.QC_BF16, 4, 1152, 8, 8, A, 1 << 30) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_qlinear_rot(A, qc.QC_BF16, 4, 1152, 8, 96, A, A, 8, 8, None, qc.QC_EPI_NONE, A,
                             qc.QC_OUT_BF16, A, 1 << 30) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_qlinear_rot(A, qc.QC_BF16, 4, 1152, 8, 128, A, A, 8, 8, None, qc.QC_EPI_NONE, None,
                             qc.QC_OUT_BF16, A, 1 << 30) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_frame_gradient_norm(None, qc.QC_F32, 4, 16, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_frame_gradient_norm(A, qc.QC_F32, 0, 16, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_frame_gradient_norm(A, 5, 4, 16, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_frame_gradient_norm(A, qc.QC_F32, 4, 16, A, A, 8) == qc.QC_ERR_WORKSPACE
    assert qc.qc_cumulative_variation(A, [A], 1, 0, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_cumulative_variation(A, None, 1, 64, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_cumulative_variation(A, [A, None], 2, 64, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_cumulative_variation(A, [A, A + 4], 2, 64, A, A, 1 << 20) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_cumulative_variation(A, [A] * 9, 9, 64, A, A, 1 << 20) == qc.QC_ERR_UNSUPPORTED
    assert qc.qc_cumulative_variation(A, [A] * 8, 8, 64, A, A, 64) == qc.QC_ERR_WORKSPACE
    assert qc.qc_frame_gradient_norm_workspace_bytes(16, 1152) == 256 * 8
    assert qc.qc_cumulative_variation_workspace_bytes(1 << 20, 3) == 256 * 8 * 8
    assert qc.qc_cumulative_variation_workspace_bytes(1 << 20, 9) == 0


def test_missing_library_is_a_loud_error(monkeypatch):
    monkeypatch.setattr(qc, "_lib", None)
    monkeypatch.setattr(qc, "LIB_PATH", "/nonexistent/libqc.so")
    with pytest.raises(ImportError):
        qc.lib()


def test_decision_rules_match_the_oracle_on_every_case_and_boundary():
    """Eq. (5), (6), (8), (10): host arithmetic, checked against the oracle's plain definitions."""
    import math

    import numpy as np

    import oracle
    f = lambda v: float(np.float32(v))
    grid = [f(v) for v in (-1.0, 0.0, 0.0999, 0.1, 0.3, 0.4999, 0.5, 0.8, 0.95, 0.951, 1.0, 9.0)]
    for d in grid:
        a = (f(0.1), f(0.5), 8, 4, 2)
        assert qc.qc_cache_interval(d, *a) == oracle.cache_interval(d, *a)
        b = (f(0.3), f(0.95), 8, 6, 4)
        assert qc.qc_activation_bits(d, *b) == oracle.activation_bits(d, *b)
        c = (f(0.8), f(0.95), f(0.25))
        assert qc.qc_prune_probability(d, *c) == oracle.prune_probability(d, *c)
    # equal thresholds: the middle case is empty for Eq. (6) and (8), a point for Eq. (10)
    assert qc.qc_cache_interval(0.5, 0.5, 0.5, 8, 4, 2) == oracle.cache_interval(0.5, 0.5, 0.5, 8, 4, 2) == 2
    assert qc.qc_prune_probability(0.5, 0.5, 0.5, 0.25) == oracle.prune_probability(0.5, 0.5, 0.5, 0.25) == 0.25
    for l1, k, g in [(12.0, 3, 0.5), (1e6, 7, 3.25), (0.0, 1, 5.0)]:
        want = np.float32(oracle.divergence_score(l1, k, g))
        assert np.float32(qc.qc_divergence_score(l1, k, g)) == want
    # error behaviour: NaN or thresholds in the wrong order
    nan = float("nan")
    assert qc.qc_cache_interval(nan, 0.1, 0.5, 8, 4, 2) == -1
    assert qc.qc_cache_interval(0.2, 0.5, 0.1, 8, 4, 2) == -1
    assert qc.qc_activation_bits(0.2, nan, 0.5, 8, 6, 4) == -1
    assert math.isnan(qc.qc_prune_probability(nan, 0.8, 0.95, 0.25))
    assert math.isnan(qc.qc_prune_probability(0.9, 0.95, 0.8, 0.25))
    assert math.isnan(qc.qc_divergence_score(1.0, 0, 1.0))


def test_build_reads_the_compilers_resource_remarks():
    """build.py fails when a kernel needs scratch memory; its parser of the compiler's remarks
    must find the kernel name, the VGPR count, the scratch bytes and the occupancy."""
    from paper_2503_06545_amd import build as qc_build
    text = (
        "csrc/x.hip:9:1: remark: Function Name: _ZN2qc4kernEv [-Rpass-analysis=kernel-resource-usage]\n"
        "csrc/x.hip:9:1: remark:     VGPRs: 212 [-Rpass-analysis=kernel-resource-usage]\n"
        "csrc/x.hip:9:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
        "csrc/x.hip:9:1: remark:     Occupancy [waves/SIMD]: 2 [-Rpass-analysis=kernel-resource-usage]\n"
        "csrc/x.hip:40:1: remark: Function Name: _ZN2qc5spillEv [-Rpass-analysis=kernel-resource-usage]\n"
        "csrc/x.hip:40:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]\n"
        "csrc/x.hip:40:1: remark:     ScratchSize [bytes/lane]: 76 [-Rpass-analysis=kernel-resource-usage]\n"
        "csrc/x.hip:40:1: remark:     Occupancy [waves/SIMD]: 2 [-Rpass-analysis=kernel-resource-usage]\n")
    assert qc_build._resources(text) == [("_ZN2qc4kernEv", 212, 0, 2), ("_ZN2qc5spillEv", 256, 76, 2)]
    # the report of the library that is built here: every kernel, none with scratch memory
    report = open(qc_build.RESOURCE_REPORT).read().splitlines()
    assert len(report) >= 60 and all("scratch_bytes_per_lane=0" in line for line in report)
    assert sum("gemm_kernel" in line for line in report) == 26
