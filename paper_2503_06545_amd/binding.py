"""ctypes binding of libqc.so: argument marshalling only.

The functions named like the C entry points take raw device addresses (ints), exactly as
``include/qc.h`` declares them.  The ``*_t`` helpers take torch tensors, which here are
nothing but device memory and a stream; every arithmetic step runs inside libqc's kernels.
There is no fallback: if the library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqc.so")

QC_OK, QC_ERR_INVALID_ARG, QC_ERR_UNSUPPORTED, QC_ERR_WORKSPACE, QC_ERR_DEVICE = range(5)
QC_F32, QC_BF16 = 0, 1
QC_EPI_NONE, QC_EPI_GELU_TANH, QC_EPI_GELU_ERF = 0, 1, 2
QC_OUT_F32, QC_OUT_BF16, QC_OUT_I32_ACC = 0, 1, 2
QC_MAX_K = 131072
QC_MAX_N = 67108864
QC_MAX_PREV = 8

EXPORTS = (
    "qc_status_string", "qc_version", "qc_packed_weight_bytes", "qc_qlinear_workspace_bytes",
    "qc_latent_delta_workspace_bytes", "qc_pack_weight", "qc_unpack_weight_codes", "qc_quant_act",
    "qc_qlinear", "qc_qlinear_quant", "qc_qlinear_gemm", "qc_quant_act_bits",
    "qc_qlinear_quant_bits", "qc_qlinear_act_bits", "qc_layer_similarity_workspace_bytes",
    "qc_layer_similarity", "qc_debug_workspace_act", "qc_debug_gemm_kernel", "qc_debug_gemm_schedule",
    "qc_latent_delta",
    "qc_frame_gradient_norm_workspace_bytes", "qc_frame_gradient_norm",
    "qc_cumulative_variation_workspace_bytes", "qc_cumulative_variation",
    "qc_divergence_score", "qc_cache_interval", "qc_activation_bits", "qc_prune_probability",
    "qc_pack_weight_rot", "qc_quant_act_rot", "qc_qlinear_quant_rot", "qc_qlinear_rot",
    "qc_qlinear_asym_workspace_bytes", "qc_weight_row_sums", "qc_quant_act_asym",
    "qc_qlinear_asym", "qc_debug_workspace_act_asym", "qc_qlinear_asym_quant",
    "qc_qlinear_asym_gemm", "qc_quant_act_tensor_workspace_bytes", "qc_quant_act_tensor",
    "qc_qlinear_tensor_workspace_bytes", "qc_qlinear_tensor", "qc_latent_delta_static",
)


class QcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libqc.so (built in-tree by ``paper_2503_06545_amd.build``).  No fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2503_06545_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        L.qc_status_string.restype = ctypes.c_char_p
        L.qc_status_string.argtypes = [i32]
        L.qc_version.restype = i32
        L.qc_version.argtypes = []
        L.qc_packed_weight_bytes.restype = sz
        L.qc_packed_weight_bytes.argtypes = [i64, i64, i32]
        L.qc_qlinear_workspace_bytes.restype = sz
        L.qc_qlinear_workspace_bytes.argtypes = [i64, i64, i64]
        L.qc_latent_delta_workspace_bytes.restype = sz
        L.qc_latent_delta_workspace_bytes.argtypes = [i64]
        L.qc_pack_weight.restype = i32
        L.qc_pack_weight.argtypes = [vp, i64, i64, i32, vp, vp, vp]
        L.qc_unpack_weight_codes.restype = i32
        L.qc_unpack_weight_codes.argtypes = [vp, i64, i64, i32, vp, vp]
        L.qc_quant_act.restype = i32
        L.qc_quant_act.argtypes = [vp, i32, i64, i64, vp, vp, vp]
        L.qc_qlinear.restype = i32
        L.qc_qlinear.argtypes = [vp, i32, i64, i64, vp, vp, i32, i64, vp, i32, vp, i32, vp, sz, vp]
        L.qc_qlinear_quant.restype = i32
        L.qc_qlinear_quant.argtypes = [vp, i32, i64, i64, vp, sz, vp]
        L.qc_qlinear_gemm.restype = i32
        L.qc_qlinear_gemm.argtypes = [vp, sz, i64, i64, vp, vp, i32, i64, vp, i32, vp, i32, vp]
        L.qc_quant_act_bits.restype = i32
        L.qc_quant_act_bits.argtypes = [vp, i32, i64, i64, i32, vp, vp, vp]
        L.qc_qlinear_quant_bits.restype = i32
        L.qc_qlinear_quant_bits.argtypes = [vp, i32, i64, i64, i32, vp, sz, vp]
        L.qc_qlinear_act_bits.restype = i32
        L.qc_qlinear_act_bits.argtypes = [vp, i32, i64, i64, i32, vp, vp, i32, i64, vp, i32, vp, i32,
                                          vp, sz, vp]
        L.qc_layer_similarity_workspace_bytes.restype = sz
        L.qc_layer_similarity_workspace_bytes.argtypes = [i64]
        L.qc_layer_similarity.restype = i32
        L.qc_layer_similarity.argtypes = [vp, vp, i32, i64, vp, vp, sz, vp]
        L.qc_debug_workspace_act.restype = i32
        L.qc_debug_workspace_act.argtypes = [vp, i64, i64, vp, vp, vp]
        L.qc_debug_gemm_kernel.restype = i32
        L.qc_debug_gemm_kernel.argtypes = [i64, i64, i64, i32]
        L.qc_debug_gemm_schedule.restype = i32
        L.qc_debug_gemm_schedule.argtypes = [i64, i64, i32, vp, i32]
        L.qc_latent_delta.restype = i32
        L.qc_latent_delta.argtypes = [vp, vp, i64, vp, vp, sz, vp]
        L.qc_latent_delta_static.restype = i32
        L.qc_latent_delta_static.argtypes = [vp, vp, i64, vp, vp]
        f32 = ctypes.c_float
        L.qc_qlinear_asym_workspace_bytes.restype = sz
        L.qc_qlinear_asym_workspace_bytes.argtypes = [i64, i64, i64]
        L.qc_weight_row_sums.restype = i32
        L.qc_weight_row_sums.argtypes = [vp, i64, i64, i32, vp, vp]
        L.qc_quant_act_asym.restype = i32
        L.qc_quant_act_asym.argtypes = [vp, i32, i64, i64, i32, vp, vp, vp, vp]
        L.qc_qlinear_asym.restype = i32
        L.qc_qlinear_asym.argtypes = [vp, i32, i64, i64, i32, vp, vp, vp, i32, i64, vp, i32, vp, i32,
                                      vp, sz, vp]
        L.qc_qlinear_asym_quant.restype = i32
        L.qc_qlinear_asym_quant.argtypes = [vp, i32, i64, i64, i32, vp, sz, vp]
        L.qc_qlinear_asym_gemm.restype = i32
        L.qc_qlinear_asym_gemm.argtypes = [vp, sz, i64, i64, vp, vp, vp, i32, i64, vp, i32, vp, i32, vp]
        L.qc_quant_act_tensor_workspace_bytes.restype = sz
        L.qc_quant_act_tensor_workspace_bytes.argtypes = [i64, i64]
        L.qc_quant_act_tensor.restype = i32
        L.qc_quant_act_tensor.argtypes = [vp, i32, i64, i64, i32, vp, vp, vp, sz, vp]
        L.qc_qlinear_tensor_workspace_bytes.restype = sz
        L.qc_qlinear_tensor_workspace_bytes.argtypes = [i64, i64, i64]
        L.qc_qlinear_tensor.restype = i32
        L.qc_qlinear_tensor.argtypes = [vp, i32, i64, i64, i32, vp, vp, i32, i64, vp, i32, vp, i32, vp,
                                        sz, vp]
        L.qc_debug_workspace_act_asym.restype = i32
        L.qc_debug_workspace_act_asym.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp]
        L.qc_pack_weight_rot.restype = i32
        L.qc_pack_weight_rot.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        L.qc_quant_act_rot.restype = i32
        L.qc_quant_act_rot.argtypes = [vp, i32, i64, i64, i32, i32, vp, vp, vp]
        L.qc_qlinear_quant_rot.restype = i32
        L.qc_qlinear_quant_rot.argtypes = [vp, i32, i64, i64, i32, i32, vp, sz, vp]
        L.qc_qlinear_rot.restype = i32
        L.qc_qlinear_rot.argtypes = [vp, i32, i64, i64, i32, i32, vp, vp, i32, i64, vp, i32, vp, i32,
                                     vp, sz, vp]
        L.qc_frame_gradient_norm_workspace_bytes.restype = sz
        L.qc_frame_gradient_norm_workspace_bytes.argtypes = [i64, i64]
        L.qc_frame_gradient_norm.restype = i32
        L.qc_frame_gradient_norm.argtypes = [vp, i32, i64, i64, vp, vp, sz, vp]
        L.qc_cumulative_variation_workspace_bytes.restype = sz
        L.qc_cumulative_variation_workspace_bytes.argtypes = [i64, i32]
        L.qc_cumulative_variation.restype = i32
        L.qc_cumulative_variation.argtypes = [vp, ctypes.POINTER(vp), i32, i64, vp, vp, sz, vp]
        L.qc_divergence_score.restype = f32
        L.qc_divergence_score.argtypes = [f32, i32, f32]
        L.qc_cache_interval.restype = i32
        L.qc_cache_interval.argtypes = [f32, f32, f32, i32, i32, i32]
        L.qc_activation_bits.restype = i32
        L.qc_activation_bits.argtypes = [f32, f32, f32, i32, i32, i32]
        L.qc_prune_probability.restype = f32
        L.qc_prune_probability.argtypes = [f32, f32, f32, f32]
        _lib = L
    return _lib


# ---- the C entry points, same names, raw addresses ---------------------------------------

def status_string(status: int) -> str:
    return lib().qc_status_string(int(status)).decode()


def qc_version() -> int:
    return int(lib().qc_version())


def qc_packed_weight_bytes(N: int, K: int, bits: int) -> int:
    return int(lib().qc_packed_weight_bytes(N, K, bits))


def qc_qlinear_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().qc_qlinear_workspace_bytes(M, K, N))


def qc_latent_delta_workspace_bytes(n: int) -> int:
    return int(lib().qc_latent_delta_workspace_bytes(n))


def qc_pack_weight(W, N, K, bits, packed, w_scale, stream=0) -> int:
    return int(lib().qc_pack_weight(W, N, K, bits, packed, w_scale, stream))


def qc_unpack_weight_codes(packed, N, K, bits, codes, stream=0) -> int:
    return int(lib().qc_unpack_weight_codes(packed, N, K, bits, codes, stream))


def qc_quant_act(X, xdt, M, K, qx, x_scale, stream=0) -> int:
    return int(lib().qc_quant_act(X, xdt, M, K, qx, x_scale, stream))


def qc_qlinear(X, xdt, M, K, packed, w_scale, bits, N, bias, epi, Y, ydt, workspace,
               workspace_bytes, stream=0) -> int:
    return int(lib().qc_qlinear(X, xdt, M, K, packed, w_scale, bits, N, bias, epi, Y, ydt,
                                workspace, workspace_bytes, stream))


def qc_qlinear_quant(X, xdt, M, K, workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_qlinear_quant(X, xdt, M, K, workspace, workspace_bytes, stream))


def qc_qlinear_gemm(workspace, workspace_bytes, M, K, packed, w_scale, bits, N, bias, epi, Y, ydt,
                    stream=0) -> int:
    return int(lib().qc_qlinear_gemm(workspace, workspace_bytes, M, K, packed, w_scale, bits, N,
                                     bias, epi, Y, ydt, stream))


def qc_quant_act_bits(X, xdt, M, K, act_bits, qx, x_scale, stream=0) -> int:
    return int(lib().qc_quant_act_bits(X, xdt, M, K, act_bits, qx, x_scale, stream))


def qc_qlinear_quant_bits(X, xdt, M, K, act_bits, workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_qlinear_quant_bits(X, xdt, M, K, act_bits, workspace, workspace_bytes,
                                           stream))


def qc_qlinear_act_bits(X, xdt, M, K, act_bits, packed, w_scale, bits, N, bias, epi, Y, ydt,
                        workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_qlinear_act_bits(X, xdt, M, K, act_bits, packed, w_scale, bits, N, bias,
                                         epi, Y, ydt, workspace, workspace_bytes, stream))


def qc_layer_similarity_workspace_bytes(n: int) -> int:
    return int(lib().qc_layer_similarity_workspace_bytes(n))


def qc_layer_similarity(a, b, dt, n, out4, workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_layer_similarity(a, b, dt, n, out4, workspace, workspace_bytes, stream))


def qc_debug_workspace_act(workspace, M, K, qx, x_scale, stream=0) -> int:
    return int(lib().qc_debug_workspace_act(workspace, M, K, qx, x_scale, stream))


def qc_debug_gemm_kernel(M, K, N, bits) -> int:
    return int(lib().qc_debug_gemm_kernel(M, K, N, bits))


def qc_debug_gemm_schedule(M, N, block, pairs, cap) -> int:
    return int(lib().qc_debug_gemm_schedule(M, N, block, pairs, cap))


def gemm_schedule(M: int, N: int, block: int):
    """The (channel tile, token chunk) rounds of one block of the resident GEMM kernel (host only)."""
    n = qc_debug_gemm_schedule(M, N, block, None, 0)
    if n < 0:
        raise QcError(QC_ERR_INVALID_ARG, "qc_debug_gemm_schedule")
    buf = (ctypes.c_int32 * (2 * max(n, 1)))()
    qc_debug_gemm_schedule(M, N, block, ctypes.cast(buf, ctypes.c_void_p), n)
    return [(buf[2 * i], buf[2 * i + 1]) for i in range(n)]


def qc_latent_delta(cur, prev, n, out3, workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_latent_delta(cur, prev, n, out3, workspace, workspace_bytes, stream))


QC_LATENT_DELTA_STATIC_MAX_N = 1 << 30


def qc_latent_delta_static(cur, prev, n, out3, stream=0) -> int:
    return int(lib().qc_latent_delta_static(cur, prev, n, out3, stream))


# ---- tensor helpers: allocate outputs with torch, pass addresses and the current stream ----

def qc_pack_weight_rot(W, N, K, bits, rot_block, packed, w_scale, stream=0) -> int:
    return int(lib().qc_pack_weight_rot(W, N, K, bits, rot_block, packed, w_scale, stream))


def qc_quant_act_rot(X, xdt, M, K, act_bits, rot_block, qx, x_scale, stream=0) -> int:
    return int(lib().qc_quant_act_rot(X, xdt, M, K, act_bits, rot_block, qx, x_scale, stream))


def qc_qlinear_quant_rot(X, xdt, M, K, act_bits, rot_block, workspace, workspace_bytes,
                         stream=0) -> int:
    return int(lib().qc_qlinear_quant_rot(X, xdt, M, K, act_bits, rot_block, workspace,
                                          workspace_bytes, stream))


def qc_qlinear_rot(X, xdt, M, K, act_bits, rot_block, packed, w_scale, bits, N, bias, epi, Y, ydt,
                   workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_qlinear_rot(X, xdt, M, K, act_bits, rot_block, packed, w_scale, bits, N,
                                    bias, epi, Y, ydt, workspace, workspace_bytes, stream))


def qc_qlinear_asym_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().qc_qlinear_asym_workspace_bytes(M, K, N))


def qc_weight_row_sums(packed, N, K, bits, w_row_sums, stream=0) -> int:
    return int(lib().qc_weight_row_sums(packed, N, K, bits, w_row_sums, stream))


def qc_quant_act_asym(X, xdt, M, K, act_bits, qx, x_scale, x_zero, stream=0) -> int:
    return int(lib().qc_quant_act_asym(X, xdt, M, K, act_bits, qx, x_scale, x_zero, stream))


def qc_qlinear_asym(X, xdt, M, K, act_bits, packed, w_scale, w_row_sums, bits, N, bias, epi, Y, ydt,
                    workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_qlinear_asym(X, xdt, M, K, act_bits, packed, w_scale, w_row_sums, bits, N,
                                     bias, epi, Y, ydt, workspace, workspace_bytes, stream))


def qc_qlinear_asym_quant(X, xdt, M, K, act_bits, workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_qlinear_asym_quant(X, xdt, M, K, act_bits, workspace, workspace_bytes,
                                           stream))


def qc_qlinear_asym_gemm(workspace, workspace_bytes, M, K, packed, w_scale, w_row_sums, bits, N,
                         bias, epi, Y, ydt, stream=0) -> int:
    return int(lib().qc_qlinear_asym_gemm(workspace, workspace_bytes, M, K, packed, w_scale,
                                          w_row_sums, bits, N, bias, epi, Y, ydt, stream))


def qc_quant_act_tensor_workspace_bytes(M: int, K: int) -> int:
    return int(lib().qc_quant_act_tensor_workspace_bytes(M, K))


def qc_quant_act_tensor(X, xdt, M, K, act_bits, qx, x_scale, workspace, workspace_bytes,
                        stream=0) -> int:
    return int(lib().qc_quant_act_tensor(X, xdt, M, K, act_bits, qx, x_scale, workspace,
                                         workspace_bytes, stream))


def qc_qlinear_tensor_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().qc_qlinear_tensor_workspace_bytes(M, K, N))


def qc_qlinear_tensor(X, xdt, M, K, act_bits, packed, w_scale, bits, N, bias, epi, Y, ydt,
                      workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_qlinear_tensor(X, xdt, M, K, act_bits, packed, w_scale, bits, N, bias, epi,
                                       Y, ydt, workspace, workspace_bytes, stream))


def qc_debug_workspace_act_asym(workspace, M, K, act_bits, qx, x_scale, x_zero, stream=0) -> int:
    return int(lib().qc_debug_workspace_act_asym(workspace, M, K, act_bits, qx, x_scale, x_zero,
                                                 stream))


def qc_frame_gradient_norm_workspace_bytes(frames: int, inner: int) -> int:
    return int(lib().qc_frame_gradient_norm_workspace_bytes(frames, inner))


def qc_frame_gradient_norm(m, dt, frames, inner, out2, workspace, workspace_bytes, stream=0) -> int:
    return int(lib().qc_frame_gradient_norm(m, dt, frames, inner, out2, workspace,
                                            workspace_bytes, stream))


def qc_cumulative_variation_workspace_bytes(n: int, count: int) -> int:
    return int(lib().qc_cumulative_variation_workspace_bytes(n, count))


def qc_cumulative_variation(cur, prevs, count, n, out, workspace, workspace_bytes, stream=0) -> int:
    """prevs: a sequence of `count` device addresses (or None for a null list)."""
    arr = None
    if prevs is not None:
        arr = (ctypes.c_void_p * len(prevs))(*prevs)
    return int(lib().qc_cumulative_variation(cur, arr, count, n, out, workspace, workspace_bytes,
                                             stream))


def qc_divergence_score(l1_change: float, k: int, grad_norm: float) -> float:
    return float(lib().qc_divergence_score(l1_change, k, grad_norm))


def qc_cache_interval(D, delta1, delta2, tau_max, tau_mid, tau_min) -> int:
    return int(lib().qc_cache_interval(D, delta1, delta2, tau_max, tau_mid, tau_min))


def qc_activation_bits(D, theta1, theta2, bit_max, bit_mid, bit_min) -> int:
    return int(lib().qc_activation_bits(D, theta1, theta2, bit_max, bit_mid, bit_min))


def qc_prune_probability(S, tau_low, tau_high, p_base) -> float:
    return float(lib().qc_prune_probability(S, tau_low, tau_high, p_base))


def _torch():
    import torch
    return torch


def _stream() -> int:
    return int(_torch().cuda.current_stream().cuda_stream)


def _check(status: int, where: str) -> None:
    if status != QC_OK:
        raise QcError(status, where)


def _xdt(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return QC_F32
    if t.dtype == torch.bfloat16:
        return QC_BF16
    raise TypeError(f"activations must be float32 or bfloat16, got {t.dtype}")


EPI = {"none": QC_EPI_NONE, "gelu_tanh": QC_EPI_GELU_TANH, "gelu_erf": QC_EPI_GELU_ERF}
OUT = {"f32": QC_OUT_F32, "bf16": QC_OUT_BF16, "i32": QC_OUT_I32_ACC}


class PackedWeight:
    """Device blob written by qc_pack_weight plus its per-channel scales."""

    def __init__(self, blob, scale, N: int, K: int, bits: int):
        self.blob, self.scale, self.N, self.K, self.bits = blob, scale, N, K, bits


def pack_weight_t(W, bits: int, rot_block: int = 0) -> PackedWeight:
    torch = _torch()
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and W.dim() == 2
    N, K = W.shape
    nbytes = qc_packed_weight_bytes(N, K, bits)
    if nbytes == 0:
        raise QcError(QC_ERR_UNSUPPORTED, "qc_packed_weight_bytes")
    blob = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    scale = torch.empty(N, dtype=torch.float32, device=W.device)
    if rot_block:
        _check(qc_pack_weight_rot(W.data_ptr(), N, K, bits, rot_block, blob.data_ptr(),
                                  scale.data_ptr(), _stream()), "qc_pack_weight_rot")
    else:
        _check(qc_pack_weight(W.data_ptr(), N, K, bits, blob.data_ptr(), scale.data_ptr(),
                              _stream()), "qc_pack_weight")
    return PackedWeight(blob, scale, N, K, bits)


def unpack_weight_codes_t(pw: PackedWeight):
    torch = _torch()
    codes = torch.empty((pw.N, pw.K), dtype=torch.int8, device=pw.blob.device)
    _check(qc_unpack_weight_codes(pw.blob.data_ptr(), pw.N, pw.K, pw.bits, codes.data_ptr(),
                                  _stream()), "qc_unpack_weight_codes")
    return codes


def quant_act_t(X, act_bits: int = 8, rot_block: int = 0):
    torch = _torch()
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2
    M, K = X.shape
    qx = torch.empty((M, K), dtype=torch.int8, device=X.device)
    sx = torch.empty(M, dtype=torch.float32, device=X.device)
    if rot_block:
        _check(qc_quant_act_rot(X.data_ptr(), _xdt(X), M, K, act_bits, rot_block, qx.data_ptr(),
                                sx.data_ptr(), _stream()), "qc_quant_act_rot")
    else:
        _check(qc_quant_act_bits(X.data_ptr(), _xdt(X), M, K, act_bits, qx.data_ptr(),
                                 sx.data_ptr(), _stream()), "qc_quant_act_bits")
    return qx, sx


def qlinear_workspace_t(M: int, K: int, N: int, device="cuda"):
    torch = _torch()
    nbytes = qc_qlinear_workspace_bytes(M, K, N)
    if nbytes == 0:
        raise QcError(QC_ERR_UNSUPPORTED, "qc_qlinear_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def qlinear_t(X, pw: PackedWeight, bias=None, epi="none", out="bf16", workspace=None, Y=None,
              act_bits: int = 8, rot_block: int = 0):
    torch = _torch()
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2 and X.shape[1] == pw.K
    M, K = X.shape
    if workspace is None:
        workspace = qlinear_workspace_t(M, K, pw.N, X.device)
    if Y is None:
        ydtype = {"f32": torch.float32, "bf16": torch.bfloat16, "i32": torch.int32}[out]
        Y = torch.empty((M, pw.N), dtype=ydtype, device=X.device)
    b = None if bias is None else bias.data_ptr()
    if rot_block:
        _check(qc_qlinear_rot(X.data_ptr(), _xdt(X), M, K, act_bits, rot_block, pw.blob.data_ptr(),
                              pw.scale.data_ptr(), pw.bits, pw.N, b, EPI[epi], Y.data_ptr(),
                              OUT[out], workspace.data_ptr(), workspace.numel(), _stream()),
               "qc_qlinear_rot")
    else:
        _check(qc_qlinear_act_bits(X.data_ptr(), _xdt(X), M, K, act_bits, pw.blob.data_ptr(),
                                   pw.scale.data_ptr(), pw.bits, pw.N, b, EPI[epi], Y.data_ptr(),
                                   OUT[out], workspace.data_ptr(), workspace.numel(), _stream()),
               "qc_qlinear_act_bits")
    return Y


def debug_workspace_act_t(workspace, M: int, K: int):
    torch = _torch()
    qx = torch.empty((M, K), dtype=torch.int8, device=workspace.device)
    sx = torch.empty(M, dtype=torch.float32, device=workspace.device)
    _check(qc_debug_workspace_act(workspace.data_ptr(), M, K, qx.data_ptr(), sx.data_ptr(),
                                  _stream()), "qc_debug_workspace_act")
    return qx, sx


def latent_delta_workspace_t(n: int, device="cuda"):
    torch = _torch()
    return torch.empty(qc_latent_delta_workspace_bytes(n), dtype=torch.uint8, device=device)


def latent_delta_t(cur, prev, workspace=None, out3=None):
    torch = _torch()
    assert cur.is_cuda and cur.dtype == torch.float32 and cur.is_contiguous()
    assert prev.shape == cur.shape and prev.dtype == torch.float32 and prev.is_contiguous()
    n = cur.numel()
    if workspace is None:
        workspace = latent_delta_workspace_t(n, cur.device)
    if out3 is None:
        out3 = torch.empty(3, dtype=torch.float32, device=cur.device)
    _check(qc_latent_delta(cur.data_ptr(), prev.data_ptr(), n, out3.data_ptr(), workspace.data_ptr(),
                           workspace.numel(), _stream()), "qc_latent_delta")
    return out3


def layer_similarity_t(a, b, workspace=None, out4=None):
    torch = _torch()
    assert a.is_cuda and a.is_contiguous() and b.is_contiguous()
    assert a.shape == b.shape and a.dtype == b.dtype
    n = a.numel()
    if workspace is None:
        workspace = torch.empty(qc_layer_similarity_workspace_bytes(n), dtype=torch.uint8,
                                device=a.device)
    if out4 is None:
        out4 = torch.empty(4, dtype=torch.float32, device=a.device)
    _check(qc_layer_similarity(a.data_ptr(), b.data_ptr(), _xdt(a), n, out4.data_ptr(),
                               workspace.data_ptr(), workspace.numel(), _stream()),
           "qc_layer_similarity")
    return out4


def frame_gradient_norm_t(m, workspace=None, out2=None):
    """m: [frames, ...] float32 or bfloat16, contiguous -> device float [2]."""
    torch = _torch()
    assert m.is_cuda and m.is_contiguous() and m.dim() >= 2
    frames = m.shape[0]
    inner = m.numel() // frames
    if workspace is None:
        workspace = torch.empty(qc_frame_gradient_norm_workspace_bytes(frames, inner),
                                dtype=torch.uint8, device=m.device)
    if out2 is None:
        out2 = torch.empty(2, dtype=torch.float32, device=m.device)
    _check(qc_frame_gradient_norm(m.data_ptr(), _xdt(m), frames, inner, out2.data_ptr(),
                                  workspace.data_ptr(), workspace.numel(), _stream()),
           "qc_frame_gradient_norm")
    return out2


def cumulative_variation_t(cur, prevs, workspace=None, out=None):
    """cur float32 [n], prevs a list of float32 tensors of the same size -> device float
    [len(prevs) + 1]."""
    torch = _torch()
    assert cur.is_cuda and cur.is_contiguous() and cur.dtype == torch.float32
    n = cur.numel()
    for p in prevs:
        assert p.is_cuda and p.is_contiguous() and p.dtype == torch.float32 and p.numel() == n
    count = len(prevs)
    if workspace is None:
        workspace = torch.empty(max(qc_cumulative_variation_workspace_bytes(n, count), 256),
                                dtype=torch.uint8, device=cur.device)
    if out is None:
        out = torch.empty(count + 1, dtype=torch.float32, device=cur.device)
    _check(qc_cumulative_variation(cur.data_ptr(), [p.data_ptr() for p in prevs], count, n,
                                   out.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                   _stream()),
           "qc_cumulative_variation")
    return out


# ---- asymmetric activations ---------------------------------------------------------------------

def weight_row_sums_t(pw: PackedWeight):
    torch = _torch()
    sums = torch.empty(pw.N, dtype=torch.int32, device=pw.blob.device)
    _check(qc_weight_row_sums(pw.blob.data_ptr(), pw.N, pw.K, pw.bits, sums.data_ptr(), _stream()),
           "qc_weight_row_sums")
    return sums


def quant_act_asym_t(X, act_bits: int = 8):
    torch = _torch()
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2
    M, K = X.shape
    qx = torch.empty((M, K), dtype=torch.uint8, device=X.device)
    sx = torch.empty(M, dtype=torch.float32, device=X.device)
    zx = torch.empty(M, dtype=torch.float32, device=X.device)
    _check(qc_quant_act_asym(X.data_ptr(), _xdt(X), M, K, act_bits, qx.data_ptr(), sx.data_ptr(),
                             zx.data_ptr(), _stream()), "qc_quant_act_asym")
    return qx, sx, zx


def qlinear_asym_workspace_t(M: int, K: int, N: int, device="cuda"):
    torch = _torch()
    nbytes = qc_qlinear_asym_workspace_bytes(M, K, N)
    if nbytes == 0:
        raise QcError(QC_ERR_UNSUPPORTED, "qc_qlinear_asym_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def qlinear_asym_t(X, pw: PackedWeight, row_sums, bias=None, epi="none", out="bf16", workspace=None,
                   Y=None, act_bits: int = 8):
    torch = _torch()
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2 and X.shape[1] == pw.K
    M, K = X.shape
    if workspace is None:
        workspace = qlinear_asym_workspace_t(M, K, pw.N, X.device)
    if Y is None:
        ydtype = {"f32": torch.float32, "bf16": torch.bfloat16, "i32": torch.int32}[out]
        Y = torch.empty((M, pw.N), dtype=ydtype, device=X.device)
    _check(qc_qlinear_asym(X.data_ptr(), _xdt(X), M, K, act_bits, pw.blob.data_ptr(),
                           pw.scale.data_ptr(), row_sums.data_ptr(), pw.bits, pw.N,
                           None if bias is None else bias.data_ptr(), EPI[epi], Y.data_ptr(),
                           OUT[out], workspace.data_ptr(), workspace.numel(), _stream()),
           "qc_qlinear_asym")
    return Y


def debug_workspace_act_asym_t(workspace, M: int, K: int, act_bits: int = 8):
    torch = _torch()
    qx = torch.empty((M, K), dtype=torch.uint8, device=workspace.device)
    sx = torch.empty(M, dtype=torch.float32, device=workspace.device)
    zx = torch.empty(M, dtype=torch.float32, device=workspace.device)
    _check(qc_debug_workspace_act_asym(workspace.data_ptr(), M, K, act_bits, qx.data_ptr(),
                                       sx.data_ptr(), zx.data_ptr(), _stream()),
           "qc_debug_workspace_act_asym")
    return qx, sx, zx


# ---- one activation scale per layer input -------------------------------------------------------

def quant_act_tensor_t(X, act_bits: int = 8):
    torch = _torch()
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2
    M, K = X.shape
    qx = torch.empty((M, K), dtype=torch.int8, device=X.device)
    sx = torch.empty(1, dtype=torch.float32, device=X.device)
    ws = torch.empty(qc_quant_act_tensor_workspace_bytes(M, K), dtype=torch.uint8, device=X.device)
    _check(qc_quant_act_tensor(X.data_ptr(), _xdt(X), M, K, act_bits, qx.data_ptr(), sx.data_ptr(),
                               ws.data_ptr(), ws.numel(), _stream()), "qc_quant_act_tensor")
    return qx, sx


def qlinear_tensor_workspace_t(M: int, K: int, N: int, device="cuda"):
    torch = _torch()
    nbytes = qc_qlinear_tensor_workspace_bytes(M, K, N)
    if nbytes == 0:
        raise QcError(QC_ERR_UNSUPPORTED, "qc_qlinear_tensor_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def qlinear_tensor_t(X, pw: PackedWeight, bias=None, epi="none", out="bf16", workspace=None, Y=None,
                     act_bits: int = 8):
    torch = _torch()
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2 and X.shape[1] == pw.K
    M, K = X.shape
    if workspace is None:
        workspace = qlinear_tensor_workspace_t(M, K, pw.N, X.device)
    if Y is None:
        ydtype = {"f32": torch.float32, "bf16": torch.bfloat16, "i32": torch.int32}[out]
        Y = torch.empty((M, pw.N), dtype=ydtype, device=X.device)
    _check(qc_qlinear_tensor(X.data_ptr(), _xdt(X), M, K, act_bits, pw.blob.data_ptr(),
                             pw.scale.data_ptr(), pw.bits, pw.N,
                             None if bias is None else bias.data_ptr(), EPI[epi], Y.data_ptr(),
                             OUT[out], workspace.data_ptr(), workspace.numel(), _stream()),
           "qc_qlinear_tensor")
    return Y
