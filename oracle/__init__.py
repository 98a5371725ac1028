"""CPU oracle for the QuantCache quantized-linear hot path -- TEST INFRASTRUCTURE ONLY.

A thin numpy/ctypes front for ``qc_oracle.c`` (plain C, built with gcc).  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library and its Python binding never do, and this package never
imports them.

Paper passages each function follows (arxiv 2503.06545):
  quant_act, quant_weight   Section 3.1 Eq. (3), Eq. (4) in symmetric signed form;
                            Section 4.1 "Quantization Scheme" (per-channel weight,
                            online activation scales); Section 3.2 AIGQ (1) for the
                            per-layer weight bit-width, AIGQ (2) Eq. (8) for the
                            activation bit-width (8, 6 or 4 in an int8 container)
  gemm_i32, epilogue,       Section 4.1 "Hardware Implementation" (low-bit GEMM with
  qlinear                   fused quantize / dequantize)
  latent_delta              Section 3.2 HLC, Eq. (5) numerator
  layer_similarity          Section 3.3 SRAP, Eq. (9)
  quant_act_tensor,         Section 4.1 "Quantization Scheme" read literally: one activation
  qlinear_tensor            scale per layer input (per tensor), computed online
  quant_act_asym,           Section 3.1 Eq. (3), Eq. (4) as printed: asymmetric, with a zero
  qlinear_asym              point per token
  rotate_rows, quant_act_   Section 3.2 AIGQ (1) (rotation against outlier channels) and
  rot, quant_weight_rot,    Section 4.1 "Hardware Implementation" (rotation fused with the
  qlinear_rot               quantization), as a block Walsh-Hadamard transform over K
  frame_gradient,           Section 3.2 HLC, Eq. (5): the inter-frame gradient factor and the
  divergence_score          score built from it and latent_delta's first sum
  cumulative_variation      Section 3.3 SRAP, Eq. (11)
  cache_interval,           the three-way threshold rules: Section 3.2 Eq. (6) and Eq. (8),
  activation_bits,          Section 3.3 Eq. (10)
  prune_probability
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qc_oracle.c")
_LIB = os.path.join(_HERE, "libqc_oracle.so")

EPI_NONE, EPI_GELU_TANH, EPI_GELU_ERF = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile qc_oracle.c with gcc (-O2, no contraction, OpenMP over rows).  QC_ORACLE_LIB names
    a differently compiled copy of the same source to load instead (the sanitizer test's)."""
    if os.environ.get("QC_ORACLE_LIB"):
        return os.environ["QC_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall",
               "-Wextra", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.orc_num_threads.restype = i32
        lib.orc_set_num_threads.argtypes = [i32]
        lib.orc_quant_rows_f32.argtypes = [vp, i64, i64, i32, vp, vp]
        lib.orc_quant_rows_bf16.argtypes = [vp, i64, i64, i32, vp, vp]
        lib.orc_pack_int4.argtypes = [vp, i64, i64, vp]
        lib.orc_unpack_int4.argtypes = [vp, i64, i64, vp]
        lib.orc_gemm_i32.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.orc_gemm_i64.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.orc_epilogue_f64.argtypes = [vp, vp, vp, vp, i32, i64, i64, vp]
        lib.orc_round_to_f32.argtypes = [vp, i64, vp]
        lib.orc_round_to_bf16.argtypes = [vp, i64, vp]
        lib.orc_qlinear.argtypes = [vp, i32, i64, i64, i32, vp, vp, i64, vp, i32, vp, vp, vp, vp]
        lib.orc_latent_delta.argtypes = [vp, vp, i64, vp]
        lib.orc_layer_similarity.argtypes = [vp, vp, i32, i64, vp]
        lib.orc_layer_similarity.restype = None
        lib.orc_quant_rows_asym.argtypes = [vp, i32, i64, i64, i32, vp, vp, vp]
        lib.orc_quant_rows_asym.restype = None
        lib.orc_qlinear_asym.argtypes = [vp, i32, i64, i64, i32, vp, vp, i64, vp, i32, vp, vp, vp, vp]
        lib.orc_qlinear_asym.restype = None
        lib.orc_rotate_rows_f32.argtypes = [vp, i64, i64, i32, ctypes.c_float, vp]
        lib.orc_rotate_rows_f32.restype = None
        lib.orc_frame_gradient.argtypes = [vp, i32, i64, i64, vp]
        lib.orc_frame_gradient.restype = None
        lib.orc_cumulative_variation.argtypes = [vp, vp, i32, i64, vp]
        lib.orc_cumulative_variation.restype = None
        for name in ("orc_set_num_threads", "orc_quant_rows_f32", "orc_quant_rows_bf16",
                     "orc_pack_int4", "orc_unpack_int4", "orc_gemm_i32", "orc_gemm_i64",
                     "orc_epilogue_f64", "orc_round_to_f32", "orc_round_to_bf16", "orc_qlinear",
                     "orc_latent_delta"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_L().orc_num_threads())


def set_num_threads(n: int) -> None:
    _L().orc_set_num_threads(int(n))


def qmax(bits: int) -> int:
    """Largest code magnitude of the symmetric b-bit quantizer: 2^(b-1) - 1."""
    return (1 << (bits - 1)) - 1


def _quant_rows(X, qm):
    """X: float32 [R, K] or uint16 (bf16 bit patterns) [R, K] -> (int8 codes, float32 scales)."""
    if X.dtype == np.uint16:
        X = _c(X, np.uint16)
        fn = _L().orc_quant_rows_bf16
    else:
        X = _c(X, np.float32)
        fn = _L().orc_quant_rows_f32
    R, K = X.shape
    q = np.empty((R, K), np.int8)
    s = np.empty((R,), np.float32)
    fn(_p(X), R, K, int(qm), _p(q), _p(s))
    return q, s


def quant_act(X, act_bits: int = 8):
    """Per-token (per-row) symmetric quantization of activations X [M, K] into an int8
    container; act_bits 8, 6 or 4 (Section 3.2 AIGQ (2), Eq. (8))."""
    return _quant_rows(X, qmax(act_bits))


def quant_weight(W, bits: int):
    """Per-output-channel symmetric quantization of W [N, K] at 8 or 4 bits."""
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    return _quant_rows(np.asarray(W, np.float32), qmax(bits))


def pack_int4(codes):
    codes = _c(codes, np.int8)
    N, K = codes.shape
    if K % 2:
        raise ValueError("int4 packing needs an even K")
    out = np.empty((N, K // 2), np.uint8)
    _L().orc_pack_int4(_p(codes), N, K, _p(out))
    return out


def unpack_int4(packed, K: int):
    packed = _c(packed, np.uint8)
    N = packed.shape[0]
    out = np.empty((N, K), np.int8)
    _L().orc_unpack_int4(_p(packed), N, K, _p(out))
    return out


def gemm_i32(qx, qw):
    qx, qw = _c(qx, np.int8), _c(qw, np.int8)
    M, K = qx.shape
    N = qw.shape[0]
    assert qw.shape[1] == K
    acc = np.empty((M, N), np.int32)
    _L().orc_gemm_i32(_p(qx), _p(qw), M, N, K, _p(acc))
    return acc


def gemm_i64(qx, qw):
    qx, qw = _c(qx, np.int8), _c(qw, np.int8)
    M, K = qx.shape
    N = qw.shape[0]
    acc = np.empty((M, N), np.int64)
    _L().orc_gemm_i64(_p(qx), _p(qw), M, N, K, _p(acc))
    return acc


def epilogue(acc, sx, sw, bias=None, epi=EPI_NONE):
    """y = acc * sx[m] * sw[n] + bias[n], optional GELU; returns float64 [M, N]."""
    acc = _c(acc, np.int32)
    sx, sw = _c(sx, np.float32), _c(sw, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    M, N = acc.shape
    y = np.empty((M, N), np.float64)
    _L().orc_epilogue_f64(_p(acc), _p(sx), _p(sw), _p(bias), int(epi), M, N, _p(y))
    return y


def round_f32(y):
    y = _c(y, np.float64)
    out = np.empty(y.shape, np.float32)
    _L().orc_round_to_f32(_p(y), y.size, _p(out))
    return out


def round_bf16_bits(y):
    y = _c(y, np.float64)
    out = np.empty(y.shape, np.uint16)
    _L().orc_round_to_bf16(_p(y), y.size, _p(out))
    return out


def bf16_bits_to_f64(bits):
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    bits = np.asarray(bits, np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def qlinear(X, qw, sw, bias=None, epi=EPI_NONE, act_bits: int = 8):
    """Whole quantized linear.  X float32 or uint16(bf16 bits) [M, K]; qw int8 codes [N, K].

    Returns dict(qx, sx, acc, y) with y in float64 before the single output rounding.
    """
    x_is_bf16 = X.dtype == np.uint16
    X = _c(X, np.uint16 if x_is_bf16 else np.float32)
    qw, sw = _c(qw, np.int8), _c(sw, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    M, K = X.shape
    N = qw.shape[0]
    assert qw.shape[1] == K and sw.shape[0] == N
    qx = np.empty((M, K), np.int8)
    sx = np.empty((M,), np.float32)
    acc = np.empty((M, N), np.int32)
    y = np.empty((M, N), np.float64)
    _L().orc_qlinear(_p(X), int(x_is_bf16), M, K, qmax(act_bits), _p(qw), _p(sw), N, _p(bias),
                     int(epi), _p(qx), _p(sx), _p(acc), _p(y))
    return {"qx": qx, "sx": sx, "acc": acc, "y": y}


def latent_delta(cur, prev):
    """(sum|cur-prev|, sum|prev|, ratio) in float64."""
    cur, prev = _c(cur, np.float32).ravel(), _c(prev, np.float32).ravel()
    assert cur.size == prev.size
    out = np.empty(3, np.float64)
    _L().orc_latent_delta(_p(cur), _p(prev), cur.size, _p(out))
    return out


def layer_similarity(a, b):
    """(<a,b>, <a,a>, <b,b>, cosine) in float64; a, b float32 or uint16 (bf16 bits)."""
    is_bf16 = a.dtype == np.uint16
    dt = np.uint16 if is_bf16 else np.float32
    a, b = _c(a, dt).ravel(), _c(b, dt).ravel()
    assert a.size == b.size
    out = np.empty(4, np.float64)
    _L().orc_layer_similarity(_p(a), _p(b), int(is_bf16), a.size, _p(out))
    return out


def frame_gradient(m):
    """m: float32 or uint16 (bf16 bits) [frames, inner] -> (sum of squared forward differences
    along the frame axis, its square root) in float64."""
    is_bf16 = m.dtype == np.uint16
    m = _c(m, np.uint16 if is_bf16 else np.float32)
    frames, inner = m.shape
    out = np.empty(2, np.float64)
    _L().orc_frame_gradient(_p(m), int(is_bf16), frames, inner, _p(out))
    return out


def cumulative_variation(cur, prevs):
    """cur float32 [n], prevs float32 [count, n] -> float64 [count + 1]: each L1 distance, then
    their sum V (Eq. (11))."""
    cur = _c(cur, np.float32).ravel()
    prevs = _c(prevs, np.float32).reshape(-1, cur.size)
    out = np.empty(prevs.shape[0] + 1, np.float64)
    _L().orc_cumulative_variation(_p(cur), _p(prevs), prevs.shape[0], cur.size, _p(out))
    return out


def divergence_score(l1_change: float, k: int, grad_norm: float) -> float:
    """Eq. (5): the L1 change since the cached step, per step, times the gradient norm."""
    return float(l1_change) / float(k) * float(grad_norm)


def _three_way(value, low, high, below, between, above):
    """below if value < low, between if low <= value < high, above if value >= high."""
    if value < low:
        return below
    if value < high:
        return between
    return above


def cache_interval(D, delta1, delta2, tau_max, tau_mid, tau_min):
    """Eq. (6): steps until the next recomputation."""
    return _three_way(D, delta1, delta2, tau_max, tau_mid, tau_min)


def activation_bits(D, theta1, theta2, bit_max, bit_mid, bit_min):
    """Eq. (8): activation bit-width of a timestep from its redundancy metric."""
    return _three_way(D, theta1, theta2, bit_max, bit_mid, bit_min)


def prune_probability(S, tau_low, tau_high, p_base):
    """Eq. (10): 1 above tau_high, p_base on [tau_low, tau_high], 0 below tau_low."""
    if S > tau_high:
        return 1.0
    if S < tau_low:
        return 0.0
    return float(p_base)


# ---- rotation before quantization ------------------------------------------------------------

def widen_f32(X):
    """float32 view of the input values: bf16 bit patterns widened exactly, float32 as is."""
    if X.dtype == np.uint16:
        return (np.ascontiguousarray(X).astype(np.uint32) << 16).view(np.float32)
    return _c(X, np.float32)


def rotate_rows(X, block: int, post_scale: float = 1.0):
    """Block Walsh-Hadamard transform of each row of X [R, K] (float32) over blocks of `block`
    consecutive columns, binary32 butterflies in ascending stride, then * post_scale."""
    X = _c(X, np.float32)
    R, K = X.shape
    if block < 2 or block & (block - 1) or K % block:
        raise ValueError("block must be a power of two that divides K")
    out = np.empty((R, K), np.float32)
    _L().orc_rotate_rows_f32(_p(X), R, K, int(block), float(post_scale), _p(out))
    return out


def quant_act_rot(X, block: int, act_bits: int = 8):
    """Per-token quantization of the rotated activations X H."""
    return _quant_rows(rotate_rows(widen_f32(X), block), qmax(act_bits))


def quant_weight_rot(W, bits: int, block: int):
    """Per-channel quantization of the counter-rotated weights W H / block."""
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    return _quant_rows(rotate_rows(np.asarray(W, np.float32), block, 1.0 / block), qmax(bits))


def qlinear_rot(X, qw, sw, block: int, bias=None, epi=EPI_NONE, act_bits: int = 8):
    """The quantized linear on rotated activations; qw / sw come from quant_weight_rot."""
    return qlinear(rotate_rows(widen_f32(X), block), qw, sw, bias, epi, act_bits)


# ---- the printed, asymmetric form of the activation quantizer ---------------------------------

def levels(bits: int) -> int:
    """Largest code of the b-bit unsigned quantizer of Eq. (3): 2^b - 1."""
    return (1 << bits) - 1


def quant_act_asym(X, act_bits: int = 8):
    """Per-token asymmetric quantization: (uint8 codes in [0, 2^b - 1], float32 scales,
    float32 integer-valued zero points); dequantized value = s * (code - z)."""
    is_bf16 = X.dtype == np.uint16
    X = _c(X, np.uint16 if is_bf16 else np.float32)
    R, K = X.shape
    q = np.empty((R, K), np.uint8)
    s = np.empty((R,), np.float32)
    z = np.empty((R,), np.float32)
    _L().orc_quant_rows_asym(_p(X), int(is_bf16), R, K, levels(act_bits), _p(q), _p(s), _p(z))
    return q, s, z


def qlinear_asym(X, qw, sw, bias=None, epi=EPI_NONE, act_bits: int = 8):
    """Quantized linear with asymmetric activations; returns dict(qx, sx, zx, y), y float64."""
    is_bf16 = X.dtype == np.uint16
    X = _c(X, np.uint16 if is_bf16 else np.float32)
    qw, sw = _c(qw, np.int8), _c(sw, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    M, K = X.shape
    N = qw.shape[0]
    assert qw.shape[1] == K and sw.shape[0] == N
    qx = np.empty((M, K), np.uint8)
    sx = np.empty((M,), np.float32)
    zx = np.empty((M,), np.float32)
    y = np.empty((M, N), np.float64)
    _L().orc_qlinear_asym(_p(X), int(is_bf16), M, K, levels(act_bits), _p(qw), _p(sw), N,
                          _p(bias), int(epi), _p(qx), _p(sx), _p(zx), _p(y))
    return {"qx": qx, "sx": sx, "zx": zx, "y": y}


# ---- one activation scale per layer input -----------------------------------------------------

def quant_act_tensor(X, act_bits: int = 8):
    """The symmetric quantizer with ONE scale for the whole activation tensor (the paper's
    "dynamic per-layer activation quantization" taken literally): the tensor is quantized as a
    single long row.  Returns (int8 codes [M, K], float32 scale)."""
    M, K = X.shape
    q, s = _quant_rows(np.ascontiguousarray(X).reshape(1, M * K), qmax(act_bits))
    return q.reshape(M, K), np.float32(s[0])


def qlinear_tensor(X, qw, sw, bias=None, epi=EPI_NONE, act_bits: int = 8):
    """Quantized linear on per-tensor activation codes; dict(qx, sx, acc, y), sx a scalar."""
    qx, s = quant_act_tensor(X, act_bits)
    acc = gemm_i32(qx, qw)
    y = epilogue(acc, np.full(X.shape[0], s, np.float32), sw, bias, epi)
    return {"qx": qx, "sx": s, "acc": acc, "y": y}
