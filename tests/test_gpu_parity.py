"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: bit-exact for int8 codes, scales (compared as bit patterns) and int32 accumulators;
outputs within |y - ref| <= rtol * |ref| + rtol * RMS(ref) with rtol 1e-3 (float output)
or 2e-2 (bf16 output); latent delta within 1e-5 relative.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2503_06545_amd import binding as qc
from paper_2503_06545_amd import synth

pytestmark = pytest.mark.gpu

RTOL = {"f32": 1e-3, "bf16": 2e-2}
EPI_ORACLE = {"none": oracle.EPI_NONE, "gelu_tanh": oracle.EPI_GELU_TANH, "gelu_erf": oracle.EPI_GELU_ERF}


def dev(a: np.ndarray):
    """numpy -> device tensor; uint16 arrays are bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def host_f64(y: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    if y.dtype == torch.bfloat16:
        return oracle.bf16_bits_to_f64(y.view(torch.int16).cpu().numpy().view(np.uint16))
    return y.cpu().numpy().astype(np.float64)


def bits_equal(a: np.ndarray, b: np.ndarray) -> bool:
    return np.array_equal(np.ascontiguousarray(a).view(np.uint32), np.ascontiguousarray(b).view(np.uint32))


def assert_outputs_close(got: np.ndarray, ref: np.ndarray, rtol: float):
    rms = math.sqrt(float(np.mean(ref ** 2)))
    err = np.abs(got - ref)
    bound = rtol * np.abs(ref) + rtol * rms
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound), (
        f"max violation at flat index {worst}: got {got.flat[worst]} ref {ref.flat[worst]} "
        f"rms {rms} rtol {rtol}")


def random_x(rng, M, K, dtype):
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.integers(0, K, size=max(1, K // 100))] *= 20
    return synth.to_bf16_bits(x) if dtype == "bf16" else x


# ------------------------------------------------------------------ qc_quant_act

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,K", [(256, 1152), (300, 4608), (1, 16), (37, 2304), (65, 1000),
                                 (5, 24), (3, 9216), (2, 10000), (130, 7)])
def test_quant_act_matches_oracle_bit_for_bit(dtype, M, K):
    rng = np.random.default_rng(M * 100003 + K)
    x = random_x(rng, M, K, dtype)
    x[M // 2] = 0  # a zero row uses the absmax floor
    q_ref, s_ref = oracle.quant_act(x)
    qx, sx = qc.quant_act_t(dev(x))
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), s_ref)
    assert np.array_equal(qx.cpu().numpy(), q_ref)


def test_quant_act_tiny_config_and_ties():
    x = synth.TINY.x()
    q_ref, s_ref = oracle.quant_act(x)
    qx, sx = qc.quant_act_t(dev(x))
    assert bits_equal(sx.cpu().numpy(), s_ref) and np.array_equal(qx.cpu().numpy(), q_ref)
    # exact half-way cases: scale 1, ties go to even
    t = np.zeros((2, 16), np.float32)
    t[0, :10] = [127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, -126.5, 125.5]
    t[1] = -t[0]
    qx, sx = qc.quant_act_t(dev(t))
    assert sx.cpu().tolist() == [1.0, 1.0]
    assert qx[0, :10].cpu().tolist() == [127, 0, 2, 2, 0, -2, -2, 126, -126, 126]
    assert torch.equal(qx[1], -qx[0])


@pytest.mark.parametrize("act_bits", [6, 4])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,K", [(256, 1152), (77, 4608), (9, 1000)])
def test_quant_act_lower_bit_widths(act_bits, dtype, M, K):
    rng = np.random.default_rng(M + K + act_bits)
    x = random_x(rng, M, K, dtype)
    q_ref, s_ref = oracle.quant_act(x, act_bits)
    qx, sx = qc.quant_act_t(dev(x), act_bits)
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), s_ref)
    assert np.array_equal(qx.cpu().numpy(), q_ref)
    assert int(qx.abs().max()) == (1 << (act_bits - 1)) - 1


# ------------------------------------------------------------------ qc_pack_weight

@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("N,K", [(1152, 1152), (200, 136), (1, 2), (129, 72), (64, 4608), (130, 100)])
def test_pack_weight_codes_and_scales_bit_exact(bits, N, K):
    rng = np.random.default_rng(N * 7919 + K + bits)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    if N > 2:
        W[1] = 0
    q_ref, s_ref = oracle.quant_weight(W, bits)
    pw = qc.pack_weight_t(dev(W), bits)
    codes = qc.unpack_weight_codes_t(pw)
    torch.cuda.synchronize()
    assert bits_equal(pw.scale.cpu().numpy(), s_ref)
    assert np.array_equal(codes.cpu().numpy(), q_ref)
    if bits == 4:  # canonical nibble container round trip of the same codes
        assert np.array_equal(oracle.unpack_int4(oracle.pack_int4(codes.cpu().numpy()), K), q_ref)


def test_pack_int4_all_nibbles_all_positions():
    """Every 4-bit code at every k position of a 64-k packing unit, K not a multiple of it."""
    K = 200
    codes = np.zeros((16, K), np.float32)
    for n in range(16):
        codes[n] = [((n + k) % 15) - 7 for k in range(K)]
        codes[n, 0] = 7  # absmax 7 -> scale 1
    pw = qc.pack_weight_t(dev(codes), 4)
    got = qc.unpack_weight_codes_t(pw).cpu().numpy()
    assert np.all(pw.scale.cpu().numpy() == 1.0)
    assert np.array_equal(got, codes.astype(np.int8))


# ------------------------------------------------------------------ qc_qlinear

def run_linear_case(x, W, b, bits, epi, out, check_acc=True, act_bits=8, rot_block=0):
    M, K = x.shape
    N = W.shape[0]
    if rot_block:
        qw_ref, sw_ref = oracle.quant_weight_rot(W, bits, rot_block)
        ref = oracle.qlinear_rot(x, qw_ref, sw_ref, rot_block, b, EPI_ORACLE[epi], act_bits)
    else:
        qw_ref, sw_ref = oracle.quant_weight(W, bits)
        ref = oracle.qlinear(x, qw_ref, sw_ref, b, EPI_ORACLE[epi], act_bits)
    xd, pw = dev(x), qc.pack_weight_t(dev(W), bits, rot_block)
    bd = None if b is None else dev(b)
    ws = qc.qlinear_workspace_t(M, K, N)
    y = qc.qlinear_t(xd, pw, bd, epi, out, workspace=ws, act_bits=act_bits, rot_block=rot_block)
    qx, sx = qc.debug_workspace_act_t(ws, M, K)
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), ref["sx"]), "activation scales differ"
    assert np.array_equal(qx.cpu().numpy(), ref["qx"]), "activation codes differ"
    if check_acc:
        acc = qc.qlinear_t(xd, pw, None, "none", "i32", workspace=ws, act_bits=act_bits,
                           rot_block=rot_block)
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), ref["acc"]), "int32 accumulators differ"
    y_ref = ref["y"]
    if out == "bf16":  # the oracle's single rounding to the output type
        y_ref = oracle.bf16_bits_to_f64(oracle.round_bf16_bits(y_ref))
    else:
        y_ref = oracle.round_f32(y_ref).astype(np.float64)
    assert_outputs_close(host_f64(y), y_ref, RTOL[out])
    return y


def test_qlinear_tiny_config_full_parity():
    c = synth.TINY
    run_linear_case(c.x(), c.weight(), c.bias(), 8, "none", "f32")


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("epi", ["none", "gelu_tanh", "gelu_erf"])
@pytest.mark.parametrize("out", ["f32", "bf16"])
def test_qlinear_variants(bits, epi, out):
    rng = np.random.default_rng(bits * 31 + len(epi) + len(out))
    M, K, N = 512, 1152, 384
    x = random_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    run_linear_case(x, W, b, bits, epi, out)


@pytest.mark.parametrize("bits,act_bits", [(4, 6), (8, 6), (4, 4)])
def test_qlinear_lower_activation_bit_widths(bits, act_bits):
    """The paper's W4A6 operating point and its neighbours: same GEMM, coarser activation codes."""
    rng = np.random.default_rng(bits * 10 + act_bits)
    M, K, N = 640, 1152, 256
    x = random_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    run_linear_case(x, W, b, bits, "gelu_tanh", "bf16", act_bits=act_bits)
    run_linear_case(x, W, b, bits, "none", "f32", act_bits=act_bits)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,K,N", [(300, 136, 200), (1, 16, 1), (257, 64, 129), (33, 200, 77),
                                   (700, 4608, 130), (256, 2, 8), (513, 1000, 260)])
def test_qlinear_ragged_shapes(bits, M, K, N):
    rng = np.random.default_rng(M + 3 * K + 5 * N + bits)
    x = random_x(rng, M, K, "f32")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    run_linear_case(x, W, b, bits, "none", "f32")
    run_linear_case(synth.to_bf16_bits(x), W, None, bits, "gelu_tanh", "bf16", check_acc=False)


@pytest.mark.parametrize("out", ["f32", "bf16"])
@pytest.mark.parametrize("epi", ["gelu_tanh", "gelu_erf"])
def test_gelu_dense_sweep_through_the_epilogue(epi, out):
    """All-zero activations give zero accumulators, so Y[m, n] = act(bias[n]): the bias sweeps
    the activation's argument densely over [-8, 8] (and far outside), every output against the
    oracle's fp64 formula rounded once.  Bars: the output tolerances with the RMS term replaced
    by 1 (the scale of an fc1 output), i.e. an absolute 1e-3 / 2e-2 near zero."""
    N, K, M = 16384 + 8, 64, 16
    b = np.concatenate([np.linspace(-8.0, 8.0, 16384), [-100, -20, -10, 10, 20, 100, 0.0, -0.0]]).astype(np.float32)
    x = np.zeros((M, K), np.float32)
    W = np.full((N, K), 0.01, np.float32)
    qw_ref, sw_ref = oracle.quant_weight(W, 8)
    ref = oracle.qlinear(x, qw_ref, sw_ref, b, EPI_ORACLE[epi])
    assert not ref["acc"].any()
    y = qc.qlinear_t(dev(x), qc.pack_weight_t(dev(W), 8), dev(b), epi, out)
    y_ref = ref["y"]
    y_ref = (oracle.bf16_bits_to_f64(oracle.round_bf16_bits(y_ref)) if out == "bf16"
             else oracle.round_f32(y_ref).astype(np.float64))
    got = host_f64(y)
    rtol = RTOL[out]
    assert np.all(np.abs(got - y_ref) <= rtol * np.abs(y_ref) + rtol), float(np.abs(got - y_ref).max())
    # the float path is far inside its bar: absolute error of the activation itself
    if out == "f32":
        assert float(np.abs(got - y_ref).max()) < 2e-6 * 8


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("K", [100, 200, 1000, 1160])
def test_qlinear_ragged_k_with_a_poisoned_workspace(bits, K):
    """K is padded to 192 inside the tiled workspace and the quantizer does not write the
    padding; the GEMM reads it and multiplies it by the zero padding of the packed weights.
    With the workspace full of 0x7f bytes beforehand the result must not change."""
    rng = np.random.default_rng(K + bits)
    M, N = 300, 200
    x = random_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    qw_ref, sw_ref = oracle.quant_weight(W, bits)
    ref = oracle.qlinear(x, qw_ref, sw_ref, None, oracle.EPI_NONE)
    ws = qc.qlinear_workspace_t(M, K, N)
    ws.fill_(0x7f)
    acc = qc.qlinear_t(dev(x), qc.pack_weight_t(dev(W), bits), None, "none", "i32", workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,N", [(4096, 4096), (4096 - 37, 4096 - 3)])
def test_qlinear_many_tiles_full_comparison(bits, M, N):
    """Several rounds of tiles on every CU (512 tiles of 256 x 128), short reduction; the whole
    output is compared with the oracle, ragged edges included."""
    rng = np.random.default_rng(M + N + bits)
    K = 320
    x = random_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    run_linear_case(x, W, b, bits, "gelu_tanh", "bf16")
    if bits == 4:
        run_asym_case(x, W, b, bits, "none", "f32", act_bits=6)


def test_qlinear_seeded_random_shapes():
    """Thirty shapes drawn from a seeded generator: any M, N, even K, every combination of input
    type, weight bits, activation bits, epilogue and output type gets hit; full comparison."""
    rng = np.random.default_rng(20250306)
    for case in range(30):
        M = int(rng.integers(1, 700))
        K = 2 * int(rng.integers(1, 400))
        N = int(rng.integers(1, 400))
        bits = int(rng.choice([8, 4]))
        act_bits = int(rng.choice([8, 8, 6, 4]))
        epi = str(rng.choice(["none", "gelu_tanh", "gelu_erf"]))
        out = str(rng.choice(["f32", "bf16"]))
        dtype = str(rng.choice(["f32", "bf16"]))
        x = random_x(rng, M, K, dtype)
        W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
        b = (rng.standard_normal(N) * 0.01).astype(np.float32) if case % 3 else None
        try:
            run_linear_case(x, W, b, bits, epi, out, act_bits=act_bits)
        except AssertionError as e:
            raise AssertionError(f"case {case}: M={M} K={K} N={N} bits={bits} act_bits={act_bits} "
                                 f"epi={epi} out={out} x={dtype}: {e}") from e


def test_qlinear_closed_form_integers_and_extremes():
    """Integer operands with unit scales reproduce X W^T + b exactly; all-127 operands reach the
    largest accumulator magnitude at K = 4608."""
    rng = np.random.default_rng(5)
    for bits, qm in ((8, 127), (4, 7)):
        M, K, N = 64, 4608, 128
        X = rng.integers(-127, 128, size=(M, K)).astype(np.float32)
        X[:, 0] = 127
        W = rng.integers(-qm, qm + 1, size=(N, K)).astype(np.float32)
        W[:, 1] = qm
        X[0], W[0] = 127, qm
        X[1] = -127
        b = rng.integers(-5, 6, size=N).astype(np.float32)
        pw = qc.pack_weight_t(dev(W), bits)
        acc = qc.qlinear_t(dev(X), pw, None, "none", "i32").cpu().numpy()
        ref = X.astype(np.int64) @ W.astype(np.int64).T
        assert np.array_equal(acc.astype(np.int64), ref)
        assert acc[0, 0] == 127 * qm * K and acc[1, 0] == -127 * qm * K
        y = qc.qlinear_t(dev(X), pw, dev(b), "none", "f32").cpu().numpy().astype(np.float64)
        assert np.allclose(y, ref + b, rtol=3e-7, atol=0)


def test_qlinear_largest_reduction_length():
    """K = QC_MAX_K: all-127 operands reach 127 * 127 * K = 2 114 060 288 < 2^31 without
    wrapping; random rows agree with an int64 product."""
    K, M, N = qc.QC_MAX_K, 33, 130
    rng = np.random.default_rng(13)
    X = rng.integers(-127, 128, size=(M, K)).astype(np.float32)
    W = rng.integers(-127, 128, size=(N, K)).astype(np.float32)
    X[:, 0], W[:, 1] = 127, 127
    X[0], W[0], X[1] = 127, 127, -127
    pw = qc.pack_weight_t(dev(W), 8)
    acc = qc.qlinear_t(dev(X), pw, None, "none", "i32").cpu().numpy()
    assert np.array_equal(acc.astype(np.int64), X.astype(np.int64) @ W.astype(np.int64).T)
    assert acc[0, 0] == 127 * 127 * K and acc[1, 0] == -127 * 127 * K
    assert qc.qc_qlinear_workspace_bytes(M, K + 1, N) == 0


def test_qlinear_one_hot_rows_return_weight_columns():
    K, N = 128, 256
    rng = np.random.default_rng(9)
    W = rng.integers(-127, 128, size=(N, K)).astype(np.float32)
    W[:, 0] = 127
    X = np.zeros((K, K), np.float32)
    X[np.arange(K), np.arange(K)] = 3.0  # scale 3/127, code 127
    pw = qc.pack_weight_t(dev(W), 8)
    acc = qc.qlinear_t(dev(X), pw, None, "none", "i32").cpu().numpy()
    assert np.array_equal(acc, 127 * W.T.astype(np.int32))


def test_qlinear_is_deterministic_and_stays_inside_its_output():
    rng = np.random.default_rng(11)
    M, K, N = 777, 1152, 392
    x = dev(random_x(rng, M, K, "bf16"))
    pw = qc.pack_weight_t(dev((rng.standard_normal((N, K)) * 0.02).astype(np.float32)), 8)
    pad = 4096
    buf = torch.full((M * N + 2 * pad,), -7.0, dtype=torch.bfloat16, device="cuda")
    Y = buf[pad:pad + M * N].view(M, N)
    first = qc.qlinear_t(x, pw, None, "none", "bf16", Y=Y).clone()
    for _ in range(5):
        again = qc.qlinear_t(x, pw, None, "none", "bf16", Y=Y)
        assert torch.equal(again.view(torch.int16), first.view(torch.int16))
    torch.cuda.synchronize()
    assert torch.all(buf[:pad] == -7.0) and torch.all(buf[pad + M * N:] == -7.0)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("N", [4, 8, 12, 129, 130, 132, 136, 260, 264])
def test_qlinear_every_store_width_stays_inside_its_output(bits, N):
    """A lane owns eight consecutive channels of a token and writes them as one 16 B store, two
    8 B or 16 B stores or single elements, depending on N mod 8, N mod 4 and the output type:
    every class, on a ragged M, against the oracle and with guard bands around Y."""
    rng = np.random.default_rng(1000 * bits + N)
    M, K = 300, 192
    x = random_x(rng, M, K, "f32")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    qw_ref, sw_ref = oracle.quant_weight(W, bits)
    ref = oracle.qlinear(x, qw_ref, sw_ref, b, EPI_ORACLE["none"], 8)
    xd, pw, bd = dev(x), qc.pack_weight_t(dev(W), bits), dev(b)
    pad = 1024  # elements; keeps Y 16-byte aligned for every element size
    for out, tdtype, fill in (("bf16", torch.bfloat16, -7.0), ("f32", torch.float32, -7.0),
                              ("i32", torch.int32, -7)):
        buf = torch.full((M * N + 2 * pad,), fill, dtype=tdtype, device="cuda")
        Y = buf[pad:pad + M * N].view(M, N)
        if out == "i32":
            y = qc.qlinear_t(xd, pw, None, "none", out, Y=Y)
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy(), ref["acc"]), out
        else:
            y = qc.qlinear_t(xd, pw, bd, "none", out, Y=Y)
            torch.cuda.synchronize()
            if out == "bf16":
                y_ref = oracle.bf16_bits_to_f64(oracle.round_bf16_bits(ref["y"]))
            else:
                y_ref = oracle.round_f32(ref["y"]).astype(np.float64)
            assert_outputs_close(host_f64(y), y_ref, RTOL[out])
        assert torch.all(buf[:pad] == fill) and torch.all(buf[pad + M * N:] == fill), out


def test_calls_on_two_streams_do_not_disturb_each_other():
    """The library keeps no device state of its own: two different linears issued on two
    streams at the same time, each with its own workspace, give the bits they give alone."""
    rng = np.random.default_rng(21)
    jobs = []
    for (M, K, N, bits, act_bits, epi) in ((3000, 1152, 1152, 8, 8, "none"), (2000, 2304, 640, 4, 6, "gelu_tanh")):
        x = dev(random_x(rng, M, K, "bf16"))
        pw = qc.pack_weight_t(dev((rng.standard_normal((N, K)) * 0.02).astype(np.float32)), bits)
        b = dev((rng.standard_normal(N) * 0.01).astype(np.float32))
        ws = qc.qlinear_workspace_t(M, K, N)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        jobs.append(dict(x=x, pw=pw, b=b, ws=ws, Y=Y, epi=epi, act_bits=act_bits))

    def run(j):
        qc.qlinear_t(j["x"], j["pw"], j["b"], j["epi"], "bf16", workspace=j["ws"], Y=j["Y"],
                     act_bits=j["act_bits"])

    alone = []
    for j in jobs:
        run(j)
        torch.cuda.synchronize()
        alone.append(j["Y"].clone())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]  # default priority
    for _ in range(10):
        for j in jobs:
            j["Y"].fill_(0)
        torch.cuda.synchronize()
        for j, st in zip(jobs, streams):
            with torch.cuda.stream(st):
                for _ in range(3):
                    run(j)
        torch.cuda.synchronize()
        for j, ref in zip(jobs, alone):
            assert torch.equal(j["Y"].view(torch.int16), ref.view(torch.int16))


def test_step_replays_from_a_hip_graph():
    """The library allocates nothing and clears nothing with memset calls, so one step (qc_qlinear
    and qc_latent_delta with caller-owned workspaces) can be captured once and replayed.  Every
    replay, with eager work and synchronizations in between, must give the eager bits."""
    rng = np.random.default_rng(5)
    M, K, N = 777, 1152, 392
    x = dev(random_x(rng, M, K, "bf16"))
    pw = qc.pack_weight_t(dev((rng.standard_normal((N, K)) * 0.02).astype(np.float32)), 4)
    b = dev((rng.standard_normal(N) * 0.01).astype(np.float32))
    n = 1 << 20
    cur, prev = (dev(a) for a in synth.latent_pair(seed=3, n=n))
    ws, dws = qc.qlinear_workspace_t(M, K, N), qc.latent_delta_workspace_t(n)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    out3 = torch.empty(3, dtype=torch.float32, device="cuda")

    def step():
        qc.qlinear_t(x, pw, b, "gelu_tanh", "bf16", workspace=ws, Y=Y, act_bits=6)
        qc.latent_delta_t(cur, prev, workspace=dws, out3=out3)

    # Captured before anything in this test ran eagerly: no call needs a set-up step (an
    # attribute, an allocation, a memset) that capture would refuse.
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    replays = []
    for _ in range(3):
        Y.fill_(0)
        out3.fill_(0)
        ws.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replays.append((Y.clone(), out3.clone()))
    Y.fill_(0)
    out3.fill_(0)
    step()  # eager
    torch.cuda.synchronize()
    for y_g, d_g in replays:
        assert torch.equal(y_g.view(torch.int16), Y.view(torch.int16))
        assert torch.equal(d_g.view(torch.int32), out3.view(torch.int32))


# ------------------------------------------------------------------ full-size configs, sampled rows

def sampled_rows_case(case: synth.LinearCase, rows_wanted=96, layer=0, x=None):
    M, K, N = case.M, case.K, case.N
    if x is None:
        x = case.x()
    W, b = case.weight(layer), case.bias(layer)
    pw = qc.pack_weight_t(dev(W), case.bits)
    ws = qc.qlinear_workspace_t(M, K, N)
    xd = dev(x)
    y = qc.qlinear_t(xd, pw, dev(b), case.epi, case.out_dtype, workspace=ws)
    acc = qc.qlinear_t(xd, pw, None, "none", "i32", workspace=ws)
    qx, sx = qc.debug_workspace_act_t(ws, M, K)
    torch.cuda.synchronize()
    rows = synth.sample_rows(M, rows_wanted)
    ridx = torch.from_numpy(rows).cuda()
    qw_ref, sw_ref = oracle.quant_weight(W, case.bits)
    assert bits_equal(pw.scale.cpu().numpy(), sw_ref)
    assert np.array_equal(qc.unpack_weight_codes_t(pw).cpu().numpy(), qw_ref)
    # rows are independent under per-token quantization: the oracle runs on the sampled rows
    ref = oracle.qlinear(x[rows], qw_ref, sw_ref, b, EPI_ORACLE[case.epi])
    assert bits_equal(sx[ridx].cpu().numpy(), ref["sx"])
    assert np.array_equal(qx[ridx].cpu().numpy(), ref["qx"])
    assert np.array_equal(acc[ridx].cpu().numpy(), ref["acc"])
    y_ref = oracle.bf16_bits_to_f64(oracle.round_bf16_bits(ref["y"]))
    assert_outputs_close(host_f64(y[ridx]), y_ref, RTOL["bf16"])
    # whole-tensor properties that hold at any size
    q_all = qx.to(torch.int16).abs().amax(dim=1)
    assert int(q_all.min()) == 127 and int(q_all.max()) == 127
    assert torch.isfinite(y.float()).all()


def test_config_qkv_256_sampled_rows():
    sampled_rows_case(synth.QKV_256)


def test_config_fc1_gelu_512_sampled_rows():
    sampled_rows_case(synth.FC1_512)


@pytest.mark.parametrize("case", [synth.FC2_512_W8, synth.FC2_512_W4], ids=["w8", "w4"])
def test_config_fc2_512_sampled_rows(case):
    sampled_rows_case(case, rows_wanted=48)


def _sweep_layer(kind, bits):
    """(index, case) of the first layer of the 28-block sweep with this shape and weight
    bit-width, as the seeded importance mask assigns them."""
    for i, c in enumerate(synth.stdit_block_layers()):
        if c.name.endswith("_" + kind) and c.bits == bits:
            return i, c
    raise AssertionError(f"the mask gives no {kind} layer at {bits} bits")


_sweep_x = {}


@pytest.mark.parametrize("kind,bits", [("out", 8), ("out", 4), ("qkv", 4), ("fc1", 4), ("fc2", 8),
                                       ("fc2", 4)])
def test_config_sweep28_sampled_rows(kind, bits):
    """Layers of the 28-block sweep at its full M = 131072 (CFG batch 2), with the weights of
    their own layer index: the shapes and bit-width mixes the single-layer configurations do
    not reach (out-projection 1152 -> 1152, 4-bit QKV and fc1, M twice as large)."""
    i, case = _sweep_layer(kind, bits)
    assert case.M == 131072
    key = (case.K, case.post_gelu, case.outliers)
    if key not in _sweep_x:
        _sweep_x.clear()             # at most one activation tensor (up to 1.2 GB) is kept
        _sweep_x[key] = case.x()
    sampled_rows_case(case, rows_wanted=48 if case.K > 2000 else 64, layer=i, x=_sweep_x[key])
    if kind == "fc2" and bits == 4:
        _sweep_x.clear()


@pytest.mark.parametrize("bits,K,epi,out,asym", [
    (8, 1000, "gelu_tanh", "bf16", False), (8, 1152, "none", "f32", False),
    (4, 2200, "gelu_erf", "bf16", False), (4, 1136, "none", "f32", True),
    (8, 1136, "gelu_tanh", "bf16", True)])
def test_qlinear_weights_resident_in_lds_ragged_shapes(bits, K, epi, out, asym):
    """The GEMM kernel that keeps its weight tile in LDS, on a problem it is chosen for whose
    edges are all ragged: 80037 tokens (the last 512-token round and the last 64-token tile are
    partial), 3401 channels (a partial last channel tile, scalar stores), K below the padded
    reduction length.  X repeats a block of 1024 generated rows, so the oracle's result for the
    block is the expected result of every repetition: all outputs are compared."""
    period, M, N = 1024, 80037, 3401
    assert qc.qc_debug_gemm_kernel(M, K, N, bits) == 2
    rng = np.random.default_rng(1000 * bits + K)
    block = post_gelu_x(rng, period, K, "bf16") if asym else random_x(rng, period, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    qw_ref, sw_ref = oracle.quant_weight(W, bits)
    xd = dev(block).repeat((M + period - 1) // period, 1)[:M].contiguous()
    pw = qc.pack_weight_t(dev(W), bits)
    if asym:
        ref = oracle.qlinear_asym(block, qw_ref, sw_ref, b, EPI_ORACLE[epi], 8)
        rs = qc.weight_row_sums_t(pw)
        ws = qc.qlinear_asym_workspace_t(M, K, N)
        y = qc.qlinear_asym_t(xd, pw, rs, dev(b), epi, out, workspace=ws)
        acc = qc.qlinear_asym_t(xd, pw, rs, None, "none", "i32", workspace=ws)
        acc_ref = oracle.gemm_i32((ref["qx"].astype(np.int16) - 128).astype(np.int8), qw_ref)
    else:
        ref = oracle.qlinear(block, qw_ref, sw_ref, b, EPI_ORACLE[epi])
        ws = qc.qlinear_workspace_t(M, K, N)
        y = qc.qlinear_t(xd, pw, dev(b), epi, out, workspace=ws)
        acc = qc.qlinear_t(xd, pw, None, "none", "i32", workspace=ws)
        acc_ref = ref["acc"]
    torch.cuda.synchronize()
    assert y.shape == (M, N) and acc.shape == (M, N)
    assert np.array_equal(acc[:period].cpu().numpy(), acc_ref)
    y_ref = ref["y"]
    y_ref = (oracle.bf16_bits_to_f64(oracle.round_bf16_bits(y_ref)) if out == "bf16"
             else oracle.round_f32(y_ref).astype(np.float64))
    assert_outputs_close(host_f64(y[:period]), y_ref, RTOL[out])
    # every other row against the one a period above it, bit for bit
    assert torch.equal(acc[period:], acc[:-period])
    as_int = torch.int16 if out == "bf16" else torch.int32
    assert torch.equal(y[period:].view(as_int), y[:-period].view(as_int))


def test_qlinear_weights_resident_in_lds_seeded_shapes():
    """Seeded shapes the resident-weight kernel is chosen for, from the shortest reduction (three
    64-k stages) to the longest that fits, with channel counts on both sides of a pass of 32
    channel tiles; raw accumulators and bf16 outputs of every row against the oracle's result for
    the repeated block of rows."""
    rng = np.random.default_rng(77)
    period, done = 512, 0
    for bits, K in ((8, 192), (8, 330), (4, 2304), (8, 768), (4, 96), (8, 1152)):
        for _ in range(40):
            M = int(rng.integers(66000, 150000))
            N = int(rng.integers(2100, 6000))
            if qc.qc_debug_gemm_kernel(M, K, N, bits) == 2:
                break
        else:
            raise AssertionError("no shape found that takes the resident kernel")
        block = random_x(rng, period, K, "bf16")
        W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
        b = (rng.standard_normal(N) * 0.01).astype(np.float32)
        qw_ref, sw_ref = oracle.quant_weight(W, bits)
        ref = oracle.qlinear(block, qw_ref, sw_ref, b, oracle.EPI_NONE)
        xd = dev(block).repeat((M + period - 1) // period, 1)[:M].contiguous()
        pw = qc.pack_weight_t(dev(W), bits)
        ws = qc.qlinear_workspace_t(M, K, N)
        y = qc.qlinear_t(xd, pw, dev(b), "none", "bf16", workspace=ws)
        acc = qc.qlinear_t(xd, pw, None, "none", "i32", workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(acc[:period].cpu().numpy(), ref["acc"]), (M, K, N, bits)
        assert torch.equal(acc[period:], acc[:-period]), (M, K, N, bits)
        y_ref = oracle.bf16_bits_to_f64(oracle.round_bf16_bits(ref["y"]))
        assert_outputs_close(host_f64(y[:period]), y_ref, RTOL["bf16"])
        assert torch.equal(y[period:].view(torch.int16), y[:-period].view(torch.int16)), (M, K, N, bits)
        del xd, y, acc, ws
        done += 1
    assert done == 6
    torch.cuda.empty_cache()


def test_qlinear_offsets_beyond_4_gib():
    """A problem whose input passes 2 GiB and whose output passes 4 GiB, so that a 32-bit byte or
    element offset anywhere on the path would wrap: M = 2^19 + 77 tokens of 1152 binary32 values
    (2.4 GB), 2304 channels of binary32 output (4.8 GB), and the same again as raw accumulators.
    X repeats a block of 8192 generated rows (tokens are independent), so the oracle runs on
    sampled rows of that block and every output row must also equal, bit for bit, the row 8192
    above it."""
    period, M, K, N = 8192, (1 << 19) + 77, 1152, 2304
    case = synth.LinearCase("offsets", M=period, K=K, N=N, x_dtype="f32", out_dtype="f32", outliers=12, seed=5)
    x_block = case.x()
    W, b = case.weight(), case.bias()
    xd = dev(x_block).repeat((M + period - 1) // period, 1)[:M].contiguous()
    assert xd.numel() * 4 > 1 << 31 and M * N * 4 > 1 << 32
    pw = qc.pack_weight_t(dev(W), 8)
    ws = qc.qlinear_workspace_t(M, K, N)
    y = qc.qlinear_t(xd, pw, dev(b), "none", "f32", workspace=ws)
    acc = qc.qlinear_t(xd, pw, None, "none", "i32", workspace=ws)
    qx, sx = qc.debug_workspace_act_t(ws, M, K)
    torch.cuda.synchronize()
    assert y.shape == (M, N) and acc.shape == (M, N)
    # rows next to the byte offsets 2^31 and 2^32 of X, of Y and of the code workspace
    edges = {0, 1, M - 1, M - 2, M - 77, M - 78}
    for row_bytes in (4 * K, 4 * N, K):
        for boundary in (1 << 30, 1 << 31, 1 << 32):
            r = boundary // row_bytes
            edges.update(q for q in (r - 1, r, r + 1) if 0 <= q < M)
    rng = np.random.default_rng(17)
    rows = np.unique(np.concatenate([np.fromiter(edges, np.int64), rng.integers(0, M, 40)]))
    ridx = torch.from_numpy(rows).cuda()
    qw_ref, sw_ref = oracle.quant_weight(W, 8)
    ref = oracle.qlinear(x_block[rows % period], qw_ref, sw_ref, b, oracle.EPI_NONE)
    assert bits_equal(sx[ridx].cpu().numpy(), ref["sx"])
    assert np.array_equal(qx[ridx].cpu().numpy(), ref["qx"])
    assert np.array_equal(acc[ridx].cpu().numpy(), ref["acc"])
    assert_outputs_close(host_f64(y[ridx]), ref["y"].astype(np.float64), RTOL["f32"])
    # every row against the one a period above it
    assert torch.equal(acc[period:], acc[:-period])
    assert torch.equal(y[period:].view(torch.int32), y[:-period].view(torch.int32))
    assert torch.equal(sx[period:M].view(torch.int32), sx[:M - period].view(torch.int32))


# ------------------------------------------------------------------ qc_latent_delta

@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 4096, 100003, 16 * 4 * 16 * 64 * 64, 9_000_001])
def test_latent_delta_matches_oracle(n):
    cur, prev = synth.latent_pair(seed=n % 97, n=n)
    ref = oracle.latent_delta(cur, prev)
    ws = qc.latent_delta_workspace_t(n)
    out = qc.latent_delta_t(dev(cur), dev(prev), workspace=ws).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(out - ref) <= 1e-5 * np.abs(ref)), (out, ref)
    # same workspace again, identical bits
    out2 = qc.latent_delta_t(dev(cur), dev(prev), workspace=ws).cpu().numpy()
    assert bits_equal(out2, out.astype(np.float32))


def test_latent_delta_closed_forms_and_determinism():
    n = 16 * 4 * 16 * 64 * 64
    cur, prev = synth.latent_pair(n=n)
    c, p = dev(cur), dev(prev)
    ws = qc.latent_delta_workspace_t(n)
    assert qc.latent_delta_t(p, p, workspace=ws).cpu().tolist()[0] == 0.0
    half = qc.latent_delta_t(p * 0.5, p, workspace=ws).cpu().numpy()
    assert abs(half[2] - 0.5) < 1e-6
    z = torch.zeros_like(p)
    assert qc.latent_delta_t(p, z, workspace=ws).cpu().tolist()[2] == math.inf
    assert qc.latent_delta_t(z, z, workspace=ws).cpu().tolist() == [0.0, 0.0, 0.0]
    first = qc.latent_delta_t(c, p, workspace=ws).cpu().numpy()
    assert 0.009 < first[2] < 0.011
    for _ in range(10):
        assert bits_equal(qc.latent_delta_t(c, p, workspace=ws).cpu().numpy(), first)


# ------------------------------------------------------------------ qc_layer_similarity

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [1, 7, 8, 9, 4096, 100003, 65536 * 1152])
def test_layer_similarity_matches_oracle(dtype, n):
    cur, prev = synth.latent_pair(seed=n % 89, n=n, delta=0.5)
    if dtype == "bf16":
        cur, prev = synth.to_bf16_bits(cur), synth.to_bf16_bits(prev)
    ref = oracle.layer_similarity(cur, prev)
    got = qc.layer_similarity_t(dev(cur), dev(prev)).cpu().numpy().astype(np.float64)
    norm = math.sqrt(ref[1] * ref[2])
    assert abs(got[0] - ref[0]) <= 1e-6 * norm + 1e-30
    assert abs(got[1] - ref[1]) <= 1e-6 * ref[1] and abs(got[2] - ref[2]) <= 1e-6 * ref[2]
    assert abs(got[3] - ref[3]) <= 2e-6
    again = qc.layer_similarity_t(dev(cur), dev(prev)).cpu().numpy()
    assert bits_equal(again, got.astype(np.float32))


def test_layer_similarity_closed_forms():
    a = torch.randn(1 << 20, device="cuda")
    assert abs(qc.layer_similarity_t(a, a).cpu().tolist()[3] - 1.0) < 1e-6
    assert abs(qc.layer_similarity_t(a, -a).cpu().tolist()[3] + 1.0) < 1e-6
    assert qc.layer_similarity_t(a, torch.zeros_like(a)).cpu().tolist()[3] == 0.0


# ------------------------------------------------------------------ qc_frame_gradient_norm

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("frames,inner", [(1, 64), (2, 1), (2, 8), (3, 7), (5, 1000), (16, 1152),
                                          (16, 9 * 1152 + 4), (16, 256 * 1152), (51, 32 * 32 * 4)])
def test_frame_gradient_norm_matches_oracle(dtype, frames, inner):
    m, _ = synth.latent_pair(seed=(frames * 131 + inner) % 83, n=frames * inner)
    m = m.reshape(frames, inner)
    if dtype == "bf16":
        m = synth.to_bf16_bits(m)
    ref = oracle.frame_gradient(m)
    got = qc.frame_gradient_norm_t(dev(m)).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2e-6 * np.abs(ref)), (got, ref)
    again = qc.frame_gradient_norm_t(dev(m)).cpu().numpy()
    assert bits_equal(again, got.astype(np.float32))


def test_frame_gradient_norm_closed_forms():
    F, inner = 12, 4096 + 8
    v = torch.randint(-8, 9, (inner,), device="cuda", dtype=torch.float32)
    ramp = torch.arange(F, device="cuda", dtype=torch.float32)[:, None] * v[None, :] + 3.0
    ss, norm = qc.frame_gradient_norm_t(ramp.contiguous()).cpu().tolist()
    want = (F - 1) * float((v.double() ** 2).sum())
    assert ss == np.float32(want) and abs(norm - math.sqrt(want)) <= 1e-6 * norm
    still = torch.randn(inner, device="cuda").expand(F, inner).contiguous()
    assert qc.frame_gradient_norm_t(still).cpu().tolist() == [0.0, 0.0]
    # the same numbers as one tensor [F, inner] or as a bf16 copy of an integer ramp
    assert qc.frame_gradient_norm_t(ramp.to(torch.bfloat16).contiguous()).cpu().tolist()[0] == \
        oracle.frame_gradient(synth.to_bf16_bits(ramp.cpu().numpy()))[0].astype(np.float32)


# ------------------------------------------------------------------ qc_cumulative_variation

@pytest.mark.parametrize("count", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("n", [1, 3, 4, 6, 2049, 100003, 16 * 4 * 16 * 64 * 64])
def test_cumulative_variation_matches_oracle(count, n):
    cur, _ = synth.latent_pair(seed=n % 79, n=n)
    prevs = np.stack([synth.latent_pair(seed=n % 79, n=n, delta=0.01 * (c + 1))[0]
                      for c in range(count)])
    ref = oracle.cumulative_variation(cur, prevs)
    dp = [dev(prevs[c]) for c in range(count)]
    got = qc.cumulative_variation_t(dev(cur), dp).cpu().numpy().astype(np.float64)
    assert got.shape == (count + 1,)
    assert np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-30), (got, ref)
    again = qc.cumulative_variation_t(dev(cur), dp).cpu().numpy()
    assert bits_equal(again, got.astype(np.float32))


def test_cumulative_variation_agrees_with_latent_delta_and_closed_forms():
    n = 1 << 20
    cur = torch.randint(-50, 50, (n,), device="cuda", dtype=torch.float32)
    out = qc.cumulative_variation_t(cur, [cur + 1, cur - 2, cur.clone()]).cpu().tolist()
    assert out == [float(n), 2.0 * n, 0.0, 3.0 * n]
    a, b = torch.randn(n, device="cuda"), torch.randn(n, device="cuda")
    one = qc.cumulative_variation_t(a, [b]).cpu().numpy()
    pair = qc.latent_delta_t(a, b).cpu().numpy()
    assert abs(one[0] - pair[0]) <= 1e-6 * pair[0] and one[1] == one[0]


def test_reductions_past_2_to_the_31_elements():
    """Tensors of 2^31 + 4099 elements (8.6 GB each): an element or byte index held in 32 bits
    anywhere in the reduction kernels would wrap.  The tensors repeat a generated block of 2^20
    elements 2048 times and end with its first 4099, so every sum is 2048 times the oracle's sum
    over the block plus its sum over that tail."""
    P, reps, tail = 1 << 20, 2048, 4099
    n = reps * P + tail
    assert n > 1 << 31
    cur_b, prev_b = synth.latent_pair(seed=9, n=P, delta=0.05)

    def tiled(block, length):
        t = torch.empty(length, dtype=torch.float32, device="cuda")
        full = length // P
        t[:full * P].view(full, P).copy_(dev(block)[None, :].expand(full, P))
        t[full * P:] = dev(block)[:length - full * P]
        return t

    def combined(fn, tail_len, *blocks):
        whole = np.asarray(fn(*blocks), np.float64)
        part = np.asarray(fn(*(b[..., :tail_len] for b in blocks)), np.float64)
        return reps * whole + part

    cur, prev = tiled(cur_b, n), tiled(prev_b, n)

    ref = combined(oracle.latent_delta, tail, cur_b, prev_b)       # the ratio is redone below
    got = qc.latent_delta_t(cur, prev).cpu().numpy().astype(np.float64)
    assert abs(got[0] - ref[0]) <= 1e-5 * ref[0] and abs(got[1] - ref[1]) <= 1e-5 * ref[1]
    assert abs(got[2] - ref[0] / ref[1]) <= 1e-5 * ref[0] / ref[1]

    ref = combined(oracle.layer_similarity, tail, cur_b, prev_b)
    got = qc.layer_similarity_t(cur, prev).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got[:3] - ref[:3]) <= 1e-6 * np.abs(ref[:3]))
    assert abs(got[3] - ref[0] / math.sqrt(ref[1] * ref[2])) <= 2e-6

    got = qc.cumulative_variation_t(cur, [prev, prev]).cpu().numpy().astype(np.float64)
    num = combined(oracle.latent_delta, tail, cur_b, prev_b)[0]
    assert np.all(np.abs(got - np.array([num, num, 2 * num])) <= 1e-5 * num)
    del cur, prev

    inner = reps * P + 4096                                           # a multiple of 8: vector path
    frames = torch.empty((2, inner), dtype=torch.float32, device="cuda")
    frames[0], frames[1] = tiled(prev_b, inner), tiled(cur_b, inner)
    ss = combined(lambda m: oracle.frame_gradient(m)[:1], 4096, np.stack([prev_b, cur_b]))[0]
    got = qc.frame_gradient_norm_t(frames).cpu().numpy().astype(np.float64)
    assert abs(got[0] - ss) <= 2e-6 * ss and abs(got[1] - math.sqrt(ss)) <= 2e-6 * math.sqrt(ss)
    del frames
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ rotation fused into quantization

@pytest.mark.parametrize("rot_block", [16, 32, 64, 128])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,K,act_bits", [(256, 1152, 8), (77, 4608, 6), (9, 128, 8), (33, 9216, 4),
                                          (5, 2304, 8), (1, 640, 8)])
def test_quant_act_rot_bit_exact(rot_block, dtype, M, K, act_bits):
    rng = np.random.default_rng(M * 1009 + K + rot_block)
    x = random_x(rng, M, K, dtype)
    q_ref, s_ref = oracle.quant_act_rot(x, rot_block, act_bits)
    qx, sx = qc.quant_act_t(dev(x), act_bits, rot_block)
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), s_ref)
    assert np.array_equal(qx.cpu().numpy(), q_ref)


@pytest.mark.parametrize("rot_block", [16, 64, 128])
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("N,K", [(1152, 1152), (200, 128), (3, 640), (129, 4608)])
def test_pack_weight_rot_codes_and_scales_bit_exact(rot_block, bits, N, K):
    rng = np.random.default_rng(N * 7919 + K + bits + rot_block)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    W[N // 2] = 0
    q_ref, s_ref = oracle.quant_weight_rot(W, bits, rot_block)
    pw = qc.pack_weight_t(dev(W), bits, rot_block)
    codes = qc.unpack_weight_codes_t(pw)
    torch.cuda.synchronize()
    assert bits_equal(pw.scale.cpu().numpy(), s_ref)
    assert np.array_equal(codes.cpu().numpy(), q_ref)


@pytest.mark.parametrize("bits,act_bits,rot_block", [(8, 8, 128), (4, 8, 128), (4, 6, 64), (8, 4, 16)])
def test_qlinear_rot_matches_oracle(bits, act_bits, rot_block):
    rng = np.random.default_rng(bits * 100 + act_bits * 10 + rot_block)
    M, K, N = 520, 1152, 300
    x = random_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    run_linear_case(x, W, b, bits, "gelu_tanh", "bf16", act_bits=act_bits, rot_block=rot_block)
    run_linear_case(x, W, b, bits, "none", "f32", act_bits=act_bits, rot_block=rot_block)


def test_qlinear_rot_leaves_the_product_and_cuts_outlier_error():
    """(X H)(W H / b)^T = X W^T: with outlier channels the rotated W4A8 linear is closer to the
    exact product than the plain one, and on integers both are exact."""
    rng = np.random.default_rng(2024)
    M, K, N = 512, 1152, 256
    x = random_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    exact = oracle.bf16_bits_to_f64(x) @ W.astype(np.float64).T
    xd = dev(x)
    err = {}
    for rot in (0, 128):
        pw = qc.pack_weight_t(dev(W), 4, rot)
        y = host_f64(qc.qlinear_t(xd, pw, None, "none", "f32", rot_block=rot))
        err[rot] = math.sqrt(float(np.mean((y - exact) ** 2)) / float(np.mean(exact ** 2)))
    assert err[128] < err[0] and err[128] < 0.2, err
    # integer operands whose rotated images stay on the code grid: every step is exact
    xi = np.zeros((256, 256), np.float32)
    xi[np.arange(256), np.arange(256)] = 127.0            # rows of 127 * identity
    wi = np.zeros((128, 256), np.float32)
    wi[np.arange(128), np.arange(128) * 2] = 7.0
    pw = qc.pack_weight_t(dev(wi), 8, 128)
    y = host_f64(qc.qlinear_t(dev(xi), pw, None, "none", "f32", rot_block=128))
    want = xi.astype(np.float64) @ wi.astype(np.float64).T
    assert np.max(np.abs(y - want)) <= 1e-3 * 889


# ------------------------------------------------------------------ asymmetric activations

def post_gelu_x(rng, M, K, dtype):
    g = rng.standard_normal((M, K))
    x = (0.5 * g * (1 + np.tanh(0.7978845608 * (g + 0.044715 * g ** 3)))).astype(np.float32)
    return synth.to_bf16_bits(x) if dtype == "bf16" else x


@pytest.mark.parametrize("act_bits", [8, 6, 4])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,K", [(256, 1152), (77, 4608), (9, 16), (33, 9216), (5, 2304)])
def test_quant_act_asym_bit_exact(act_bits, dtype, M, K):
    rng = np.random.default_rng(M * 31 + K + act_bits)
    x = post_gelu_x(rng, M, K, dtype) if M % 2 else random_x(rng, M, K, dtype)
    if dtype == "f32" and M > 8:
        x[3] += np.float32(1000.0)     # a row far from zero: large zero point
        x[4] = np.float32(-2.5)        # a constant row: range floor
        x[5] = 0
    q_ref, s_ref, z_ref = oracle.quant_act_asym(x, act_bits)
    qx, sx, zx = qc.quant_act_asym_t(dev(x), act_bits)
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), s_ref)
    assert bits_equal(zx.cpu().numpy(), z_ref)
    assert np.array_equal(qx.cpu().numpy(), q_ref)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("N,K", [(1152, 1152), (200, 136), (3, 16), (129, 4608)])
def test_weight_row_sums_exact(bits, N, K):
    rng = np.random.default_rng(N + K + bits)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    W[0] = np.abs(W[0])                     # a channel whose codes do not cancel
    q_ref, _ = oracle.quant_weight(W, bits)
    pw = qc.pack_weight_t(dev(W), bits)
    sums = qc.weight_row_sums_t(pw).cpu().numpy()
    assert np.array_equal(sums, q_ref.astype(np.int64).sum(axis=1))


def run_asym_case(x, W, b, bits, epi, out, act_bits=8):
    M, K = x.shape
    N = W.shape[0]
    qw_ref, sw_ref = oracle.quant_weight(W, bits)
    ref = oracle.qlinear_asym(x, qw_ref, sw_ref, b, EPI_ORACLE[epi], act_bits)
    xd, pw = dev(x), qc.pack_weight_t(dev(W), bits)
    rs = qc.weight_row_sums_t(pw)
    bd = None if b is None else dev(b)
    ws = qc.qlinear_asym_workspace_t(M, K, N)
    y = qc.qlinear_asym_t(xd, pw, rs, bd, epi, out, workspace=ws, act_bits=act_bits)
    qx, sx, zx = qc.debug_workspace_act_asym_t(ws, M, K, act_bits)
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), ref["sx"]), "activation scales differ"
    assert np.array_equal(zx.cpu().numpy(), ref["zx"]), "zero points differ"
    assert np.array_equal(qx.cpu().numpy(), ref["qx"]), "activation codes differ"
    # the MFMA loop's own sum, on the stored signed bytes
    acc = qc.qlinear_asym_t(xd, pw, rs, None, "none", "i32", workspace=ws, act_bits=act_bits)
    shifted = (ref["qx"].astype(np.int16) - (128 if act_bits == 8 else 0)).astype(np.int8)
    assert np.array_equal(acc.cpu().numpy(), oracle.gemm_i32(shifted, qw_ref))
    y_ref = ref["y"]
    if out == "bf16":
        y_ref = oracle.bf16_bits_to_f64(oracle.round_bf16_bits(y_ref))
    else:
        y_ref = oracle.round_f32(y_ref).astype(np.float64)
    assert_outputs_close(host_f64(y), y_ref, RTOL[out])
    return host_f64(y)


@pytest.mark.parametrize("bits,act_bits", [(8, 8), (4, 8), (4, 6), (8, 4)])
@pytest.mark.parametrize("epi,out", [("none", "f32"), ("gelu_tanh", "bf16")])
def test_qlinear_asym_matches_oracle(bits, act_bits, epi, out):
    rng = np.random.default_rng(bits * 100 + act_bits)
    M, K, N = 520, 1152, 300
    x = post_gelu_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    run_asym_case(x, W, b, bits, epi, out, act_bits=act_bits)


@pytest.mark.parametrize("M,K,N", [(1, 16, 1), (257, 64, 129), (33, 208, 77), (700, 4608, 130)])
def test_qlinear_asym_ragged_shapes(M, K, N):
    rng = np.random.default_rng(M + 3 * K + 5 * N)
    x = random_x(rng, M, K, "f32") + np.float32(0.75)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    run_asym_case(x, W, b, 8, "none", "f32")
    run_asym_case(x, W, None, 4, "gelu_erf", "bf16")


def test_qlinear_asym_gains_on_one_sided_input_and_is_exact_on_integers():
    rng = np.random.default_rng(7)
    M, K, N = 512, 4608, 256
    x = post_gelu_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    qw, sw = oracle.quant_weight(W, 8)
    exact = oracle.bf16_bits_to_f64(x) @ (sw.astype(np.float64)[:, None] * qw.astype(np.float64)).T
    pw = qc.pack_weight_t(dev(W), 8)
    rs = qc.weight_row_sums_t(pw)
    for act_bits in (8, 4):
        e_sym = np.abs(host_f64(qc.qlinear_t(dev(x), pw, None, "none", "f32", act_bits=act_bits)) - exact).mean()
        e_asym = np.abs(host_f64(qc.qlinear_asym_t(dev(x), pw, rs, None, "none", "f32", act_bits=act_bits)) - exact).mean()
        assert e_asym < 0.7 * e_sym, (act_bits, e_asym, e_sym)
    Xi = rng.integers(0, 256, size=(64, 1152)).astype(np.float32)
    Xi[:, 0], Xi[:, 1] = 0, 255
    Wi = rng.integers(-127, 128, size=(128, 1152)).astype(np.float32)
    Wi[:, 0] = 127
    pwi = qc.pack_weight_t(dev(Wi), 8)
    y = host_f64(qc.qlinear_asym_t(dev(Xi - 100), pwi, qc.weight_row_sums_t(pwi), None, "none", "f32"))
    want = (Xi.astype(np.float64) - 100) @ Wi.astype(np.float64).T
    assert np.max(np.abs(y - want)) <= 2e-7 * np.max(np.abs(want)) * 4


# ------------------------------------------------------------------ one scale per layer input

@pytest.mark.parametrize("act_bits", [8, 6, 4])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,K", [(256, 1152), (77, 4608), (1, 16), (9, 1000), (130, 7), (3, 10000),
                                 (2048, 1152)])
def test_quant_act_tensor_bit_exact(act_bits, dtype, M, K):
    rng = np.random.default_rng(M * 17 + K + act_bits)
    x = random_x(rng, M, K, dtype)
    q_ref, s_ref = oracle.quant_act_tensor(x, act_bits)
    qx, sx = qc.quant_act_tensor_t(dev(x), act_bits)
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), np.array([s_ref], np.float32))
    assert np.array_equal(qx.cpu().numpy(), q_ref)


def _quantizer_on_a_repeated_block(how, dtype, M, K):
    """X repeats a generated block of 2048 rows, so the oracle's codes for the block are the
    expected codes of every repetition (for the one-scale-per-tensor form too: the tensor's
    absmax is the block's); every code and scale of the large tensor is compared."""
    period = 2048
    block = random_x(np.random.default_rng(23), period, K, dtype)
    xd = dev(block).repeat((M + period - 1) // period, 1)[:M].contiguous()
    aux = None
    if how == "token":
        q_ref, s_ref = oracle.quant_act(block)
        qx, sx = qc.quant_act_t(xd)
    elif how == "rot128":
        q_ref, s_ref = oracle.quant_act_rot(block, 128, 8)
        qx, sx = qc.quant_act_t(xd, 8, 128)
    elif how == "asym":
        q_ref, s_ref, z_ref = oracle.quant_act_asym(block, 8)
        qx, sx, aux = qc.quant_act_asym_t(xd, 8)
    else:
        q_ref, s_one = oracle.quant_act_tensor(block, 8)
        s_ref = None
        qx, sx = qc.quant_act_tensor_t(xd, 8)
        assert bits_equal(sx.cpu().numpy(), np.array([s_one], np.float32))
    torch.cuda.synchronize()
    del xd
    q_ref_d = torch.from_numpy(q_ref.view(np.int8)).cuda()
    reps, rest = divmod(M, period)
    codes = qx.view(torch.int8)
    assert torch.equal(codes[:reps * period].view(reps, period, K), q_ref_d[None].expand(reps, period, K))
    assert torch.equal(codes[reps * period:], q_ref_d[:rest])
    if s_ref is not None:
        s_ref_d = torch.from_numpy(s_ref.view(np.int32)).cuda()
        bits = sx.view(torch.int32)
        assert torch.equal(bits[:reps * period].view(reps, period), s_ref_d[None].expand(reps, period))
        assert torch.equal(bits[reps * period:], s_ref_d[:rest])
    if aux is not None:
        z_ref_d = torch.from_numpy(z_ref.view(np.int32)).cuda()
        bits = aux.view(torch.int32)
        assert torch.equal(bits[:reps * period].view(reps, period), z_ref_d[None].expand(reps, period))
        assert torch.equal(bits[reps * period:], z_ref_d[:rest])
    del qx, sx, codes
    torch.cuda.empty_cache()


@pytest.mark.parametrize("how", ["token", "rot128", "asym", "tensor"])
def test_quantizers_offsets_beyond_4_gib(how):
    """2^19 + 5 rows of 4608 bf16 values: 4.8 GB of input and 2.4 GB of codes, past what 32-bit
    byte offsets reach, on the kernel that cuts a row into four column slices (and, with codes
    beyond the last-level cache, the variant with non-temporal stores)."""
    M, K = (1 << 19) + 5, 4608
    assert M * K * 2 > 1 << 32 and M * K > 1 << 31
    _quantizer_on_a_repeated_block(how, "bf16", M, K)


@pytest.mark.parametrize("how", ["token", "rot128", "asym"])
@pytest.mark.parametrize("dtype,M", [("bf16", 98304 + 5), ("f32", 65536 + 5)])
def test_quantizers_sizes_that_stream_their_input(how, dtype, M):
    """Input plus codes beyond 256 MiB with the codes below it: the kernel variant that reads X
    with non-temporal loads."""
    K = 1152
    assert M * K <= 256 << 20 < M * K * ((2 if dtype == "bf16" else 4) + 1)
    _quantizer_on_a_repeated_block(how, dtype, M, K)


@pytest.mark.parametrize("bits,act_bits", [(8, 8), (4, 8), (4, 6)])
@pytest.mark.parametrize("M,K,N", [(520, 1152, 300), (33, 200, 77), (700, 4608, 130)])
def test_qlinear_tensor_matches_oracle(bits, act_bits, M, K, N):
    rng = np.random.default_rng(M + K + N + bits + act_bits)
    x = random_x(rng, M, K, "bf16")
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    qw_ref, sw_ref = oracle.quant_weight(W, bits)
    ref = oracle.qlinear_tensor(x, qw_ref, sw_ref, b, oracle.EPI_GELU_TANH, act_bits)
    xd, pw = dev(x), qc.pack_weight_t(dev(W), bits)
    ws = qc.qlinear_tensor_workspace_t(M, K, N)
    y = qc.qlinear_tensor_t(xd, pw, dev(b), "gelu_tanh", "bf16", workspace=ws, act_bits=act_bits)
    qx, sx = qc.debug_workspace_act_t(ws, M, K)
    acc = qc.qlinear_tensor_t(xd, pw, None, "none", "i32", workspace=ws, act_bits=act_bits)
    torch.cuda.synchronize()
    assert bits_equal(sx.cpu().numpy(), np.full(M, ref["sx"], np.float32))
    assert np.array_equal(qx.cpu().numpy(), ref["qx"])
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    y_ref = oracle.bf16_bits_to_f64(oracle.round_bf16_bits(ref["y"]))
    assert_outputs_close(host_f64(y), y_ref, RTOL["bf16"])
