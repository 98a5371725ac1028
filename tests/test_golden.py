"""Stored oracle outputs (tests/golden/oracle_outputs.json, written by tests/golden/make_golden.py
from the oracle alone): the oracle still reproduces them, and the GPU path matches them."""
import importlib.util
import json
import os
import zlib

import numpy as np
import pytest

import oracle
from paper_2503_06545_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
GOLDEN = os.path.join(HERE, "golden", "oracle_outputs.json")


def load_maker():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def stored():
    with open(GOLDEN) as f:
        return json.load(f)


def test_oracle_reproduces_the_stored_outputs():
    assert load_maker().build() == stored()


def crc(a) -> int:
    return zlib.crc32(np.ascontiguousarray(a).tobytes()) & 0xFFFFFFFF


CASES = {"tiny_w8a8": synth.TINY, "stdit_qkv_256": synth.QKV_256}


@pytest.mark.gpu
@pytest.mark.parametrize("index", range(5))
def test_gpu_path_matches_the_stored_outputs(index):
    import torch

    from paper_2503_06545_amd import binding as qc
    g = stored()["linear"][index]
    case = CASES[g["case"]]
    x = case.x() if g["rows"] == case.M else case.x_rows(0, g["rows"])
    M, K = x.shape
    if x.dtype == np.uint16:
        xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        xd = torch.from_numpy(x).cuda()
    pw = qc.pack_weight_t(torch.from_numpy(case.weight()).cuda(), g["bits"], g["rot_block"])
    bd = torch.from_numpy(case.bias()).cuda()
    ws = qc.qlinear_workspace_t(M, K, case.N)
    kw = dict(workspace=ws, act_bits=g["act_bits"], rot_block=g["rot_block"])
    y = qc.qlinear_t(xd, pw, bd, g["epi"], "f32", **kw).cpu().numpy().astype(np.float64)
    qx, sx = qc.debug_workspace_act_t(ws, M, K)
    acc = qc.qlinear_t(xd, pw, None, "none", "i32", **kw).cpu().numpy()
    assert crc(qc.unpack_weight_codes_t(pw).cpu().numpy()) == g["qw_crc32"]
    assert crc(pw.scale.cpu().numpy()) == g["sw_crc32"]
    assert crc(qx.cpu().numpy()) == g["qx_crc32"] and crc(sx.cpu().numpy()) == g["sx_crc32"]
    assert [int(v) for v in sx.cpu().numpy()[:4].view(np.uint32)] == g["sx_bits_first4"]
    assert crc(acc) == g["acc_crc32"]
    N = case.N
    pts = [(m % M, n % N) for m, n in load_maker().SAMPLES]
    assert [int(acc[m, n]) for m, n in pts] == g["acc_samples"]
    want = np.array([float.fromhex(h) for h in g["y_samples_hex"]])
    got = np.array([y[m, n] for m, n in pts])
    rms = abs(float.fromhex(g["y_sum_hex"])) / y.size + float(np.sqrt(np.mean(y ** 2)))
    assert np.all(np.abs(got - want) <= 1e-3 * np.abs(want) + 1e-3 * rms)
    assert abs(float(np.sum(y)) - float.fromhex(g["y_sum_hex"])) <= 1e-4 * float(np.sum(np.abs(y)))


@pytest.mark.gpu
def test_gpu_reductions_match_the_stored_outputs():
    import torch

    from paper_2503_06545_amd import binding as qc
    g = stored()["reductions"]
    val = lambda key: np.array([float.fromhex(h) for h in g[key]])
    cur, prev = synth.latent_pair(seed=3, n=100003)
    c, p = torch.from_numpy(cur).cuda(), torch.from_numpy(prev).cuda()
    near = lambda got, want, tol: np.all(np.abs(got.astype(np.float64) - want) <= tol * np.abs(want) + 1e-30)
    assert near(qc.latent_delta_t(c, p).cpu().numpy(), val("latent_delta_seed3_n100003_hex"), 1e-5)
    sim, want = qc.layer_similarity_t(c, p).cpu().numpy(), val("layer_similarity_seed3_n100003_hex")
    assert near(sim[1:], want[1:], 2e-6) and abs(sim[0] - want[0]) <= 1e-6 * np.sqrt(want[1] * want[2])
    m = c[:7 * 14286].reshape(7, 14286).contiguous()
    assert near(qc.frame_gradient_norm_t(m).cpu().numpy(), val("frame_gradient_seed3_7x14286_hex"), 2e-6)
    out = qc.cumulative_variation_t(c, [p, (p * 0.5).contiguous()]).cpu().numpy()
    assert near(out, val("cumulative_variation_seed3_n100003_hex"), 1e-5)
