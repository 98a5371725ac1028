"""qc_latent_delta_static (the entry point that allocates nothing) against qc_latent_delta.

Collected last on purpose: the file name sorts after every other test file.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_06545_amd import binding as qc
from paper_2503_06545_amd import synth

pytestmark = pytest.mark.gpu


def _both(cur, prev, n, out_static, out_ws, ws):
    stream = torch.cuda.current_stream().cuda_stream
    st = qc.qc_latent_delta_static(cur.data_ptr(), prev.data_ptr(), n, out_static.data_ptr(), stream)
    assert st == qc.QC_OK, qc.status_string(st)
    st = qc.qc_latent_delta(cur.data_ptr(), prev.data_ptr(), n, out_ws.data_ptr(), ws.data_ptr(),
                            ws.numel(), stream)
    assert st == qc.QC_OK, qc.status_string(st)
    torch.cuda.synchronize()
    return out_static.cpu().numpy(), out_ws.cpu().numpy()


def test_static_scratch_call_equals_the_workspace_call_twice_in_a_row():
    n_big, n_small = 4_194_304 + 3, 70_001       # the second call is the smaller one
    cur_h, prev_h = synth.latent_pair(seed=5, n=n_big)
    cur, prev = torch.from_numpy(cur_h).cuda(), torch.from_numpy(prev_h).cuda()
    ws = qc.latent_delta_workspace_t(n_big)
    # every buffer exists before the calls under test: they must not need an allocation
    outs = [torch.full((3,), -1.0, device="cuda") for _ in range(4)]
    torch.cuda.synchronize()
    for k, n in enumerate((n_big, n_small)):
        got, want = _both(cur, prev, n, outs[2 * k], outs[2 * k + 1], ws)
        assert got.view(np.uint32).tolist() == want.view(np.uint32).tolist(), (n, got, want)
        ref = np.asarray(oracle.latent_delta(cur_h[:n], prev_h[:n]), np.float64)
        assert np.all(np.abs(got.astype(np.float64) - ref) <= 1e-5 * np.abs(ref)), (n, got, ref)


def test_static_scratch_call_rejects_bad_arguments_before_any_launch():
    a = torch.zeros(16, device="cuda")
    out = torch.zeros(3, device="cuda")
    A, O = a.data_ptr(), out.data_ptr()
    assert qc.qc_latent_delta_static(0, A, 8, O) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_latent_delta_static(A, A, 0, O) == qc.QC_ERR_INVALID_ARG
    assert qc.qc_latent_delta_static(A, A + 4, 8, O) == qc.QC_ERR_INVALID_ARG   # misaligned
    assert qc.qc_latent_delta_static(A, A, qc.QC_LATENT_DELTA_STATIC_MAX_N + 1, O) == qc.QC_ERR_UNSUPPORTED
    assert "UNSUPPORTED" in qc.status_string(qc.QC_ERR_UNSUPPORTED)
