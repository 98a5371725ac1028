"""The seeded input generators: deterministic, row-addressable, shaped like the STDiT layers."""
import numpy as np

from paper_2503_06545_amd import synth


def test_rows_are_addressable_and_deterministic():
    c = synth.QKV_256
    a = c.x_rows(100, 300)
    b = c.x_rows(0, 512)[100:300]
    assert a.dtype == np.uint16 and a.shape == (200, 1152)
    assert np.array_equal(a, b)
    assert np.array_equal(c.x_rows(100, 300), a)


def test_tiny_case_recipe():
    c = synth.TINY
    x = c.x()
    assert x.dtype == np.float32 and x.shape == (256, 1152)
    cols = synth.outlier_columns(c.seed, c.K, 8)
    assert len(set(cols.tolist())) == 8
    col_rms = np.sqrt((x.astype(np.float64) ** 2).mean(axis=0))
    assert np.all(col_rms[cols] > 10) and np.all(np.delete(col_rms, cols) < 2)
    w, b = c.weight(), c.bias()
    assert w.shape == (1152, 1152) and abs(w.std() - 0.02) < 1e-3
    assert b.shape == (1152,) and abs(b.std() - 0.01) < 2e-3


def test_post_gelu_distribution_is_one_sided():
    x = synth.FC2_512_W8.x_rows(0, 64)
    f = (x.astype(np.uint32) << 16).view(np.float32)
    assert f.min() > -0.18 and f.max() > 2.5


def test_bf16_cast_matches_torch():
    import torch
    x = synth.normal_rows(0, 99, 0, 64, 256)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(synth.to_bf16_bits(x), ref)


def test_latent_pair_and_layer_mask():
    cur, prev = synth.latent_pair(n=100000)
    rel = np.abs(cur - prev).sum() / np.abs(prev).sum()
    assert 0.009 < rel < 0.011
    layers = synth.stdit_block_layers()
    assert len(layers) == 112
    w4 = sum(l.bits == 4 for l in layers)
    assert 20 <= w4 <= 48
    rows = synth.sample_rows(65536, 64)
    assert rows.min() == 0 and rows.max() == 65535 and len(rows) >= 64
