"""Host checks of the synthetic input generators (no attention arithmetic here)."""
import numpy as np
import pytest
import torch

import workloads as wl


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(100000).astype(np.float32) * np.float32(3.0)
    x[:4] = [0.0, -0.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8]      # ties -> even
    bits = wl.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, want)
    np.testing.assert_array_equal(wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(bits)), bits)


def test_qkv_seeded_and_padded():
    a = wl.make_qkv(1, 2, 128, 64, 100, seed=3)
    b = wl.make_qkv(1, 2, 128, 64, 100, seed=3)
    c = wl.make_qkv(1, 2, 128, 64, 100, seed=4)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    assert not np.array_equal(a[0], c[0])
    assert all((x[:, :, 100:] == 0).all() for x in a)
    n = wl.make_qkv(1, 2, 128, 64, 100, seed=3, pad_fill="nan")
    assert all((x[:, :, 100:] == wl.BF16_NAN).all() for x in n)
    f = wl.bf16_bits_to_f32(a[0][:, :, :100])
    assert abs(f.mean()) < 0.05 and abs(f.std() - 1.0) < 0.05


def test_workload_table_shapes():
    w = wl.WORKLOADS
    assert (w["sd3_1024"].nb, w["flux_1024"].nb, w["flux_2048"].nb, w["tiny"].nb) == (35, 36, 132, 4)
    assert w["sd3_1024"].N == 4480 and w["sd3_1024"].kv_len == 4096 + 333
    assert w["flux_1024"].kv_len == 4096 + 512 and w["flux_2048"].kv_len == 16384 + 512
    assert abs(w["flux_1024"].dense_flops() / 1e9 - 260.92) < 0.01
    assert abs(w["sd3_1024"].dense_flops() / 1e9 - 120.52) < 0.01
    assert abs(w["grpo_sd3"].dense_flops() / 1e9 - 964.17) < 0.01
    for x in w.values():
        assert x.N % x.block == 0 and x.N - x.kv_len < x.block


def test_tiny_mask():
    w = wl.WORKLOADS["tiny"]
    m = w.mask(0.5)
    assert m.shape == (1, 2, 4, 4) and (m[:, :, np.arange(4), np.arange(4)] == 1).all()
    assert (w.mask(1.0) == 1).all()
    assert not np.array_equal(m[0, 0], m[0, 1])


@pytest.mark.parametrize("name,density,img_kept,eff", [
    ("sd3_1024", 0.25, 256, (201 + 256) / 1225),
    ("flux_1024", 0.5, 512, (272 + 512) / 1296),
    ("flux_1024", 0.2, 205, (272 + 205) / 1296),
])
def test_text_dense_masks_hit_exact_counts(name, density, img_kept, eff):
    w = wl.WORKLOADS[name]
    m = w.mask(density)
    nI = w.nb - w.n_text_blocks
    assert (m[:, :, nI:, :] == 1).all() and (m[:, :, :, nI:] == 1).all()
    assert (m[:, :, np.arange(nI), np.arange(nI)] == 1).all()
    assert (m[:, :, :nI, :nI].sum(axis=(2, 3)) == img_kept).all()
    assert abs(wl.effective_density(m, w.block, w.kv_len) - eff) < 1e-9
    assert not np.array_equal(m[0, 0], m[0, 1])               # per-head masks
    assert (w.mask(1.0) == 1).all()
    np.testing.assert_array_equal(m, w.mask(density))           # seeded


def test_grpo_per_sample_densities():
    w = wl.WORKLOADS["grpo_sd3"]
    ds = w.sample_densities()
    assert len(ds) == 8 and set(ds) <= {1.0, 0.5, 0.3, 0.15} and len(set(ds)) >= 2
    m = w.mask("mixed")
    nI = 32
    for b, d in enumerate(ds):
        want = nI * nI if d >= 1.0 else round(d * nI * nI)
        assert (m[b, :, :nI, :nI].sum(axis=(1, 2)) == want).all()


@pytest.mark.parametrize("density,half_width,total", [(0.1, 1, 1742), (0.3, 8, 5227)])
def test_band_masks_total_density(density, half_width, total):
    w = wl.WORKLOADS["flux_2048"]
    m = w.mask(density)
    assert (m.sum(axis=(2, 3)) == total).all()
    nI = 128
    i, j = np.meshgrid(np.arange(nI), np.arange(nI), indexing="ij")
    assert (m[0, 5, :nI, :nI][np.abs(i - j) <= half_width] == 1).all()
    assert (m[:, :, nI:, :] == 1).all() and (m[:, :, :, nI:] == 1).all()
    assert abs(wl.effective_density(m, 128, w.kv_len) - total / 132 ** 2) < 1e-12


def test_sample_rows_cover_edges():
    rows = wl.sample_rows(2, 3, 4480, 4429, 128, 64, seed=1)
    assert rows.shape == (64, 3) and len({tuple(r) for r in rows}) == 64
    t = {tuple(r) for r in rows}
    assert (0, 0, 0) in t and (1, 2, 4428) in t and (0, 2, 4479) in t


def test_block_structured_inputs_have_a_prunable_map():
    """The generator for the mask-selection legs: seeded, padded like make_qkv, and (checked with
    the selection oracle) its pooled attention map concentrates on few key-blocks per row, which
    i.i.d. inputs of the same shape do not."""
    from oracle import mask_oracle as mo
    B, H, nb, block, D = 1, 2, 12, 64, 64
    N = nb * block
    a = wl.make_qkv_block_structured(B, H, N, D, block, kv_len=N - 10, seed=5, n_text_blocks=2, pad_fill="nan")
    b = wl.make_qkv_block_structured(B, H, N, D, block, kv_len=N - 10, seed=5, n_text_blocks=2, pad_fill="nan")
    for x, y in zip(a, b):
        assert x.dtype == np.uint16 and x.shape == (B, H, N, D) and (x == y).all()
        assert (x[:, :, N - 10:] == wl.BF16_NAN).all() and not (x[:, :, :N - 10] == wl.BF16_NAN).any()
    structured = mo.select_mask(a[0], a[1], block, N - 10, N, 0.9)
    plain_q, plain_k, _ = wl.make_qkv(B, H, N, D, N - 10, seed=5)
    plain = mo.select_mask(plain_q, plain_k, block, N - 10, N, 0.9)
    assert structured.mean() < 0.3 < 0.8 < plain.mean()
