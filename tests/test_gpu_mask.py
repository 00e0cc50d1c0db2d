"""GPU parity of the block-mask selection against its oracle.  The cut compares fp32 partial
sums, the oracle fp64 ones: a block whose inclusion decides whether a row's mass reaches tau to
within rounding may fall on either side, so the GPU mask must lie between the oracle's masks
for tau - 1e-5 and tau + 1e-5 (the rule is monotone in tau), and agree with the oracle's mask
for tau itself almost everywhere."""
import numpy as np
import pytest
import torch

import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import to_dev
from oracle import mask_oracle as mo

pytestmark = pytest.mark.gpu
DELTA = 1e-5


def run(q, k, block, kv_len, text_start, tau, scale=0.0):
    B, H, N, D = q.shape
    m = torch.full((B, H, N // block, N // block), 9, dtype=torch.uint8, device="cuda")
    ra.rapid_mask_select(to_dev(q), to_dev(k), m, block, kv_len, text_start, tau, scale)
    torch.cuda.synchronize()
    return m.cpu().numpy()


def check(q, k, block, kv_len, text_start, tau, scale=0.0):
    got = run(q, k, block, kv_len, text_start, tau, scale)
    assert set(np.unique(got)) <= {0, 1}
    lo = mo.select_mask(q, k, block, kv_len, text_start, tau - DELTA, scale)
    hi = mo.select_mask(q, k, block, kv_len, text_start, tau + DELTA, scale)
    mid = mo.select_mask(q, k, block, kv_len, text_start, tau, scale)
    assert (lo <= got).all() and (got <= hi).all(), ((lo > got).sum(), (got > hi).sum())
    assert (got == mid).mean() >= 0.999
    return got


CASES = [
    # B, H, N, D, block, kv_len, text_start, gain
    (1, 2, 256, 64, 64, 256, 256, 3.0),
    (2, 3, 640, 64, 64, 600, 512, 3.0),
    (1, 2, 1152, 128, 128, 1100, 1024, 2.0),
    (2, 2, 4608, 128, 128, 4608, 4096, 2.5),
    (1, 3, 4480, 64, 128, 4429, 4096, 3.0),
    (1, 1, 8192, 64, 64, 8192, 9000, 3.0),      # 128 blocks per row: two per lane
    (1, 2, 16896, 128, 128, 16896, 16384, 2.5), # the 2048^2 FLUX-like shape: 132 blocks per side
]


@pytest.mark.parametrize("B,H,N,D,block,kv_len,text_start,gain", CASES)
@pytest.mark.parametrize("tau", [0.5, 0.9, 0.98])
def test_mask_matches_the_oracle(B, H, N, D, block, kv_len, text_start, gain, tau):
    q, k, _ = wl.make_qkv(B, H, N, D, kv_len, seed=N + D, gain=gain, pad_fill="nan")
    got = check(q, k, block, kv_len, text_start, tau)
    live = -(-kv_len // block)
    assert (got[:, :, live:] == 0).all() and (got[:, :, :, live:] == 0).all()
    if tau <= 0.5 and live >= 8:
        assert got[:, :, :live, :live].mean() < 0.95           # it does prune on these inputs


def test_more_than_256_blocks_per_row_take_the_bisection_kernel():
    B, H, N, D, block, kv_len = 1, 1, 64 * 300, 64, 64, 64 * 300 - 17
    q, k, _ = wl.make_qkv(B, H, N, D, kv_len, seed=19, gain=3.0)
    got = check(q, k, block, kv_len, 64 * 290, 0.7)
    assert got[0, 0, :290, :290].mean() < 0.9


def test_levels_are_nested_and_tau_one_is_dense():
    B, H, N, D, block = 1, 2, 2048, 128, 128
    q, k, _ = wl.make_qkv(B, H, N, D, N, seed=3, gain=3.0)
    masks = [run(q, k, block, N, 1792, ra.rapid_mask_level_tau(a)) for a in (3, 2, 1, 0)]
    for a, b in zip(masks, masks[1:]):
        assert (a <= b).all()
    assert (masks[-1] == 1).all()
    assert (run(q, k, block, N, N, 7.0) == 1).all()           # any tau >= 1


def test_custom_scale_and_block_structured_inputs():
    rng = np.random.default_rng(4)
    B, H, nb, block, D = 1, 2, 16, 128, 128
    N = nb * block
    centers_k = rng.normal(size=(H, nb, D)) * 1.5
    centers_q = centers_k[:, rng.permutation(nb)] + rng.normal(size=(H, nb, D)) * 0.3
    q = np.repeat(centers_q, block, axis=1)[None] + rng.normal(size=(B, H, N, D)) * 0.2
    k = np.repeat(centers_k, block, axis=1)[None] + rng.normal(size=(B, H, N, D)) * 0.2
    qb, kb = wl.f32_to_bf16_bits(q.astype(np.float32)), wl.f32_to_bf16_bits(k.astype(np.float32))
    got = check(qb, kb, block, N, N + 1, 0.9)
    assert got.mean() < 0.5
    check(qb, kb, block, N, N + 1, 0.9, scale=0.03)


def test_selected_mask_feeds_the_sparse_attention():
    """The two calls chain on one stream without a host round trip, and the sparse attention
    under the selected mask equals the oracle's attention under the same mask."""
    import oracle
    from gpu_common import assert_close, from_dev
    B, H, N, D, block, kv_len = 1, 2, 1024, 64, 128, 1000
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=12)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    m = torch.empty((B, H, N // block, N // block), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(dq)
    ra.rapid_mask_select(dq, dk, m, block, kv_len, 896, 0.8)
    ra.rapid_attn_block_sparse(dq, dk, dv, o, m, block, kv_len)
    torch.cuda.synchronize()
    assert_close(from_dev(o), oracle.attention(q, k, v, kv_len, m.cpu().numpy(), block), "select + sparse")
