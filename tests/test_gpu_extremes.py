"""Shapes at the edges of what the entry points accept: more mask blocks per side than the launch
plan sorts (its natural-order fallback), many (sample, head) pairs, a long ragged dense call."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import assert_close, from_dev, to_dev

pytestmark = pytest.mark.gpu


def sparse_rows_mask(nb, per_row, seed):
    """[1,1,nb,nb] with the diagonal, the first column and `per_row` random blocks per row."""
    rng = np.random.default_rng(seed)
    m = np.zeros((1, 1, nb, nb), np.uint8)
    idx = np.arange(nb)
    m[0, 0, idx, idx] = 1
    m[0, 0, :, 0] = 1
    for _ in range(per_row):
        m[0, 0, idx, rng.integers(nb, size=nb)] = 1
    return m


@pytest.mark.parametrize("block", [128, 64])
def test_more_blocks_per_side_than_the_plan_sorts(block):
    nb, D = 8192, 64                                       # the plan sorts up to 8176 blocks per side
    N = nb * block
    kv_len = N - 100
    q, k, v = wl.make_qkv(1, 1, N, D, kv_len, seed=400 + block)
    mask = sparse_rows_mask(nb, 2, seed=block)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full_like(dq, float("nan"))
    ws = torch.empty(ra.rapid_attn_workspace_bytes(1, 1, N, D, block), dtype=torch.uint8, device="cuda")
    ra.rapid_attn_block_sparse(dq, dk, dv, o, torch.from_numpy(mask).cuda(), block, kv_len, 0.0, ws)
    torch.cuda.synchronize()
    got = from_dev(o)
    rows = wl.sample_rows(1, 1, N, kv_len, block, 96, seed=3)
    ref = oracle.attention_rows(q, k, v, rows, kv_len, mask, block)
    assert_close(got[rows[:, 0], rows[:, 1], rows[:, 2]], ref, f"nb={nb} block={block}")
    assert np.isfinite(wl.bf16_bits_to_f32(got)).all()
    # the fallback plan: items in natural order, whole, on the XCD of their (sample, head)
    head = ws[:256].cpu().numpy()                          # counts of the first rows: diag + column 0 + <= 2
    counts = head.view(np.int32)[:8]
    assert ((counts >= 1) & (counts <= 4)).all()


def test_many_sample_head_pairs():
    B, H, N, D, block, kv_len = 64, 16, 256, 64, 128, 250
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=410)
    mask = wl.mask_bernoulli_diag(B, H, N // block, 0.5, seed=8)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full_like(dq, float("nan"))
    ra.rapid_attn_dense(dq, dk, dv, o, kv_len)
    torch.cuda.synchronize()
    assert_close(from_dev(o), oracle.attention(q, k, v, kv_len), "dense, 1024 (sample, head) pairs")
    o.fill_(float("nan"))
    ra.rapid_attn_block_sparse(dq, dk, dv, o, torch.from_numpy(mask).cuda(), block, kv_len)
    torch.cuda.synchronize()
    assert_close(from_dev(o), oracle.attention(q, k, v, kv_len, mask, block), "sparse, 1024 (sample, head) pairs")


def test_long_ragged_dense_call():
    B, H, N, D, kv_len = 1, 1, 40000, 128, 39990           # N a multiple of nothing the kernels tile by
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=420)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full_like(dq, float("nan"))
    ra.rapid_attn_dense(dq, dk, dv, o, kv_len)
    torch.cuda.synchronize()
    got = from_dev(o)
    rows = wl.sample_rows(B, H, N, kv_len, 128, 64, seed=5)
    assert_close(got[rows[:, 0], rows[:, 1], rows[:, 2]], oracle.attention_rows(q, k, v, rows, kv_len), "N=40000")
    assert (got[0, 0, kv_len:] == 0).all()
