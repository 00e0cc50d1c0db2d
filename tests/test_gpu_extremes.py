"""Shapes at the edges of what the entry points accept: many (sample, head) pairs of few tokens, a long
ragged dense call.  (The large end -- more mask blocks than the planners sort, a million tokens,
more items than the planner caches -- is in test_gpu_limits.py.)"""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import assert_close, from_dev, to_dev

pytestmark = pytest.mark.gpu


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
