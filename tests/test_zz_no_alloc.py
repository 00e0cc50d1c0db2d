"""The entry point that allocates nothing (rapid_attn_block_sparse_static: scratch in a fixed
array inside the library) against rapid_attn_block_sparse on a caller's workspace: same kernels,
so whenever the whole workspace fits the array the outputs are bit-identical; with fewer
partial-result slots than the split rule asks for (large batches) fewer rows are cut and the
outputs agree within the tolerances against the oracle.  Calls share the array, so the second
call (smaller, other head size) runs on whatever the first one left there."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import assert_close, from_dev, to_dev

pytestmark = pytest.mark.gpu


def both(B, H, N, D, block, kv_len, p, seed, long_rows=()):
    nb = N // block
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=seed, pad_fill="nan")
    mask = wl.mask_bernoulli_diag(B, H, nb, p, seed=seed + 1)
    for r in long_rows:
        mask[:, :, r, :] = 1
    dq, dk, dv, dm = to_dev(q), to_dev(k), to_dev(v), torch.from_numpy(mask).cuda()
    o_ws = torch.full_like(dq, float("nan"))
    o_st = torch.full_like(dq, float("nan"))
    ws = torch.full((ra.rapid_attn_workspace_bytes(B, H, N, D, block),), 0xAB, dtype=torch.uint8, device="cuda")
    ra.rapid_attn_block_sparse(dq, dk, dv, o_ws, dm, block, kv_len, 0.0, ws)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ra.rapid_attn_block_sparse_static(dq, dk, dv, o_st, dm, block, kv_len)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return (q, k, v, mask), from_dev(o_ws), from_dev(o_st), ws.numel()


def test_two_calls_in_a_row_match_the_workspace_entry_point():
    # first call: long rows are cut into pieces and merged through the partial-result slots
    B, H, N, D, block, kv_len = 1, 16, 4608, 128, 128, 4500
    _, want, got, need = both(B, H, N, D, block, kv_len, 0.1, seed=301, long_rows=(5, 35))
    assert need <= ra.STATIC_SCRATCH_BYTES
    assert np.isfinite(wl.bf16_bits_to_f32(got)).all()
    np.testing.assert_array_equal(got, want)
    # second call: smaller, other head size, 64-token tiles; the array still holds the first call's plan
    B, H, N, D, block, kv_len = 2, 3, 1152, 64, 64, 1100
    (q, k, v, mask), want, got, need = both(B, H, N, D, block, kv_len, 0.4, seed=302)
    np.testing.assert_array_equal(got, want)
    assert_close(got, oracle.attention(q, k, v, kv_len, mask, block), "static, second call")
    # and a 128-token-tile call again, smaller than the first
    B, H, N, D, block, kv_len = 1, 8, 2304, 128, 128, 2304
    _, want, got, need = both(B, H, N, D, block, kv_len, 0.3, seed=303, long_rows=(17,))
    np.testing.assert_array_equal(got, want)


def test_fewer_slots_than_the_rule_asks_for():
    """A batch whose full workspace exceeds the array: the plan gets the slots that fit."""
    B, H, N, D, block, kv_len = 8, 24, 2560, 128, 128, 2500
    (q, k, v, mask), want, got, need = both(B, H, N, D, block, kv_len, 0.15, seed=304, long_rows=(3, 11, 19))
    assert need > ra.STATIC_SCRATCH_BYTES
    rows = wl.sample_rows(B, H, N, kv_len, block, 256, seed=9)
    rows = np.concatenate([rows, np.array([(b, h, r * block + 7) for b in (0, 7) for h in (0, 23) for r in (3, 11, 19)], np.int32)])
    ref = oracle.attention_rows(q, k, v, rows, kv_len, mask, block)
    assert_close(got[rows[:, 0], rows[:, 1], rows[:, 2]], ref, "static, capped slots")
    assert_close(got, wl.bf16_bits_to_f32(want).astype(np.float64), "static vs workspace entry")
