"""GPU parity at the large end of what the library accepts: sequences long enough that a row of
the mask has more blocks than the planners sort (they then hand the items out in natural order,
whole), that the selection kernel holds its maximum of blocks per side, and that byte offsets
inside one (sample, head) pass 2^26.  Same oracle and tolerances as the other parity tests; the
oracle computes sampled rows (a whole tensor at a million tokens would take it hours)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import assert_close, from_dev, to_dev, widen
from oracle import mask_oracle as mo
from test_gpu_parity import check_plan, read_plan

pytestmark = pytest.mark.gpu


def long_mask(nb, live, seed):
    """[1,1,nb,nb]: diagonal and both neighbours, five random blocks per row, the last live block
    for every row; row 5 keeps nothing, row 100 keeps 600 blocks; blocks beyond `live` are set in
    places and must be ignored."""
    rng = np.random.Generator(np.random.PCG64(seed))
    m = np.zeros((1, 1, nb, nb), np.uint8)
    r = np.arange(nb)
    for d in (-1, 0, 1):
        c = np.clip(r + d, 0, nb - 1)
        m[0, 0, r, c] = 1
    m[0, 0, np.repeat(r, 5), rng.integers(0, nb, 5 * nb)] = 1
    m[0, 0, :, live - 1] = 1
    m[0, 0, 5, :] = 0
    m[0, 0, 100, rng.choice(nb, 600, replace=False)] = 1
    m[0, 0, :, live:] = rng.integers(0, 2, (nb, nb - live), dtype=np.uint8)
    return m


def sampled_rows(N, kv_len, block, n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    fixed = [0, 1, block - 1, block, 5 * block, 5 * block + 77, 100 * block + 3, kv_len - 1, kv_len, N - 1,
             (kv_len // block) * block, N // 2 + 1]
    rows = sorted(set(fixed) | set(int(x) for x in rng.integers(0, N, n)))
    return np.array([(0, 0, r) for r in rows], np.int32)


@pytest.mark.parametrize("block", [64, 128])
def test_more_mask_blocks_than_the_planner_sorts(block):
    """nb = 8192 per side (half a million tokens at 64-token tiles, a million at 128): lists bit
    for bit, a valid plan without pieces, sampled rows against the oracle; then the dense entry on
    the same tensors."""
    D, nb = 64, 8192
    N = nb * block
    kv_len = N - 3 * block - 37                       # ragged last live block, three dead blocks
    live = -(-kv_len // block)
    print(f"long sequence: N={N} block={block} nb={nb} kv_len={kv_len}", flush=True)
    q, k, v = wl.make_qkv(1, 1, N, D, kv_len, seed=8192 + block, pad_fill="nan")
    mask = long_mask(nb, live, seed=block)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    ws = torch.full((ra.rapid_attn_workspace_bytes(1, 1, N, D, block),), 0xAB, dtype=torch.uint8, device="cuda")
    o = torch.full_like(dq, float("nan"))
    ra.rapid_attn_block_sparse(dq, dk, dv, o, torch.from_numpy(mask).cuda(), block, kv_len, 0.0, ws)
    torch.cuda.synchronize()
    got = from_dev(o)
    counts, order, index, g = read_plan(ws.cpu().numpy(), 1, 1, nb, D, block)
    want_counts, want_index = oracle.kept_tiles(mask, block, kv_len)
    np.testing.assert_array_equal(counts, want_counts.reshape(-1))
    want_index = want_index.reshape(-1, nb)
    for r in range(nb):
        np.testing.assert_array_equal(index[r, :counts[r]], want_index[r, :counts[r]])
    assert counts[5] == 0 and counts[100] >= 590
    assert check_plan(counts, order, g, 1, 1, nb, block, D) == {}          # nothing is cut at this size

    rows = sampled_rows(N, kv_len, block, 300, seed=3)
    ref = oracle.attention_rows(q, k, v, rows, kv_len, mask, block)
    e = assert_close(got[rows[:, 0], rows[:, 1], rows[:, 2]], ref, f"long sparse block={block}")
    print(f"  sparse entry, {len(rows)} rows: max-abs {e['max_abs']:.3e} mean-abs {e['mean_abs']:.3e}", flush=True)
    full = widen(got)
    assert np.isfinite(full).all()
    assert (full[0, 0, kv_len:] == 0).all() and (full[0, 0, 5 * block:6 * block] == 0).all()

    o.fill_(float("nan"))
    ra.rapid_attn_dense(dq, dk, dv, o, kv_len)
    torch.cuda.synchronize()
    got = from_dev(o)
    rows = sampled_rows(N, kv_len, block, 40, seed=4)
    ref = oracle.attention_rows(q, k, v, rows, kv_len)
    e = assert_close(got[rows[:, 0], rows[:, 1], rows[:, 2]], ref, f"long dense N={N}")
    print(f"  dense entry, {len(rows)} rows: max-abs {e['max_abs']:.3e} mean-abs {e['mean_abs']:.3e}", flush=True)
    full = widen(got)
    assert np.isfinite(full).all() and (full[0, 0, kv_len:] == 0).all()


def test_long_dense_with_wide_heads():
    """D = 128, two heads of 131072 tokens: 32 MB per (sample, head), 512 workgroup tiles per head."""
    B, H, N, D, kv_len = 1, 2, 131072, 128, 131072 - 200
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=131, pad_fill="inf")
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full_like(dq, float("nan"))
    ra.rapid_attn_dense(dq, dk, dv, o, kv_len)
    torch.cuda.synchronize()
    got = from_dev(o)
    rng = np.random.Generator(np.random.PCG64(5))
    rows = np.array([(0, h, r) for h in range(H) for r in sorted({0, 255, 256, kv_len - 1, kv_len, N - 1}
                                                                  | set(int(x) for x in rng.integers(0, N, 60)))], np.int32)
    ref = oracle.attention_rows(q, k, v, rows, kv_len)
    e = assert_close(got[rows[:, 0], rows[:, 1], rows[:, 2]], ref, "long dense D=128")
    print(f"long dense D=128, {len(rows)} rows: max-abs {e['max_abs']:.3e} mean-abs {e['mean_abs']:.3e}", flush=True)
    full = widen(got)
    assert np.isfinite(full).all() and (full[:, :, kv_len:] == 0).all()


def test_selection_at_its_maximum_of_blocks_per_side():
    """2048 blocks per side (the limit of rapid_mask_select): the mask inside the oracle's band."""
    B, H, D, block, nb = 1, 1, 64, 64, 2048
    N = nb * block
    kv_len, text_start, tau = N - 100, N - 4 * block, 0.8
    q, k, _ = wl.make_qkv(B, H, N, D, kv_len, seed=2048, gain=3.0, pad_fill="nan")
    m = torch.full((B, H, nb, nb), 9, dtype=torch.uint8, device="cuda")
    ra.rapid_mask_select(to_dev(q), to_dev(k), m, block, kv_len, text_start, tau, 0.0)
    torch.cuda.synchronize()
    got = m.cpu().numpy()
    assert set(np.unique(got)) <= {0, 1}
    lo = mo.select_mask(q, k, block, kv_len, text_start, tau - 1e-5, 0.0)
    hi = mo.select_mask(q, k, block, kv_len, text_start, tau + 1e-5, 0.0)
    mid = mo.select_mask(q, k, block, kv_len, text_start, tau, 0.0)
    assert (lo <= got).all() and (got <= hi).all(), ((lo > got).sum(), (got > hi).sum())
    assert (got == mid).mean() >= 0.999
    assert got[0, 0, :nb - 4, :nb - 4].mean() < 0.95


def test_more_items_per_xcd_than_the_planner_caches():
    """4096 (sample, head) pairs of 9 query-blocks: 4608 items per XCD, more than the 4096 whose
    lengths the planner keeps in LDS; the general planner (the one-launch planner stops at 1024
    items per XCD).  Lists bit for bit, plan valid, sampled rows of a thousand items and of every
    cut item against the oracle."""
    B, H, N, D, block, kv_len = 2, 2048, 1152, 64, 128, 1100
    nb = N // block
    print(f"many items: B={B} H={H} N={N} items per XCD={B * H * nb // 8}", flush=True)
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=4096, pad_fill="nan")
    rng = np.random.Generator(np.random.PCG64(77))
    mask = (rng.random((B, H, nb, nb)) < 0.4).astype(np.uint8)
    mask[:, :, np.arange(nb), np.arange(nb)] = 1
    mask[:, ::97, 3, :] = 1                             # some full rows
    mask[1, 5::211, 2, :] = 0                           # some empty ones
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    ws = torch.full((ra.rapid_attn_workspace_bytes(B, H, N, D, block),), 0xAB, dtype=torch.uint8, device="cuda")
    o = torch.full_like(dq, float("nan"))
    ra.rapid_attn_block_sparse(dq, dk, dv, o, torch.from_numpy(mask).cuda(), block, kv_len, 0.0, ws)
    torch.cuda.synchronize()
    got = from_dev(o)
    counts, order, index, g = read_plan(ws.cpu().numpy(), B, H, nb, D, block)
    want_counts, want_index = oracle.kept_tiles(mask, block, kv_len)
    np.testing.assert_array_equal(counts, want_counts.reshape(-1))
    want_index = want_index.reshape(-1, nb)
    live = np.arange(nb)[None, :] < counts[:, None]
    np.testing.assert_array_equal(np.where(live, index, -1), np.where(live, want_index, -1))
    cut = check_plan(counts, order, g, B, H, nb, block, D)
    print(f"  {len(cut)} of {B * H * nb} rows ran as pieces", flush=True)
    items = sorted(set(int(x) for x in rng.integers(0, B * H * nb, 1000)) | set(cut))
    rows = np.array([(it // nb // H, it // nb % H, (it % nb) * block + int(r)) for it in items
                     for r in rng.integers(0, block, 2)], np.int32)
    ref = oracle.attention_rows(q, k, v, rows, kv_len, mask, block)
    e = assert_close(got[rows[:, 0], rows[:, 1], rows[:, 2]], ref, "many items")
    print(f"  {len(rows)} rows of {len(items)} items: max-abs {e['max_abs']:.3e} mean-abs {e['mean_abs']:.3e}", flush=True)
    full = widen(got)
    assert np.isfinite(full).all() and (full[:, :, kv_len:] == 0).all()
    assert (full[1, 5::211, 2 * block:3 * block] == 0).all()
