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
    B, H, nb, block, D = 1, 2, 16, 128, 128
    N = nb * block
    qb, kb, _ = wl.make_qkv_block_structured(B, H, N, D, block, seed=4)
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


# ---------------------------------------------------------------- the model-shaped form
def oracle_joint_mask(q, k, block, kv_lens, text_start, tau):
    """Per sample (each has its own valid length), on the contiguous data padded to whole blocks
    with NaN rows (beyond every valid length, so the oracle must ignore them)."""
    B, H, N, D = q.shape
    nb = -(-N // block)
    pad = lambda x: np.concatenate([x, np.full((B, H, nb * block - N, D), wl.BF16_NAN, np.uint16)], axis=2)
    qp, kp = pad(q), pad(k)
    out = np.zeros((B, H, nb, nb), np.uint8)
    for b in range(B):
        if kv_lens[b] > 0:
            out[b] = mo.select_mask(qp[b:b + 1], kp[b:b + 1], block, int(kv_lens[b]), text_start, tau)[0]
    return out


JOINT = [
    # B, H, n_img, n_txt, D, block, lens (None = all tokens), fused
    (2, 3, 512, 77, 64, 128, None, False),
    (3, 2, 640, 100, 128, 128, (740, 0, 655), True),       # per-sample lengths, one sample empty
    (2, 2, 256, 64, 128, 64, (300, 320), True),
    (1, 2, 333, 0, 64, 64, (301,), False),                 # one ragged token-major segment
    (1, 2, 4096, 333, 64, 128, None, True),                # the SD3-like joint shape, ragged last block
]


@pytest.mark.parametrize("B,H,n_img,n_txt,D,block,lens,fused", JOINT)
@pytest.mark.parametrize("tau", [0.6, 0.95])
def test_joint_selection_matches_the_oracle(B, H, n_img, n_txt, D, block, lens, fused, tau):
    from test_gpu_joint import as_model_tensors
    N = n_img + n_txt
    nb = -(-N // block)
    lens = np.array([N] * B if lens is None else lens, np.int32)
    q, k, v = wl.make_qkv_block_structured(B, H, N, D, block, seed=N + D, n_text_blocks=-(-n_txt // block))
    segs, _ = as_model_tensors(q, k, v, n_img, fused)
    m = torch.full((B, H, nb, nb), 9, dtype=torch.uint8, device="cuda")
    ra.rapid_mask_select_joint(segs, m, block, kv_lens=torch.from_numpy(lens).cuda(), text_start=n_img, tau=tau)
    torch.cuda.synchronize()
    got = m.cpu().numpy()
    assert set(np.unique(got)) <= {0, 1}
    lo, hi, mid = (oracle_joint_mask(q, k, block, lens, n_img, t) for t in (tau - DELTA, tau + DELTA, tau))
    assert (lo <= got).all() and (got <= hi).all(), ((lo > got).sum(), (got > hi).sum())
    assert (got == mid).mean() >= 0.999
    live_img = min(n_img, int(lens.max())) // block
    if live_img >= 4:
        assert got[lens.argmax(), :, :live_img, :live_img].mean() < 0.9      # it prunes on these inputs
    # the same bits as the contiguous entry point on a contiguous copy, where that one applies
    if N % block == 0 and len(set(lens.tolist())) == 1 and lens[0] > 0:
        m2 = torch.empty_like(m)
        ra.rapid_mask_select(to_dev(q), to_dev(k), m2, block, int(lens[0]), n_img, tau)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(got, m2.cpu().numpy())


def test_joint_select_then_joint_attend_on_the_same_tensors():
    """The composition the model needs: mask from the image and text tensors as they are, then
    attention on the same tensors, per-sample lengths in both; against the oracle's attention
    under the selected mask."""
    import oracle
    from gpu_common import assert_close
    from test_gpu_joint import as_model_tensors, gather, oracle_joint
    B, H, n_img, n_txt, D, block = 2, 3, 1024, 154, 128, 128
    N = n_img + n_txt
    nb = -(-N // block)
    lens = np.array([N, N - 60], np.int32)
    q, k, v = wl.make_qkv_block_structured(B, H, N, D, block, seed=77, n_text_blocks=2)
    segs, guards = as_model_tensors(q, k, v, n_img, True)
    dl = torch.from_numpy(lens).cuda()
    m = torch.empty((B, H, nb, nb), dtype=torch.uint8, device="cuda")
    ra.rapid_mask_select_joint(segs, m, block, kv_lens=dl, text_start=n_img, tau=0.9)
    ra.rapid_attn_joint(segs, m, block, kv_lens=dl)
    torch.cuda.synchronize()
    mask = m.cpu().numpy()
    assert 0.2 < mask.mean() < 0.9
    got = gather(segs)
    for b in range(B):
        ref = oracle_joint(q[b:b + 1], k[b:b + 1], v[b:b + 1], int(lens[b]), mask[b:b + 1], block)
        assert_close(got[b:b + 1], ref, f"sample {b}")


SELECT_ATTEND = [
    # B, H, n_img, n_txt, D, block, lens, fused
    (2, 3, 1024, 154, 128, 128, (1178, 1118), True),      # ragged last block, per-sample lengths
    (1, 24, 4096, 512, 128, 128, None, True),             # the FLUX-like 1024^2 joint shape: one-launch planner size
    (2, 2, 512, 64, 64, 64, (576, 0), False),             # 64-token tiles, an empty sample
    (1, 3, 8192, 256, 64, 128, None, False),              # 66 blocks per side: the general planner either way
]


@pytest.mark.parametrize("B,H,n_img,n_txt,D,block,lens,fused", SELECT_ATTEND)
def test_select_and_attend_in_one_call(B, H, n_img, n_txt, D, block, lens, fused):
    """rapid_attn_joint_select against its two-call form: the mask it reports equals the one
    rapid_mask_select_joint writes (same kernel, same arithmetic: bit for bit), the kept lists it
    left in the workspace are that mask compacted (the oracle's kept_tiles of it), and the output
    matches the oracle's attention under that mask."""
    import oracle
    from gpu_common import assert_close
    from test_gpu_joint import as_model_tensors, gather, oracle_joint
    from test_gpu_parity import read_plan, check_plan
    tau = 0.9
    N = n_img + n_txt
    nb = -(-N // block)
    lens_h = np.array([N] * B if lens is None else lens, np.int32)
    dl = torch.from_numpy(lens_h).cuda()
    q, k, v = wl.make_qkv_block_structured(B, H, N, D, block, seed=N + 3 * D, n_text_blocks=-(-n_txt // block))
    segs, guards = as_model_tensors(q, k, v, n_img, fused)
    m_two = torch.full((B, H, nb, nb), 9, dtype=torch.uint8, device="cuda")
    ra.rapid_mask_select_joint(segs, m_two, block, kv_lens=dl, text_start=n_img, tau=tau)
    ra.rapid_attn_joint(segs, m_two, block, kv_lens=dl)
    torch.cuda.synchronize()
    want = gather(segs)

    segs1, guards1 = as_model_tensors(q, k, v, n_img, fused)
    m_one = torch.full((B, H, nb, nb), 9, dtype=torch.uint8, device="cuda")
    ws = torch.full((ra.rapid_attn_joint_select_workspace_bytes(B, H, N, D, block),), 0xAB, dtype=torch.uint8, device="cuda")
    ra.rapid_attn_joint_select(segs1, block, kv_lens=dl, text_start=n_img, tau=tau, mask_out=m_one, workspace=ws)
    torch.cuda.synchronize()
    mask = m_one.cpu().numpy()
    np.testing.assert_array_equal(mask, m_two.cpu().numpy())
    assert 0.15 < mask[lens_h.argmax()].mean() < 0.9
    got = gather(segs1)
    # lists and plan left in the workspace: the mask compacted, a valid plan
    counts, order, index, g = read_plan(ws.cpu().numpy(), B, H, nb, D, block)
    for b in range(B):
        wc, wi = oracle.kept_tiles(mask[b:b + 1], block, max(int(lens_h[b]), 1))
        rows = slice(b * H * nb, (b + 1) * H * nb)
        np.testing.assert_array_equal(counts[rows], wc.reshape(-1) if lens_h[b] > 0 else 0)
        if lens_h[b] > 0:
            wi = wi.reshape(-1, nb)
            for r in range(H * nb):
                np.testing.assert_array_equal(index[rows][r, :wc.reshape(-1)[r]], wi[r, :wc.reshape(-1)[r]])
    check_plan(counts, order, g, B, H, nb, block, D)
    # output: the oracle under the selected mask; and the two-call form to rounding (its planner may
    # cut rows differently, so not bit for bit)
    for b in range(B):
        if lens_h[b] == 0:
            assert (got[b] == 0).all()
            continue
        ref = oracle_joint(q[b:b + 1], k[b:b + 1], v[b:b + 1], int(lens_h[b]), mask[b:b + 1], block)
        assert_close(got[b:b + 1], ref, f"one call, sample {b}")
        assert_close(want[b:b + 1], ref, f"two calls, sample {b}")
    for gbuf in guards1:
        assert (gbuf[:, :, 0] == 7.0).all() and (gbuf[:, :, -1] == 7.0).all()
    # without mask_out the same output
    segs2, _ = as_model_tensors(q, k, v, n_img, fused)
    ra.rapid_attn_joint_select(segs2, block, kv_lens=dl, text_start=n_img, tau=tau, workspace=ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(gather(segs2), got)
