"""GPU parity of the model-shaped entry point (separate image and text tensors, strided
layouts, ragged joint length, per-sample lengths) against the same fp64 oracle, run on a
contiguous [B,H,N,D] copy of the same data."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import assert_close, from_dev, to_dev

pytestmark = pytest.mark.gpu


def oracle_joint(q, k, v, kv_len, mask, block):
    """The oracle wants N % block == 0 with a mask: pad with rows beyond kv_len (it ignores them)."""
    B, H, N, D = q.shape
    if mask is None or N % block == 0:
        return oracle.attention(q, k, v, kv_len, mask, block if mask is not None else 64)
    Np = -(-N // block) * block
    pad = lambda x: np.concatenate([x, np.full((B, H, Np - N, D), wl.BF16_NAN, np.uint16)], axis=2)
    return oracle.attention(pad(q), pad(k), pad(v), kv_len, mask, block)[:, :, :N]


def as_model_tensors(q, k, v, n0, fused):
    """Store the joint [B,H,N,D] data the way an MM-DiT block holds it: an image tensor with
    tokens [0,n0) and a text tensor with the rest, each [B,n,H,D] (or fused [B,n,3,H,D]).
    Returns per segment (q, k, v, o) views indexed [B,H,n,D] plus the guard buffers of o."""
    B, H, N, D = q.shape
    segs, guards = [], []
    for a, b in ((0, n0), (n0, N)) if n0 < N else ((0, N),):
        n = b - a
        if fused:
            buf = torch.empty(B, n, 3, H, D, dtype=torch.bfloat16, device="cuda")
            for j, x in enumerate((q, k, v)):
                buf[:, :, j] = to_dev(x[:, :, a:b]).permute(0, 2, 1, 3)
            views = [buf[:, :, j].permute(0, 2, 1, 3) for j in range(3)]
        else:
            views = [to_dev(x[:, :, a:b]).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for x in (q, k, v)]
        # o lives inside a larger buffer (two guard channels-blocks per token) that must stay untouched
        obuf = torch.full((B, n, H + 2, D), 7.0, dtype=torch.bfloat16, device="cuda")
        o = obuf[:, :, 1:H + 1].permute(0, 2, 1, 3)
        o.fill_(float("nan"))
        segs.append((views[0], views[1], views[2], o))
        guards.append(obuf)
    return segs, guards


def gather(segs):
    return np.concatenate([from_dev(o.contiguous()) for (_, _, _, o) in segs], axis=2)


CASES = [
    # B, H, n_img, n_txt, D, block, p_keep, fused
    (2, 3, 256, 77, 64, 128, 0.5, False),
    (1, 2, 384, 100, 128, 128, 0.4, True),
    (2, 2, 256, 64, 128, 64, 0.5, True),
    (1, 3, 512, 33, 64, 64, 0.4, False),
    (2, 2, 333, 0, 128, 128, 0.5, True),       # one segment, ragged, token-major layout
    (1, 2, 384, 1, 64, 128, 0.5, False),       # a one-token text segment: torch leaves its token stride at D
]


@pytest.mark.parametrize("B,H,n_img,n_txt,D,block,p,fused", CASES)
def test_joint_dense_and_sparse_match_the_oracle(B, H, n_img, n_txt, D, block, p, fused):
    N = n_img + n_txt
    q, k, v = wl.make_qkv(B, H, N, D, N, seed=300 + N + D)
    nb = -(-N // block)
    mask = wl.mask_bernoulli_diag(B, H, nb, p, seed=N)
    for m in (None, mask):
        segs, guards = as_model_tensors(q, k, v, n_img, fused)
        ra.rapid_attn_joint(segs, None if m is None else torch.from_numpy(m).cuda(), block)
        torch.cuda.synchronize()
        assert_close(gather(segs), oracle_joint(q, k, v, N, m, block), f"joint {'dense' if m is None else 'sparse'}")
        for g in guards:                                   # nothing outside the o views was written
            assert (g[:, :, 0] == 7.0).all() and (g[:, :, -1] == 7.0).all()


def test_per_sample_lengths():
    B, H, n_img, n_txt, D, block = 4, 2, 256, 128, 64, 128
    N = n_img + n_txt
    lens = np.array([N, n_img + 5, 0, 300], np.int32)      # full, short prompt, empty sample, ragged
    q, k, v = wl.make_qkv(B, H, N, D, N, seed=77)
    mask = wl.mask_bernoulli_diag(B, H, N // block, 0.6, seed=4)
    for m in (None, mask):
        segs, _ = as_model_tensors(q, k, v, n_img, True)
        ra.rapid_attn_joint(segs, None if m is None else torch.from_numpy(m).cuda(), block,
                            kv_lens=torch.from_numpy(lens).cuda())
        torch.cuda.synchronize()
        got = gather(segs)
        for b in range(B):
            if lens[b] == 0:
                assert (got[b] == 0).all()
                continue
            ref = oracle.attention(q[b:b + 1], k[b:b + 1], v[b:b + 1], int(lens[b]),
                                   None if m is None else m[b:b + 1], block)
            assert_close(got[b:b + 1], ref, f"sample {b} kv_len {lens[b]}")


def test_joint_equals_the_contiguous_entry_points_bit_for_bit():
    B, H, N, D, block = 1, 4, 512, 128, 128
    q, k, v = wl.make_qkv(B, H, N, D, 500, seed=5)
    mask = wl.mask_bernoulli_diag(B, H, N // block, 0.5, seed=6)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    for m in (None, torch.from_numpy(mask).cuda()):
        o1, o2 = torch.empty_like(dq), torch.empty_like(dq)
        if m is None:
            ra.rapid_attn_dense(dq, dk, dv, o1, 500)
        else:
            ra.rapid_attn_block_sparse(dq, dk, dv, o1, m, block, 500)
        ra.rapid_attn_joint([(dq, dk, dv, o2)], m, block, kv_len=500)
        torch.cuda.synchronize()
        assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))


def test_strides_of_size_one_dimensions_are_not_looked_at():
    """B = 1, H = 1 and a one-token second segment, with strides in those dimensions that would be
    refused (odd, unequal between the segments) if they addressed anything."""
    B, H, n_img, n_txt, D, block = 1, 1, 256, 1, 128, 128
    N = n_img + n_txt
    q, k, v = wl.make_qkv(B, H, N, D, N, seed=91)
    mask = wl.mask_bernoulli_diag(B, H, -(-N // block), 0.5, seed=9)
    segs, _ = as_model_tensors(q, k, v, n_img, False)

    def odd(t, sb, sh, sn):
        return torch.as_strided(t, t.shape, (sb, sh, sn, 1), t.storage_offset())

    (q0, k0, v0, o0), (q1, k1, v1, o1) = segs
    segs = [(odd(q0, 3, 5, q0.stride(2)), odd(k0, 3, 5, k0.stride(2)), odd(v0, 3, 5, v0.stride(2)), odd(o0, 7, 9, o0.stride(2))),
            (odd(q1, 11, 13, 17), odd(k1, 11, 13, 17), odd(v1, 11, 13, 17), odd(o1, 19, 21, 23))]
    for m in (None, mask):
        for (_, _, _, o) in segs:
            o.fill_(float("nan"))
        ra.rapid_attn_joint(segs, None if m is None else torch.from_numpy(m).cuda(), block)
        torch.cuda.synchronize()
        assert_close(gather(segs), oracle_joint(q, k, v, N, m, block), "size-one dimensions")
    got = torch.full((B, H, 3, 3), 9, dtype=torch.uint8, device="cuda")
    ra.rapid_mask_select_joint(segs, got, block, tau=0.9)
    torch.cuda.synchronize()
    want = torch.full_like(got, 9)
    ra.rapid_mask_select_joint(as_model_tensors(q, k, v, n_img, False)[0], want, block, tau=0.9)
    torch.cuda.synchronize()
    assert torch.equal(got, want) and set(np.unique(got.cpu().numpy())) <= {0, 1}


def test_per_sample_lengths_outside_the_range_are_clamped():
    """kv_lens below 0 count as 0 (the sample outputs zeros), above N as N: attention (dense and
    sparse), selection and the one-call form give what the clamped lengths give, bit for bit."""
    B, H, n_img, n_txt, D, block = 3, 2, 256, 77, 64, 128
    N = n_img + n_txt
    nb = -(-N // block)
    q, k, v = wl.make_qkv(B, H, N, D, N, seed=55)
    mask = torch.from_numpy(wl.mask_bernoulli_diag(B, H, nb, 0.5, seed=2)).cuda()
    wild = torch.tensor([-7, N + 1000, 200], dtype=torch.int32, device="cuda")
    tame = torch.tensor([0, N, 200], dtype=torch.int32, device="cuda")
    outs = {}
    for name, lens in (("wild", wild), ("tame", tame)):
        res = []
        for m in (None, mask):
            segs, _ = as_model_tensors(q, k, v, n_img, True)
            ra.rapid_attn_joint(segs, m, block, kv_lens=lens)
            torch.cuda.synchronize()
            res.append(gather(segs))
        segs, _ = as_model_tensors(q, k, v, n_img, True)
        sel = torch.full((B, H, nb, nb), 9, dtype=torch.uint8, device="cuda")
        ra.rapid_mask_select_joint(segs, sel, block, kv_lens=lens, text_start=n_img, tau=0.8)
        sel2 = torch.full_like(sel, 9)
        ra.rapid_attn_joint_select(segs, block, kv_lens=lens, text_start=n_img, tau=0.8, mask_out=sel2)
        torch.cuda.synchronize()
        res += [sel.cpu().numpy(), sel2.cpu().numpy(), gather(segs)]
        outs[name] = res
    for a, b in zip(outs["wild"], outs["tame"]):
        np.testing.assert_array_equal(a, b)
    assert (outs["wild"][0][0] == 0).all() and (outs["wild"][3][0] == 0).all()
    assert_close(outs["wild"][0][1:2], oracle_joint(q[1:2], k[1:2], v[1:2], N, None, block), "length above N")
