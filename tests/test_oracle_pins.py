"""Pins for the fp64 oracle: each test fixes it to something other than itself.

P1  library brute force (scipy softmax + matmul with an explicit 0/-inf bias)
P2  all-ones mask == dense
P3  V == 1  ->  O == 1  (softmax rows sum to one, seen through the public result)
P4  V = indicator of one key block -> O = probability mass of that block
P5  perturbing / poisoning masked-out and padded K,V leaves O unchanged
P6  exactly one allowed key -> O = that key's V row
P7  identical allowed keys -> O = mean of allowed V rows
P8  adding a common vector to every key shifts all scores of a row equally -> O unchanged
P9  permuting keys together with their values -> O unchanged
P10 samples / heads independent; duplicated sample+mask -> duplicated output
P11 every output channel lies in [min, max] of the allowed V values
P12 all scores equal (Q = 0) -> uniform average; large-gain inputs still agree with brute force
No number printed in the paper pins attention: printed-value parity is unpinned.
"""
import numpy as np
import pytest
from scipy.special import softmax

import oracle
import workloads as wl


def widen(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def brute(q, k, v, kv_len, mask, block, scale=None):
    """softmax(scale*QK^T + bias)V with library routines and an explicit N x N bias."""
    B, H, N, D = q.shape
    Q, K, V = widen(q), widen(k), widen(v)
    K = np.where(np.arange(N)[None, None, :, None] < kv_len, K, 0.0)
    V = np.where(np.arange(N)[None, None, :, None] < kv_len, V, 0.0)
    Q = np.where(np.arange(N)[None, None, :, None] < kv_len, Q, 0.0)
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    allowed = np.ones((B, H, N, N), dtype=bool)
    if mask is not None:
        allowed &= np.kron(mask, np.ones((block, block), dtype=np.uint8)).astype(bool)
    allowed &= (np.arange(N) < kv_len)[None, None, None, :]
    bias = np.where(allowed, 0.0, -np.inf)
    S = scale * np.matmul(Q, K.transpose(0, 1, 3, 2)) + bias
    empty = ~allowed.any(axis=-1)
    S[empty] = 0.0
    P = softmax(S, axis=-1)
    O = np.matmul(P, V)
    O[empty] = 0.0
    O[:, :, kv_len:, :] = 0.0
    return O


CASES = [
    # B, H, N, D, block, kv_len, p_keep
    (1, 2, 256, 64, 64, 256, 0.5),
    (2, 3, 192, 64, 64, 150, 0.4),
    (1, 2, 256, 128, 128, 201, 0.5),
    (2, 2, 128, 128, 64, 65, 0.3),
    (1, 1, 96, 32, 32, 96, 0.6),
]


@pytest.mark.parametrize("B,H,N,D,block,kv_len,p", CASES)
def test_p1_brute_force_masked(B, H, N, D, block, kv_len, p):
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=11, pad_fill="nan")
    rng = np.random.default_rng(5)
    mask = (rng.random((B, H, N // block, N // block)) < p).astype(np.uint8)
    got = oracle.attention(q, k, v, kv_len, mask, block)
    want = brute(q, k, v, kv_len, mask, block)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("B,H,N,D,block,kv_len,p", CASES)
def test_p1_brute_force_dense_and_scale(B, H, N, D, block, kv_len, p):
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=12, pad_fill="inf")
    got = oracle.attention(q, k, v, kv_len)
    np.testing.assert_allclose(got, brute(q, k, v, kv_len, None, block), rtol=0, atol=1e-12)
    got = oracle.attention(q, k, v, kv_len, scale=0.37)
    np.testing.assert_allclose(got, brute(q, k, v, kv_len, None, block, 0.37), rtol=0, atol=1e-12)


def test_p1_rows_entry_matches_full():
    B, H, N, D, block, kv_len = 2, 2, 192, 64, 64, 170
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=13)
    mask = wl.mask_bernoulli_diag(B, H, N // block, 0.5, 3)
    full = oracle.attention(q, k, v, kv_len, mask, block)
    rows = wl.sample_rows(B, H, N, kv_len, block, 40, seed=1)
    part = oracle.attention_rows(q, k, v, rows, kv_len, mask, block)
    want = brute(q, k, v, kv_len, mask, block)
    for i, (b, h, r) in enumerate(rows):
        np.testing.assert_array_equal(part[i], full[b, h, r])
        np.testing.assert_allclose(part[i], want[b, h, r], rtol=0, atol=1e-12)


def test_p2_all_ones_mask_equals_dense():
    q, k, v = wl.make_qkv(1, 2, 256, 64, 230, seed=21)
    ones = np.ones((1, 2, 4, 4), np.uint8)
    np.testing.assert_array_equal(oracle.attention(q, k, v, 230, ones, 64),
                                  oracle.attention(q, k, v, 230))


def test_p3_rows_sum_to_one_via_unit_values():
    B, H, N, D, block, kv_len = 1, 2, 256, 64, 64, 200
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=22)
    v[:] = wl.BF16_ONE
    mask = wl.mask_bernoulli_diag(B, H, 4, 0.5, 9)
    o = oracle.attention(q, k, v, kv_len, mask, block)
    np.testing.assert_allclose(o[:, :, :kv_len], 1.0, rtol=0, atol=1e-13)
    assert (o[:, :, kv_len:] == 0).all()


def test_p4_block_indicator_gives_block_mass():
    B, H, N, D, block = 1, 2, 256, 64, 64
    q, k, v = wl.make_qkv(B, H, N, D, seed=23)
    mask = np.ones((B, H, 4, 4), np.uint8)
    mask[:, :, :, 2] = 0
    mask[:, :, 2, 2] = 1
    total = np.zeros((B, H, N))
    for j in range(4):
        vj = np.zeros_like(v)
        vj[:, :, j * block:(j + 1) * block, :] = wl.BF16_ONE
        o = oracle.attention(q, k, vj, N, mask, block)
        assert np.ptp(o, axis=-1).max() < 1e-15          # same mass in every channel
        mass = o[..., 0]
        assert (mass >= 0).all()
        if j == 2:                                        # masked out for q-blocks 0,1,3
            assert (mass[:, :, :128] == 0).all() and (mass[:, :, 192:] == 0).all()
            assert (mass[:, :, 128:192] > 0).all()
        total += mass
    np.testing.assert_allclose(total, 1.0, rtol=0, atol=1e-13)
    # cross-check the mass against the library softmax
    S = np.matmul(widen(q), widen(k).transpose(0, 1, 3, 2)) / 8.0
    P = softmax(S[:, :, :64, :][..., np.r_[0:128, 192:256]], axis=-1)
    v0 = np.zeros_like(v)
    v0[:, :, :64, :] = wl.BF16_ONE
    o0 = oracle.attention(q, k, v0, N, mask, block)
    np.testing.assert_allclose(o0[:, :, :64, 0], P[..., :64].sum(-1), rtol=0, atol=1e-13)


def test_p5_masked_and_padded_kv_do_not_matter():
    B, H, N, D, block, kv_len = 1, 2, 256, 64, 64, 180
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=24)
    mask = np.ones((B, H, 4, 4), np.uint8)
    mask[:, :, :, 1] = 0                   # key block 1 masked for every query block
    base = oracle.attention(q, k, v, kv_len, mask, block)
    for poison in (wl.BF16_NAN, wl.BF16_INF, 0x4700):
        k2, v2 = k.copy(), v.copy()
        k2[:, :, 64:128] = poison
        v2[:, :, 64:128] = poison
        k2[:, :, kv_len:] = poison
        v2[:, :, kv_len:] = poison
        np.testing.assert_array_equal(oracle.attention(q, k2, v2, kv_len, mask, block), base)
    # and an unmasked perturbation DOES change it (the test can fail)
    k3 = k.copy()
    k3[:, :, 0:64] = 0x4000
    assert np.abs(oracle.attention(q, k3, v, kv_len, mask, block) - base).max() > 1e-3


def test_p6_single_allowed_key_returns_its_value():
    B, H, N, D, block = 1, 1, 128, 64, 64
    q, k, v = wl.make_qkv(B, H, N, D, seed=25)
    o = oracle.attention(q, k, v, kv_len=1)               # only key 0 valid
    np.testing.assert_array_equal(o[0, 0, 0], widen(v)[0, 0, 0])
    assert (o[0, 0, 1:] == 0).all()
    # one key per row via a one-token-wide mask grid (block = 1)
    mask = np.zeros((1, 1, 16, 16), np.uint8)
    perm = np.random.default_rng(0).permutation(16)
    mask[0, 0, np.arange(16), perm] = 1
    q2, k2, v2 = wl.make_qkv(1, 1, 16, 32, seed=26)
    o2 = oracle.attention(q2, k2, v2, 16, mask, 1)
    np.testing.assert_array_equal(o2[0, 0], widen(v2)[0, 0, perm])


def test_p7_identical_keys_give_mean_of_values():
    B, H, N, D, block, kv_len = 1, 2, 192, 64, 64, 160
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=27)
    k[:, :, :kv_len] = k[:, :, :1]
    mask = np.ones((B, H, 3, 3), np.uint8)
    mask[:, :, 0, 1] = 0
    o = oracle.attention(q, k, v, kv_len, mask, block)
    V = widen(v)
    np.testing.assert_allclose(o[:, :, 64:kv_len], np.broadcast_to(
        V[:, :, :kv_len].mean(axis=2, keepdims=True), o[:, :, 64:kv_len].shape), atol=1e-13)
    allowed0 = np.r_[0:64, 128:kv_len]
    np.testing.assert_allclose(o[:, :, :64], np.broadcast_to(
        V[:, :, allowed0].mean(axis=2, keepdims=True), o[:, :, :64].shape), atol=1e-13)


def test_p8_shift_invariance():
    B, H, N, D, block = 1, 2, 128, 64, 64
    q, k, v = wl.make_qkv(B, H, N, D, seed=28)
    u = np.zeros(D, np.float32)
    u[:4] = [8.0, -16.0, 4.0, 32.0]                       # exactly representable shifts
    kf = wl.bf16_bits_to_f32(k)
    # keep K + u exactly representable in bf16: quantise K coarsely first
    kq = np.round(kf * 4) / 4
    k1 = wl.f32_to_bf16_bits(kq)
    k2 = wl.f32_to_bf16_bits(kq + u)
    assert np.array_equal(wl.bf16_bits_to_f32(k2), kq + u)
    mask = wl.mask_bernoulli_diag(B, H, 2, 0.5, 4)
    a = oracle.attention(q, k1, v, N, mask, block)
    b = oracle.attention(q, k2, v, N, mask, block)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-10)


def test_p9_key_permutation_invariance():
    B, H, N, D, block = 1, 2, 256, 64, 64
    q, k, v = wl.make_qkv(B, H, N, D, seed=29)
    mask = wl.mask_bernoulli_diag(B, H, 4, 0.5, 8)
    base = oracle.attention(q, k, v, N, mask, block)
    rng = np.random.default_rng(1)
    # permute tokens inside each key block
    perm = np.concatenate([j * block + rng.permutation(block) for j in range(4)])
    o1 = oracle.attention(q, k[:, :, perm], v[:, :, perm], N, mask, block)
    np.testing.assert_allclose(o1, base, rtol=0, atol=1e-13)
    # permute whole key blocks together with the mask columns
    bp = rng.permutation(4)
    tok = np.concatenate([np.arange(j * block, (j + 1) * block) for j in bp])
    o2 = oracle.attention(q, k[:, :, tok], v[:, :, tok], N, mask[:, :, :, bp], block)
    np.testing.assert_allclose(o2, base, rtol=0, atol=1e-13)


def test_p10_sample_head_independence_and_cfg_duplicate():
    B, H, N, D, block, kv_len = 2, 2, 128, 64, 64, 100
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=30)
    mask = wl.mask_bernoulli_diag(B, H, 2, 0.5, 2)
    base = oracle.attention(q, k, v, kv_len, mask, block)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[1, 0], k2[1, 0], v2[1, 0] = q[0, 1], k[0, 0], v[0, 1]
    o2 = oracle.attention(q2, k2, v2, kv_len, mask, block)
    keep = np.ones((B, H), bool)
    keep[1, 0] = False
    np.testing.assert_array_equal(o2[keep], base[keep])
    assert np.abs(o2[1, 0] - base[1, 0]).max() > 1e-3
    # CFG pair: the same sample twice with the same mask gives the same output twice
    qd, kd, vd = (np.concatenate([x[:1], x[:1]]) for x in (q, k, v))
    md = np.concatenate([mask[:1], mask[:1]])
    od = oracle.attention(qd, kd, vd, kv_len, md, block)
    np.testing.assert_array_equal(od[0], od[1])
    np.testing.assert_array_equal(od[0], base[0])


def test_p11_convex_combination_bounds():
    B, H, N, D, block, kv_len = 1, 2, 256, 64, 64, 222
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=31)
    mask = wl.mask_bernoulli_diag(B, H, 4, 0.4, 6)
    o = oracle.attention(q, k, v, kv_len, mask, block)
    V = widen(v)
    for h in range(H):
        for i in range(4):
            cols = np.concatenate([np.arange(j * block, min((j + 1) * block, kv_len))
                                   for j in range(4) if mask[0, h, i, j]])
            lo, hi = V[0, h, cols].min(0), V[0, h, cols].max(0)
            rows = slice(i * block, min((i + 1) * block, kv_len))
            assert (o[0, h, rows] >= lo - 1e-12).all() and (o[0, h, rows] <= hi + 1e-12).all()


def test_p12_zero_queries_uniform_and_peaky_regime():
    B, H, N, D, block, kv_len = 1, 2, 128, 64, 64, 97
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=32)
    q0 = np.zeros_like(q)
    o = oracle.attention(q0, k, v, kv_len)
    np.testing.assert_allclose(o[:, :, :kv_len], np.broadcast_to(
        widen(v)[:, :, :kv_len].mean(2, keepdims=True), o[:, :, :kv_len].shape), atol=1e-13)
    qp, kp, vp = wl.make_qkv(B, H, N, D, kv_len, seed=33, gain=4.0)
    np.testing.assert_allclose(oracle.attention(qp, kp, vp, kv_len),
                               brute(qp, kp, vp, kv_len, None, block), rtol=0, atol=1e-12)


def test_empty_row_is_zero_not_nan():
    B, H, N, D, block = 1, 1, 128, 64, 64
    q, k, v = wl.make_qkv(B, H, N, D, seed=34)
    mask = np.array([[[[0, 0], [1, 1]]]], np.uint8)
    o = oracle.attention(q, k, v, N, mask, block)
    assert (o[0, 0, :64] == 0).all() and np.isfinite(o).all()
    # a kept tile lying wholly in the padding contributes nothing
    mask = np.array([[[[0, 1], [1, 1]]]], np.uint8)
    o = oracle.attention(q, k, v, 60, mask, block)
    assert (o[0, 0, :64] == 0).all()


def test_kept_tiles_lists():
    mask = np.zeros((1, 2, 4, 4), np.uint8)
    mask[0, 0] = [[1, 0, 0, 1], [0, 0, 0, 0], [1, 1, 1, 1], [0, 7, 0, 0]]
    mask[0, 1] = np.eye(4)
    counts, idx = oracle.kept_tiles(mask, 64, 200)         # block 3 starts at 192 < 200
    assert counts[0, 0].tolist() == [2, 0, 4, 1]
    assert idx[0, 0].tolist() == [[0, 3, -1, -1], [-1] * 4, [0, 1, 2, 3], [1, -1, -1, -1]]
    counts, idx = oracle.kept_tiles(mask, 64, 192)         # block 3 now wholly padding
    assert counts[0, 0].tolist() == [1, 0, 3, 1]
    assert counts[0, 1].tolist() == [1, 1, 1, 0]
    assert idx[0, 0, 2].tolist() == [0, 1, 2, -1]


def test_bad_arguments_are_rejected():
    q, k, v = wl.make_qkv(1, 1, 64, 32, seed=1)
    with pytest.raises(ValueError):
        oracle.attention(q, k, v, kv_len=0)
    with pytest.raises(ValueError):
        oracle.attention(q, k, v, kv_len=65)
    with pytest.raises(ValueError):
        oracle.attention(q, k, v, 64, np.ones((1, 1, 2, 2), np.uint8), 48)
