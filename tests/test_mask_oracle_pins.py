"""Pins of the block-mask selection oracle.  The rule is this build's own (the paper does not
define one: parity against the paper is unpinned); these tests pin that the oracle computes
the stated rule: a hand-worked example, brute force over all subsets, invariants."""
import itertools

import numpy as np
import pytest

import workloads as wl
from oracle import mask_oracle as mo


def bits(a):
    b = wl.f32_to_bf16_bits(np.asarray(a, np.float32))
    assert (wl.bf16_bits_to_f32(b) == np.asarray(a, np.float32)).all(), "test values must be bf16 numbers"
    return b


def hand_example():
    """One head, 3 blocks of 2 tokens, D = 2, scale 1.  Query block means are (1, 0); key block
    means are (s_j, 0) with s = ln 6, ln 3, ln 1 -> every row has phat = (0.6, 0.3, 0.1).
    The means are formed from two different tokens each (a +/- 0.5 around the mean)."""
    s = np.log([6.0, 3.0, 1.0])
    q = np.zeros((1, 1, 6, 2), np.float64)
    k = np.zeros((1, 1, 6, 2), np.float64)
    for j in range(3):
        q[0, 0, 2 * j] = (1.5, 0.25)
        q[0, 0, 2 * j + 1] = (0.5, -0.25)
        k[0, 0, 2 * j] = (s[j] + 0.5, 1.0)
        k[0, 0, 2 * j + 1] = (s[j] - 0.5, -1.0)
    return q, k


def test_hand_worked_probabilities_and_selection():
    q, k = hand_example()
    # the oracle takes bf16 bits; feed it exact fp64 through a shim on its widening step
    orig = mo._widen
    mo._widen = lambda x: np.asarray(x, np.float64)
    try:
        p, live = mo.block_probabilities(q, k, 2, 6, scale=1.0)
        assert live == 3
        np.testing.assert_allclose(p[0, 0], np.tile([0.6, 0.3, 0.1], (3, 1)), atol=1e-15)
        # the scale multiplies the scores: scale 2 squares the ratios, the default is 1/sqrt(D)
        p2x, _ = mo.block_probabilities(q, k, 2, 6, scale=2.0)
        np.testing.assert_allclose(p2x[0, 0, 0], np.array([36.0, 9.0, 1.0]) / 46.0, atol=1e-15)
        pd, _ = mo.block_probabilities(q, k, 2, 6)
        wd = np.array([6.0, 3.0, 1.0]) ** (1 / np.sqrt(2.0))
        np.testing.assert_allclose(pd[0, 0, 2], wd / wd.sum(), atol=1e-15)
        far = 100                                          # no text blocks
        rows = lambda tau: mo.select_mask(q, k, 2, 6, far, tau, scale=1.0)[0, 0]
        # row 0 (diagonal = block 0, already the heaviest): exactly the cumulative rule
        assert rows(0.5)[0].tolist() == [1, 0, 0]
        assert rows(0.6)[0].tolist() == [1, 0, 0]          # reaching tau exactly is enough
        assert rows(0.61)[0].tolist() == [1, 1, 0]
        assert rows(0.9)[0].tolist() == [1, 1, 0]
        assert rows(0.91)[0].tolist() == [1, 1, 1]
        # rows 1 and 2 add their diagonal
        assert rows(0.5)[1].tolist() == [1, 1, 0] and rows(0.5)[2].tolist() == [1, 0, 1]
        # text starts at token 4 -> block 2 is text: its column and its row are kept
        m = mo.select_mask(q, k, 2, 6, 4, 0.5, scale=1.0)[0, 0]
        assert m.tolist() == [[1, 0, 1], [1, 1, 1], [1, 1, 1]]
        # kv_len = 3: block 1 has one valid token (its mean is that token), block 2 is dead
        p2, live2 = mo.block_probabilities(q, k, 2, 3, scale=1.0)
        assert live2 == 2 and (p2[0, 0, 2] == 0).all() and (p2[0, 0, :, 2] == 0).all()
        # row 1: its query mean is token 2 alone = (1.5, 0.25); key means: block 0 = (ln 6, 0),
        # block 1 = token 2 alone = (ln 3 + 0.5, 1)
        want = np.exp([1.5 * np.log(6.0), 1.5 * (np.log(3.0) + 0.5) + 0.25 * 1.0])
        np.testing.assert_allclose(p2[0, 0, 1, :2], want / want.sum(), rtol=1e-14)
        m2 = mo.select_mask(q, k, 2, 3, far, 0.5, scale=1.0)[0, 0]
        assert (m2[2] == 0).all() and (m2[:, 2] == 0).all()
    finally:
        mo._widen = orig


def brute_force_row(p, tau):
    """Smallest subset with mass >= tau * total; among those of that size the heaviest; then
    everything tying with its lightest member."""
    n, total = len(p), p.sum()
    for size in range(0, n + 1):
        best = None
        for sub in itertools.combinations(range(n), size):
            m = p[list(sub)].sum()
            if m >= tau * total and (best is None or m > best[0]):
                best = (m, sub)
        if best is not None:
            keep = np.zeros(n, bool)
            keep[list(best[1])] = True
            if size:
                keep |= p == p[list(best[1])].min()
            return keep
    return np.ones(n, bool)


def test_selection_against_brute_force_over_subsets():
    rng = np.random.default_rng(2)
    for trial in range(300):
        n = int(rng.integers(1, 8))
        p = rng.random(n) ** 3 + 1e-3
        if trial % 3 == 0:                                  # plant ties
            p[rng.integers(n)] = p[rng.integers(n)]
        p /= p.sum()
        for tau in (0.3, 0.5, 0.9, 0.99, 1.0):
            got = mo.select_row(p, tau)
            want = brute_force_row(p, tau)
            # float sums over different orders: skip cases that sit on the threshold
            order = np.sort(p)[::-1]
            if np.any(np.abs(np.cumsum(order) - tau * p.sum()) < 1e-12):
                continue
            np.testing.assert_array_equal(got, want, err_msg=f"{p} tau={tau}")


def test_uniform_rows_tie_and_keep_everything():
    assert mo.select_row(np.full(7, 1 / 7), 0.2).all()
    assert mo.select_row(np.array([0.4, 0.2, 0.2, 0.2]), 0.5).tolist() == [True, True, True, True]
    assert mo.select_row(np.array([0.4, 0.2, 0.2, 0.2]), 0.4).tolist() == [True, False, False, False]
    assert mo.select_row(np.array([0.5, 0.3, 0.2]), 1.5).all()       # tau out of reach: keep all


def test_invariants_on_random_inputs():
    B, H, N, D, block, kv_len, text_start = 2, 3, 640, 64, 64, 600, 512
    q, k, _ = wl.make_qkv(B, H, N, D, kv_len, seed=8, gain=3.0, pad_fill="nan")
    p, live = mo.block_probabilities(q, k, block, kv_len)
    assert live == 10 and np.allclose(p[:, :, :live].sum(-1), 1.0, atol=1e-12)
    masks = [mo.select_mask(q, k, block, kv_len, text_start, tau) for tau in (0.5, 0.8, 0.95, 1.0)]
    for lo, hi in zip(masks, masks[1:]):                   # nested in tau
        assert (lo <= hi).all()
    assert (masks[-1][:, :, :live, :live] == 1).all()      # tau = 1 keeps every live block
    m = masks[1]
    idx = np.arange(live)
    assert (m[:, :, idx, idx] == 1).all()                  # diagonal
    assert (m[:, :, 8:live, :live] == 1).all() and (m[:, :, :live, 8:live] == 1).all()   # text rows / columns
    assert (m[:, :, live:] == 0).all() and (m[:, :, :, live:] == 0).all()               # dead blocks
    # kept mass reaches tau, and dropping the lightest kept (unforced) block would fall below it
    for b, h, i in itertools.product(range(B), range(H), range(8)):
        row, pr = m[b, h, i, :8].astype(bool), p[b, h, i]
        forced = np.zeros(live, bool)
        forced[i] = True
        forced[8:] = True
        sel = mo.select_row(pr[:live], 0.8)
        assert pr[:live][sel].sum() >= 0.8 - 1e-12
        assert pr[:live][sel].sum() - pr[:live][sel].min() < 0.8 + 1e-12
        assert (m[b, h, i, :live].astype(bool) == (sel | forced)).all()
    # poison in the padding rows (NaN beyond kv_len) changed nothing: same mask with zeros there
    q0, k0, _ = wl.make_qkv(B, H, N, D, kv_len, seed=8, gain=3.0, pad_fill="zero")
    np.testing.assert_array_equal(mo.select_mask(q0, k0, block, kv_len, text_start, 0.8), m)


def test_recall_of_true_attention_mass_on_block_structured_inputs():
    """When the tokens of a block share a direction (plus noise), the pooled scores predict where
    the true attention mass lies: the kept blocks hold nearly tau of it."""
    rng = np.random.default_rng(4)
    B, H, nb, block, D = 1, 2, 8, 64, 64
    N = nb * block
    centers_k = rng.normal(size=(H, nb, D)) * 1.5
    centers_q = centers_k[:, rng.permutation(nb)] + rng.normal(size=(H, nb, D)) * 0.3
    q = np.repeat(centers_q, block, axis=1)[None] + rng.normal(size=(B, H, N, D)) * 0.2
    k = np.repeat(centers_k, block, axis=1)[None] + rng.normal(size=(B, H, N, D)) * 0.2
    qb, kb = wl.f32_to_bf16_bits(q.astype(np.float32)), wl.f32_to_bf16_bits(k.astype(np.float32))
    tau = 0.9
    m = mo.select_mask(qb, kb, block, N, N + 1, tau)
    qf, kf = mo._widen(qb), mo._widen(kb)
    s = np.einsum("bhid,bhjd->bhij", qf, kf) / np.sqrt(D)
    pt = np.exp(s - s.max(-1, keepdims=True))
    pt /= pt.sum(-1, keepdims=True)
    token_keep = np.kron(m, np.ones((block, block), np.uint8)).astype(bool)
    recall = (pt * token_keep).sum(-1).mean()
    assert recall >= tau - 0.05, recall
    assert m.mean() < 0.6                                  # and it is actually sparse


MUTANTS = [
    ("ascending_order", "order = np.argsort(-p_row, kind=\"stable\")", "order = np.argsort(p_row, kind=\"stable\")"),
    ("strict_threshold", "if mass >= tau * total and p_row[j] != last:", "if mass > tau * total and p_row[j] != last:"),
    ("ties_dropped", "if mass >= tau * total and p_row[j] != last:", "if mass >= tau * total:"),
    ("mean_over_whole_block", "out[:, :, i] = x[:, :, lo:hi].sum(axis=2) / (hi - lo)", "out[:, :, i] = x[:, :, lo:hi].sum(axis=2) / block"),
    ("no_scale", "scale * float(np.dot(qb[b, h, i], kb[b, h, j]))", "float(np.dot(qb[b, h, i], kb[b, h, j]))"),
    ("transposed_scores", "np.dot(qb[b, h, i], kb[b, h, j])", "np.dot(qb[b, h, j], kb[b, h, i])"),
    ("no_diagonal", "                keep[i] = True\n", ""),
    ("text_rows_not_dense", "                if i >= first_text:\n                    keep[:] = True\n", ""),
    ("text_columns_not_kept", "                keep[first_text:live] = True\n", ""),
]


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(monkeypatch, name, find, repl):
    import inspect
    import types
    src = inspect.getsource(mo)
    assert src.count(find) >= 1, name
    mod = types.ModuleType("mask_oracle_mutant")
    exec(compile(src.replace(find, repl), "mask_oracle_mutant", "exec"), mod.__dict__)
    caught = 0
    for test in (test_hand_worked_probabilities_and_selection, test_selection_against_brute_force_over_subsets,
                 test_uniform_rows_tie_and_keep_everything, test_invariants_on_random_inputs):
        monkeypatch.setitem(globals(), "mo", mod)
        try:
            test()
        except AssertionError:
            caught += 1
        finally:
            monkeypatch.setitem(globals(), "mo", mo)
    assert caught, f"mutant {name} survived every pin"
