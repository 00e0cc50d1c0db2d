"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by
element on the same seeded inputs.  Tolerances: max-abs 1e-2, mean-abs 1e-3, plus a
relative Frobenius bound of 1e-2; integer work (mask compaction) is bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import assert_close, from_dev, to_dev, widen

pytestmark = pytest.mark.gpu


def run_dense(q, k, v, kv_len, scale=0.0):
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full_like(dq, float("nan"))
    ra.rapid_attn_dense(dq, dk, dv, o, kv_len, scale)
    torch.cuda.synchronize()
    return from_dev(o)


def run_sparse(q, k, v, mask, block, kv_len, scale=0.0, return_ws=False):
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    dm = torch.from_numpy(mask).cuda()
    B, H, N, D = q.shape
    ws = torch.full((ra.rapid_attn_workspace_bytes(B, H, N, D, block),), 0xAB, dtype=torch.uint8, device="cuda")
    o = torch.full_like(dq, float("nan"))
    ra.rapid_attn_block_sparse(dq, dk, dv, o, dm, block, kv_len, scale, ws)
    torch.cuda.synchronize()
    return (from_dev(o), ws.cpu().numpy()) if return_ws else from_dev(o)


# ---------------------------------------------------------------- small, every element
SMALL = [
    # B, H, N, D, block, kv_len, p_keep, pad_fill
    (1, 2, 256, 64, 64, 256, 0.5, "zero"),      # the Tiny workload's shape
    (2, 3, 384, 64, 64, 300, 0.4, "nan"),       # ragged tail inside a tile, several tiles
    (1, 2, 512, 128, 128, 512, 0.5, "zero"),
    (2, 2, 384, 128, 128, 333, 0.5, "nan"),
    (1, 3, 640, 64, 128, 577, 0.3, "inf"),
    (1, 2, 320, 128, 64, 259, 0.5, "nan"),
    (3, 1, 128, 64, 64, 1, 1.0, "nan"),         # a single valid token
    (1, 1, 1152, 128, 128, 1100, 0.35, "nan"),
]


@pytest.mark.parametrize("B,H,N,D,block,kv_len,p,fill", SMALL)
def test_dense_small(B, H, N, D, block, kv_len, p, fill):
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=101, pad_fill=fill)
    got = run_dense(q, k, v, kv_len)
    ref = oracle.attention(q, k, v, kv_len)
    assert_close(got, ref, "dense")
    assert (got[:, :, kv_len:] == 0).all()


@pytest.mark.parametrize("B,H,N,D,block,kv_len,p,fill", SMALL)
def test_sparse_small(B, H, N, D, block, kv_len, p, fill):
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=102, pad_fill=fill)
    mask = wl.mask_bernoulli_diag(B, H, N // block, p, seed=7)
    got = run_sparse(q, k, v, mask, block, kv_len)
    ref = oracle.attention(q, k, v, kv_len, mask, block)
    assert_close(got, ref, "sparse")
    assert (got[:, :, kv_len:] == 0).all()


@pytest.mark.parametrize("N,kv_len,D", [(200, 200, 64), (77, 50, 128), (130, 129, 64)])
def test_dense_any_token_count(N, kv_len, D):
    q, k, v = wl.make_qkv(2, 2, N, D, kv_len, seed=103, pad_fill="nan")
    assert_close(run_dense(q, k, v, kv_len), oracle.attention(q, k, v, kv_len), "dense odd N")


@pytest.mark.parametrize("B,H,N,D,kv_len", [(2, 9, 2048, 128, 2000), (1, 20, 2304, 64, 2250)])
def test_dense_mid_size_every_element(B, H, N, D, kv_len):
    """Several 256-query workgroup tiles per head, dozens of key tiles, ragged tail: every
    element against the oracle."""
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=107, pad_fill="nan")
    got = run_dense(q, k, v, kv_len)
    assert_close(got, oracle.attention(q, k, v, kv_len), "dense mid-size")
    assert (got[:, :, kv_len:] == 0).all()


def test_tiny_workload_both_masks_and_dense():
    w = wl.WORKLOADS["tiny"]
    q, k, v = w.qkv()
    ref_dense = oracle.attention(q, k, v, w.kv_len)
    assert_close(run_dense(q, k, v, w.kv_len), ref_dense, "tiny dense")
    assert_close(run_sparse(q, k, v, w.mask(1.0), w.block, w.kv_len), ref_dense, "tiny all-ones")
    m = w.mask(0.5)
    assert_close(run_sparse(q, k, v, m, w.block, w.kv_len),
                 oracle.attention(q, k, v, w.kv_len, m, w.block), "tiny 0.5")


def test_custom_scale_and_peaky_inputs():
    B, H, N, D, kv_len = 1, 2, 384, 64, 350
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=104)
    assert_close(run_dense(q, k, v, kv_len, 0.07), oracle.attention(q, k, v, kv_len, scale=0.07), "scale")
    # a large scale concentrates the softmax: |O| reaches ~3, where half a bf16 ulp of the
    # OUTPUT is already 2^-7; the absolute bounds (stated for 1/sqrt(D) on unit-normal
    # inputs, |O| << 1) are therefore applied relative to max(1, |O|max)
    ref = oracle.attention(q, k, v, kv_len, scale=0.31)
    got = widen(run_dense(q, k, v, kv_len, 0.31))
    mag = max(1.0, np.abs(ref).max())
    assert np.abs(got - ref).max() <= 1e-2 * mag and np.abs(got - ref).mean() <= 1e-3
    # scores with std ~16: the running max moves a lot, probabilities are near one-hot
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=105, gain=4.0)
    ref = oracle.attention(q, k, v, kv_len)
    got = widen(run_dense(q, k, v, kv_len))
    assert np.isfinite(got).all()
    # values reach ~12 here (half a bf16 ulp of the output is 2^-5): bounds relative to |O|max
    mag = max(1.0, np.abs(ref).max())
    assert np.abs(got - ref).max() <= 1e-2 * mag and np.abs(got - ref).mean() <= 1e-3 * mag
    assert np.sqrt(((got - ref) ** 2).sum() / (ref ** 2).sum()) <= 1e-2


def plan_geometry(B, H, nb, D, block):
    """Workspace geometry of the sparse entry point, as its header states it."""
    up = lambda x: (x + 255) // 256 * 256
    rows = B * H * nb
    items = (B * H + 7) // 8 * nb
    if block == 128:
        pmax = min(256, items)
        chunk = items + pmax
        rec_bytes = 16
    else:
        pmax, chunk, rec_bytes = 0, items, 4
    off_order = up(rows * 4)
    off_index = off_order + up(8 * chunk * rec_bytes)
    return dict(rows=rows, pmax=pmax, chunk=chunk, off_order=off_order, off_index=off_index)


def read_plan(ws, B, H, nb, D, block):
    g = plan_geometry(B, H, nb, D, block)
    rows, chunk = g["rows"], g["chunk"]
    counts = ws[:rows * 4].view(np.int32)
    width = 4 if block == 128 else 1
    order = ws[g["off_order"]:g["off_order"] + 8 * chunk * 4 * width].view(np.int32).reshape(8, chunk, width)
    index = ws[g["off_index"]:g["off_index"] + rows * nb * 4].view(np.int32).reshape(rows, nb)
    return counts, order, index, g


def split_rule(counts_x, D):
    """The rule of one XCD whose items keep counts_x blocks: (granules g, p_all).  P(c) =
    round(c * g / total) pieces, or p_all for every item when that is not 0; at most c // 8 and 16.
    D = 128: g = 32 x 2.5; rows all alike (8 n max <= 9 total): p_all = the first P in 1 .. max // 8
    that minimises rounds(P) x (piece length + 2 + 2 [P > 1]) over the XCD's 64 places.
    D = 64: g = 32 x 4, rows all alike: 32 x 12."""
    n, total, longest = len(counts_x), int(np.sum(counts_x)), int(np.max(counts_x, initial=0))
    alike = 8 * n * longest <= 9 * total
    if D != 128:
        return 32 * (12 if alike else 4), 0
    p_all = 0
    if alike and total:
        cost = lambda P: -(-n * P // 64) * (-(-longest // P) + 2 + (2 if P > 1 else 0))
        p_all = min(range(1, max(1, min(longest // 8, 16)) + 1), key=lambda P: (cost(P), P))
    return 80, p_all


def split_pieces(c, total, rule):
    if total == 0:
        return 1
    g, p_all = rule
    return max(1, min(p_all if p_all else (2 * c * g + total) // (2 * total), c // 8, 16))


def check_plan(counts, order, g, B, H, nb, block, D=64):
    """The launch plan, entry for entry.  Every XCD segment holds the entries of the (b,h) pairs
    with (b*H+h) % 8 == x, longest first, then -1.  With 64-token tiles an entry is an item; with
    128-token tiles it is a record (item, first list position, kept blocks, w) and an item that is
    long against a CU's share of the work is cut into pieces by the rule in the header."""
    rows = B * H * nb
    n_split = 0
    for x in range(8):
        seg = order[x]
        valid = seg[:, 0] >= 0
        n = int(valid.sum())
        assert valid[:n].all() and (seg[n:, 0] == -1).all()
        ent = seg[:n]
        mine = [i for i in range(rows) if (i // nb) % 8 == x]          # ascending item id
        assert ((ent[:, 0] // nb) % 8 == x).all()
        if block != 128:
            assert sorted(ent[:, 0].tolist()) == mine
            assert (np.diff(counts[ent[:, 0]]) <= 0).all()
            continue
        most = (B * H + 7) // 8 * nb                                    # items of the fullest XCD
        if nb <= 64 and most <= 1024 and most * nb <= 8192:
            # the one-launch planner: the odd rounds of 32 of the first wave (one record per place
            # of the XCD: 32 CUs x 2 at D = 128, x 4 at D = 64) are stored backwards
            ent = ent.copy()
            for lo in range(32, min(n, 32 * (2 if D == 128 else 4)), 64):
                ent[lo:lo + 32] = ent[lo:lo + 32][::-1].copy()
        assert (np.diff(ent[:, 2]) <= 0).all()
        total = int(counts[mine].sum())
        rule = split_rule(counts[mine], D)
        want, run = [], 0
        for it in mine:
            c = int(counts[it])
            P = split_pieces(c, total, rule)
            slot0 = -1
            if P > 1:
                if run + P <= g["pmax"]:
                    slot0 = run
                run += P
                if slot0 < 0:
                    P = 1
            for k in range(P):
                b0 = c * k // P
                w = ((x * g["pmax"] + slot0) << 8 | k << 4 | (P - 1)) if P > 1 else -1
                want.append((it, b0, c * (k + 1) // P - b0, w))
            n_split += P > 1
        assert sorted(map(tuple, ent.tolist())) == sorted(want)
    return n_split


def test_compaction_is_bit_exact():
    B, H, N, D, block, kv_len = 2, 3, 1152, 64, 128, 1100
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=106)
    mask = wl.mask_bernoulli_diag(B, H, N // block, 0.4, seed=9)
    mask[0, 0, 2, :] = 0                                   # an empty row
    mask[1, 2, :, :] = 3                                   # nonzero, not 1
    _, ws = run_sparse(q, k, v, mask, block, kv_len, return_ws=True)
    nb = N // block
    rows = B * H * nb
    counts, order, index, g = read_plan(ws, B, H, nb, D, block)
    want_counts, want_index = oracle.kept_tiles(mask, block, kv_len)
    np.testing.assert_array_equal(counts, want_counts.reshape(-1))
    want_index = want_index.reshape(rows, nb)
    for r in range(rows):
        np.testing.assert_array_equal(index[r, :counts[r]], want_index[r, :counts[r]])
    check_plan(counts, order, g, B, H, nb, block)


def test_compaction_is_bit_exact_with_64_token_tiles():
    B, H, N, D, block, kv_len = 2, 5, 576, 64, 64, 530
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=107)
    nb = N // block
    mask = wl.mask_bernoulli_diag(B, H, nb, 0.5, seed=10)
    _, ws = run_sparse(q, k, v, mask, block, kv_len, return_ws=True)
    counts, order, index, g = read_plan(ws, B, H, nb, D, block)
    want_counts, want_index = oracle.kept_tiles(mask, block, kv_len)
    np.testing.assert_array_equal(counts, want_counts.reshape(-1))
    for r in range(B * H * nb):
        np.testing.assert_array_equal(index[r, :counts[r]], want_index.reshape(-1, nb)[r, :counts[r]])
    check_plan(counts, order, g, B, H, nb, block)


PLANNERS = [
    # B, H, N, kv_len, p_keep, D: 128-token tiles.  Up to 64 blocks per side, 1024 items and
    # 8 KB of mask rows per XCD the one-launch planner runs, beyond that compaction + planner.
    (1, 3, 128, 100, 1.0, 64),        # one block per side, XCDs 3..7 without items
    (1, 2, 8192, 8100, 0.3, 64),      # 64 blocks per side: a row fills the whole 64-bit word
    (2, 8, 8192, 8192, 0.2, 128),     # two pairs per XCD: exactly 8 KB of mask rows
    (3, 8, 8192, 8000, 0.2, 64),      # three pairs per XCD: past the limit
    (1, 8, 10240, 10200, 0.25, 128),  # 80 blocks per side: past the limit
    (37, 3, 640, 520, 0.6, 64),       # 111 pairs: 14 per XCD on some, 13 on others
    (1, 24, 2816, 2816, 1.0, 128),    # all-ones mask with about as many items as the chip has places
]


@pytest.mark.parametrize("B,H,N,kv_len,p,D", PLANNERS)
def test_lists_and_plan_on_both_planners(B, H, N, kv_len, p, D):
    """Kept-block lists against the oracle's and the launch plan record for record, on shapes on
    both sides of the limits that choose between the two planners and with both head sizes (the
    split rule depends on it); the outputs themselves are compared with the oracle in the other
    tests, here on a few sampled rows."""
    block = 128
    nb = N // block
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=B * 1000 + nb)
    mask = wl.mask_bernoulli_diag(B, H, nb, p, seed=nb)
    mask[0, 0, nb // 2, :] = 0                              # an empty row
    mask[-1, -1, 0, :] = 7                                  # a full row, nonzero but not 1
    got, ws = run_sparse(q, k, v, mask, block, kv_len, return_ws=True)
    counts, order, index, g = read_plan(ws, B, H, nb, D, block)
    want_counts, want_index = oracle.kept_tiles(mask, block, kv_len)
    np.testing.assert_array_equal(counts, want_counts.reshape(-1))
    want_index = want_index.reshape(-1, nb)
    for r in range(B * H * nb):
        np.testing.assert_array_equal(index[r, :counts[r]], want_index[r, :counts[r]])
    check_plan(counts, order, g, B, H, nb, block, D)
    rows = wl.sample_rows(B, H, N, kv_len, block, 48, seed=5)
    ref = oracle.attention_rows(q, k, v, rows, kv_len, mask, block)
    assert_close(got[rows[:, 0], rows[:, 1], rows[:, 2]], ref, "sampled rows")


@pytest.mark.parametrize("D", [64, 128])
def test_long_rows_are_split_into_pieces_and_merged(D):
    """A few rows keep every tile while the rest keep few: the long rows are cut into pieces
    and combined by the last piece to finish.
    The ragged tail block (kv_len inside it) is the last block of the last piece."""
    B, H, N, block, kv_len = 2, 8, 4608, 128, 4500
    nb = N // block
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=108 + D)
    mask = wl.mask_bernoulli_diag(B, H, nb, 0.08, seed=12)
    mask[:, :, 5, :] = 1
    mask[:, :, nb - 1, :] = 1
    mask[1, :, 17, ::2] = 1
    got, ws = run_sparse(q, k, v, mask, block, kv_len, return_ws=True)
    counts, order, _, g = read_plan(ws, B, H, nb, D, block)
    np.testing.assert_array_equal(counts, oracle.kept_tiles(mask, block, kv_len)[0].reshape(-1))
    assert check_plan(counts, order, g, B, H, nb, block, D) >= 2 * B * H
    rng = np.random.default_rng(3)
    rows_ = np.stack([rng.integers(B, size=160), rng.integers(H, size=160),
                      rng.choice(np.r_[5 * block:6 * block, (nb - 1) * block:kv_len, 17 * block:18 * block,
                                       0:block], size=160)], axis=1).astype(np.int32)
    ref = oracle.attention_rows(q, k, v, rows_, kv_len, mask, block)
    assert_close(got[rows_[:, 0], rows_[:, 1], rows_[:, 2]], ref, "split rows")


# ---------------------------------------------------------------- full sizes, sampled rows
FULL = [("sd3_1024", 1.0), ("sd3_1024", 0.25), ("flux_1024", 1.0), ("flux_1024", 0.5),
        ("flux_1024", 0.2), ("grpo_sd3", "mixed"), ("flux_2048", 0.1), ("flux_2048", 0.3)]


@pytest.mark.parametrize("name,density", FULL)
def test_full_size_sampled_rows(name, density):
    """The bench's launch configuration at the full workload sizes; the oracle
    computes a seeded sample of output rows (first/last/boundary/pad rows included)."""
    w = wl.WORKLOADS[name]
    q, k, v = w.qkv(pad_fill="nan")
    mask = w.mask(density)
    rows = wl.sample_rows(w.B, w.H, w.N, w.kv_len, w.block, 384, seed=w.seed() + 1)
    got = run_sparse(q, k, v, mask, w.block, w.kv_len)
    ref = oracle.attention_rows(q, k, v, rows, w.kv_len, mask, w.block)
    sel = got[rows[:, 0], rows[:, 1], rows[:, 2]]
    assert_close(sel, ref, f"{name} d={density} sparse entry")
    assert (got[:, :, w.kv_len:] == 0).all()
    assert np.isfinite(widen(got)).all()
    if density == 1.0:
        got_d = run_dense(q, k, v, w.kv_len)
        assert_close(got_d[rows[:, 0], rows[:, 1], rows[:, 2]], ref, f"{name} dense entry")
        # action 0 == all-ones mask, up to summation order (the sparse path splits the key
        # list between two wavefront groups and merges them)
        assert_close(got, widen(got_d), f"{name} all-ones vs dense")
