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
    """Where the arrays of the sparse entry point's workspace lie, as its header states it."""
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
    off_arrived = off_index + up(rows * nb * 4)
    return dict(rows=rows, pmax=pmax, chunk=chunk, off_order=off_order, off_index=off_index,
                off_arrived=off_arrived)


def read_plan(ws, B, H, nb, D, block):
    g = plan_geometry(B, H, nb, D, block)
    rows, chunk = g["rows"], g["chunk"]
    counts = ws[:rows * 4].view(np.int32)
    width = 4 if block == 128 else 1
    order = ws[g["off_order"]:g["off_order"] + 8 * chunk * 4 * width].view(np.int32).reshape(8, chunk, width)
    index = ws[g["off_index"]:g["off_index"] + rows * nb * 4].view(np.int32).reshape(rows, nb)
    g["arrived"] = ws[g["off_arrived"]:g["off_arrived"] + 8 * g["pmax"] * 4].view(np.int32)
    return counts, order, index, g


def check_plan(counts, order, g, B, H, nb, block, D=64):
    """The launch plan is one of many correct ones (how rows are cut and in which order they
    run is tuning), so it is checked for VALIDITY, after the call has run:
      * a segment is entries, then only "none" entries; segment x holds items of the (b,h)
        pairs with (b*H+h) % 8 == x and nothing else;
      * every item appears: once as a whole (first 0, n = its count, w = -1), or as pieces
        0..P-1 of P that cover its kept list exactly once, in order, none empty;
      * the P partial-result slots of a cut item lie inside its segment's pmax slots and no
        two items share a slot;
      * arrived[] holds P at the first slot of every cut item (all pieces counted in) and 0
        everywhere else.
    Returns {item: [(first, n, k, P), ...]} for the cut items."""
    rows = B * H * nb
    recs = {}
    for x in range(8):
        seg = order[x]
        valid = seg[:, 0] >= 0
        n = int(valid.sum())
        assert valid[:n].all(), "entries first, then none"
        if block == 128:
            assert (seg[n:] == np.array([-1, 0, 0, -1])).all()
        else:
            assert (seg[n:, 0] == -1).all()
        ent = seg[:n]
        assert (ent[:, 0] < rows).all() and ((ent[:, 0] // nb) % 8 == x).all()
        for e in ent.tolist():
            recs.setdefault(e[0], []).append(tuple(e[1:]))
    assert sorted(recs) == list(range(rows)), "every item has an entry"
    if block != 128:
        assert all(len(r) == 1 for r in recs.values())
        return {}
    pmax = g["pmax"]
    cut, slots_taken = {}, np.zeros(8 * pmax, bool)
    want_arrived = np.zeros(8 * pmax, np.int32)
    for item, rs in recs.items():
        c = int(counts[item])
        if len(rs) == 1 and rs[0][2] == -1:
            assert rs[0][:2] == (0, c), (item, rs, c)
            continue
        P = len(rs)
        assert 2 <= P <= 16
        rs = sorted(rs)
        x = (item // nb) % 8
        slot0 = rs[0][2] >> 8
        pos = 0
        for k, (first, nblk, w) in enumerate(rs):
            assert w >= 0 and (w & 15) == P - 1 and ((w >> 4) & 15) == k and (w >> 8) == slot0, (item, rs)
            assert first == pos and nblk >= 1, (item, rs)
            pos += nblk
        assert pos == c, (item, rs, c)
        assert x * pmax <= slot0 and slot0 + P <= (x + 1) * pmax
        assert not slots_taken[slot0:slot0 + P].any(), "two items share a partial-result slot"
        slots_taken[slot0:slot0 + P] = True
        want_arrived[slot0] = P
        cut[item] = [(first, nblk, k, P) for k, (first, nblk, w) in enumerate(rs)]
    np.testing.assert_array_equal(g["arrived"], want_arrived)
    return cut


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
    cut = check_plan(counts, order, g, B, H, nb, block, D)
    long_items = [(b * H + h) * nb + r for b in range(B) for h in range(H) for r in (5, nb - 1)]
    assert all(it in cut for it in long_items), "the rows that keep every tile are cut into pieces"
    rng = np.random.default_rng(3)
    rows_ = np.stack([rng.integers(B, size=160), rng.integers(H, size=160),
                      rng.choice(np.r_[5 * block:6 * block, (nb - 1) * block:kv_len, 17 * block:18 * block,
                                       0:block], size=160)], axis=1).astype(np.int32)
    ref = oracle.attention_rows(q, k, v, rows_, kv_len, mask, block)
    assert_close(got[rows_[:, 0], rows_[:, 1], rows_[:, 2]], ref, "split rows")


# ---------------------------------------------------------------- full sizes
def per_block_errors(got_bits, ref, block, what):
    """Beyond the whole-tensor bounds: every (sample, head, query-block) on its own, so that one
    wrong block (one plan record, one piece of a cut row) cannot hide in the average of millions
    of good elements."""
    B, H, N, D = ref.shape
    g = widen(got_bits)
    d2 = ((g - ref) ** 2).reshape(B, H, N // block, block * D).sum(-1)
    r2 = (ref ** 2).reshape(B, H, N // block, block * D).sum(-1)
    live = r2 > 0
    rel = np.sqrt(d2[live] / r2[live])
    worst = np.unravel_index(np.argmax(np.where(live, d2 / np.maximum(r2, 1e-300), 0)), d2.shape)
    assert rel.max() <= 1e-2, f"{what}: (b, h, query-block) {worst} is off by {rel.max():.3e} (relative Frobenius)"
    assert (d2[~live] == 0).all(), f"{what}: rows that must be zero are not"


EVERY = [("sd3_1024", 1.0), ("sd3_1024", 0.25), ("sd3_1024", "total0.25"), ("flux_1024", 1.0),
         ("flux_1024", 0.5), ("flux_1024", 0.2), ("grpo_sd3", "mixed")]


@pytest.mark.parametrize("name,density", EVERY)
def test_full_size_every_element(name, density):
    """The workloads at their full sizes, in the launch configuration the bench times, EVERY
    output element against the oracle: all (sample, head) pairs, all query-blocks, all plan
    records whatever their kind.  The plan that ran is read back and checked for validity."""
    w = wl.WORKLOADS[name]
    q, k, v = w.qkv(pad_fill="nan")
    mask = w.mask(density)
    got, ws = run_sparse(q, k, v, mask, w.block, w.kv_len, return_ws=True)
    ref = oracle.attention(q, k, v, w.kv_len, mask, w.block)
    e = assert_close(got, ref, f"{name} d={density} sparse entry")
    print(f"{name} d={density} sparse entry, every element: max-abs {e['max_abs']:.3e} mean-abs {e['mean_abs']:.3e} "
          f"rel-Frobenius {e['rel_fro']:.3e}")
    per_block_errors(got, ref, w.block, f"{name} d={density} sparse entry")
    assert (got[:, :, w.kv_len:] == 0).all()
    counts, order, index, g = read_plan(ws, w.B, w.H, w.nb, w.D, w.block)
    np.testing.assert_array_equal(counts, oracle.kept_tiles(mask, w.block, w.kv_len)[0].reshape(-1))
    cut = check_plan(counts, order, g, w.B, w.H, w.nb, w.block, w.D)
    print(f"{name} d={density}: {len(cut)} of {w.B * w.H * w.nb} rows ran as pieces")   # every one of them is compared
    if density == 1.0 or name == "grpo_sd3":
        mask_is_full = density == 1.0
        got_d = run_dense(q, k, v, w.kv_len)
        ref_d = ref if mask_is_full else oracle.attention(q, k, v, w.kv_len)
        e = assert_close(got_d, ref_d, f"{name} dense entry")
        print(f"{name} dense entry, every element: max-abs {e['max_abs']:.3e} mean-abs {e['mean_abs']:.3e} "
              f"rel-Frobenius {e['rel_fro']:.3e}")
        per_block_errors(got_d, ref_d, w.block, f"{name} dense entry")
        assert (got_d[:, :, w.kv_len:] == 0).all()


def stratified_blocks(w, extra, per_head, seed):
    """Query-blocks to check, per (sample, head): the first and last image block, the blocks at
    the edge of the local band, every text block, the blocks in `extra` (per pair), then random
    ones up to per_head."""
    rng = np.random.Generator(np.random.PCG64(seed))
    nI = w.nb - w.n_text_blocks
    out = {}
    for b in range(w.B):
        for h in range(w.H):
            s = {0, 1, 8, 9, nI - 10, nI - 9, nI - 2, nI - 1} | set(range(nI, w.nb)) | set(extra.get((b, h), ()))
            while len(s) < per_head:
                s.add(int(rng.integers(w.nb)))
            out[(b, h)] = sorted(s)
    return out


@pytest.mark.parametrize("density", [0.1, 0.3])
def test_flux_2048_sparse_stratified(density):
    """The largest workload (the oracle would need minutes for all of it): the plan is read
    back and the rows are chosen from it on purpose -- every (sample, head); at least 10 % of
    the query-blocks of each, among them the first, the last, the band edges, all text blocks
    and every block whose row was cut into pieces; all 128 rows (all four wavefronts) of each
    chosen block."""
    w = wl.WORKLOADS["flux_2048"]
    q, k, v = w.qkv(pad_fill="nan")
    mask = w.mask(density)
    got, ws = run_sparse(q, k, v, mask, w.block, w.kv_len, return_ws=True)
    counts, order, index, g = read_plan(ws, w.B, w.H, w.nb, w.D, w.block)
    want_counts, want_index = oracle.kept_tiles(mask, w.block, w.kv_len)
    np.testing.assert_array_equal(counts, want_counts.reshape(-1))
    want_index = want_index.reshape(-1, w.nb)
    for r in range(w.B * w.H * w.nb):
        np.testing.assert_array_equal(index[r, :counts[r]], want_index[r, :counts[r]])
    cut = check_plan(counts, order, g, w.B, w.H, w.nb, w.block, w.D)
    print(f"flux_2048 d={density}: {len(cut)} of {w.B * w.H * w.nb} rows ran as pieces")
    extra = {}
    for item in cut:
        extra.setdefault((item // w.nb // w.H, item // w.nb % w.H), []).append(item % w.nb)
    per_head = max(14, -(-w.nb // 10))
    blocks = stratified_blocks(w, extra, per_head, seed=w.seed() + 11)
    assert len(blocks) == w.B * w.H and all(len(v_) >= 0.10 * w.nb for v_ in blocks.values())
    assert all(set(extra.get(key, ())) <= set(v_) for key, v_ in blocks.items())
    rows = np.array([(b, h, i * w.block + r) for (b, h), bl in blocks.items() for i in bl for r in range(w.block)],
                    np.int32)
    ref = oracle.attention_rows(q, k, v, rows, w.kv_len, mask, w.block)
    sel = got[rows[:, 0], rows[:, 1], rows[:, 2]]
    e = assert_close(sel, ref, f"flux_2048 d={density}")
    print(f"flux_2048 d={density} sparse entry, {len(rows)} rows of {len(blocks)} (sample, head) pairs: max-abs {e['max_abs']:.3e} "
          f"mean-abs {e['mean_abs']:.3e} rel-Frobenius {e['rel_fro']:.3e}")
    per_block_errors(sel.reshape(1, 1, -1, w.D), ref.reshape(1, 1, -1, w.D), w.block, f"flux_2048 d={density}")
    assert np.isfinite(widen(got)).all()


def test_flux_2048_dense_stratified():
    """Dense entry at the largest workload: every (sample, head), 8 of the 66 workgroup tiles of
    256 queries of each (first, last, the one holding the image/text border, random ones), all
    256 rows (both wavefront groups) of each."""
    w = wl.WORKLOADS["flux_2048"]
    q, k, v = w.qkv(pad_fill="nan")
    got = run_dense(q, k, v, w.kv_len)
    rng = np.random.Generator(np.random.PCG64(w.seed() + 13))
    nt = w.N // 256
    rows = []
    for h in range(w.H):
        tiles = {0, nt - 1, (w.N - 512) // 256 - 1, (w.N - 512) // 256}
        while len(tiles) < 8:
            tiles.add(int(rng.integers(nt)))
        assert len(tiles) >= 0.10 * nt
        rows += [(0, h, t * 256 + r) for t in sorted(tiles) for r in range(256)]
    rows = np.array(rows, np.int32)
    ref = oracle.attention_rows(q, k, v, rows, w.kv_len)
    sel = got[rows[:, 0], rows[:, 1], rows[:, 2]]
    e = assert_close(sel, ref, "flux_2048 dense")
    print(f"flux_2048 dense entry, {len(rows)} rows: max-abs {e['max_abs']:.3e} mean-abs {e['mean_abs']:.3e} "
          f"rel-Frobenius {e['rel_fro']:.3e}")
    per_block_errors(sel.reshape(1, 1, -1, w.D), ref.reshape(1, 1, -1, w.D), 256, "flux_2048 dense")
    assert np.isfinite(widen(got)).all()
