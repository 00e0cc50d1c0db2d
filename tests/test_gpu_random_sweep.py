"""Seeded random sweeps over shapes, tile sizes, lengths, mask densities, layouts and fill values,
every output element against the oracles: the contiguous entries (dense, sparse, the entry that
allocates nothing), the model-shaped entry with per-sample lengths, selection and the one-call
select + attend form, the Cache-Reuse operations.  The hand-picked cases of the other files aim at
known edges; these look for the ones nobody thought of (a first run of the model-shaped sweep
found that a one-token text segment was refused for the arbitrary stride torch leaves on a
dimension of size one)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import errors, from_dev, to_dev
from oracle import cache_oracle as co

pytestmark = pytest.mark.gpu


def close(got_bits, ref, what):
    e = errors(got_bits, ref)
    scale = max(1.0, float(np.abs(ref).max()))          # high-gain cases: bounds relative to |O|max
    assert e["finite"] and e["max_abs"] <= 1e-2 * scale and e["rel_fro"] <= 1.2e-2, (what, e)


def test_contiguous_entries():
    rng = np.random.default_rng(20250922)
    for it in range(60):
        D, block = int(rng.choice([64, 128])), int(rng.choice([64, 128]))
        B, H, nb = int(rng.integers(1, 4)), int(rng.integers(1, 13)), int(rng.integers(1, 33))
        N = nb * block
        kv = int(rng.integers(1, N + 1)) if rng.random() < 0.7 else N
        p, fill, gain = float(rng.choice([0.1, 0.3, 0.6, 1.0])), str(rng.choice(["nan", "inf", "zero"])), float(rng.choice([1.0, 1.0, 3.0]))
        what = f"case {it}: B={B} H={H} N={N} D={D} block={block} kv_len={kv} p={p} fill={fill} gain={gain}"
        print(what, flush=True)
        q, k, v = wl.make_qkv(B, H, N, D, kv, seed=1000 + it, gain=gain, pad_fill=fill)
        mask = (rng.random((B, H, nb, nb)) < p).astype(np.uint8)
        if rng.random() < 0.5:
            mask[:, :, np.arange(nb), np.arange(nb)] = 1
        if rng.random() < 0.3:
            mask[:, :, nb - 1, :] = 1
        if rng.random() < 0.2:
            mask[:, :, 0, :] = 0
        dq, dk, dv, dm = to_dev(q), to_dev(k), to_dev(v), torch.from_numpy(mask).cuda()
        o = torch.full_like(dq, float("nan"))
        ra.rapid_attn_dense(dq, dk, dv, o, kv)
        torch.cuda.synchronize()
        close(from_dev(o), oracle.attention(q, k, v, kv), what + " dense")
        o.fill_(float("nan"))
        ra.rapid_attn_block_sparse(dq, dk, dv, o, dm, block, kv)
        torch.cuda.synchronize()
        close(from_dev(o), oracle.attention(q, k, v, kv, mask, block), what + " sparse")
        o2 = torch.full_like(dq, float("nan"))
        ra.rapid_attn_block_sparse_static(dq, dk, dv, o2, dm, block, kv)
        torch.cuda.synchronize()
        assert torch.equal(o.view(torch.int16), o2.view(torch.int16)), what + " static entry"


def test_model_shaped_entries():
    from test_gpu_joint import as_model_tensors, gather, oracle_joint
    from test_gpu_mask import oracle_joint_mask
    rng = np.random.default_rng(20250923)
    for it in range(40):
        D, block = int(rng.choice([64, 128])), int(rng.choice([64, 128]))
        B, H = int(rng.integers(1, 4)), int(rng.integers(1, 6))
        n_img, n_txt = 128 * int(rng.integers(1, 11)), int(rng.choice([0, 1, 33, 64, 77, 128, 200, 333]))
        fused = bool(rng.random() < 0.5)
        N = n_img + n_txt
        nb = -(-N // block)
        lens = np.array([int(rng.choice([0, N, N, int(rng.integers(1, N + 1))])) for _ in range(B)], np.int32)
        tau, text_start = float(rng.choice([0.3, 0.6, 0.9, 0.98, 1.0])), int(rng.choice([n_img, N, 0]))
        what = (f"case {it}: B={B} H={H} n_img={n_img} n_txt={n_txt} D={D} block={block} fused={fused} "
                f"lens={lens.tolist()} tau={tau} text_start={text_start}")
        print(what, flush=True)
        if rng.random() < 0.6:
            q, k, v = wl.make_qkv_block_structured(B, H, N, D, block, seed=7000 + it, n_text_blocks=-(-n_txt // block))
        else:
            q, k, v = wl.make_qkv(B, H, N, D, N, seed=7000 + it, gain=3.0)
        dl = torch.from_numpy(lens).cuda()

        def per_sample(got, m, label):
            for b in range(B):
                if lens[b] == 0:
                    assert (got[b] == 0).all(), what + label
                else:
                    close(got[b:b + 1], oracle_joint(q[b:b + 1], k[b:b + 1], v[b:b + 1], int(lens[b]),
                                                     None if m is None else m[b:b + 1], block), what + label)

        given = (rng.random((B, H, nb, nb)) < 0.4).astype(np.uint8)
        given[:, :, np.arange(nb), np.arange(nb)] = 1
        for m in (None, given):
            segs, guards = as_model_tensors(q, k, v, n_img, fused)
            ra.rapid_attn_joint(segs, None if m is None else torch.from_numpy(m).cuda(), block, kv_lens=dl)
            torch.cuda.synchronize()
            per_sample(gather(segs), m, " joint dense" if m is None else " joint sparse")
            for g in guards:
                assert (g[:, :, 0] == 7.0).all() and (g[:, :, -1] == 7.0).all(), what + " guard"
        # selection: inside the oracle's band; the one-call form reports the same mask and attends under it
        segs, _ = as_model_tensors(q, k, v, n_img, fused)
        sel = torch.full((B, H, nb, nb), 9, dtype=torch.uint8, device="cuda")
        ra.rapid_mask_select_joint(segs, sel, block, kv_lens=dl, text_start=text_start, tau=tau)
        torch.cuda.synchronize()
        got = sel.cpu().numpy()
        lo = oracle_joint_mask(q, k, block, lens, text_start, max(tau - 1e-5, 1e-6))
        hi = oracle_joint_mask(q, k, block, lens, text_start, min(tau + 1e-5, 1.0))
        mid = oracle_joint_mask(q, k, block, lens, text_start, tau)
        assert set(np.unique(got)) <= {0, 1} and (lo <= got).all() and (got <= hi).all(), what + " selection band"
        assert (got == mid).mean() >= 0.995, what + " selection"
        sel2 = torch.full_like(sel, 9)
        ra.rapid_attn_joint_select(segs, block, kv_lens=dl, text_start=text_start, tau=tau, mask_out=sel2)
        torch.cuda.synchronize()
        assert torch.equal(sel, sel2), what + " one-call mask"
        per_sample(gather(segs), got, " one-call attention")


def test_cache_operations():
    from test_gpu_cache import dev, host, same, tensors
    rng = np.random.default_rng(20250924)
    for it in range(120):
        B = int(rng.choice([1, 1, 2, 3, 7]))
        per = int(rng.choice([1, 7, 8, 9, 63, 64, 1000, 4096, 4099, 65536 + int(rng.integers(0, 9)), 300001]))
        off = int(rng.choice([0, 0, 1, 3, 8])) if B == 1 else 0          # element offset of the views: alignment
        inplace, store = int(rng.choice([0, 0, 1, 2])), bool(rng.random() < 0.5)
        flags = (rng.random(B) < 0.5).astype(np.uint8) if rng.random() < 0.4 else None
        what = f"case {it}: B={B} per_sample={per} offset={off} flags={None if flags is None else flags.tolist()} in_place={inplace} store={store}"
        a, b = tensors((B, per), seed=9000 + it)
        out0 = np.full((B, per), 0x1234, np.uint16)

        def view(bits):
            if off == 0:
                return dev(bits)
            return dev(np.concatenate([np.zeros(off, np.uint16), bits.reshape(-1)]))[off:].view(B, per)

        da, db = view(a), view(b)
        do = da if inplace == 1 else db if inplace == 2 else view(out0)
        before = a if inplace == 1 else b if inplace == 2 else out0
        (ra.rapid_cache_store if store else ra.rapid_cache_reuse)(da, db, do, None if flags is None else torch.from_numpy(flags).cuda())
        torch.cuda.synchronize()
        full = co.cache_store(a, b) if store else co.cache_reuse(a, b)
        want = full if flags is None else np.where(flags[:, None] != 0, full, before)
        try:
            same(host(do.contiguous()).reshape(B, per), want)
        except AssertionError as e:
            raise AssertionError(what + ": " + str(e)[:300])
