"""GPU parity of the Cache-Reuse residual operations against the oracle: bit for bit (bf16
outputs of a correctly rounded sum are unique), NaN compared as NaN."""
import numpy as np
import pytest
import torch

import paper_2509_22323_amd as ra
import workloads as wl
from oracle import cache_oracle as co

pytestmark = pytest.mark.gpu


def dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def same(got, want):
    g, w = co.bf16_to_f64(got), co.bf16_to_f64(want)
    nan = np.isnan(w)
    assert (np.isnan(g) == nan).all()
    np.testing.assert_array_equal(got[~nan], want[~nan])


def tensors(shape, seed, special=True):
    rng = np.random.default_rng(seed)
    x = wl.f32_to_bf16_bits((rng.normal(size=shape) * rng.choice([1e-3, 1.0, 30.0], size=shape)).astype(np.float32))
    y = wl.f32_to_bf16_bits((rng.normal(size=shape) * rng.choice([1e-3, 1.0, 30.0], size=shape)).astype(np.float32))
    if special:
        fx, fy = x.reshape(-1), y.reshape(-1)
        n = fx.size
        pick = rng.choice(n, size=min(n, 64), replace=False)
        vals = np.array([0x0000, 0x8000, 0x7F80, 0xFF80, 0x7FC0, 0x0001, 0x8001, 0x007F, 0x0080, 0x7F7F, 0xFF7F,
                         0x3F80, 0x3B80, 0x3F81, 0x4380, 0x3C00], np.uint16)
        fx[pick] = rng.choice(vals, size=pick.size)
        fy[pick[::-1]] = rng.choice(vals, size=pick.size)
        fx[pick[:8]] = fy[pick[:8]]                        # equal operands: exact zero
    return x, y


SHAPES = [(1, 8), (1, 1), (1, 7), (1, 4099), (3, 40), (2, 4096), (5, 1001), (4, 16, 12, 8), (1, 300001), (8, 65536),
          (1, 4608 * 3072)]          # the last: one layer's hidden states, the size bench.py times


@pytest.mark.parametrize("shape", SHAPES, ids=[str(s) for s in SHAPES])
def test_store_and_reuse_bit_exact(shape):
    o, x = tensors(shape, seed=sum(shape))
    d_out = torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    ra.rapid_cache_store(dev(o), dev(x), d_out)
    same(host(d_out), co.cache_store(o, x))
    r_out = torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    ra.rapid_cache_reuse(dev(x), dev(o), r_out)
    same(host(r_out), co.cache_reuse(x, o))


def test_misaligned_views_take_the_scalar_path():
    o, x = tensors((1, 5000), seed=9)
    big_o, big_x = dev(np.concatenate([[0], o[0]]).astype(np.uint16)), dev(np.concatenate([[0], x[0]]).astype(np.uint16))
    out = torch.zeros(5001, dtype=torch.bfloat16, device="cuda")
    ra.rapid_cache_reuse(big_x[1:], big_o[1:], out[1:])                    # 2-byte aligned only
    same(host(out)[1:], co.cache_reuse(x[0], o[0]))
    assert host(out)[0] == 0


def test_image_wise_flags_and_in_place_update():
    x, d = tensors((6, 2048), seed=21)
    flags = np.array([1, 0, 0, 1, 1, 0], np.uint8)
    out0 = np.full((6, 2048), 0x1234, np.uint16)
    out = dev(out0)
    ra.rapid_cache_reuse(dev(x), dev(d), out, torch.from_numpy(flags).cuda())
    same(host(out), co.cache_reuse_batch(x, d, out0, flags))
    # in place: X <- X + Delta and Delta <- O - X written over O
    xd = dev(x)
    ra.rapid_cache_reuse(xd, dev(d), xd)
    same(host(xd), co.cache_reuse(x, d))
    od = dev(d)
    ra.rapid_cache_store(od, dev(x), od)
    same(host(od), co.cache_store(d, x))


def test_binding_rejects_wrong_tensors():
    a = torch.zeros(2, 8, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(TypeError):
        ra.rapid_cache_reuse(a.float(), a, a)
    with pytest.raises(ValueError):
        ra.rapid_cache_reuse(a, a[:, :4].contiguous(), a)
    with pytest.raises(TypeError):
        ra.rapid_cache_reuse(a, a, a, torch.zeros(3, dtype=torch.uint8, device="cuda"))


def test_more_than_two_to_the_32_elements():
    """One sample of 2^32 + 24 elements (8.6 GB per tensor): element indices do not fit 32 bits.
    The inputs repeat a seeded pattern whose length (2^20 + 7) does not divide 2^32, so an index
    that wrapped would read another phase of it; the expected result is the oracle's for one
    period, repeated the same way."""
    period, n = (1 << 20) + 7, (1 << 32) + 24
    o, x = tensors((1, period), seed=32, special=False)
    reps = -(-n // period)

    def tiled(bits):
        return dev(bits).reshape(-1).repeat(reps)[:n].reshape(1, n)

    d_o, d_x = tiled(o), tiled(x)
    d_out = torch.empty((1, n), dtype=torch.bfloat16, device="cuda")
    ra.rapid_cache_store(d_o, d_x, d_out)
    want = co.cache_store(o, x)
    assert torch.equal(d_out.view(torch.int16), tiled(want).view(torch.int16))
    ra.rapid_cache_reuse(d_x, d_out, d_o)                     # d_o <- x + delta
    assert torch.equal(d_o.view(torch.int16), tiled(co.cache_reuse(x, want)).view(torch.int16))
