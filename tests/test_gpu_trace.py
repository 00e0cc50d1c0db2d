"""The step-level driver issues exactly the calls the trace asks for and leaves the outputs of
its last computing / reusing step in place."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import assert_close, from_dev, to_dev
from oracle import cache_oracle as co
from oracle import mask_oracle as mo
from paper_2509_22323_amd.sampler import run_action_trace

pytestmark = pytest.mark.gpu


def test_driver_follows_the_trace():
    B, H, N, D, block, kv_len, text_start, layers = 1, 2, 512, 64, 128, 500, 384, 3
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=31)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full_like(dq, float("nan"))
    rng = np.random.default_rng(1)
    x = wl.f32_to_bf16_bits(rng.normal(size=(B, 4096)).astype(np.float32))
    g = wl.f32_to_bf16_bits(rng.normal(size=(B, 4096)).astype(np.float32))     # the stub generator's output
    dx, dout, ddelta = to_dev(x), to_dev(g), torch.zeros(B, 4096, dtype=torch.bfloat16, device="cuda")
    trace = [(0, 0), (1, 0), (0, 2), (1, 0), (0, 0), (0, 3), (1, 0)]
    res = run_action_trace(trace, dq, dk, dv, o, layers, block, kv_len, text_start, dx, ddelta, dout)
    assert [s["kind"] for s in res.steps] == ["full", "cached", "sparse-2", "cached", "full", "sparse-3", "cached"]
    assert res.calls == {"rapid_attn_dense": 2 * layers, "rapid_attn_block_sparse": 2 * layers,
                         "rapid_mask_select": 2 * layers, "rapid_cache_reuse": 3, "rapid_cache_store": 4}
    assert all(s["ms"] > 0 for s in res.steps) and abs(sum(s["ms"] for s in res.steps) - res.total_ms) < 1e-6
    # residual kept by the computing steps (out is the stub's fixed output), reused by the last step
    delta = co.cache_store(g, x)
    np.testing.assert_array_equal(from_dev(ddelta), delta)
    np.testing.assert_array_equal(from_dev(dout), co.cache_reuse(x, delta))
    # o holds the attention of the last computing step: sparse level 3 under the selected mask
    m = mo.select_mask(q, k, block, kv_len, text_start, mo.LEVEL_TAU[3])
    assert_close(from_dev(o), oracle.attention(q, k, v, kv_len, m, block), "last computing step")


def test_first_step_cannot_reuse():
    z = torch.zeros(1, 1, 128, 64, dtype=torch.bfloat16, device="cuda")
    y = torch.zeros(1, 8, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):
        run_action_trace([(1, 0)], z, z, z, z.clone(), 1, 128, 128, 128, y, y.clone(), y.clone())
