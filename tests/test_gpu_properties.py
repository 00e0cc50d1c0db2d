"""GPU property tests: invariants that hold at any size, checked through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import assert_close, from_dev, to_dev, widen
from test_gpu_parity import run_dense, run_sparse

pytestmark = pytest.mark.gpu


def test_unit_values_give_unit_rows():
    B, H, N, D, block, kv_len = 1, 2, 512, 64, 64, 470
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=201)
    v[:] = wl.BF16_ONE
    mask = wl.mask_bernoulli_diag(B, H, N // block, 0.5, 3)
    o = widen(run_sparse(q, k, v, mask, block, kv_len))
    assert np.abs(o[:, :, :kv_len] - 1.0).max() <= 2 ** -7      # one bf16 ulp at 1.0
    assert (o[:, :, kv_len:] == 0).all()


def test_masked_and_padded_kv_are_never_read_into_the_result():
    B, H, N, D, block, kv_len = 2, 2, 640, 128, 128, 600
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=202)
    mask = wl.mask_bernoulli_diag(B, H, N // block, 0.5, 4)
    mask[:, :, :, 1] = 0
    mask[:, :, 1, 1] = 1
    base = run_sparse(q, k, v, mask, block, kv_len)
    m2 = mask.copy()
    m2[:, :, 1, 1] = 0                                       # block 1 now unused by everyone
    base2 = run_sparse(q, k, v, m2, block, kv_len)
    for poison in (wl.BF16_NAN, wl.BF16_INF, 0x4700):
        k2, v2 = k.copy(), v.copy()
        k2[:, :, 128:256], v2[:, :, 128:256] = poison, poison
        k2[:, :, kv_len:], v2[:, :, kv_len:] = poison, poison
        np.testing.assert_array_equal(run_sparse(q, k2, v2, m2, block, kv_len), base2)
    # padding poison alone leaves the first result bit-identical too
    k3, v3, q3 = k.copy(), v.copy(), q.copy()
    k3[:, :, kv_len:], v3[:, :, kv_len:], q3[:, :, kv_len:] = wl.BF16_NAN, wl.BF16_INF, wl.BF16_NAN
    np.testing.assert_array_equal(run_sparse(q3, k3, v3, mask, block, kv_len), base)
    np.testing.assert_array_equal(run_dense(q3, k3, v3, kv_len), run_dense(q, k, v, kv_len))


def test_single_allowed_key_is_exact():
    B, H, N, D = 1, 2, 128, 64
    q, k, v = wl.make_qkv(B, H, N, D, seed=203)
    got = run_dense(q, k, v, 1)
    np.testing.assert_array_equal(got[:, :, 0], v[:, :, 0])
    assert (got[:, :, 1:] == 0).all()


def test_rows_without_kept_keys_are_zero():
    B, H, N, D, block = 1, 2, 256, 64, 64
    q, k, v = wl.make_qkv(B, H, N, D, seed=204)
    mask = np.ones((B, H, 4, 4), np.uint8)
    mask[:, :, 1, :] = 0
    mask[0, 1, 3, :] = [0, 0, 0, 1]
    got = run_sparse(q, k, v, mask, block, 190)              # block 3 starts at 192: all padding
    assert (got[:, :, 64:128] == 0).all()
    assert (got[0, 1, 190:] == 0).all()
    assert_close(got, oracle.attention(q, k, v, 190, mask, block), "empty rows")


def test_deterministic_and_batch_invariant():
    B, H, N, D, block, kv_len = 2, 2, 512, 128, 128, 480
    q, k, v = wl.make_qkv(1, H, N, D, kv_len, seed=205)
    q, k, v = (np.concatenate([x, x]) for x in (q, k, v))   # a CFG pair sharing one action
    m1 = wl.mask_bernoulli_diag(1, H, N // block, 0.5, 5)
    mask = np.concatenate([m1, m1])
    a = run_sparse(q, k, v, mask, block, kv_len)
    b = run_sparse(q, k, v, mask, block, kv_len)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(a[0], a[1])
    # another sample's inputs do not leak in
    q2 = q.copy()
    q2[1] = wl.make_qkv(1, H, N, D, kv_len, seed=206)[0][0]
    c = run_sparse(q2, k, v, mask, block, kv_len)
    np.testing.assert_array_equal(c[0], a[0])
    assert not np.array_equal(c[1], a[1])


def test_all_ones_mask_equals_dense():
    """Action 0 and an all-ones mask are the same function; the two entry points sum the
    keys in a different order, so they agree to rounding, not bit for bit."""
    for (N, D, block, kv_len) in [(512, 64, 64, 450), (512, 128, 128, 512), (384, 64, 128, 300)]:
        q, k, v = wl.make_qkv(1, 2, N, D, kv_len, seed=207)
        ones = np.ones((1, 2, N // block, N // block), np.uint8)
        a, b = run_sparse(q, k, v, ones, block, kv_len), run_dense(q, k, v, kv_len)
        assert_close(a, widen(b), "all-ones vs dense")
        assert np.abs(widen(a) - widen(b)).max() <= 2 ** -8          # a bf16 ulp or two at |O| < 1


def test_runs_on_a_side_stream_without_sync_inside():
    B, H, N, D = 1, 2, 256, 64
    q, k, v = wl.make_qkv(B, H, N, D, seed=208)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    o = torch.zeros_like(dq)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        ra.rapid_attn_dense(dq, dk, dv, o)
    s.synchronize()
    assert_close(from_dev(o), oracle.attention(q, k, v), "side stream")


def test_two_streams_with_their_own_workspaces():
    """Sparse calls of two different problems issued alternately on two streams (default
    priority), each with its own workspace: kernels of the two overlap on the chip, results are
    bit-identical to the same calls made one after the other.  Both masks have rows long enough
    to be cut into pieces, so partial results and piece counters of the two are live together."""
    probs = []
    for (H, N, D, seed) in [(24, 2304, 64, 231), (16, 2048, 128, 232)]:
        q, k, v = wl.make_qkv(1, H, N, D, N - 40, seed=seed)
        nb = N // 128
        mask = wl.mask_bernoulli_diag(1, H, nb, 0.3, seed)
        mask[:, :, nb - 2:, :] = 1                                   # two full rows per head
        dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
        dm = torch.from_numpy(mask).cuda()
        ws = torch.empty(ra.rapid_attn_workspace_bytes(1, H, N, D, 128), dtype=torch.uint8, device="cuda")
        o = torch.full_like(dq, float("nan"))
        ra.rapid_attn_block_sparse(dq, dk, dv, o, dm, 128, N - 40, 0.0, ws)
        torch.cuda.synchronize()
        probs.append(dict(q=dq, k=dk, v=dv, m=dm, ws=ws, kv=N - 40, want=from_dev(o), o=torch.empty_like(dq),
                          stream=torch.cuda.Stream()))
        assert_close(probs[-1]["want"], oracle.attention(q, k, v, N - 40, mask, 128), "reference call")
    for p in probs:
        p["stream"].wait_stream(torch.cuda.current_stream())
    for rep in range(12):
        for p in probs:
            with torch.cuda.stream(p["stream"]):
                if rep == 11:
                    p["o"].fill_(float("nan"))
                ra.rapid_attn_block_sparse(p["q"], p["k"], p["v"], p["o"], p["m"], 128, p["kv"], 0.0, p["ws"])
    for p in probs:
        p["stream"].synchronize()
        np.testing.assert_array_equal(from_dev(p["o"]), p["want"])


def test_status_errors_raise_from_the_binding():
    q = torch.zeros(1, 1, 128, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ra.RapidAttnError) as e:
        ra.rapid_attn_dense(q, q.clone(), q.clone(), q.clone(), kv_len=129)
    assert e.value.status == ra.STATUS["RAPID_ERR_SHAPE"]
    q32 = torch.zeros(1, 1, 128, 32, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ra.RapidAttnError) as e:
        ra.rapid_attn_dense(q32, q32.clone(), q32.clone(), q32.clone())
    assert e.value.status == ra.STATUS["RAPID_ERR_UNSUPPORTED"]
