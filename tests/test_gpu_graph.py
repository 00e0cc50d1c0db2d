"""The entry points inside a captured HIP graph: a serving loop replays one step's calls without
going through the host again.  Every replay must reproduce the eager result bit for bit, with
other work and synchronisations between the replays, and after the inputs have changed in
place (the plan of the sparse path is rebuilt by its own kernels on every replay)."""
import numpy as np
import pytest
import torch

import paper_2509_22323_amd as ra
import workloads as wl
from gpu_common import from_dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("D,N", [(128, 1152), (64, 8320)])     # one-launch planner / compaction + planner
def test_select_attend_and_cache_in_a_graph(D, N):
    B, H, block, kv_len, text_start = 2, 3, 128, N - 40, N - 256
    nb = N // block
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=77 + D, gain=2.0)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    o_dense, o_sparse = torch.empty_like(dq), torch.empty_like(dq)
    o_static, o_one = torch.empty_like(dq), torch.empty_like(dq)
    ws_one = torch.empty(ra.rapid_attn_joint_select_workspace_bytes(B, H, N, D, block), dtype=torch.uint8, device="cuda")
    mask = torch.zeros(B, H, nb, nb, dtype=torch.uint8, device="cuda")
    sel_ws = torch.empty(ra.rapid_mask_select_workspace_bytes(B, H, N, D, block), dtype=torch.uint8, device="cuda")
    ws = torch.empty(ra.rapid_attn_workspace_bytes(B, H, N, D, block), dtype=torch.uint8, device="cuda")
    delta, out = torch.empty_like(dq), torch.empty_like(dq)
    tau = 0.5                                               # low enough to drop blocks of these near-uniform rows

    def step():
        ra.rapid_attn_dense(dq, dk, dv, o_dense, kv_len)
        ra.rapid_mask_select(dq, dk, mask, block, kv_len, text_start, tau, 0.0, sel_ws)
        ra.rapid_attn_block_sparse(dq, dk, dv, o_sparse, mask, block, kv_len, 0.0, ws)
        # the entry that allocates nothing (its scratch is inside the library) and the one-call form
        ra.rapid_attn_block_sparse_static(dq, dk, dv, o_static, mask, block, kv_len)
        ra.rapid_attn_joint_select([(dq, dk, dv, o_one)], block, kv_len=kv_len, text_start=text_start, tau=tau,
                                   workspace=ws_one)
        ra.rapid_cache_store(o_sparse.view(B, -1), dq.view(B, -1), delta.view(B, -1))
        ra.rapid_cache_reuse(dq.view(B, -1), delta.view(B, -1), out.view(B, -1))

    def results():
        torch.cuda.synchronize()
        return [from_dev(t).copy() for t in (o_dense, o_sparse, delta, out)] + [mask.cpu().numpy().copy()] + \
               [from_dev(t).copy() for t in (o_static, o_one)]

    step()
    eager = results()
    assert 0.05 < eager[4].mean() < 0.999, "the mask should be neither empty nor full on this input"
    np.testing.assert_array_equal(eager[5], eager[1])     # static scratch: same kernels, same plan as the workspace entry
    two, one = (wl.bf16_bits_to_f32(eager[i]).astype(np.float64) for i in (1, 6))
    assert np.abs(one - two).max() <= 2e-2 * max(1.0, np.abs(two).max())   # another planner, so equal to rounding only

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    for replay in range(3):
        for t in (o_dense, o_sparse, delta, out, o_static, o_one):
            t.fill_(float("nan"))
        mask.fill_(7)
        ws.fill_(0xAB)                                     # stale plan, counters and partial results
        ws_one.fill_(0xCD)
        torch.cuda.synchronize()
        graph.replay()
        for got, want in zip(results(), eager):
            np.testing.assert_array_equal(got, want, err_msg=f"replay {replay}")

    # new inputs in the same buffers: the replay must follow them (other mask, other plan)
    q2, k2, v2 = wl.make_qkv(B, H, N, D, kv_len, seed=78 + D, gain=2.0)
    dq.copy_(to_dev(q2)); dk.copy_(to_dev(k2)); dv.copy_(to_dev(v2))
    step()
    eager2 = results()
    assert (eager2[4] != eager[4]).any()
    for t in (o_dense, o_sparse, delta, out, o_static, o_one):
        t.fill_(float("nan"))
    graph.replay()
    for got, want in zip(results(), eager2):
        np.testing.assert_array_equal(got, want, err_msg="replay on new inputs")
