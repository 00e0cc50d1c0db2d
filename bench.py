#!/usr/bin/env python3
"""Bench of the MM-DiT joint-attention hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload flux_1024]

A step is one attention call of one DiT layer at the FLUX-like 1024^2 shape
(B=1, H=24, N=4608, D=128, bf16): the dense entry point (Sparse-Attention action 0),
the shape the headline metric is quoted on.  Inputs are synthetic (i.i.d. N(0,1)
rounded to bf16), resident in HBM before the timed region (which is preceded by --ramp-ms
of the same calls, so that the GPU clock has come up from idle, and by the W warm-up
steps).  The same run then times
the block-sparse entry point (mask compaction + attention) at each density of the
workload and reports time / (effective density x dense time), and times the fp64
CPU oracle on a bounded sample of rows of the same workload.

Prints ONE JSON line:
  value      effective TFLOP/s = 4 B H kv_len^2 D density / time  (density 1 for dense)
  roofline   dominant kernel (the attention kernel) against the bf16 MFMA peak, from
             HIP-event durations of each launch on the launch stream
  cpu_baseline  the oracle, as it stands, on this machine's host cores
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak (published, no sparsity)


def source_digest():
    """sha256 of the attention kernels' source: a counter summary under profiles/ names the
    source it was taken from."""
    import hashlib
    path = os.path.join(ROOT, "paper_2509_22323_amd", "csrc", "rapid_attn.hip")
    return hashlib.sha256(open(path, "rb").read()).hexdigest()


def measured_traffic(workload, D):
    """HBM bytes per launch of the dense kernel, from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE runs scaled by a plain copy).  The counters cannot be read from
    inside this process, so the figure comes from a file: it is reported with the file's name and
    only if the file says it was taken from the kernel source that is being run now."""
    name = f"attn_dense_pp_kernel_{workload}.txt"
    info = {"file": f"profiles/{name}", "kernel_source_sha256": None, "matches_source_in_tree": False}
    traffic = None
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                traffic = int(line.split("=", 1)[1])
            if line.startswith("KERNEL_SOURCE_SHA256="):
                info["kernel_source_sha256"] = line.split("=", 1)[1].strip()
    except OSError:
        return None, {"file": None}
    info["matches_source_in_tree"] = info["kernel_source_sha256"] == source_digest()
    return (traffic if info["matches_source_in_tree"] else None), info


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--ramp-ms", type=float, default=150.0,
                    help="before the warm-up steps, keep the GPU under the same load for this long: after "
                         "idling, its clock takes some tens of milliseconds to come up (the first ~100 "
                         "calls run ~13 %% slower)")
    ap.add_argument("--leg-ramp-ms", type=float, default=40.0,
                    help="the same before every further timed leg (sparse densities, joint layout, other workloads)")
    ap.add_argument("--workload", default="flux_1024")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sparse", action="store_true")
    ap.add_argument("--no-mfma-probe", action="store_true")
    ap.add_argument("--no-cache-ops", action="store_true")
    ap.add_argument("--no-joint", action="store_true")
    ap.add_argument("--no-mask-select", action="store_true")
    ap.add_argument("--no-trace", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-config table (all five workloads)")
    ap.add_argument("--only-attention", action="store_true",
                    help="time the dense call and the sparse densities of --workload and nothing else "
                         "(what the per-kernel profiles under profiles/ are taken from)")
    ap.add_argument("--only-cache-case", type=int, default=None,
                    help="time only the Cache-Reuse kernels on tensor case 0, 1 or 2 (latent / one layer / 8 layers) "
                         "and nothing else besides the headline leg (for per-size profiles)")
    ap.add_argument("--only-mask-select", action="store_true",
                    help="time only the mask selection besides the headline leg (for its profile)")
    ap.add_argument("--density", default=None,
                    help="with --only-attention: time only this nominal density of the sparse entry point")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of the Q tensor (known size) so that HBM "
                         "counters collected around this process can be scaled")
    return ap.parse_args()


def main():
    args = parse()
    if args.only_attention:
        args.no_cpu_baseline = args.no_mfma_probe = args.no_cache_ops = args.no_joint = True
        args.no_mask_select = args.no_trace = args.no_configs = True
    if args.only_cache_case is not None or args.only_mask_select:
        args.no_cpu_baseline = args.no_mfma_probe = args.no_joint = args.no_sparse = True
        args.no_trace = args.no_configs = True
        args.no_cache_ops = args.only_cache_case is None
        args.no_mask_select = not args.only_mask_select
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2509_22323_amd as ra
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    ra.library()                                   # fail loudly if the HIP library is missing

    w = wl.WORKLOADS[args.workload]
    q, k, v = w.qkv()

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    dq, dk, dv = dev(q), dev(k), dev(v)
    do = torch.empty_like(dq)
    ws = torch.empty(ra.rapid_attn_workspace_bytes(w.B, w.H, w.N, w.D, w.block), dtype=torch.uint8,
                     device="cuda")
    dense_flops = w.dense_flops()

    def time_calls(fn, steps, warmup):
        """(wall ms per step, mean and min HIP-event ms per call) over `steps` calls."""
        for _ in range(warmup):
            fn()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        durs = [a.elapsed_time(b) for a, b in ev]
        return wall, float(np.mean(durs)), float(np.min(durs))

    def ramp(fn, ms):
        """Keep the GPU under the load of `fn` for `ms`: while the host prepares the next input
        the GPU idles and its clock drops; the first ~25 ms of calls after that run ~13 % slower."""
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(8):
                fn()
            torch.cuda.synchronize()

    def time_graph(fn, calls, replays=20):
        """GPU ms per call with the host out of the way: `calls` calls captured in one HIP graph,
        replayed; for calls so short that issuing them from Python takes longer than running them."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()                                   # the library is loaded and warm before capture
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(calls):
                fn()
        ramp(graph.replay, args.leg_ramp_ms)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(replays):
            graph.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / (replays * calls)

    def time_region(fn, steps, warmup, ramp_ms=None):
        """The timed region proper: `steps` calls back to back, nothing else in the stream; wall ms
        per step between synchronisations and HIP-event ms per step over the same region.  Every
        leg is preceded by its own ramp (see ramp)."""
        ramp(fn, args.leg_ramp_ms if ramp_ms is None else ramp_ms)
        for _ in range(warmup):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a.record()
        for _ in range(steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, a.elapsed_time(b) / steps

    # ---- the timed K steps: dense entry point
    dense_call = lambda: ra.rapid_attn_dense(dq, dk, dv, do, w.kv_len)
    t_ramp = time.perf_counter()
    while (time.perf_counter() - t_ramp) * 1e3 < args.ramp_ms:
        for _ in range(20):
            dense_call()
        torch.cuda.synchronize()
    wall_ms, ev_mean = time_region(dense_call, args.steps, args.warmup, ramp_ms=0.0)
    value = dense_flops / (wall_ms * 1e-3) / 1e12
    achieved = dense_flops / (ev_mean * 1e-3) / 1e12
    # one launch at a time between its own pair of events (the events themselves open a gap of a
    # few microseconds between launches, which is why the timed region above has none inside)
    _, _, ev_min = time_calls(dense_call, min(args.steps, 200), 0)

    traffic, traffic_info = measured_traffic(w.name, w.D)
    out = {
        "metric": "effective TFLOP/s (4*B*H*N^2*D*density), dense joint attention",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall_ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} N={w.N} kv_len={w.kv_len} D={w.D} "
                               f"dense (action 0), one layer's attention per step",
                   "flops_per_step": dense_flops, "entry": "rapid_attn_dense"},
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "roofline": {"bound": "mfma", "kernel": f"attn_dense_pp_kernel<{w.D}>", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_source": traffic_info,
                     "algorithmic_bytes": 4 * dq.numel() * 2,
                     "launch_ms_mean": round(ev_mean, 5), "launch_ms_min": round(ev_min, 5)},
    }

    # ---- what the matrix pipe alone sustains on this machine (context for the roofline fraction):
    # an MFMA-only loop, once on constant operands and once on this workload's kind of data.
    # The published peak assumes the nominal clock; random bf16 operands throttle it.
    if not args.no_mfma_probe:
        import ctypes
        probe = ctypes.CDLL(os.path.join(ROOT, "paper_2509_22323_amd", "libmfma_probe.so"))
        probe.rapid_probe_mfma.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                                           ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        # each thread reads 256 bytes of operands: size the grid to the tensor that supplies them
        blocks = int(min(512, dq.numel() * 2 // (256 * 256)))
        iters = 2000
        pout = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        mfma_only = {}
        ones = torch.ones(blocks * 256 * 128, dtype=torch.bfloat16, device="cuda")
        for kind, data in (("constant_operands", ones), ("unit_normal_operands", dq)):
            nbytes = data.numel() * data.element_size()
            run = lambda: probe.rapid_probe_mfma(data.data_ptr(), nbytes, pout.data_ptr(), pout.numel() * 4,
                                                 blocks, iters, stream)
            rc = run()
            if rc != 0:
                raise RuntimeError(f"rapid_probe_mfma refused the launch: {rc}")
            _, p_mean, _ = time_calls(run, 5, 2)
            mfma_only[kind] = round(blocks * 4 * iters * 32 * 32768.0 / (p_mean * 1e-3) / 1e12, 1)
        mfma_only["unit"] = "TFLOP/s"
        out["mfma_only_loop"] = mfma_only

    if args.calibrate_copy:                        # 2 x Q bytes of HBM traffic, for counter calibration
        for _ in range(5):
            do.copy_(dq)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = 2 * dq.numel() * 2

    # ---- block-sparse entry point at the workload's densities (compaction included)
    if not args.no_sparse:
        sparse = []
        for d in w.densities:
            if args.density is not None and str(d) != args.density:
                continue
            mask = w.mask(d)
            eff = wl.effective_density(mask, w.block, w.kv_len)
            dm = torch.from_numpy(mask).cuda()
            _, s_mean = time_region(
                lambda: ra.rapid_attn_block_sparse(dq, dk, dv, do, dm, w.block, w.kv_len, 0.0, ws),
                max(20, min(200, args.steps // 2)), max(5, args.warmup // 2))
            sparse.append({"density_nominal": d, "density_effective": round(eff, 4),
                           "ms": round(s_mean, 5),
                           "eff_tflops": round(dense_flops * eff / (s_mean * 1e-3) / 1e12, 2),
                           "time_over_density_x_dense": round(s_mean / (eff * ev_mean), 3)})
        out["sparse"] = sparse

    # ---- the same dense call on tensors as an MM-DiT block holds them: image and text stream in
    # separate fused-QKV tensors [B, n, 3, H, D], outputs [B, n, H, D] (no concatenated copy)
    n_txt = 512 if w.N > 1024 else 0
    if not args.no_joint and (w.N - n_txt) % 128 == 0:
        segs = []
        for a, b in ((0, w.N - n_txt), (w.N - n_txt, w.N)) if n_txt else ((0, w.N),):
            fused = torch.empty(w.B, b - a, 3, w.H, w.D, dtype=torch.bfloat16, device="cuda")
            for j, x in enumerate((dq, dk, dv)):
                fused[:, :, j] = x[:, :, a:b].permute(0, 2, 1, 3)
            o_seg = torch.empty(w.B, b - a, w.H, w.D, dtype=torch.bfloat16, device="cuda")
            segs.append(tuple(fused[:, :, j].permute(0, 2, 1, 3) for j in range(3)) + (o_seg.permute(0, 2, 1, 3),))
        _, j_mean = time_region(lambda: ra.rapid_attn_joint(segs, None, w.block, kv_len=w.kv_len),
                                max(20, min(200, args.steps // 2)), max(5, args.warmup // 2))
        out["joint_layout"] = {"layout": f"{len(segs)} segment(s), fused [B,n,3,H,D] inputs, [B,n,H,D] outputs",
                               "ms": round(j_mean, 5), "tflops": round(dense_flops / (j_mean * 1e-3) / 1e12, 2),
                               "time_over_contiguous": round(j_mean / ev_mean, 3)}
        del segs

    # ---- block-mask selection for the Sparse-Attention levels (block means -> softmax -> mass cut):
    # streams Q and K once (HBM-bound), then one wavefront per mask row.  Timed by graph replay (the
    # host's issue time is out of the way), twice: on ONE set of Q, K, which the 256 MB memory-side
    # cache then serves, and rotating over enough copies of Q, K that every call reads from HBM.
    if not args.no_mask_select and w.N % w.block == 0 and w.N // w.block <= 2048:
        nbk = w.N // w.block
        sel_mask = torch.empty(w.B, w.H, nbk, nbk, dtype=torch.uint8, device="cuda")
        sel_ws = torch.empty(ra.rapid_mask_select_workspace_bytes(w.B, w.H, w.N, w.D, w.block), dtype=torch.uint8,
                             device="cuda")
        text_start = w.N - 512 if w.N > 1024 else w.N
        read_bytes = 2 * dq.numel() * 2
        n_sets = int(-(-600e6 // read_bytes)) + 1
        qk_sets = [(dq, dk)] + [(dq.clone(), dk.clone()) for _ in range(n_sets - 1)]
        turn = [0]
        levels = []
        bq, bk, _ = w.qkv_block_structured()
        bq, bk = dev(bq), dev(bk)
        for action in (1, 2, 3):
            tau = ra.rapid_mask_level_tau(action)
            sel_call = lambda: ra.rapid_mask_select(dq, dk, sel_mask, w.block, w.kv_len, text_start, tau, 0.0, sel_ws)
            ra.rapid_mask_select(bq, bk, sel_mask, w.block, w.kv_len, text_start, tau, 0.0, sel_ws)
            kept_structured = round(float(sel_mask.float().mean()), 4)

            def sel_rotating():
                i = turn[0] = (turn[0] + 1) % n_sets
                ra.rapid_mask_select(qk_sets[i][0], qk_sets[i][1], sel_mask, w.block, w.kv_len, text_start, tau, 0.0,
                                     sel_ws)

            levels.append({"action": action, "tau": round(tau, 3),
                           "ms": round(time_graph(sel_rotating, 4 * n_sets), 5),
                           "ms_inputs_in_memory_side_cache": round(time_graph(sel_call, 20), 5),
                           "kept_fraction_iid_inputs": round(float(sel_mask.float().mean()), 4),
                           "kept_fraction_block_structured_inputs": kept_structured})
        gbs = read_bytes / (levels[0]["ms"] * 1e-3) / 1e9
        gbs_c = read_bytes / (levels[0]["ms_inputs_in_memory_side_cache"] * 1e-3) / 1e9
        out["mask_select"] = {"levels": levels, "qk_sets_rotated": n_sets,
                              "roofline": {"bound": "hbm", "kernel": "block_mean_kernel (+ select_blocks_kernel in the time)",
                                           "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s",
                                           "frac": round(gbs / 8000.0, 4), "algorithmic_bytes": read_bytes,
                                           "achieved_inputs_in_memory_side_cache": round(gbs_c, 1)}}
        if not args.only_mask_select:
            # one layer of a sparse step on the block-structured inputs: selection + attention as two calls
            # (byte mask in between) and as the one call that writes the kept lists directly
            tau3 = ra.rapid_mask_level_tau(3)
            ws1 = torch.empty(ra.rapid_attn_joint_select_workspace_bytes(w.B, w.H, w.N, w.D, w.block), dtype=torch.uint8,
                              device="cuda")
            one_seg = [(bq, bk, dv, do)]

            def two_calls():
                ra.rapid_mask_select(bq, bk, sel_mask, w.block, w.kv_len, text_start, tau3, 0.0, sel_ws)
                ra.rapid_attn_block_sparse(bq, bk, dv, do, sel_mask, w.block, w.kv_len, 0.0, ws)

            one_call = lambda: ra.rapid_attn_joint_select(one_seg, w.block, kv_len=w.kv_len, text_start=text_start,
                                                          tau=tau3, workspace=ws1)
            _, t2 = time_region(two_calls, 100, 10)
            _, t1 = time_region(one_call, 100, 10)
            out["mask_select"]["select_and_attend_level_3"] = {
                "inputs": "block-structured", "kept_fraction": levels[2]["kept_fraction_block_structured_inputs"],
                "two_calls_ms": round(t2, 5), "one_call_ms": round(t1, 5), "dense_ms": round(ev_mean, 5)}
            del ws1
        del qk_sets, bq, bk

    # ---- a scripted action trace of one image (counts as in the paper's appendix: 12-16 steps, 4-8 of
    # them reuse the cache, 2-4 run sparse attention) played against the library: the attention side
    # of every layer of every computing step, the residual operations, mask selection on the GPU.
    # Twice: on Q, K with a block-structured attention map (the kind of map the selection is for; the
    # sparse steps then prune) and on the i.i.d. tensors of the headline leg (nearly uniform pooled
    # scores: nothing to prune, so a "sparse" step only adds the selection and the plan).
    if not args.no_trace and w.N % w.block == 0 and w.N // w.block <= 2048:
        from paper_2509_22323_amd.sampler import run_action_trace
        n_layers, base_steps = (57, 28) if w.D == 128 else (24, 28)    # FLUX.1 / SD3-medium attention layers
        trace = wl.action_trace(20250922)
        lat = torch.randn(w.B, 4096 * 64, device="cuda").bfloat16()
        dl, oo = torch.zeros_like(lat), torch.randn(w.B, 4096 * 64, device="cuda").bfloat16()
        text_start = w.N - 512 if w.N > 1024 else w.N
        sq, sk, sv = (dev(x) for x in w.qkv_block_structured())
        base_ms = base_steps * n_layers * ev_mean

        def play(tq, tk, tv):
            run_action_trace(trace[:3], tq, tk, tv, do, 2, w.block, w.kv_len, text_start, lat, dl, oo)   # warm
            ramp(dense_call, args.leg_ramp_ms)
            tr = run_action_trace(trace, tq, tk, tv, do, n_layers, w.block, w.kv_len, text_start, lat, dl, oo)
            kinds = [s_["kind"] for s_ in tr.steps]
            mean_ms = lambda pred: float(np.mean([s_["ms"] for s_ in tr.steps if pred(s_["kind"])] or [float("nan")]))
            full_ms = mean_ms(lambda kd: kd == "full")
            sparse_ms = mean_ms(lambda kd: kd.startswith("sparse"))
            kept = {}
            sel_mask = torch.empty(w.B, w.H, w.N // w.block, w.N // w.block, dtype=torch.uint8, device="cuda")
            for action in (1, 2, 3):
                ra.rapid_mask_select(tq, tk, sel_mask, w.block, w.kv_len, text_start, ra.rapid_mask_level_tau(action))
                kept[f"level_{action}"] = round(float(sel_mask.float().mean()), 4)
            return tr, kinds, {
                "attention_ms": round(tr.total_ms, 3), "full_step_ms": round(full_ms, 3),
                "sparse_step_ms": round(sparse_ms, 3), "cached_step_ms": round(mean_ms(lambda kd: kd == "cached"), 4),
                "attention_time_ratio_vs_base_schedule": round(base_ms / tr.total_ms, 3),
                "measured_sparse_step_cost_reduction": round(1.0 - sparse_ms / full_ms, 3),
                "equivalent_steps_measured_attention": round(tr.total_ms / full_ms, 3),
                "kept_fraction_of_selected_masks": kept}

        tr, kinds, structured = play(sq, sk, sv)
        _, _, iid = play(dq, dk, dv)
        cc = [0.95 if kd == "cached" else 0.0 for kd in kinds]
        cs = [{"sparse-1": 0.05, "sparse-2": 0.07, "sparse-3": 0.10}.get(kd, 0.0) for kd in kinds]
        k_exact, k_round = ra.rapid_equivalent_steps(cc, cs)
        out["sampler_trace"] = {
            "layers": n_layers, "steps": len(trace), "cached_steps": kinds.count("cached"),
            "sparse_steps": sum(kd.startswith("sparse") for kd in kinds),
            "base_schedule": f"{base_steps} dense steps", "base_schedule_ms": round(base_ms, 3),
            "equivalent_steps_paper_constants": {"K_exact": round(k_exact, 3), "K": k_round},
            "block_structured_inputs": structured, "iid_inputs": iid,
            "note": "masks selected on the GPU per layer; the same Q, K, V stand in for every layer; quality "
                    "is not measured (no generator)"}
        del sq, sk, sv

    # ---- Cache-Reuse residual operations (O = X + Delta, Delta = G(X) - X): streaming kernels,
    # bound by HBM (6 bytes per element).  Two sizes: the latent of one image at this workload's
    # resolution (launch-latency bound) and one layer's hidden states (joint tokens x 3072 channels).
    if not args.no_cache_ops:
        cache = []
        cases = (("latent of one image: 4096 tokens x 64 channels", 4096 * 64),
                 (f"hidden states of one layer: {w.N} tokens x 3072 channels", w.N * 3072),
                 (f"hidden states of 8 layers: 8 x {w.N} tokens x 3072 channels", 8 * w.N * 3072))
        if args.only_cache_case is not None:
            cases = cases[args.only_cache_case:args.only_cache_case + 1]
        for label, elems in cases:
            # rotate over enough tensor sets to exceed the 256 MB memory-side cache, so that the
            # large case streams from HBM and not from that cache
            sets = max(1, min(8, int(600e6 // (6 * elems))))
            g = torch.Generator(device="cuda")
            g.manual_seed(3)
            xs = [torch.randn(1, elems, device="cuda", generator=g).bfloat16() for _ in range(sets)]
            ds = [torch.randn(1, elems, device="cuda", generator=g).bfloat16() for _ in range(sets)]
            os_ = [torch.empty_like(x) for x in xs]
            turn = [0]

            def reuse():
                i = turn[0] = (turn[0] + 1) % sets
                ra.rapid_cache_reuse(xs[i], ds[i], os_[i])

            def store():
                i = turn[0] = (turn[0] + 1) % sets
                ra.rapid_cache_store(os_[i], xs[i], ds[i])

            # GPU time per call by graph replay (every tensor set visited the same number of times)
            r_mean = time_graph(reuse, 4 * sets)
            s_mean = time_graph(store, 4 * sets)
            gbs = 6.0 * elems / (r_mean * 1e-3) / 1e9
            cache.append({"tensor": label, "elements": elems, "tensor_sets_rotated": sets,
                          "reuse_ms": round(r_mean, 5), "store_ms": round(s_mean, 5),
                          "roofline": {"bound": "hbm", "kernel": "cache_residual_kernel", "achieved": round(gbs, 1),
                                       "peak": 8000.0, "unit": "GB/s", "frac": round(gbs / 8000.0, 4),
                                       "algorithmic_bytes": 6 * elems}})
            del xs, ds, os_
        out["cache_reuse"] = cache

    # ---- all five workloads, dense and at every listed density, in this same process: ms, effective
    # TFLOP/s, fraction of the bf16 MFMA peak, and the sparse time over (effective density x dense
    # time).  The headline workload's entry repeats the figures measured above.  With the cpu_baseline
    # leg on, 128 sampled output rows of every (workload, density) are also checked against the oracle.
    if not args.no_configs:
        if not args.no_cpu_baseline:
            import oracle

        def widen(t):
            return wl.bf16_bits_to_f32(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)

        def config_entry(cw, cq, ck, cv, co, cws, host, dense_ms=None, sparse_done=None):
            flops = cw.dense_flops()
            n_calls = lambda ms: int(max(10, min(400, 60.0 / max(ms, 1e-3))))
            call = lambda: ra.rapid_attn_dense(cq, ck, cv, co, cw.kv_len)
            if dense_ms is None:
                _, rough = time_region(call, 5, 3)
                _, dense_ms = time_region(call, n_calls(rough), 5, ramp_ms=0.0)
            entry = {"workload": cw.name, "B": cw.B, "H": cw.H, "N": cw.N, "kv_len": cw.kv_len, "D": cw.D,
                     "block": cw.block, "dense_gflop": round(flops / 1e9, 2),
                     "dense": {"ms": round(dense_ms, 5), "tflops": round(flops / (dense_ms * 1e-3) / 1e12, 2),
                               "frac_of_bf16_mfma_peak": round(flops / (dense_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
                     "sparse": []}
            rows = None
            if not args.no_cpu_baseline:
                rows = wl.sample_rows(cw.B, cw.H, cw.N, cw.kv_len, cw.block, 128, seed=cw.seed() + 5)
                call()
                got = widen(co)[rows[:, 0], rows[:, 1], rows[:, 2]]
                err = np.abs(got - oracle.attention_rows(host[0], host[1], host[2], rows, cw.kv_len))
                entry["dense"]["oracle_check_128_rows"] = {"max_abs": float(f"{err.max():.3e}"),
                                                           "mean_abs": float(f"{err.mean():.3e}")}
            for d in cw.densities:
                mask = cw.mask(d)
                eff = wl.effective_density(mask, cw.block, cw.kv_len)
                dm = torch.from_numpy(mask).cuda()
                scall = lambda: ra.rapid_attn_block_sparse(cq, ck, cv, co, dm, cw.block, cw.kv_len, 0.0, cws)
                done = None if sparse_done is None else [x for x in sparse_done if x["density_nominal"] == d]
                if done:
                    s_ms = done[0]["ms"]
                else:
                    _, rough = time_region(scall, 5, 3)
                    _, s_ms = time_region(scall, n_calls(rough), 5, ramp_ms=0.0)
                e = {"density_nominal": d, "density_effective": round(eff, 4), "ms": round(s_ms, 5),
                     "eff_tflops": round(flops * eff / (s_ms * 1e-3) / 1e12, 2),
                     "time_over_density_x_dense": round(s_ms / (eff * dense_ms), 3)}
                if rows is not None:
                    scall()
                    got = widen(co)[rows[:, 0], rows[:, 1], rows[:, 2]]
                    err = np.abs(got - oracle.attention_rows(host[0], host[1], host[2], rows, cw.kv_len, mask, cw.block))
                    e["oracle_check_128_rows"] = {"max_abs": float(f"{err.max():.3e}"), "mean_abs": float(f"{err.mean():.3e}")}
                entry["sparse"].append(e)
            return entry

        configs = []
        for name in ("tiny", "sd3_1024", "flux_1024", "grpo_sd3", "flux_2048"):
            cw = wl.WORKLOADS[name]
            if name == w.name:
                configs.append(config_entry(w, dq, dk, dv, do, ws, (q, k, v), dense_ms=ev_mean,
                                            sparse_done=out.get("sparse")))
                continue
            host = cw.qkv()
            cq, ck, cv = (dev(x) for x in host)
            co = torch.empty_like(cq)
            cws = torch.empty(ra.rapid_attn_workspace_bytes(cw.B, cw.H, cw.N, cw.D, cw.block), dtype=torch.uint8,
                              device="cuda")
            configs.append(config_entry(cw, cq, ck, cv, co, cws, host))
            del cq, ck, cv, co, cws, host
        out["configs"] = configs

    # ---- the oracle on this machine's host cores, bounded sample of rows of the same workload
    if not args.no_cpu_baseline:
        import oracle
        rng = np.random.default_rng(1)

        def rows(n):
            return np.stack([rng.integers(w.B, size=n), rng.integers(w.H, size=n),
                             rng.integers(w.kv_len, size=n)], axis=1).astype(np.int32)

        flops_per_row = 4.0 * w.kv_len * w.D
        t0 = time.perf_counter()
        oracle.attention_rows(q, k, v, rows(256), w.kv_len)
        pilot = time.perf_counter() - t0
        n = int(max(256, min(w.B * w.H * w.kv_len, args.cpu_seconds / max(pilot, 1e-6) * 256)))
        t0 = time.perf_counter()
        oracle.attention_rows(q, k, v, rows(n), w.kv_len)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(n * flops_per_row / dt / 1e12, 6), "unit": "TFLOP/s",
                               "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"{n} random output rows of {w.name} dense "
                                         f"({n * flops_per_row / 1e9:.1f} GFLOP fp64) in {dt:.1f} s; "
                                         f"full call would take {dense_flops / (n * flops_per_row) * dt:.0f} s"}

    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
