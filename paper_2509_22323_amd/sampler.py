"""Step-level driver: plays a scripted RAPID^3 action trace against the library.

There is no generator here (that would need trained weights): every denoising step issues what
the ATTENTION side of a DiT would issue under the step's actions (Sec. 3.2 / 3.3: Step-Skip is
the length of the trace; a step that reuses the cache runs no layer at all and outputs
X + Delta; a computing step runs every layer's joint attention, dense for sparse action 0 and
block-sparse under the selected mask for actions 1..3, and then refreshes the cached residual).
The same Q/K/V stand in for every layer.  All work is library calls on torch's current stream;
this module only sequences them and reads HIP events.
"""
from __future__ import annotations

from dataclasses import dataclass, field

from . import binding as _b


@dataclass
class TraceResult:
    steps: list = field(default_factory=list)       # per step: dict(kind, ms)
    total_ms: float = 0.0
    calls: dict = field(default_factory=dict)       # library calls issued, by name


def run_action_trace(trace, q, k, v, o, n_layers, block, kv_len, text_start, x, delta, out, masks=None):
    """Play `trace` (list of (a_cache, a_sparse)).  q, k, v, o: CUDA bf16 [B,H,N,D]; x, delta, out:
    CUDA bf16 [B, elems] (the generator's input, the cached residual, its output).  masks: optional
    dict action -> CUDA uint8 mask to use instead of selecting one on the GPU per layer."""
    import torch
    B, H, N, D = (int(s) for s in q.shape)
    nb = N // block
    res = TraceResult(calls={"rapid_attn_dense": 0, "rapid_attn_block_sparse": 0, "rapid_mask_select": 0,
                             "rapid_cache_reuse": 0, "rapid_cache_store": 0})
    mask = torch.empty(B, H, nb, nb, dtype=torch.uint8, device=q.device)
    ws_attn = torch.empty(max(_b.rapid_attn_workspace_bytes(B, H, N, D, block), 16), dtype=torch.uint8, device=q.device)
    ws_mask = torch.empty(max(_b.rapid_mask_select_workspace_bytes(B, H, N, D, block), 16), dtype=torch.uint8,
                          device=q.device)
    events = []
    for step, (a_cache, a_sparse) in enumerate(trace):
        if step == 0 and a_cache:
            raise ValueError("the first step has no cache to reuse")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if a_cache:
            _b.rapid_cache_reuse(x, delta, out)
            res.calls["rapid_cache_reuse"] += 1
            kind = "cached"
        else:
            for _ in range(n_layers):
                if a_sparse == 0:
                    _b.rapid_attn_dense(q, k, v, o, kv_len)
                    res.calls["rapid_attn_dense"] += 1
                else:
                    if masks is not None:
                        m = masks[a_sparse]
                    else:
                        m = _b.rapid_mask_select(q, k, mask, block, kv_len, text_start,
                                                 _b.rapid_mask_level_tau(a_sparse), 0.0, ws_mask)
                        res.calls["rapid_mask_select"] += 1
                    _b.rapid_attn_block_sparse(q, k, v, o, m, block, kv_len, 0.0, ws_attn)
                    res.calls["rapid_attn_block_sparse"] += 1
            _b.rapid_cache_store(out, x, delta)
            res.calls["rapid_cache_store"] += 1
            kind = "full" if a_sparse == 0 else f"sparse-{a_sparse}"
        e1.record()
        events.append((kind, e0, e1))
    torch.cuda.synchronize()
    for kind, e0, e1 in events:
        ms = e0.elapsed_time(e1)
        res.steps.append({"kind": kind, "ms": ms})
        res.total_ms += ms
    return res
