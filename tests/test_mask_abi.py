"""Host-only checks of the mask-selection part of the C ABI."""
import ctypes
import math
import os
import re

import paper_2509_22323_amd as ra
from oracle import mask_oracle as mo
from paper_2509_22323_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "rapid_mask.h")).read()
A, M, WS = 0x10000, 0x500000, 0x7000000       # fake aligned "device" addresses: never dereferenced


def call(q=A, k=A + 0x100000, B=1, H=2, N=256, D=64, block=64, kv_len=256, text_start=256, tau=0.9, scale=0.0,
         mask=M, ws=WS, ws_bytes=1 << 30):
    return ra.library().rapid_mask_select(q, k, B, H, N, D, block, kv_len, text_start, tau, scale, mask, ws, ws_bytes, None)


def test_header_and_library_agree():
    declared = re.findall(r"RAPID_API\s+[\w\s\*]+?\b(rapid_\w+)\s*\(", HEADER)
    assert set(declared) == set(binding.MASK_EXPORTS)
    ra.library()
    lib = ctypes.CDLL(ra.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_argument_errors_come_before_any_launch():
    S = ra.STATUS
    assert call(q=None) == S["RAPID_ERR_NULL"] and call(k=None) == S["RAPID_ERR_NULL"] and call(mask=None) == S["RAPID_ERR_NULL"]
    for bad in (dict(B=0), dict(H=0), dict(N=0), dict(kv_len=0), dict(kv_len=257), dict(text_start=-1),
                dict(tau=0.0), dict(tau=-1.0), dict(tau=float("nan")), dict(N=320, kv_len=300, block=128)):
        assert call(**bad) == S["RAPID_ERR_SHAPE"], bad
    for bad in (dict(D=96), dict(block=32), dict(N=64 * 2049, kv_len=64, block=64)):
        assert call(**bad) == S["RAPID_ERR_UNSUPPORTED"], bad
    assert call(q=A + 2) == S["RAPID_ERR_ALIGN"] and call(ws=WS + 4) == S["RAPID_ERR_ALIGN"]
    need = ra.rapid_mask_select_workspace_bytes(1, 2, 256, 64, 64)
    assert need == 2 * 1 * 2 * 4 * 64 * 4
    assert call(ws=None) == S["RAPID_ERR_WORKSPACE"] and call(ws_bytes=need - 1) == S["RAPID_ERR_WORKSPACE"]
    assert ra.rapid_mask_select_workspace_bytes(1, 2, 250, 64, 64) == 0


def test_default_levels_are_nested_and_match_the_oracle_table():
    taus = [ra.rapid_mask_level_tau(a) for a in range(4)]
    assert taus[0] == 1.0 and taus == sorted(taus, reverse=True) and len(set(taus)) == 4
    assert all(abs(t - w) < 1e-7 for t, w in zip(taus, mo.LEVEL_TAU))
    assert math.isnan(ra.rapid_mask_level_tau(4)) and math.isnan(ra.rapid_mask_level_tau(-1))


def seg(n=256, q=A, k=A + 0x100000, H=2, D=64, **over):
    g = binding.Segment()
    g.q, g.k, g.v, g.o, g.n = q, k, None, None, n
    g.in_stride_b, g.in_stride_h, g.in_stride_n = n * H * D, D, H * D
    for name, val in over.items():
        setattr(g, name, val)
    return g


def joint(segs, B=1, H=2, D=64, block=128, kv_len=0, text_start=256, tau=0.9, mask=M, ws=WS, ws_bytes=1 << 30):
    arr = (binding.Segment * max(len(segs), 1))(*segs)
    return ra.library().rapid_mask_select_joint(arr if segs else None, len(segs), B, H, D, block, kv_len, None,
                                                text_start, tau, 0.0, mask, ws, ws_bytes, None)


def test_joint_selection_argument_errors_come_before_any_launch():
    S = ra.STATUS
    assert joint([]) == S["RAPID_ERR_NULL"] and joint([seg()], mask=None) == S["RAPID_ERR_NULL"]
    assert joint([seg(q=None)]) == S["RAPID_ERR_NULL"] and joint([seg(k=None)]) == S["RAPID_ERR_NULL"]
    assert joint([seg(), seg(), seg()]) == S["RAPID_ERR_SHAPE"]
    assert joint([seg(n=0)]) == S["RAPID_ERR_SHAPE"] and joint([seg()], kv_len=257) == S["RAPID_ERR_SHAPE"]
    assert joint([seg()], tau=0.0) == S["RAPID_ERR_SHAPE"] and joint([seg()], text_start=-1) == S["RAPID_ERR_SHAPE"]
    assert joint([seg(n=200), seg(n=77)]) == S["RAPID_ERR_SHAPE"]             # first segment not a multiple of 128
    assert joint([seg(n=256), seg(n=77, in_stride_n=3 * 2 * 64)]) == S["RAPID_ERR_SHAPE"]
    assert joint([seg(in_stride_n=32)]) == S["RAPID_ERR_SHAPE"]
    assert joint([seg(q=A + 8)]) == S["RAPID_ERR_ALIGN"] and joint([seg(in_stride_n=2 * 64 + 4)]) == S["RAPID_ERR_ALIGN"]
    assert joint([seg()], D=96) == S["RAPID_ERR_UNSUPPORTED"] and joint([seg()], block=32) == S["RAPID_ERR_UNSUPPORTED"]
    need = ra.rapid_mask_select_joint_workspace_bytes(1, 2, 333, 64, 128)
    assert need == ra.rapid_mask_select_workspace_bytes(1, 2, 384, 64, 128) > 0
    assert joint([seg(n=256), seg(n=77)], ws=None) == S["RAPID_ERR_WORKSPACE"]
    assert joint([seg(n=256), seg(n=77)], ws_bytes=need - 1) == S["RAPID_ERR_WORKSPACE"]
    assert ra.rapid_mask_select_joint_workspace_bytes(1, 2, 0, 64, 128) == 0


def test_select_and_attend_argument_errors_come_before_any_launch():
    S = ra.STATUS

    def full(n=256, **over):
        g = seg(n=n, **over)
        g.v, g.o = g.v or A + 0x200000, g.o or A + 0x300000
        g.out_stride_b, g.out_stride_h, g.out_stride_n = n * 2 * 64, 64, 2 * 64
        return g

    def one(segs, B=1, H=2, D=64, block=128, kv_len=0, text_start=256, tau=0.9, ws=WS, ws_bytes=1 << 30):
        arr = (binding.Segment * max(len(segs), 1))(*segs)
        return ra.library().rapid_attn_joint_select(arr if segs else None, len(segs), B, H, D, block, kv_len, None,
                                                    text_start, tau, 0.0, None, ws, ws_bytes, None)

    assert one([]) == S["RAPID_ERR_NULL"]
    g = full(); g.v = None
    assert one([g]) == S["RAPID_ERR_NULL"]                                   # v is needed here
    assert one([full()], tau=0.0) == S["RAPID_ERR_SHAPE"] and one([full()], kv_len=300) == S["RAPID_ERR_SHAPE"]
    assert one([full()], block=32) == S["RAPID_ERR_UNSUPPORTED"] and one([full()], D=96) == S["RAPID_ERR_UNSUPPORTED"]
    assert one([full(n=200), full(n=77)]) == S["RAPID_ERR_SHAPE"]
    need = ra.rapid_attn_joint_select_workspace_bytes(1, 2, 256, 64, 128)
    assert need == ra.rapid_attn_joint_workspace_bytes(1, 2, 256, 64, 128) + ra.rapid_mask_select_joint_workspace_bytes(1, 2, 256, 64, 128)
    assert one([full()], ws=None) == S["RAPID_ERR_WORKSPACE"] and one([full()], ws_bytes=need - 1) == S["RAPID_ERR_WORKSPACE"]
    assert one([full()], ws=WS + 4) == S["RAPID_ERR_ALIGN"]
    assert ra.rapid_attn_joint_select_workspace_bytes(1, 2, 0, 64, 128) == 0
