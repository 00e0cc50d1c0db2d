"""Host-only checks of the C ABI: the library loads without a GPU, exports every
symbol the header declares, and every argument error is reported before any launch."""
import ctypes
import os
import re

import pytest

import paper_2509_22323_amd as ra
from paper_2509_22323_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "rapid_attn.h")).read()


def declared_symbols():
    return re.findall(r"RAPID_API\s+[\w\s\*]+?\b(rapid_attn_\w+)\s*\(", HEADER)


def test_header_declares_the_expected_entry_points():
    assert set(declared_symbols()) == set(binding.EXPORTS)


def test_library_exports_every_declared_symbol():
    ra.library()                                  # brings in the HIP runtime it binds to
    lib = ctypes.CDLL(ra.library_path())
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_version_and_status_strings():
    assert ra.rapid_attn_version() == int(re.search(r"#define RAPID_ATTN_VERSION (\d+)", HEADER).group(1))
    for name, code in ra.STATUS.items():
        assert re.search(rf"{name}\s*=\s*{code}\b", HEADER), name
        assert ra.rapid_attn_status_string(code) not in ("", "unknown status")
    assert ra.rapid_attn_status_string(12345) == "unknown status"


def test_workspace_bytes():
    f = ra.rapid_attn_workspace_bytes
    nb = 36
    rows = 24 * nb
    need = f(1, 24, 4608, 128, 128)
    assert need >= rows * 4 * 2 + rows * nb * 4 and need % 256 == 0
    assert f(8, 24, 4480, 64, 128) > f(1, 24, 4480, 64, 128)
    assert f(1, 2, 256, 64, 64) > 0
    for bad in [(0, 1, 128, 64, 64), (1, 0, 128, 64, 64), (1, 1, 0, 64, 64), (1, 1, 128, 32, 64),
                (1, 1, 128, 64, 32), (1, 1, 192, 64, 128), (1, 1, 128, 64, 0)]:
        assert f(*bad) == 0, bad


A = 0x10000          # fake, 16-byte aligned "device" addresses: never dereferenced,
WS = 0x7000000       # every call below must fail validation before any launch


def dense(q=A, k=A + 0x100000, v=A + 0x200000, o=A + 0x300000, B=1, H=2, N=256, D=64,
          kv_len=256, scale=0.0):
    return ra.library().rapid_attn_dense(q, k, v, o, B, H, N, D, kv_len, scale, None, 0, None)


def sparse(q=A, k=A + 0x100000, v=A + 0x200000, o=A + 0x300000, B=1, H=2, N=256, D=64, block=64,
           mask=A + 0x400000, kv_len=256, scale=0.0, ws=WS, ws_bytes=1 << 20):
    return ra.library().rapid_attn_block_sparse(q, k, v, o, B, H, N, D, block, mask, kv_len, scale,
                                                ws, ws_bytes, None)


S = ra.STATUS


@pytest.mark.parametrize("kw,code", [
    (dict(q=None), "RAPID_ERR_NULL"), (dict(k=None), "RAPID_ERR_NULL"),
    (dict(v=None), "RAPID_ERR_NULL"), (dict(o=None), "RAPID_ERR_NULL"),
    (dict(B=0), "RAPID_ERR_SHAPE"), (dict(H=-1), "RAPID_ERR_SHAPE"), (dict(N=0), "RAPID_ERR_SHAPE"),
    (dict(kv_len=0), "RAPID_ERR_SHAPE"), (dict(kv_len=257), "RAPID_ERR_SHAPE"),
    (dict(D=96), "RAPID_ERR_UNSUPPORTED"), (dict(D=256), "RAPID_ERR_UNSUPPORTED"),
    (dict(q=A + 8), "RAPID_ERR_ALIGN"), (dict(o=A + 0x300002), "RAPID_ERR_ALIGN"),
])
def test_dense_argument_errors(kw, code):
    assert dense(**kw) == S[code]


@pytest.mark.parametrize("kw,code", [
    (dict(mask=None), "RAPID_ERR_NULL"), (dict(v=None), "RAPID_ERR_NULL"),
    (dict(B=0), "RAPID_ERR_SHAPE"), (dict(kv_len=300), "RAPID_ERR_SHAPE"),
    (dict(N=320, kv_len=300, block=128), "RAPID_ERR_SHAPE"),
    (dict(block=32), "RAPID_ERR_UNSUPPORTED"), (dict(block=256), "RAPID_ERR_UNSUPPORTED"),
    (dict(D=80), "RAPID_ERR_UNSUPPORTED"),
    (dict(k=A + 0x100004), "RAPID_ERR_ALIGN"), (dict(ws=WS + 4), "RAPID_ERR_ALIGN"),
    (dict(ws=None), "RAPID_ERR_WORKSPACE"), (dict(ws_bytes=0), "RAPID_ERR_WORKSPACE"),
    (dict(ws_bytes=ra.rapid_attn_workspace_bytes(1, 2, 256, 64, 64) - 1), "RAPID_ERR_WORKSPACE"),
])
def test_sparse_argument_errors(kw, code):
    assert sparse(**kw) == S[code]


def test_output_must_not_overlap_an_input():
    size = 1 * 2 * 256 * 64 * 2
    assert dense(o=A) == S["RAPID_ERR_ALIAS"]                          # o is q
    assert dense(o=A + 0x100000 + size - 16) == S["RAPID_ERR_ALIAS"]    # o starts in k's last row
    assert dense(o=A + 0x200000 - size + 16) == S["RAPID_ERR_ALIAS"]    # o ends in v's first row
    assert sparse(o=A + 0x200000) == S["RAPID_ERR_ALIAS"]
    assert dense(o=A + 0x100000 + size, kv_len=0) == S["RAPID_ERR_SHAPE"]   # adjacent is fine (fails later, on kv_len)


def test_documented_size_limits():
    assert dense(N=(1 << 22) + 64, kv_len=64) == S["RAPID_ERR_SHAPE"]
    assert dense(B=1024, H=512) == S["RAPID_ERR_SHAPE"]                 # B*H = 524288
    assert re.search(r"2\^22", HEADER) and "524287" in HEADER


def static(q=A, k=A + 0x100000, v=A + 0x200000, o=A + 0x300000, B=1, H=2, N=256, D=64, block=64,
           mask=A + 0x400000, kv_len=256):
    return ra.library().rapid_attn_block_sparse_static(q, k, v, o, B, H, N, D, block, mask, kv_len, 0.0, None)


@pytest.mark.parametrize("kw,code", [
    (dict(mask=None), "RAPID_ERR_NULL"), (dict(q=None), "RAPID_ERR_NULL"),
    (dict(H=0), "RAPID_ERR_SHAPE"), (dict(N=320, kv_len=300, block=128), "RAPID_ERR_SHAPE"),
    (dict(block=96), "RAPID_ERR_UNSUPPORTED"), (dict(D=32), "RAPID_ERR_UNSUPPORTED"),
    (dict(v=A + 0x200008), "RAPID_ERR_ALIGN"), (dict(o=A), "RAPID_ERR_ALIAS"),
    # the kept-block lists alone (B*H*nb*nb*4 bytes = 512 MiB) exceed the fixed array
    (dict(B=64, H=32, N=16384, kv_len=16384, q=1 << 40, k=2 << 40, v=3 << 40, o=4 << 40), "RAPID_ERR_WORKSPACE"),
])
def test_static_scratch_entry_argument_errors(kw, code):
    assert static(**kw) == S[code]
    limit = int(re.search(r"#define RAPID_ATTN_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", HEADER).group(1)) << 20
    assert limit == ra.STATIC_SCRATCH_BYTES


def test_binding_rejects_non_tensors_and_raises_on_status():
    with pytest.raises(TypeError):
        ra.rapid_attn_dense(1, 2, 3, 4)
    err = ra.RapidAttnError(-2, ra.rapid_attn_status_string(-2))
    assert err.status == -2 and "shape" in str(err)


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2509_22323_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    orc = open(os.path.join(ROOT, "oracle", "__init__.py")).read()
    assert "paper_2509_22323_amd" not in orc


# ---------------------------------------------------------------- rapid_attn_joint
def seg(n=256, q=A, k=A + 0x100000, v=A + 0x200000, o=A + 0x300000, H=2, D=64, **over):
    g = binding.Segment()
    g.q, g.k, g.v, g.o, g.n = q, k, v, o, n
    g.in_stride_b, g.in_stride_h, g.in_stride_n = n * H * D, D, H * D
    g.out_stride_b, g.out_stride_h, g.out_stride_n = n * H * D, D, H * D
    for name, val in over.items():
        setattr(g, name, val)
    return g


def joint(segs, B=1, H=2, D=64, block=128, mask=None, kv_len=0, ws=None, ws_bytes=0):
    arr = (binding.Segment * max(len(segs), 1))(*segs)
    return ra.library().rapid_attn_joint(arr if segs else None, len(segs), B, H, D, block, mask, kv_len, None, 0.0,
                                         ws, ws_bytes, None)


def test_joint_argument_errors_come_before_any_launch():
    S = ra.STATUS
    assert joint([]) == S["RAPID_ERR_NULL"]
    assert joint([seg(), seg(), seg()]) == S["RAPID_ERR_SHAPE"]
    assert joint([seg(q=None)]) == S["RAPID_ERR_NULL"]
    assert joint([seg(n=0)]) == S["RAPID_ERR_SHAPE"]
    assert joint([seg(q=A + 8)]) == S["RAPID_ERR_ALIGN"]
    assert joint([seg(in_stride_n=2 * 64 + 4)]) == S["RAPID_ERR_ALIGN"]      # rows off the 16-byte grid
    assert joint([seg(in_stride_n=32)]) == S["RAPID_ERR_SHAPE"]              # rows overlap
    assert joint([seg(out_stride_n=1 << 24)]) == S["RAPID_ERR_SHAPE"]
    assert joint([seg()], D=96) == S["RAPID_ERR_UNSUPPORTED"]
    assert joint([seg()], block=32, mask=A) == S["RAPID_ERR_UNSUPPORTED"]
    assert joint([seg()], kv_len=257) == S["RAPID_ERR_SHAPE"]
    assert joint([seg(n=200), seg(n=77)]) == S["RAPID_ERR_SHAPE"]            # first segment not a multiple of 128
    assert joint([seg(n=256), seg(n=77, in_stride_n=3 * 2 * 64)]) == S["RAPID_ERR_SHAPE"]   # token strides differ
    assert joint([seg(n=256), seg(n=77)], mask=A, ws=None) == S["RAPID_ERR_WORKSPACE"]
    # strides of dimensions of size 1 address nothing and are not looked at: with B = 1, H = 1 and a
    # one-token second segment, values that are refused elsewhere get as far as the workspace check
    odd = dict(in_stride_b=3, out_stride_b=5, in_stride_h=7, out_stride_h=9)
    assert joint([seg(n=256, H=1, **odd), seg(n=1, H=1, in_stride_n=17, out_stride_n=19, **odd)], H=1, mask=A,
                 ws=None) == S["RAPID_ERR_WORKSPACE"]
    assert joint([seg(n=256, **odd)], B=2, H=2, mask=A, ws=None) == S["RAPID_ERR_ALIGN"]
    assert joint([seg(n=256), seg(n=2, in_stride_n=17)], mask=A, ws=None) == S["RAPID_ERR_ALIGN"]
    need = ra.rapid_attn_joint_workspace_bytes(1, 2, 333, 64, 128)
    assert need > 0 and need == ra.rapid_attn_joint_workspace_bytes(1, 2, 384, 64, 128)
    assert need == ra.rapid_attn_workspace_bytes(1, 2, 384, 64, 128)
    assert joint([seg(n=256), seg(n=77)], mask=A, ws=WS, ws_bytes=need - 1) == S["RAPID_ERR_WORKSPACE"]
    assert ra.rapid_attn_joint_workspace_bytes(1, 2, 0, 64, 128) == 0
