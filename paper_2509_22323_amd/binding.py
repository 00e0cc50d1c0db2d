"""ctypes binding of librapid_attn.so: same names as the C ABI, marshalling only.

PyTorch is used for device memory and streams, nothing else: tensors are passed as
raw device pointers, kernels go to torch's current HIP stream.  There is no fallback:
if the shared library is missing the first call raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "librapid_attn.so")
_lib = None

STATUS = {
    "RAPID_OK": 0, "RAPID_ERR_NULL": -1, "RAPID_ERR_SHAPE": -2, "RAPID_ERR_UNSUPPORTED": -3,
    "RAPID_ERR_ALIGN": -4, "RAPID_ERR_WORKSPACE": -5, "RAPID_ERR_DEVICE": -6, "RAPID_ERR_ALIAS": -7,
}

EXPORTS = ("rapid_attn_dense", "rapid_attn_block_sparse", "rapid_attn_block_sparse_static",
           "rapid_attn_workspace_bytes",
           "rapid_attn_joint", "rapid_attn_joint_workspace_bytes",
           "rapid_attn_status_string", "rapid_attn_version")


class Segment(ctypes.Structure):
    """rapid_attn_segment of include/rapid_attn.h."""
    _fields_ = [("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("o", ctypes.c_void_p),
                ("n", ctypes.c_int),
                ("in_stride_b", ctypes.c_longlong), ("in_stride_h", ctypes.c_longlong), ("in_stride_n", ctypes.c_longlong),
                ("out_stride_b", ctypes.c_longlong), ("out_stride_h", ctypes.c_longlong),
                ("out_stride_n", ctypes.c_longlong)]
MASK_EXPORTS = ("rapid_mask_select", "rapid_mask_select_workspace_bytes", "rapid_mask_select_joint",
                "rapid_mask_select_joint_workspace_bytes", "rapid_attn_joint_select",
                "rapid_attn_joint_select_workspace_bytes", "rapid_mask_level_tau")
CACHE_EXPORTS = ("rapid_cache_store", "rapid_cache_reuse", "rapid_equivalent_steps", "rapid_reward")


class RapidAttnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"rapid_attn status {status}: {message}")
        self.status = status


def library_path() -> str:
    return _SO


def _load_hip_runtime():
    """librapid_attn.so is linked WITHOUT a HIP runtime of its own, so that its
    launches go to the runtime that owns the caller's streams and allocations.
    With PyTorch that is the libamdhip64.so bundled in torch/lib: make its symbols
    global before the library (whose constructor registers the kernels) is opened."""
    import torch
    bundled = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    ctypes.CDLL(bundled if os.path.exists(bundled) else "libamdhip64.so", mode=ctypes.RTLD_GLOBAL)


def library():
    """The loaded C library with argtypes set.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_SO):
        raise ImportError(
            f"{_SO} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
            "or python paper_2509_22323_amd/build.py). There is no CPU fallback.")
    _load_hip_runtime()
    lib = ctypes.CDLL(_SO)
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.rapid_attn_dense.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, cf, vp, sz, vp]
    lib.rapid_attn_dense.restype = ci
    lib.rapid_attn_block_sparse.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, ci, cf, vp, sz, vp]
    lib.rapid_attn_block_sparse.restype = ci
    lib.rapid_attn_block_sparse_static.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, ci, cf, vp]
    lib.rapid_attn_block_sparse_static.restype = ci
    lib.rapid_attn_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.rapid_attn_workspace_bytes.restype = sz
    lib.rapid_attn_joint.argtypes = [ctypes.POINTER(Segment), ci, ci, ci, ci, ci, vp, ci, vp, cf, vp, sz, vp]
    lib.rapid_attn_joint.restype = ci
    lib.rapid_attn_joint_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.rapid_attn_joint_workspace_bytes.restype = sz
    lib.rapid_attn_status_string.argtypes = [ci]
    lib.rapid_attn_status_string.restype = ctypes.c_char_p
    lib.rapid_attn_version.argtypes = []
    lib.rapid_attn_version.restype = ci
    lib.rapid_mask_select.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, cf, vp, vp, sz, vp]
    lib.rapid_mask_select.restype = ci
    lib.rapid_mask_select_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.rapid_mask_select_workspace_bytes.restype = sz
    lib.rapid_mask_select_joint.argtypes = [ctypes.POINTER(Segment), ci, ci, ci, ci, ci, ci, vp, ci, cf, cf, vp, vp, sz, vp]
    lib.rapid_mask_select_joint.restype = ci
    lib.rapid_mask_select_joint_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.rapid_mask_select_joint_workspace_bytes.restype = sz
    lib.rapid_attn_joint_select.argtypes = [ctypes.POINTER(Segment), ci, ci, ci, ci, ci, ci, vp, ci, cf, cf, vp, vp, sz, vp]
    lib.rapid_attn_joint_select.restype = ci
    lib.rapid_attn_joint_select_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.rapid_attn_joint_select_workspace_bytes.restype = sz
    lib.rapid_mask_level_tau.argtypes = [ci]
    lib.rapid_mask_level_tau.restype = cf
    cd, dp = ctypes.c_double, ctypes.POINTER(ctypes.c_double)
    lib.rapid_cache_store.argtypes = [vp, vp, vp, ci, sz, vp, vp]
    lib.rapid_cache_store.restype = ci
    lib.rapid_cache_reuse.argtypes = [vp, vp, vp, ci, sz, vp, vp]
    lib.rapid_cache_reuse.restype = ci
    lib.rapid_equivalent_steps.argtypes = [dp, dp, ci, dp]
    lib.rapid_equivalent_steps.restype = ci
    lib.rapid_reward.argtypes = [cd, cd, cd, cd, ci]
    lib.rapid_reward.restype = cd
    _lib = lib
    return lib


def rapid_attn_status_string(status: int) -> str:
    return library().rapid_attn_status_string(int(status)).decode()


def rapid_attn_version() -> int:
    return library().rapid_attn_version()


def rapid_attn_workspace_bytes(B: int, H: int, N: int, D: int, block: int) -> int:
    return int(library().rapid_attn_workspace_bytes(B, H, N, D, block))


def _check(status: int):
    if status != 0:
        raise RapidAttnError(status, rapid_attn_status_string(status))


def _qkvo(q, k, v, o):
    import torch
    for name, t in (("q", q), ("k", k), ("v", v), ("o", o)):
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.bfloat16
                and t.dim() == 4 and t.is_contiguous()):
            raise TypeError(f"{name} must be a contiguous CUDA bfloat16 tensor [B,H,N,D]")
        if t.shape != q.shape or t.device != q.device:
            raise ValueError(f"{name} shape/device differs from q")
    return tuple(int(s) for s in q.shape)


def _stream(t):
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def rapid_attn_dense(q, k, v, o, kv_len=None, scale=0.0):
    """o <- softmax(scale q k^T) v over the first kv_len tokens (all heads, samples).
    Tensors: CUDA bf16 [B,H,N,D], contiguous.  Enqueued on torch's current stream."""
    B, H, N, D = _qkvo(q, k, v, o)
    kv_len = N if kv_len is None else int(kv_len)
    _check(library().rapid_attn_dense(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                      B, H, N, D, kv_len, float(scale), None, 0, _stream(q)))
    return o


def rapid_attn_block_sparse(q, k, v, o, mask, block, kv_len=None, scale=0.0, workspace=None):
    """As rapid_attn_dense, restricted to the tiles kept by `mask` (CUDA uint8
    [B,H,N/block,N/block]).  `workspace`: CUDA uint8 tensor of at least
    rapid_attn_workspace_bytes(...) bytes; allocated with torch if None.  Returns o."""
    import torch
    B, H, N, D = _qkvo(q, k, v, o)
    kv_len = N if kv_len is None else int(kv_len)
    if not (isinstance(mask, torch.Tensor) and mask.is_cuda and mask.dtype == torch.uint8
            and mask.is_contiguous() and mask.device == q.device):
        raise TypeError("mask must be a contiguous CUDA uint8 tensor")
    if block > 0 and N % block == 0 and tuple(mask.shape) != (B, H, N // block, N // block):
        raise ValueError(f"mask shape {tuple(mask.shape)} != {(B, H, N // block, N // block)}")
    if workspace is None:
        need = rapid_attn_workspace_bytes(B, H, N, D, int(block))
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    if not (workspace.is_cuda and workspace.is_contiguous() and workspace.device == q.device):
        raise TypeError("workspace must be a contiguous CUDA tensor on q's device")
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(library().rapid_attn_block_sparse(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), B, H, N, D, int(block),
        mask.data_ptr(), kv_len, float(scale), workspace.data_ptr(), ws_bytes, _stream(q)))
    return o


STATIC_SCRATCH_BYTES = 64 << 20


def rapid_attn_block_sparse_static(q, k, v, o, mask, block, kv_len=None, scale=0.0):
    """rapid_attn_block_sparse on the library's own fixed scratch array: neither this wrapper nor
    the call allocates device memory.  All calls on one GPU share the array."""
    import torch
    B, H, N, D = _qkvo(q, k, v, o)
    kv_len = N if kv_len is None else int(kv_len)
    if not (isinstance(mask, torch.Tensor) and mask.is_cuda and mask.dtype == torch.uint8
            and mask.is_contiguous() and mask.device == q.device):
        raise TypeError("mask must be a contiguous CUDA uint8 tensor")
    if block > 0 and N % block == 0 and tuple(mask.shape) != (B, H, N // block, N // block):
        raise ValueError(f"mask shape {tuple(mask.shape)} != {(B, H, N // block, N // block)}")
    _check(library().rapid_attn_block_sparse_static(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), B, H, N, D, int(block),
        mask.data_ptr(), kv_len, float(scale), _stream(q)))
    return o


def rapid_attn_joint_workspace_bytes(B: int, H: int, N: int, D: int, block: int) -> int:
    return int(library().rapid_attn_joint_workspace_bytes(B, H, N, D, block))


def _segments(segments):
    """(descriptor array, B, H, N, D) of a sequence of (q, k, v, o) tensors indexed [B, H, n, D]."""
    import torch
    if len(segments) not in (1, 2):
        raise ValueError("one or two segments")
    descr = (Segment * len(segments))()
    B = H = D = None
    N = 0
    for i, (q, k, v, o) in enumerate(segments):
        for name, t in (("q", q), ("k", k), ("v", v), ("o", o)):
            if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.bfloat16 and t.dim() == 4
                    and t.stride(3) == 1):
                raise TypeError(f"segment {i}: {name} must be a CUDA bfloat16 tensor [B,H,n,D] with contiguous D")
            if t.shape != q.shape or t.device != q.device:
                raise ValueError(f"segment {i}: {name} shape/device differs from q")
        if k.stride() != q.stride() or v.stride() != q.stride():
            raise ValueError(f"segment {i}: q, k, v must share their strides")
        if B is None:
            B, H, _, D = (int(x) for x in q.shape)
        elif (int(q.shape[0]), int(q.shape[1]), int(q.shape[3])) != (B, H, D):
            raise ValueError("segments differ in B, H or D")
        g = descr[i]
        g.q, g.k, g.v, g.o, g.n = q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), int(q.shape[2])
        g.in_stride_b, g.in_stride_h, g.in_stride_n = q.stride(0), q.stride(1), q.stride(2)
        g.out_stride_b, g.out_stride_h, g.out_stride_n = o.stride(0), o.stride(1), o.stride(2)
        N += int(q.shape[2])
    return descr, B, H, N, D


def _kv_lens_ptr(kv_lens, B, device):
    import torch
    if kv_lens is None:
        return None
    if not (isinstance(kv_lens, torch.Tensor) and kv_lens.is_cuda and kv_lens.dtype == torch.int32
            and kv_lens.is_contiguous() and kv_lens.numel() == B and kv_lens.device == device):
        raise TypeError("kv_lens must be a contiguous CUDA int32 tensor [B]")
    return kv_lens.data_ptr()


def rapid_attn_joint(segments, mask=None, block=128, kv_len=None, kv_lens=None, scale=0.0, workspace=None):
    """Joint attention over one or two token segments.  `segments`: sequence of (q, k, v, o),
    each a CUDA bf16 tensor indexed [B, H, n, D] with a contiguous last dimension and any other
    strides (a permuted view of a [B, n, H, D] or fused [B, n, 3, H, D] tensor is fine); q, k, v
    of a segment share their strides.  mask None = dense.  kv_lens: CUDA int32 [B] or None."""
    import torch
    descr, B, H, N, D = _segments(segments)
    q0 = segments[0][0]
    mask_ptr, ws_ptr, ws_bytes = None, None, 0
    if mask is not None:
        if not (isinstance(mask, torch.Tensor) and mask.is_cuda and mask.dtype == torch.uint8
                and mask.is_contiguous() and mask.device == q0.device):
            raise TypeError("mask must be a contiguous CUDA uint8 tensor")
        nb = -(-N // int(block)) if block > 0 else 0
        if tuple(mask.shape) != (B, H, nb, nb):
            raise ValueError(f"mask shape {tuple(mask.shape)} != {(B, H, nb, nb)}")
        if workspace is None:
            workspace = torch.empty(max(rapid_attn_joint_workspace_bytes(B, H, N, D, int(block)), 16),
                                    dtype=torch.uint8, device=q0.device)
        mask_ptr, ws_ptr, ws_bytes = mask.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size()
    lens_ptr = _kv_lens_ptr(kv_lens, B, q0.device)
    _check(library().rapid_attn_joint(descr, len(segments), B, H, D, int(block), mask_ptr,
                                      0 if kv_len is None else int(kv_len), lens_ptr, float(scale),
                                      ws_ptr, ws_bytes, _stream(q0)))
    return [seg[3] for seg in segments]


# ---------------------------------------------------------------- Cache-Reuse residual operations
def _residual_args(a, b, out, sample_flags):
    import torch
    for name, t in (("first input", a), ("second input", b), ("output", out)):
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()
                and t.dim() >= 1):
            raise TypeError(f"{name} must be a contiguous CUDA bfloat16 tensor [B, ...]")
        if t.shape != a.shape or t.device != a.device:
            raise ValueError(f"{name}: shape/device differs")
    B = int(a.shape[0])
    per_sample = a.numel() // B if B > 0 else 0
    flags = None
    if sample_flags is not None:
        if not (isinstance(sample_flags, torch.Tensor) and sample_flags.is_cuda and sample_flags.dtype == torch.uint8
                and sample_flags.is_contiguous() and sample_flags.numel() == B and sample_flags.device == a.device):
            raise TypeError("sample_flags must be a contiguous CUDA uint8 tensor [B]")
        flags = sample_flags.data_ptr()
    return B, per_sample, flags


def rapid_cache_store(gen_out, x, delta, sample_flags=None):
    """delta <- gen_out - x (the residual a cache-updating step keeps), per flagged sample."""
    B, per_sample, flags = _residual_args(gen_out, x, delta, sample_flags)
    _check(library().rapid_cache_store(gen_out.data_ptr(), x.data_ptr(), delta.data_ptr(), B, per_sample, flags,
                                       _stream(x)))
    return delta


def rapid_cache_reuse(x, delta, out, sample_flags=None):
    """out <- x + delta (the output of a step that reuses the cache), per flagged sample."""
    B, per_sample, flags = _residual_args(x, delta, out, sample_flags)
    _check(library().rapid_cache_reuse(x.data_ptr(), delta.data_ptr(), out.data_ptr(), B, per_sample, flags,
                                       _stream(x)))
    return out


def rapid_equivalent_steps(c_cache, c_sparse):
    """(K exact, K rounded) for the per-step cost reductions (host arithmetic in the library)."""
    n = len(c_cache)
    if len(c_sparse) != n:
        raise ValueError("c_cache and c_sparse differ in length")
    arr = ctypes.c_double * max(n, 1)
    exact = ctypes.c_double(0.0)
    k = library().rapid_equivalent_steps(arr(*c_cache), arr(*c_sparse), n, ctypes.byref(exact))
    if k < 0:
        _check(k)
    return exact.value, k


def rapid_reward(q, d, K, lam=0.97, omega=1.0):
    return library().rapid_reward(float(q), float(d), float(omega), float(lam), int(K))


# ---------------------------------------------------------------- block-mask selection
def rapid_mask_level_tau(action: int) -> float:
    return float(library().rapid_mask_level_tau(int(action)))


def rapid_mask_select_workspace_bytes(B: int, H: int, N: int, D: int, block: int) -> int:
    return int(library().rapid_mask_select_workspace_bytes(B, H, N, D, block))


def rapid_mask_select(q, k, mask, block, kv_len=None, text_start=None, tau=0.95, scale=0.0, workspace=None):
    """mask <- block mask [B,H,N/block,N/block] (uint8) keeping, per row, the key-blocks that hold
    `tau` of the pooled attention mass, plus the diagonal and the text rows/columns.  q, k: CUDA
    bf16 [B,H,N,D] contiguous."""
    import torch
    for name, t in (("q", q), ("k", k)):
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.bfloat16 and t.dim() == 4
                and t.is_contiguous() and t.shape == q.shape and t.device == q.device):
            raise TypeError(f"{name} must be a contiguous CUDA bfloat16 tensor [B,H,N,D]")
    B, H, N, D = (int(x) for x in q.shape)
    kv_len = N if kv_len is None else int(kv_len)
    text_start = N if text_start is None else int(text_start)
    if not (isinstance(mask, torch.Tensor) and mask.is_cuda and mask.dtype == torch.uint8 and mask.is_contiguous()
            and mask.device == q.device):
        raise TypeError("mask must be a contiguous CUDA uint8 tensor")
    if block > 0 and N % block == 0 and tuple(mask.shape) != (B, H, N // block, N // block):
        raise ValueError(f"mask shape {tuple(mask.shape)} != {(B, H, N // block, N // block)}")
    if workspace is None:
        workspace = torch.empty(max(rapid_mask_select_workspace_bytes(B, H, N, D, int(block)), 16), dtype=torch.uint8,
                                device=q.device)
    _check(library().rapid_mask_select(q.data_ptr(), k.data_ptr(), B, H, N, D, int(block), kv_len, text_start,
                                       float(tau), float(scale), mask.data_ptr(), workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(), _stream(q)))
    return mask


def rapid_mask_select_joint_workspace_bytes(B: int, H: int, N: int, D: int, block: int) -> int:
    return int(library().rapid_mask_select_joint_workspace_bytes(B, H, N, D, block))


def rapid_mask_select_joint(segments, mask, block, kv_len=None, kv_lens=None, text_start=None, tau=0.95, scale=0.0,
                            workspace=None):
    """rapid_mask_select on Q and K given as one or two token segments: `segments` is a sequence of
    (q, k) pairs (tuples as passed to rapid_attn_joint work too: only their first two tensors are
    used), each a CUDA bf16 tensor indexed [B, H, n, D] with a contiguous last dimension; q and k of
    a segment share their strides.  mask: CUDA uint8 [B, H, nb, nb], nb = ceil(N / block)."""
    import torch
    if len(segments) not in (1, 2):
        raise ValueError("one or two segments")
    descr = (Segment * len(segments))()
    B = H = D = None
    N = 0
    for i, seg in enumerate(segments):
        q, k = seg[0], seg[1]
        for name, t in (("q", q), ("k", k)):
            if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.bfloat16 and t.dim() == 4
                    and t.stride(3) == 1):
                raise TypeError(f"segment {i}: {name} must be a CUDA bfloat16 tensor [B,H,n,D] with contiguous D")
            if t.shape != q.shape or t.device != q.device:
                raise ValueError(f"segment {i}: {name} shape/device differs from q")
        if k.stride() != q.stride():
            raise ValueError(f"segment {i}: q and k must share their strides")
        if B is None:
            B, H, _, D = (int(x) for x in q.shape)
        elif (int(q.shape[0]), int(q.shape[1]), int(q.shape[3])) != (B, H, D):
            raise ValueError("segments differ in B, H or D")
        g = descr[i]
        g.q, g.k, g.v, g.o, g.n = q.data_ptr(), k.data_ptr(), None, None, int(q.shape[2])
        g.in_stride_b, g.in_stride_h, g.in_stride_n = q.stride(0), q.stride(1), q.stride(2)
        N += int(q.shape[2])
    q0 = segments[0][0]
    nb = -(-N // int(block)) if block > 0 else 0
    if not (isinstance(mask, torch.Tensor) and mask.is_cuda and mask.dtype == torch.uint8 and mask.is_contiguous()
            and mask.device == q0.device):
        raise TypeError("mask must be a contiguous CUDA uint8 tensor")
    if tuple(mask.shape) != (B, H, nb, nb):
        raise ValueError(f"mask shape {tuple(mask.shape)} != {(B, H, nb, nb)}")
    lens_ptr = None
    if kv_lens is not None:
        if not (isinstance(kv_lens, torch.Tensor) and kv_lens.is_cuda and kv_lens.dtype == torch.int32
                and kv_lens.is_contiguous() and kv_lens.numel() == B and kv_lens.device == q0.device):
            raise TypeError("kv_lens must be a contiguous CUDA int32 tensor [B]")
        lens_ptr = kv_lens.data_ptr()
    if workspace is None:
        workspace = torch.empty(max(rapid_mask_select_joint_workspace_bytes(B, H, N, D, int(block)), 16),
                                dtype=torch.uint8, device=q0.device)
    _check(library().rapid_mask_select_joint(
        descr, len(segments), B, H, D, int(block), 0 if kv_len is None else int(kv_len), lens_ptr,
        N if text_start is None else int(text_start), float(tau), float(scale), mask.data_ptr(),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(q0)))
    return mask


def rapid_attn_joint_select_workspace_bytes(B: int, H: int, N: int, D: int, block: int) -> int:
    return int(library().rapid_attn_joint_select_workspace_bytes(B, H, N, D, block))


def rapid_attn_joint_select(segments, block=128, kv_len=None, kv_lens=None, text_start=None, tau=0.95, scale=0.0,
                            mask_out=None, workspace=None):
    """Mask selection at `tau` and block-sparse attention under it in one call, on (q, k, v, o)
    segments as rapid_attn_joint takes them; mask_out: optional CUDA uint8 [B,H,nb,nb] that receives
    the selected mask.  Returns the o tensors."""
    import torch
    descr, B, H, N, D = _segments(segments)
    q0 = segments[0][0]
    nb = -(-N // int(block)) if block > 0 else 0
    mask_ptr = None
    if mask_out is not None:
        if not (isinstance(mask_out, torch.Tensor) and mask_out.is_cuda and mask_out.dtype == torch.uint8
                and mask_out.is_contiguous() and mask_out.device == q0.device and tuple(mask_out.shape) == (B, H, nb, nb)):
            raise TypeError(f"mask_out must be a contiguous CUDA uint8 tensor {(B, H, nb, nb)}")
        mask_ptr = mask_out.data_ptr()
    if workspace is None:
        workspace = torch.empty(max(rapid_attn_joint_select_workspace_bytes(B, H, N, D, int(block)), 16),
                                dtype=torch.uint8, device=q0.device)
    _check(library().rapid_attn_joint_select(
        descr, len(segments), B, H, D, int(block), 0 if kv_len is None else int(kv_len),
        _kv_lens_ptr(kv_lens, B, q0.device), N if text_start is None else int(text_start), float(tau), float(scale),
        mask_ptr, workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(q0)))
    return [seg[3] for seg in segments]
