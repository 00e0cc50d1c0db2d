"""fp64 CPU oracle for MM-DiT joint attention (dense / block-masked).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
bench's cpu_baseline leg.  The product package never imports this module, and
this module never imports the product package.

The arithmetic lives in ``attn_oracle.c`` (plain C, fp64, OpenMP over rows);
this file only compiles it with gcc when needed and marshals numpy arrays.
Operation followed: RAPID^3 Sec. 3.1 Eq. 1 (self-attention block), Sec. 3.2
Level-3 / Eq. 4 (sparse replacement), Sec. 3.3 (c) (action semantics).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_SO = os.path.join(_HERE, "libattn_oracle.so")
_lib = None


def build(force: bool = False, src: str = _SRC, out: str = _SO) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the .so path."""
    stale = (not os.path.exists(out)) or os.path.getmtime(out) < os.path.getmtime(src)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
               "-Wall", "-Wextra", "-o", out, src, "-lm"]
        subprocess.run(cmd, check=True)
    return out


def _bind(lib):
    u16p = ctypes.POINTER(ctypes.c_uint16)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    f64p = ctypes.POINTER(ctypes.c_double)
    i32p = ctypes.POINTER(ctypes.c_int32)
    ci = ctypes.c_int
    lib.rapid_oracle_attn.argtypes = [u16p, u16p, u16p, f64p, ci, ci, ci, ci, ci,
                                      u8p, ci, ctypes.c_double]
    lib.rapid_oracle_attn.restype = ci
    lib.rapid_oracle_attn_rows.argtypes = [u16p, u16p, u16p, f64p, ci, ci, ci, ci, ci,
                                           u8p, ci, ctypes.c_double, ci, i32p]
    lib.rapid_oracle_attn_rows.restype = ci
    lib.rapid_oracle_kept_tiles.argtypes = [u8p, ci, ci, ci, ci, ci, i32p, i32p]
    lib.rapid_oracle_kept_tiles.restype = ci
    lib.rapid_oracle_threads.argtypes = []
    lib.rapid_oracle_threads.restype = ci
    return lib


def load(path: str | None = None):
    """Load (building first if needed) the oracle library."""
    global _lib
    if path is not None:
        return _bind(ctypes.CDLL(path))
    if _lib is None:
        _lib = _bind(ctypes.CDLL(build()))
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("q/k/v must be bf16 bit patterns stored as uint16")
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _mask_arg(mask, B, H, N, block):
    if mask is None:
        return None, None
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    nb = N // block
    if m.shape != (B, H, nb, nb):
        raise ValueError(f"mask shape {m.shape} != {(B, H, nb, nb)}")
    return m, _ptr(m, ctypes.c_uint8)


def attention(q, k, v, kv_len=None, mask=None, block=0, scale=0.0, lib=None):
    """O[B,H,N,D] in fp64.  q,k,v: uint16 bf16 bits [B,H,N,D]; mask: uint8
    [B,H,N/block,N/block] or None (dense); scale<=0 -> 1/sqrt(D)."""
    lib = lib or load()
    q, k, v = _u16(q), _u16(k), _u16(v)
    B, H, N, D = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    kv_len = N if kv_len is None else int(kv_len)
    m, mp = _mask_arg(mask, B, H, N, block)
    o = np.empty((B, H, N, D), dtype=np.float64)
    rc = lib.rapid_oracle_attn(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16),
                               _ptr(v, ctypes.c_uint16), _ptr(o, ctypes.c_double),
                               B, H, N, D, int(block), mp, kv_len, float(scale))
    if rc != 0:
        raise ValueError(f"rapid_oracle_attn failed with code {rc}")
    return o


def attention_rows(q, k, v, rows, kv_len=None, mask=None, block=0, scale=0.0, lib=None):
    """Selected output rows.  rows: int array [n,3] of (b,h,r).  Returns fp64 [n,D]."""
    lib = lib or load()
    q, k, v = _u16(q), _u16(k), _u16(v)
    B, H, N, D = q.shape
    kv_len = N if kv_len is None else int(kv_len)
    m, mp = _mask_arg(mask, B, H, N, block)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    o = np.empty((rows.shape[0], D), dtype=np.float64)
    rc = lib.rapid_oracle_attn_rows(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16),
                                    _ptr(v, ctypes.c_uint16), _ptr(o, ctypes.c_double),
                                    B, H, N, D, int(block), mp, kv_len, float(scale),
                                    rows.shape[0], _ptr(rows, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"rapid_oracle_attn_rows failed with code {rc}")
    return o


def kept_tiles(mask, block, kv_len, lib=None):
    """(counts int32 [B,H,nb], indices int32 [B,H,nb,nb], -1 padded)."""
    lib = lib or load()
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    B, H, nb, nb2 = m.shape
    assert nb == nb2
    counts = np.empty((B, H, nb), dtype=np.int32)
    idx = np.empty((B, H, nb, nb), dtype=np.int32)
    rc = lib.rapid_oracle_kept_tiles(_ptr(m, ctypes.c_uint8), B, H, nb * block, block,
                                     int(kv_len), _ptr(counts, ctypes.c_int32),
                                     _ptr(idx, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"rapid_oracle_kept_tiles failed with code {rc}")
    return counts, idx


def threads(lib=None) -> int:
    return (lib or load()).rapid_oracle_threads()
