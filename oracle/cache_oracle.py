"""Oracle for the Cache-Reuse residual operations and the cost accounting of RAPID^3.

TEST INFRASTRUCTURE ONLY (imported by tests, the smoke check and the bench's CPU leg;
never by the product package, and it imports nothing from it).

What is defined where (RAPID^3):
  Sec. 3.2 "Level-2: Cache-Reuse" and Eq. 3: the cached residual is the difference between the
      generator's output and its input at the step where the cache was last updated,
      Delta = G(X) - X, and a step that reuses the cache outputs O = X + Delta.
  Sec. 3.3 "Training policy heads with reinforcement learning": the equivalent steps
      K = sum_k (1 - C_k^cache)(1 - C_k^sparse), rounded to the nearest integer, and the reward
      r = (1/K) sum_{k=1..K} lambda^(K-k) (q + omega d).
  App. (hyper-parameter table): lambda = 0.97, omega = 1.0, C^cache = 0.95,
      C^sparse = 0.05 / 0.07 / 0.10 for the three sparse candidates.

Arithmetic: tensors are bf16 bit patterns (uint16).  The exact sum or difference is formed in
fp64 and rounded ONCE to bf16, round-to-nearest-even (inputs have 8 significant bits, so the
fp64 result is either exact or so far from a bf16 tie that its own rounding cannot matter).
Readings of the paper (it is silent on both): a tie in "nearest integer" rounds away from
zero, and K is at least 1.
"""
from __future__ import annotations

import numpy as np

C_CACHE = 0.95                        # cost reduction of a step that reuses the cache
C_SPARSE = (0.0, 0.05, 0.07, 0.10)    # cost reduction of sparse action 0 (dense), 1, 2, 3
LAMBDA = 0.97
OMEGA = 1.0


def bf16_to_f64(bits) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f64_to_bf16(x) -> np.ndarray:
    """Round float64 to bf16 (1 sign, 8 exponent, 7 fraction bits), nearest, ties to even,
    with subnormals, overflow to infinity, NaN kept as a NaN.  Returns uint16 bit patterns.

    A bf16 value with |x| in [2^(e-1), 2^e) is a multiple of 2^(e-8); below the normal range
    the spacing stays 2^-133.  Dividing by that power of two is exact, numpy.rint rounds half
    to even, and multiplying back is exact."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    finite = np.isfinite(a)
    _, e = np.frexp(np.where(finite, a, 1.0))              # a = m * 2^e, m in [0.5, 1)
    quantum_exp = np.maximum(e - 8, -133)
    y = np.ldexp(np.rint(np.ldexp(np.where(finite, a, 0.0), -quantum_exp)), quantum_exp)
    y = np.where(y >= 2.0 ** 128, np.inf, y)               # past the largest bf16 (2^128 - 2^120)
    y = np.where(finite, y, a)                             # inf and nan pass through
    with np.errstate(over="ignore"):
        f32 = np.copysign(y, x).astype(np.float32)         # exact: y is a bf16 value
    bits = (f32.view(np.uint32) >> 16).astype(np.uint16)
    return np.where(np.isnan(x), np.uint16(0x7FC0), bits).astype(np.uint16)


def cache_store(o_bits, x_bits) -> np.ndarray:
    """Delta = G(X) - X: the residual that a cache-updating step leaves behind."""
    with np.errstate(invalid="ignore"):                   # inf - inf is a NaN, as it should be
        return f64_to_bf16(bf16_to_f64(o_bits) - bf16_to_f64(x_bits))


def cache_reuse(x_bits, delta_bits) -> np.ndarray:
    """O = X + Delta: the output of a step that reuses the cached residual."""
    with np.errstate(invalid="ignore"):
        return f64_to_bf16(bf16_to_f64(x_bits) + bf16_to_f64(delta_bits))


def cache_reuse_batch(x_bits, delta_bits, out_bits, flags) -> np.ndarray:
    """Image-wise decision over a batch [B, ...]: samples with a nonzero flag take X + Delta,
    the others keep what `out_bits` already holds."""
    out = np.array(out_bits, dtype=np.uint16, copy=True)
    for b, f in enumerate(np.asarray(flags)):
        if f:
            out[b] = cache_reuse(np.asarray(x_bits)[b], np.asarray(delta_bits)[b])
    return out


def step_costs(cache_actions, sparse_actions):
    """(C^cache_k, C^sparse_k) of an action trace: a_cache = 1 reuses the cache, a_sparse in
    0..3 picks the sparse candidate; the sparse policy is inactive on a step that reuses the
    cache (Sec. 3.3 (c)), so its reduction is 0 there."""
    cc, cs = [], []
    for ac, asp in zip(cache_actions, sparse_actions):
        cc.append(C_CACHE if ac else 0.0)
        cs.append(0.0 if ac else C_SPARSE[asp])
    return cc, cs


def equivalent_steps(c_cache, c_sparse):
    """K = sum_k (1 - C_k^cache)(1 - C_k^sparse); returns (K exact, K rounded to the nearest
    integer, ties away from zero, at least 1)."""
    k = 0.0
    for a, b in zip(c_cache, c_sparse):
        k += (1.0 - a) * (1.0 - b)
    return k, max(1, int(np.floor(k + 0.5)))


def reward(q, d, K, lam=LAMBDA, omega=OMEGA):
    """r = (1/K) sum_{k=1..K} lambda^(K-k) (q + omega d), the sum written out."""
    s = 0.0
    for k in range(1, K + 1):
        s += lam ** (K - k) * (q + omega * d)
    return s / K
