"""Oracle for the block-mask selection that turns a Sparse-Attention level into a mask.

TEST INFRASTRUCTURE ONLY (imported by tests, the smoke check and the bench's CPU leg; never
by the product package, and it imports nothing from it).

PARITY UNPINNED against the paper: RAPID^3 (Sec. 3.2 "Level-3: Sparse-Attention", Sec. 3.3 (c),
App. hyper-parameter table) takes its sparse attention from a third-party method and states
only that each action 1..3 selects a candidate hyper-parameter of progressively higher
sparsity, per layer and head; the selection rule itself is not in the paper.  The rule below
is this build's own, in the spirit the paper describes (a cheap per-head prediction of which
blocks of the attention map matter); what is pinned is that THIS rule is computed correctly.

Rule, for one (sample, head), mask tiles of `block` tokens, nb = N / block:
  1. live blocks: those that start below kv_len.
  2. block means qbar_i, kbar_j over the valid tokens (row < kv_len) of each live block.
  3. block scores s_ij = scale * qbar_i . kbar_j; phat_i = softmax of s_i over the live j.
  4. row i keeps the fewest key-blocks, taken in order of decreasing phat_ij, whose mass
     reaches tau; blocks that tie with the last one taken are kept too.  Equivalently: with
     v* the largest value among phat_i. for which the blocks with phat_ij >= v* hold at least
     tau of the row's mass, keep { j : phat_ij >= v* }; if even all blocks do not reach tau
     (tau > 1 or rounding), keep all.
  5. always kept: the diagonal; the rows and the columns of text blocks (blocks that hold a
     token at or after text_start) -- the paper's configurations keep text tokens dense.
  6. blocks that are not live: row and column 0.
"""
from __future__ import annotations

import numpy as np

LEVEL_TAU = (1.0, 0.98, 0.95, 0.90)   # action 0 (dense) .. 3: this build's defaults, not the paper's


def _widen(bits):
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def block_means(x_bits, block, kv_len):
    """fp64 mean over the valid tokens of each block: [B,H,N,D] bf16 bits -> [B,H,nb,D];
    blocks without a valid token give 0."""
    x = _widen(x_bits)
    B, H, N, D = x.shape
    nb = N // block
    out = np.zeros((B, H, nb, D))
    for i in range(nb):
        lo, hi = i * block, min((i + 1) * block, kv_len)
        if hi > lo:
            out[:, :, i] = x[:, :, lo:hi].sum(axis=2) / (hi - lo)
    return out


def block_probabilities(q_bits, k_bits, block, kv_len, scale=None):
    """phat [B,H,nb,nb] (0 outside the live blocks) and the number of live blocks."""
    B, H, N, D = q_bits.shape
    nb = N // block
    live = -(-kv_len // block)
    scale = 1.0 / np.sqrt(D) if not scale or scale <= 0 else scale
    qb, kb = block_means(q_bits, block, kv_len), block_means(k_bits, block, kv_len)
    p = np.zeros((B, H, nb, nb))
    for b in range(B):
        for h in range(H):
            for i in range(live):
                s = np.array([scale * float(np.dot(qb[b, h, i], kb[b, h, j])) for j in range(live)])
                e = np.exp(s - s.max())
                p[b, h, i, :live] = e / e.sum()
    return p, live


def select_row(p_row, tau):
    """Step 4 for one row of live probabilities: boolean keep vector."""
    order = np.argsort(-p_row, kind="stable")
    total = p_row.sum()
    keep = np.zeros(len(p_row), bool)
    mass = 0.0
    last = None
    for j in order:
        if mass >= tau * total and p_row[j] != last:
            break
        keep[j] = True
        mass += p_row[j]
        last = p_row[j]
    return keep


def select_mask(q_bits, k_bits, block, kv_len, text_start, tau, scale=None):
    """uint8 mask [B,H,nb,nb] by the rule in the module header."""
    p, live = block_probabilities(q_bits, k_bits, block, kv_len, scale)
    B, H, nb, _ = p.shape
    first_text = min(text_start // block, nb) if text_start < kv_len else nb
    mask = np.zeros((B, H, nb, nb), np.uint8)
    for b in range(B):
        for h in range(H):
            for i in range(live):
                keep = select_row(p[b, h, i, :live], tau)
                keep[i] = True
                keep[first_text:live] = True
                if i >= first_text:
                    keep[:] = True
                mask[b, h, i, :live] = keep
    return mask
