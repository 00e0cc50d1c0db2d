"""Seeded synthetic inputs for MM-DiT joint attention: Q/K/V tensors and block masks.

Shared by the oracle-side tests and the GPU-side tests/bench.  Holds NO attention
arithmetic: only random draws, bf16 rounding of the drawn values, and the block-mask
structure rules.  Everything is numpy on the host; tensors are bf16 bit patterns
stored as uint16 so both sides see identical bits.

The five workloads stand in for SD3 / FLUX joint text+image attention (RAPID^3
Sec. 4 setup; App. B for the CFG batch shapes; Table "Default Implementation
Details" for the GRPO group size): token layout is [image | text | zero padding].
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20250922
BF16_NAN = 0x7FC0
BF16_INF = 0x7F80
BF16_ONE = 0x3F80


# --------------------------------------------------------------------------- bf16
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    nan = np.isnan(x)
    rnd = ((bits >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((bits + rnd) >> np.uint32(16)).astype(np.uint16)
    out[nan] = BF16_NAN
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- Q/K/V
def make_qkv(B, H, N, D, kv_len=None, seed=BASE_SEED, gain=1.0, pad_fill="zero"):
    """Q, K, V as uint16 bf16 bits [B,H,N,D]; i.i.d. N(0, gain^2) drawn Q, K, V in
    that order, rounded RNE.  Rows >= kv_len hold zeros ("zero"), NaN ("nan") or
    +Inf ("inf")."""
    kv_len = N if kv_len is None else kv_len
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for _ in range(3):
        x = rng.standard_normal((B, H, N, D), dtype=np.float32)
        if gain != 1.0:
            x *= np.float32(gain)
        bits = f32_to_bf16_bits(x)
        if kv_len < N:
            fill = {"zero": 0, "nan": BF16_NAN, "inf": BF16_INF}[pad_fill]
            bits[:, :, kv_len:, :] = fill
        out.append(bits)
    return tuple(out)


def make_qkv_block_structured(B, H, N, D, block, kv_len=None, seed=BASE_SEED, n_text_blocks=0,
                              peak=5.5, link_noise=0.3, token_noise=0.2, pad_fill="zero"):
    """Q, K, V (uint16 bf16 bits [B,H,N,D]) whose attention map has block structure, as the maps of
    a trained DiT have and i.i.d. inputs have not: every key-block has a centre c_j ~ N(0, g^2),
    every query-block looks at one key-block (a seeded permutation; the diagonal for text blocks)
    with centre c_perm(i) + N(0, link_noise^2), tokens are their block's centre + N(0, token_noise^2).
    g^2 = peak / sqrt(D), so that under the 1/sqrt(D) scale the linked block's score stands about
    `peak` above the others whatever the head size (at 5.5: most of a row's mass, not all of it, so
    that selection levels of different strictness keep different numbers of blocks).
    V is i.i.d. N(0,1).  Only draws and the structure rule: no attention arithmetic."""
    kv_len = N if kv_len is None else kv_len
    rng = np.random.Generator(np.random.PCG64(seed))
    nb = -(-N // block)
    nI = nb - n_text_blocks
    center_gain = float(np.sqrt(peak / np.sqrt(D)))
    ck = (rng.standard_normal((B, H, nb, D)) * center_gain).astype(np.float32)
    cq = np.empty_like(ck)
    for b in range(B):
        for h in range(H):
            perm = np.concatenate([rng.permutation(nI), np.arange(nI, nb)])
            cq[b, h] = ck[b, h, perm]
    cq += (rng.standard_normal((B, H, nb, D)) * link_noise).astype(np.float32)
    out = []
    for centres in (cq, ck, None):
        x = rng.standard_normal((B, H, N, D), dtype=np.float32)
        if centres is not None:
            x *= np.float32(token_noise)
            x += np.repeat(centres, block, axis=2)[:, :, :N]
        bits = f32_to_bf16_bits(x)
        if kv_len < N:
            bits[:, :, kv_len:, :] = {"zero": 0, "nan": BF16_NAN, "inf": BF16_INF}[pad_fill]
        out.append(bits)
    return tuple(out)


# --------------------------------------------------------------------------- masks
def mask_bernoulli_diag(B, H, nb, p, seed):
    """Each tile kept with probability p; the diagonal forced on."""
    rng = np.random.Generator(np.random.PCG64(seed))
    m = (rng.random((B, H, nb, nb)) < p).astype(np.uint8)
    i = np.arange(nb)
    m[:, :, i, i] = 1
    return m


def _pick_extra(rng, sub, target):
    """Turn on uniformly-random zero tiles of 2-D array `sub` (in place) until
    sub.sum() == target (no-op if already >= target)."""
    need = int(target) - int(sub.sum())
    if need <= 0:
        return
    zr, zc = np.nonzero(sub == 0)
    sel = rng.choice(zr.size, size=min(need, zr.size), replace=False)
    sub[zr[sel], zc[sel]] = 1


def mask_text_dense(B, H, nb, n_text, density, seed, per_sample_density=None):
    """Text rows/cols (the trailing n_text blocks) all kept; image diagonal kept;
    further image x image tiles drawn uniformly without replacement, per (sample,
    head), until round(density * nI^2) image tiles are kept.  `density` is nominal,
    over the image x image sub-grid."""
    rng = np.random.Generator(np.random.PCG64(seed))
    nI = nb - n_text
    m = np.zeros((B, H, nb, nb), dtype=np.uint8)
    m[:, :, nI:, :] = 1
    m[:, :, :, nI:] = 1
    i = np.arange(nI)
    for b in range(B):
        d = density if per_sample_density is None else per_sample_density[b]
        for h in range(H):
            sub = np.zeros((nI, nI), dtype=np.uint8)
            sub[i, i] = 1
            if d >= 1.0:
                sub[:] = 1
            else:
                _pick_extra(rng, sub, round(d * nI * nI))
            m[b, h, :nI, :nI] = sub
    return m


def mask_band_plus_random(B, H, nb, n_text, half_width, total_density, seed):
    """Text rows/cols kept; image band |i-j| <= half_width kept (one block = one row
    of the 2-D latent grid, so this is a local 2-D window); then per-head random
    off-band image tiles until round(total_density * nb^2) tiles are kept in all."""
    rng = np.random.Generator(np.random.PCG64(seed))
    nI = nb - n_text
    m = np.zeros((B, H, nb, nb), dtype=np.uint8)
    m[:, :, nI:, :] = 1
    m[:, :, :, nI:] = 1
    ii, jj = np.meshgrid(np.arange(nI), np.arange(nI), indexing="ij")
    band = (np.abs(ii - jj) <= half_width).astype(np.uint8)
    n_text_tiles = nb * nb - nI * nI
    target_img = round(total_density * nb * nb) - n_text_tiles
    for b in range(B):
        for h in range(H):
            sub = band.copy()
            _pick_extra(rng, sub, target_img)
            m[b, h, :nI, :nI] = sub
    return m


def effective_density(mask, block, kv_len):
    """Kept tiles whose key-block starts below kv_len and whose query-block starts
    below kv_len, over nb^2, averaged over (sample, head)."""
    nb = mask.shape[-1]
    live = (np.arange(nb) * block < kv_len)
    kept = (mask != 0) & live[None, None, :, None] & live[None, None, None, :]
    return float(kept.sum()) / float(mask.shape[0] * mask.shape[1] * nb * nb)


# --------------------------------------------------------------------------- configs
@dataclass
class Workload:
    name: str
    B: int
    H: int
    N: int          # allocated tokens (multiple of block)
    kv_len: int     # valid tokens (image + text)
    D: int
    block: int
    n_text_blocks: int
    densities: tuple            # nominal densities; 1.0 = all-ones mask
    index: int
    notes: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def nb(self):
        return self.N // self.block

    def seed(self, density_index=0):
        return BASE_SEED + 100 * self.index + density_index

    def dense_flops(self):
        return 4.0 * self.B * self.H * float(self.kv_len) ** 2 * self.D

    def qkv(self, pad_fill="zero", gain=1.0):
        return make_qkv(self.B, self.H, self.N, self.D, self.kv_len,
                        seed=self.seed(), gain=gain, pad_fill=pad_fill)

    def qkv_block_structured(self, pad_fill="zero"):
        """The same shape with a block-structured attention map (what the mask selection is for)."""
        return make_qkv_block_structured(self.B, self.H, self.N, self.D, self.block, self.kv_len,
                                         seed=self.seed() + 50, n_text_blocks=self.n_text_blocks, pad_fill=pad_fill)

    def mask(self, density):
        """uint8 [B,H,nb,nb] for a nominal density listed in `densities`
        ("mixed" for the per-sample GRPO draw)."""
        di = self.densities.index(density)
        seed = self.seed(di) + 7
        if self.name == "tiny":
            if density >= 1.0:
                return np.ones((self.B, self.H, self.nb, self.nb), np.uint8)
            return mask_bernoulli_diag(self.B, self.H, self.nb, density, seed)
        if self.name in ("sd3_1024", "flux_1024"):
            if isinstance(density, str) and density.startswith("total"):
                # the density as a TOTAL over the whole grid, text rows/columns included:
                # the image x image sub-grid keeps whatever is left after the text tiles
                nI = self.nb - self.n_text_blocks
                kept_image = round(float(density[5:]) * self.nb ** 2) - (self.nb ** 2 - nI ** 2)
                density = max(kept_image, nI) / nI ** 2
            return mask_text_dense(self.B, self.H, self.nb, self.n_text_blocks, density, seed)
        if self.name == "grpo_sd3":
            return mask_text_dense(self.B, self.H, self.nb, self.n_text_blocks, None, seed,
                                   per_sample_density=self.sample_densities())
        if self.name == "flux_2048":
            w = {0.1: 1, 0.3: 8}[density]
            return mask_band_plus_random(self.B, self.H, self.nb, self.n_text_blocks, w,
                                         density, seed)
        raise KeyError(self.name)

    def sample_densities(self):
        """GRPO rollout group: each sample's sparse action drawn uniformly."""
        rng = np.random.Generator(np.random.PCG64(self.seed() + 3))
        return [float(x) for x in rng.choice([1.0, 0.5, 0.3, 0.15], size=self.B)]


WORKLOADS = {
    w.name: w for w in [
        Workload("tiny", 1, 2, 256, 256, 64, 64, 0, (1.0, 0.5), 1,
                 "4x4 block grid, Bernoulli(0.5) with diagonal on"),
        Workload("sd3_1024", 1, 24, 4480, 4429, 64, 128, 3, (1.0, 0.25, "total0.25"), 2,
                 "4096 image + 333 text tokens, padded to 35 blocks"),
        Workload("flux_1024", 1, 24, 4608, 4608, 128, 128, 4, (1.0, 0.5, 0.2), 3,
                 "4096 image + 512 text tokens"),
        Workload("grpo_sd3", 8, 24, 4480, 4429, 64, 128, 3, ("mixed",), 4,
                 "rollout group, per-sample density from {1.0,0.5,0.3,0.15}"),
        Workload("flux_2048", 1, 24, 16896, 16896, 128, 128, 4, (0.1, 0.3), 5,
                 "16384 image + 512 text tokens, band + random tiles, total density"),
    ]
}


def sample_rows(B, H, N, kv_len, block, n, seed):
    """n distinct (b,h,r) triples: the first/last valid rows, a row of the block that
    holds kv_len, one pad row if any, and uniform draws over valid rows."""
    rng = np.random.Generator(np.random.PCG64(seed))
    fixed = [(0, 0, 0), (B - 1, H - 1, kv_len - 1), (B - 1, 0, (kv_len - 1) // block * block)]
    if kv_len < N:
        fixed.append((0, H - 1, N - 1))
    seen = set(fixed)
    while len(seen) < max(n, len(fixed)):
        seen.add((int(rng.integers(B)), int(rng.integers(H)), int(rng.integers(kv_len))))
    rows = fixed + sorted(seen - set(fixed))
    return np.asarray(rows, dtype=np.int32)


def action_trace(seed, n_steps=None, n_cached=None, n_sparse=None):
    """A scripted action trace of one image with the statistics the paper reports for its learned
    policies (App. "distribution of learned strategies": 12-16 sampling steps per image, of which
    4-8 reuse the cache and 2-4 run sparse attention): a list of (a_cache, a_sparse) per step,
    a_cache in {0, 1}, a_sparse in 0..3 (0 on the steps that reuse the cache, where the sparse
    policy is inactive).  The first step always computes (there is no cache yet).  Only the
    counts follow the paper; which steps get which action is a seeded draw."""
    rng = np.random.default_rng(seed)
    n_steps = int(rng.integers(12, 17)) if n_steps is None else n_steps
    n_cached = int(rng.integers(4, 9)) if n_cached is None else n_cached
    n_sparse = int(rng.integers(2, 5)) if n_sparse is None else n_sparse
    n_cached = min(n_cached, n_steps - 1)
    n_sparse = min(n_sparse, n_steps - n_cached)
    cached = set((1 + rng.choice(n_steps - 1, size=n_cached, replace=False)).tolist())
    free = [s for s in range(n_steps) if s not in cached]
    sparse = set(rng.choice(free, size=n_sparse, replace=False).tolist())
    return [(1, 0) if s in cached else (0, int(rng.integers(1, 4)) if s in sparse else 0) for s in range(n_steps)]
