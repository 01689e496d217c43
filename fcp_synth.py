"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This module draws random lengths and random bf16 tensors and does nothing else:
none of the method's arithmetic (no attention, no chunking, no merge) lives here,
so both the CPU oracle and the HIP path can be fed from it without sharing code.

Workloads (stand-ins for the long-tailed text / video corpora the paper trains
on, Fig. 1a; no item of those corpora is used):

  cfg 0  one sequence, L=512, degree 1, 4/4 heads, D=64, forward only
  cfg 1  one sequence, L=4096, degree 3, 8/8 heads, D=128, report rank 1
  cfg 2  24 lognormal(6.5, 1.2) lengths totalling 32768, degree ceil(len/4096)<=6,
         32/8 heads, D=128, report rank 0            (the benchmark workload)
  cfg 3  one sequence, L=131072, degree 5, 32/8 heads, D=128, report rank 2
  cfg 4  one 49152-token sequence (degree 6) + 64 lengths in [128, 512] totalling
         16384, 40/8 heads, D=128, report rank 0

Draw order for a workload: lengths first, then Q, K, V, dO (standard normal,
float32, rounded to bf16 with round-to-nearest-even), all from one
numpy.random.default_rng(seed).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


# ----------------------------------------------------------------------------
# bf16 <-> float conversions (storage format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    out = r.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = out.copy()
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


# ----------------------------------------------------------------------------
# workload descriptions
# ----------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    seq_lens: np.ndarray          # int32 [n_seqs]
    cp_degree: np.ndarray         # int32 [n_seqs]
    hq: int
    hkv: int
    head_dim: int
    rank: int                     # the rank whose share is reported
    backward: bool = True
    seed: int = 0
    _rng: np.random.Generator = field(default=None, repr=False)

    @property
    def total_tokens(self) -> int:
        return int(self.seq_lens.sum())

    @property
    def cu_seqlens(self) -> np.ndarray:
        cu = np.zeros(len(self.seq_lens) + 1, dtype=np.int32)
        np.cumsum(self.seq_lens, out=cu[1:])
        return cu

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


def degree_rule(lens: np.ndarray, per_rank: int = 4096, cap: int = 6) -> np.ndarray:
    """Per-sequence CP degree = ceil(len / per_rank), capped."""
    d = (np.asarray(lens, dtype=np.int64) + per_rank - 1) // per_rank
    return np.clip(d, 1, cap).astype(np.int32)


def lognormal_lengths(rng: np.random.Generator, n: int = 24, total: int = 32768,
                      mu: float = 6.5, sigma: float = 1.2,
                      lo: int = 64, hi: int = 16384, mult: int = 16) -> np.ndarray:
    """n long-tailed lengths: lognormal, clipped to [lo, hi], rounded to a multiple
    of `mult`; the last one is set so the sum is `total`; the vector is redrawn
    while the last one falls outside [lo, hi]."""
    while True:
        x = rng.lognormal(mu, sigma, size=n - 1)
        x = np.clip(x, lo, hi)
        x = (np.round(x / mult) * mult).astype(np.int64)
        x = np.clip(x, lo, hi)
        last = total - int(x.sum())
        if lo <= last <= hi:
            return np.concatenate([x, [last]]).astype(np.int32)


def uniform_lengths(rng: np.random.Generator, n: int = 64, total: int = 16384,
                    lo: int = 128, hi: int = 512) -> np.ndarray:
    """n lengths uniform in [lo, hi]; last adjusted to hit `total`; redrawn while
    the last one falls outside [lo, hi]."""
    while True:
        x = rng.integers(lo, hi + 1, size=n - 1).astype(np.int64)
        last = total - int(x.sum())
        if lo <= last <= hi:
            return np.concatenate([x, [last]]).astype(np.int32)


def make_workload(cfg: int, seed: int = 0) -> Workload:
    rng = np.random.default_rng(seed)
    if cfg == 0:
        wl = Workload("L512_d1_h4x4_D64", np.array([512], np.int32), np.array([1], np.int32),
                      4, 4, 64, rank=0, backward=False)
    elif cfg == 1:
        wl = Workload("L4096_d3_h8x8_D128", np.array([4096], np.int32), np.array([3], np.int32),
                      8, 8, 128, rank=1)
    elif cfg == 2:
        lens = lognormal_lengths(rng)
        wl = Workload("packed32k_lognormal24_h32x8_D128", lens, degree_rule(lens), 32, 8, 128, rank=0)
    elif cfg == 3:
        wl = Workload("L131072_d5_h32x8_D128", np.array([131072], np.int32), np.array([5], np.int32),
                      32, 8, 128, rank=2)
    elif cfg == 4:
        shorts = uniform_lengths(rng)
        lens = np.concatenate([np.array([49152], np.int32), shorts]).astype(np.int32)
        deg = np.concatenate([np.array([6], np.int32), np.ones(64, np.int32)]).astype(np.int32)
        wl = Workload("mm65k_1x49152_64short_h40x8_D128", lens, deg, 40, 8, 128, rank=0)
    else:
        raise ValueError(f"unknown workload {cfg}")
    wl.seed = seed
    wl._rng = rng
    return wl


def image_spans(seq_lens, seed: int = 0, span_len: int = 576, image_fraction: float = 0.35):
    """Full-attention spans of a synthetic multimodal batch: every sequence longer than one image gets images of
    `span_len` tokens (a 24 x 24 patch grid) separated by text runs, until about `image_fraction` of its tokens
    are image tokens; shorter sequences stay text only.  Returns [(seq, start, len), ...] sorted by (seq, start)."""
    rng = np.random.default_rng(seed + 77)
    spans = []
    for k, L in enumerate(int(x) for x in seq_lens):
        n_img = int(L * image_fraction) // span_len
        if n_img == 0:
            continue
        text = L - n_img * span_len
        cuts = np.sort(rng.integers(0, text + 1, size=n_img))     # text tokens before each image
        for i, c in enumerate(cuts):
            spans.append((k, int(c) + i * span_len, span_len))
    return spans


def custom_workload(seq_lens, cp_degree, hq, hkv, head_dim, rank=0, seed=0, name="custom") -> Workload:
    wl = Workload(name, np.asarray(seq_lens, np.int32), np.asarray(cp_degree, np.int32),
                  hq, hkv, head_dim, rank=rank, seed=seed)
    wl._rng = np.random.default_rng(seed)
    return wl


def draw_tensor_bits(rng: np.random.Generator, shape, block_rows: int = 1 << 14) -> np.ndarray:
    """Standard-normal float32 rounded to bf16 bits, drawn in row blocks to bound memory.
    The stream of draws is the same as one call of standard_normal over the whole shape."""
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(shape[0], -1)
    for r0 in range(0, shape[0], block_rows):
        r1 = min(shape[0], r0 + block_rows)
        blk = rng.standard_normal((r1 - r0, flat.shape[1]), dtype=np.float32)
        flat[r0:r1] = f32_to_bf16_bits(blk)
    return out


def draw_qkvdo(wl: Workload):
    """Q [T,Hq,D], K [T,Hkv,D], V [T,Hkv,D], dO [T,Hq,D] as bf16 bit patterns (uint16),
    for the unsharded packed batch (T = total tokens), in that draw order."""
    rng = wl._rng
    T, D = wl.total_tokens, wl.head_dim
    q = draw_tensor_bits(rng, (T, wl.hq, D))
    k = draw_tensor_bits(rng, (T, wl.hkv, D))
    v = draw_tensor_bits(rng, (T, wl.hkv, D))
    do = draw_tensor_bits(rng, (T, wl.hq, D))
    return q, k, v, do
