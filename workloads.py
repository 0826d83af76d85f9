"""Seeded synthetic inputs for the MemoSight decode hot path.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark, so it deliberately holds NONE of the method's arithmetic: no RoPE, no
position-layout rule, no rounding rule, no allocator, no softmax.  It only draws
random numbers with the shapes, value distributions and structure of the
workloads (long chain-of-thought decode with compressed caches) and hands the
same bytes to either side.  It imports neither `oracle` nor the product package.

bfloat16 tensors are produced as uint16 bit patterns by cutting a float32 sample
down to its upper 16 bits (truncation, not a rounding rule): every value is then
exactly representable, so both sides read identical inputs.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 20260414
PAGE_SIZE = 16


def hash_stream(stream: Tuple[int, ...]) -> int:
    h = 1469598103934665603
    for s in stream:
        h ^= int(s) & 0xFFFFFFFFFFFFFFFF
        h = (h * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    return h


def make_rng(*stream: int) -> np.random.Generator:
    """Counter-based (Philox) generator; the `stream` integers select an independent stream."""
    return np.random.Generator(np.random.Philox(key=[BASE_SEED, hash_stream(stream)]))


def normal_f32(rng: np.random.Generator, shape, sigma: float = 1.0) -> np.ndarray:
    return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def normal_bf16_bits(rng: np.random.Generator, shape, sigma: float = 0.5) -> np.ndarray:
    """N(0, sigma) samples cut to bfloat16 bit patterns (uint16)."""
    x = normal_f32(rng, shape, sigma)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def bits_as_f32(bits: np.ndarray) -> np.ndarray:
    """Exact float32 view of uint16 bfloat16 bit patterns."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def normal_bf16_exact(rng: np.random.Generator, shape, sigma: float = 0.5) -> np.ndarray:
    """float32 array whose every value is exactly representable in bfloat16."""
    return bits_as_f32(normal_bf16_bits(rng, shape, sigma))


def ragged_lengths(rng: np.random.Generator, batch: int, lo: int, hi: int) -> List[int]:
    """Cache lengths drawn uniformly from [lo, hi]."""
    return [int(x) for x in rng.integers(lo, hi + 1, size=batch)]


def shuffled_page_tables(rng: np.random.Generator, n_pages: int, lengths: List[int]) -> List[List[int]]:
    """Disjoint page lists for each sequence taken from a random permutation of the pool."""
    counts = [-(-n // PAGE_SIZE) for n in lengths]
    assert sum(counts) <= n_pages
    perm = rng.permutation(n_pages)
    out, off = [], 0
    for c in counts:
        out.append([int(p) for p in perm[off:off + c]])
        off += c
    return out


def draft_and_target(rng: np.random.Generator, batch: int, n: int, vocab: int = 1000,
                     forced_prefix: Optional[List[int]] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Draft tokens and greedy targets, uniform over the vocabulary.

    With `forced_prefix[b] = a` the first a targets of sequence b are made equal to
    the drafts and (if a < n) the next one is made different, so that every
    acceptance length occurs.
    """
    draft = rng.integers(0, vocab, size=(batch, n)).astype(np.int32)
    target = rng.integers(0, vocab, size=(batch, n)).astype(np.int32)
    if forced_prefix is not None:
        for b, a in enumerate(forced_prefix):
            target[b, :a] = draft[b, :a]
            if a < n:
                target[b, a] = (draft[b, a] + 1 + rng.integers(0, vocab - 1)) % vocab
    return draft, target


# --------------------------------------------------------------------------
# named workload shapes
# --------------------------------------------------------------------------

@dataclass
class AttnShape:
    """Shape of one predict+verify attention call."""
    name: str
    dtype: str                 # "f32" or "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_verify: int
    n_foresight: int
    lengths: List[int]         # compressed cache length per sequence
    sigma: float
    rope_base: float = 10000.0
    n_layers: int = 1
    slack_pages: float = 0.10  # extra pool pages beyond what the sequences own
    shuffle_pages: bool = True

    @property
    def n_q(self) -> int:
        return self.n_verify + self.n_foresight

    @property
    def pages_owned(self) -> int:
        return sum(-(-n // PAGE_SIZE) for n in self.lengths)

    @property
    def n_pages(self) -> int:
        return int(self.pages_owned * (1.0 + self.slack_pages)) + 1

    def first_query_pid(self, b: int) -> int:
        """PID of the first verify token: caches hold about a third of the raw tokens."""
        return 3 * self.lengths[b] + 1


def config2() -> AttnShape:
    """Qwen2.5-7B-shaped layer, one sequence, 4096 cached tokens, 4 verify + 3 foresight."""
    return AttnShape("config2_b1_4k", "bf16", 1, 28, 4, 128, 4, 3, [4096], 0.5, 1000000.0)


def metric_point(batch: int = 32, length: int = 8192, n_layers: int = 1) -> AttnShape:
    """The headline point: batch 32, 8192 cached tokens each, 5 verify + 4 foresight."""
    return AttnShape(f"b{batch}_kv{length}", "bf16", batch, 28, 4, 128, 5, 4,
                     [length] * batch, 0.5, 1000000.0, n_layers=n_layers)


def config3(seed_stream: int = 3, batch: int = 32, lo: int = 1024, hi: int = 16384,
            n_layers: int = 1) -> AttnShape:
    """Ragged batch: lengths uniform in [1k, 16k], 5 verify + 4 foresight, shuffled pages."""
    rng = make_rng(seed_stream, 0)
    return AttnShape("config3_ragged", "bf16", batch, 28, 4, 128, 5, 4,
                     ragged_lengths(rng, batch, lo, hi), 0.5, 1000000.0, n_layers=n_layers)


@dataclass
class AttnInputs:
    shape: AttnShape
    page_tables: List[List[int]]
    pool: np.ndarray           # f32: float32 [layers, pages, Hkv, 2, 16, D]; bf16: uint16 same shape
    q: np.ndarray              # f32: float32; bf16: uint16 bit patterns  [B, n_q, Hq, D]
    k_new: np.ndarray          # [B, n_q, Hkv, D]
    v_new: np.ndarray
    first_pid: List[int] = field(default_factory=list)


def attention_inputs(shape: AttnShape, *stream: int, peaked: float = 0.0) -> AttnInputs:
    """Random pre-filled pool (cached K is taken as already rotated), page tables and queries.

    `peaked` > 0 multiplies that fraction of each sequence's cached keys by 8 (exact
    in either storage type), which widens the score range and stresses the softmax.
    """
    rng = make_rng(*stream, 11)
    pts = shuffled_page_tables(rng, shape.n_pages, shape.lengths) if shape.shuffle_pages else None
    if pts is None:
        pts, off = [], 0
        for n in shape.lengths:
            c = -(-n // PAGE_SIZE)
            pts.append(list(range(off, off + c)))
            off += c
    pool_shape = (shape.n_layers, shape.n_pages, shape.n_kv_heads, 2, PAGE_SIZE, shape.head_dim)
    b, nq = shape.batch, shape.n_q
    if shape.dtype == "bf16":
        gen = lambda shp: normal_bf16_bits(rng, shp, shape.sigma)
    else:
        gen = lambda shp: normal_f32(rng, shp, shape.sigma)
    pool = gen(pool_shape)
    q = gen((b, nq, shape.n_q_heads, shape.head_dim))
    k_new = gen((b, nq, shape.n_kv_heads, shape.head_dim))
    v_new = gen((b, nq, shape.n_kv_heads, shape.head_dim))
    if peaked > 0.0:
        for bi, n in enumerate(shape.lengths):
            cnt = max(1, int(n * peaked))
            toks = rng.choice(n, size=cnt, replace=False)
            for t in toks:
                blk = pool[:, pts[bi][t // PAGE_SIZE], :, 0, t % PAGE_SIZE, :]
                if shape.dtype == "bf16":
                    big = bits_as_f32(blk) * np.float32(8.0)
                    pool[:, pts[bi][t // PAGE_SIZE], :, 0, t % PAGE_SIZE, :] = \
                        (big.view(np.uint32) >> 16).astype(np.uint16)
                else:
                    pool[:, pts[bi][t // PAGE_SIZE], :, 0, t % PAGE_SIZE, :] = blk * np.float32(8.0)
    return AttnInputs(shape, pts, pool, q, k_new, v_new,
                      [shape.first_query_pid(i) for i in range(b)])
