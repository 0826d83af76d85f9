"""Plain CPU oracle for the MemoSight per-step decode hot path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct definition
that the HIP library is checked against.  It shares no code with the HIP path,
imports nothing from the product package, and must only be imported by tests,
the smoke check and the benchmark's CPU-baseline leg.

Everything floating point is evaluated in float64 on inputs that were first
rounded to the storage type (float32 or bfloat16), so the oracle is the exact
masked-softmax attention over the surviving KV up to fp64 rounding.

What each function follows (MemoSight paper):
  * ama_count            -- Section 2.1.2, "Adaptive Memory Allocation": l = ceil(|R_i| / c)
  * upl_positions        -- Section 2.1.2, "Uniform Position Layout", its footnote on the
                            short last group, and Section 2.2 "Position ID Assignment"
                            (Figure 3: c = 3, span 1..3 -> memory PID 2)
  * output_token_pid     -- Section 2.2 "Position ID Assignment" (<o> gets last PID + 1)
  * foresight_pids       -- Section 2.1.1 (a foresight token's PID is one less than the
                            PID of the token it predicts; PIDs increase by one)
  * default_ctx_new      -- Section 2.1.1 / Section 2.3 "MTP Attention" (a foresight
                            token sees the regular prefix and itself, nothing else sees it)
  * rope                 -- Section 2.1.2 names RoPE as the positional mechanism; the
                            rotate-half convention of the evaluated model families is a
                            reading, pinned against the public library routine in tests
  * PagedCache.append    -- Algorithm 1, "S <- S (+) A"
  * PagedCache.compact   -- Section 2.1.2 and Algorithm 1 "UpdateCache" (evict the step's
                            regular tokens, keep its memory tokens)
  * attention            -- Section 2.3 "Compression Attention" / "MTP Attention",
                            Section 2.1.1 (Predict and Verify)
  * accept               -- footnote of Section 2.1.1 (accept the prefix of drafts that
                            coincide with the argmax predictions)

Parity pins (tests/test_oracle_*.py): printed worked values of Figure 3 and
Section 2.1.1, dense brute-force masked softmax written with python loops,
torch scaled_dot_product_attention reductions, the public rotary-embedding
routine of the `transformers` package, closed forms and invariants.
"""

from __future__ import annotations

import bisect
from typing import List, Optional, Sequence

import numpy as np

PAGE_SIZE = 16

F32 = "f32"
BF16 = "bf16"


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------

def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even); returns float32."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    out = rounded.astype(np.uint32).view(np.float32).reshape(a.shape)
    nan = np.isnan(a)
    if nan.any():
        out = out.copy()
        out[nan] = np.float32(np.nan)
    return out


def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round to the cache storage type; the result is held in float32."""
    if dtype == F32:
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == BF16:
        return round_bf16(np.asarray(x, dtype=np.float64).astype(np.float32))
    raise ValueError(f"unknown dtype {dtype!r}")


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Reinterpret uint16 bfloat16 bit patterns as float32 values (exact)."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------
# position layout helpers (integers only)
# --------------------------------------------------------------------------

def ama_count(n_tokens: int, c: int) -> int:
    """Number of memory tokens for a reasoning step of n_tokens at ratio c."""
    if n_tokens < 0 or c <= 0:
        raise ValueError("need n_tokens >= 0 and c > 0")
    return -(-n_tokens // c)


def upl_positions(first_pid: int, n_tokens: int, c: int) -> List[int]:
    """Memory-token PIDs for a step whose tokens hold PIDs first_pid .. first_pid+n-1.

    The step is cut into ceil(n/c) consecutive groups of c tokens (the last one
    may be shorter); each memory token takes the centre PID of its group.  For a
    group with an even number of tokens the lower of the two middle PIDs is taken
    (a reading: the paper only prints an odd-sized example).
    """
    out = []
    for g in range(ama_count(n_tokens, c)):
        lo = g * c
        hi = min(lo + c, n_tokens) - 1          # inclusive, step-local
        out.append(first_pid + (lo + hi) // 2)
    return out


def output_token_pid(last_pid: int) -> int:
    """PID of the <o> token that follows a step whose last token has PID last_pid."""
    return last_pid + 1


def next_step_first_pid(last_pid: int) -> int:
    """PID of the first token of the step after <o> (consecutive positions)."""
    return last_pid + 2


def foresight_pids(last_prefix_pid: int, d: int) -> List[int]:
    """PIDs of d foresight tokens appended after a prefix ending at last_prefix_pid.

    The j-th foresight token (j = 1..d) predicts the token at PID last+j+1 and
    holds the PID immediately before its target.
    """
    return [last_prefix_pid + j for j in range(1, d + 1)]


def default_ctx_new(n_verify: int, n_foresight: int) -> List[int]:
    """How many in-flight tokens (besides itself) each query sees.

    Verify token i is causal inside the verify block (sees i earlier ones).
    Every foresight token sees the whole verify block and no other foresight token.
    """
    return list(range(n_verify)) + [n_verify] * n_foresight


def per_position_layout(first_pid: int, n_verify: int, d: int):
    """Step layout with d foresight tokens behind every verify token (Section 2.2, "CoT
    Augmentation" and "Position ID Assignment"; Section 2.3, "MTP Attention").

    Queries: the n_verify verify tokens (PIDs first_pid ..), then, for verify token j in turn, its
    d foresight tokens.  Foresight token k = 1..d behind verify token j plays the role of the
    training-time foresight token placed before the token after j with offset d' = k: it holds the
    PID just before its target, pid_j + k, and sees what that next token would see of the step --
    verify tokens 0..j -- plus itself.  Returns (pids, ctx_new).
    """
    pids = [first_pid + j for j in range(n_verify)]
    ctx = list(range(n_verify))
    for j in range(n_verify):
        for k in range(1, d + 1):
            pids.append(first_pid + j + k)
            ctx.append(j + 1)
    return pids, ctx


def consecutive_memory_positions(last_pid: int, n_mem: int) -> List[int]:
    """Memory-token PIDs without UPL (Appendix B, "w/o UPL"; Section 2.1.2 on prior methods):
    consecutive new PIDs after the step's last token.  <o> then follows the last memory token."""
    return [last_pid + 1 + j for j in range(n_mem)]


def upl_positions_fixed(first_pid: int, n_tokens: int, n_mem: int) -> List[int]:
    """UPL for a fixed budget of n_mem memory tokens (Appendix B, "w/o AMA": 9 per step).

    A reading: the paper defines the groups only through the ratio c.  Here the step is cut into
    n_mem contiguous groups whose boundaries are floor(g * n / n_mem); a group left empty because
    the step has fewer tokens than memory tokens stands for the single token at its boundary.
    """
    if n_tokens < 1 or n_mem < 1:
        raise ValueError("need n_tokens >= 1 and n_mem >= 1")
    out = []
    for g in range(n_mem):
        lo = g * n_tokens // n_mem
        hi = (g + 1) * n_tokens // n_mem - 1
        if hi < lo:
            hi = lo
        out.append(first_pid + (lo + hi) // 2)
    return out


# --------------------------------------------------------------------------
# RoPE
# --------------------------------------------------------------------------

def rope_inv_freq(head_dim: int, base: float) -> np.ndarray:
    """inv_freq_i = base^(-2i/D), i < D/2, computed in double and rounded once to fp32."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return (np.float64(base) ** (-2.0 * i / head_dim)).astype(np.float32)


def rope(x: np.ndarray, pos: np.ndarray, inv_freq: np.ndarray) -> np.ndarray:
    """Rotate x[..., D] by integer positions pos[...] (broadcast over leading dims).

    Pairing is (i, i + D/2).  The angle is the fp32 product of the fp32 position
    and the fp32 inverse frequency; sine and cosine of that fp32 angle and the
    rotation itself are evaluated in float64.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    p32 = np.asarray(pos).astype(np.float32)
    theta = (p32[..., None] * inv_freq.astype(np.float32)).astype(np.float32)
    theta = theta.astype(np.float64)
    c, s = np.cos(theta), np.sin(theta)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


# --------------------------------------------------------------------------
# paged KV cache
# --------------------------------------------------------------------------

class OutOfPages(Exception):
    pass


class PagedCache:
    """Logical KV cache S of Algorithm 1, realised as fixed 16-token pages.

    pool[layer, page, kv_head, 0 (K) | 1 (V), slot, d] holds storage-rounded
    values as float32.  Logical token t of a sequence lives in page
    page_table[t // 16], slot t % 16.  The page table is shared by all layers.

    Allocation policy (needed so page tables can be compared bit for bit):
    the free set is ordered and the lowest free page index is always taken;
    released pages go back into the set.
    """

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int, n_pages: int,
                 dtype: str = BF16, rope_base: float = 10000.0, max_seqs: int = 64,
                 pool: Optional[np.ndarray] = None):
        self.n_layers, self.n_kv_heads, self.head_dim = n_layers, n_kv_heads, head_dim
        self.n_pages, self.dtype, self.rope_base = n_pages, dtype, rope_base
        self.max_seqs = max_seqs
        shape = (n_layers, n_pages, n_kv_heads, 2, PAGE_SIZE, head_dim)
        if pool is None:
            pool = np.zeros(shape, dtype=np.float32)
        assert pool.shape == shape and pool.dtype == np.float32
        self.pool = pool
        self.inv_freq = rope_inv_freq(head_dim, rope_base)
        self.free: List[int] = list(range(n_pages))      # kept sorted
        self.page_table: dict[int, List[int]] = {}
        self.seq_len: dict[int, int] = {}
        self.peak_pages = 0

    # ---- allocator -------------------------------------------------------
    def _alloc(self) -> int:
        if not self.free:
            raise OutOfPages()
        p = self.free.pop(0)
        self.peak_pages = max(self.peak_pages, self.n_pages - len(self.free))
        return p

    def _release(self, page: int) -> None:
        bisect.insort(self.free, page)

    def free_page_count(self) -> int:
        return len(self.free)

    # ---- sequences -------------------------------------------------------
    def seq_create(self) -> int:
        for sid in range(self.max_seqs):
            if sid not in self.seq_len:
                self.page_table[sid] = []
                self.seq_len[sid] = 0
                return sid
        raise RuntimeError("no free sequence id")

    def seq_import(self, length: int, pages: Sequence[int]) -> int:
        """Adopt an already-filled set of pages (in logical order) as a new sequence."""
        pages = [int(p) for p in pages]
        if len(pages) != -(-length // PAGE_SIZE):
            raise ValueError("page count does not match length")
        if len(set(pages)) != len(pages):
            raise ValueError("duplicate page")
        for p in pages:
            i = bisect.bisect_left(self.free, p)
            if i >= len(self.free) or self.free[i] != p:
                raise ValueError("page not free")
        sid = self.seq_create()
        for p in pages:
            self.free.pop(bisect.bisect_left(self.free, p))
        self.page_table[sid] = pages
        self.seq_len[sid] = int(length)
        self.peak_pages = max(self.peak_pages, self.n_pages - len(self.free))
        return sid

    def seq_free(self, sid: int) -> None:
        for p in self.page_table.pop(sid):
            self._release(p)
        del self.seq_len[sid]

    # ---- row access ------------------------------------------------------
    def _slot(self, sid: int, t: int):
        return self.page_table[sid][t // PAGE_SIZE], t % PAGE_SIZE

    def _push_row(self, sid: int, k_rows: np.ndarray, v_rows: np.ndarray) -> None:
        """k_rows, v_rows: [layers, Hkv, D], already storage-rounded float32."""
        t = self.seq_len[sid]
        if t % PAGE_SIZE == 0:
            self.page_table[sid].append(self._alloc())
        page, slot = self._slot(sid, t)
        self.pool[:, page, :, 0, slot, :] = k_rows
        self.pool[:, page, :, 1, slot, :] = v_rows
        self.seq_len[sid] = t + 1

    def gather(self, layer: int, sid: int):
        """Dense copies K[L, Hkv, D], V[L, Hkv, D] (float32) of a sequence in logical order."""
        n = self.seq_len[sid]
        pt = np.asarray(self.page_table[sid], dtype=np.int64)
        if n == 0:
            z = np.zeros((0, self.n_kv_heads, self.head_dim), np.float32)
            return z, z.copy()
        blk = self.pool[layer, pt]                       # [pages, Hkv, 2, 16, D]
        k = blk[:, :, 0].transpose(0, 2, 1, 3).reshape(-1, self.n_kv_heads, self.head_dim)[:n]
        v = blk[:, :, 1].transpose(0, 2, 1, 3).reshape(-1, self.n_kv_heads, self.head_dim)[:n]
        return k, v

    # ---- Algorithm 1: S <- S (+) A ----------------------------------------
    def append(self, seq_ids: Sequence[int], n_tok: Sequence[int], k: np.ndarray,
               v: np.ndarray, pos_ids: Sequence[int], apply_rope: bool = True) -> None:
        """Append tokens at the logical end of each sequence, in argument order.

        k, v: [layers, sum(n_tok), Hkv, D]; pos_ids: [sum(n_tok)].  K is rotated by
        its PID unless it already is; both are rounded to the storage type.  A page is
        taken exactly when the length before the push is a multiple of 16.  If the
        pool cannot hold the whole call, nothing changes and OutOfPages is raised.
        """
        k = np.asarray(k, dtype=np.float64)
        v = np.asarray(v, dtype=np.float64)
        need = 0
        for sid, n in zip(seq_ids, n_tok):
            cur = self.seq_len[sid]
            need += -(-(cur + n) // PAGE_SIZE) - len(self.page_table[sid])
        if need > len(self.free):
            raise OutOfPages()
        pos = np.asarray(pos_ids, dtype=np.int64)
        if apply_rope:
            k = rope(k, pos[None, :, None], self.inv_freq)
        ks = round_storage(k, self.dtype)
        vs = round_storage(v, self.dtype)
        off = 0
        for sid, n in zip(seq_ids, n_tok):
            for j in range(n):
                self._push_row(sid, ks[:, off + j], vs[:, off + j])
            off += n

    # ---- Algorithm 1: UpdateCache ------------------------------------------
    def compact(self, seq_ids: Sequence[int], seg_begin: Sequence[int], seg_len: Sequence[int],
                n_mem: Sequence[int], mem_k: np.ndarray, mem_v: np.ndarray,
                mem_pos: Sequence[int], apply_rope: bool = True) -> None:
        """Replace logical rows [seg_begin, seg_begin+seg_len) by n_mem memory-token rows.

        mem_k, mem_v: [layers, sum(n_mem), Hkv, D]; mem_pos: [sum(n_mem)].
        Rows after the segment (normally none: Algorithm 1 compacts the cache
        suffix) keep their stored values and follow the memory tokens.

        Page policy, per sequence in argument order: pages that hold any row below
        seg_begin are kept; every later page of the sequence is released first;
        then the memory rows and the tail rows are pushed one by one, each new
        page being the lowest free index.
        """
        mem_k = np.asarray(mem_k, dtype=np.float64)
        mem_v = np.asarray(mem_v, dtype=np.float64)
        mpos = np.asarray(mem_pos, dtype=np.int64)
        # validate first so that a bad call leaves the state untouched
        for sid, s, n, l in zip(seq_ids, seg_begin, seg_len, n_mem):
            L = self.seq_len[sid]
            if s < 0 or n < 0 or l < 0 or s + n > L:
                raise ValueError("segment out of range")
        # page need can only exceed what is released if n_mem > seg_len
        sim_free = len(self.free)
        for sid, s, n, l in zip(seq_ids, seg_begin, seg_len, n_mem):
            L = self.seq_len[sid]
            keep = -(-s // PAGE_SIZE)
            sim_free += len(self.page_table[sid]) - keep
            sim_free -= -(-(L - n + l) // PAGE_SIZE) - keep
            if sim_free < 0:
                raise OutOfPages()
        if apply_rope:
            mem_k = rope(mem_k, mpos[None, :, None], self.inv_freq)
        mk = round_storage(mem_k, self.dtype)
        mv = round_storage(mem_v, self.dtype)
        off = 0
        for sid, s, n, l in zip(seq_ids, seg_begin, seg_len, n_mem):
            L = self.seq_len[sid]
            tail_k = [None] * (L - s - n)
            tail_v = [None] * (L - s - n)
            for idx, t in enumerate(range(s + n, L)):
                page, slot = self._slot(sid, t)
                tail_k[idx] = self.pool[:, page, :, 0, slot, :].copy()
                tail_v[idx] = self.pool[:, page, :, 1, slot, :].copy()
            keep = -(-s // PAGE_SIZE)
            for p in self.page_table[sid][keep:]:
                self._release(p)
            del self.page_table[sid][keep:]
            self.seq_len[sid] = s
            for j in range(l):
                self._push_row(sid, mk[:, off + j], mv[:, off + j])
            for tk, tv in zip(tail_k, tail_v):
                self._push_row(sid, tk, tv)
            off += l

    # ---- integrity ---------------------------------------------------------
    def check_integrity(self) -> None:
        owned = []
        for sid, pt in self.page_table.items():
            assert len(pt) == -(-self.seq_len[sid] // PAGE_SIZE), "page count vs length"
            owned += pt
        assert len(set(owned)) == len(owned), "page owned twice"
        assert not (set(owned) & set(self.free)), "page both owned and free"
        assert sorted(owned + self.free) == list(range(self.n_pages)), "page leaked"
        assert self.free == sorted(self.free)


# --------------------------------------------------------------------------
# fused Predict+Verify attention
# --------------------------------------------------------------------------

def attention_rows(cache: PagedCache, layer: int, sid: int, q: np.ndarray, k_new: np.ndarray,
                   v_new: np.ndarray, pos: Sequence[int], ctx_new: Sequence[int],
                   scale: Optional[float] = None,
                   rows: Optional[Sequence[tuple]] = None) -> np.ndarray:
    """Attention outputs of one sequence.

    q [n_q, Hq, D]; k_new, v_new [n_q, Hkv, D] (K not yet rotated); pos [n_q];
    ctx_new [n_q].  Query i sees every cached token of the sequence, the in-flight
    tokens j < ctx_new[i], and itself.  Query head h reads KV head h // (Hq / Hkv).
    Returns out [n_q, Hq, D] in float64; if `rows` (a list of (i, h)) is given only
    those rows are computed and the rest is NaN.
    """
    q = np.asarray(q, dtype=np.float64)
    k_new = np.asarray(k_new, dtype=np.float64)
    v_new = np.asarray(v_new, dtype=np.float64)
    n_q, n_qh, d = q.shape
    n_kvh = cache.n_kv_heads
    group = n_qh // n_kvh
    assert group * n_kvh == n_qh and d == cache.head_dim
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(float(d))
    pos = np.asarray(pos, dtype=np.int64)
    qr = rope(q, pos[:, None], cache.inv_freq)            # [n_q, Hq, D]
    kr = rope(k_new, pos[:, None], cache.inv_freq)        # [n_q, Hkv, D]
    kc, vc = cache.gather(layer, sid)                     # [L, Hkv, D]
    kc = kc.astype(np.float64)
    vc = vc.astype(np.float64)
    out = np.full((n_q, n_qh, d), np.nan, dtype=np.float64)
    todo = rows if rows is not None else [(i, h) for i in range(n_q) for h in range(n_qh)]
    for i, h in todo:
        g = h // group
        vis = [j for j in range(n_q) if j < ctx_new[i] or j == i]
        keys = np.concatenate([kc[:, g, :], kr[vis, g, :]], axis=0)
        vals = np.concatenate([vc[:, g, :], v_new[vis, g, :]], axis=0)
        s = (keys @ qr[i, h]) * scale
        p = np.exp(s - s.max())
        out[i, h] = (p / p.sum()) @ vals
    return out


def attention(cache: PagedCache, layer: int, seq_ids: Sequence[int], n_verify: int,
              n_foresight: int, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
              pos_ids: np.ndarray, ctx_new: Optional[np.ndarray] = None,
              scale: Optional[float] = None) -> np.ndarray:
    """Batched Predict+Verify attention.

    q [B, n_q, Hq, D]; k_new, v_new [B, n_q, Hkv, D]; pos_ids [B, n_q];
    ctx_new [B, n_q] or None for the default layout.  Inputs are taken as given
    (the caller rounds them to the storage type first).  Returns float64
    [B, n_q, Hq, D].
    """
    n_q = n_verify + n_foresight
    q = np.asarray(q)
    assert q.shape[1] == n_q
    outs = []
    for b, sid in enumerate(seq_ids):
        cn = default_ctx_new(n_verify, n_foresight) if ctx_new is None else list(ctx_new[b])
        outs.append(attention_rows(cache, layer, sid, q[b], k_new[b], v_new[b],
                                   pos_ids[b], cn, scale))
    return np.stack(outs, axis=0)


# --------------------------------------------------------------------------
# greedy longest-prefix acceptance
# --------------------------------------------------------------------------

def accept(draft: np.ndarray, target: np.ndarray, stop_ids: Sequence[int] = ()):
    """Per sequence: number of leading drafts equal to the model's own argmax tokens.

    draft, target: int [B, n], aligned (target[b, j] is the greedy token for the
    slot draft[b, j] fills).  If stop ids are given, acceptance ends just after the
    first accepted stop id so that a finished step is always a cache suffix.
    Returns (accept_len [B], next_token [B]); next_token is target[b, a] when
    a < n (the model's own token at the first non-accepted slot), else -1.
    """
    draft = np.asarray(draft, dtype=np.int64)
    target = np.asarray(target, dtype=np.int64)
    b_sz, n = draft.shape
    stops = set(int(s) for s in stop_ids)
    acc = np.zeros(b_sz, dtype=np.int32)
    nxt = np.full(b_sz, -1, dtype=np.int32)
    for b in range(b_sz):
        a = 0
        while a < n and draft[b, a] == target[b, a]:
            a += 1
            if int(draft[b, a - 1]) in stops:
                break
        acc[b] = a
        if a < n:
            nxt[b] = target[b, a]
    return acc, nxt
