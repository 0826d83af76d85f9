"""CPU oracle of one full MemoSight decode step (test infrastructure only -- never imported by the
product path).

Scope: Algorithm 1's SpeculativeStep (Appendix A) on the models the paper fine-tunes (Section 3.1:
Qwen2.5-7B, Llama-3.1-8B).  The paper does not restate the decoder block; it is the public
pre-norm architecture of those models -- RMSNorm, Q/K/V projections (with bias in Qwen2.5), rotary
attention with grouped KV heads, output projection, SwiGLU MLP, final norm and LM head -- and this
file writes it out in plain numpy fp64 around the attention oracle.  It is pinned against the
`transformers` implementation of that architecture in tests/test_oracle_decoder.py (tiny random
model, the paper's attention mask and position ids).

Everything is computed in fp64 without intermediate rounding; only the K/V rows that enter the
cache are rounded to the cache's storage type (by the cache itself).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

from . import memosight_oracle as O


@dataclass
class LayerWeights:
    ln1: np.ndarray          # [H]        RMSNorm weight before attention
    wq: np.ndarray           # [Hq*D, H]
    bq: Optional[np.ndarray]  # [Hq*D] or None
    wk: np.ndarray           # [Hkv*D, H]
    bk: Optional[np.ndarray]
    wv: np.ndarray           # [Hkv*D, H]
    bv: Optional[np.ndarray]
    wo: np.ndarray           # [H, Hq*D]
    ln2: np.ndarray          # [H]        RMSNorm weight before the MLP
    w_gate: np.ndarray       # [I, H]
    w_up: np.ndarray         # [I, H]
    w_down: np.ndarray       # [H, I]


@dataclass
class DecoderWeights:
    embed: np.ndarray        # [V, H]
    layers: List[LayerWeights]
    norm: np.ndarray         # [H]        final RMSNorm weight
    lm_head: np.ndarray      # [V, H]
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    eps: float = 1e-6


def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * w over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * w


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def _linear(x, w, b=None):
    y = x @ np.asarray(w, dtype=np.float64).T
    return y if b is None else y + b


@dataclass
class StepResult:
    logits: np.ndarray       # [B, n_q, V] fp64
    k_new: np.ndarray        # [L, B, n_q, Hkv, D] unrotated keys of the step's tokens
    v_new: np.ndarray        # [L, B, n_q, Hkv, D]
    hidden: np.ndarray       # [B, n_q, H] before the final norm
    targets: np.ndarray = field(default=None)   # [B, n_q] greedy tokens


def speculative_step(wts: DecoderWeights, cache: "O.PagedCache", seq_ids: Sequence[int], tokens: np.ndarray,
                     pos: np.ndarray, n_verify: int, n_foresight: int,
                     ctx_new: Optional[np.ndarray] = None) -> StepResult:
    """One forward pass of the model over the step's tokens (Algorithm 1, SpeculativeStep; the
    fused Predict + Verify pass of Section 2.1.1): tokens [B, n_q] are the verify block followed
    by the foresight tokens, pos their position ids.  The cache is read, not changed; the K/V of
    the step's tokens are returned so the caller can append the accepted ones.

    Greedy targets take the lowest index among equal maxima.
    """
    tokens = np.asarray(tokens)
    B, n_q = tokens.shape
    assert n_q == n_verify + n_foresight
    hq, hkv, d = wts.n_q_heads, wts.n_kv_heads, wts.head_dim
    h = np.asarray(wts.embed, dtype=np.float64)[tokens]                     # [B, n_q, H]
    ks, vs = [], []
    for li, lw in enumerate(wts.layers):
        x = rmsnorm(h, lw.ln1, wts.eps)
        q = _linear(x, lw.wq, lw.bq).reshape(B, n_q, hq, d)
        k = _linear(x, lw.wk, lw.bk).reshape(B, n_q, hkv, d)
        v = _linear(x, lw.wv, lw.bv).reshape(B, n_q, hkv, d)
        attn = O.attention(cache, li, list(seq_ids), n_verify, n_foresight, q, k, v, pos, ctx_new, None)
        h = h + _linear(attn.reshape(B, n_q, hq * d), lw.wo)
        x = rmsnorm(h, lw.ln2, wts.eps)
        h = h + _linear(silu(_linear(x, lw.w_gate)) * _linear(x, lw.w_up), lw.w_down)
        ks.append(k)
        vs.append(v)
    logits = _linear(rmsnorm(h, wts.norm, wts.eps), wts.lm_head)
    res = StepResult(logits, np.stack(ks), np.stack(vs), h)
    res.targets = np.argmax(logits, axis=-1).astype(np.int64)              # first maximum wins
    return res


def greedy_accept(verify_tokens: np.ndarray, targets: np.ndarray, stop_ids: Sequence[int] = ()):
    """Acceptance for a verify block [t_0, draft_1, .., draft_{n-1}] (t_0 is already decided: it
    is the previous step's next token).  targets[j] is the greedy token after verify token j, so
    draft_{j+1} is accepted while it equals targets[j] (footnote of Section 2.1.1).  Returns
    (n_commit, next_token) per sequence: how many verify tokens enter the cache (1 + accepted
    drafts) and the token that follows them.
    """
    verify_tokens = np.asarray(verify_tokens)
    B, n = verify_tokens.shape
    n_commit, nxt = [], []
    for b in range(B):
        a, _ = O.accept(verify_tokens[b:b + 1, 1:], np.asarray(targets)[b:b + 1, :n - 1], stop_ids)
        c = 1 + int(a[0])
        n_commit.append(c)
        nxt.append(int(targets[b, c - 1]))
    return n_commit, nxt
