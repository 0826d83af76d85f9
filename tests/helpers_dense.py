"""A second, deliberately dumb reference used only to pin the oracle.

Dense masked softmax over a FULL, uncompressed token sequence, with the boolean
attention mask written token pair by token pair from the paper's description
(Section 2.3, "Compression Attention" and "MTP Attention"), in python loops and
math.exp.  Rotary embedding comes from the public `transformers` routine, not
from the oracle.  Nothing here is imported by the oracle or by the product.
"""
import math

import torch
from transformers import LlamaConfig
from transformers.models.llama.modeling_llama import LlamaRotaryEmbedding, apply_rotary_pos_emb


def hf_rope(x, pids, base):
    """x: [T, H, D] float64 numpy; pids: [T] ints.  Rotated copy via the HF routine."""
    import numpy as np
    t, h, d = x.shape
    cfg = LlamaConfig(hidden_size=d * h, num_attention_heads=h, num_key_value_heads=h,
                      rope_theta=float(base), num_hidden_layers=1, intermediate_size=8,
                      vocab_size=8)
    emb = LlamaRotaryEmbedding(cfg)
    xt = torch.from_numpy(np.ascontiguousarray(x)).to(torch.float64).permute(1, 0, 2)[None]  # [1,H,T,D]
    cos, sin = emb(xt, torch.tensor(list(pids), dtype=torch.long)[None])
    out, _ = apply_rotary_pos_emb(xt, xt, cos.to(torch.float64), sin.to(torch.float64))
    return out[0].permute(1, 0, 2).numpy()


# token kinds in the full sequence
PROMPT, REASON, MEMORY, OUTPUT, FORESIGHT = "P", "R", "M", "O", "F"


def paper_mask(kinds, steps):
    """mask[i][j] = may token i attend to token j, from the paper's rules.

    kinds[i] in {P, R, M, O, F}; steps[i] = index of the reasoning step the token
    belongs to (prompt: -1; memory/output tokens carry the step they close).
      * everything is causal (j <= i);
      * nobody but the foresight token itself attends to a foresight token;
      * a token of step s does not attend to the reasoning tokens of steps < s;
      * it attends to the prompt, to memory and output tokens of earlier steps and to
        the earlier reasoning tokens of its own step.
    """
    n = len(kinds)
    m = [[False] * n for _ in range(n)]
    for i in range(n):
        for j in range(i + 1):
            if j == i:
                m[i][j] = True
                continue
            if kinds[j] == FORESIGHT:
                continue
            if kinds[j] == REASON and steps[j] < steps[i]:
                continue
            m[i][j] = True
    return m


def dense_masked_attention(q, k, v, mask, rows, scale):
    """q, k, v: python lists of vectors (already rotated); returns {row: out vector}."""
    out = {}
    d = len(v[0])
    for i in rows:
        idx = [j for j in range(len(k)) if mask[i][j]]
        s = [scale * sum(a * b for a, b in zip(q[i], k[j])) for j in idx]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        z = sum(e)
        out[i] = [sum(e[t] * v[idx[t]][c] for t in range(len(idx))) / z for c in range(d)]
    return out
