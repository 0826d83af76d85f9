"""Pins the full-decode-step oracle against the public implementation of the architecture.

The reference side is `transformers`' Qwen2 model (tiny random configuration, fp64, eager
attention) run ONCE over the full, uncompressed token sequence with the attention mask written
from the paper's rules (tests/helpers_dense.py) and the paper's position ids.  The oracle side
walks Algorithm 1 (Appendix A): prefill, a reasoning step, the memory-token pass, compaction, the
next step's prefix and finally a fused verify + foresight pass -- the cache only ever holds what
compression kept.  Logits must agree at every position.
"""
import numpy as np
import pytest
import torch

from tests import helpers_dense as H
from oracle import decoder_oracle as DO
from oracle import memosight_oracle as O


def tiny_model(seed, hq=4, hkv=2, d=16, layers=2, vocab=50, inter=96):
    from transformers import Qwen2Config, Qwen2ForCausalLM
    torch.manual_seed(seed)
    cfg = Qwen2Config(hidden_size=hq * d, intermediate_size=inter, num_hidden_layers=layers,
                      num_attention_heads=hq, num_key_value_heads=hkv, vocab_size=vocab, rope_theta=1e6,
                      rms_norm_eps=1e-6, max_position_embeddings=512, tie_word_embeddings=False,
                      attn_implementation="eager")
    model = Qwen2ForCausalLM(cfg).double().eval()
    with torch.no_grad():                       # default init leaves biases at zero and norms at one
        for n, p in model.named_parameters():
            if n.endswith("bias"):
                p.normal_(0.0, 0.3)
            elif "norm" in n:
                p.uniform_(0.5, 1.5)
            else:
                p.normal_(0.0, 0.15)
    sd = {k: v.detach().numpy().astype(np.float64) for k, v in model.state_dict().items()}
    lay = []
    for i in range(layers):
        p = f"model.layers.{i}."
        lay.append(DO.LayerWeights(
            ln1=sd[p + "input_layernorm.weight"],
            wq=sd[p + "self_attn.q_proj.weight"], bq=sd[p + "self_attn.q_proj.bias"],
            wk=sd[p + "self_attn.k_proj.weight"], bk=sd[p + "self_attn.k_proj.bias"],
            wv=sd[p + "self_attn.v_proj.weight"], bv=sd[p + "self_attn.v_proj.bias"],
            wo=sd[p + "self_attn.o_proj.weight"], ln2=sd[p + "post_attention_layernorm.weight"],
            w_gate=sd[p + "mlp.gate_proj.weight"], w_up=sd[p + "mlp.up_proj.weight"],
            w_down=sd[p + "mlp.down_proj.weight"]))
    wts = DO.DecoderWeights(embed=sd["model.embed_tokens.weight"], layers=lay, norm=sd["model.norm.weight"],
                            lm_head=sd["lm_head.weight"], n_q_heads=hq, n_kv_heads=hkv, head_dim=d, eps=1e-6)
    return model, wts


def test_rmsnorm_and_silu_closed_forms():
    x = np.array([[3.0, 4.0]])
    assert np.allclose(DO.rmsnorm(x, np.array([1.0, 2.0]), 0.0), [[3 / np.sqrt(12.5), 8 / np.sqrt(12.5)]])
    assert np.allclose(DO.rmsnorm(7.0 * x, np.ones(2), 0.0), DO.rmsnorm(x, np.ones(2), 0.0))   # scale invariant
    assert DO.silu(np.array([0.0]))[0] == 0.0
    assert np.isclose(DO.silu(np.array([1.0]))[0], 1.0 / (1.0 + np.exp(-1.0)))
    assert np.isclose(DO.silu(np.array([-30.0]))[0], 0.0, atol=1e-11)


@pytest.mark.parametrize("seed,n_verify,n_foresight", [(1, 3, 2), (2, 1, 3), (3, 4, 0)])
def test_algorithm1_walk_matches_transformers_on_the_full_sequence(seed, n_verify, n_foresight):
    model, wts = tiny_model(seed)
    rng = np.random.default_rng(seed)
    c = 3
    n_p, n_r1, n_r2 = 5, 6, 3
    # full sequence: P | R_1 | M_1 (2 memory tokens) <o> | R_2 prefix | verify | foresight
    kinds = ["P"] * n_p + ["R"] * n_r1 + ["M", "M", "O"] + ["R"] * n_r2 + ["R"] * n_verify + ["F"] * n_foresight
    steps = [-1] * n_p + [0] * n_r1 + [0, 0, 0] + [1] * (n_r2 + n_verify + n_foresight)
    first_r1 = n_p + 1
    mem_pids = [first_r1 + 1, first_r1 + 4]                  # centres of {6,7,8} and {9,10,11}: written by hand
    o_pid = first_r1 + n_r1                                   # the position after the step's last token
    first_r2 = o_pid + 1
    pids = (list(range(1, n_p + 1)) + list(range(first_r1, first_r1 + n_r1)) + mem_pids + [o_pid] +
            list(range(first_r2, first_r2 + n_r2 + n_verify + n_foresight)))
    T = len(kinds)
    tokens = rng.integers(0, 50, size=T)
    mask = torch.tensor(H.paper_mask(kinds, steps))
    add = torch.zeros(T, T, dtype=torch.float64).masked_fill(~mask, float("-inf"))
    with torch.no_grad():
        ref = model(input_ids=torch.tensor(tokens)[None], attention_mask=add[None, None],
                    position_ids=torch.tensor(pids)[None]).logits[0].numpy()

    # ---- the oracle walks Algorithm 1 with a cache that only holds what compression keeps
    cache = O.PagedCache(len(wts.layers), wts.n_kv_heads, wts.head_dim, n_pages=8, dtype=O.F32, rope_base=1e6)
    sid = cache.seq_create()
    got = np.full_like(ref, np.nan)

    def forward(lo, hi, nv, nf):
        r = DO.speculative_step(wts, cache, [sid], tokens[None, lo:hi], np.asarray(pids)[None, lo:hi], nv, nf)
        got[lo:hi] = r.logits[0]
        return r

    r = forward(0, n_p, n_p, 0)                                               # prefill
    cache.append([sid], [n_p], r.k_new[:, 0], r.v_new[:, 0], pids[:n_p])
    lo = n_p
    r = forward(lo, lo + n_r1, n_r1, 0)                                       # reasoning step 1
    cache.append([sid], [n_r1], r.k_new[:, 0], r.v_new[:, 0], pids[lo:lo + n_r1])
    lo += n_r1
    assert pids[lo:lo + 2] == O.upl_positions(first_r1, n_r1, c) and pids[lo + 2] == O.output_token_pid(first_r1 + n_r1 - 1)
    r = forward(lo, lo + 3, 3, 0)                                             # memory tokens and <o>
    cache.compact([sid], [n_p], [n_r1], [3], r.k_new[:, 0], r.v_new[:, 0], pids[lo:lo + 3])
    assert cache.seq_len[sid] == n_p + 3
    lo += 3
    r = forward(lo, lo + n_r2, n_r2, 0)                                       # prefix of step 2
    cache.append([sid], [n_r2], r.k_new[:, 0], r.v_new[:, 0], pids[lo:lo + n_r2])
    lo += n_r2
    r = forward(lo, T, n_verify, n_foresight)                                 # fused verify + foresight
    assert not np.isnan(got).any()
    assert np.abs(got - ref).max() < 2e-5 * max(1.0, np.abs(ref).max())      # fp32 storage of cached K/V
    assert np.array_equal(r.targets[0], ref[lo:].argmax(axis=-1))


def test_greedy_accept_prefix_semantics():
    verify = np.array([[7, 3, 4, 5], [7, 3, 9, 5], [7, 8, 4, 5], [1, 2, 3, 4]])
    targets = np.array([[3, 4, 5, 6], [3, 4, 5, 6], [3, 4, 5, 6], [2, 3, 4, 9]])
    n_commit, nxt = DO.greedy_accept(verify, targets)
    assert n_commit == [4, 2, 1, 4]
    assert nxt == [6, 4, 3, 9]
    n_commit, nxt = DO.greedy_accept(verify[:, :1], targets[:, :1])
    assert n_commit == [1, 1, 1, 1] and nxt == [3, 3, 3, 2]
