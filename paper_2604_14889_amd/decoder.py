"""One full decode step (Algorithm 1, SpeculativeStep, of the MemoSight paper) on the GPU.

Everything in the step is this library's HIP kernels: the attention, the residual/RMSNorm and
greedy-token kernels, acceptance, the cache update, and the dense projections (ms_gemm_bf16 and its
fused forms: one launch fills the three Q/K/V tensors, the gate/up projection applies SwiGLU in its
epilogue, the down projection's partial sums are added up by the kernel that also adds the
residual and applies the next norm, the LM head can leave the greedy token instead of the logits).
Up to 16 rows (one or two sequences) the projections run on the library's few-row kernel.

Nothing here computes on the CPU or in a library GEMM; every call fails if the HIP library is
missing, and shapes the kernels do not take are refused when the Decoder is built.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from . import binding as M
from .session import Session


@dataclass
class DecoderConfig:
    n_layers: int
    hidden: int
    inter: int
    vocab: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    eps: float = 1e-6
    rope_base: float = 1000000.0

    @staticmethod
    def qwen2_5_7b() -> "DecoderConfig":
        return DecoderConfig(28, 3584, 18944, 152064, 28, 4, 128, 1e-6, 1000000.0)


class LayerTensors:
    """bf16 device tensors of one block; projection weights are [out_features, in_features]."""

    def __init__(self, ln1, wq, bq, wk, bk, wv, bv, wo, ln2, w_gate_up, w_down):
        self.ln1, self.wo, self.ln2, self.w_down = ln1, wo, ln2, w_down
        # one weight for the fused Q/K/V projection (rows: Q heads, then K heads, then V heads)
        self.wqkv = torch.cat([wq, wk, wv], dim=0).contiguous()
        self.bqkv = torch.cat([bq, bk, bv], dim=0).contiguous()
        # gate and up rows interleaved in blocks of 32: the layout the gate/up projection with SwiGLU
        # in its epilogue reads (a one-off re-ordering of rows at load time)
        inter = w_gate_up.shape[0] // 2
        self.w_gate_up_blocked = M.interleave_gate_up(w_gate_up[:inter], w_gate_up[inter:])


class DecoderTensors:
    def __init__(self, embed, layers: List[LayerTensors], norm, lm_head):
        self.embed, self.layers, self.norm, self.lm_head = embed, layers, norm, lm_head

    @staticmethod
    def random(cfg: DecoderConfig, seed: int, device="cuda:0") -> "DecoderTensors":
        """Random-init weights of the given shape, drawn on the device: projections N(0, 1/sqrt(fan_in)),
        biases N(0, 0.1), norm weights 1."""
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)

        def w(out_f, in_f):
            return torch.empty(out_f, in_f, dtype=torch.bfloat16, device=device).normal_(0.0, in_f ** -0.5, generator=gen)

        def b(n):
            return torch.empty(n, dtype=torch.bfloat16, device=device).normal_(0.0, 0.1, generator=gen)

        def ones(n):
            return torch.ones(n, dtype=torch.bfloat16, device=device)

        qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
        layers = [LayerTensors(ones(cfg.hidden), w(qd, cfg.hidden), b(qd), w(kd, cfg.hidden), b(kd), w(kd, cfg.hidden), b(kd),
                               w(cfg.hidden, qd), ones(cfg.hidden), w(2 * cfg.inter, cfg.hidden), w(cfg.hidden, cfg.inter))
                  for _ in range(cfg.n_layers)]
        embed = torch.empty(cfg.vocab, cfg.hidden, dtype=torch.bfloat16, device=device).normal_(0.0, 1.0, generator=gen)
        return DecoderTensors(embed, layers, ones(cfg.hidden), w(cfg.vocab, cfg.hidden))


class Decoder:
    """Buffers and the step driver for up to max_rows = B * n_q tokens per step."""

    def __init__(self, cfg: DecoderConfig, weights: DecoderTensors, session: Session, max_rows: int, fused_lm_head: bool = False):
        """fused_lm_head: LM head and greedy token in one kernel (the token is taken on the fp32 sums,
        the logits are never written); step() then returns None for the logits."""
        self.cfg, self.w, self.ses = cfg, weights, session
        dev = weights.embed.device
        qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
        if qd % 128 or kd % 128 or cfg.hidden % 128 or cfg.inter % 256:
            raise M.MsError(M.MS_ERR_UNSUPPORTED, "the projection kernels need head widths and the hidden size in multiples of 128 "
                                                  "and an MLP width in multiples of 256")
        # the LM head's width in multiples of 128: rows of zeros are appended once, here; the greedy
        # token is taken over the real vocabulary only
        self.vocab_pad = -(-cfg.vocab // 128) * 128
        self.lm_head = weights.lm_head
        if self.vocab_pad != cfg.vocab:
            self.lm_head = torch.zeros(self.vocab_pad, cfg.hidden, dtype=torch.bfloat16, device=dev)
            self.lm_head[:cfg.vocab].copy_(weights.lm_head)
        if fused_lm_head and self.vocab_pad != cfg.vocab:
            raise M.MsError(M.MS_ERR_UNSUPPORTED, "fused_lm_head needs a vocabulary size in multiples of 128")
        self.fused_lm_head = fused_lm_head

        def buf(*shape, dtype=torch.bfloat16):
            return torch.empty(*shape, dtype=dtype, device=dev)

        self.max_rows = max_rows
        self.h = buf(max_rows, cfg.hidden, dtype=torch.float32)
        self.x = buf(max_rows, cfg.hidden)
        self.q = buf(max_rows, qd)
        self._kv = {}             # rows -> (k_new, v_new), each [L, rows, Hkv*D] contiguous for the commit
        self._prepared = {}       # rows -> prepared argument tuples of the library calls
        self.attn = buf(max_rows, qd)
        self.act = buf(max_rows, cfg.inter)
        self.logits = None if fused_lm_head else buf(max_rows, self.vocab_pad)
        self.targets = buf(max_rows, dtype=torch.int32)
        # K is divided over workgroups where a projection has few output tiles (one 256 x 256 tile per
        # workgroup, one workgroup per compute unit); measured at Qwen2.5-7B widths: Q/K/V 7 ways up to
        # 256 rows (one row tile) and 4 above, output 8 and 7, down 16 and 8.  Other widths take the
        # largest divisor of their K steps below those.
        def split(k, want):
            steps = k // 32
            return max(s for s in range(1, want + 1) if steps % s == 0 and (s == 1 or steps // s >= 4))
        self.splits_few = (split(cfg.hidden, 7), max(2, split(qd, 8)), max(2, split(cfg.inter, 16)))
        self.splits_many = (split(cfg.hidden, 4), max(2, split(qd, 7)), max(2, split(cfg.inter, 8)))
        rows_few = range(1, min(max_rows, 16) + 1)
        need = max([M.ms_gemm_workspace_bytes(max_rows, qd + 2 * kd, cfg.hidden, self.splits_few[0]),
                    M.ms_gemm_add_rmsnorm_workspace_bytes(max_rows, cfg.hidden, qd, self.splits_few[1]),
                    M.ms_gemm_workspace_bytes(max_rows, 2 * cfg.inter, cfg.hidden, 1),
                    M.ms_gemm_workspace_bytes(max_rows, self.vocab_pad, cfg.hidden, 1),
                    M.ms_gemm_add_rmsnorm_workspace_bytes(max_rows, cfg.hidden, cfg.inter, self.splits_few[2])] +
                   [M.ms_gemm_workspace_bytes(r, n, k, 1) for r in rows_few
                    for n, k in ((qd + 2 * kd, cfg.hidden), (2 * cfg.inter, cfg.hidden), (self.vocab_pad, cfg.hidden))] +
                   [M.ms_gemm_add_rmsnorm_workspace_bytes(r, cfg.hidden, k, s) for r in rows_few
                    for k, s in ((qd, self.splits_few[1]), (cfg.inter, self.splits_few[2]))])
        self.gemm_ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        self.lm_ws = None
        if fused_lm_head:
            self.lm_ws = torch.empty(M.ms_lm_head_argmax_workspace_bytes(max_rows, cfg.vocab, cfg.hidden), dtype=torch.uint8, device=dev)

    # ---- argument tuples of the library calls, prepared once per row count ---------------------------
    def _prepare(self, rows: int):
        """All buffers are this object's and all weights are fixed, so the addresses never change; a
        step with a single sequence is otherwise bound by re-deriving them in Python for its ~200
        calls.  Whoever swaps a weight tensor for another one afterwards calls forget_prepared()."""
        cfg, w = self.cfg, self.w
        ptr = lambda t: t.data_ptr()
        qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
        h, x, q, attn, act = (ptr(t) for t in (self.h, self.x, self.q, self.attn, self.act))
        k_all, v_all = self._kv[rows]
        ws, ws_bytes = ptr(self.gemm_ws), self.gemm_ws.numel()
        qkv_split, o_split, down_split = self.splits_few if rows <= 256 else self.splits_many
        cols_qkv = M.int_array([0, qd, qd + kd, qd + 2 * kd])
        layers = []
        for li, lw in enumerate(w.layers):
            k, v = ptr(k_all[li]), ptr(v_all[li])
            layers.append(dict(
                keep=(cols_qkv,),
                norm1=(h, None, ptr(lw.ln1), cfg.eps, x, rows, cfg.hidden),   # used by the first block only
                qkv=(x, ptr(lw.wqkv), ptr(lw.bqkv), rows, qd + 2 * kd, cfg.hidden, 3, (C.c_void_p * 3)(q, k, v), cols_qkv,
                     qkv_split, ws, ws_bytes),
                k=k, v=v,
                # the output projection with the residual add and the post-attention norm that follow it
                o_norm=(attn, ptr(lw.wo), rows, cfg.hidden, qd, o_split, h, ptr(lw.ln2), cfg.eps, x, ws, ws_bytes),
                # gate/up with SwiGLU in the product's epilogue, from the row-interleaved weight
                mlp=(x, ptr(lw.w_gate_up_blocked), rows, cfg.inter, cfg.hidden, act, ws, ws_bytes),
                # the down projection with the residual add and the norm that follow it (the next block's, or the final one)
                down_norm=(act, ptr(lw.w_down), rows, cfg.hidden, cfg.inter, down_split, h,
                           ptr(w.layers[li + 1].ln1 if li + 1 < len(w.layers) else w.norm), cfg.eps, x, ws, ws_bytes)))
        return dict(layers=layers, q=q, attn=attn)

    def forget_prepared(self) -> None:
        """Drops the prepared argument tuples (they hold device addresses of the weights)."""
        self._prepared.clear()

    def step(self, seq_ids: Sequence[int], tokens: torch.Tensor, pos: torch.Tensor, n_verify: int, n_foresight: int,
             ctx_new: Optional[torch.Tensor] = None):
        """tokens, pos: int32 device [B, n_q].  Returns (logits [B*n_q, vocab] bf16, greedy tokens
        [B*n_q] int32), both views of this object's buffers (logits is None with fused_lm_head);
        step_kv() gives the step's keys and values for ms_commit_accepted."""
        cfg, w, lib, check = self.cfg, self.w, M.lib, M._check
        B, n_q = len(seq_ids), n_verify + n_foresight
        rows = B * n_q
        if rows > self.max_rows:
            raise M.MsError(M.MS_ERR_INVALID, f"step of {rows} rows exceeds the buffers ({self.max_rows})")
        if tokens.numel() != rows or pos.numel() != rows or (ctx_new is not None and ctx_new.numel() != rows):
            raise M.MsError(M.MS_ERR_INVALID, "tokens / pos / ctx_new do not have one entry per row")
        if rows not in self._kv:
            kd = cfg.n_kv_heads * cfg.head_dim
            self._kv[rows] = (torch.empty(cfg.n_layers, rows, kd, dtype=torch.bfloat16, device=self.h.device),
                              torch.empty(cfg.n_layers, rows, kd, dtype=torch.bfloat16, device=self.h.device))
        self.k_new, self.v_new = self._kv[rows]
        if rows not in self._prepared:
            self._prepared[rows] = self._prepare(rows)
        prep = self._prepared[rows]
        st = M._stream(None)
        ids = seq_ids if isinstance(seq_ids, C.Array) else M.int_array(seq_ids)
        att_ws = self.ses.ensure_workspace(B, n_q)
        att_ws_ptr, att_ws_bytes = att_ws.data_ptr(), att_ws.numel() * att_ws.element_size()
        pos_ptr, ctx_ptr = M._dev(pos), M._dev(ctx_new)
        cache, q, attn = self.ses.cache, prep["q"], prep["attn"]
        M.ms_embed_rows(w.embed, tokens, self.h[:rows])
        for li, c in enumerate(prep["layers"]):
            if li == 0:     # the later blocks' input norm is applied by the block before, with its down projection
                check(lib.ms_add_rmsnorm(*c["norm1"], st))
            check(lib.ms_gemm_bf16(*c["qkv"], st))
            check(lib.ms_predict_verify_attention(cache, li, B, ids, n_verify, n_foresight, q, c["k"], c["v"], pos_ptr, ctx_ptr, 0.0,
                                                  attn, att_ws_ptr, att_ws_bytes, st))
            check(lib.ms_gemm_add_rmsnorm_bf16(*c["o_norm"], st))
            check(lib.ms_gemm_swiglu_bf16(*c["mlp"], st))
            check(lib.ms_gemm_add_rmsnorm_bf16(*c["down_norm"], st))
        return self._greedy_tokens(self.x[:rows], rows)

    def _greedy_tokens(self, x, rows):
        targets = self.targets[:rows]
        if self.fused_lm_head:
            # the workspace was sized for max_rows; fewer rows may run on another kernel with more column groups
            need = M.ms_lm_head_argmax_workspace_bytes(rows, self.cfg.vocab, self.cfg.hidden)
            if need > self.lm_ws.numel():
                self.lm_ws = torch.empty(need, dtype=torch.uint8, device=self.lm_ws.device)
            M.ms_lm_head_argmax_bf16(x, self.lm_head, targets, self.lm_ws)
            return None, targets
        logits = self.logits[:rows]
        M.ms_gemm_bf16(x, self.lm_head, None, [logits], 1, self.gemm_ws)
        M.ms_argmax_rows(logits, self.cfg.vocab, targets)
        return logits[:, :self.cfg.vocab], targets

    def step_kv(self):
        """The last step's K / V as contiguous [L, rows, Hkv, D] tensors (input of ms_commit_accepted)."""
        cfg = self.cfg
        rows = self.k_new.shape[1]
        return (self.k_new.view(cfg.n_layers, rows, cfg.n_kv_heads, cfg.head_dim),
                self.v_new.view(cfg.n_layers, rows, cfg.n_kv_heads, cfg.head_dim))
