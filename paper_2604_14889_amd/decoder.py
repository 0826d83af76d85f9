"""One full decode step (Algorithm 1, SpeculativeStep, of the MemoSight paper) on the GPU.

The attention, the residual/RMSNorm, SwiGLU and greedy-token kernels, acceptance and the cache
update are this library's HIP kernels.  Of the dense projections, the fused Q/K/V projection and
the MLP down projection run on this library's MFMA GEMM (ms_gemm_bf16: one launch fills the three
Q/K/V tensors; the down projection's deep K is split over workgroups), where it is faster than the
library GEMM at a few hundred rows; the output, gate/up and LM-head projections go through torch
(hipBLASLt underneath), which is still ahead on those shapes.  fused_mlp=True moves the gate/up
projection onto this library's GEMM as well, with SwiGLU applied in its epilogue
(ms_gemm_swiglu_bf16): no hipBLASLt in the MLP, about a tenth slower on that projection.

Nothing here computes on the CPU; every call fails if the HIP library is missing.
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
        self.ln1, self.wq, self.bq, self.wk, self.bk, self.wv, self.bv = ln1, wq, bq, wk, bk, wv, bv
        self.wo, self.ln2, self.w_gate_up, self.w_down = wo, ln2, w_gate_up, w_down
        # one weight for the fused Q/K/V projection (rows: Q heads, then K heads, then V heads)
        self.wqkv = torch.cat([wq, wk, wv], dim=0).contiguous()
        self.bqkv = torch.cat([bq, bk, bv], dim=0).contiguous()
        self.w_gate_up_blocked = None   # rows re-ordered for the fused gate/up + SwiGLU GEMM, made on demand

    def gate_up_blocked(self):
        if self.w_gate_up_blocked is None:
            inter = self.w_gate_up.shape[0] // 2
            self.w_gate_up_blocked = M.interleave_gate_up(self.w_gate_up[:inter], self.w_gate_up[inter:])
        return self.w_gate_up_blocked


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

    def __init__(self, cfg: DecoderConfig, weights: DecoderTensors, session: Session, max_rows: int,
                 hand_gemm: bool = True, fused_mlp: bool = False, tune_library_gemms: bool = False,
                 fused_lm_head: bool = False):
        """hand_gemm: run the Q/K/V and down projections on this library's GEMM (needs widths that
        are multiples of 128 and depths that are multiples of 128); otherwise everything dense goes
        through torch."""
        self.cfg, self.w, self.ses = cfg, weights, session
        dev = weights.embed.device
        if tune_library_gemms:
            # the projections left to torch: let it time the library's solutions for each new shape
            # once (a few seconds at the first call) instead of taking the default pick.  Process-wide.
            import torch.cuda.tunable as tunable
            tunable.enable(True)
            tunable.tuning_enable(True)
            tunable.set_max_tuning_duration(200)
            import os
            import tempfile
            tunable.set_filename(os.path.join(tempfile.gettempdir(), "memosight_library_gemms.csv"))   # its results file
        qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim

        def buf(*shape, dtype=torch.bfloat16):
            return torch.empty(*shape, dtype=dtype, device=dev)

        self.max_rows = max_rows
        self.h = buf(max_rows, cfg.hidden, dtype=torch.float32)
        self.x = buf(max_rows, cfg.hidden)
        self.q = buf(max_rows, qd)
        self._kv = {}             # rows -> (k_new, v_new), each [L, rows, Hkv*D] contiguous for the commit
        self._prepared = {}       # rows -> prepared argument tuples of the library calls
        self.attn = buf(max_rows, qd)
        self.proj = buf(max_rows, cfg.hidden)
        self.gate_up = buf(max_rows, 2 * cfg.inter)
        self.act = buf(max_rows, cfg.inter)
        self.logits = buf(max_rows, cfg.vocab)
        self.targets = buf(max_rows, dtype=torch.int32)
        self.attn_events = None   # optional list of (start, stop) events around every attention call
        # K is split further when a step has few rows (one row tile: half as many workgroups);
        # measured at Qwen2.5-7B widths: Q/K/V 4 ways up to 256 rows, 2 above; down 8 and 4
        self.splits_few, self.splits_many = (4, 8), (2, 4)
        self.hand_gemm = (hand_gemm and qd % 128 == 0 and kd % 128 == 0 and cfg.hidden % 128 == 0 and
                          cfg.hidden % (32 * 4) == 0 and cfg.inter % (32 * 8) == 0)
        # gate/up + SwiGLU in one GEMM: keeps a second, row-interleaved copy of the gate/up weights
        self.fused_mlp = fused_mlp and self.hand_gemm and cfg.inter % 64 == 0
        # LM head and greedy token in one kernel of the library (fp32 sums, no logits): step() then
        # returns None for the logits
        self.fused_lm_head = fused_lm_head and cfg.vocab % 128 == 0 and cfg.hidden % 32 == 0
        self.lm_ws = None
        if self.fused_lm_head:
            self.lm_ws = torch.empty(M.ms_lm_head_argmax_workspace_bytes(max_rows, cfg.vocab, cfg.hidden), dtype=torch.uint8, device=dev)
        self.gemm_ws = None
        if self.hand_gemm:
            need = max(M.ms_gemm_workspace_bytes(max_rows, qd + 2 * kd, cfg.hidden, self.splits_few[0]),
                       M.ms_gemm_workspace_bytes(max_rows, cfg.hidden, cfg.inter, self.splits_few[1]),
                       max(M.ms_gemm_workspace_bytes(r, qd + 2 * kd, cfg.hidden, 1) for r in range(1, min(max_rows, 16) + 1)),
                       max(M.ms_gemm_workspace_bytes(r, 2 * cfg.inter, cfg.hidden, 1) for r in range(1, min(max_rows, 16) + 1)),
                       max(M.ms_gemm_workspace_bytes(r, cfg.vocab, cfg.hidden, 1) for r in range(1, min(max_rows, 16) + 1))
                       if cfg.vocab % 128 == 0 else 0,
                       max(M.ms_gemm_workspace_bytes(r, cfg.hidden, qd, 1) for r in range(1, min(max_rows, 16) + 1)),
                       M.ms_gemm_add_rmsnorm_workspace_bytes(max_rows, cfg.hidden, cfg.inter, self.splits_few[1]),
                       max(M.ms_gemm_add_rmsnorm_workspace_bytes(r, cfg.hidden, cfg.inter, self.splits_few[1])
                           for r in range(1, min(max_rows, 16) + 1)),
                       M.ms_gemm_workspace_bytes(max_rows, 2 * cfg.inter, cfg.hidden, 1) if self.fused_mlp else 0)
            self.gemm_ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

    def step(self, seq_ids: Sequence[int], tokens: torch.Tensor, pos: torch.Tensor, n_verify: int, n_foresight: int,
             ctx_new: Optional[torch.Tensor] = None):
        """tokens, pos: int32 device [B, n_q].  Returns (logits [B*n_q, vocab] bf16, greedy tokens
        [B*n_q] int32), both views of this object's buffers (logits is None with fused_lm_head);
        step_kv() gives the step's keys and values for ms_commit_accepted."""
        cfg, w = self.cfg, self.w
        B = len(seq_ids)
        n_q = n_verify + n_foresight
        rows = B * n_q
        if rows > self.max_rows:
            raise M.MsError(M.MS_ERR_INVALID, f"step of {rows} rows exceeds the buffers ({self.max_rows})")
        hq, hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
        h, x, q, attn, proj = self.h[:rows], self.x[:rows], self.q[:rows], self.attn[:rows], self.proj[:rows]
        gate_up, act = self.gate_up[:rows], self.act[:rows]
        if rows not in self._kv:
            kd = hkv * d
            self._kv[rows] = (torch.empty(cfg.n_layers, rows, kd, dtype=torch.bfloat16, device=h.device),
                              torch.empty(cfg.n_layers, rows, kd, dtype=torch.bfloat16, device=h.device))
        self.k_new, self.v_new = self._kv[rows]
        if self.hand_gemm and not self.fused_mlp:
            return self._step_prepared(seq_ids, tokens, pos, n_verify, n_foresight, ctx_new, rows)
        qkv_split, down_split = self.splits_few if rows <= 256 else self.splits_many
        M.ms_embed_rows(w.embed, tokens, h)
        delta = None
        for li, lw in enumerate(w.layers):
            M.ms_add_rmsnorm(h, delta, lw.ln1, cfg.eps, x)
            k, v = self.k_new[li], self.v_new[li]
            if self.hand_gemm:
                M.ms_gemm_bf16(x, lw.wqkv, lw.bqkv, [q, k, v], qkv_split, self.gemm_ws)
            else:
                torch.addmm(lw.bq, x, lw.wq.t(), out=q)
                torch.addmm(lw.bk, x, lw.wk.t(), out=k)
                torch.addmm(lw.bv, x, lw.wv.t(), out=v)
            self.ses.attention(li, seq_ids, n_verify, n_foresight, q.view(B, n_q, hq, d), k.view(B, n_q, hkv, d),
                               v.view(B, n_q, hkv, d), pos, ctx_new, 0.0, attn.view(B, n_q, hq, d))
            torch.mm(attn, lw.wo.t(), out=proj)
            M.ms_add_rmsnorm(h, proj, lw.ln2, cfg.eps, x)
            if self.fused_mlp:
                M.ms_gemm_swiglu_bf16(x, lw.gate_up_blocked(), act, self.gemm_ws)
            else:
                torch.mm(x, lw.w_gate_up.t(), out=gate_up)
                M.ms_swiglu(gate_up, act)
            if self.hand_gemm:
                M.ms_gemm_bf16(act, lw.w_down, None, [proj], down_split, self.gemm_ws)
            else:
                torch.mm(act, lw.w_down.t(), out=proj)
            delta = proj
        M.ms_add_rmsnorm(h, delta, w.norm, cfg.eps, x)
        return self._greedy_tokens(x, rows)

    # ---- the same step with the library calls' arguments prepared once -------------------------------
    def _prepare(self, rows: int):
        """Argument tuples of every per-layer library call of a step of `rows` rows.  All buffers are
        this object's and all weights are fixed, so the addresses never change; a step with a single
        sequence is otherwise bound by re-deriving them in Python for its ~200 calls.  Whoever swaps
        a weight tensor for another one afterwards calls forget_prepared()."""
        cfg, w = self.cfg, self.w
        ptr = lambda t: t.data_ptr()
        qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
        h, x, q, attn, proj, gate_up, act = (ptr(t) for t in (self.h, self.x, self.q, self.attn, self.proj, self.gate_up, self.act))
        k_all, v_all = self._kv[rows]
        ws, ws_bytes = ptr(self.gemm_ws), self.gemm_ws.numel()
        qkv_split, down_split = self.splits_few if rows <= 256 else self.splits_many
        cols_qkv = M.int_array([0, qd, qd + kd, qd + 2 * kd])
        cols_h = M.int_array([0, cfg.hidden])
        outs_proj = (C.c_void_p * 1)(proj)
        layers = []
        for li, lw in enumerate(w.layers):
            k, v = ptr(k_all[li]), ptr(v_all[li])
            layers.append(dict(
                keep=(outs_proj, cols_qkv, cols_h),
                norm1=(h, proj if li else None, ptr(lw.ln1), cfg.eps, x, rows, cfg.hidden),
                qkv=(x, ptr(lw.wqkv), ptr(lw.bqkv), rows, qd + 2 * kd, cfg.hidden, 3, (C.c_void_p * 3)(q, k, v), cols_qkv,
                     qkv_split, ws, ws_bytes),
                k=k, v=v,
                o=(attn, ptr(lw.wo), None, rows, cfg.hidden, qd, 1, outs_proj, cols_h, 1, ws, ws_bytes),
                wo_t=lw.wo.t(), w_gate_up_t=lw.w_gate_up.t(),
                norm2=(h, proj, ptr(lw.ln2), cfg.eps, x, rows, cfg.hidden),
                swiglu=(gate_up, act, rows, cfg.inter),
                # few rows: gate/up with SwiGLU in the product's epilogue, from the row-interleaved copy of the weight
                mlp_few=(x, ptr(lw.gate_up_blocked()), rows, cfg.inter, cfg.hidden, act, ws, ws_bytes) if self._few(rows) else None,
                # the down projection with the residual add and the norm that follow it (the next block's, or the final one)
                down_norm=(act, ptr(lw.w_down), rows, cfg.hidden, cfg.inter, down_split, h,
                           ptr(w.layers[li + 1].ln1 if li + 1 < len(w.layers) else w.norm), cfg.eps, x, ws, ws_bytes)))
        return dict(layers=layers, q=q, attn=attn)

    def _few(self, rows: int) -> bool:
        """Steps of at most 16 rows (one or two sequences) run every projection on this library's
        few-row kernel, gate/up fused with SwiGLU (which keeps a row-interleaved second copy
        of that weight, made at the first such step)."""
        return rows <= 16 and self.cfg.inter % 128 == 0

    def forget_prepared(self) -> None:
        """Drops the prepared argument tuples (they hold device addresses of the weights)."""
        self._prepared.clear()

    def _step_prepared(self, seq_ids, tokens, pos, n_verify, n_foresight, ctx_new, rows):
        cfg, w, lib, check = self.cfg, self.w, M.lib, M._check
        if rows not in self._prepared:
            self._prepared[rows] = self._prepare(rows)
        prep = self._prepared[rows]
        B, n_q = len(seq_ids), n_verify + n_foresight
        if tokens.numel() != rows or pos.numel() != rows or (ctx_new is not None and ctx_new.numel() != rows):
            raise M.MsError(M.MS_ERR_INVALID, "tokens / pos / ctx_new do not have one entry per row")
        st = M._stream(None)
        ids = M.int_array(seq_ids)
        att_ws = self.ses.ensure_workspace(B, n_q)
        att_ws_ptr, att_ws_bytes = att_ws.data_ptr(), att_ws.numel() * att_ws.element_size()
        pos_ptr, ctx_ptr = M._dev(pos), M._dev(ctx_new)
        cache, q, attn = self.ses.cache, prep["q"], prep["attn"]
        x_t, attn_t, proj_t, gate_up_t = self.x[:rows], self.attn[:rows], self.proj[:rows], self.gate_up[:rows]
        few = self._few(rows)
        M.ms_embed_rows(w.embed, tokens, self.h[:rows])
        for li, c in enumerate(prep["layers"]):
            if li == 0:     # the later blocks' input norm is applied by the block before, with its down projection
                check(lib.ms_add_rmsnorm(*c["norm1"], st))
            check(lib.ms_gemm_bf16(*c["qkv"], st))
            if self.attn_events is not None:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            check(lib.ms_predict_verify_attention(cache, li, B, ids, n_verify, n_foresight, q, c["k"], c["v"], pos_ptr, ctx_ptr, 0.0,
                                                  attn, att_ws_ptr, att_ws_bytes, st))
            if self.attn_events is not None:
                e1.record()
                self.attn_events.append((e0, e1))
            if few:
                check(lib.ms_gemm_bf16(*c["o"], st))
            else:
                torch.mm(attn_t, c["wo_t"], out=proj_t)
            check(lib.ms_add_rmsnorm(*c["norm2"], st))
            if few:
                check(lib.ms_gemm_swiglu_bf16(*c["mlp_few"], st))
            else:
                torch.mm(x_t, c["w_gate_up_t"], out=gate_up_t)
                check(lib.ms_swiglu(*c["swiglu"], st))
            check(lib.ms_gemm_add_rmsnorm_bf16(*c["down_norm"], st))
        return self._greedy_tokens(x_t, rows)

    def _greedy_tokens(self, x, rows):
        targets = self.targets[:rows]
        if self.fused_lm_head:
            # the workspace was sized for max_rows; fewer rows may run on another kernel with more column groups
            need = M.ms_lm_head_argmax_workspace_bytes(rows, self.cfg.vocab, self.cfg.hidden)
            if need > self.lm_ws.numel():
                self.lm_ws = torch.empty(need, dtype=torch.uint8, device=self.lm_ws.device)
            M.ms_lm_head_argmax_bf16(x, self.w.lm_head, targets, self.lm_ws)
            return None, targets
        logits = self.logits[:rows]
        if self.hand_gemm and self._few(rows) and self.cfg.vocab % 128 == 0:
            M.ms_gemm_bf16(x, self.w.lm_head, None, [logits], 1, self.gemm_ws)
        else:
            torch.mm(x, self.w.lm_head.t(), out=logits)
        M.ms_argmax_rows(logits, self.cfg.vocab, targets)
        return logits, targets

    def step_kv(self):
        """The last step's K / V as contiguous [L, rows, Hkv, D] tensors (input of ms_commit_accepted)."""
        cfg = self.cfg
        rows = self.k_new.shape[1]
        return (self.k_new.view(cfg.n_layers, rows, cfg.n_kv_heads, cfg.head_dim),
                self.v_new.view(cfg.n_layers, rows, cfg.n_kv_heads, cfg.head_dim))
