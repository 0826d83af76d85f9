"""MemoSight's iterative inference (Appendix A, Algorithm 1 of the paper) on the GPU step by step.

Phase 1, foresight-based acceleration (Section 2.1.1).  A sequence that holds drafts runs the fused
pass: the verify block [next token, d drafts] and d foresight tokens behind it; the drafts that match
the model's own greedy tokens are accepted and the accepted tokens' K/V enter the paged cache.  Only
when the whole block was kept do the foresight rows stand at the position ids of the tokens that
follow it, and only then are their greedy tokens the next drafts.  A sequence without valid drafts
(a new step, or a block that was cut short) runs the Predict pass alone: its next token and d
foresight tokens right behind it, which yields the next token's successor and d drafts.  Both kinds
share one forward pass of the batch: every query carries its own position id and visibility bound.
Phase 2, compression: when a step delimiter is among the accepted tokens, l = ceil(|R| / c) memory tokens and the output token <o> are run through the model
(causal among themselves, position ids from the uniform position layout, Section 2.1.2 / 2.2), and
the step's tokens are replaced in the cache by those l + 1 rows; generation continues from <o>'s
greedy token.

All model arithmetic runs in `Decoder.step` (this library's kernels + library GEMMs); this file is
host control flow only.  An observer, if given, is told about every forward pass and every cache
change -- the tests use it to keep a CPU oracle in lockstep.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as M
from .decoder import Decoder


@dataclass
class SpecialTokens:
    memory: int                 # <m>
    output: int                 # <o>
    foresight: int              # <f>
    delimiters: Sequence[int]   # step boundaries <e>
    eos: int


@dataclass
class SeqState:
    seq_id: int
    next_token: int             # decided but not yet in the cache: the next verify block starts with it
    next_pid: int               # its position id
    drafts: List[int]           # d draft tokens for the positions after next_token
    step_begin: int             # cache length at which the open reasoning step begins
    step_first_pid: int         # position id of the open step's first token
    prompt_len: int = 0
    generated: List[int] = field(default_factory=list)
    finished: bool = False
    steps_closed: int = 0
    drafts_valid: bool = False  # False: `drafts` are placeholders, the next pass is a Predict pass for this sequence


class Observer:
    def forward(self, kind, seq_ids, tokens, pos, n_verify, n_foresight, logits, targets, ctx_new=None):  # noqa: D401
        pass

    def commit(self, seq_ids, n_commit, pos):
        pass

    def compact(self, seq_id, seg_begin, seg_len, n_rows, pos):
        pass


class MemoSightDriver:
    def __init__(self, decoder: Decoder, d: int, c: int, special: SpecialTokens, observer: Optional[Observer] = None,
                 per_position: bool = False, upl: bool = True, fixed_memory: Optional[int] = None):
        """upl=False and fixed_memory=n select the ablation layouts of Appendix B: memory tokens on the
        consecutive position ids after the step ("w/o UPL"), n memory tokens for every step whatever
        its length ("w/o AMA").
        per_position: put d foresight tokens behind EVERY verify token (the layout the model is
        trained on, Section 2.2) instead of behind the block only, so that the drafts for the next
        pass are valid whatever number of verify tokens was kept; costs (d + 1) d instead of d extra
        queries per pass."""
        if d < 0 or c < 1:
            raise ValueError("need d >= 0 and c >= 1")
        if per_position and (d + 1) * (d + 1) > M.MS_MAX_QUERIES:
            raise ValueError("too many queries per pass")
        if fixed_memory is not None and not 1 <= fixed_memory < M.MS_MAX_QUERIES:
            raise ValueError("fixed_memory out of range")
        self.per_position, self.upl, self.fixed_memory = per_position, upl, fixed_memory
        self.dec, self.ses, self.d, self.c, self.sp = decoder, decoder.ses, d, c, special
        self.obs = observer or Observer()
        self.state: Dict[int, SeqState] = {}
        self.passes = {"speculative": 0, "memory": 0, "prefill": 0}
        self.blocks = {"verify": 0, "predict": 0}   # per sequence and pass: which kind it ran
        self.committed = 0         # tokens committed by speculative passes
        self.raw_tokens = 0        # tokens that would be cached without compression

    # ---- helpers --------------------------------------------------------------------------------
    def _forward(self, kind, seq_ids, tokens: np.ndarray, pos: np.ndarray, n_verify: int, n_foresight: int, ctx_d=None):
        tok_d = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).cuda()
        pos_d = torch.from_numpy(np.ascontiguousarray(pos, dtype=np.int32)).cuda()
        logits, targets = self.dec.step(seq_ids, tok_d, pos_d, n_verify, n_foresight, ctx_d)
        self.passes[kind] += 1
        ctx = None if ctx_d is None else ctx_d.cpu().numpy()
        self.obs.forward(kind, list(seq_ids), tokens, pos, n_verify, n_foresight, logits, targets, ctx)
        return pos_d, targets

    # ---- Algorithm 1, initialisation: prefill -------------------------------------------------------------
    def prefill(self, seq_ids: Sequence[int], prompts: Sequence[Sequence[int]], chunk: int = M.MS_MAX_QUERIES):
        """Runs each prompt through the model in causal chunks and caches all of it; the greedy token
        after the prompt's last token becomes the first token of the first reasoning step."""
        for sid, prompt in zip(seq_ids, prompts):
            prompt = [int(t) for t in prompt]
            if not prompt:
                raise ValueError("empty prompt")
            at, last_target = 0, None
            while at < len(prompt):
                n = min(chunk, len(prompt) - at)
                tokens = np.asarray([prompt[at:at + n]], np.int32)
                pos = np.arange(1 + at, 1 + at + n, dtype=np.int32)[None]
                pos_d, targets = self._forward("prefill", [sid], tokens, pos, n, 0)
                k_new, v_new = self.dec.step_kv()
                M.ms_commit_accepted(self.ses.cache, [sid], [n], n, k_new, v_new, pos_d)
                self.obs.commit([sid], [n], pos)
                last_target = int(targets[n - 1].item())
                at += n
            self.raw_tokens += len(prompt)
            self.state[sid] = SeqState(sid, last_target, len(prompt) + 1, [self.sp.foresight] * self.d, len(prompt),
                                       len(prompt) + 1, prompt_len=len(prompt))

    # ---- Algorithm 1, phase 1: one speculative step for every unfinished sequence ---------------------
    def speculative_step(self) -> List[int]:
        """Returns the ids of the sequences whose reasoning step closed in this pass."""
        act = [s for s in self.state.values() if not s.finished]
        if not act:
            return []
        d = self.d
        ids = [s.seq_id for s in act]
        B = len(act)
        F = self.sp.foresight
        ctx_d = None
        if self.per_position:
            # d foresight tokens behind every verify token: whatever is kept, drafts follow it
            nv, nf = d + 1, (d + 1) * d
            tokens = np.asarray([[s.next_token] + s.drafts + [F] * nf for s in act], np.int32)
            lay = [M.ms_per_position_layout(s.next_pid, nv, d) for s in act]
            pos = np.asarray([p for p, _ in lay], np.int32)
            ctx_d = torch.tensor([c_ for _, c_ in lay], dtype=torch.int32, device="cuda")
            verifying = [True] * B
        else:
            verifying = [s.drafts_valid and d > 0 for s in act]
            first = np.asarray([s.next_pid for s in act], np.int32)
            if not any(verifying):
                # Predict pass for everyone: the next token and d foresight tokens behind it
                nv, nf = 1, d
                tokens = np.asarray([[s.next_token] + [F] * d for s in act], np.int32)
                pos = M.ms_step_positions(first, 1, d)
            else:
                # fused pass; a sequence without drafts runs its Predict pass inside it: its d
                # foresight tokens take the place of the drafts (each sees the next token and
                # itself) and the block's last d rows are padding that sees, and is seen by, nothing
                nv, nf = d + 1, d
                tokens = np.asarray([[s.next_token] + (s.drafts if v else [F] * d) + [F] * d for s, v in zip(act, verifying)], np.int32)
                pos = M.ms_step_positions(first, nv, d)
                if not all(verifying):
                    pred = M.ms_step_positions(first, 1, d)
                    fused_ctx, pred_ctx = M.ms_default_ctx_new(nv, d), M.ms_default_ctx_new(1, d) + [0] * d
                    for b, v in enumerate(verifying):
                        if not v:
                            pos[b, :1 + d] = pred[b]
                    ctx_d = torch.tensor([fused_ctx if v else pred_ctx for v in verifying], dtype=torch.int32, device="cuda")
        pos_d, targets = self._forward("speculative", ids, tokens, pos, nv, nf, ctx_d)
        nq = nv + nf
        tg = targets.view(B, nq)
        n_commit = [1] * B
        if nv > 1:
            acc_d = torch.empty(B, dtype=torch.int32, device="cuda")
            nxt_d = torch.empty(B, dtype=torch.int32, device="cuda")
            stops = torch.tensor(list(self.sp.delimiters) + [self.sp.eos], dtype=torch.int32, device="cuda")
            draft_d = torch.from_numpy(np.ascontiguousarray(tokens[:, 1:nv])).cuda()
            M.ms_accept(B, d, draft_d, tg[:, :d].contiguous(), stops, acc_d, nxt_d)
            n_commit = [1 + int(a) if v else 1 for a, v in zip(acc_d.cpu().numpy(), verifying)]
        tg_h = tg.cpu().numpy()
        boundary = set(self.sp.delimiters) | {self.sp.eos}
        for b, s in enumerate(act):
            if int(tokens[b, 0]) in boundary:      # the block's first token already ends the step
                n_commit[b] = 1
        k_new, v_new = self.dec.step_kv()
        M.ms_commit_accepted(self.ses.cache, ids, n_commit, nq, k_new, v_new, pos_d)
        self.obs.commit(ids, n_commit, pos)
        closing = []
        for b, s in enumerate(act):
            kept = [int(t) for t in tokens[b, :n_commit[b]]]
            s.generated += kept
            self.raw_tokens += len(kept)
            self.committed += len(kept)
            self.blocks["verify" if verifying[b] else "predict"] += 1
            last = kept[-1]
            s.next_pid += len(kept)
            s.next_token = int(tg_h[b, len(kept) - 1])          # the greedy token after the last kept one
            # drafts for the next pass: the greedy tokens of the foresight rows that stand right
            # behind the last kept token.  Per-position layout: the d rows of that verify token.
            # Otherwise the foresight rows follow the whole block (or, in a Predict pass, the next
            # token): their position ids and what they saw fit only if all of it was kept.
            if self.per_position:
                f0 = nv + (len(kept) - 1) * d
                s.drafts, s.drafts_valid = [int(t) for t in tg_h[b, f0:f0 + d]], True
            elif not verifying[b]:
                s.drafts, s.drafts_valid = [int(t) for t in tg_h[b, 1:1 + d]], True
            elif len(kept) == nv:
                s.drafts, s.drafts_valid = [int(t) for t in tg_h[b, nv:nv + d]], True
            else:
                s.drafts, s.drafts_valid = [F] * d, False
            if last == self.sp.eos:
                s.finished = True
            elif last in self.sp.delimiters:
                closing.append(s.seq_id)
        return closing

    # ---- Algorithm 1, phase 2: compress a finished step ------------------------------------------------
    def close_step(self, sid: int) -> None:
        s = self.state[sid]
        cur = M.ms_seq_len(self.ses.cache, sid)
        seg_len = cur - s.step_begin
        last_pid = s.step_first_pid + seg_len - 1
        # how many memory tokens: one per c tokens of the step (adaptive memory allocation), or a
        # fixed budget (Appendix B, "w/o AMA")
        l = M.ms_ama_count(seg_len, self.c) if self.fixed_memory is None else self.fixed_memory
        if l + 1 > M.MS_MAX_QUERIES:
            raise M.MsError(M.MS_ERR_UNSUPPORTED, f"step of {seg_len} tokens needs {l + 1} queries in one pass")
        # where they stand: spread over the step's position span (uniform position layout), or on
        # the consecutive positions after the step (Appendix B, "w/o UPL")
        if not self.upl:
            mem_pids = M.ms_consecutive_memory_positions(last_pid, l)
            o_pid = M.ms_output_token_pid(last_pid + l)
        elif self.fixed_memory is None:
            mem_pids = M.ms_upl_positions(s.step_first_pid, seg_len, self.c)
            o_pid = M.ms_output_token_pid(last_pid)
        else:
            mem_pids = M.ms_upl_positions_fixed(s.step_first_pid, seg_len, l)
            o_pid = M.ms_output_token_pid(last_pid)
        tokens = np.asarray([[self.sp.memory] * l + [self.sp.output]], np.int32)
        pos = np.asarray([mem_pids + [o_pid]], np.int32)
        pos_d, targets = self._forward("memory", [sid], tokens, pos, l + 1, 0)
        k_new, v_new = self.dec.step_kv()
        L = k_new.shape[0]
        M.ms_compact_segment(self.ses.cache, [sid], [s.step_begin], [seg_len], [l + 1], k_new.reshape(L, l + 1, *k_new.shape[2:]),
                             v_new.reshape(L, l + 1, *v_new.shape[2:]), pos_d.view(-1))
        self.obs.compact(sid, s.step_begin, seg_len, l + 1, pos[0])
        s.steps_closed += 1
        s.next_token = int(targets[l].item())      # generation continues from <o>'s greedy token
        s.next_pid = o_pid + 1
        s.drafts, s.drafts_valid = [self.sp.foresight] * self.d, False    # no drafts yet for the new step
        s.step_begin = M.ms_seq_len(self.ses.cache, sid)
        s.step_first_pid = s.next_pid

    # ---- the loop -------------------------------------------------------------------------------------
    def run(self, max_passes: int) -> dict:
        """Alternates the two phases until every sequence has produced <eos> or max_passes
        speculative passes were made.  Returns counters, among them the peak number of cache pages
        and what an uncompressed cache would need."""
        for _ in range(max_passes):
            if all(s.finished for s in self.state.values()):
                break
            for sid in self.speculative_step():
                self.close_step(sid)
        return {
            "passes": dict(self.passes),
            "generated": {sid: list(s.generated) for sid, s in self.state.items()},
            "steps_closed": {sid: s.steps_closed for sid, s in self.state.items()},
            "peak_pages": M.ms_peak_pages(self.ses.cache),
            "pages_without_compression": sum(-(-(s.prompt_len + len(s.generated)) // M.MS_PAGE_SIZE)
                                             for s in self.state.values()),
            "cached_tokens": {sid: M.ms_seq_len(self.ses.cache, sid) for sid in self.state},
            "raw_tokens": self.raw_tokens,
            "blocks": dict(self.blocks),
            # tokens committed per sequence and speculative pass (1 = no gain over plain decoding)
            "mean_committed": self.committed / max(1, sum(self.blocks.values())),
        }
