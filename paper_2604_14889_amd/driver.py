"""MemoSight's iterative inference (Appendix A, Algorithm 1 of the paper) on the GPU step by step.

Phase 1, foresight-based acceleration: one fused pass per step over the verify block
[next token, drafts] and d foresight tokens (Section 2.1.1); the drafts that match the model's own
greedy tokens are accepted, the accepted tokens' K/V enter the paged cache, the foresight rows'
greedy tokens are the next drafts.  Phase 2, compression: when a step delimiter is among the
accepted tokens, l = ceil(|R| / c) memory tokens and the output token <o> are run through the model
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


class Observer:
    def forward(self, kind, seq_ids, tokens, pos, n_verify, n_foresight, logits, targets, ctx_new=None):  # noqa: D401
        pass

    def commit(self, seq_ids, n_commit, pos):
        pass

    def compact(self, seq_id, seg_begin, seg_len, n_rows, pos):
        pass


class MemoSightDriver:
    def __init__(self, decoder: Decoder, d: int, c: int, special: SpecialTokens, observer: Optional[Observer] = None,
                 per_position: bool = False):
        """per_position: put d foresight tokens behind EVERY verify token (the layout the model is
        trained on, Section 2.2) instead of behind the block only, so that the drafts for the next
        pass are valid whatever number of verify tokens was kept; costs (d + 1) d instead of d extra
        queries per pass."""
        if d < 0 or c < 1:
            raise ValueError("need d >= 0 and c >= 1")
        if per_position and (d + 1) * (d + 1) > M.MS_MAX_QUERIES:
            raise ValueError("too many queries per pass")
        self.per_position = per_position
        self.dec, self.ses, self.d, self.c, self.sp = decoder, decoder.ses, d, c, special
        self.obs = observer or Observer()
        self.state: Dict[int, SeqState] = {}
        self.passes = {"speculative": 0, "memory": 0, "prefill": 0}
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
        d, nv = self.d, self.d + 1
        ids = [s.seq_id for s in act]
        nf = nv * d if self.per_position else d
        tokens = np.asarray([[s.next_token] + s.drafts + [self.sp.foresight] * nf for s in act], np.int32)
        ctx_d = None
        if self.per_position:
            lay = [M.ms_per_position_layout(s.next_pid, nv, d) for s in act]
            pos = np.asarray([p for p, _ in lay], np.int32)
            ctx_d = torch.tensor([c_ for _, c_ in lay], dtype=torch.int32, device="cuda")
        else:
            pos = M.ms_step_positions(np.asarray([s.next_pid for s in act], np.int32), nv, d)
        pos_d, targets = self._forward("speculative", ids, tokens, pos, nv, nf, ctx_d)
        B, nq = len(act), nv + nf
        tg = targets.view(B, nq)
        n_commit = [1] * B
        if d > 0:
            acc_d = torch.empty(B, dtype=torch.int32, device="cuda")
            nxt_d = torch.empty(B, dtype=torch.int32, device="cuda")
            stops = torch.tensor(list(self.sp.delimiters) + [self.sp.eos], dtype=torch.int32, device="cuda")
            draft_d = torch.from_numpy(np.ascontiguousarray(tokens[:, 1:nv])).cuda()
            M.ms_accept(B, d, draft_d, tg[:, :d].contiguous(), stops, acc_d, nxt_d)
            n_commit = [1 + int(a) for a in acc_d.cpu().numpy()]
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
            last = kept[-1]
            s.next_pid += len(kept)
            s.next_token = int(tg_h[b, len(kept) - 1])          # the greedy token after the last kept one
            # drafts for the next pass: the greedy tokens of the foresight rows behind the last kept
            # verify token; with foresight tokens behind the block only, those are conditioned on the
            # whole block and only have a chance when all of it was kept
            f0 = nv + (len(kept) - 1) * d if self.per_position else nv
            s.drafts = [int(t) for t in tg_h[b, f0:f0 + d]]
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
        l = M.ms_ama_count(seg_len, self.c)
        if l + 1 > M.MS_MAX_QUERIES:
            raise M.MsError(M.MS_ERR_UNSUPPORTED, f"step of {seg_len} tokens needs {l + 1} queries in one pass")
        mem_pids = M.ms_upl_positions(s.step_first_pid, seg_len, self.c)
        o_pid = M.ms_output_token_pid(s.step_first_pid + seg_len - 1)
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
        s.drafts = [self.sp.foresight] * self.d    # no drafts yet for the new step
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
        }
