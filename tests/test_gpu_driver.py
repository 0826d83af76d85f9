"""Algorithm 1 end to end on the GPU (prefill, speculative steps, memory-token passes, compaction)
with the fp64 decoder oracle kept in lockstep: every forward pass is repeated by the oracle on the
same tokens and position ids against its own cache, every cache change is applied to the oracle's
cache with the oracle's own K/V, and logits, greedy tokens (where the margin is clear), page tables
and lengths are compared after each.  Reduced model, bf16, random weights."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import decoder_oracle as DO
from oracle import memosight_oracle as O
from tests.test_gpu_decoder import make_weights

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("per_position,upl,fixed_memory", [(False, True, None), (True, True, None),
                                                           (False, False, None),     # Appendix B, "w/o UPL"
                                                           (False, True, 9)])        # Appendix B, "w/o AMA"
def test_algorithm1_driver_runs_in_lockstep_with_the_oracle(per_position, upl, fixed_memory):
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import decoder as D
    from paper_2604_14889_amd import driver as DR
    from paper_2604_14889_amd import session as S

    cfg = D.DecoderConfig(n_layers=2, hidden=512, inter=1024, vocab=1000, n_q_heads=8, n_kv_heads=2, head_dim=128)
    rng = W.make_rng(800)
    layers, top = make_weights(rng, cfg)
    f64 = lambda b: O.bf16_bits_to_f32(b).astype(np.float64)
    wts = DO.DecoderWeights(
        embed=f64(top["embed"]), norm=f64(top["norm"]), lm_head=f64(top["lm_head"]),
        layers=[DO.LayerWeights(ln1=f64(l["ln1"]), wq=f64(l["wq"]), bq=f64(l["bq"]), wk=f64(l["wk"]), bk=f64(l["bk"]),
                                wv=f64(l["wv"]), bv=f64(l["bv"]), wo=f64(l["wo"]), ln2=f64(l["ln2"]),
                                w_gate=f64(l["w_gate"]), w_up=f64(l["w_up"]), w_down=f64(l["w_down"])) for l in layers],
        n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, eps=cfg.eps)
    dev = lambda b: S.to_device(b, M.MS_BF16)
    gw = D.DecoderTensors(
        dev(top["embed"]),
        [D.LayerTensors(dev(l["ln1"]), dev(l["wq"]), dev(l["bq"]), dev(l["wk"]), dev(l["bk"]), dev(l["wv"]), dev(l["bv"]),
                        dev(l["wo"]), dev(l["ln2"]), dev(np.concatenate([l["w_gate"], l["w_up"]], axis=0)), dev(l["w_down"]))
         for l in layers],
        dev(top["norm"]), dev(top["lm_head"]))

    n_pages = 48
    ses = S.Session(cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, n_pages, M.MS_BF16, cfg.rope_base,
                    max_seqs=4, max_pages_per_seq=24)
    ora = O.PagedCache(cfg.n_layers, cfg.n_kv_heads, cfg.head_dim, n_pages, dtype=O.BF16, rope_base=cfg.rope_base, max_seqs=4)
    special = DR.SpecialTokens(memory=996, output=997, foresight=998, delimiters=list(range(0, 80)), eos=999)
    d_off, ratio = 3, 5

    class Lockstep(DR.Observer):
        def __init__(self):
            self.last = None
            self.n_forward = 0
            self.worst = (0.0, 0.0)
            self.clear = 0
            self.rows = 0
            self.kinds = set()

        def check_state(self, seq_ids):
            for s in seq_ids:
                assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s]
                assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s]
            assert M.ms_free_page_count(ses.cache) == ora.free_page_count()

        def forward(self, kind, seq_ids, tokens, pos, nv, nf, logits, targets, ctx_new=None):
            torch.cuda.synchronize()
            if kind == "speculative":
                if per_position:
                    assert (nv, nf) == (d_off + 1, (d_off + 1) * d_off) and ctx_new is not None
                else:
                    # everyone predicting, everyone verifying (default visibility), or a mix (explicit)
                    assert (nv, nf) in ((1, d_off), (d_off + 1, d_off))
                    if ctx_new is not None:
                        rows = {tuple(r_) for r_ in ctx_new.tolist()}
                        assert rows == {tuple(O.default_ctx_new(d_off + 1, d_off)), tuple(O.default_ctx_new(1, d_off) + [0] * d_off)}
                    self.kinds.add((nv, ctx_new is not None))
            r = DO.speculative_step(wts, ora, seq_ids, tokens, pos, nv, nf, ctx_new)
            got = logits.float().cpu().numpy().reshape(r.logits.shape).astype(np.float64)
            err = np.abs(got - r.logits)
            scale = np.abs(r.logits).max()
            assert err.max() <= 4e-2 * scale, f"{kind} pass {self.n_forward}: max-abs {err.max():.3e} of scale {scale:.2f}"
            mean_rel = err.mean() / np.abs(r.logits).mean()
            assert mean_rel <= 2e-2
            self.worst = (max(self.worst[0], err.max() / scale), max(self.worst[1], mean_rel))
            srt = np.sort(r.logits, axis=-1)
            clear = (srt[..., -1] - srt[..., -2]) > 2 * err.max()
            tg = targets.cpu().numpy().reshape(clear.shape)
            assert np.array_equal(tg[clear], r.targets[clear])
            self.clear += int(clear.sum())
            self.rows += clear.size
            self.last = r
            self.n_forward += 1

        def commit(self, seq_ids, n_commit, pos):
            for b, (s, n) in enumerate(zip(seq_ids, n_commit)):
                ora.append([s], [n], self.last.k_new[:, b, :n], self.last.v_new[:, b, :n], pos[b, :n])
            self.check_state(seq_ids)
            M.ms_check_integrity(ses.cache)

        def compact(self, sid, seg_begin, seg_len, n_rows, pos):
            l = O.ama_count(seg_len, ratio) if fixed_memory is None else fixed_memory
            assert n_rows == l + 1
            last = self.step_first[sid] + seg_len - 1
            if not upl:
                want = O.consecutive_memory_positions(last, l)
                want.append(O.output_token_pid(want[-1]))
            elif fixed_memory is None:
                want = O.upl_positions(self.step_first[sid], seg_len, ratio) + [O.output_token_pid(last)]
            else:
                want = O.upl_positions_fixed(self.step_first[sid], seg_len, l) + [O.output_token_pid(last)]
            assert list(pos) == want
            self.step_first[sid] = want[-1] + 1
            ora.compact([sid], [seg_begin], [seg_len], [n_rows], self.last.k_new[:, 0], self.last.v_new[:, 0], pos)
            self.check_state([sid])

    with ses:
        obs = Lockstep()
        dec = D.Decoder(cfg, gw, ses, 64)
        drv = DR.MemoSightDriver(dec, d_off, ratio, special, obs, per_position=per_position, upl=upl, fixed_memory=fixed_memory)
        ids = [M.ms_seq_create(ses.cache) for _ in range(2)]
        assert ids == [ora.seq_create() for _ in range(2)]
        prompts = [rng.integers(100, 990, size=70).tolist(), rng.integers(100, 990, size=9).tolist()]
        drv.prefill(ids, prompts)
        obs.step_first = {s_: len(p_) + 1 for s_, p_ in zip(ids, prompts)}
        assert obs.n_forward == 3                            # 64 + 6 tokens, then 9
        out = drv.run(max_passes=36)
        print(f"passes {out['passes']}, steps closed {out['steps_closed']}, cached {out['cached_tokens']}, raw {out['raw_tokens']}, "
              f"peak pages {out['peak_pages']} vs {out['pages_without_compression']} uncompressed; "
              f"worst logits error {obs.worst[0]:.2e} of scale, mean-rel {obs.worst[1]:.2e}; clear greedy rows {obs.clear}/{obs.rows}")
        assert out["passes"]["speculative"] >= 10
        assert sum(out["steps_closed"].values()) >= 2 and out["passes"]["memory"] == sum(out["steps_closed"].values())
        assert out["peak_pages"] == ora.peak_pages
        assert obs.clear > obs.rows // 2
        for s in ids:
            assert out["cached_tokens"][s] == ora.seq_len[s]
            # what is cached: the prompt, l + 1 rows per closed step, the open step
            # (a fixed budget of 9 memory tokens is more than these short steps hold: there the cache grows)
            if fixed_memory is None:
                assert out["cached_tokens"][s] <= len(prompts[ids.index(s)]) + len(out["generated"][s])
        if fixed_memory is None:
            assert sum(out["cached_tokens"].values()) < out["raw_tokens"]
        if not per_position:
            assert (1, False) in obs.kinds, obs.kinds      # the first pass after the prompts: Predict only
            assert out["blocks"]["predict"] > 0
        assert 1.0 <= out["mean_committed"] <= d_off + 1


class ToyModel:
    """Stands in for the decoder so that acceptance can be predicted: the "text" is a fixed function
    of the position id, truth(p).  A regular token's row yields truth(p + 1) if the row and every
    in-flight token it sees carry the true tokens of their positions, else a wrong token.  A foresight
    row at position p yields truth(p + 1) under the same condition -- except at every 7th position,
    where foresight is "too hard" and yields a wrong token.  So: drafts taken from foresight rows that
    stood at the right positions and saw only true tokens are mostly right; drafts from rows that
    saw rejected tokens, or stood behind tokens that were not kept, are wrong."""

    def __init__(self, ses, n_layers, n_kv_heads, head_dim, special, truth):
        self.ses, self.sp, self.truth = ses, special, truth
        self.shape = (n_layers, n_kv_heads, head_dim)
        self.gen = torch.Generator(device="cuda")
        self.gen.manual_seed(5)

    def step(self, seq_ids, tokens, pos, n_verify, n_foresight, ctx_new=None):
        tok, p = tokens.cpu().numpy(), pos.cpu().numpy()
        B, nq = tok.shape
        ctx = np.asarray([O.default_ctx_new(n_verify, n_foresight)] * B) if ctx_new is None else ctx_new.cpu().numpy()
        regular = lambda t: t not in (self.sp.foresight, self.sp.memory, self.sp.output)
        targets = np.zeros((B, nq), np.int32)
        for b in range(B):
            for i in range(nq):
                seen = [j for j in range(nq) if j < ctx[b, i] or j == i]
                clean = all(tok[b, j] == self.truth(p[b, j]) for j in seen if regular(tok[b, j]))
                # a foresight token stands in for the tokens between the last regular one it sees and its own position
                behind = max([p[b, j] for j in seen if regular(tok[b, j])], default=None)
                hard = tok[b, i] == self.sp.foresight and (p[b, i] % 7 == 3 or behind is None or not 0 <= p[b, i] - behind <= 4)
                right = self.truth(int(p[b, i]) + 1)
                targets[b, i] = right if clean and not hard else right + 1
        L, hkv, d = self.shape
        self.kv = tuple(torch.randn(L, B * nq, hkv, d, device="cuda", generator=self.gen) for _ in range(2))
        return None, torch.from_numpy(targets.reshape(-1)).cuda()

    def step_kv(self):
        return self.kv


@pytest.mark.parametrize("per_position", [False, True])
def test_drafts_are_accepted_when_foresight_is_right(per_position):
    """Algorithm 1 with a predictable stand-in for the model: the committed tokens must be exactly
    the text (speculation never changes what greedy decoding produces), and more than one token per
    sequence and pass must be committed on average -- drafts that come from the right foresight rows
    are accepted (Section 2.1.1: up to d + 1 tokens per pass)."""
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import driver as DR
    from paper_2604_14889_amd import session as S

    d_off, ratio = 3, 5
    special = DR.SpecialTokens(memory=996, output=997, foresight=998, delimiters=[5], eos=999)
    truth = lambda p: 999 if p >= 330 else (5 if p % 19 == 0 else 100 + (p * 37) % 700)
    ses = S.Session(1, 4, 2, 64, 64, M.MS_F32, 10000.0, max_seqs=4, max_pages_per_seq=32)

    class Pids(DR.Observer):
        def __init__(self):
            self.pids = {}

        def commit(self, seq_ids, n_commit, pos):
            for b, (s_, n) in enumerate(zip(seq_ids, n_commit)):
                self.pids.setdefault(s_, []).extend(int(x) for x in pos[b, :n])

    with ses:
        obs = Pids()
        toy = ToyModel(ses, 1, 2, 64, special, truth)
        drv = DR.MemoSightDriver(toy, d_off, ratio, special, obs, per_position=per_position)
        ids = [M.ms_seq_create(ses.cache) for _ in range(3)]
        prompts = [[truth(p) for p in range(1, n + 1)] for n in (40, 7, 18)]
        drv.prefill(ids, prompts)
        out = drv.run(max_passes=400)
        for s_, prompt in zip(ids, prompts):
            gen_pids = obs.pids[s_][len(prompt):]
            assert len(gen_pids) == len(out["generated"][s_]) > 250
            assert out["generated"][s_] == [truth(p) for p in gen_pids]       # the text, token for token
            assert out["generated"][s_][-1] == special.eos
            assert out["steps_closed"][s_] >= 10
        print(f"per_position={per_position}: {out['mean_committed']:.2f} tokens per sequence and pass, blocks {out['blocks']}, passes {out['passes']}")
        assert out["mean_committed"] > 1.8, out["mean_committed"]
        if not per_position:
            assert out["blocks"]["verify"] > out["blocks"]["predict"] > 0
        M.ms_check_integrity(ses.cache)
