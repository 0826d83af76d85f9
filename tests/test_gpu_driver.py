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


@pytest.mark.parametrize("per_position", [False, True])
def test_algorithm1_driver_runs_in_lockstep_with_the_oracle(per_position):
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

        def check_state(self, seq_ids):
            for s in seq_ids:
                assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s]
                assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s]
            assert M.ms_free_page_count(ses.cache) == ora.free_page_count()

        def forward(self, kind, seq_ids, tokens, pos, nv, nf, logits, targets, ctx_new=None):
            torch.cuda.synchronize()
            if kind == "speculative":
                assert nf == ((d_off + 1) * d_off if per_position else d_off) and (ctx_new is not None) == per_position
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
            assert n_rows == O.ama_count(seg_len, ratio) + 1
            ora.compact([sid], [seg_begin], [seg_len], [n_rows], self.last.k_new[:, 0], self.last.v_new[:, 0], pos)
            self.check_state([sid])

    with ses:
        obs = Lockstep()
        dec = D.Decoder(cfg, gw, ses, 64)
        drv = DR.MemoSightDriver(dec, d_off, ratio, special, obs, per_position=per_position)
        ids = [M.ms_seq_create(ses.cache) for _ in range(2)]
        assert ids == [ora.seq_create() for _ in range(2)]
        prompts = [rng.integers(100, 990, size=70).tolist(), rng.integers(100, 990, size=9).tolist()]
        drv.prefill(ids, prompts)
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
            assert out["cached_tokens"][s] <= len(prompts[ids.index(s)]) + len(out["generated"][s])
        assert sum(out["cached_tokens"].values()) < out["raw_tokens"]
