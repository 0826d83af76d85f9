"""Full decode step on the GPU against the fp64 decoder oracle (bf16; a reduced model, and one block at the real widths).

Tolerances: the GPU rounds every GEMM output and activation to bf16 (relative
2^-9 each) through 2 layers and the LM head, so logits carry an error of a few 1e-3 of their scale;
the test allows max-abs 4e-2 x max|ref| and mean-rel 2e-2.  Greedy tokens must agree wherever the
oracle's margin between best and second-best logit exceeds twice the measured max-abs error; accept
lengths and page tables are compared exactly on rows whose decisions have that margin.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import decoder_oracle as DO
from oracle import memosight_oracle as O

pytestmark = pytest.mark.gpu


def _mods():
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import decoder as D
    from paper_2604_14889_amd import session as S
    return M, S, D



def make_weights(rng, cfg):
    """bf16-valued random weights as (uint16 bit arrays for the GPU, float64 arrays for the oracle)."""
    def bits(shape, std, mean=0.0):
        x = (rng.standard_normal(shape) * std + mean).astype(np.float32)
        b = (x.view(np.uint32) >> 16).astype(np.uint16)           # truncation: exact bf16 values
        return b
    qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    layers = []
    for _ in range(cfg.n_layers):
        layers.append(dict(ln1=bits(cfg.hidden, 0.2, 1.0), wq=bits((qd, cfg.hidden), cfg.hidden ** -0.5), bq=bits(qd, 0.1),
                           wk=bits((kd, cfg.hidden), cfg.hidden ** -0.5), bk=bits(kd, 0.1),
                           wv=bits((kd, cfg.hidden), cfg.hidden ** -0.5), bv=bits(kd, 0.1),
                           wo=bits((cfg.hidden, qd), qd ** -0.5), ln2=bits(cfg.hidden, 0.2, 1.0),
                           w_gate=bits((cfg.inter, cfg.hidden), cfg.hidden ** -0.5),
                           w_up=bits((cfg.inter, cfg.hidden), cfg.hidden ** -0.5),
                           w_down=bits((cfg.hidden, cfg.inter), cfg.inter ** -0.5)))
    top = dict(embed=bits((cfg.vocab, cfg.hidden), 1.0), norm=bits(cfg.hidden, 0.2, 1.0),
               lm_head=bits((cfg.vocab, cfg.hidden), cfg.hidden ** -0.5))
    return layers, top


def test_decode_step_matches_oracle_and_commits_accepted_rows():
    M, S, D = _mods()
    cfg = D.DecoderConfig(n_layers=2, hidden=512, inter=1024, vocab=1024, n_q_heads=8, n_kv_heads=2, head_dim=128)
    rng = W.make_rng(700)
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

    # a cache with random (already rotated) contents, shared bit for bit by both sides
    B, nv, nf = 3, 4, 3
    nq = nv + nf
    lengths = [300, 40, 0]
    sh = W.AttnShape("dec", "bf16", B, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, nv, nf, lengths, 0.5, cfg.rope_base,
                     n_layers=cfg.n_layers)
    inp = W.attention_inputs(sh, 701)
    ses = S.Session(cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, sh.n_pages + 8, M.MS_BF16, cfg.rope_base,
                    max_seqs=4, max_pages_per_seq=32, pool=np.concatenate(
                        [inp.pool, np.zeros((cfg.n_layers, 8) + inp.pool.shape[2:], inp.pool.dtype)], axis=1))
    ora = O.PagedCache(cfg.n_layers, cfg.n_kv_heads, cfg.head_dim, sh.n_pages + 8, dtype=O.BF16, rope_base=cfg.rope_base,
                       max_seqs=4, pool=np.concatenate(
                           [O.bf16_bits_to_f32(inp.pool), np.zeros((cfg.n_layers, 8) + inp.pool.shape[2:], np.float32)], axis=1))
    with ses:
        ids = [M.ms_seq_import(ses.cache, n, pt) for n, pt in zip(lengths, inp.page_tables)]
        assert ids == [ora.seq_import(n, pt) for n, pt in zip(lengths, inp.page_tables)]
        first_pid = np.asarray([3 * n + 1 for n in lengths], np.int32)
        pos = M.ms_step_positions(first_pid, nv, nf)

        # verify blocks built with the oracle so that 3, 1 and 0 drafts are right: token j+1 is the
        # greedy continuation of tokens 0..j where a draft is meant to be accepted
        tokens = rng.integers(0, cfg.vocab, size=(B, nq)).astype(np.int32)
        want_ok = [3, 1, 0]
        need_margin = 0.12            # decisions the test relies on must not hinge on bf16 rounding
        for attempt in range(40):
            for j in range(nv - 1):
                r = DO.speculative_step(wts, ora, ids, tokens, pos, nv, nf)
                for b in range(B):
                    if j < want_ok[b]:
                        tokens[b, j + 1] = r.targets[b, j]
                    elif tokens[b, j + 1] == r.targets[b, j]:
                        tokens[b, j + 1] = (tokens[b, j + 1] + 1) % cfg.vocab
            ref = DO.speculative_step(wts, ora, ids, tokens, pos, nv, nf)
            srt = np.sort(ref.logits, axis=-1)
            margin = srt[..., -1] - srt[..., -2]
            weak = [b for b in range(B) if margin[b, :min(want_ok[b] + 1, nv - 1)].min() < need_margin]
            if not weak:
                break
            for b in weak:                                   # another first token, another chain
                tokens[b] = rng.integers(0, cfg.vocab, size=nq)
        assert not weak, "no verify block with clear greedy decisions found"

        dec = D.Decoder(cfg, gw, ses, B * nq)
        logits, targets = dec.step(ids, S.ints_dev(tokens).view(B, nq), S.ints_dev(pos).view(B, nq), nv, nf)
        torch.cuda.synchronize()
        got = logits.float().cpu().numpy().reshape(B, nq, cfg.vocab).astype(np.float64)
        err = np.abs(got - ref.logits)
        scale = np.abs(ref.logits).max()
        max_abs, mean_rel = err.max(), err.mean() / np.abs(ref.logits).mean()
        print(f"logits: max-abs {max_abs:.3e} (scale {scale:.2f}), mean-rel {mean_rel:.3e}")
        assert max_abs <= 4e-2 * scale and mean_rel <= 2e-2
        # LM head and greedy token in one kernel (fp32 sums, no logits): same tokens wherever the decision is clear
        dec_g = D.Decoder(cfg, gw, ses, B * nq, fused_lm_head=True)
        assert dec_g.fused_lm_head
        none_logits, targets_g = dec_g.step(ids, S.ints_dev(tokens).view(B, nq), S.ints_dev(pos).view(B, nq), nv, nf)
        torch.cuda.synchronize()
        assert none_logits is None
        srt_g = np.sort(ref.logits, axis=-1)
        clear_g = (srt_g[..., -1] - srt_g[..., -2]) > 2 * max_abs
        assert (targets_g.cpu().numpy().reshape(B, nq)[clear_g] == ref.targets[clear_g]).all()
        # a single sequence (7 rows): every projection on the few-row kernel, gate/up with SwiGLU in
        # its epilogue, the LM head with and without the greedy token; rows of a step do not depend
        # on the other sequences, so the batch's reference serves
        for b in (0, 2):
            dec_1 = D.Decoder(cfg, gw, ses, nq, fused_lm_head=(b == 2))
            logits_1, targets_1 = dec_1.step(ids[b:b + 1], S.ints_dev(tokens[b:b + 1]).view(1, nq), S.ints_dev(pos[b:b + 1]).view(1, nq), nv, nf)
            torch.cuda.synchronize()
            if b == 0:
                err_1 = np.abs(logits_1.float().cpu().numpy().astype(np.float64) - ref.logits[b])
                print(f"logits (single sequence): max-abs {err_1.max():.3e}, mean-rel {err_1.mean() / np.abs(ref.logits[b]).mean():.3e}")
                assert err_1.max() <= 4e-2 * scale and err_1.mean() / np.abs(ref.logits[b]).mean() <= 2e-2
            else:
                assert logits_1 is None
            assert (targets_1.cpu().numpy()[clear_g[b]] == ref.targets[b][clear_g[b]]).all()
            k_1, _ = dec_1.step_kv()
            assert np.abs(k_1.float().cpu().numpy().reshape(cfg.n_layers, nq, cfg.n_kv_heads, cfg.head_dim) - ref.k_new[:, b]).max() \
                <= 4e-2 * np.abs(ref.k_new).max()
        # greedy tokens wherever the oracle's decision has a margin
        srt = np.sort(ref.logits, axis=-1)
        margin = srt[..., -1] - srt[..., -2]
        clear = margin > 2 * max_abs
        assert clear.mean() > 0.5
        tg = targets.cpu().numpy().reshape(B, nq)
        assert np.array_equal(tg[clear], ref.targets[clear])

        # the step's keys and values (unrotated projections) against the oracle's
        k_new, v_new = dec.step_kv()
        kg = k_new.float().cpu().numpy().reshape(cfg.n_layers, B, nq, cfg.n_kv_heads, cfg.head_dim)
        assert np.abs(kg - ref.k_new).max() <= 4e-2 * np.abs(ref.k_new).max()

        # acceptance on the device from the device's own greedy tokens, then the commit
        acc_d = torch.empty(B, dtype=torch.int32, device="cuda")
        nxt_d = torch.empty(B, dtype=torch.int32, device="cuda")
        tok_d = S.ints_dev(tokens).view(B, nq)
        draft = tok_d[:, 1:nv].contiguous()
        targ = targets.view(B, nq)[:, :nv - 1].contiguous()
        M.ms_accept(B, nv - 1, draft, targ, None, acc_d, nxt_d)
        acc = acc_d.cpu().numpy()
        n_commit_ref, nxt_ref = DO.greedy_accept(tokens[:, :nv], ref.targets[:, :nv])
        decided = [bool(clear[b, :min(n_commit_ref[b], nv - 1)].all()) for b in range(B)]
        assert all(decided), "the test's forced drafts must sit on clear-margin rows"
        assert [1 + int(a) for a in acc] == n_commit_ref == [4, 2, 1]
        n_commit = [1 + int(a) for a in acc]
        M.ms_commit_accepted(ses.cache, ids, n_commit, nq, k_new, v_new, S.ints_dev(pos).view(B, nq))
        for b in range(B):
            ora.append([ids[b]], [n_commit[b]], ref.k_new[:, b, :n_commit[b]], ref.v_new[:, b, :n_commit[b]],
                       pos[b, :n_commit[b]])
            assert M.ms_seq_page_table(ses.cache, ids[b]) == ora.page_table[ids[b]]
            assert M.ms_seq_len(ses.cache, ids[b]) == ora.seq_len[ids[b]] == lengths[b] + n_commit[b]
        M.ms_check_integrity(ses.cache)
        # the committed rows as stored (rotated K, V) agree with the oracle's cache to bf16-GEMM accuracy
        torch.cuda.synchronize()
        gp = O.bf16_bits_to_f32(ses.pool.view(torch.int16).cpu().numpy().view(np.uint16))
        for b in range(B):
            for t in range(lengths[b], lengths[b] + n_commit[b]):
                page, slot = ora.page_table[ids[b]][t // 16], t % 16
                for li in range(cfg.n_layers):
                    a, w = gp[li, page, :, :, slot], ora.pool[li, page, :, :, slot]
                    assert np.abs(a - w).max() <= 4e-2 * max(1.0, np.abs(w).max())


def test_decoder_helper_kernels_against_closed_forms():
    """RMSNorm, SwiGLU, embedding and greedy-token kernels alone, on shapes with ragged tails."""
    M, S, D = _mods()
    rng = W.make_rng(702)
    n, hidden, inter, vocab = 5, 3584, 1000 * 8, 152064 + 0
    bf = lambda b: O.bf16_bits_to_f32(b).astype(np.float64)
    hb = W.normal_bf16_bits(rng, (n, hidden))
    db = W.normal_bf16_bits(rng, (n, hidden))
    wb = W.normal_bf16_bits(rng, (hidden,))
    h = torch.from_numpy(O.bf16_bits_to_f32(hb)).cuda()
    out = torch.empty(n, hidden, dtype=torch.bfloat16, device="cuda")
    M.ms_add_rmsnorm(h, S.to_device(db, M.MS_BF16), S.to_device(wb, M.MS_BF16), 1e-6, out)
    want_h = bf(hb) + bf(db)
    want = DO.rmsnorm(want_h, bf(wb), 1e-6)
    assert np.abs(h.cpu().numpy() - want_h).max() <= 1e-6 * np.abs(want_h).max()          # fp32 residual stream
    assert np.abs(out.float().cpu().numpy() - want).max() <= 2 ** -8 * np.abs(want).max()   # one bf16 rounding
    M.ms_add_rmsnorm(h, None, S.to_device(wb, M.MS_BF16), 1e-6, out)                        # no delta: h unchanged
    assert np.abs(h.cpu().numpy() - want_h).max() <= 1e-6 * np.abs(want_h).max()

    gu = W.normal_bf16_bits(rng, (n, 2 * inter))
    act = torch.empty(n, inter, dtype=torch.bfloat16, device="cuda")
    M.ms_swiglu(S.to_device(gu, M.MS_BF16), act)
    g = bf(gu)
    want = DO.silu(g[:, :inter]) * g[:, inter:]
    assert np.abs(act.float().cpu().numpy() - want).max() <= 2 ** -8 * max(1.0, np.abs(want).max())

    table = W.normal_bf16_bits(rng, (300, hidden))
    toks = np.asarray([0, 299, 17, 17, 5], np.int32)
    hh = torch.empty(n, hidden, dtype=torch.float32, device="cuda")
    M.ms_embed_rows(S.to_device(table, M.MS_BF16), S.ints_dev(toks), hh)
    assert np.array_equal(hh.cpu().numpy(), O.bf16_bits_to_f32(table)[toks])

    for v in (vocab, 1003, 8):
        ld = -(-v // 8) * 8
        lg = W.normal_bf16_bits(rng, (n, ld))
        lg[0, 5] = lg[0, 3] = 0x4200            # 32.0 twice: the lower index wins
        lg[1, v - 1] = 0x4300                    # the last valid column
        if ld > v:
            lg[2, v:] = 0x4400                   # padding columns past the vocabulary are ignored
        lg[3, 0] = 0x7fc0                        # NaN never wins
        res = torch.empty(n, dtype=torch.int32, device="cuda")
        M.ms_argmax_rows(S.to_device(lg, M.MS_BF16), v, res)
        vals = O.bf16_bits_to_f32(lg)[:, :v].astype(np.float64)
        vals[np.isnan(vals)] = -np.inf
        want = vals.argmax(axis=1)
        assert res.cpu().numpy().tolist() == want.tolist()
        assert res[0].item() == 3 and res[1].item() == v - 1


def test_config5_full_widths_one_block_final_norm_and_lm_head():
    """Config 5 at its real widths (hidden 3584, FFN 18944, vocabulary 152064, 28/4 heads x 128) and
    row count (batch 64 x (4 verify + 3 foresight) = 448 rows): one decoder block, the final norm and
    the LM head against the fp64 oracle (0.7 TFLOP of numpy).  One sequence holds 8192 cached tokens,
    the others 16 to 300.  Same tolerances and margin rule as the reduced-model test above."""
    M, S, D = _mods()
    cfg = D.DecoderConfig(n_layers=1, hidden=3584, inter=18944, vocab=152064, n_q_heads=28, n_kv_heads=4, head_dim=128)
    rng = W.make_rng(710)

    def bits(shape, std, mean=0.0):
        x = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if mean:
            x += np.float32(mean)
        return (x.view(np.uint32) >> 16).astype(np.uint16)

    qd, kd, H, I, V = 28 * 128, 4 * 128, cfg.hidden, cfg.inter, cfg.vocab
    l = dict(ln1=bits(H, 0.2, 1.0), wq=bits((qd, H), H ** -0.5), bq=bits(qd, 0.1), wk=bits((kd, H), H ** -0.5), bk=bits(kd, 0.1),
             wv=bits((kd, H), H ** -0.5), bv=bits(kd, 0.1), wo=bits((H, qd), qd ** -0.5), ln2=bits(H, 0.2, 1.0),
             w_gate=bits((I, H), H ** -0.5), w_up=bits((I, H), H ** -0.5), w_down=bits((H, I), I ** -0.5))
    top = dict(embed=bits((V, H), 1.0), norm=bits(H, 0.2, 1.0), lm_head=bits((V, H), H ** -0.5))
    f32 = O.bf16_bits_to_f32                                   # the oracle widens to fp64 where it computes
    wts = DO.DecoderWeights(
        embed=f32(top["embed"]), norm=f32(top["norm"]).astype(np.float64), lm_head=f32(top["lm_head"]),
        layers=[DO.LayerWeights(**{k: f32(v).astype(np.float64) for k, v in l.items()})],
        n_q_heads=28, n_kv_heads=4, head_dim=128, eps=cfg.eps)
    dev = lambda b: S.to_device(b, M.MS_BF16)
    gw = D.DecoderTensors(
        dev(top["embed"]),
        [D.LayerTensors(dev(l["ln1"]), dev(l["wq"]), dev(l["bq"]), dev(l["wk"]), dev(l["bk"]), dev(l["wv"]), dev(l["bv"]),
                        dev(l["wo"]), dev(l["ln2"]), dev(np.concatenate([l["w_gate"], l["w_up"]], axis=0)), dev(l["w_down"]))],
        dev(top["norm"]), dev(top["lm_head"]))

    B, nv, nf = 64, 4, 3
    nq = nv + nf
    lengths = [8192] + [int(x) for x in rng.integers(16, 301, size=B - 1)]
    sh = W.AttnShape("c5", "bf16", B, 28, 4, 128, nv, nf, lengths, 0.5, cfg.rope_base, n_layers=1)
    inp = W.attention_inputs(sh, 711)
    ses, ora, ids = None, None, None
    from tests.test_gpu_parity import setup_pair
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = M.ms_step_positions(np.asarray([3 * n + 1 for n in lengths], np.int32), nv, nf)
        tokens = rng.integers(0, V, size=(B, nq)).astype(np.int32)
        dec = D.Decoder(cfg, gw, ses, B * nq)
        logits, targets = dec.step(ids, S.ints_dev(tokens).view(B, nq), S.ints_dev(pos).view(B, nq), nv, nf)
        torch.cuda.synchronize()
        got = logits.float().cpu().numpy().reshape(B, nq, V)
        tg = targets.cpu().numpy().reshape(B, nq)
        ref = DO.speculative_step(wts, ora, ids, tokens, pos, nv, nf)
        err = np.abs(got - ref.logits)
        scale = np.abs(ref.logits).max()
        max_abs, mean_rel = err.max(), err.mean() / np.abs(ref.logits).mean()
        print(f"config 5 widths, 448 rows: logits max-abs {max_abs:.3e} (scale {scale:.2f}), mean-rel {mean_rel:.3e}")
        assert max_abs <= 4e-2 * scale and mean_rel <= 2e-2
        part = np.partition(ref.logits, V - 2, axis=-1)
        clear = (part[..., -1] - part[..., -2]) > 2 * max_abs
        assert clear.mean() > 0.3, clear.mean()
        assert np.array_equal(tg[clear], ref.targets[clear])
        k_new, v_new = dec.step_kv()
        kg = k_new.float().cpu().numpy().reshape(1, B, nq, 4, 128)
        vg = v_new.float().cpu().numpy().reshape(1, B, nq, 4, 128)
        assert np.abs(kg - ref.k_new).max() <= 4e-2 * np.abs(ref.k_new).max()
        assert np.abs(vg - ref.v_new).max() <= 4e-2 * np.abs(ref.v_new).max()
        # the greedy token straight from the fp32 sums (no logits) at the same widths
        dec_g = D.Decoder(cfg, gw, ses, B * nq, fused_lm_head=True)
        none_logits, targets_g = dec_g.step(ids, S.ints_dev(tokens).view(B, nq), S.ints_dev(pos).view(B, nq), nv, nf)
        torch.cuda.synchronize()
        assert none_logits is None
        assert np.array_equal(targets_g.cpu().numpy().reshape(B, nq)[clear], ref.targets[clear])
