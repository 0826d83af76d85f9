"""GPU parity at the full sizes of the named configurations, in the launch configuration the
benchmark times: every (query, head) row of whole sequences against the fp64 oracle, attention
at layer indices deep in the pool (0, 13, 27 of 28), after a full-size compaction, and with a
softmax scale of the caller's.  Tolerances as in test_gpu_parity.py (the build target's)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import memosight_oracle as O
from tests.test_gpu_parity import (as_f32, assert_k_rows_close, check_out, oracle_attention, pids_for, run_gpu_attention,
                                   setup_pair)

pytestmark = pytest.mark.gpu


def _mods():
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    return M, S


def whole_sequences_check(sh: W.AttnShape, stream: int, seqs, deterministic: bool = False):
    """All n_q x Hq rows of the given sequences, each over that sequence's whole cache."""
    M, S = _mods()
    inp = W.attention_inputs(sh, stream)
    ses, ora, ids = setup_pair(inp)
    with ses:
        M.ms_attention_set_deterministic(ses.cache, deterministic)
        pos = pids_for(inp, M)
        got = run_gpu_attention(ses, inp, ids, pos)
        assert np.isfinite(got).all()
        worst = (0.0, 0.0)
        for b in seqs:
            want = O.attention_rows(ora, 0, ids[b], as_f32(inp.q[b], "bf16"), as_f32(inp.k_new[b], "bf16"),
                                    as_f32(inp.v_new[b], "bf16"), pos[b], O.default_ctx_new(sh.n_verify, sh.n_foresight))
            assert not np.isnan(want).any()
            r = check_out(got[b], want, "bf16", f"{sh.name} seq {b} len {sh.lengths[b]}")
            worst = (max(worst[0], r[0]), max(worst[1], r[1]))
        print(f"{sh.name}: {len(seqs)} whole sequences, max-abs {worst[0]:.3e} mean-rel {worst[1]:.3e}")
        M.ms_check_integrity(ses.cache)


@pytest.mark.parametrize("deterministic", [False, True])
def test_metric_point_all_rows_of_whole_sequences(deterministic):
    """Batch 32 x 8192 tokens, 5 verify + 4 foresight: all 252 rows of six sequences, in both
    tile-assignment modes."""
    whole_sequences_check(W.metric_point(), 5, [0, 7, 13, 16, 24, 31], deterministic)


def test_config3_ragged_all_rows_of_whole_sequences():
    sh = W.config3()
    order = np.argsort(sh.lengths)
    whole_sequences_check(sh, 3, [int(order[0]), int(order[1]), int(order[len(order) // 2]), int(order[-2]), int(order[-1])])


def test_batch32_kv4096_all_rows_of_whole_sequences():
    whole_sequences_check(W.metric_point(32, 4096), 8, [0, 15, 31])


def test_config4_full_shape_compaction_then_attention_at_layers_0_13_27():
    """Config 4 at its full shape: batch 16, 28 layers, every sequence closes a 256-token segment
    into 8 memory tokens (c = 32), then 4 verify + 3 foresight queries attend over the 2k-8k tokens
    that remain.  The oracle holds layers 0, 13 and 27 (the pool offsets layer * layer_elems reach
    4.8 GB); all 196 rows of the shortest, the longest and a middle sequence are compared at each."""
    M, S = _mods()
    rng = W.make_rng(4, 1)
    B, L, Hq, Hkv, D = 16, 28, 28, 4, 128
    layers = [0, 13, 27]
    lens = [int(16 * x) for x in rng.integers(2304 // 16, 8448 // 16 + 1, size=B)]
    sh3 = W.AttnShape("c4full", "bf16", B, Hq, Hkv, D, 4, 3, lens, 0.5, 1000000.0, n_layers=len(layers), slack_pages=0.02)
    inp = W.attention_inputs(sh3, 44)                        # pool of the three compared layers
    ses = S.Session(L, Hq, Hkv, D, sh3.n_pages, M.MS_BF16, 1000000.0, max_seqs=B, max_pages_per_seq=600)
    ora = O.PagedCache(len(layers), Hkv, D, sh3.n_pages, dtype=O.BF16, rope_base=1000000.0, max_seqs=B,
                       pool=O.bf16_bits_to_f32(inp.pool).copy())
    with ses:
        assert ses.pool.numel() * 2 > 4 << 30
        for i, li in enumerate(layers):
            ses.pool[li].copy_(S.to_device(inp.pool[i], M.MS_BF16))
        ids = [M.ms_seq_import(ses.cache, n, pt) for n, pt in zip(lens, inp.page_tables)]
        assert ids == [ora.seq_import(n, pt) for n, pt in zip(lens, inp.page_tables)]
        c = 32
        n_mem = [M.ms_ama_count(256, c)] * B
        assert n_mem[0] == 8
        begin = [n - 256 for n in lens]
        first_pid = [3 * n for n in lens]
        mpos = sum((M.ms_upl_positions(fp, 256, c) for fp in first_pid), [])
        assert mpos == sum((O.upl_positions(fp, 256, c) for fp in first_pid), [])
        mk = W.normal_bf16_bits(rng, (L, 8 * B, Hkv, D))
        mv = W.normal_bf16_bits(rng, (L, 8 * B, Hkv, D))
        M.ms_compact_segment(ses.cache, ids, begin, [256] * B, n_mem, S.to_device(mk, M.MS_BF16), S.to_device(mv, M.MS_BF16),
                             S.ints_dev(mpos))
        ora.compact(ids, begin, [256] * B, n_mem, O.bf16_bits_to_f32(mk[layers]), O.bf16_bits_to_f32(mv[layers]), mpos)
        for s in ids:
            assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s]
            assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s] == lens[s] - 248
        M.ms_check_integrity(ses.cache)
        new_lens = [n - 248 for n in lens]
        sh_after = W.AttnShape("c4full", "bf16", B, Hq, Hkv, D, 4, 3, new_lens, 0.5, 1000000.0, n_layers=1)
        order = np.argsort(new_lens)
        picks = [int(order[0]), int(order[B // 2]), int(order[-1])]
        worst = (0.0, 0.0)
        for i, li in enumerate(layers):
            q = W.normal_bf16_bits(rng, (B, 7, Hq, D))
            kn, vn = W.normal_bf16_bits(rng, (B, 7, Hkv, D)), W.normal_bf16_bits(rng, (B, 7, Hkv, D))
            step = W.AttnInputs(sh_after, inp.page_tables, None, q, kn, vn, [3 * n + 1 for n in lens])
            pos = pids_for(step, M)
            got = run_gpu_attention(ses, step, ids, pos, layer=li)
            assert np.isfinite(got).all()
            for b in picks:
                want = O.attention_rows(ora, i, ids[b], as_f32(q[b], "bf16"), as_f32(kn[b], "bf16"), as_f32(vn[b], "bf16"),
                                        pos[b], O.default_ctx_new(4, 3))
                r = check_out(got[b], want, "bf16", f"config 4, layer {li}, seq {b} ({new_lens[b]} tokens)")
                worst = (max(worst[0], r[0]), max(worst[1], r[1]))
            # the memory-token rows as stored in this layer
            torch.cuda.synchronize()
            for b in picks:
                for j in (0, 7):
                    t = begin[b] + j
                    p, sl = ora.page_table[ids[b]][t // 16], t % 16
                    row = S.to_host_f32(ses.pool[li, p, :, :, sl])
                    assert np.array_equal(row[:, 1], ora.pool[i, p, :, 1, sl])
                    assert_k_rows_close(row[:, 0], ora.pool[i, p, :, 0, sl])
        print(f"config 4 full shape: layers {layers}, sequences {picks}: max-abs {worst[0]:.3e} mean-rel {worst[1]:.3e}")


@pytest.mark.parametrize("dtype,hq,hkv,d,nv,nf,lengths,scale", [
    ("bf16", 28, 4, 128, 5, 4, [3000, 70, 0, 517], 0.2),        # streaming kernel; default would be 0.088
    ("bf16", 28, 4, 128, 41, 0, [700], 0.03),                   # wide step
    ("f32", 8, 8, 64, 4, 3, [80, 333], 0.31),                   # general kernel; default would be 0.125
    ("bf16", 8, 2, 64, 2, 5, [77, 500], 1.0),
])
def test_attention_with_a_scale_of_the_callers(dtype, hq, hkv, d, nv, nf, lengths, scale):
    """scale != 0 replaces 1 / sqrt(head_dim); compared with the oracle at the same scale, and shown
    to differ from the default-scale result (so the argument is not ignored)."""
    M, S = _mods()
    sh = W.AttnShape("scale", dtype, len(lengths), hq, hkv, d, nv, nf, lengths, 1.0 if dtype == "f32" else 0.5,
                     10000.0 if dtype == "f32" else 1000000.0)
    inp = W.attention_inputs(sh, 460, hq, nv)
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        dt = M.MS_BF16 if dtype == "bf16" else M.MS_F32
        q, kn, vn = (S.to_device(x, dt) for x in (inp.q, inp.k_new, inp.v_new))
        p = S.ints_dev(pos).view(sh.batch, sh.n_q)
        got = S.to_host_f32(ses.attention(0, ids, nv, nf, q, kn, vn, p, None, scale))
        base = S.to_host_f32(ses.attention(0, ids, nv, nf, q, kn, vn, p, None, 0.0))
        want = O.attention(ora, 0, ids, nv, nf, as_f32(inp.q, dtype), as_f32(inp.k_new, dtype), as_f32(inp.v_new, dtype), pos,
                           None, scale)
        check_out(got, want, dtype, f"scale {scale}")
        check_out(base, oracle_attention(ora, inp, ids, pos), dtype, "default scale")
        assert np.abs(got - base).max() > 1e-2
