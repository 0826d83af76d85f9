"""ms_predict_verify_attention_static (the entry point for callers that cannot allocate) against
ms_predict_verify_attention on the same inputs: two calls in a row on the library's fixed workspace,
the second with a smaller input; bit-identical with the fixed tile assignment, inside the bf16 /
fp32 attention tolerances otherwise; and against the oracle on the small case.  Collected last."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import memosight_oracle as O
from tests.test_gpu_parity import (BF16_MAX_ABS, BF16_MEAN_REL, as_f32, check_out, oracle_attention, pids_for,
                                   setup_pair)

pytestmark = pytest.mark.gpu


def _mods():
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    return M, S


def both_entry_points(ses, inp, gids, pos, M, S):
    """(existing entry point's output, static entry point's output), device tensors."""
    sh = inp.shape
    dt = M.MS_BF16 if sh.dtype == "bf16" else M.MS_F32
    q, kn, vn = S.to_device(inp.q, dt), S.to_device(inp.k_new, dt), S.to_device(inp.v_new, dt)
    p = S.ints_dev(pos).view(sh.batch, sh.n_q)
    ref = ses.attention(0, gids, sh.n_verify, sh.n_foresight, q, kn, vn, p)
    torch.cuda.synchronize()
    out = torch.full_like(q, float("nan"))
    M.ms_predict_verify_attention_static(ses.cache, 0, gids, sh.n_verify, sh.n_foresight, q, kn, vn, p, None, 0.0, out)
    torch.cuda.synchronize()
    return ref, out


def test_static_workspace_matches_the_workspace_entry_point_twice_in_a_row():
    M, S = _mods()
    # first call: ragged batch with shares that cross sequences and pairs with several partials;
    # second call: a smaller batch, which leaves most of the first call's partials behind it
    big = W.AttnShape("static_big", "bf16", 6, 28, 4, 128, 5, 4, [5000, 64, 3000, 9000, 130, 1], 0.5, 1000000.0)
    small = W.AttnShape("static_small", "bf16", 2, 28, 4, 128, 4, 3, [700, 33], 0.5, 1000000.0)
    results = []
    for deterministic in (True, False):
        for sh, stream in ((big, 71), (small, 72)):
            inp = W.attention_inputs(sh, stream)
            ses, ora, gids = setup_pair(inp, with_oracle_pool=sh is small)
            with ses:
                M.ms_attention_set_deterministic(ses.cache, deterministic)
                pos = pids_for(inp, M)
                ref, out = both_entry_points(ses, inp, gids, pos, M, S)
                assert not torch.isnan(out.float()).any()
                if deterministic:
                    assert torch.equal(ref.view(torch.int16), out.view(torch.int16)), sh.name
                else:
                    g, w = S.to_host_f32(out).astype(np.float64), S.to_host_f32(ref).astype(np.float64)
                    assert np.abs(g - w).max() <= BF16_MAX_ABS and np.abs(g - w).mean() / np.abs(w).mean() <= BF16_MEAN_REL
                if ora is not None:
                    check_out(S.to_host_f32(out), oracle_attention(ora, inp, gids, pos), "bf16", sh.name)
                results.append(sh.name)
    assert len(results) == 4


def test_static_workspace_general_kernel_fp32():
    M, S = _mods()
    for lengths, stream in (([333, 64, 15], 73), ([80], 74)):
        sh = W.AttnShape("static_f32", "f32", len(lengths), 6, 2, 64, 3, 2, lengths, 1.0, 10000.0)
        inp = W.attention_inputs(sh, stream)
        ses, ora, gids = setup_pair(inp)
        with ses:
            pos = pids_for(inp, M)
            ref, out = both_entry_points(ses, inp, gids, pos, M, S)
            assert torch.equal(ref, out)
            check_out(S.to_host_f32(out), oracle_attention(ora, inp, gids, pos), "f32", "static fp32")


def test_static_workspace_rejects_what_does_not_fit():
    M, S = _mods()
    n = 200   # (64 shares + 200 sequences) x 4 KV heads x 33 280 bytes > 32 MiB
    sh = W.AttnShape("static_many", "bf16", n, 28, 4, 128, 1, 0, [16] * n, 0.5, 1000000.0)
    inp = W.attention_inputs(sh, 75)
    ses, _, gids = setup_pair(inp, with_oracle_pool=False)
    with ses:
        assert M.ms_attention_workspace_bytes(ses.cache, n, 1) > M.MS_STATIC_SCRATCH_BYTES
        q, kn, vn = (S.to_device(x, M.MS_BF16) for x in (inp.q, inp.k_new, inp.v_new))
        out = torch.zeros_like(q)
        with pytest.raises(M.MsError) as e:
            M.ms_predict_verify_attention_static(ses.cache, 0, gids, 1, 0, q, kn, vn, S.ints_dev(pids_for(inp, M)).view(n, 1),
                                                 None, 0.0, out)
        assert e.value.code == M.MS_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert not out.float().abs().sum().item()      # nothing was launched
        # the workspace entry point still serves the same call
        ref = ses.attention(0, gids, 1, 0, q, kn, vn, S.ints_dev(pids_for(inp, M)).view(n, 1))
        torch.cuda.synchronize()
        assert torch.isfinite(ref.float()).all()
