"""CPU-side checks of the C-ABI library: it loads, exports everything the header declares, and its
pure host helpers agree with the paper's printed values.  No GPU compute is called here."""
import os
import re

import pytest

from paper_2604_14889_amd import binding as M
from tests.test_oracle_layout import G

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "memosight.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ms_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    syms = declared_symbols()
    assert len(syms) >= 20
    for s in syms:
        assert hasattr(M.lib, s), f"{s} declared in memosight.h but not exported"
    assert sorted(M.EXPORTED) == syms


def test_helpers_match_paper_values():
    inp, exp = G["upl"]
    assert M.ms_upl_positions(inp["first_pid"], inp["n"], inp["c"]) == [exp]
    inp, exp = G["ama"]
    assert M.ms_ama_count(inp["n"], inp["c"]) == exp
    inp, exp = G["ama_long"]
    assert M.ms_ama_count(inp["n"], inp["c"]) == exp
    inp, exp = G["output_pid"]
    assert M.ms_output_token_pid(inp["last_pid"]) == exp
    inp, exp = G["foresight_pid"]
    assert M.ms_foresight_pids(exp - 1, 1) == [exp]
    inp, exp = G["drafts_per_pass"]
    assert 1 + len(M.ms_foresight_pids(7, inp["d"])) == exp


def test_helpers_match_oracle_exhaustively():
    from oracle import memosight_oracle as O
    for c in range(1, 10):
        for n in range(0, 70):
            assert M.ms_ama_count(n, c) == O.ama_count(n, c)
            for first in (0, 1, 257):
                assert M.ms_upl_positions(first, n, c) == O.upl_positions(first, n, c)
    for nv in range(0, 7):
        for d in range(0, 6):
            if nv + d == 0:
                continue
            assert M.ms_default_ctx_new(nv, d) == O.default_ctx_new(nv, d)
            assert M.ms_foresight_pids(100 + nv, d) == O.foresight_pids(100 + nv, d)
            pos, ctx = M.ms_per_position_layout(100, nv, d)
            assert (pos, ctx) == O.per_position_layout(100, nv, d)
    for n in range(1, 60):
        for l in (1, 2, 9, 13):
            assert M.ms_upl_positions_fixed(3, n, l) == O.upl_positions_fixed(3, n, l)
    for l in range(0, 12):
        assert M.ms_consecutive_memory_positions(41, l) == O.consecutive_memory_positions(41, l)
    import numpy as np
    first = np.asarray([1, 50, 7000], dtype=np.int32)
    for nv, d in ((5, 4), (1, 0), (0, 3), (4, 3)):
        got = M.ms_step_positions(first, nv, d)
        for b, p0 in enumerate(first):
            ver = list(range(p0, p0 + nv))
            assert got[b].tolist() == ver + O.foresight_pids(int(p0) + nv - 1, d)
    with pytest.raises(M.MsError):
        M.ms_upl_positions_fixed(1, 0, 9)


def test_bad_arguments_return_errors_not_crashes():
    assert M.ms_ama_count(3, 0) < 0
    d = M.make_desc(1, 8, 8, 64, 8, 2, 8, M.MS_F32, 10000.0)
    assert M.ms_pool_bytes(d) == 1 * 8 * 8 * 2 * 16 * 64 * 4
    bad = M.make_desc(1, 7, 4, 64, 8, 2, 8, M.MS_F32, 10000.0)        # 7 not a multiple of 4
    assert M.ms_pool_bytes(bad) == 0
    bad = M.make_desc(1, 8, 8, 96, 8, 2, 8, M.MS_F32, 10000.0)        # unsupported head_dim
    assert M.ms_pool_bytes(bad) == 0
    with pytest.raises(M.MsError) as e:
        M.ms_cache_create(d)                                           # pool is NULL
    assert e.value.code == M.MS_ERR_INVALID and "pool" in str(e.value)
    with pytest.raises(M.MsError):
        M.ms_accept(-1, 4, None, None, None, None, None)
    assert M.lib.ms_hbm_read_probe(None, 1 << 20, 0, None, None, None) == M.MS_ERR_INVALID     # null pointers: refused on the host


def test_projection_workspace_sizes_follow_the_launch_shapes():
    """Host-only sizing functions of the projections (256 compute units assumed without a device).
    Up to 16 rows the few-row kernel divides K only where all rows of A do not fit its LDS share."""
    f = 4   # bytes per fp32 partial sum
    assert M.ms_gemm_workspace_bytes(7, 4608, 3584, 1) == 0                     # a single sequence's Q/K/V: one K part
    assert M.ms_gemm_workspace_bytes(14, 4608, 3584, 1) == 7 * 14 * 4608 * f    # two sequences: A needs two parts, seven fill the chip
    assert M.ms_gemm_workspace_bytes(7, 3584, 18944, 1) == 8 * 7 * 3584 * f     # down projection: eight parts
    assert M.ms_gemm_workspace_bytes(448, 3584, 18944, 4) == 4 * 448 * 3584 * f  # tiled kernel, caller's split
    assert M.ms_gemm_workspace_bytes(448, 4608, 3584, 1) == 0                   # tiled, one round of tiles
    assert M.ms_gemm_workspace_bytes(7, 4600, 3584, 1) == 0                     # unsupported width
    # with the residual add and the norm the K parts are summed by the norm's kernel: at least two
    assert M.ms_gemm_add_rmsnorm_workspace_bytes(7, 3584, 18944, 1) == 8 * 7 * 3584 * f
    assert M.ms_gemm_add_rmsnorm_workspace_bytes(7, 3584, 3584, 1) == 7 * 7 * 3584 * f
    assert M.ms_gemm_add_rmsnorm_workspace_bytes(448, 3584, 18944, 4) == 4 * 448 * 3584 * f
    assert M.ms_gemm_add_rmsnorm_workspace_bytes(448, 3584, 18944, 1) == 0      # above 16 rows the caller must divide K
    # the greedy-token LM head leaves one 8-byte key per row and column group
    assert M.ms_lm_head_argmax_workspace_bytes(7, 152064, 3584) == 152064 // 32 * 7 * 8     # two 16-row tiles per wave
    assert M.ms_lm_head_argmax_workspace_bytes(448, 152064, 3584) == 152064 // 128 * 2 * 448 * 8
