"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Tolerances (from the build target): page tables, lengths, accept lengths and tokens bit-exact;
attention outputs max-abs <= 1e-5 for float32 caches, and max-abs <= 2e-2 with mean-rel <= 1e-2
(mean |a-b| / mean |b| over the tensor) for bfloat16 caches against the fp64 oracle on the same
bf16-valued inputs.  Stored K rows of bfloat16 caches may differ from the oracle by one bf16 ulp
(fp32 vs fp64 rotation before the rounding); stored V rows are exact.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import memosight_oracle as O

pytestmark = pytest.mark.gpu

F32_MAX_ABS = 1e-5
BF16_MAX_ABS = 2e-2
BF16_MEAN_REL = 1e-2


def _mods():
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    return M, S


def check_out(got: np.ndarray, want: np.ndarray, dtype: str, what: str = ""):
    mask = ~np.isnan(want)
    g, w = got[mask].astype(np.float64), want[mask]
    max_abs = float(np.abs(g - w).max())
    mean_rel = float(np.abs(g - w).mean() / max(np.abs(w).mean(), 1e-30))
    if dtype == "f32":
        assert max_abs <= F32_MAX_ABS, f"{what}: max-abs {max_abs:.3e}"
    else:
        assert max_abs <= BF16_MAX_ABS and mean_rel <= BF16_MEAN_REL, \
            f"{what}: max-abs {max_abs:.3e} mean-rel {mean_rel:.3e}"
    return max_abs, mean_rel



def assert_k_rows_close(a: np.ndarray, b: np.ndarray):
    """Stored bf16 K rows: at most one bf16 ulp from the oracle (fp32 vs fp64 rotation ahead of the
    rounding), plus the fp32 rotation error itself where cancellation leaves a tiny result."""
    bad = np.abs(a - b) > np.abs(b) * 2.0 ** -7 + 1e-6
    assert not bad.any(), f"{int(bad.sum())} elements off, worst {float(np.abs(a - b).max()):.3e}"


def as_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    return O.bf16_bits_to_f32(x) if dtype == "bf16" else x


def pids_for(inp: W.AttnInputs, M):
    """Position ids [B, n_q]: verify block consecutive from first_pid, foresight after it; from the
    library's helper on the GPU side and the oracle's on the other, asserted equal."""
    sh = inp.shape
    rows_lib, rows_ora = [], []
    for b in range(sh.batch):
        ver = list(range(inp.first_pid[b], inp.first_pid[b] + sh.n_verify))
        last = ver[-1] if ver else inp.first_pid[b] - 1
        rows_lib.append(ver + M.ms_foresight_pids(last, sh.n_foresight))
        rows_ora.append(ver + O.foresight_pids(last, sh.n_foresight))
    assert rows_lib == rows_ora
    return np.asarray(rows_ora, dtype=np.int32)


def setup_pair(inp: W.AttnInputs, with_oracle_pool: bool = True):
    """Session (GPU) and oracle cache holding the same imported sequences."""
    M, S = _mods()
    sh = inp.shape
    dt = M.MS_BF16 if sh.dtype == "bf16" else M.MS_F32
    max_pp = max(4, max(len(p) for p in inp.page_tables) + 2)
    ses = S.Session(sh.n_layers, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.n_pages, dt, sh.rope_base,
                    max_seqs=max(4, sh.batch), max_pages_per_seq=max_pp, pool=inp.pool)
    ora = None
    if with_oracle_pool:
        ora = O.PagedCache(sh.n_layers, sh.n_kv_heads, sh.head_dim, sh.n_pages,
                           dtype=O.BF16 if sh.dtype == "bf16" else O.F32, rope_base=sh.rope_base,
                           max_seqs=max(4, sh.batch), pool=as_f32(inp.pool, sh.dtype).copy())
    gids, oids = [], []
    for n, pt in zip(sh.lengths, inp.page_tables):
        gids.append(M.ms_seq_import(ses.cache, n, pt))
        if ora is not None:
            oids.append(ora.seq_import(n, pt))
    if ora is not None:
        assert gids == oids
    return ses, ora, gids


def run_gpu_attention(ses, inp, gids, pos, layer=0, ctx_new=None):
    M, S = _mods()
    sh = inp.shape
    dt = M.MS_BF16 if sh.dtype == "bf16" else M.MS_F32
    q, kn, vn = S.to_device(inp.q, dt), S.to_device(inp.k_new, dt), S.to_device(inp.v_new, dt)
    cn = None if ctx_new is None else S.ints_dev(ctx_new).view(sh.batch, sh.n_q)
    out = ses.attention(layer, gids, sh.n_verify, sh.n_foresight, q, kn, vn,
                        S.ints_dev(pos).view(sh.batch, sh.n_q), cn)
    torch.cuda.synchronize()
    return S.to_host_f32(out)


def oracle_attention(ora, inp, oids, pos, layer=0, ctx_new=None):
    sh = inp.shape
    return O.attention(ora, layer, oids, sh.n_verify, sh.n_foresight, as_f32(inp.q, sh.dtype),
                       as_f32(inp.k_new, sh.dtype), as_f32(inp.v_new, sh.dtype), pos, ctx_new)


# ------------------------------------------------------------------ attention, small shapes ---

SMALL = [
    # dtype, Hq, Hkv, D, n_verify, n_foresight, lengths
    ("f32", 8, 8, 64, 4, 3, [80]),
    ("f32", 4, 2, 128, 1, 0, [0, 1, 17, 200]),
    ("f32", 6, 2, 64, 3, 2, [333, 64, 15]),
    ("bf16", 28, 4, 128, 4, 3, [300, 1, 0, 129]),
    ("bf16", 28, 4, 128, 5, 4, [1000, 2047, 16, 700]),
    ("bf16", 8, 2, 64, 2, 5, [77, 500]),
    ("bf16", 28, 4, 128, 0, 3, [260]),
    ("bf16", 28, 4, 128, 9, 0, [515, 31]),
    ("bf16", 4, 4, 128, 12, 4, [100, 1500]),
    ("bf16", 28, 4, 128, 1, 0, [777, 32, 33]),          # plain decode: one query, 7 rows per KV head
    ("bf16", 28, 4, 128, 4, 3, [0, 0]),                 # nothing cached yet: in-flight tokens only
    ("bf16", 32, 8, 128, 5, 4, [4096 + 17, 31, 2048]),  # group of 4: 36 rows per KV head
    ("bf16", 28, 4, 128, 5, 4, [5000, 64, 3000, 9000, 130, 7000, 1, 2500]),  # shares cross sequences
    # wide steps (more than 64 rows per KV head or more than 16 queries): several query chunks
    ("bf16", 28, 4, 128, 10, 0, [100, 33]),             # 70 rows: two chunks, one in-flight tile
    ("bf16", 28, 4, 128, 41, 0, [700]),                 # memory-token pass, l + 1 = 41: two in-flight tiles
    ("bf16", 28, 4, 128, 64, 0, [300, 0, 2100]),        # the largest step
    ("bf16", 32, 8, 128, 5, 20, [513, 64]),             # 25 queries, group of 4
    ("bf16", 4, 4, 128, 33, 7, [90]),                   # one head per KV head, 40 queries in one chunk
    ("f32", 8, 2, 64, 30, 10, [70, 5]),                 # general kernel, 40 queries
    ("bf16", 8, 2, 64, 17, 0, [129]),
    ("bf16", 28, 4, 128, 41, 0, [5000, 64, 3000, 0]),   # wide steps over caches cut into many shares: several partials per chunk
    ("bf16", 28, 4, 128, 64, 0, [9000]),
    ("bf16", 64, 4, 128, 40, 0, [700, 33]),             # 16 query heads per KV head: 4 queries per chunk, two launches
    ("bf16", 28, 4, 128, 17, 8, [2048, 2047, 31]),      # foresight rows in a wide step
    # the largest batch: 256 short sequences (many segments per workgroup, some sequences empty)
    ("bf16", 28, 4, 128, 2, 1, [(37 * i) % 97 for i in range(256)]),
    ("f32", 4, 2, 64, 1, 1, [(11 * i) % 40 for i in range(256)]),
]


@pytest.mark.parametrize("dtype,hq,hkv,d,nv,nf,lengths", SMALL)
def test_attention_small_shapes_match_oracle(dtype, hq, hkv, d, nv, nf, lengths):
    M, S = _mods()
    sh = W.AttnShape("small", dtype, len(lengths), hq, hkv, d, nv, nf, lengths,
                     1.0 if dtype == "f32" else 0.5, 10000.0 if dtype == "f32" else 1000000.0, n_layers=2)
    inp = W.attention_inputs(sh, 400, hq, d, nv, len(lengths))
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        for layer in (0, 1):
            got = run_gpu_attention(ses, inp, ids, pos, layer)
            want = oracle_attention(ora, inp, ids, pos, layer)
            check_out(got, want, dtype, f"layer {layer}")
        M.ms_check_integrity(ses.cache)


BOUNDARY_LENGTHS = [0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 511, 512, 513, 1000, 2047, 2048, 4095, 4096, 4097]


@pytest.mark.parametrize("case", range(16))
def test_attention_random_batches_of_boundary_lengths(case):
    """Seeded random batches whose lengths sit on page (16), tile (32) and round (256) boundaries,
    with random head groupings and step shapes: exercises the share planner (empty sequences,
    segments that end exactly on a tile, shares crossing several sequences) on the streaming kernel."""
    M, S = _mods()
    rng = W.make_rng(450, case)
    hq, hkv = [(28, 4), (32, 8), (8, 8), (16, 2), (64, 1)][case % 5]
    g = hq // hkv
    batch = int(rng.integers(1, 13))
    lengths = [int(rng.choice(BOUNDARY_LENGTHS)) for _ in range(batch)]
    if case % 4 == 0:
        lengths[int(rng.integers(batch))] = int(rng.integers(5000, 12000))   # one long sequence among short ones
    n_q = int(rng.integers(1, 17 if g <= 4 else max(2, 64 // g + 3)))
    nv = int(rng.integers(0, n_q + 1))
    nf = n_q - nv
    sh = W.AttnShape(f"rand{case}", "bf16", batch, hq, hkv, 128, nv, nf, lengths, 0.5, 1000000.0)
    inp = W.attention_inputs(sh, 451, case)
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        got = run_gpu_attention(ses, inp, ids, pos)
        want = oracle_attention(ora, inp, ids, pos)
        assert np.isfinite(got).all()
        check_out(got, want, "bf16", f"case {case}: heads {hq}/{hkv}, verify {nv} foresight {nf}, lengths {lengths}")
        M.ms_check_integrity(ses.cache)


def test_attention_custom_ctx_new_and_peaked_scores():
    M, S = _mods()
    sh = W.AttnShape("ctx", "bf16", 2, 28, 4, 128, 4, 3, [450, 130], 0.5, 1000000.0)
    inp = W.attention_inputs(sh, 401, peaked=0.05)
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        # per-position foresight layout: foresight j hangs off verify token j (sees j+1 verify tokens)
        ctx = np.asarray([[0, 1, 2, 3, 1, 2, 3], [0, 1, 2, 3, 4, 4, 4]], dtype=np.int32)
        got = run_gpu_attention(ses, inp, ids, pos, ctx_new=ctx)
        want = oracle_attention(ora, inp, ids, pos, ctx_new=ctx)
        check_out(got, want, "bf16", "custom ctx_new, peaked")


def test_per_position_foresight_layout_wide_step():
    """Foresight tokens after every verify token (the layout the model is trained on, Section 2.3
    "MTP Attention"; at inference it keeps drafts alive after a partial acceptance): 5 verify
    tokens, 4 foresight tokens behind each, plus rows that see no other in-flight token at all,
    some of them in the second in-flight tile."""
    M, S = _mods()
    nv, d = 5, 4
    n_extra = 12                      # rows with ctx 0 at query indices 25 .. 36
    nq = nv + nv * d + n_extra
    sh = W.AttnShape("ppf", "bf16", 2, 28, 4, 128, nv, nq - nv, [450, 40], 0.5, 1000000.0)
    inp = W.attention_inputs(sh, 402)
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = np.zeros((2, nq), np.int32)
        ctx = np.zeros((2, nq), np.int32)
        for b in range(2):
            p0 = inp.first_pid[b]
            lay = M.ms_per_position_layout(p0, nv, d)
            assert lay == O.per_position_layout(p0, nv, d)
            pos[b, :nv * (1 + d)], ctx[b, :nv * (1 + d)] = lay
            pos[b, nv + nv * d:] = p0 + nv + np.arange(n_extra)
        got = run_gpu_attention(ses, inp, ids, pos, ctx_new=ctx)
        want = oracle_attention(ora, inp, ids, pos, ctx_new=ctx)
        assert np.isfinite(got).all()
        check_out(got, want, "bf16", "per-position foresight")


def test_gpu_foresight_rows_independent_and_page_permutation_invariant():
    M, S = _mods()
    sh = W.AttnShape("inv", "bf16", 1, 28, 4, 128, 4, 3, [700], 0.5, 1000000.0)
    inp = W.attention_inputs(sh, 402)
    ses, _, ids = setup_pair(inp, with_oracle_pool=False)
    with ses:
        pos = pids_for(inp, M)
        loose = run_gpu_attention(ses, inp, ids, pos)       # default mode: reproducible to rounding
        M.ms_attention_set_deterministic(ses.cache, True)   # bitwise statements need the fixed tile order
        base = run_gpu_attention(ses, inp, ids, pos)
        assert np.array_equal(run_gpu_attention(ses, inp, ids, pos), base)
        check_out(loose, base, "bf16", "default against deterministic mode")
        inp2 = W.attention_inputs(sh, 402)
        inp2.q[0, 5] ^= 0x0100          # perturb foresight query 5 and its key / value
        inp2.k_new[0, 5] ^= 0x0080
        inp2.v_new[0, 5] ^= 0x0040
        got = run_gpu_attention(ses, inp2, ids, pos)
        others = [0, 1, 2, 3, 4, 6]
        assert np.array_equal(got[0, others], base[0, others])
        assert not np.array_equal(got[0, 5], base[0, 5])
    # same logical content under a different physical page placement: bit-identical output
    rng = W.make_rng(4020)
    perm = rng.permutation(sh.n_pages)
    pool2 = np.zeros_like(inp.pool)
    pool2[:, perm] = inp.pool
    inp3 = W.AttnInputs(sh, [[int(perm[p]) for p in inp.page_tables[0]]], pool2, inp.q, inp.k_new, inp.v_new,
                        inp.first_pid)
    ses3, _, ids3 = setup_pair(inp3, with_oracle_pool=False)
    with ses3:
        M.ms_attention_set_deterministic(ses3.cache, True)
        got3 = run_gpu_attention(ses3, inp3, ids3, pos)
    assert np.array_equal(got3, base)


def test_layer_pool_above_4_gib():
    """A 4.6 GB layer pool (140 000 pages): byte offsets of pages no longer fit 32 bits, the
    streaming kernel's build with 64-bit page bases runs.  The same logical content is placed once
    in a small pool and once on pages spread over the large one (some beyond the 4 GiB mark); with
    the fixed tile assignment both must give the same bits, and match the oracle."""
    M, S = _mods()
    sh = W.AttnShape("bigpool", "bf16", 3, 28, 4, 128, 5, 4, [3000, 70, 1500], 0.5, 1000000.0)
    inp = W.attention_inputs(sh, 404)
    ses, ora, ids = setup_pair(inp)
    with ses:
        M.ms_attention_set_deterministic(ses.cache, True)
        pos = pids_for(inp, M)
        base = run_gpu_attention(ses, inp, ids, pos)
        check_out(base, oracle_attention(ora, inp, ids, pos), "bf16", "small pool")
    n_big = 140000
    assert n_big * 4 * 2 * 16 * 128 * 2 > 1 << 32
    to_big = lambda p: n_big - 1 - 440 * p               # page 0 -> the last page, later ones further down
    assert sh.n_pages * 440 < n_big and to_big(10) * 32768 > 1 << 32
    big = S.Session(1, 28, 4, 128, n_big, M.MS_BF16, 1000000.0, max_seqs=4, max_pages_per_seq=256)
    with big:
        small_pool = S.to_device(inp.pool, M.MS_BF16)
        big.pool[0, torch.tensor([to_big(p) for p in range(sh.n_pages)], device="cuda")] = small_pool[0]
        del small_pool
        gids = [M.ms_seq_import(big.cache, n, [to_big(p) for p in pt]) for n, pt in zip(sh.lengths, inp.page_tables)]
        M.ms_attention_set_deterministic(big.cache, True)
        got = run_gpu_attention(big, inp, gids, pos)
        assert np.array_equal(got, base)
        M.ms_attention_set_deterministic(big.cache, False)
        check_out(run_gpu_attention(big, inp, gids, pos), base, "bf16", "large pool, default assignment")
        M.ms_check_integrity(big.cache)


def test_repeated_launches_agree_with_many_partials_per_pair():
    """Race check for the closing of (sequence, KV head) pairs: long sequences in a small batch are
    cut into many shares (up to ~25 partials per pair here), and whichever share finishes last folds
    the others.  Thirty launches in a row must give the same bits with the fixed tile assignment and
    stay within rounding of them with the default one."""
    M, S = _mods()
    sh = W.AttnShape("rep", "bf16", 5, 28, 4, 128, 5, 4, [9000, 100, 4000, 33, 7000], 0.5, 1000000.0, n_layers=2)
    inp = W.attention_inputs(sh, 403)
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        want = oracle_attention(ora, inp, ids, pos, 1)
        M.ms_attention_set_deterministic(ses.cache, True)
        base = run_gpu_attention(ses, inp, ids, pos, 1)
        check_out(base, want, "bf16", "fixed assignment")
        for i in range(30):
            again = run_gpu_attention(ses, inp, ids, pos, i % 2)
            if i % 2 == 1:
                assert np.array_equal(again, base), f"launch {i} differs"
        M.ms_attention_set_deterministic(ses.cache, False)
        for i in range(30):
            again = run_gpu_attention(ses, inp, ids, pos, 1)
            # a different summation order moves a result by a bf16 unit in the last place at most
            assert (np.abs(again - base) <= 2.0 ** -7 * np.abs(base) + 2e-4).all(), f"launch {i}: {np.abs(again - base).max():.3e}"
            check_out(again, want, "bf16", f"default assignment, launch {i}")


def test_profiling_spans_count_calls_and_leave_results_alone():
    """The event pairs of ms_profile_attention: every stride-th call opens a span of `span` calls, an
    unfinished span is not reported, a read resets the count, the outputs do not change."""
    M, S = _mods()
    sh = W.AttnShape("prof", "bf16", 3, 28, 4, 128, 4, 3, [700, 2100, 50], 0.5, 1000000.0, n_layers=2)
    inp = W.attention_inputs(sh, 404)
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        M.ms_attention_set_deterministic(ses.cache, True)
        base = run_gpu_attention(ses, inp, ids, pos, 0)
        check_out(base, oracle_attention(ora, inp, ids, pos, 0), "bf16", "before profiling")
        for bad in ((4, 0, 1), (4, 2, 3), (4, 2, 0), (-1, 1, 1)):
            with pytest.raises(M.MsError):
                M.ms_profile_attention(ses.cache, *bad)
        M.ms_profile_attention(ses.cache, 8, 3, 2)
        for i in range(7):      # spans open at calls 0, 3, 6; the last one stays open
            assert np.array_equal(run_gpu_attention(ses, inp, ids, pos, 0), base), f"call {i}"
        ms = M.ms_profile_read(ses.cache, 8)
        assert len(ms) == 2 and all(0.0 < t < 50.0 for t in ms), ms
        assert M.ms_profile_read(ses.cache, 8) == []
        run_gpu_attention(ses, inp, ids, pos, 0)      # the read dropped the open span: nothing to close
        assert M.ms_profile_read(ses.cache, 8) == []
        M.ms_profile_attention(ses.cache, 2, 1, 1)
        for i in range(5):      # capacity 2: only the first two calls are recorded
            run_gpu_attention(ses, inp, ids, pos, 0)
        assert len(M.ms_profile_read(ses.cache, 8)) == 2
        M.ms_profile_attention(ses.cache, 0, 1, 1)
        assert np.array_equal(run_gpu_attention(ses, inp, ids, pos, 0), base)
        assert M.ms_profile_read(ses.cache, 8) == []


# ------------------------------------------------------------------ the named configurations ---

def test_config1_fp32_built_through_append_and_compact():
    """One layer, fp32, 8 heads x 64: four 64-token segments each compacted to 4 memory tokens
    (c = 16), a 64-token live tail, then 4 verify + 3 foresight queries; acceptance on vocab 1000."""
    M, S = _mods()
    rng = W.make_rng(1)
    H, D = 8, 64
    ses = S.Session(1, H, H, D, 12, M.MS_F32, 10000.0, max_seqs=2, max_pages_per_seq=8)
    ora = O.PagedCache(1, H, D, 12, dtype=O.F32, rope_base=10000.0, max_seqs=2)
    with ses:
        g, o = M.ms_seq_create(ses.cache), ora.seq_create()
        assert g == o
        pid = 1
        for seg in range(4):
            k, v = W.normal_f32(rng, (1, 64, H, D)), W.normal_f32(rng, (1, 64, H, D))
            pos = list(range(pid, pid + 64))
            begin = M.ms_seq_len(ses.cache, g)
            M.ms_append_kv(ses.cache, [g], [64], S.to_device(k, M.MS_F32), S.to_device(v, M.MS_F32), S.ints_dev(pos))
            ora.append([o], [64], k, v, pos)
            l = M.ms_ama_count(64, 16)
            assert l == O.ama_count(64, 16) == 4
            mpos = M.ms_upl_positions(pid, 64, 16)
            assert mpos == O.upl_positions(pid, 64, 16)
            mk, mv = W.normal_f32(rng, (1, l, H, D)), W.normal_f32(rng, (1, l, H, D))
            M.ms_compact_segment(ses.cache, [g], [begin], [64], [l], S.to_device(mk, M.MS_F32),
                                 S.to_device(mv, M.MS_F32), S.ints_dev(mpos))
            ora.compact([o], [begin], [64], [l], mk, mv, mpos)
            assert M.ms_seq_len(ses.cache, g) == ora.seq_len[o] == 4 * (seg + 1)
            assert M.ms_seq_page_table(ses.cache, g) == ora.page_table[o]
            M.ms_check_integrity(ses.cache)
            pid += 64
        k, v = W.normal_f32(rng, (1, 64, H, D)), W.normal_f32(rng, (1, 64, H, D))
        pos = list(range(257, 321))
        M.ms_append_kv(ses.cache, [g], [64], S.to_device(k, M.MS_F32), S.to_device(v, M.MS_F32), S.ints_dev(pos))
        ora.append([o], [64], k, v, pos)
        assert M.ms_seq_len(ses.cache, g) == 80
        assert M.ms_seq_page_table(ses.cache, g) == ora.page_table[o] == [0, 1, 2, 3, 4]
        assert M.ms_free_page_count(ses.cache) == ora.free_page_count() == 7
        assert M.ms_peak_pages(ses.cache) == ora.peak_pages
        M.ms_check_integrity(ses.cache)
        # stored rows
        torch.cuda.synchronize()
        gp = ses.pool_host_f32()
        for p in ora.page_table[o]:
            assert np.abs(gp[0, p] - ora.pool[0, p]).max() < 3e-6
        # attention: PIDs 321..324 verify, 325..327 foresight
        ver = list(range(321, 325))
        fpos = M.ms_foresight_pids(ver[-1], 3)
        assert fpos == O.foresight_pids(ver[-1], 3) == [325, 326, 327]
        pos_q = np.asarray([ver + fpos], dtype=np.int32)
        q = W.normal_f32(rng, (1, 7, H, D))
        kn, vn = W.normal_f32(rng, (1, 7, H, D)), W.normal_f32(rng, (1, 7, H, D))
        out = ses.attention(0, [g], 4, 3, S.to_device(q, M.MS_F32), S.to_device(kn, M.MS_F32),
                            S.to_device(vn, M.MS_F32), S.ints_dev(pos_q).view(1, 7))
        want = O.attention(ora, 0, [o], 4, 3, q, kn, vn, pos_q)
        check_out(S.to_host_f32(out), want, "f32", "config 1")
        # acceptance, every accepted length 0..4 forced plus free draws
        forced = [0, 1, 2, 3, 4]
        draft, target = W.draft_and_target(rng, 5, 4, 1000, forced)
        d2, t2 = W.draft_and_target(rng, 27, 4, 1000)
        draft, target = np.concatenate([draft, d2]), np.concatenate([target, t2])
        acc, nxt = torch.empty(32, dtype=torch.int32, device="cuda"), torch.empty(32, dtype=torch.int32, device="cuda")
        M.ms_accept(32, 4, S.ints_dev(draft), S.ints_dev(target), None, acc, nxt)
        wa, wn = O.accept(draft, target)
        assert np.array_equal(acc.cpu().numpy(), wa) and np.array_equal(nxt.cpu().numpy(), wn)
        assert wa[:5].tolist() == forced


def test_config2_bf16_batch1_4k_all_rows():
    M, S = _mods()
    sh = W.config2()
    inp = W.attention_inputs(sh, 2)
    assert inp.first_pid == [12289]
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        assert pos[0].tolist() == [12289, 12290, 12291, 12292, 12293, 12294, 12295]
        got = run_gpu_attention(ses, inp, ids, pos)
        want = oracle_attention(ora, inp, ids, pos)
        print("config2 max-abs %.3e mean-rel %.3e" % check_out(got, want, "bf16", "config 2"))
        inp_p = W.attention_inputs(sh, 2, peaked=0.01)
    ses, ora, ids = setup_pair(inp_p)
    with ses:
        got = run_gpu_attention(ses, inp_p, ids, pos)
        want = oracle_attention(ora, inp_p, ids, pos)
        check_out(got, want, "bf16", "config 2 peaked")


def sampled_rows_check(sh: W.AttnShape, stream: int, seqs_to_check, rows_per_seq: int):
    """Full-size run on the GPU in the benchmark's launch configuration; the oracle computes sampled
    (query, head) rows one by one, each over that sequence's whole cache."""
    M, S = _mods()
    inp = W.attention_inputs(sh, stream)
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        got = run_gpu_attention(ses, inp, ids, pos)
        assert np.isfinite(got).all()
        rng = W.make_rng(stream, 77)
        worst = (0.0, 0.0)
        for b in seqs_to_check:
            rows = [(int(rng.integers(sh.n_q)), int(rng.integers(sh.n_q_heads))) for _ in range(rows_per_seq)]
            rows += [(sh.n_q - 1, sh.n_q_heads - 1), (0, 0)]
            want = O.attention_rows(ora, 0, ids[b], as_f32(inp.q[b], "bf16"), as_f32(inp.k_new[b], "bf16"),
                                    as_f32(inp.v_new[b], "bf16"), pos[b],
                                    O.default_ctx_new(sh.n_verify, sh.n_foresight), rows=rows)
            r = check_out(got[b], want, "bf16", f"{sh.name} seq {b} len {sh.lengths[b]}")
            worst = (max(worst[0], r[0]), max(worst[1], r[1]))
        print(f"{sh.name}: sampled max-abs {worst[0]:.3e} mean-rel {worst[1]:.3e}")
        M.ms_check_integrity(ses.cache)


def test_config3_ragged_batch32_sampled():
    sh = W.config3()
    order = np.argsort(sh.lengths)
    picks = [int(order[0]), int(order[-1]), int(order[len(order) // 2]), 0, 31]
    sampled_rows_check(sh, 3, picks, 4)


def test_one_very_long_sequence_sampled():
    """131k cached tokens in one sequence next to a short one: every workgroup but one works on the
    same sequence (64 partials per KV head to combine), position ids near 4e5 (large RoPE angles)."""
    sh = W.AttnShape("long", "bf16", 2, 28, 4, 128, 5, 4, [131072 + 13, 100], 0.5, 1000000.0)
    sampled_rows_check(sh, 6, [0, 1], 4)


def test_metric_point_batch32_kv8192_sampled():
    sampled_rows_check(W.metric_point(), 5, [0, 13, 31], 4)


# ------------------------------------------------------------------ append / commit ----------

def test_append_bf16_rows_and_page_tables():
    M, S = _mods()
    rng = W.make_rng(410)
    L, Hkv, D, NP = 3, 4, 128, 40
    ses = S.Session(L, 28, Hkv, D, NP, M.MS_BF16, 1000000.0, max_seqs=4, max_pages_per_seq=16)
    ora = O.PagedCache(L, Hkv, D, NP, dtype=O.BF16, rope_base=1000000.0, max_seqs=4)
    with ses:
        gs = [M.ms_seq_create(ses.cache) for _ in range(3)]
        os_ = [ora.seq_create() for _ in range(3)]
        assert gs == os_
        for step, counts in enumerate([[5, 40, 16], [30, 1, 0], [13, 7, 100]]):
            n = sum(counts)
            k, v = W.normal_bf16_bits(rng, (L, n, Hkv, D)), W.normal_bf16_bits(rng, (L, n, Hkv, D))
            pos = rng.integers(0, 50000, size=n).astype(np.int32)
            order = [2, 0, 1] if step == 1 else [0, 1, 2]
            sid = [gs[i] for i in order]
            cnt = [counts[i] for i in order]
            M.ms_append_kv(ses.cache, sid, cnt, S.to_device(k, M.MS_BF16), S.to_device(v, M.MS_BF16), S.ints_dev(pos))
            ora.append(sid, cnt, O.bf16_bits_to_f32(k), O.bf16_bits_to_f32(v), pos)
            for s in gs:
                assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s]
                assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s]
            M.ms_check_integrity(ses.cache)
        torch.cuda.synchronize()
        gp = ses.pool_host_f32()
        n_diff = n_tot = 0
        for s in gs:
            for li in range(L):
                for t in range(ora.seq_len[s]):
                    p, sl = ora.page_table[s][t // 16], t % 16
                    assert np.array_equal(gp[li, p, :, 1, sl], ora.pool[li, p, :, 1, sl])          # V exact
                    a, b = gp[li, p, :, 0, sl], ora.pool[li, p, :, 0, sl]
                    assert_k_rows_close(a, b)
                    n_diff += int((a != b).sum())
                    n_tot += a.size
        assert n_diff <= 0.01 * n_tot, (n_diff, n_tot)


def test_commit_accepted_appends_only_accepted_verify_rows():
    M, S = _mods()
    rng = W.make_rng(411)
    L, Hq, Hkv, D, NP, B, nq = 2, 28, 4, 128, 24, 4, 7
    ses = S.Session(L, Hq, Hkv, D, NP, M.MS_BF16, 1000000.0, max_seqs=4, max_pages_per_seq=8)
    ora = O.PagedCache(L, Hkv, D, NP, dtype=O.BF16, rope_base=1000000.0, max_seqs=4)
    with ses:
        gs = [M.ms_seq_create(ses.cache) for _ in range(B)]
        for _ in range(B):
            ora.seq_create()
        start = [14, 15, 16, 30]
        n = sum(start)
        k, v = W.normal_bf16_bits(rng, (L, n, Hkv, D)), W.normal_bf16_bits(rng, (L, n, Hkv, D))
        pos = np.arange(n, dtype=np.int32)
        M.ms_append_kv(ses.cache, gs, start, S.to_device(k, M.MS_BF16), S.to_device(v, M.MS_BF16), S.ints_dev(pos))
        ora.append(gs, start, O.bf16_bits_to_f32(k), O.bf16_bits_to_f32(v), pos)
        kn, vn = W.normal_bf16_bits(rng, (L, B, nq, Hkv, D)), W.normal_bf16_bits(rng, (L, B, nq, Hkv, D))
        pq = (np.arange(nq)[None] + np.asarray([100, 200, 300, 400])[:, None]).astype(np.int32)
        acc = [4, 0, 1, 3]
        M.ms_commit_accepted(ses.cache, gs, acc, nq, S.to_device(kn, M.MS_BF16), S.to_device(vn, M.MS_BF16),
                             S.ints_dev(pq).view(B, nq))
        knf, vnf = O.bf16_bits_to_f32(kn), O.bf16_bits_to_f32(vn)
        for b in range(B):          # oracle: plain append of the accepted rows, sequence by sequence
            ora.append([gs[b]], [acc[b]], knf[:, b, :acc[b]], vnf[:, b, :acc[b]], pq[b, :acc[b]])
        torch.cuda.synchronize()
        gp = ses.pool_host_f32()
        for s in gs:
            assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s]
            assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s]
            for li in range(L):
                for t in range(ora.seq_len[s]):
                    p, sl = ora.page_table[s][t // 16], t % 16
                    assert np.array_equal(gp[li, p, :, 1, sl], ora.pool[li, p, :, 1, sl])
                    a, b_ = gp[li, p, :, 0, sl], ora.pool[li, p, :, 0, sl]
                    assert_k_rows_close(a, b_)
        M.ms_check_integrity(ses.cache)


def test_device_side_commit_keeps_pace_with_host_commit_and_oracle():
    """ms_commit_accepted_device over several steps with no host synchronisation in between: the
    attention that follows goes by the device's lengths (the host's lag behind), and once the host
    has caught up its page tables, lengths and free set are the oracle's, and the pool holds the same
    bits as a twin cache driven through the host-side ms_commit_accepted."""
    M, S = _mods()
    rng = W.make_rng(415)
    L, Hq, Hkv, D, NP, nv, nf = 2, 28, 4, 128, 80, 4, 3
    nq = nv + nf
    start = [14, 15, 16, 30, 0, 250, 31]
    B = len(start)
    order = [3, 0, 6, 1, 5, 2, 4]                 # argument order differs from id order
    bf = O.bf16_bits_to_f32
    dev = S.Session(L, Hq, Hkv, D, NP, M.MS_BF16, 1000000.0, max_seqs=8, max_pages_per_seq=24)
    host = S.Session(L, Hq, Hkv, D, NP, M.MS_BF16, 1000000.0, max_seqs=8, max_pages_per_seq=24)
    ora = O.PagedCache(L, Hkv, D, NP, dtype=O.BF16, rope_base=1000000.0, max_seqs=8)
    with dev, host:
        ids = [M.ms_seq_create(dev.cache) for _ in range(B)]
        assert ids == [M.ms_seq_create(host.cache) for _ in range(B)] == [ora.seq_create() for _ in range(B)]
        n = sum(start)
        k, v = W.normal_bf16_bits(rng, (L, n, Hkv, D)), W.normal_bf16_bits(rng, (L, n, Hkv, D))
        pos = np.concatenate([np.arange(1, c + 1) for c in start]).astype(np.int32)
        for ses in (dev, host):
            M.ms_append_kv(ses.cache, ids, start, S.to_device(k, M.MS_BF16), S.to_device(v, M.MS_BF16), S.ints_dev(pos))
        ora.append(ids, start, bf(k), bf(v), pos)
        sid = [ids[i] for i in order]
        first_pid = np.asarray([start[i] + 1 for i in order], np.int32)
        first_d = S.ints_dev(first_pid)
        pos_d = torch.empty(B, nq, dtype=torch.int32, device="cuda")
        accepts = [[4, 0, 1, 3, 2, 4, 1], [1, 1, 4, 4, 4, 2, 1], [0, 0, 0, 0, 0, 0, 0], [4, 4, 4, 4, 4, 4, 4], [2, 3, 4, 1, 0, 4, 4],
                   [4, 4, 4, 4, 4, 4, 4], [3, 4, 4, 2, 4, 4, 4]]
        for step, acc in enumerate(accepts):
            kn, vn = W.normal_bf16_bits(rng, (L, B, nq, Hkv, D)), W.normal_bf16_bits(rng, (L, B, nq, Hkv, D))
            M.ms_step_positions_device(first_d, nv, nf, pos_d)
            pq = M.ms_step_positions(first_pid, nv, nf)
            # attention first: it reads the cache as the commits so far left it, the host none the wiser
            q = W.normal_bf16_bits(rng, (B, nq, Hq, D))
            got = dev.attention(1, sid, nv, nf, S.to_device(q, M.MS_BF16), S.to_device(kn[1], M.MS_BF16), S.to_device(vn[1], M.MS_BF16), pos_d)
            want = O.attention(ora, 1, sid, nv, nf, bf(q), bf(kn[1]), bf(vn[1]), pq)
            check_out(S.to_host_f32(got), want, "bf16", f"step {step}")
            assert np.array_equal(pos_d.cpu().numpy(), pq)
            acc_d = S.ints_dev(acc)
            M.ms_commit_accepted_device(dev.cache, sid, acc_d, nq, nv, S.to_device(kn, M.MS_BF16), S.to_device(vn, M.MS_BF16), pos_d, first_d)
            M.ms_commit_accepted(host.cache, sid, acc, nq, S.to_device(kn, M.MS_BF16), S.to_device(vn, M.MS_BF16), S.ints_dev(pq).view(B, nq))
            for b in range(B):
                ora.append([sid[b]], [acc[b]], bf(kn)[:, b, :acc[b]], bf(vn)[:, b, :acc[b]], pq[b, :acc[b]])
            first_pid = first_pid + np.asarray(acc, np.int32)
            if step == 3:        # the host catches up in the middle (any call that needs its tables does)
                for s_ in ids:
                    assert M.ms_seq_len(dev.cache, s_) == ora.seq_len[s_]
        assert np.array_equal(first_d.cpu().numpy(), first_pid)
        M.ms_cache_sync(dev.cache)
        for s_ in ids:
            assert M.ms_seq_page_table(dev.cache, s_) == M.ms_seq_page_table(host.cache, s_) == ora.page_table[s_]
            assert M.ms_seq_len(dev.cache, s_) == ora.seq_len[s_]
        assert M.ms_free_page_count(dev.cache) == ora.free_page_count()
        assert M.ms_peak_pages(dev.cache) == M.ms_peak_pages(host.cache) == ora.peak_pages
        M.ms_check_integrity(dev.cache)
        torch.cuda.synchronize()
        assert torch.equal(dev.pool.view(torch.int16), host.pool.view(torch.int16))     # the same bits as the host-side commit
        # compaction after device-side commits, then device-side commits again
        seg = [5, 3]
        cids = [ids[5], ids[0]]
        begin = [M.ms_seq_len(dev.cache, s_) - n_ for s_, n_ in zip(cids, seg)]
        mk, mv = W.normal_bf16_bits(rng, (L, 2, Hkv, D)), W.normal_bf16_bits(rng, (L, 2, Hkv, D))
        M.ms_compact_segment(dev.cache, cids, begin, seg, [1, 1], S.to_device(mk, M.MS_BF16), S.to_device(mv, M.MS_BF16), S.ints_dev([400, 50]))
        ora.compact(cids, begin, seg, [1, 1], bf(mk), bf(mv), [400, 50])
        kn, vn = W.normal_bf16_bits(rng, (L, B, nq, Hkv, D)), W.normal_bf16_bits(rng, (L, B, nq, Hkv, D))
        acc = [4, 4, 1, 0, 4, 4, 2]
        M.ms_step_positions_device(first_d, nv, nf, pos_d)
        M.ms_commit_accepted_device(dev.cache, sid, S.ints_dev(acc), nq, nv, S.to_device(kn, M.MS_BF16), S.to_device(vn, M.MS_BF16), pos_d, first_d)
        pq = M.ms_step_positions(first_pid, nv, nf)
        for b in range(B):
            ora.append([sid[b]], [acc[b]], bf(kn)[:, b, :acc[b]], bf(vn)[:, b, :acc[b]], pq[b, :acc[b]])
        for s_ in ids:
            assert M.ms_seq_page_table(dev.cache, s_) == ora.page_table[s_]
        M.ms_check_integrity(dev.cache)


def test_wide_step_after_device_side_commits():
    """A pass of 41 causal queries (the memory-token pass) right after device-side commits: the wide kernel goes by
    the device's lengths and looks up the pages the commits added, while the host still holds the old tables."""
    M, S = _mods()
    rng = W.make_rng(418)
    L, Hq, Hkv, D, NP, nv, nf = 1, 28, 4, 128, 240, 4, 3
    nq = nv + nf
    start = [1000, 15, 2040, 0, 333]
    B = len(start)
    bf = O.bf16_bits_to_f32
    ses = S.Session(L, Hq, Hkv, D, NP, M.MS_BF16, 1000000.0, max_seqs=8, max_pages_per_seq=140)
    ora = O.PagedCache(L, Hkv, D, NP, dtype=O.BF16, rope_base=1000000.0, max_seqs=8)
    with ses:
        ids = [M.ms_seq_create(ses.cache) for _ in range(B)]
        assert ids == [ora.seq_create() for _ in range(B)]
        n = sum(start)
        k, v = W.normal_bf16_bits(rng, (L, n, Hkv, D)), W.normal_bf16_bits(rng, (L, n, Hkv, D))
        pos = np.concatenate([np.arange(1, c + 1) for c in start]).astype(np.int32)
        M.ms_append_kv(ses.cache, ids, start, S.to_device(k, M.MS_BF16), S.to_device(v, M.MS_BF16), S.ints_dev(pos))
        ora.append(ids, start, bf(k), bf(v), pos)
        first = np.asarray([c + 1 for c in start], np.int32)
        first_d = S.ints_dev(first)
        pos_d = torch.empty(B, nq, dtype=torch.int32, device="cuda")
        wide_q = 41
        for step, acc in enumerate([[4, 4, 4, 4, 4], [4, 1, 4, 0, 3], [4, 4, 4, 4, 4], [2, 4, 4, 4, 4]]):
            # a wide pass first: it sees what the commits so far have left (the plan is the one cut before them)
            qw = W.normal_bf16_bits(rng, (B, wide_q, Hq, D))
            kw, vw = W.normal_bf16_bits(rng, (B, wide_q, Hkv, D)), W.normal_bf16_bits(rng, (B, wide_q, Hkv, D))
            pw = np.stack([np.arange(f, f + wide_q) for f in first]).astype(np.int32)
            got = ses.attention(0, ids, wide_q, 0, S.to_device(qw, M.MS_BF16), S.to_device(kw, M.MS_BF16), S.to_device(vw, M.MS_BF16),
                                S.ints_dev(pw).view(B, wide_q))
            want = O.attention(ora, 0, ids, wide_q, 0, bf(qw), bf(kw), bf(vw), pw)
            check_out(S.to_host_f32(got), want, "bf16", f"wide pass before commit {step}")
            kn, vn = W.normal_bf16_bits(rng, (L, B, nq, Hkv, D)), W.normal_bf16_bits(rng, (L, B, nq, Hkv, D))
            M.ms_step_positions_device(first_d, nv, nf, pos_d)
            pq = M.ms_step_positions(first, nv, nf)
            M.ms_commit_accepted_device(ses.cache, ids, S.ints_dev(acc), nq, nv, S.to_device(kn, M.MS_BF16), S.to_device(vn, M.MS_BF16), pos_d, first_d)
            for b in range(B):
                ora.append([ids[b]], [acc[b]], bf(kn)[:, b, :acc[b]], bf(vn)[:, b, :acc[b]], pq[b, :acc[b]])
            first = first + np.asarray(acc, np.int32)
        M.ms_cache_sync(ses.cache)
        for s_ in ids:
            assert M.ms_seq_page_table(ses.cache, s_) == ora.page_table[s_] and M.ms_seq_len(ses.cache, s_) == ora.seq_len[s_]
        M.ms_check_integrity(ses.cache)


def test_device_side_commit_general_kernel_and_errors():
    M, S = _mods()
    rng = W.make_rng(416)
    L, Hq, Hkv, D, NP, nv, nf = 1, 4, 2, 64, 6, 3, 2
    nq = nv + nf
    ses = S.Session(L, Hq, Hkv, D, NP, M.MS_F32, 10000.0, max_seqs=3, max_pages_per_seq=3)
    ora = O.PagedCache(L, Hkv, D, NP, dtype=O.F32, rope_base=10000.0, max_seqs=3)
    with ses:
        ids = [M.ms_seq_create(ses.cache) for _ in range(2)]
        [ora.seq_create() for _ in range(2)]
        start = [15, 2]
        k, v = W.normal_f32(rng, (L, 17, Hkv, D)), W.normal_f32(rng, (L, 17, Hkv, D))
        pos = np.concatenate([np.arange(1, c + 1) for c in start]).astype(np.int32)
        M.ms_append_kv(ses.cache, ids, start, S.to_device(k, M.MS_F32), S.to_device(v, M.MS_F32), S.ints_dev(pos))
        ora.append(ids, start, k, v, pos)
        first_pid = np.asarray([16, 3], np.int32)
        first_d = S.ints_dev(first_pid)
        pos_d = torch.empty(2, nq, dtype=torch.int32, device="cuda")
        for acc in ([3, 1], [2, 3], [3, 3]):
            kn, vn = W.normal_f32(rng, (L, 2, nq, Hkv, D)), W.normal_f32(rng, (L, 2, nq, Hkv, D))
            q = W.normal_f32(rng, (2, nq, Hq, D))
            M.ms_step_positions_device(first_d, nv, nf, pos_d)
            pq = M.ms_step_positions(first_pid, nv, nf)
            got = ses.attention(0, ids, nv, nf, S.to_device(q, M.MS_F32), S.to_device(kn[0], M.MS_F32), S.to_device(vn[0], M.MS_F32), pos_d)
            check_out(S.to_host_f32(got), O.attention(ora, 0, ids, nv, nf, q, kn[0], vn[0], pq), "f32", "general kernel, lengths on the device")
            M.ms_commit_accepted_device(ses.cache, ids, S.ints_dev(acc), nq, nv, S.to_device(kn, M.MS_F32), S.to_device(vn, M.MS_F32), pos_d, first_d)
            for b in range(2):
                ora.append([ids[b]], [acc[b]], kn[:, b, :acc[b]], vn[:, b, :acc[b]], pq[b, :acc[b]])
            first_pid = first_pid + np.asarray(acc, np.int32)
        for s_ in ids:
            assert M.ms_seq_page_table(ses.cache, s_) == ora.page_table[s_] and M.ms_seq_len(ses.cache, s_) == ora.seq_len[s_]
        torch.cuda.synchronize()
        gp = ses.pool_host_f32()
        for s_ in ids:
            for t in range(ora.seq_len[s_]):
                p_, sl = ora.page_table[s_][t // 16], t % 16
                assert np.abs(gp[0, p_, :, :, sl] - ora.pool[0, p_, :, :, sl]).max() < 3e-6
        # 23 and 9 rows in 2 + 1 of 6 pages; a third sequence and four more steps use up the worst-case room
        kn, vn = S.to_device(W.normal_f32(rng, (L, 2, nq, Hkv, D)), M.MS_F32), S.to_device(W.normal_f32(rng, (L, 2, nq, Hkv, D)), M.MS_F32)
        with pytest.raises(M.MsError) as e:
            M.ms_commit_accepted_device(ses.cache, [ids[0], ids[0]], S.ints_dev([1, 1]), nq, nv, kn, vn, pos_d)
        assert e.value.code == M.MS_ERR_INVALID                                        # listed twice
        with pytest.raises(M.MsError) as e:
            M.ms_commit_accepted_device(ses.cache, ids, S.ints_dev([1, 1]), nq, nq + 1, kn, vn, pos_d)
        assert e.value.code == M.MS_ERR_INVALID                                        # n_max above n_q
        third = M.ms_seq_create(ses.cache)
        ora.seq_create()
        k3 = S.to_device(W.normal_f32(rng, (L, 40, Hkv, D)), M.MS_F32)
        M.ms_append_kv(ses.cache, [third], [40], k3, k3, S.ints_dev(np.arange(40)))    # 3 pages: the pool is full
        with pytest.raises(M.MsError) as e:
            M.ms_commit_accepted_device(ses.cache, ids, S.ints_dev([0, 0]), nq, nv, kn, vn, pos_d)
        assert e.value.code == M.MS_ERR_OOM_PAGES                                      # no room for the worst case
        assert M.ms_seq_len(ses.cache, ids[0]) == 23 and M.ms_free_page_count(ses.cache) == 0
        M.ms_check_integrity(ses.cache)


# ------------------------------------------------------------------ compaction ---------------

def test_config4_page_tables_batch16_28_layers():
    """Batch 16, 28 layers: each sequence closes a 256-token segment (16 whole pages released) and
    keeps 8 memory tokens in fresh pages.  Page tables, lengths and free counts must equal the
    oracle's; memory-token rows are checked in sampled layers."""
    M, S = _mods()
    rng = W.make_rng(4)
    B, L, Hq, Hkv, D = 16, 28, 28, 4, 128
    lens = [int(16 * x) for x in rng.integers(2304 // 16, 8448 // 16 + 1, size=B)]
    shape = W.AttnShape("c4", "bf16", B, Hq, Hkv, D, 4, 3, lens, 0.5, 1000000.0, n_layers=L, slack_pages=0.02)
    pts = W.shuffled_page_tables(rng, shape.n_pages, lens)
    ses = S.Session(L, Hq, Hkv, D, shape.n_pages, M.MS_BF16, 1000000.0, max_seqs=B, max_pages_per_seq=600)
    ora = O.PagedCache(1, 1, 8, shape.n_pages, dtype=O.BF16, max_seqs=B)     # tables only
    with ses:
        gs = [M.ms_seq_import(ses.cache, n, pt) for n, pt in zip(lens, pts)]
        os_ = [ora.seq_import(n, pt) for n, pt in zip(lens, pts)]
        assert gs == os_
        c = 32
        n_mem = [M.ms_ama_count(256, c)] * B
        assert n_mem[0] == 8
        begin = [n - 256 for n in lens]
        first_pid = [3 * n for n in lens]
        mpos = sum((M.ms_upl_positions(fp, 256, c) for fp in first_pid), [])
        assert mpos == sum((O.upl_positions(fp, 256, c) for fp in first_pid), [])
        mk = W.normal_bf16_bits(rng, (L, 8 * B, Hkv, D))
        mv = W.normal_bf16_bits(rng, (L, 8 * B, Hkv, D))
        free_before = M.ms_free_page_count(ses.cache)
        M.ms_compact_segment(ses.cache, gs, begin, [256] * B, n_mem, S.to_device(mk, M.MS_BF16),
                             S.to_device(mv, M.MS_BF16), S.ints_dev(mpos))
        ora.compact(os_, begin, [256] * B, n_mem, np.zeros((1, 8 * B, 1, 8)), np.zeros((1, 8 * B, 1, 8)), mpos)
        assert M.ms_free_page_count(ses.cache) == ora.free_page_count() == free_before + 15 * B
        for s in gs:
            assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s]
            assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s]
        M.ms_check_integrity(ses.cache)
        torch.cuda.synchronize()
        inv = O.rope_inv_freq(D, 1000000.0)
        for li in (0, 13, 27):
            want_k = O.round_bf16(O.rope(O.bf16_bits_to_f32(mk[li]), np.asarray(mpos)[:, None], inv).astype(np.float32))
            for b in (0, 7, 15):
                s = gs[b]
                for j in range(8):
                    t = begin[b] + j
                    p, sl = ora.page_table[s][t // 16], t % 16
                    row = S.to_host_f32(ses.pool[li, p, :, :, sl])          # [Hkv, 2, D]
                    assert np.array_equal(row[:, 1], O.bf16_bits_to_f32(mv[li, 8 * b + j]))
                    wk = want_k[8 * b + j]
                    assert_k_rows_close(row[:, 0], wk)


def test_compaction_content_attention_and_recompute_equivalence():
    """Reduced config 4 (2 layers, batch 4) with real data: after compaction the cache rows and the
    attention over them match the oracle, and match a GPU cache rebuilt from the kept rows only."""
    M, S = _mods()
    rng = W.make_rng(41)
    B, L, Hq, Hkv, D = 4, 2, 28, 4, 128
    lens = [1024 + 256, 2048 + 256, 640 + 256, 1296 + 256]
    sh = W.AttnShape("c4small", "bf16", B, Hq, Hkv, D, 4, 3, lens, 0.5, 1000000.0, n_layers=L)
    inp = W.attention_inputs(sh, 41)
    ses, ora, ids = setup_pair(inp)
    with ses:
        M.ms_attention_set_deterministic(ses.cache, True)   # for the bitwise comparison at the end
        n_mem = [8] * B
        begin = [n - 256 for n in lens]
        mpos = sum((M.ms_upl_positions(3 * n, 256, 32) for n in lens), [])
        mk = W.normal_bf16_bits(rng, (L, 8 * B, Hkv, D))
        mv = W.normal_bf16_bits(rng, (L, 8 * B, Hkv, D))
        M.ms_compact_segment(ses.cache, ids, begin, [256] * B, n_mem, S.to_device(mk, M.MS_BF16),
                             S.to_device(mv, M.MS_BF16), S.ints_dev(mpos))
        ora.compact(ids, begin, [256] * B, n_mem, O.bf16_bits_to_f32(mk), O.bf16_bits_to_f32(mv), mpos)
        for s in ids:
            assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s]
            assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s] == lens[s] - 256 + 8
        M.ms_check_integrity(ses.cache)
        sh2 = W.AttnShape("c4small", "bf16", B, Hq, Hkv, D, 4, 3, [n - 248 for n in lens], 0.5, 1000000.0, n_layers=L)
        inp2 = W.AttnInputs(sh2, inp.page_tables, inp.pool, inp.q, inp.k_new, inp.v_new,
                            [3 * n + 1 for n in lens])
        pos = pids_for(inp2, M)
        outs = []
        for layer in range(L):
            got = run_gpu_attention(ses, inp2, ids, pos, layer)
            want = oracle_attention(ora, inp2, ids, pos, layer)
            check_out(got, want, "bf16", f"after compaction, layer {layer}")
            outs.append(got)
        # rebuild on the GPU from the kept rows only (download, re-append pre-rotated)
        torch.cuda.synchronize()
        gp = ses.pool.view(torch.int16).cpu().numpy().view(np.uint16)
        tables = ses.page_tables(ids)
        new_lens = ses.lengths(ids)
    ses2 = S.Session(L, Hq, Hkv, D, sh.n_pages, M.MS_BF16, 1000000.0, max_seqs=B, max_pages_per_seq=200)
    with ses2:
        M.ms_attention_set_deterministic(ses2.cache, True)
        ids2 = [M.ms_seq_create(ses2.cache) for _ in range(B)]
        for b in range(B):
            pt = np.asarray(tables[b])
            rows = gp[:, pt].transpose(0, 1, 4, 2, 3, 5).reshape(L, -1, Hkv, 2, D)[:, :new_lens[b]]
            k = np.ascontiguousarray(rows[:, :, :, 0])
            v = np.ascontiguousarray(rows[:, :, :, 1])
            M.ms_append_kv(ses2.cache, [ids2[b]], [new_lens[b]], S.to_device(k, M.MS_BF16), S.to_device(v, M.MS_BF16),
                           None, flags=M.MS_PRE_ROTATED)
        for layer in range(L):
            again = run_gpu_attention(ses2, inp2, ids2, pos, layer)
            assert np.array_equal(again, outs[layer]), "compaction must equal recomputation over the kept KV"
        M.ms_attention_set_deterministic(ses2.cache, False)
        for layer in range(L):
            check_out(run_gpu_attention(ses2, inp2, ids2, pos, layer), outs[layer], "bf16", "default mode, recomputation")


def test_compaction_in_the_middle_moves_the_tail():
    M, S = _mods()
    rng = W.make_rng(412)
    L, Hkv, D, NP = 2, 2, 64, 16
    ses = S.Session(L, 4, Hkv, D, NP, M.MS_F32, 10000.0, max_seqs=2, max_pages_per_seq=8)
    ora = O.PagedCache(L, Hkv, D, NP, dtype=O.F32, rope_base=10000.0, max_seqs=2)
    with ses:
        gs = [M.ms_seq_create(ses.cache), M.ms_seq_create(ses.cache)]
        ora.seq_create(), ora.seq_create()
        counts = [50, 37]
        k, v = W.normal_f32(rng, (L, 87, Hkv, D)), W.normal_f32(rng, (L, 87, Hkv, D))
        pos = np.arange(87, dtype=np.int32)
        M.ms_append_kv(ses.cache, gs, counts, S.to_device(k, M.MS_F32), S.to_device(v, M.MS_F32), S.ints_dev(pos))
        ora.append(gs, counts, k, v, pos)
        mk, mv = W.normal_f32(rng, (L, 5, Hkv, D)), W.normal_f32(rng, (L, 5, Hkv, D))
        mpos = [12, 17, 22, 3, 9]
        args = (gs, [10, 2], [25, 20], [3, 2])
        need = M.ms_compact_workspace_bytes(ses.cache, *args[:3])
        assert need == (15 + 15) * 2 * L * Hkv * D * 4
        with pytest.raises(M.MsError) as e:
            M.ms_compact_segment(ses.cache, *args, S.to_device(mk, M.MS_F32), S.to_device(mv, M.MS_F32), S.ints_dev(mpos))
        assert e.value.code == M.MS_ERR_WORKSPACE
        assert M.ms_seq_len(ses.cache, gs[0]) == 50                      # unchanged by the failed call
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        M.ms_compact_segment(ses.cache, *args, S.to_device(mk, M.MS_F32), S.to_device(mv, M.MS_F32), S.ints_dev(mpos),
                             workspace=ws)
        ora.compact(*args, mk, mv, mpos)
        torch.cuda.synchronize()
        gp = ses.pool_host_f32()
        for s in gs:
            assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s]
            assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s]
            for li in range(L):
                for t in range(ora.seq_len[s]):
                    p, sl = ora.page_table[s][t // 16], t % 16
                    assert np.abs(gp[li, p, :, :, sl] - ora.pool[li, p, :, :, sl]).max() < 3e-6
        M.ms_check_integrity(ses.cache)


def test_random_cache_operation_sequence_stays_in_step_with_the_oracle():
    """300 seeded random cache operations -- create, free, append (batched), compaction of a random
    segment (suffix or middle, batched), failing calls (pool exhausted, segment out of range) --
    applied to both sides; page tables, lengths and free counts must agree after every one, the
    stored rows at the end."""
    M, S = _mods()
    rng = W.make_rng(414)
    L, Hkv, D, NP, MAXS = 2, 2, 64, 40, 6
    ses = S.Session(L, 4, Hkv, D, NP, M.MS_F32, 10000.0, max_seqs=MAXS, max_pages_per_seq=NP)
    ora = O.PagedCache(L, Hkv, D, NP, dtype=O.F32, rope_base=10000.0, max_seqs=MAXS)
    live, next_pos = [], {}
    n_ops = {"create": 0, "free": 0, "append": 0, "compact": 0, "oom": 0, "range": 0}
    with ses:
        for op_i in range(300):
            r = rng.random()
            if (r < 0.12 and len(live) < MAXS) or not live:
                s = M.ms_seq_create(ses.cache)
                assert s == ora.seq_create()
                live.append(s)
                next_pos[s] = 1
                n_ops["create"] += 1
            elif r < 0.2:
                s = live.pop(int(rng.integers(len(live))))
                M.ms_seq_free(ses.cache, s)
                ora.seq_free(s)
                n_ops["free"] += 1
            elif r < 0.65:
                k_seqs = int(rng.integers(1, len(live) + 1))
                seqs = [int(x) for x in rng.choice(live, size=k_seqs, replace=False)]
                counts = [int(rng.integers(0, 41)) for _ in seqs]
                tot = sum(counts)
                k, v = W.normal_f32(rng, (L, max(tot, 1), Hkv, D)), W.normal_f32(rng, (L, max(tot, 1), Hkv, D))
                pos = np.concatenate([np.arange(next_pos[s], next_pos[s] + c) for s, c in zip(seqs, counts)] + [np.zeros(0)]).astype(np.int32)
                pos_d = S.ints_dev(pos if tot else [0])
                try:
                    ora.append(seqs, counts, k[:, :tot], v[:, :tot], pos)
                except O.OutOfPages:
                    with pytest.raises(M.MsError) as e:
                        M.ms_append_kv(ses.cache, seqs, counts, S.to_device(k, M.MS_F32), S.to_device(v, M.MS_F32), pos_d)
                    assert e.value.code == M.MS_ERR_OOM_PAGES
                    n_ops["oom"] += 1
                else:
                    M.ms_append_kv(ses.cache, seqs, counts, S.to_device(k, M.MS_F32), S.to_device(v, M.MS_F32), pos_d)
                    for s, c in zip(seqs, counts):
                        next_pos[s] += c
                    n_ops["append"] += 1
            else:
                cands = [s for s in live if ora.seq_len[s] >= 4]
                if not cands:
                    continue
                k_seqs = int(rng.integers(1, min(3, len(cands)) + 1))
                seqs = [int(x) for x in rng.choice(cands, size=k_seqs, replace=False)]
                begin, seg, n_mem = [], [], []
                for s in seqs:
                    n = ora.seq_len[s]
                    b0 = int(rng.integers(0, n - 1))
                    ln = n - b0 if rng.random() < 0.5 else int(rng.integers(1, n - b0 + 1))    # suffix or middle
                    begin.append(b0)
                    seg.append(ln)
                    n_mem.append(int(rng.integers(0, max(1, ln // 3) + 1)))
                bad = rng.random() < 0.1
                if bad:
                    seg[0] = ora.seq_len[seqs[0]] - begin[0] + 1                               # one past the end
                tot = sum(n_mem)
                mk, mv = W.normal_f32(rng, (L, max(tot, 1), Hkv, D)), W.normal_f32(rng, (L, max(tot, 1), Hkv, D))
                mpos = rng.integers(1, 500, size=max(tot, 1)).astype(np.int32)
                args = (seqs, begin, seg, n_mem)
                if bad:
                    big = torch.empty(1 << 22, dtype=torch.uint8, device="cuda")
                    with pytest.raises(M.MsError) as e:
                        M.ms_compact_segment(ses.cache, *args, S.to_device(mk, M.MS_F32), S.to_device(mv, M.MS_F32), S.ints_dev(mpos),
                                             workspace=big)
                    assert e.value.code == M.MS_ERR_RANGE
                    n_ops["range"] += 1
                else:
                    need = M.ms_compact_workspace_bytes(ses.cache, *args[:3])
                    ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
                    M.ms_compact_segment(ses.cache, *args, S.to_device(mk, M.MS_F32), S.to_device(mv, M.MS_F32), S.ints_dev(mpos),
                                         workspace=ws)
                    ora.compact(*args, mk[:, :tot], mv[:, :tot], mpos[:tot])
                    n_ops["compact"] += 1
            for s in live:
                assert M.ms_seq_page_table(ses.cache, s) == ora.page_table[s], f"op {op_i}"
                assert M.ms_seq_len(ses.cache, s) == ora.seq_len[s]
            assert M.ms_free_page_count(ses.cache) == ora.free_page_count()
        M.ms_check_integrity(ses.cache)
        assert M.ms_peak_pages(ses.cache) == ora.peak_pages
        assert min(n_ops["append"], n_ops["compact"]) > 40 and n_ops["free"] > 5, n_ops
        torch.cuda.synchronize()
        gp = ses.pool_host_f32()
        for s in live:
            for li in range(L):
                for t in range(ora.seq_len[s]):
                    p, sl = ora.page_table[s][t // 16], t % 16
                    assert np.abs(gp[li, p, :, :, sl] - ora.pool[li, p, :, :, sl]).max() < 3e-6
        print("operations:", n_ops)


# ------------------------------------------------------------------ acceptance ---------------

def test_accept_matches_oracle_including_stop_ids():
    M, S = _mods()
    rng = W.make_rng(413)
    for n in (1, 4, 5, 9):
        B = 200
        forced = [int(x) for x in rng.integers(0, n + 1, size=B)]
        draft, target = W.draft_and_target(rng, B, n, 50, forced)
        for stops in (None, [7, 11, 13]):
            acc = torch.full((B,), -9, dtype=torch.int32, device="cuda")
            nxt = torch.full((B,), -9, dtype=torch.int32, device="cuda")
            M.ms_accept(B, n, S.ints_dev(draft), S.ints_dev(target), None if stops is None else S.ints_dev(stops), acc, nxt)
            wa, wn = O.accept(draft, target, stops or ())
            assert np.array_equal(acc.cpu().numpy(), wa)
            assert np.array_equal(nxt.cpu().numpy(), wn)
            if stops is None:
                assert wa.tolist() == forced
            a = acc.cpu().numpy()
            for b in range(B):      # accepted tokens form a prefix of the drafts
                assert np.array_equal(draft[b, :a[b]], target[b, :a[b]])


# ------------------------------------------------------------------ error paths --------------

def test_errors_are_reported_and_leave_state_unchanged():
    M, S = _mods()
    ses = S.Session(1, 4, 2, 64, 3, M.MS_F32, 10000.0, max_seqs=2, max_pages_per_seq=2)
    with ses:
        s = M.ms_seq_create(ses.cache)
        k = torch.zeros(1, 40, 2, 64, device="cuda")
        pos = torch.zeros(40, dtype=torch.int32, device="cuda")
        M.ms_append_kv(ses.cache, [s], [20], k, k, pos)
        with pytest.raises(M.MsError) as e:
            M.ms_append_kv(ses.cache, [s], [20], k, k, pos)              # 40 rows -> 3 pages > max_pages_per_seq
        assert e.value.code == M.MS_ERR_OOM_PAGES
        s2 = M.ms_seq_create(ses.cache)
        with pytest.raises(M.MsError) as e:
            M.ms_append_kv(ses.cache, [s2, s], [17, 12], k, k, pos)      # needs 2 pages, 1 free
        assert e.value.code == M.MS_ERR_OOM_PAGES
        assert M.ms_seq_len(ses.cache, s) == 20 and M.ms_seq_len(ses.cache, s2) == 0
        assert M.ms_free_page_count(ses.cache) == 1
        with pytest.raises(M.MsError) as e:
            M.ms_append_kv(ses.cache, [5], [1], k, k, pos)
        assert e.value.code == M.MS_ERR_INVALID
        with pytest.raises(M.MsError) as e:
            M.ms_compact_segment(ses.cache, [s], [10], [11], [1], k, k, pos)
        assert e.value.code == M.MS_ERR_RANGE
        with pytest.raises(M.MsError) as e:
            M.ms_seq_import(ses.cache, 16, [0])                           # page 0 is owned
        assert e.value.code == M.MS_ERR_INVALID
        q = torch.zeros(1, 3, 4, 64, device="cuda")
        kn = torch.zeros(1, 3, 2, 64, device="cuda")
        pq = torch.zeros(1, 3, dtype=torch.int32, device="cuda")
        with pytest.raises(M.MsError) as e:
            M.ms_predict_verify_attention(ses.cache, 0, [s], 2, 1, q, kn, kn, pq, None, 0.0, q.clone(),
                                          torch.empty(256, dtype=torch.uint8, device="cuda"))
        assert e.value.code == M.MS_ERR_WORKSPACE
        with pytest.raises(M.MsError) as e:
            M.ms_predict_verify_attention(ses.cache, 1, [s], 2, 1, q, kn, kn, pq, None, 0.0, q.clone(), None)
        assert e.value.code == M.MS_ERR_INVALID
        with pytest.raises(M.MsError) as e:
            ses.attention(0, [s], 12, 5, q, kn, kn, pq)
        assert e.value.code == M.MS_ERR_INVALID
        M.ms_check_integrity(ses.cache)
        M.ms_seq_free(ses.cache, s)
        with pytest.raises(M.MsError):
            M.ms_seq_len(ses.cache, s)
        assert M.ms_free_page_count(ses.cache) == 3


# ------------------------------------------------------------------ Algorithm 1 as a state machine ---

def test_algorithm1_loop_keeps_gpu_and_oracle_in_step():
    """Drives both sides through the paper's inference loop (Appendix A, Algorithm 1) with random
    stand-ins for the model: speculative steps (attention, acceptance, commit of the accepted rows),
    and, whenever a sequence's step closes, the memory-token pass (l + 1 causal queries, no foresight)
    followed by compaction of that sequence only.  After every call the page tables, lengths and
    attention outputs must agree; this also exercises the cached work plan across cache changes."""
    M, S = _mods()
    rng = W.make_rng(500)
    B, L, Hq, Hkv, D, NP = 3, 2, 28, 4, 128, 96
    nv, nf, c_ratio = 4, 3, 5
    nq = nv + nf
    ses = S.Session(L, Hq, Hkv, D, NP, M.MS_BF16, 1000000.0, max_seqs=B, max_pages_per_seq=40)
    ora = O.PagedCache(L, Hkv, D, NP, dtype=O.BF16, rope_base=1000000.0, max_seqs=B)
    bf = O.bf16_bits_to_f32
    with ses:
        ids = [M.ms_seq_create(ses.cache) for _ in range(B)]
        assert ids == [ora.seq_create() for _ in range(B)]
        # "prefill": prompts of different lengths
        prompt = [37, 5, 64]
        n = sum(prompt)
        k, v = W.normal_bf16_bits(rng, (L, n, Hkv, D)), W.normal_bf16_bits(rng, (L, n, Hkv, D))
        pos = np.concatenate([np.arange(1, p + 1) for p in prompt]).astype(np.int32)
        M.ms_append_kv(ses.cache, ids, prompt, S.to_device(k, M.MS_BF16), S.to_device(v, M.MS_BF16), S.ints_dev(pos))
        ora.append(ids, prompt, bf(k), bf(v), pos)
        next_pid = [p + 1 for p in prompt]
        seg_start_len = list(prompt)            # cache length at which the open step began
        seg_first_pid = list(next_pid)
        close_at = [11, 23, 17]                 # a step closes once it holds this many tokens
        n_compactions = 0
        closed = [0] * B                        # steps closed so far: each took one position id for <o>
        for step in range(30):
            q = W.normal_bf16_bits(rng, (B, nq, Hq, D))
            kn = W.normal_bf16_bits(rng, (L, B, nq, Hkv, D))
            vn = W.normal_bf16_bits(rng, (L, B, nq, Hkv, D))
            pq = np.asarray([list(range(p, p + nv)) + M.ms_foresight_pids(p + nv - 1, nf) for p in next_pid], np.int32)
            for layer in range(L):
                out = ses.attention(layer, ids, nv, nf, S.to_device(q, M.MS_BF16), S.to_device(kn[layer], M.MS_BF16),
                                    S.to_device(vn[layer], M.MS_BF16), S.ints_dev(pq).view(B, nq))
                want = O.attention(ora, layer, ids, nv, nf, bf(q), bf(kn[layer]), bf(vn[layer]), pq)
                check_out(S.to_host_f32(out), want, "bf16", f"step {step} layer {layer}")
            forced = [int(x) for x in rng.integers(0, nv + 1, size=B)]
            draft, target = W.draft_and_target(rng, B, nv, 1000, forced)
            acc_d = torch.empty(B, dtype=torch.int32, device="cuda")
            nxt_d = torch.empty(B, dtype=torch.int32, device="cuda")
            M.ms_accept(B, nv, S.ints_dev(draft), S.ints_dev(target), None, acc_d, nxt_d)
            acc = acc_d.cpu().numpy()
            wa, _ = O.accept(draft, target)
            assert np.array_equal(acc, wa)
            acc = [max(1, int(a)) for a in acc]          # the first draft is the previous bonus token
            M.ms_commit_accepted(ses.cache, ids, acc, nq, S.to_device(kn, M.MS_BF16), S.to_device(vn, M.MS_BF16),
                                 S.ints_dev(pq).view(B, nq))
            for b in range(B):
                ora.append([ids[b]], [acc[b]], bf(kn)[:, b, :acc[b]], bf(vn)[:, b, :acc[b]], pq[b, :acc[b]])
                next_pid[b] += acc[b]
            # close finished steps: memory-token pass, then compaction, for those sequences only
            closing = [b for b in range(B) if M.ms_seq_len(ses.cache, ids[b]) - seg_start_len[b] >= close_at[b]]
            if closing:
                seg_len = [M.ms_seq_len(ses.cache, ids[b]) - seg_start_len[b] for b in closing]
                n_mem = [M.ms_ama_count(s_, c_ratio) for s_ in seg_len]
                assert n_mem == [O.ama_count(s_, c_ratio) for s_ in seg_len]
                cids = [ids[b] for b in closing]
                # memory tokens take UPL position ids, <o> the position after the step
                mpos = [M.ms_upl_positions(seg_first_pid[b], s_, c_ratio) for b, s_ in zip(closing, seg_len)]
                assert mpos == [O.upl_positions(seg_first_pid[b], s_, c_ratio) for b, s_ in zip(closing, seg_len)]
                for bi, b in enumerate(closing):        # memory-token forward: l + 1 causal queries, one sequence
                    lq = n_mem[bi] + 1
                    if lq > 16:
                        continue
                    qm = W.normal_bf16_bits(rng, (1, lq, Hq, D))
                    km = W.normal_bf16_bits(rng, (1, lq, Hkv, D))
                    vm = W.normal_bf16_bits(rng, (1, lq, Hkv, D))
                    pm = np.asarray([mpos[bi] + [M.ms_output_token_pid(next_pid[b] - 1)]], np.int32)
                    out = ses.attention(1, [ids[b]], lq, 0, S.to_device(qm, M.MS_BF16), S.to_device(km, M.MS_BF16),
                                        S.to_device(vm, M.MS_BF16), S.ints_dev(pm).view(1, lq))
                    want = O.attention(ora, 1, [ids[b]], lq, 0, bf(qm), bf(km), bf(vm), pm)
                    check_out(S.to_host_f32(out), want, "bf16", f"memory-token pass, step {step}, seq {b}")
                tot = sum(n_mem)
                mk, mv = W.normal_bf16_bits(rng, (L, tot, Hkv, D)), W.normal_bf16_bits(rng, (L, tot, Hkv, D))
                flat = sum(mpos, [])
                begin = [seg_start_len[b] for b in closing]
                M.ms_compact_segment(ses.cache, cids, begin, seg_len, n_mem, S.to_device(mk, M.MS_BF16),
                                     S.to_device(mv, M.MS_BF16), S.ints_dev(flat))
                ora.compact(cids, begin, seg_len, n_mem, bf(mk), bf(mv), flat)
                n_compactions += len(closing)
                for b in closing:
                    closed[b] += 1
                    next_pid[b] = M.ms_output_token_pid(next_pid[b] - 1) + 1
                    seg_start_len[b] = M.ms_seq_len(ses.cache, ids[b])
                    seg_first_pid[b] = next_pid[b]
            for b in range(B):
                assert M.ms_seq_page_table(ses.cache, ids[b]) == ora.page_table[ids[b]]
                assert M.ms_seq_len(ses.cache, ids[b]) == ora.seq_len[ids[b]]
            assert M.ms_free_page_count(ses.cache) == ora.free_page_count()
            M.ms_check_integrity(ses.cache)
        assert n_compactions >= 6
        assert M.ms_peak_pages(ses.cache) == ora.peak_pages
        # what compression buys (Appendix C.1 reports it as peak context tokens): without it every
        # committed token would still be cached
        raw_tokens = [p - 1 - n_o for p, n_o in zip(next_pid, closed)]
        pages_without = sum(-(-t // 16) for t in raw_tokens)
        assert ora.peak_pages < pages_without
        kept = sum(M.ms_seq_len(ses.cache, s) for s in ids)
        assert kept - sum(prompt) < (sum(raw_tokens) - sum(prompt)) / 2     # prompts are never compressed


# ------------------------------------------------------------------ failure path of the split-KV combine ---

def test_closing_timeout_is_reported_and_the_cache_recovers():
    """The condition is forced from the host (every pair's "published" counter starts at -3 and the
    closing workgroups' bounded wait is cut to 200 polls): the launch must end normally, leave the
    output rows unwritten, and be reported by the next call -- which resets the counters so that the
    call after it is right again."""
    M, S = _mods()
    sh = W.AttnShape("fault", "bf16", 3, 28, 4, 128, 5, 4, [3000, 40, 9000], 0.5, 1000000.0)
    inp = W.attention_inputs(sh, 470)
    ses, ora, ids = setup_pair(inp)
    with ses:
        pos = pids_for(inp, M)
        want = oracle_attention(ora, inp, ids, pos)
        check_out(run_gpu_attention(ses, inp, ids, pos), want, "bf16", "before")
        q, kn, vn = (S.to_device(x, M.MS_BF16) for x in (inp.q, inp.k_new, inp.v_new))
        p = S.ints_dev(pos).view(sh.batch, sh.n_q)
        M.ms_attention_fault_injection(ses.cache, 200, -3)
        marker = torch.full_like(q, 7.0)
        ses.attention(0, ids, 5, 4, q, kn, vn, p, out=marker)          # runs to the end, writes nothing
        torch.cuda.synchronize()
        assert (marker.float() == 7.0).all()
        with pytest.raises(M.MsError) as e:
            M.ms_check_integrity(ses.cache)
        assert e.value.code == M.MS_ERR_HIP
        with pytest.raises(M.MsError) as e:
            ses.attention(0, ids, 5, 4, q, kn, vn, p)                   # reports, resets the counters
        assert e.value.code == M.MS_ERR_HIP and "timed out" in str(e.value)
        M.ms_attention_fault_injection(ses.cache, 0, 0)                 # default bound again
        check_out(run_gpu_attention(ses, inp, ids, pos), want, "bf16", "after the reset")
        M.ms_check_integrity(ses.cache)
