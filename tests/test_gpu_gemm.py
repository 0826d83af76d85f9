"""The bf16 projection GEMM against the definition C = A W^T + bias evaluated in fp64 (numpy) on
the same bf16-valued operands.  The kernel accumulates in fp32 and rounds once to bf16, so an
element may differ by one bf16 rounding (2^-8 relative with a safety factor) plus an fp32
accumulation error far below that."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import memosight_oracle as O

pytestmark = pytest.mark.gpu

CASES = [
    # M, N, K, output widths, split_k, bias
    (1, 128, 32, [128], 1, False),
    (7, 256, 64, [128, 128], 1, True),
    (257, 256, 128, [256], 2, True),              # second row tile holds a single row
    (448, 512, 3584, [512], 1, True),             # K / V projection of a 64 x 7 token step
    (448, 4608, 3584, [3584, 512, 512], 1, True),  # fused Q / K / V projection into three tensors
    (448, 3584, 18944, [3584], 4, False),         # MLP down projection, K split four ways
    (300, 1024, 2048, [128, 512, 256, 128], 8, True),
    (448, 37888, 512, [37888], 1, True),          # gate/up width: 296 tiles on 256 compute units, the last round split over K
    (100, 67584, 512, [67584], 1, False),         # one row tile: 264 tiles, the last 8 split over K
    (1024, 640, 256, [640], 1, True),             # four row tiles, a last column tile that is half past N
    (700, 384, 512, [256, 128], 2, False),        # a ragged third row tile (188 rows: 4 and 2 row blocks of its waves), K in two parts
    # at most 16 rows and K a multiple of 128: the few-row kernel that streams the weight once (split_k is not used there)
    (1, 128, 512, [128], 1, False),
    (7, 4608, 3584, [3584, 512, 512], 1, True),   # a single sequence's fused Q / K / V projection
    (5, 256, 1024, [128, 128], 1, True),
    (8, 3584, 18944, [3584], 1, False),           # down projection: K in parts, fp32 partials
    (3, 3584, 18944, [3584], 1, True),            # fewer rows: fewer, longer K parts
    (4, 37888, 512, [37888], 1, True),            # gate/up width
    (7, 16384, 1536, [16384], 1, False),          # 12 K steps against 4 in flight
    # the same kernel's launch shapes: waves that split K, several tiles per wave, K in parts
    (16, 256, 128, [128, 128], 1, True),          # a single K step
    (9, 4608, 3584, [3584, 512, 512], 1, True),   # four waves split K over the same weight rows
    (7, 3584, 3584, [3584], 1, False),            # output projection of a single sequence
    (14, 3584, 18944, [3584], 1, False),          # two sequences' down projection: K in parts, fp32 partials
    (16, 37888, 384, [37888], 1, True),           # gate/up width, 3 steps against 4 in flight
    (2, 152064, 256, [152064], 1, False),         # LM-head width: two 16-row tiles per wave, 2 steps
    (12, 1024, 640, [512, 512], 1, False),        # 5 steps over 4 waves (1, 1, 1, 2)
    (11, 128, 2176, [128], 1, True),              # 17 steps over 4 waves
    (14, 37888, 3584, [37888], 1, True),          # two sequences' gate/up width: all of A (100 KB) in one compute unit's LDS
]


@pytest.mark.parametrize("m,n,k,widths,split,with_bias", CASES)
def test_gemm_matches_fp64_definition(m, n, k, widths, split, with_bias):
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    rng = W.make_rng(900, m, n, k)
    a = W.normal_bf16_bits(rng, (m, k), 1.0)
    w = W.normal_bf16_bits(rng, (n, k), k ** -0.5)
    b = W.normal_bf16_bits(rng, (n,), 0.5) if with_bias else None
    f64 = lambda x: O.bf16_bits_to_f32(x).astype(np.float64)
    ref = f64(a) @ f64(w).T + (f64(b) if with_bias else 0.0)
    outs = [torch.full((m, wd), float("nan"), dtype=torch.bfloat16, device="cuda") for wd in widths]
    ws = None
    need = M.ms_gemm_workspace_bytes(m, n, k, split)
    if split > 1:
        assert need == split * m * n * 4
    elif n >= 37888 and m > 16:
        assert need > 0, "this shape is meant to exercise the K-split last round"
    if need:
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    M.ms_gemm_bf16(S.to_device(a, M.MS_BF16), S.to_device(w, M.MS_BF16), None if b is None else S.to_device(b, M.MS_BF16),
                   outs, split, ws)
    torch.cuda.synchronize()
    got = np.concatenate([o.float().cpu().numpy() for o in outs], axis=1).astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    bound = 2.0 ** -8 * np.abs(ref) + 1e-5 * np.abs(ref).max()
    assert (err <= bound).all(), f"max excess {np.max(err - bound):.3e} at {np.unravel_index(np.argmax(err - bound), err.shape)}"


@pytest.mark.parametrize("case", range(10))
def test_gemm_random_shapes(case):
    """Seeded random shapes: ragged row counts (also across the 256-row tile), several destinations,
    every split depth the shape allows."""
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    rng = W.make_rng(905, case)
    m = int(rng.choice([1, 3, 63, 64, 65, 255, 256, 257, 300, 511, 513, 600]))
    n_blocks = int(rng.integers(1, 17))
    split = int(rng.choice([1, 1, 2, 3, 4, 8]))
    k = 32 * split * int(rng.integers(1, 9))
    n = 128 * n_blocks
    cuts = sorted(set(int(c) for c in rng.integers(1, n_blocks, size=int(rng.integers(0, 4)))) if n_blocks > 1 else [])[:3]
    bounds = [0] + [128 * c for c in cuts] + [n]
    widths = [b - a for a, b in zip(bounds, bounds[1:])]
    with_bias = bool(rng.integers(0, 2))
    a = W.normal_bf16_bits(rng, (m, k), 1.0)
    w = W.normal_bf16_bits(rng, (n, k), k ** -0.5)
    b = W.normal_bf16_bits(rng, (n,), 0.5) if with_bias else None
    f64 = lambda x: O.bf16_bits_to_f32(x).astype(np.float64)
    ref = f64(a) @ f64(w).T + (f64(b) if with_bias else 0.0)
    outs = [torch.full((m, wd), float("nan"), dtype=torch.bfloat16, device="cuda") for wd in widths]
    need = M.ms_gemm_workspace_bytes(m, n, k, split)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
    M.ms_gemm_bf16(S.to_device(a, M.MS_BF16), S.to_device(w, M.MS_BF16), None if b is None else S.to_device(b, M.MS_BF16),
                   outs, split, ws)
    torch.cuda.synchronize()
    got = np.concatenate([o.float().cpu().numpy() for o in outs], axis=1).astype(np.float64)
    assert np.isfinite(got).all(), f"m {m} n {n} k {k} split {split} widths {widths}"
    err = np.abs(got - ref)
    bound = 2.0 ** -8 * np.abs(ref) + 1e-5 * np.abs(ref).max()
    assert (err <= bound).all(), f"m {m} n {n} k {k} split {split} widths {widths}: max excess {np.max(err - bound):.3e}"


@pytest.mark.parametrize("case", range(12))
def test_few_row_gemm_random_shapes(case):
    """Seeded random shapes of the few-row kernel: 1 to 16 rows, K a multiple of 128 (one step to
    dozens, also more than one K part), several destinations, bias or none; every third case the
    SwiGLU product, every fourth the greedy token as well."""
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    from oracle import decoder_oracle as DO
    rng = W.make_rng(908, case)
    m = int(rng.integers(1, 17))
    n_blocks = int(rng.choice([1, 2, 3, 8, 20, 37]))
    k = 128 * int(rng.choice([1, 2, 3, 5, 8, 13, 28, 40]))
    n = 128 * n_blocks
    cuts = sorted(set(int(c) for c in rng.integers(1, n_blocks, size=int(rng.integers(0, 3)))) if n_blocks > 1 else [])[:3]
    bounds = [0] + [128 * c for c in cuts] + [n]
    widths = [b - a for a, b in zip(bounds, bounds[1:])]
    with_bias = bool(rng.integers(0, 2))
    a = W.normal_bf16_bits(rng, (m, k), 1.0)
    w = W.normal_bf16_bits(rng, (n, k), k ** -0.5)
    b = W.normal_bf16_bits(rng, (n,), 0.5) if with_bias else None
    f64 = lambda x: O.bf16_bits_to_f32(x).astype(np.float64)
    prod = f64(a) @ f64(w).T
    ref = prod + (f64(b) if with_bias else 0.0)
    what = f"m {m} n {n} k {k} widths {widths} bias {with_bias}"
    ad, wd = S.to_device(a, M.MS_BF16), S.to_device(w, M.MS_BF16)
    outs = [torch.full((m, wd_), float("nan"), dtype=torch.bfloat16, device="cuda") for wd_ in widths]
    need = M.ms_gemm_workspace_bytes(m, n, k, 1)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    M.ms_gemm_bf16(ad, wd, None if b is None else S.to_device(b, M.MS_BF16), outs, 1, ws)
    torch.cuda.synchronize()
    got = np.concatenate([o.float().cpu().numpy() for o in outs], axis=1).astype(np.float64)
    assert np.isfinite(got).all(), what
    err = np.abs(got - ref)
    bound = 2.0 ** -8 * np.abs(ref) + 1e-5 * np.abs(ref).max()
    assert (err <= bound).all(), f"{what}: max excess {np.max(err - bound):.3e}"
    if case % 3 == 0 and n % 256 == 0:      # the same weight read as interleaved gate / up blocks
        inter = n // 2
        wv = f64(w).reshape(inter // 32, 2, 32, k)
        gate, up = f64(a) @ wv[:, 0].reshape(inter, k).T, f64(a) @ wv[:, 1].reshape(inter, k).T
        want = DO.silu(gate) * up
        act = torch.full((m, inter), float("nan"), dtype=torch.bfloat16, device="cuda")
        M.ms_gemm_swiglu_bf16(ad, wd, act, ws)
        torch.cuda.synchronize()
        ga = act.float().cpu().numpy().astype(np.float64)
        tol = 2.0 ** -8 * np.abs(want) + 2e-5 * (np.abs(gate) + 1.0) * (np.abs(up) + 1.0)
        assert np.isfinite(ga).all() and (np.abs(ga - want) <= tol).all(), what
    if case % 4 == 0:
        tok = torch.full((m,), -1, dtype=torch.int32, device="cuda")
        kws = torch.empty(M.ms_lm_head_argmax_workspace_bytes(m, n, k), dtype=torch.uint8, device="cuda")
        M.ms_lm_head_argmax_bf16(ad, wd, tok, kws)
        torch.cuda.synchronize()
        srt = np.sort(prod, axis=1)
        clear = (srt[:, -1] - srt[:, -2]) > 1e-4 * np.abs(prod).max() if n > 1 else np.ones(m, bool)
        assert (tok.cpu().numpy()[clear] == np.argmax(prod, axis=1)[clear]).all(), what


def test_gemm_last_round_split_is_optional():
    """Without workspace the same shape runs whole tiles throughout; both ways give the product."""
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    m, n, k = 448, 37888, 512
    rng = W.make_rng(901)
    a = W.normal_bf16_bits(rng, (m, k), 1.0)
    w = W.normal_bf16_bits(rng, (n, k), k ** -0.5)
    ad, wd = S.to_device(a, M.MS_BF16), S.to_device(w, M.MS_BF16)
    ws = torch.empty(M.ms_gemm_workspace_bytes(m, n, k, 1), dtype=torch.uint8, device="cuda")
    assert ws.numel() > 0
    o1 = torch.zeros(m, n, dtype=torch.bfloat16, device="cuda")
    o2 = torch.zeros_like(o1)
    M.ms_gemm_bf16(ad, wd, None, [o1], 1, ws)
    M.ms_gemm_bf16(ad, wd, None, [o2], 1, None)
    torch.cuda.synchronize()
    main_cols = 16 * 8 * 256    # the first round's columns (16 groups of 8 column tiles on 256 compute units) do not depend on the workspace
    assert torch.equal(o1[:, :main_cols], o2[:, :main_cols])
    d = (o1.float() - o2.float()).abs()
    assert float(d.max()) <= 2.0 ** -7 * float(o2.float().abs().max())   # other order of fp32 additions: one bf16 step at most


def test_gemm_results_do_not_depend_on_timing():
    """The K parts are summed in a fixed order and no tile depends on which workgroup ran first: repeated calls
    give the same bits, with K divided over workgroups, with the last round divided, and with whole tiles."""
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    rng = W.make_rng(906)
    for m, n, k, split in ((448, 4608, 3584, 4), (448, 37888, 512, 1), (300, 1280, 2048, 8), (448, 3584, 3584, 7)):
        ad = S.to_device(W.normal_bf16_bits(rng, (m, k), 1.0), M.MS_BF16)
        wd = S.to_device(W.normal_bf16_bits(rng, (n, k), k ** -0.5), M.MS_BF16)
        ws = torch.empty(max(16, M.ms_gemm_workspace_bytes(m, n, k, split)), dtype=torch.uint8, device="cuda")
        first = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
        M.ms_gemm_bf16(ad, wd, None, [first], split, ws)
        for _ in range(4):
            again = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device="cuda")
            M.ms_gemm_bf16(ad, wd, None, [again], split, ws)
            assert torch.equal(again.view(torch.int16), first.view(torch.int16)), (m, n, k, split)


SWIGLU_CASES = [(7, 64, 32), (300, 1088, 256), (448, 18944, 512),
                (7, 18944, 512), (16, 128, 128), (5, 1152, 384), (1, 2048, 3584),   # few rows: the few-row kernel
                (14, 18944, 3584), (16, 16384, 3584)]                               # ... with a whole compute unit's LDS for A


@pytest.mark.parametrize("m,inter,k", SWIGLU_CASES)
def test_gate_up_gemm_with_swiglu_epilogue(m, inter, k):
    """silu(A Wg^T) * (A Wu^T) (the models' MLP, Section 3.1) in fp64 against the fused GEMM, which
    applies SwiGLU to its fp32 sums and rounds once."""
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    from oracle import decoder_oracle as DO
    rng = W.make_rng(902, m, inter, k)
    a = W.normal_bf16_bits(rng, (m, k), 1.0)
    wg = W.normal_bf16_bits(rng, (inter, k), k ** -0.5)
    wu = W.normal_bf16_bits(rng, (inter, k), k ** -0.5)
    f64 = lambda x: O.bf16_bits_to_f32(x).astype(np.float64)
    gate, up = f64(a) @ f64(wg).T, f64(a) @ f64(wu).T
    ref = DO.silu(gate) * up
    blocked = M.interleave_gate_up(S.to_device(wg, M.MS_BF16), S.to_device(wu, M.MS_BF16))
    out = torch.full((m, inter), float("nan"), dtype=torch.bfloat16, device="cuda")
    need = M.ms_gemm_workspace_bytes(m, 2 * inter, k, 1)
    if inter == 18944 and m > 16:
        assert need > 0      # the tiled kernel's K-split last round
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
    M.ms_gemm_swiglu_bf16(S.to_device(a, M.MS_BF16), blocked, out, ws)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    # one bf16 rounding of the result + the fp32 sums' error carried through silu and the product
    bound = 2.0 ** -8 * np.abs(ref) + 2e-5 * (np.abs(gate) + 1.0) * (np.abs(up) + 1.0)
    assert (err <= bound).all(), f"max excess {np.max(err - bound):.3e} at {np.unravel_index(np.argmax(err - bound), err.shape)}"


ARGMAX_CASES = [(7, 16384, 1536), (5, 2048, 512), (1, 128, 512), (8, 37888, 1024), (9, 1024, 512), (300, 4096, 256), (448, 2048, 3584),
                (16, 152064, 256), (12, 37888, 384), (3, 1024, 128), (7, 152064, 256), (12, 32768, 3584)]


@pytest.mark.parametrize("m,vocab,k", ARGMAX_CASES)
def test_lm_head_with_greedy_token(m, vocab, k):
    """Greedy token straight from the fp32 sums of the LM-head product (Algorithm 1, SpeculativeStep:
    the model's own next token): against the argmax of the fp64 product wherever that one is clear;
    equal maxima resolve to the lowest column and NaN never wins."""
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    rng = W.make_rng(906, m, vocab, k)
    a = W.normal_bf16_bits(rng, (m, k), 1.0)
    w = W.normal_bf16_bits(rng, (vocab, k), k ** -0.5)
    # planted cases: row 0's best column duplicated further down (a tie: the lower one must win) ...
    f64 = lambda x: O.bf16_bits_to_f32(x).astype(np.float64)
    ref = f64(a) @ f64(w).T
    top0 = int(np.argmax(ref[0]))
    dup = (top0 + vocab // 2) % vocab
    w[dup] = w[top0]
    # ... and a weight row of NaN (0x7fc0), which must never be chosen
    nan_col = (top0 + 7) % vocab
    if nan_col == dup:
        nan_col = (nan_col + 1) % vocab
    w[nan_col] = 0x7FC0
    ref = f64(a) @ f64(w).T
    ref_valid = np.where(np.isnan(ref), -np.inf, ref)
    want = np.argmax(ref_valid, axis=1)                      # numpy: first among equal maxima
    srt = np.sort(ref_valid, axis=1)
    margin = srt[:, -1] - srt[:, -2]
    out = torch.full((m,), -1, dtype=torch.int32, device="cuda")
    ws = torch.empty(M.ms_lm_head_argmax_workspace_bytes(m, vocab, k), dtype=torch.uint8, device="cuda")
    M.ms_lm_head_argmax_bf16(S.to_device(a, M.MS_BF16), S.to_device(w, M.MS_BF16), out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert got[0] == min(top0, dup), f"tie between columns {top0} and {dup} went to {got[0]}"
    assert (got != nan_col).all()
    clear = margin > 1e-4 * np.abs(ref[np.isfinite(ref)]).max()
    clear[0] = False                                          # row 0 is the planted tie (margin 0)
    assert clear.sum() >= (m - 1) * 0.8
    assert (got[clear] == want[clear]).all(), f"rows {np.nonzero(clear & (got != want))[0]}"
    with pytest.raises(M.MsError) as e:
        M.ms_lm_head_argmax_bf16(S.to_device(a, M.MS_BF16), S.to_device(w, M.MS_BF16), out, None)
    assert e.value.code == M.MS_ERR_WORKSPACE


NORM_CASES = [
    # M, N, K, split_k, same K parts as the two-call path (then the bits must agree)
    (7, 3584, 18944, 1, True),      # a single sequence's down projection: 8 K parts either way
    (448, 3584, 18944, 4, True),    # a batch's down projection on the tiled kernel
    (300, 1024, 2048, 8, True),
    (16, 128, 256, 1, False),       # few rows, short K: one part in the two-call path, two here
    (14, 512, 1024, 1, False),
    (257, 8192, 64, 2, True),       # the widest row the norm takes
]


@pytest.mark.parametrize("m,n,k,split,same_parts", NORM_CASES)
def test_projection_with_residual_add_and_rmsnorm(m, n, k, split, same_parts):
    """h += bf16(A W^T), out = rmsnorm(h) * g in one call: against the fp64 definition, and against
    ms_gemm_bf16 followed by ms_add_rmsnorm (the same bits where both divide K alike)."""
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    rng = W.make_rng(907, m, n, k)
    a = W.normal_bf16_bits(rng, (m, k), 1.0)
    w = W.normal_bf16_bits(rng, (n, k), k ** -0.5)
    gam = W.normal_bf16_bits(rng, (n,), 0.3) 
    h0 = rng.standard_normal((m, n)).astype(np.float32)
    eps = 1e-6
    f64 = lambda x: O.bf16_bits_to_f32(x).astype(np.float64)
    delta = f64(a) @ f64(w).T
    h_ref = h0.astype(np.float64) + delta
    out_ref = h_ref / np.sqrt((h_ref ** 2).mean(axis=1, keepdims=True) + eps) * f64(gam)
    ad, wd, gd = S.to_device(a, M.MS_BF16), S.to_device(w, M.MS_BF16), S.to_device(gam, M.MS_BF16)
    need = M.ms_gemm_add_rmsnorm_workspace_bytes(m, n, k, split)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    h1 = torch.from_numpy(h0).cuda()
    out1 = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device="cuda")
    M.ms_gemm_add_rmsnorm_bf16(ad, wd, h1, gd, eps, out1, split, ws)
    torch.cuda.synchronize()
    got_h, got = h1.cpu().numpy().astype(np.float64), out1.float().cpu().numpy().astype(np.float64)
    # delta is rounded to bf16 before it is added (2^-9 relative), the output once more
    assert (np.abs(got_h - h_ref) <= 2.0 ** -8 * np.abs(delta) + 1e-5 * np.abs(delta).max() + 1e-6 * np.abs(h_ref)).all()
    tol = 2.0 ** -8 * np.abs(out_ref) + 2.0 ** -7 * np.abs(f64(gam)) * (np.abs(delta) / np.sqrt((h_ref ** 2).mean(axis=1, keepdims=True))) + 1e-4
    assert np.isfinite(got).all() and (np.abs(got - out_ref) <= tol).all(), f"max excess {np.max(np.abs(got - out_ref) - tol):.3e}"
    # the two-call path
    d2 = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    need2 = M.ms_gemm_workspace_bytes(m, n, k, split)
    ws2 = torch.empty(max(need2, 16), dtype=torch.uint8, device="cuda")
    M.ms_gemm_bf16(ad, wd, None, [d2], split, ws2)
    h2 = torch.from_numpy(h0).cuda()
    out2 = torch.empty_like(out1)
    M.ms_add_rmsnorm(h2, d2, gd, eps, out2)
    torch.cuda.synchronize()
    if same_parts:
        assert torch.equal(h1, h2) and torch.equal(out1.view(torch.int16), out2.view(torch.int16))
    else:
        assert float((h1 - h2).abs().max()) <= 2.0 ** -7 * float(d2.float().abs().max())
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_add_rmsnorm_bf16(ad, wd, h1, gd, eps, out1, split, None)
    assert e.value.code == M.MS_ERR_WORKSPACE
    if m > 16:
        with pytest.raises(M.MsError) as e:
            M.ms_gemm_add_rmsnorm_bf16(ad, wd, h1, gd, eps, out1, 1, ws)     # above 16 rows the caller divides K
        assert e.value.code == M.MS_ERR_INVALID


def test_gemm_rejects_what_it_is_not_built_for():
    from paper_2604_14889_amd import binding as M
    a = torch.zeros(4, 64, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(192, 64, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4, 192, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_bf16(a, w, None, [out])                       # 192 is not a multiple of 128
    assert e.value.code == M.MS_ERR_UNSUPPORTED
    w = torch.zeros(256, 64, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4, 256, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_bf16(a, w, None, [out], split_k=2)            # no workspace
    assert e.value.code == M.MS_ERR_WORKSPACE
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_bf16(a, w, None, [out], split_k=4)            # 64 is not a multiple of 32 x 4
    assert e.value.code == M.MS_ERR_UNSUPPORTED
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_bf16(a, w, None, [out[:, :64].contiguous(), torch.zeros(4, 192, dtype=torch.bfloat16, device="cuda")])
    assert e.value.code == M.MS_ERR_INVALID                     # boundary at column 64
