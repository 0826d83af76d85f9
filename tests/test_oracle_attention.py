"""Pins for the oracle's RoPE and Predict+Verify attention (CPU only)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import memosight_oracle as O
from tests import helpers_dense as H


# ---------------------------------------------------------------- RoPE ------

def test_rope_matches_public_library_routine():
    rng = W.make_rng(100)
    for d, base in ((64, 10000.0), (128, 1000000.0), (8, 10000.0)):
        x = rng.standard_normal((9, 3, d))
        pids = [0, 1, 2, 7, 100, 321, 4097, 12289, 49153]
        got = O.rope(x, np.asarray(pids)[:, None], O.rope_inv_freq(d, base))
        ref = H.hf_rope(x, pids, base)
        # The library builds inv_freq in fp32 arithmetic (it can sit one ulp away from the
        # double-then-rounded value used here), so angles may differ by about p * 2^-23:
        # tight at small positions, proportionally looser at large ones.  A wrong pairing,
        # sign or frequency formula is an O(1) error and fails either bound.
        err = np.abs(got - ref).max(axis=(1, 2))
        bound = 5e-6 + np.asarray(pids) * 2.0 ** -23 * np.abs(x).max()
        assert np.all(err < bound), (err, bound)


def test_rope_two_dims_is_plane_rotation():
    # D = 2: one pair, inv_freq = 1, so position p rotates (1, 0) to (cos p, sin p)
    inv = O.rope_inv_freq(2, 10000.0)
    assert inv.tolist() == [1.0]
    for p in (0, 1, 2, 3):
        y = O.rope(np.array([1.0, 0.0]), np.array(p), inv)
        assert np.allclose(y, [np.cos(np.float32(p)), np.sin(np.float32(p))], atol=1e-15)


def test_rope_position_zero_is_identity_and_norm_kept():
    rng = W.make_rng(101)
    x = rng.standard_normal((5, 64))
    inv = O.rope_inv_freq(64, 10000.0)
    assert np.array_equal(O.rope(x, np.zeros(5, int), inv), x)
    y = O.rope(x, np.arange(5) * 1000, inv)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)


def test_rope_scores_depend_on_relative_position_only():
    # exact in exact arithmetic; here angles are fp32-rounded, so rounding-level only
    rng = W.make_rng(102)
    inv = O.rope_inv_freq(64, 10000.0)
    q, k = rng.standard_normal(64), rng.standard_normal(64)
    base = O.rope(q, np.array(40), inv) @ O.rope(k, np.array(33), inv)
    for shift in (1, 64, 1000):
        s = O.rope(q, np.array(40 + shift), inv) @ O.rope(k, np.array(33 + shift), inv)
        assert abs(s - base) < 2e-3 * (1 + shift / 100)


def test_inv_freq_closed_form():
    inv = O.rope_inv_freq(128, 1000000.0)
    assert inv.dtype == np.float32 and inv.shape == (64,)
    assert inv[0] == 1.0
    assert abs(float(inv[32]) - 1e-3) < 1e-9          # base^(-64/128) = 1e-3
    assert np.all(np.diff(inv) < 0)


# ------------------------------------------------------- bf16 rounding ------

def test_round_bf16_against_torch():
    rng = W.make_rng(103)
    x = (rng.standard_normal(20000) * 10 ** rng.uniform(-6, 6, 20000)).astype(np.float32)
    x[:6] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38]   # ties both ways, near max
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.round_bf16(x).view(np.uint32), ref.view(np.uint32))


# ------------------------------------------------ dense brute-force pin -----

def build_paper_sequence(rng, n_kv_heads, group, d, base, n_verify, n_foresight):
    """A full training-style sequence [P, R_1, M_1, <o>, R_2, M_2, <o>, R_3 prefix, verify, foresight].

    PIDs are written out by hand from the paper's rules (c = 3):
      P: 4 tokens PIDs 1..4;  R_1: 6 tokens PIDs 5..10 -> groups {5,6,7} {8,9,10} -> memory PIDs 6, 9;
      <o> PID 11;  R_2: 5 tokens PIDs 12..16 -> groups {12,13,14} {15,16} -> memory PIDs 13, 15;
      <o> PID 17;  R_3 prefix: 3 tokens PIDs 18..20;  verify: 21..;  foresight continue after.
    """
    kinds = ["P"] * 4 + ["R"] * 6 + ["M", "M", "O"] + ["R"] * 5 + ["M", "M", "O"] + ["R"] * 3
    steps = [-1] * 4 + [0] * 6 + [0, 0, 0] + [1] * 5 + [1, 1, 1] + [2] * 3
    pids = [1, 2, 3, 4] + list(range(5, 11)) + [6, 9, 11] + list(range(12, 17)) + [13, 15, 17] + [18, 19, 20]
    kinds += ["R"] * n_verify + ["F"] * n_foresight
    steps += [2] * (n_verify + n_foresight)
    pids += list(range(21, 21 + n_verify + n_foresight))
    n = len(kinds)
    hq = n_kv_heads * group
    q = rng.standard_normal((n, hq, d))
    k = rng.standard_normal((n, n_kv_heads, d))
    v = rng.standard_normal((n, n_kv_heads, d))
    return kinds, steps, pids, q, k, v


@pytest.mark.parametrize("n_kv_heads,group,d,n_verify,n_foresight",
                         [(1, 1, 8, 1, 0), (2, 2, 16, 4, 3), (1, 3, 8, 2, 2), (2, 1, 64, 3, 0)])
def test_oracle_equals_dense_masked_softmax_over_full_sequence(n_kv_heads, group, d, n_verify, n_foresight):
    base = 10000.0
    rng = W.make_rng(110, n_kv_heads, group, d, n_verify)
    kinds, steps, pids, q, k, v = build_paper_sequence(rng, n_kv_heads, group, d, base, n_verify, n_foresight)
    n = len(kinds)
    n_q = n_verify + n_foresight
    scale = 1.0 / np.sqrt(d)
    # --- dense side: rotate with the library routine, mask from the paper's rules
    mask = H.paper_mask(kinds, steps)
    qr = H.hf_rope(q, pids, base)
    kr = H.hf_rope(k, pids, base)
    rows = list(range(n - n_q, n))
    dense = {}
    for h in range(n_kv_heads * group):
        g = h // group
        dense[h] = H.dense_masked_attention(qr[:, h].tolist(), kr[:, g].tolist(), v[:, g].tolist(),
                                            mask, rows, scale)
    # --- oracle side: drive the cache the way Algorithm 1 does (append, compact, append ...)
    cache = O.PagedCache(1, n_kv_heads, d, n_pages=8, dtype=O.F32, rope_base=base)
    sid = cache.seq_create()

    def app(lo, hi):
        cache.append([sid], [hi - lo], k[None, lo:hi], v[None, lo:hi], pids[lo:hi])

    app(0, 4)                                                # prompt
    app(4, 10)                                               # R_1
    cache.compact([sid], [4], [6], [3], k[None, 10:13], v[None, 10:13], pids[10:13])   # M_1 + <o>
    app(13, 18)                                              # R_2
    cache.compact([sid], [7], [5], [3], k[None, 18:21], v[None, 18:21], pids[18:21])   # M_2 + <o>
    app(21, 24)                                              # R_3 prefix
    assert cache.seq_len[sid] == 4 + 3 + 3 + 3
    lo = n - n_q
    # float32 storage rounding of the cached rows is the only difference (~1e-7)
    qs = q[lo:].astype(np.float32)
    out = O.attention(cache, 0, [sid], n_verify, n_foresight, qs[None], k[None, lo:].astype(np.float32),
                      v[None, lo:].astype(np.float32), np.asarray(pids[lo:])[None], None, None)[0]
    for h in range(n_kv_heads * group):
        for r, i in enumerate(rows):
            assert np.abs(out[r, h] - np.asarray(dense[h][i])).max() < 3e-6


@pytest.mark.parametrize("n_kv_heads,group,d,n_verify,depth", [(1, 2, 8, 3, 2), (2, 1, 16, 4, 3), (1, 1, 8, 1, 4)])
def test_per_position_layout_equals_training_style_sequence(n_kv_heads, group, d, n_verify, depth):
    """The per-position foresight step against the dense reference over the training-style
    sequence: foresight tokens sit between the step's tokens (Section 2.2, "CoT Augmentation"),
    hold PID t + d' - 1 when placed before token t with offset d' (Section 2.2, Foresight
    Tokens), and are masked from everyone else (Section 2.3).  PIDs and mask on the dense side are
    written from those rules, not from the oracle's helper."""
    base = 10000.0
    rng = W.make_rng(111, n_kv_heads, group, d, n_verify)
    n_prompt, n_cached = 5, 4
    first = n_prompt + n_cached + 1                     # PID of the first verify token (PIDs from 1)
    kinds = ["P"] * n_prompt + ["R"] * n_cached
    steps = [-1] * n_prompt + [0] * n_cached
    pids = list(range(1, first))
    where_verify, where_foresight = [], {}
    for j in range(n_verify):
        where_verify.append(len(kinds))
        kinds.append("R"); steps.append(0); pids.append(first + j)
        t_next = first + j + 1                           # the foresight tokens stand before token t_next
        for dp in range(1, depth + 1):
            where_foresight[(j, dp)] = len(kinds)
            kinds.append("F"); steps.append(0); pids.append(t_next + dp - 1)
    n = len(kinds)
    hq = n_kv_heads * group
    q = rng.standard_normal((n, hq, d))
    k = rng.standard_normal((n, n_kv_heads, d))
    v = rng.standard_normal((n, n_kv_heads, d))
    mask = H.paper_mask(kinds, steps)
    qr, kr = H.hf_rope(q, pids, base), H.hf_rope(k, pids, base)
    scale = 1.0 / np.sqrt(d)
    # the step's queries in the helper's order: verify tokens, then each verify token's foresight block
    order = where_verify + [where_foresight[(j, dp)] for j in range(n_verify) for dp in range(1, depth + 1)]
    dense = {h: H.dense_masked_attention(qr[:, h].tolist(), kr[:, h // group].tolist(), v[:, h // group].tolist(),
                                         mask, order, scale) for h in range(hq)}
    lay_pids, lay_ctx = O.per_position_layout(first, n_verify, depth)
    assert lay_pids == [pids[i] for i in order]
    cache = O.PagedCache(1, n_kv_heads, d, n_pages=4, dtype=O.F32, rope_base=base)
    sid = cache.seq_create()
    nc = n_prompt + n_cached
    cache.append([sid], [nc], k[None, :nc], v[None, :nc], pids[:nc])
    f32 = lambda x: x[order].astype(np.float32)[None]
    out = O.attention(cache, 0, [sid], n_verify, n_verify * depth, f32(q), f32(k), f32(v),
                      np.asarray(lay_pids)[None], np.asarray(lay_ctx)[None], None)[0]
    for h in range(hq):
        for r, i in enumerate(order):
            assert np.abs(out[r, h] - np.asarray(dense[h][i])).max() < 3e-6


# ------------------------------------------------- textbook reductions ------

def sdpa_reference(cache, sid, q_rot, k_new_rot, v_new, group, causal_new):
    """torch SDPA over dense gathered K/V; queries bottom-right aligned when causal."""
    kc, vc = cache.gather(0, sid)
    kk = np.concatenate([kc.astype(np.float64), k_new_rot], axis=0)      # [T, Hkv, D]
    vv = np.concatenate([vc.astype(np.float64), v_new], axis=0)
    kt = torch.from_numpy(kk).permute(1, 0, 2).repeat_interleave(group, dim=0)[None]
    vt = torch.from_numpy(vv).permute(1, 0, 2).repeat_interleave(group, dim=0)[None]
    qt = torch.from_numpy(q_rot).permute(1, 0, 2)[None]
    n_q, t = q_rot.shape[0], kk.shape[0]
    m = torch.ones(n_q, t, dtype=torch.bool)
    if causal_new:
        m = torch.tril(m, diagonal=t - n_q)
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=m)
    return o[0].permute(1, 0, 2).numpy()


@pytest.mark.parametrize("n_verify", [1, 4])
def test_no_foresight_reduces_to_causal_decode_attention(n_verify):
    rng = W.make_rng(120, n_verify)
    hkv, group, d, L = 2, 3, 32, 37
    cache = O.PagedCache(1, hkv, d, n_pages=4, dtype=O.F32)
    sid = cache.seq_create()
    cache.append([sid], [L], rng.standard_normal((1, L, hkv, d)), rng.standard_normal((1, L, hkv, d)),
                 list(range(L)))
    q = rng.standard_normal((n_verify, hkv * group, d))
    kn = rng.standard_normal((n_verify, hkv, d))
    vn = rng.standard_normal((n_verify, hkv, d))
    pos = np.arange(L, L + n_verify)
    out = O.attention(cache, 0, [sid], n_verify, 0, q[None], kn[None], vn[None], pos[None])[0]
    ref = sdpa_reference(cache, sid, H.hf_rope(q, pos, 10000.0), H.hf_rope(kn, pos, 10000.0), vn, group, True)
    assert np.abs(out - ref).max() < 3e-6


# ------------------------------------------------------------ invariants ----

def small_case(rng, dtype=O.F32, L=45, n_verify=3, n_foresight=2, hkv=2, group=2, d=16):
    cache = O.PagedCache(1, hkv, d, n_pages=6, dtype=dtype)
    sid = cache.seq_create()
    cache.append([sid], [L], rng.standard_normal((1, L, hkv, d)), rng.standard_normal((1, L, hkv, d)),
                 list(range(L)))
    n_q = n_verify + n_foresight
    q = rng.standard_normal((1, n_q, hkv * group, d))
    kn = rng.standard_normal((1, n_q, hkv, d))
    vn = rng.standard_normal((1, n_q, hkv, d))
    pos = np.arange(L, L + n_q)[None]
    return cache, sid, q, kn, vn, pos


def test_constant_values_give_constant_output_and_weights_sum_to_one():
    rng = W.make_rng(130)
    cache, sid, q, kn, vn, pos = small_case(rng)
    cache.pool[:, :, :, 1] = 1.0
    out = O.attention(cache, 0, [sid], 3, 2, q, kn, np.ones_like(vn), pos)
    assert np.abs(out - 1.0).max() < 1e-12


def test_foresight_queries_are_independent_of_each_other():
    rng = W.make_rng(131)
    cache, sid, q, kn, vn, pos = small_case(rng, n_verify=3, n_foresight=3)
    base = O.attention(cache, 0, [sid], 3, 3, q, kn, vn, pos)
    for j in (3, 4, 5):
        q2, k2, v2 = q.copy(), kn.copy(), vn.copy()
        q2[0, j] += 1.0
        k2[0, j] -= 2.0
        v2[0, j] *= 3.0
        out = O.attention(cache, 0, [sid], 3, 3, q2, k2, v2, pos)
        others = [i for i in range(6) if i != j]
        assert np.array_equal(out[0, others], base[0, others])      # bit-identical
        assert not np.array_equal(out[0, j], base[0, j])


def test_verify_is_causal_and_foresight_sees_whole_verify_block():
    rng = W.make_rng(132)
    cache, sid, q, kn, vn, pos = small_case(rng, n_verify=3, n_foresight=2)
    base = O.attention(cache, 0, [sid], 3, 2, q, kn, vn, pos)
    k2 = kn.copy()
    k2[0, 1] += 1.0                      # change verify token 1's key
    out = O.attention(cache, 0, [sid], 3, 2, q, k2, vn, pos)
    assert np.array_equal(out[0, 0], base[0, 0])                    # earlier verify: unaffected
    for i in (1, 2, 3, 4):                                          # itself, later verify, all foresight
        assert not np.array_equal(out[0, i], base[0, i])


def test_page_permutation_invariance():
    rng = W.make_rng(133)
    cache, sid, q, kn, vn, pos = small_case(rng)
    base = O.attention(cache, 0, [sid], 3, 2, q, kn, vn, pos)
    perm = [5, 3, 0]                                                # new homes for the 3 pages
    old = list(cache.page_table[sid])
    pool2 = np.zeros_like(cache.pool)
    for o, n in zip(old, perm):
        pool2[:, n] = cache.pool[:, o]
    c2 = O.PagedCache(1, 2, 16, n_pages=6, dtype=O.F32, pool=pool2)
    s2 = c2.seq_import(cache.seq_len[sid], perm)
    out = O.attention(c2, 0, [s2], 3, 2, q, kn, vn, pos)
    assert np.array_equal(out, base)


def test_identical_query_rows_in_a_group_give_identical_outputs():
    rng = W.make_rng(134)
    cache, sid, q, kn, vn, pos = small_case(rng, hkv=2, group=3)
    q[0, :, 1] = q[0, :, 0]
    q[0, :, 2] = q[0, :, 0]
    out = O.attention(cache, 0, [sid], 3, 2, q, kn, vn, pos)
    assert np.array_equal(out[0, :, 1], out[0, :, 0]) and np.array_equal(out[0, :, 2], out[0, :, 0])
    # heads 3.. read the other KV head: different result
    q[0, :, 3] = q[0, :, 0]
    out = O.attention(cache, 0, [sid], 3, 2, q, kn, vn, pos)
    assert not np.array_equal(out[0, :, 3], out[0, :, 0])


def test_custom_ctx_new_reproduces_separate_predict_and_verify_passes():
    # the fused default equals: verify rows from a verify-only pass, foresight rows from a
    # pass whose "verify block" is all of them, with the same PIDs
    rng = W.make_rng(135)
    cache, sid, q, kn, vn, pos = small_case(rng, n_verify=3, n_foresight=2)
    fused = O.attention(cache, 0, [sid], 3, 2, q, kn, vn, pos)
    ver = O.attention(cache, 0, [sid], 3, 0, q[:, :3], kn[:, :3], vn[:, :3], pos[:, :3])
    assert np.array_equal(fused[0, :3], ver[0])
    explicit = O.attention(cache, 0, [sid], 3, 2, q, kn, vn, pos, ctx_new=np.array([[0, 1, 2, 3, 3]]))
    assert np.array_equal(fused, explicit)


def test_empty_cache_and_single_query():
    cache = O.PagedCache(1, 1, 8, n_pages=2, dtype=O.F32)
    sid = cache.seq_create()
    rng = W.make_rng(136)
    q = rng.standard_normal((1, 1, 1, 8))
    kn = rng.standard_normal((1, 1, 1, 8))
    vn = rng.standard_normal((1, 1, 1, 8))
    out = O.attention(cache, 0, [sid], 1, 0, q, kn, vn, np.array([[0]]))
    assert np.allclose(out[0, 0, 0], vn[0, 0, 0])                   # sees only itself
