"""Pins for the oracle's paged cache: append, compaction, allocator policy (CPU only)."""
import numpy as np
import pytest

import workloads as W
from oracle import memosight_oracle as O


def kv(rng, n, hkv=2, d=8, layers=1):
    return rng.standard_normal((layers, n, hkv, d)), rng.standard_normal((layers, n, hkv, d))


def test_append_allocates_lowest_page_at_each_16_token_boundary():
    rng = W.make_rng(200)
    c = O.PagedCache(1, 2, 8, n_pages=6, dtype=O.F32)
    a, b = c.seq_create(), c.seq_create()
    assert (a, b) == (0, 1)
    k, v = kv(rng, 17)
    c.append([a], [17], k, v, list(range(17)))
    assert c.page_table[a] == [0, 1] and c.seq_len[a] == 17
    k, v = kv(rng, 16)
    c.append([b], [16], k, v, list(range(16)))
    assert c.page_table[b] == [2]
    k, v = kv(rng, 1)
    c.append([b], [1], k, v, [16])
    assert c.page_table[b] == [2, 3]
    c.seq_free(a)
    assert c.free == [0, 1, 4, 5]
    k, v = kv(rng, 40)
    c.append([b], [40], k, v, list(range(17, 57)))
    assert c.page_table[b] == [2, 3, 0, 1]          # lowest free first
    c.check_integrity()


def test_append_batch_order_and_stored_values():
    rng = W.make_rng(201)
    c = O.PagedCache(2, 2, 8, n_pages=8, dtype=O.F32)
    a, b = c.seq_create(), c.seq_create()
    k, v = kv(rng, 5 + 20, layers=2)
    pos = list(range(5)) + list(range(100, 120))
    c.append([b, a], [5, 20], k, v, pos)            # b first: it gets page 0
    assert c.page_table[b] == [0] and c.page_table[a] == [1, 2]
    ka, va = c.gather(1, a)
    assert np.array_equal(va, v[1, 5:].astype(np.float32))
    want = O.rope(k[1, 5:], np.asarray(pos[5:])[:, None], c.inv_freq).astype(np.float32)
    assert np.array_equal(ka, want)
    kb, _ = c.gather(0, b)
    assert np.array_equal(kb[0], k[0, 0].astype(np.float32))       # position 0: unrotated


def test_append_out_of_pages_leaves_state_unchanged():
    rng = W.make_rng(202)
    c = O.PagedCache(1, 1, 8, n_pages=2, dtype=O.F32)
    a = c.seq_create()
    k, v = kv(rng, 10, hkv=1)
    c.append([a], [10], k, v, list(range(10)))
    k, v = kv(rng, 30, hkv=1)
    with pytest.raises(O.OutOfPages):
        c.append([a], [30], k, v, list(range(30)))
    assert c.seq_len[a] == 10 and c.page_table[a] == [0] and c.free == [1]


def test_bf16_cache_stores_bf16_representable_values():
    rng = W.make_rng(203)
    c = O.PagedCache(1, 1, 8, n_pages=2, dtype=O.BF16)
    a = c.seq_create()
    k, v = kv(rng, 9, hkv=1)
    c.append([a], [9], k, v, list(range(9)))
    kk, vv = c.gather(0, a)
    assert np.all((kk.view(np.uint32) & 0xFFFF) == 0) and np.all((vv.view(np.uint32) & 0xFFFF) == 0)
    assert np.abs(vv - v[0]).max() <= np.abs(v).max() * 2.0 ** -8


def test_config1_compaction_closed_form():
    """4 segments x 64 tokens, each compacted to 4 memory tokens (c = 16), then a 64-token tail."""
    rng = W.make_rng(204)
    c = O.PagedCache(1, 8, 64, n_pages=12, dtype=O.F32)
    s = c.seq_create()
    pid = 1
    for seg in range(4):
        k, v = kv(rng, 64, hkv=8, d=64)
        begin = c.seq_len[s]
        c.append([s], [64], k, v, list(range(pid, pid + 64)))
        l = O.ama_count(64, 16)
        assert l == 4
        mk, mv = kv(rng, l, hkv=8, d=64)
        mpos = O.upl_positions(pid, 64, 16)
        assert mpos == [pid + 7, pid + 23, pid + 39, pid + 55]
        c.compact([s], [begin], [64], [l], mk, mv, mpos)
        assert c.seq_len[s] == 4 * (seg + 1)
        c.check_integrity()
        pid += 64
    k, v = kv(rng, 64, hkv=8, d=64)
    c.append([s], [64], k, v, list(range(257, 321)))
    assert c.seq_len[s] == 80 and len(c.page_table[s]) == 5
    assert c.page_table[s] == [0, 1, 2, 3, 4]
    assert c.peak_pages == 5                     # 4 kept rows + 64 new rows never need more
    c.check_integrity()


def test_compaction_equals_cache_rebuilt_from_kept_tokens():
    """Attention after compaction is bit-identical to attention over a cache that only ever
    received the kept rows, and (built in the same order) the page tables agree too."""
    rng = W.make_rng(205)
    hkv, d = 2, 16
    a = O.PagedCache(1, hkv, d, n_pages=10, dtype=O.BF16)
    b = O.PagedCache(1, hkv, d, n_pages=10, dtype=O.BF16)
    sa, sb = a.seq_create(), b.seq_create()
    kp, vp = kv(rng, 21, hkv, d)                  # prefix that survives
    ks, vs = kv(rng, 50, hkv, d)                  # segment that is evicted
    km, vm = kv(rng, 7, hkv, d)                   # memory tokens
    mpos = O.upl_positions(21, 50, 8)
    assert len(mpos) == 7
    a.append([sa], [21], kp, vp, list(range(21)))
    a.append([sa], [50], ks, vs, list(range(21, 71)))
    a.compact([sa], [21], [50], [7], km, vm, mpos)
    b.append([sb], [21], kp, vp, list(range(21)))
    b.append([sb], [7], km, vm, mpos)
    assert a.seq_len[sa] == b.seq_len[sb] == 28
    assert a.page_table[sa] == b.page_table[sb] == [0, 1]
    assert a.free == b.free
    q = rng.standard_normal((1, 5, 4, d))
    kn, vn = rng.standard_normal((1, 5, hkv, d)), rng.standard_normal((1, 5, hkv, d))
    pos = np.arange(71, 76)[None]
    oa = O.attention(a, 0, [sa], 3, 2, q, kn, vn, pos)
    ob = O.attention(b, 0, [sb], 3, 2, q, kn, vn, pos)
    assert np.array_equal(oa, ob)
    a.check_integrity()


def test_compaction_page_policy_release_then_allocate_lowest():
    rng = W.make_rng(206)
    c = O.PagedCache(1, 1, 8, n_pages=12, dtype=O.F32)
    x, y = c.seq_create(), c.seq_create()
    k, v = kv(rng, 40, 1)
    c.append([x], [40], k, v, list(range(40)))                 # pages 0 1 2
    k, v = kv(rng, 16, 1)
    c.append([y], [16], k, v, list(range(16)))                 # page 3
    k, v = kv(rng, 60, 1)
    c.append([x], [60], k, v, list(range(40, 100)))            # x: 0 1 2 4 5 6 7 (100 rows -> 7 pages)
    assert c.page_table[x] == [0, 1, 2, 4, 5, 6, 7]
    mk, mv = kv(rng, 20, 1)
    # evict rows [20, 100): page 0 full kept, page 1 partially kept, the rest released first
    c.compact([x], [20], [80], [20], mk, mv, list(range(20, 40)))
    assert c.seq_len[x] == 40
    assert c.page_table[x] == [0, 1, 2]                        # 2 is again the lowest free one
    assert c.free == [4, 5, 6, 7, 8, 9, 10, 11]
    c.check_integrity()


def test_compaction_in_the_middle_keeps_tail_rows_in_order():
    rng = W.make_rng(207)
    c = O.PagedCache(1, 1, 8, n_pages=8, dtype=O.F32)
    s = c.seq_create()
    k, v = kv(rng, 50, 1)
    c.append([s], [50], k, v, [0] * 50)                        # PID 0: keys stored as given
    mk, mv = kv(rng, 3, 1)
    c.compact([s], [10], [25], [3], mk, mv, [0, 0, 0])
    kk, vv = c.gather(0, s)
    want_k = np.concatenate([k[0, :10], mk[0], k[0, 35:]]).astype(np.float32)
    want_v = np.concatenate([v[0, :10], mv[0], v[0, 35:]]).astype(np.float32)
    assert np.array_equal(kk, want_k) and np.array_equal(vv, want_v)
    assert c.seq_len[s] == 28 and c.page_table[s] == [0, 1]
    c.check_integrity()


def test_compaction_rejects_bad_ranges_without_side_effects():
    rng = W.make_rng(208)
    c = O.PagedCache(1, 1, 8, n_pages=4, dtype=O.F32)
    s = c.seq_create()
    k, v = kv(rng, 20, 1)
    c.append([s], [20], k, v, list(range(20)))
    mk, mv = kv(rng, 1, 1)
    with pytest.raises(ValueError):
        c.compact([s], [10], [11], [1], mk, mv, [0])
    assert c.seq_len[s] == 20 and c.page_table[s] == [0, 1]


def test_seq_import_and_integrity():
    c = O.PagedCache(1, 1, 8, n_pages=6, dtype=O.F32)
    s = c.seq_import(33, [5, 2, 4])
    assert c.page_table[s] == [5, 2, 4] and c.free == [0, 1, 3]
    with pytest.raises(ValueError):
        c.seq_import(5, [2])
    with pytest.raises(ValueError):
        c.seq_import(40, [0, 1])
    c.check_integrity()
    t = c.seq_create()
    assert t == 1
    c.seq_free(s)
    assert c.free == [0, 1, 2, 3, 4, 5]
