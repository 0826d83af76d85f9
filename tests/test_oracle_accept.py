"""Pins for greedy longest-prefix acceptance (CPU only)."""
import itertools

import numpy as np

import workloads as W
from oracle import memosight_oracle as O


def test_all_match_patterns_brute_force():
    # every pattern of per-slot agreement for n <= 5: accepted count = leading run of matches
    for n in range(1, 6):
        for pattern in itertools.product([0, 1], repeat=n):
            draft = np.arange(10, 10 + n)[None]
            target = draft.copy()
            for j, m in enumerate(pattern):
                if not m:
                    target[0, j] = 999 - j
            a, nxt = O.accept(draft, target)
            lead = 0
            for m in pattern:
                if not m:
                    break
                lead += 1
            assert a[0] == lead
            assert nxt[0] == (target[0, lead] if lead < n else -1)


def test_accepted_tokens_are_a_prefix_of_the_drafts():
    rng = W.make_rng(300)
    forced = [0, 1, 2, 3, 4, 2, 4, 0]
    draft, target = W.draft_and_target(rng, 8, 4, 1000, forced)
    a, nxt = O.accept(draft, target)
    assert a.tolist() == forced
    for b in range(8):
        assert np.array_equal(draft[b, :a[b]], target[b, :a[b]])
        if a[b] < 4:
            assert nxt[b] == target[b, a[b]] and nxt[b] != draft[b, a[b]]
        else:
            assert nxt[b] == -1


def test_random_drafts_mostly_rejected_at_slot_zero():
    rng = W.make_rng(301)
    draft, target = W.draft_and_target(rng, 512, 4, 1000)
    a, _ = O.accept(draft, target)
    assert 0 <= a.min() and a.max() <= 4
    assert (a == 0).mean() > 0.98                 # chance of a match is 1/1000 per slot


def test_stop_id_truncates_just_after_the_delimiter():
    draft = np.array([[5, 7, 9, 11], [5, 7, 9, 11], [7, 1, 2, 3]])
    target = draft.copy()
    target[1, 0] = 6
    a, nxt = O.accept(draft, target, stop_ids=[7])
    assert a.tolist() == [2, 0, 1]
    assert nxt.tolist() == [9, 6, 1]
    a, _ = O.accept(draft, target, stop_ids=[])
    assert a.tolist() == [4, 0, 4]
