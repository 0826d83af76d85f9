"""Pins for the oracle's integer position-layout helpers.

Expected values come from tests/golden/paper_worked_values.txt (values the paper
prints) and from closed forms, never from the oracle itself.
"""
import os

import pytest

from oracle import memosight_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_values.txt")


def load_golden():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, inputs, expected, _cite = [x.strip() for x in line.split("|", 3)]
            kv = dict(tok.split("=") for tok in inputs.split())
            rows[name] = ({k: int(v) for k, v in kv.items()}, int(expected))
    return rows


G = load_golden()


def test_golden_file_has_all_rows():
    assert set(G) == {"upl", "ama", "output_pid", "foresight_pid", "foresight_train_pid",
                      "drafts_per_pass", "ama_long"}


def test_upl_printed_example():
    inp, exp = G["upl"]
    assert O.upl_positions(inp["first_pid"], inp["n"], inp["c"]) == [exp]


def test_ama_printed_examples():
    inp, exp = G["ama"]
    assert O.ama_count(inp["n"], inp["c"]) == exp
    inp, exp = G["ama_long"]
    assert O.ama_count(inp["n"], inp["c"]) == exp
    assert len(O.upl_positions(1, inp["n"], inp["c"])) == exp


def test_output_pid_printed_example():
    inp, exp = G["output_pid"]
    assert O.output_token_pid(inp["last_pid"]) == exp
    assert O.next_step_first_pid(inp["last_pid"]) == exp + 1


def test_foresight_pid_printed_example():
    # the token that predicts PID 4 holds PID 3; with the prefix ending at PID 2 it is
    # the first foresight token (the prefix's last token itself predicts PID 3)
    inp, exp = G["foresight_pid"]
    target = inp["target_pid"]
    pids = O.foresight_pids(last_prefix_pid=exp - 1, d=1)
    assert pids == [exp] and pids[0] + 1 == target


def test_foresight_training_rule_consistent():
    # training rule: foresight before r_t with offset d' has PID t + d' - 1
    inp, exp = G["foresight_train_pid"]
    t, dp = inp["t"], inp["dprime"]
    assert t + dp - 1 == exp
    # inference: prefix ends at r_{t-1}... the j-th appended foresight token plays the
    # role of offset d' = j placed before r_{t}, where t - 1 is the last prefix PID
    for last in (0, 5, 99):
        for d in (1, 2, 3, 4):
            pids = O.foresight_pids(last, d)
            assert pids == [(last + 1) + j - 1 for j in range(1, d + 1)]


def test_drafts_per_pass():
    inp, exp = G["drafts_per_pass"]
    d = inp["d"]
    # verify block of the next pass = next-token prediction + d foresight predictions
    assert 1 + len(O.foresight_pids(10, d)) == exp


@pytest.mark.parametrize("c", [1, 3, 5, 7, 9])
def test_upl_closed_form_odd_ratio(c):
    # full groups of odd size: centre is first + g*c + (c-1)/2
    for first in (1, 17):
        for groups in (1, 2, 5):
            n = groups * c
            assert O.upl_positions(first, n, c) == [first + g * c + (c - 1) // 2 for g in range(groups)]


def test_upl_properties_brute_force():
    for c in range(1, 9):
        for n in range(0, 40):
            for first in (0, 1, 100):
                pids = O.upl_positions(first, n, c)
                assert len(pids) == -(-n // c)
                # each PID lies inside its own group and is the group's (lower) median
                for g, p in enumerate(pids):
                    members = list(range(first + g * c, first + min((g + 1) * c, n)))
                    assert members, "group must not be empty"
                    assert p == members[(len(members) - 1) // 2]
                assert pids == sorted(set(pids))


def test_upl_short_last_group():
    # n = 7, c = 3: groups {0,1,2} {3,4,5} {6}; PIDs first+1, first+4, first+6
    assert O.upl_positions(10, 7, 3) == [11, 14, 16]
    # even group: lower middle
    assert O.upl_positions(1, 16, 16) == [8]
    assert O.upl_positions(1, 64, 16) == [8, 24, 40, 56]


def test_default_ctx_new():
    assert O.default_ctx_new(4, 3) == [0, 1, 2, 3, 4, 4, 4]
    assert O.default_ctx_new(1, 0) == [0]
    assert O.default_ctx_new(5, 4) == [0, 1, 2, 3, 4, 5, 5, 5, 5]


def test_ama_rejects_bad_input():
    with pytest.raises(ValueError):
        O.ama_count(3, 0)
    with pytest.raises(ValueError):
        O.ama_count(-1, 2)


def test_per_position_layout_from_the_training_rule():
    # foresight before token t with offset d' holds PID t + d' - 1 (golden row foresight_train_pid
    # is the d' = 1, t = 1 case) and sees what token t sees of the step: the tokens before t
    inp, exp = G["foresight_train_pid"]
    pids, ctx = O.per_position_layout(inp["t"] - 1, 1, 1)      # one verify token r_0 at PID t - 1
    assert pids == [inp["t"] - 1, exp] and ctx == [0, 1]
    for first in (1, 40):
        for nv in (1, 2, 5):
            for d in (0, 1, 4):
                pids, ctx = O.per_position_layout(first, nv, d)
                assert len(pids) == len(ctx) == nv * (1 + d)
                assert pids[:nv] == list(range(first, first + nv)) and ctx[:nv] == list(range(nv))
                at = nv
                for j in range(nv):
                    t = first + j + 1                          # the token these foresight tokens precede
                    for dp in range(1, d + 1):
                        assert pids[at] == t + dp - 1
                        assert ctx[at] == t - first            # verify tokens with PID below t
                        at += 1
    # with a single verify token it is the plain step layout
    assert O.per_position_layout(7, 1, 3) == ([7] + O.foresight_pids(7, 3), O.default_ctx_new(1, 3))


def test_consecutive_memory_positions():
    assert O.consecutive_memory_positions(10, 3) == [11, 12, 13]
    assert O.consecutive_memory_positions(10, 0) == []


def test_upl_fixed_budget_reduces_to_ratio_rule_and_stays_in_span():
    # whenever the budget divides the step evenly the groups are the ratio rule's groups
    for c in range(1, 8):
        for groups in range(1, 10):
            for first in (1, 33):
                assert O.upl_positions_fixed(first, groups * c, groups) == O.upl_positions(first, groups * c, c)
    assert O.upl_positions_fixed(1, 56, 8) == [1 + 7 * g + 3 for g in range(8)]      # closed form, c = 7
    for n in range(1, 40):
        for l in range(1, 12):
            pids = O.upl_positions_fixed(5, n, l)
            assert len(pids) == l and pids == sorted(pids)
            assert 5 <= pids[0] and pids[-1] <= 5 + n - 1
            # brute force: token t belongs to the last group whose boundary floor(g n / l) is <= t
            members = [[] for _ in range(l)]
            for t in range(n):
                members[max(g for g in range(l) if g * n // l <= t)].append(t)
            for g in range(l):
                if members[g]:
                    assert pids[g] == 5 + members[g][(len(members[g]) - 1) // 2]
                else:
                    assert pids[g] == 5 + g * n // l
            if l <= n:
                assert len(set(pids)) == l and all(members)
    with pytest.raises(ValueError):
        O.upl_positions_fixed(1, 0, 9)
