"""Pins of oracle/sparse_tree.py: the draft-side control of a round (Sec. IV-A truncation, Sec. IV-B
merging of the kept suffix, Sec. IV-C marks and second-pass branches) against trees worked out by
hand from those passages and the stated readings (threshold strict, the uncertain token kept,
window +-1, branch hangs off the trunk token before the mark, concatenation copies the trunk's
tail).  The draft model is a hand-made table path -> (top1, top2, prob)."""
import numpy as np

from oracle import sparse_tree as st


class Table:
    """read_out(path): explicit entries, else "next token = last + 1, second = last + 50, p = 0.9"."""

    def __init__(self, entries=None):
        self.entries = dict(entries or {})
        self.calls = []

    def __call__(self, path):
        self.calls.append(path)
        if path in self.entries:
            return self.entries[path]
        return path[-1] + 1, path[-1] + 50, 0.9


def test_asp_truncates_behind_the_first_token_strictly_below_the_threshold():
    t = Table({(5, 6, 7): (8, 58, 0.4),           # exactly at the threshold: still certain
               (5, 6, 7, 8): (9, 59, 0.39)})      # below: token 9 is kept, drafting stops
    r = st.build_round(t, 5, 100, {}, st.Params(mode="asp"))
    assert r.tokens == [5, 6, 7, 8, 9] and r.parents == [-1, 0, 1, 2, 3] and r.trunk == [0, 1, 2, 3, 4]
    assert r.read_outs == 4 and r.marks == []
    # the same table without truncation runs to the maximum prediction length of 24 drafted tokens
    r = st.build_round(Table(), 5, 100, {}, st.Params(mode="asp"))
    assert r.tokens == list(range(5, 30)) and r.parents == [-1] + list(range(24)) and r.read_outs == 24


def test_tsp_marks_instead_of_truncating_and_hangs_the_second_token_off_the_previous_trunk_node():
    # uncertain at the LAST trunk position (max_draft 4): the alternative 59 to trunk token 9 is a
    # child of trunk token 8; the branch never meets the trunk again and grows to 5 nodes
    t = Table({(5, 6, 7, 8): (9, 59, 0.1),
               (5, 6, 7, 8, 59): (900, 0, 0.9), (5, 6, 7, 8, 59, 900): (901, 0, 0.9),
               (5, 6, 7, 8, 59, 900, 901): (902, 0, 0.9), (5, 6, 7, 8, 59, 900, 901, 902): (903, 0, 0.9)})
    r = st.build_round(t, 5, 0, {}, st.Params(max_draft=4))
    assert r.marks == [(4, 59, 0.1)]
    assert r.tokens == [5, 6, 7, 8, 9, 59, 900, 901, 902, 903]
    assert r.parents == [-1, 0, 1, 2, 3, 3, 5, 6, 7, 8]
    assert r.read_outs == 4 + 4                   # trunk + one per branch level; the full branch is not consulted
    # a second candidate equal to the trunk token would be no alternative: no branch
    t = Table({(5, 6, 7, 8): (9, 9, 0.1)})
    r = st.build_round(t, 5, 0, {}, st.Params(max_draft=4))
    assert r.tokens == [5, 6, 7, 8, 9] and len(r.marks) == 1


def test_branch_is_concatenated_to_the_trunk_at_the_corresponding_or_an_adjacent_position():
    # trunk 5 6 7 8 9 10 11; mark at position 2 (token 7, second candidate 70)
    base = {(5, 6): (7, 70, 0.2)}
    # the branch 70 continues with 9: position 3 holds 8, position 4 holds 9 -> joins one later and
    # takes the trunk's tail 9 10 11 without consulting the draft model again
    r = st.build_round(Table({**base, (5, 6, 70): (9, 0, 0.9)}), 5, 0, {}, st.Params(max_draft=6))
    assert r.tokens == [5, 6, 7, 8, 9, 10, 11, 70, 9, 10, 11]
    assert r.parents == [-1, 0, 1, 2, 3, 4, 5, 1, 7, 8, 9]
    assert r.read_outs == 6 + 1
    # continues with 8 = the corresponding position 3: tail 8 9 10 11, cut at 5 branch nodes
    r = st.build_round(Table({**base, (5, 6, 70): (8, 0, 0.9)}), 5, 0, {}, st.Params(max_draft=6))
    assert r.tokens[7:] == [70, 8, 9, 10, 11] and r.parents[7:] == [1, 7, 8, 9, 10] and r.read_outs == 7
    # continues with 7 = one position earlier: tail 7 8 9 10 (branch size 5 reached before 11)
    r = st.build_round(Table({**base, (5, 6, 70): (7, 0, 0.9)}), 5, 0, {}, st.Params(max_draft=6))
    assert r.tokens[7:] == [70, 7, 8, 9, 10] and r.read_outs == 7          # copied, not drafted
    # continues with 10 = two positions later: outside the window, an ordinary branch token
    r = st.build_round(Table({**base, (5, 6, 70): (10, 0, 0.9)}), 5, 0, {}, st.Params(max_draft=6))
    assert r.tokens[7:9] == [70, 10] and r.read_outs > 7


def test_recycling_reuses_the_kept_suffix_on_a_match_at_the_same_or_an_adjacent_position():
    prm = st.Params(mode="asp", max_draft=8)
    # root 5 at position 100; kept from the last round: 8 9 10 at positions 103..105.  The new trunk
    # 6 7 8 reaches 8 at position 103 = the corresponding position: 9 and 10 follow without drafting
    t = Table()
    r = st.build_round(t, 5, 100, {103: 8, 104: 9, 105: 10}, prm)
    assert r.tokens == list(range(5, 14)) and r.recycled == 2 and r.read_outs == 8 - 2
    assert (5, 6, 7, 8) not in t.calls and (5, 6, 7, 8, 9) not in t.calls      # tokens 9, 10 were not drafted
    assert (5, 6, 7, 8, 9, 10) in t.calls                                      # drafting resumes behind them
    # kept tokens one position later than where they are drafted now (pos + 1): 7 kept at 103, drafted at 102
    r = st.build_round(Table(), 5, 100, {103: 7, 104: 8, 105: 9}, prm)
    assert r.tokens == list(range(5, 14)) and r.recycled == 2
    # one position earlier (pos - 1): 7 kept at 101, drafted at 102
    r = st.build_round(Table(), 5, 100, {101: 7, 102: 8}, prm)
    assert r.recycled == 1 and r.tokens == list(range(5, 14))
    # two positions off: no reuse
    r = st.build_round(Table(), 5, 100, {104: 7, 105: 8}, prm)
    assert r.recycled == 0 and r.read_outs == 8
    # the kept suffix is spent by its first use: a hole ends the reuse, later kept tokens are ignored
    r = st.build_round(Table(), 5, 100, {102: 7, 103: 8, 105: 10}, prm)
    assert r.recycled == 1 and r.read_outs == 7
    # switched off
    r = st.build_round(Table(), 5, 100, {103: 8, 104: 9}, st.Params(mode="asp", max_draft=8, recycle=False))
    assert r.recycled == 0
    # the reuse respects the maximum prediction length
    r = st.build_round(Table(), 5, 100, {101: 6, 102: 7, 103: 8, 104: 9}, st.Params(mode="asp", max_draft=3))
    assert r.tokens == [5, 6, 7, 8] and r.recycled == 2


def test_node_cap_is_reached_in_the_middle_of_a_branch_level():
    # 24 drafted tokens, every even position uncertain: the 8 least confident of 12 marks get a branch
    entries = {}
    for k in range(1, 25):
        path = tuple(range(5, 5 + k))
        p = 0.01 * k if k % 2 == 0 else 0.9
        entries[path] = (path[-1] + 1, path[-1] + 500, p)
    r = st.build_round(Table(entries), 5, 0, {}, st.Params())
    assert len(r.marks) == 12 and len(r.tokens) == 64
    firsts = [i for i in range(25, 64) if r.parents[i] in r.trunk]
    assert firsts == list(range(25, 33))                                   # branch heads right behind the trunk
    # least confident = positions 2, 4, ..., 16, in trunk order; each head hangs off the node before its mark
    assert [r.parents[i] for i in firsts] == [r.trunk[k - 1] for k in range(2, 17, 2)]
    sizes = []
    for h in firsts:
        n, node = 1, h
        while True:
            kids = [i for i in range(64) if r.parents[i] == node]
            if not kids:
                break
            node, n = kids[0], n + 1
        sizes.append(n)
    assert sizes == [5, 5, 5, 5, 5, 5, 5, 4]                               # 25 + 8 * 5 = 65 > 64: the last branch stops short


def test_structure_invariants_on_random_tables():
    rng = np.random.default_rng(7)
    for trial in range(200):
        memo = {}

        def read_out(path):
            if path not in memo:
                t1, t2 = rng.choice(12, 2, replace=False)
                memo[path] = (int(t1), int(t2), float(rng.random()))
            return memo[path]

        prm = st.Params(mode="tsp" if trial % 2 else "asp", max_draft=int(rng.integers(1, 25)),
                        max_branches=int(rng.integers(1, 9)), branch_depth=int(rng.integers(1, 6)),
                        max_nodes=int(rng.integers(2, 65)))
        kept = {50 + int(q): int(rng.integers(12)) for q in rng.choice(30, 6, replace=False)}
        r = st.build_round(read_out, 3, 50, kept, prm)
        n = len(r.tokens)
        assert 1 <= n <= prm.max_nodes and len(r.trunk) - 1 <= prm.max_draft
        assert r.parents[0] == -1 and all(0 <= r.parents[i] < i for i in range(1, n))
        assert r.trunk == list(range(len(r.trunk)))                         # trunk first, in order
        for i in range(n):                                                  # alternatives differ from their siblings
            kids = [r.tokens[j] for j in range(n) if r.parents[j] == i]
            assert len(kids) <= 2 and len(set(kids)) == len(kids)
        assert len(st.path_set(r.tokens, r.parents)) == n                   # no path twice
        if prm.mode == "asp":
            assert n == len(r.trunk)


def test_kept_suffix_after_a_round():
    # trunk tokens t0..t6 at positions 40..46; 3 nodes accepted (positions 40..42), the target's own
    # token takes position 43: positions 44.. are kept
    assert st.kept_after([9, 1, 2, 3, 4, 5, 6], 40, 3) == {44: 4, 45: 5, 46: 6}
    assert st.kept_after([9, 1, 2], 40, 3) == {}
    assert st.kept_after([9, 1, 2, 3], 40, 1) == {42: 2, 43: 3}
