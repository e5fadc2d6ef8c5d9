"""Pins for the oracle's majority vote (no GPU): the paper's worked example, brute force over
an explicitly built token tree, and special cases."""
import itertools
import os

import numpy as np
import pytest

from oracle import minions_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "vote_worked_example.txt")


def _golden_cases():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w, d, v, s = [f.strip() for f in line.split("|")]
        cases.append(([float(x) for x in w.split()],
                      [[int(t) for t in row.split()] for row in d.split(";")],
                      [int(t) for t in v.split()], int(s)))
    return cases


@pytest.mark.parametrize("w,drafts,voted,ssm", _golden_cases())
def test_worked_example_section_3_2(w, drafts, voted, ssm):
    got_v, got_s = orc.vote_tree(drafts, len(voted), w)
    assert got_v == voted and got_s == ssm


# ---- an independent formulation: build the explicit tree, weight the nodes, walk it ----

class _Node:
    def __init__(self, tok):
        self.tok, self.weight, self.children, self.first, self.members = tok, 0.0, [], None, []


def _tree_reference(drafts, k, w):
    root = _Node(None)
    for j, d in enumerate(drafts):                 # insert every draft as a root-to-leaf branch
        node = root
        for t in range(k):
            nxt = next((c for c in node.children if c.tok == d[t]), None)
            if nxt is None:
                nxt = _Node(d[t])
                nxt.first = j
                node.children.append(nxt)
            nxt.members.append(j)
            node = nxt
    def weigh(node):
        node.weight = np.float32(0)
        for j in sorted(node.members):
            node.weight = np.float32(node.weight + np.float32(w[j]))
        for c in node.children:
            weigh(c)
    for c in root.children:
        weigh(c)
    out, node = [], root
    for _ in range(k):
        best = max(node.children, key=lambda c: (c.weight, -c.first))
        out.append(best.tok)
        node = best
    return out, (min(node.members) if k > 0 else 0)


@pytest.mark.parametrize("V,n,k", [(2, 3, 3), (3, 3, 2), (3, 4, 2), (2, 4, 3), (3, 2, 3)])
def test_bruteforce_all_draft_sets(V, n, k):
    seqs = list(itertools.product(range(V), repeat=k))
    weight_sets = [[1.0] * n, [float(i + 1) for i in range(n)], [float(n - i) for i in range(n)],
                   [0.5, 0.25, 0.75, 0.5][:n]]
    count = 0
    for combo in itertools.product(seqs, repeat=n):
        for w in weight_sets:
            want = _tree_reference(combo, k, w)
            got = orc.vote_tree(combo, k, w)
            assert got == want, (combo, w)
            count += 1
    assert count > 100


def test_random_against_tree_reference():
    rng = np.random.default_rng(7)
    for _ in range(300):
        n, k, V = int(rng.integers(1, 7)), int(rng.integers(1, 9)), int(rng.integers(2, 5))
        d = rng.integers(0, V, size=(n, k)).tolist()
        w = rng.random(n).astype(np.float32).tolist()
        assert orc.vote_tree(d, k, w) == _tree_reference(d, k, w)


def test_special_cases():
    rng = np.random.default_rng(3)
    d = rng.integers(0, 50, size=(1, 6)).tolist()
    assert orc.vote_tree(d, 6, [0.3]) == (d[0], 0)                    # one SSM: identity
    same = [d[0]] * 4
    assert orc.vote_tree(same, 6, [1, 2, 3, 4]) == (d[0], 0)          # all equal
    a, b = [1, 2, 3], [4, 5, 6]
    assert orc.vote_tree([a, b], 3, [1, 1]) == (a, 0)                 # two SSMs, unit weights: draft 0
    assert orc.vote_tree([a, b], 3, [1, 2]) == (b, 1)
    assert orc.vote_tree([a, b, b], 0, [1, 1, 1]) == ([], 0)          # k = 0: nothing to vote on


def test_output_is_one_ssms_whole_output():
    # section 3.2: the majority-approved output is the output of exactly one SSM (voted_SSM)
    rng = np.random.default_rng(11)
    for _ in range(200):
        n, k = int(rng.integers(1, 6)), int(rng.integers(1, 10))
        d = rng.integers(0, 3, size=(n, k))
        w = (rng.random(n) + 0.1).astype(np.float32)
        v, s = orc.vote_tree(d, k, w)
        assert list(d[s]) == v
        assert all(list(d[j]) != v for j in range(s))                 # and s is the lowest such index


def test_tree_and_column_modes():
    # they differ when the column vote splices drafts
    d = [[1, 2], [1, 3], [4, 3]]
    assert orc.vote_tree(d, 2, [1, 1, 1]) == ([1, 2], 0)
    assert orc.vote_column(d, 2, [1, 1, 1]) == ([1, 3], 1)
    d2 = [[1, 2], [5, 3], [4, 3]]
    assert orc.vote_column(d2, 2, [1, 1, 1]) == ([1, 3], -1)           # spliced: no single SSM
    # a strict (weighted) majority on the whole sequence: both modes agree
    rng = np.random.default_rng(5)
    for _ in range(100):
        k = int(rng.integers(1, 7))
        major = rng.integers(0, 9, size=k).tolist()
        others = rng.integers(0, 9, size=(2, k)).tolist()
        d = [major, others[0], major, others[1], major]
        w = [1, 1, 1, 1, 1]
        assert orc.vote_tree(d, k, w)[0] == major
        assert orc.vote_column(d, k, w)[0] == major


def test_batch_padding_and_ragged_lengths():
    d = np.array([[[1, 2, 3], [1, 2, 4]], [[7, 8, -1], [9, 8, -1]]], np.int32)
    voted, ssm = orc.vote_batch(d, [3, 1], [1.0, 2.0])
    assert voted.tolist() == [[1, 2, 4], [9, -1, -1]] and ssm.tolist() == [1, 1]


def test_fp32_weight_sum_order_is_part_of_the_contract():
    # 2^24 + 1 + 1 in fp32, summed left to right, stays 2^24; a lone 2^24+2 beats it
    big = float(2 ** 24)
    d = [[1], [1], [1], [2]]
    w = [big, 1.0, 1.0, big + 2.0]
    assert orc.vote_tree(d, 1, w) == ([2], 3)
