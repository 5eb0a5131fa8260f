"""Pins of the oracle's lookahead / verification mask (Sec. 3.3, Fig. 2(b), Algorithm 2).

The mask rule inside oracle/la_oracle.c is a closed-form test on (branch, level, column).
Here it is checked against formulations that share nothing with it: a parent-pointer walk
(each step token has exactly one predecessor on its trajectory), the position-chain
invariant that the causal principle implies, a closed-form count, and the paper's own
worked example.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import la_oracle as orc

SMALL = [(W, N, G) for W in range(0, 6) for N in range(2, 6) for G in range(0, 4)]
PAPER = [(15, 5, 15), (10, 5, 10), (7, 5, 7), (5, 4, 2), (5, 3, 2), (30, 5, 30)]


def row_of_lookahead(l, j, W):
    return 1 + l * W + j


def row_of_candidate(g, k, W, N):
    return 1 + W * (N - 1) + g * (N - 1) + k


def parent(r, W, N, G):
    """Predecessor of step token r on its own trajectory, None for the current token.

    Algorithm 2 conditions a new window token on its column in the later levels and on the
    oldest level up to its column; read backwards, the token before (l, j) is (l-1, j) and
    the token before (0, j) is (0, j-1), ending at the current token.  A candidate token
    follows the previous token of the same n-gram (Sec. 3.2), the first one follows the
    current token.
    """
    if r == 0:
        return None
    nl = W * (N - 1)
    if r <= nl:
        l, j = divmod(r - 1, W)
        if l > 0:
            return row_of_lookahead(l - 1, j, W)
        return row_of_lookahead(0, j - 1, W) if j > 0 else 0
    g, k = divmod(r - 1 - nl, N - 1)
    return row_of_candidate(g, k - 1, W, N) if k > 0 else 0


def ancestors_mask(W, N, G):
    T = 1 + (W + G) * (N - 1)
    m = np.zeros((T, T), dtype=bool)
    for r in range(T):
        c = r
        while c is not None:
            m[r, c] = True
            c = parent(c, W, N, G)
    return m


@pytest.mark.parametrize("W,N,G", SMALL + PAPER)
def test_mask_equals_trajectory_ancestors(W, N, G):
    assert orc.num_rows(W, N, G) == 1 + (W + G) * (N - 1)
    np.testing.assert_array_equal(orc.step_mask(W, N, G), ancestors_mask(W, N, G))


@pytest.mark.parametrize("W,N,G", SMALL + PAPER)
def test_position_chain_invariant(W, N, G):
    """A row at relative position p sees exactly one step token at each position 0..p."""
    m = orc.step_mask(W, N, G)
    T = m.shape[0]
    pos = np.array([orc.position(r, W, N, G) for r in range(T)])
    for r in range(T):
        seen = sorted(pos[m[r]])
        assert seen == list(range(pos[r] + 1)), (r, seen)
        # nothing at a larger position is ever visible (causal principle, Sec. 2)
        assert not np.any(m[r] & (pos > pos[r]))


def test_positions_follow_fig2b():
    # W = 5, N = 4 window: level l column j carries the digit 1 + l + j; candidates 1..N-1
    W, N, G = 5, 4, 2
    assert orc.position(0, W, N, G) == 0
    for l in range(N - 1):
        for j in range(W):
            assert orc.position(row_of_lookahead(l, j, W), W, N, G) == 1 + l + j
    for g in range(G):
        for k in range(N - 1):
            assert orc.position(row_of_candidate(g, k, W, N), W, N, G) == 1 + k


def visible_pairs_closed_form(W, N, G):
    n1 = N - 1
    # current token: itself.  level 0, column j: current + j + 1 tokens.  level l >= 1,
    # column j: current + (j + 1) of level 0 + l of its own column.  candidate token k:
    # current + k + 1.
    level0 = sum(1 + j + 1 for j in range(W))
    upper = sum(1 + (j + 1) + l for l in range(1, n1) for j in range(W))
    cands = G * sum(1 + k + 1 for k in range(n1))
    return 1 + level0 + upper + cands


@pytest.mark.parametrize("W,N,G,count", [(4, 3, 2, 43), (5, 4, 2, 94), (15, 5, 15, 841),
                                           (10, 5, 10, 461), (7, 5, 7, 281)])
def test_visible_pair_counts(W, N, G, count):
    assert visible_pairs_closed_form(W, N, G) == count
    assert int(orc.step_mask(W, N, G).sum()) == count


@pytest.mark.parametrize("W,N,G", SMALL)
def test_visible_pair_count_formula_everywhere(W, N, G):
    assert int(orc.step_mask(W, N, G).sum()) == visible_pairs_closed_form(W, N, G)


def test_paper_worked_example(golden_dir):
    path = os.path.join(golden_dir, "sec3_3_visibility_example.txt")
    cases = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        shape, row, vis = [x.strip() for x in line.split("|")]
        W, N, G = [int(x) for x in shape.split()]
        l, j = [int(x) for x in row.split(",")]
        want = set()
        for tok in vis.split():
            if tok == "cur":
                want.add(0)
            else:
                a, b = [int(x) for x in tok.split(",")]
                want.add(row_of_lookahead(a, b, W))
        m = orc.step_mask(W, N, G)
        got = set(np.nonzero(m[row_of_lookahead(l, j, W)])[0].tolist())
        assert got == want, (line, sorted(got))
        cases += 1
    assert cases == 3


@pytest.mark.parametrize("W,N,G", [(5, 4, 2), (4, 3, 3), (15, 5, 15)])
def test_branches_do_not_see_each_other(W, N, G):
    m = orc.step_mask(W, N, G)
    nl = W * (N - 1)
    look = slice(1, 1 + nl)
    cand = slice(1 + nl, None)
    assert not m[look, cand].any() and not m[cand, look].any()
    assert not m[0, 1:].any() and m[:, 0].all()
    # candidates are block diagonal with lower-triangular blocks
    n1 = N - 1
    blk = m[cand, cand]
    want = np.kron(np.eye(G, dtype=bool), np.tril(np.ones((n1, n1), dtype=bool)))
    np.testing.assert_array_equal(blk, want)
    # disjoint columns above the oldest level do not interact (Sec. 3.4)
    for l1, l2 in itertools.product(range(1, N - 1), repeat=2):
        for j1 in range(W):
            for j2 in range(W):
                if j1 != j2:
                    assert not m[row_of_lookahead(l1, j1, W), row_of_lookahead(l2, j2, W)]
