"""Pins of the oracle's step_rope (rotary position embedding at the step's positions) against
things that are not the oracle: the digits printed in Fig. 2(b), invariants of a rotation, the
property rotary embeddings exist for (a score depends on the distance of the two positions only), a
quarter turn written out by hand, and complex multiplication."""
import numpy as np
import pytest

from oracle import la_oracle as orc
from paper_2402_02057_amd import workloads as wl


def tables(max_pos, d):
    return wl.rope_tables(max_pos, d)


def test_positions_are_the_digits_of_figure_2b():
    """W = 5, N = 4, G = 2: the current token 0; the three window levels 1-5, 2-6, 3-7; the
    candidates' tokens 1, 2, 3 (Fig. 2(b)).  A table whose 'angle' encodes the position shows which
    row the oracle reads."""
    W, N, G, d = 5, 4, 2, 2
    digits = [0] + [1, 2, 3, 4, 5] + [2, 3, 4, 5, 6] + [3, 4, 5, 6, 7] + [1, 2, 3] * 2
    T = len(digits)
    P = 10
    cos = np.arange(40, dtype=np.float64)[:, None] * 1.0     # not a cosine: a label
    sin = np.zeros((40, 1))
    q = np.ones((T, 1, d))
    rq, rk = orc.step_rope(q, q, cos, sin, P, W, N, G)
    assert rq[:, 0, 0].tolist() == [float(P + x) for x in digits]
    assert rk[:, 0, 1].tolist() == [float(P + x) for x in digits]


@pytest.mark.parametrize("interleaved", [False, True])
def test_rotation_keeps_pair_norms_and_is_the_identity_at_position_zero(interleaved):
    W, N, G, d, H = 3, 3, 2, 16, 2
    T = 1 + (W + G) * (N - 1)
    rng = np.random.default_rng(0)
    q, k = rng.standard_normal((T, H, d)), rng.standard_normal((T, 1, d))
    cos, sin = tables(64, d)
    rq, rk = orc.step_rope(q, k, cos, sin, 7, W, N, G, interleaved)
    pairs = (lambda x: (x[..., 0::2], x[..., 1::2])) if interleaved else (lambda x: (x[..., :d // 2], x[..., d // 2:]))
    for x, y in ((q, rq), (k, rk)):
        a, b = pairs(x)
        ra, rb = pairs(y)
        np.testing.assert_allclose(ra ** 2 + rb ** 2, a ** 2 + b ** 2, rtol=1e-6)   # (tables are fp32)
    rq0, _ = orc.step_rope(q, k, cos, sin, 0, W, N, G, interleaved)
    np.testing.assert_array_equal(rq0[0], q[0])                 # row 0 at P = 0: angle zero
    assert not np.allclose(rq0[1], q[1])


@pytest.mark.parametrize("interleaved", [False, True])
def test_scores_depend_on_the_distance_only(interleaved):
    """<rope(q, m), rope(k, n)> is a function of m - n: shifting the prefix length moves every
    row by the same amount and must leave all scores between step rows unchanged."""
    W, N, G, d = 4, 4, 3, 32
    T = 1 + (W + G) * (N - 1)
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((T, 1, d)), rng.standard_normal((T, 1, d))
    i = np.arange(d // 2)
    angle = np.arange(400)[:, None] * 10000.0 ** (-2.0 * i / d)[None, :]
    cos, sin = np.cos(angle), np.sin(angle)                     # fp64 tables: the identity is exact up to rounding
    scores = []
    for P in (0, 5, 300):
        rq, rk = orc.step_rope(q, k, cos, sin, P, W, N, G, interleaved)
        scores.append(rq[:, 0] @ rk[:, 0].T)
    np.testing.assert_allclose(scores[1], scores[0], atol=1e-9)
    np.testing.assert_allclose(scores[2], scores[0], atol=1e-9)
    # and they do depend on it: rows at different positions see a different score than unrotated
    assert not np.allclose(scores[0], q[:, 0] @ k[:, 0].T)


def test_quarter_turn_by_hand():
    """All angles pi/2 at position 1, zero at position 0: (a, b) -> (-b, a) for the rows at
    relative position 1, nothing for row 0; both pairings written out."""
    W, N, G, d = 1, 2, 1, 4
    cos = np.array([[1.0, 1.0], [0.0, 0.0]])
    sin = np.array([[0.0, 0.0], [1.0, 1.0]])
    x = np.array([1.0, 2.0, 3.0, 4.0])
    q = np.tile(x, (3, 1, 1))                                   # rows: current (0), lookahead (1), candidate (1)
    rq, _ = orc.step_rope(q, q, cos, sin, 0, W, N, G, interleaved=False)
    assert rq[0, 0].tolist() == [1.0, 2.0, 3.0, 4.0]
    assert rq[1, 0].tolist() == [-3.0, -4.0, 1.0, 2.0]          # pairs (x0, x2), (x1, x3)
    assert rq[2, 0].tolist() == [-3.0, -4.0, 1.0, 2.0]
    rq, _ = orc.step_rope(q, q, cos, sin, 0, W, N, G, interleaved=True)
    assert rq[1, 0].tolist() == [-2.0, 1.0, -4.0, 3.0]          # pairs (x0, x1), (x2, x3)


@pytest.mark.parametrize("interleaved", [False, True])
def test_equals_complex_multiplication(interleaved):
    W, N, G, d, H = 5, 4, 2, 8, 3
    T = 1 + (W + G) * (N - 1)
    rng = np.random.default_rng(2)
    q, k = rng.standard_normal((T, H, d)), rng.standard_normal((T, 2, d))
    cos, sin = tables(64, d)
    P = 11
    rq, rk = orc.step_rope(q, k, cos, sin, P, W, N, G, interleaved)
    pos = np.array([P + orc.position(r, W, N, G) for r in range(T)])
    turn = (cos[pos].astype(np.float64) + 1j * sin[pos].astype(np.float64))[:, None, :]
    for x, y in ((q, rq), (k, rk)):
        z = (x[..., 0::2] + 1j * x[..., 1::2]) if interleaved else (x[..., :d // 2] + 1j * x[..., d // 2:])
        w = z * turn
        want = np.empty_like(x)
        if interleaved:
            want[..., 0::2], want[..., 1::2] = w.real, w.imag
        else:
            want[..., :d // 2], want[..., d // 2:] = w.real, w.imag
        np.testing.assert_allclose(y, want, atol=1e-12)


def test_the_two_pairings_differ_by_a_permutation():
    W, N, G, d = 2, 3, 1, 8
    T = 1 + (W + G) * (N - 1)
    rng = np.random.default_rng(3)
    q = rng.standard_normal((T, 2, d))
    cos, sin = tables(32, d)
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])      # interleaved order -> halves order
    a, _ = orc.step_rope(q, q, cos, sin, 4, W, N, G, interleaved=True)
    b, _ = orc.step_rope(q[..., perm], q[..., perm], cos, sin, 4, W, N, G, interleaved=False)
    np.testing.assert_array_equal(a[..., perm], b)


def test_tables_are_the_published_frequencies():
    cos, sin = wl.rope_tables(8, 4, base=100.0)
    assert cos.dtype == np.float32 and cos.shape == (8, 2)
    np.testing.assert_allclose(cos[3], [np.cos(3.0), np.cos(3.0 / 10.0)], rtol=1e-6)
    np.testing.assert_allclose(sin[5], [np.sin(5.0), np.sin(0.5)], rtol=1e-6)
