"""Pins of the oracle's greedy verification reduction (Sec. 2 guess-and-verify, Algorithm 3)."""
import itertools

import numpy as np
import pytest

from oracle import la_oracle as orc
from paper_2402_02057_amd import workloads as wl


def logits_with_argmax(am, V, rng):
    """fp32 rows whose unique maximum sits at the given indices."""
    am = np.asarray(am)
    x = rng.standard_normal(size=am.shape + (V,)).astype(np.float32)
    np.put_along_axis(x, am[..., None], 50.0, axis=-1)
    return x


@pytest.mark.parametrize("V,N,G", [(V, N, G) for V in (2, 3) for N in (2, 3, 4) for G in (1, 2)]
                         + [(4, 3, 1), (2, 2, 3)])
def test_accept_length_exhaustive(V, N, G):
    """Every candidate tuple against every argmax tuple: accept_len is the longest common prefix."""
    rng = np.random.default_rng(V * 100 + N * 10 + G)
    n1 = N - 1
    tuples = list(itertools.product(range(V), repeat=n1))
    combos = list(itertools.product(tuples, repeat=G))
    if len(combos) > 300:
        combos = [combos[i] for i in rng.choice(len(combos), 300, replace=False)]
    for cands in combos:
        for ams in itertools.product(tuples, repeat=G) if len(tuples) ** G <= 64 else \
                [tuple(tuples[i] for i in rng.integers(0, len(tuples), G)) for _ in range(40)]:
            cand = np.array(cands, dtype=np.int32).reshape(G, n1)
            am = np.array(ams, dtype=np.int32).reshape(G, n1)
            logits = logits_with_argmax(am, V, rng)
            alen, acc = orc.verify(logits, cand, G, N, V)
            np.testing.assert_array_equal(acc, am)
            for g in range(G):
                L = 0
                for a, b in zip(cands[g], ams[g]):
                    if a != b:
                        break
                    L += 1
                assert alen[g] == L


@pytest.mark.parametrize("V", [1, 2, 5, 63, 64, 65, 255, 1000, 32000, 32016])
def test_argmax_matches_library_first_occurrence(V):
    rng = np.random.default_rng(V)
    G, N = 3, 4
    logits = rng.standard_normal(size=(G, N - 1, V)).astype(np.float32)
    # deliberate ties: quantise half of the rows so the maximum repeats
    logits[1] = np.round(logits[1])
    logits[2, 0] = 0.0
    cand = rng.integers(0, V, size=(G, N - 1)).astype(np.int32)
    alen, acc = orc.verify(logits, cand, G, N, V)
    np.testing.assert_array_equal(acc, np.argmax(logits, axis=-1).astype(np.int32))
    assert acc[2, 0] == 0


def test_negative_and_extreme_values():
    V = 17
    logits = np.full((1, 2, V), -np.float32(3.0e38), dtype=np.float32)
    logits[0, 0, 9] = -1.0e-30
    logits[0, 1, 16] = -np.float32(2.9e38)
    cand = np.array([[9, 16]], dtype=np.int32)
    alen, acc = orc.verify(logits, cand, 1, 3, V)
    assert acc.tolist() == [[9, 16]] and alen.tolist() == [2]


def test_planted_workload_lengths():
    for s in (wl.LLAMA2_7B, wl.LLAMA2_13B, wl.LLAMA2_70B, wl.ragged_shape(0, 30)):
        logits, cand, lens = wl.verify_inputs(s)
        alen, acc = orc.verify(logits, cand, s.G, s.N, s.V)
        np.testing.assert_array_equal(alen, lens)
        # every accept length 0..N-1 occurs when G >= N
        if s.G >= s.N:
            assert set(lens.tolist()) == set(range(s.N))
        # a match counter (instead of the leading run) would differ somewhere
        matches = (acc == cand).sum(axis=1)
        assert np.any(matches != alen)


def toy_model_argmax(prefix, V):
    """A deterministic stand-in for the model: greedy next token as a function of the prefix."""
    h = 1469598103934665603
    for t in prefix:
        h = ((h ^ (int(t) + 1)) * 1099511628211) % (1 << 64)
    return (h >> 20) % V


@pytest.mark.parametrize("seed", range(40))
def test_reduction_agrees_with_algorithm3(seed):
    """With distributions that depend only on the token prefix (as a real model's do), the
    tokens Algorithm 3 returns are the best candidate's accepted run plus the model's own
    token at the first mismatch (or the bonus token after a full match)."""
    rng = np.random.default_rng(seed)
    V, N, G = 3, int(rng.integers(2, 6)), int(rng.integers(1, 6))
    n1 = N - 1
    last = int(rng.integers(0, V))
    cands = [tuple(int(t) for t in rng.integers(0, V, n1)) for _ in range(G)]
    # bias some candidates towards the true continuation so long accepts occur
    truth, pre = [], [last]
    for _ in range(N):
        truth.append(toy_model_argmax(pre, V))
        pre.append(truth[-1])
    for g in range(G):
        if rng.random() < 0.5:
            keep = int(rng.integers(0, n1 + 1))
            cands[g] = tuple(truth[:keep]) + cands[g][keep:]
    dist = [[toy_model_argmax([last] + list(c[:i]), V) for i in range(N)] for c in cands]
    out = orc.greedy_verification(cands, dist)

    am = np.array([d[:n1] for d in dist], dtype=np.int32)
    logits = logits_with_argmax(am, V, rng)
    alen, acc = orc.verify(logits, np.array(cands, dtype=np.int32).reshape(G, n1), G, N, V)
    np.testing.assert_array_equal(acc, am)
    best = int(np.argmax(alen))          # lowest g among the longest
    L = int(alen[best])
    assert 1 <= len(out) <= N
    assert len(out) - 1 == L
    assert tuple(out[:L]) == cands[best][:L]
    assert out[L] == dist[best][L]
    # and the output is what plain greedy autoregressive decoding would have produced
    assert out == truth[:L + 1]


def test_zero_candidates_is_a_noop():
    alen, acc = orc.verify(np.zeros((0, 3, 8), np.float32), np.zeros((0, 3), np.int32), 0, 4, 8)
    assert alen.shape == (0,) and acc.shape == (0, 3)
