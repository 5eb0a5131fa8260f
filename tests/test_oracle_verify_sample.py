"""Pins of the oracle's sampling verification (Algorithm 4).

The paper's claim (Theorem A, App. B) is that every token the procedure emits follows the model's
own distribution given the tokens before it.  The tests below (i) compute, independently of the
oracle, the exact law of the token emitted at every node of Algorithm 4's decision tree and check
that it IS the model's distribution (so the reading of the algorithm is the one the theorem is
about), (ii) check the oracle's outputs against that exact tree by seeded Monte Carlo, and (iii)
check special cases with library routines.
"""
import math

import numpy as np
import pytest
import scipy.special

from oracle import la_oracle as orc


def toy_logits(prefix, V):
    """A deterministic stand-in for the model: logits as a function of the token prefix."""
    h = 1469598103934665603
    for t in prefix:
        h = ((h ^ (int(t) + 1)) * 1099511628211) % (1 << 64)
    return np.random.default_rng(h).standard_normal(V).astype(np.float32) * 1.5


def model_dist(prefix, V, temperature):
    return scipy.special.softmax(toy_logits(prefix, V).astype(np.float64) / temperature)


def inputs_for(last, cands, V):
    """logits_cur, logits_cand for candidates (tuples of N-1 tokens) continuing the token `last`."""
    G, n1 = len(cands), len(cands[0]) if cands else 1
    cur = toy_logits([last], V)
    cnd = np.zeros((G, n1, V), dtype=np.float32)
    for g, c in enumerate(cands):
        for k in range(n1):
            cnd[g, k] = toy_logits([last] + list(c[:k + 1]), V)
    return cur, cnd


def exact_tree(last, cands, V, temperature):
    """{output tuple: probability} of Algorithm 4, by walking its decision tree with exact
    branch probabilities, and at every position the law of the emitted token given the accepted
    prefix (a list of (prefix, distribution) pairs to compare with the model)."""
    n1 = len(cands[0])
    out, emitted = {}, []

    def walk(i, alive, prefix, prob):
        if i == n1:
            P = model_dist([last] + prefix, V, temperature)
            for v in range(V):
                out[tuple(prefix + [v])] = out.get(tuple(prefix + [v]), 0.0) + prob * P[v]
            return
        P = model_dist([last] + prefix, V, temperature).copy()
        law = np.zeros(V)
        reach = 1.0                      # probability of getting to the j-th test of this position
        for j, g in enumerate(alive):
            s = cands[g][i]
            a = P[s]
            law[s] += reach * a
            if a > 0:
                walk(i + 1, [k for k in alive[j:] if cands[k][i] == s], prefix + [s], prob * reach * a)
            reach *= 1.0 - a
            P[s] = 0.0
            if P.sum() > 0:
                P = P / P.sum()
        law += reach * P
        for v in range(V):
            if reach * P[v] > 0:
                out[tuple(prefix + [v])] = out.get(tuple(prefix + [v]), 0.0) + prob * reach * P[v]
        emitted.append((list(prefix), law))

    walk(0, list(range(len(cands))), [], 1.0)
    return out, emitted


CASES = [
    (3, [(0,), (1,)]),
    (3, [(2,), (2,), (0,)]),                      # a repeated candidate token
    (4, [(1, 2), (1, 3), (0, 0)]),
    (3, [(0, 1, 2), (0, 1, 1), (0, 2, 2), (1, 0, 0)]),
    (5, [(4, 4), (3, 1)]),
]


@pytest.mark.parametrize("V,cands", CASES)
@pytest.mark.parametrize("temperature", [1.0, 0.5])
def test_every_emitted_token_follows_the_model(V, cands, temperature):
    """Theorem A on the reading implemented here: at every node of the decision tree the token
    emitted (accepted candidate token or residual sample) has the model's distribution."""
    out, emitted = exact_tree(0, cands, V, temperature)
    assert abs(sum(out.values()) - 1.0) < 1e-12
    assert emitted
    for prefix, law in emitted:
        np.testing.assert_allclose(law, model_dist([0] + prefix, V, temperature), atol=1e-12)


@pytest.mark.parametrize("V,cands", CASES)
def test_oracle_samples_follow_the_exact_tree(V, cands):
    """Seeded Monte Carlo through the oracle against the exact law of the whole output."""
    temperature = 0.8
    G, n1 = len(cands), len(cands[0])
    N = n1 + 1
    cur, cnd = inputs_for(0, cands, V)
    cand = np.array(cands, dtype=np.int32).reshape(G, n1)
    want, _ = exact_tree(0, cands, V, temperature)
    rng = np.random.default_rng(V * 1000 + G)
    n = 60000
    u_test = rng.random((n, n1, G), dtype=np.float32)
    u_final = rng.random(n, dtype=np.float32)
    counts = {}
    for t in range(n):
        o = tuple(orc.verify_sample(cur, cnd, cand, u_test[t], u_final[t], temperature, N, G, V))
        counts[o] = counts.get(o, 0) + 1
    assert set(counts) <= {k for k, p in want.items() if p > 0}
    for k, p in want.items():
        sigma = math.sqrt(p * (1 - p) / n)
        assert abs(counts.get(k, 0) / n - p) <= 5 * sigma + 1e-4, (k, counts.get(k, 0) / n, p)


def test_decisions_follow_the_draws_exactly():
    """One position, two candidates: the outcome as a function of the draws, region by region."""
    V, N, G = 4, 2, 2
    cur = np.log(np.array([0.1, 0.2, 0.3, 0.4])).astype(np.float32)
    cand = np.array([[3], [1]], dtype=np.int32)
    cnd = np.zeros((G, 1, V), dtype=np.float32)
    cnd[0, 0] = np.log(np.array([0.7, 0.1, 0.1, 0.1]))     # after accepting token 3
    cnd[1, 0] = np.log(np.array([0.1, 0.1, 0.1, 0.7]))     # after accepting token 1

    def run(r0, r1, u):
        return orc.verify_sample(cur, cnd, cand, np.array([[r0, r1]], np.float32), u, 1.0, N, G, V)
    # first candidate accepted (P(3) = 0.4); bonus token from its own next distribution
    assert run(0.39, 0.9, 0.65) == [3, 0] and run(0.39, 0.9, 0.75) == [3, 1]
    # rejected; residual is (1/6, 2/6, 3/6, 0): second candidate (token 1) accepted below 1/3
    assert run(0.41, 0.33, 0.95) == [1, 3] and run(0.41, 0.33, 0.05) == [1, 0]
    # both rejected; residual (1/4, 0, 3/4, 0)
    assert run(0.41, 0.34, 0.2) == [0] and run(0.41, 0.34, 0.3) == [2] and run(0.99, 0.99, 0.999) == [2]


def test_zero_temperature_limit_is_greedy_verification():
    """Sharp distributions of a prefix-deterministic model: whatever the draws, the result is
    Algorithm 3's (and plain greedy decoding's)."""
    rng = np.random.default_rng(11)

    def sharp_logits(prefix, V):
        x = toy_logits(prefix, V)
        x[int(np.argmax(x))] += 30.0
        return x
    for _ in range(40):
        V, N, G = 7, int(rng.integers(2, 6)), int(rng.integers(1, 5))
        n1 = N - 1
        last = int(rng.integers(0, V))
        truth, pre = [], [last]
        for _ in range(N):
            truth.append(int(np.argmax(sharp_logits(pre, V))))
            pre.append(truth[-1])
        cands = rng.integers(0, V, size=(G, n1)).astype(np.int32)
        for g in range(G):
            keep = int(rng.integers(0, N))
            cands[g, :keep] = truth[:keep]
        cur = sharp_logits([last], V)
        cnd = np.stack([np.stack([sharp_logits([last] + cands[g, :k + 1].tolist(), V) for k in range(n1)])
                        for g in range(G)])
        want, _, _, _ = orc.verify_step(cur, np.zeros((0, V), np.float32), cnd, cands, 0, N, G, V)
        assert want == truth[:len(want)]
        u = rng.random((n1, G), dtype=np.float32) * 0.98 + 0.01
        got = orc.verify_sample(cur, cnd, cands, u, float(rng.random() * 0.98 + 0.01), 0.05, N, G, V)
        assert got == want


@pytest.mark.parametrize("V", [1, 2, 17, 1000, 32000])
def test_no_candidates_is_inverse_cdf_sampling_of_the_library_softmax(V):
    rng = np.random.default_rng(V)
    cur = (rng.standard_normal(V) * 2).astype(np.float32)
    cdf = np.cumsum(scipy.special.softmax(cur.astype(np.float64) / 0.7))
    for u in [0.0, 0.1, 0.5, 0.9, 0.999] + rng.random(20).tolist():
        u = float(np.float32(u))
        got = orc.verify_sample(cur, np.zeros((0, 1, V), np.float32), np.zeros((0, 1), np.int32),
                                np.zeros((1, 0), np.float32), u, 0.7, 2, 0, V)
        want = min(int(np.searchsorted(cdf, u, side="right")), V - 1)
        # (a draw within rounding of a CDF step may fall on either side)
        assert len(got) == 1 and (got[0] == want or abs(cdf[min(got[0], want)] - u) < 1e-9)


def test_a_rejected_token_is_never_accepted_later():
    V, N, G = 3, 2, 3
    cur = np.log(np.array([0.5, 0.3, 0.2])).astype(np.float32)
    cand = np.array([[0], [0], [1]], dtype=np.int32)
    cnd = np.zeros((G, 1, V), dtype=np.float32)
    # token 0 rejected by the first draw; the second candidate proposes it again: P = 0 now
    got = orc.verify_sample(cur, cnd, cand, np.array([[0.6, 0.0, 0.59]], np.float32), 0.5, 1.0, N, G, V)
    assert got[0] == 1            # third candidate: residual P(1) = 0.6 > 0.59
    got = orc.verify_sample(cur, cnd, cand, np.array([[0.6, 0.0, 0.61]], np.float32), 0.5, 1.0, N, G, V)
    assert got == [2]             # all rejected; residual is (0, 0, 1)


def test_a_token_outside_the_vocabulary_has_probability_zero():
    """A candidate token outside 0 .. V-1 (a padding id) spends its draw, is never accepted and
    rules nothing out: the walk equals the one over the other candidates with the draws they saw."""
    rng = np.random.default_rng(11)
    V, N = 7, 3
    cur = (rng.standard_normal(V) * 2).astype(np.float32)
    for bad in (-1, V, V + 5, -2**31, 2**31 - 1):
        for trial in range(40):
            tok = rng.integers(0, V, size=(1, N - 1)).astype(np.int32)
            cnd1 = (rng.standard_normal((1, N - 1, V)) * 2).astype(np.float32)
            u = rng.random((N - 1, 2), dtype=np.float32)
            u_final = float(rng.random())
            # the bad candidate first: it uses up draw [0][0]; the good one is examined second
            cand2 = np.concatenate([np.full((1, N - 1), bad, np.int32), tok])
            cnd2 = np.concatenate([np.zeros_like(cnd1), cnd1])
            got = orc.verify_sample(cur, cnd2, cand2, u, u_final, 0.8, N, 2, V)
            # position 0 examines both (draws u[0][0], u[0][1]); from position 1 on only the good one
            # is alive if it was accepted, and it is examined first there (draw u[1][0])
            want = orc.verify_sample(cur, cnd1, tok, np.array([[u[0, 1]], [u[1, 0]]], np.float32), u_final, 0.8, N, 1, V)
            assert got == want
        # alone, it is the same as no candidate at all
        u = rng.random((N - 1, 1), dtype=np.float32)
        got = orc.verify_sample(cur, np.zeros((1, N - 1, V), np.float32), np.full((1, N - 1), bad, np.int32), u, 0.3, 0.8, N, 1, V)
        want = orc.verify_sample(cur, np.zeros((0, N - 1, V), np.float32), np.zeros((0, N - 1), np.int32),
                                 np.zeros((N - 1, 0), np.float32), 0.3, 0.8, N, 0, V)
        assert got == want
