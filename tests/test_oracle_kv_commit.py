"""Pin of the oracle's cache append: after any number of lookahead steps the cache must be the one
plain autoregressive decoding builds, row t holding the keys/values of token t at position t.

The keys/values here are an arbitrary function of (token, absolute position, head): what a model
with position-dependent keys (RoPE) computes.  The step computes them for every row of the step at
the row's position (Fig. 2(b): the digits on the tokens, written out below independently of the
oracle); the append then has to pick exactly the rows of the accepted tokens."""
import numpy as np
import pytest

from oracle import la_oracle as orc
from oracle import lookahead_loop as loop

KV, D = 2, 8


def kv_of(token, position, which):
    h = (int(token) * 1000003 + int(position) * 7919 + which * 104729 + 12345) % (1 << 31)
    return np.random.default_rng(h).standard_normal((KV, D)).astype(np.float32)


def relative_positions(W, N, g):
    """Digits of Fig. 2(b), shifted by one for the separate current-token row: lookahead level l,
    column j sits l + j + 1 after the current token; candidate token k sits k + 1 after it."""
    pos = [0]
    for l in range(N - 1):
        pos += [1 + l + j for j in range(W)]
    for _ in range(g):
        pos += [1 + k for k in range(N - 1)]
    return pos


@pytest.mark.parametrize("W,N,G,seed", [(5, 4, 5, 0), (3, 3, 2, 1), (0, 3, 3, 3), (4, 2, 4, 2), (8, 5, 8, 4)])
def test_cache_after_lookahead_steps_is_the_autoregressive_cache(W, N, G, seed):
    model = loop.ToyModel(seed)
    prompt = [0, 5, 9, 5] if W else [0, 5, 9] + loop.greedy_decode(model, [0, 5, 9], 40)
    n_tokens = 80
    tokens, steps, trace = loop.lookahead_decode(model, prompt, W, N, G, n_tokens, seed=seed,
                                                 prompt_as_reference=(W == 0))
    seq = list(prompt)
    capacity = len(prompt) + n_tokens + 2 * N
    kc = np.zeros((KV, capacity, D), np.float32)
    vc = np.zeros((KV, capacity, D), np.float32)
    P = len(prompt) - 1
    for t in range(P):                      # prefill: every prompt token but the last
        kc[:, t], vc[:, t] = kv_of(seq[t], t, 0), kv_of(seq[t], t, 1)
    multi = 0
    for rec in trace:
        g = (len(rec["tokens"]) - 1) // (N - 1) - W
        rel = relative_positions(W, N, g)
        assert len(rel) == len(rec["tokens"])
        step_k = np.stack([kv_of(tok, P + r, 0) for tok, r in zip(rec["tokens"], rel)])
        step_v = np.stack([kv_of(tok, P + r, 1) for tok, r in zip(rec["tokens"], rel)])
        P = orc.kv_commit(kc, vc, step_k, step_v, P, W, N, g, rec["best"], len(rec["accepted"]))
        multi += len(rec["accepted"]) > 1
        seq.extend(rec["accepted"])
        assert P == len(seq) - 1
        # rows past the prefix are untouched
        assert not kc[:, P:].any() and not vc[:, P:].any()
    assert multi > 3                        # steps that append several rows did occur
    for t in range(P):
        np.testing.assert_array_equal(kc[:, t], kv_of(seq[t], t, 0))
        np.testing.assert_array_equal(vc[:, t], kv_of(seq[t], t, 1))


def test_rows_by_hand():
    W, N, G = 2, 3, 2                        # T = 1 + 4 + 4; candidate rows 5,6 and 7,8
    T = 9
    step_k = np.arange(T * 1 * 2, dtype=np.float32).reshape(T, 1, 2)
    step_v = -step_k
    kc = np.full((1, 10, 2), 99.0, np.float32)
    vc = np.full((1, 10, 2), 99.0, np.float32)
    assert orc.kv_commit(kc, vc, step_k, step_v, 4, W, N, G, 1, 3) == 7
    np.testing.assert_array_equal(kc[0, 4:7], step_k[[0, 7, 8], 0])
    np.testing.assert_array_equal(vc[0, 4:7], step_v[[0, 7, 8], 0])
    assert (kc[0, :4] == 99).all() and (kc[0, 7:] == 99).all()
    assert orc.kv_commit(kc, vc, step_k, step_v, 7, W, N, G, -1, 1) == 8    # nothing accepted
    np.testing.assert_array_equal(kc[0, 7], step_k[0, 0])
    assert (kc[0, 8:] == 99).all()
