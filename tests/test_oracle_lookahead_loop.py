"""Pins of the decoding loop (Algorithm 2) written out in oracle/lookahead_loop.py."""
import numpy as np
import pytest

from oracle import lookahead_loop as loop
from paper_2402_02057_amd import workloads as wl


@pytest.mark.parametrize("W,N,G", [(5, 4, 5), (1, 2, 1), (3, 3, 0), (0, 3, 3), (8, 5, 8), (15, 5, 15)])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_output_equals_plain_greedy_decoding(W, N, G, seed):
    """Lossless (Sec. 3.2, Sec. 5.3): whatever W, N, G and the window's random content, the tokens
    are exactly those of step-by-step greedy decoding."""
    model = loop.ToyModel(seed)
    prompt = [0, 3 + seed, 7, 3 + seed]
    want = loop.greedy_decode(model, prompt, 120)
    got, steps, trace = loop.lookahead_decode(model, prompt, W, N, G, 120, seed=seed)
    assert got == want
    assert steps <= 120
    assert all(1 <= len(t["accepted"]) <= N for t in trace)


def test_steps_are_compressed_when_candidates_exist():
    """The toy model's sequences become periodic, the pool fills with their n-grams and several
    tokens are accepted per step: S = tokens / steps > 1 (Eq. 6); with no lookahead and no
    candidates the loop degenerates to one token per step."""
    model = loop.ToyModel(0)
    prompt = [0, 5, 9]
    _, steps, trace = loop.lookahead_decode(model, prompt, 5, 4, 5, 200, seed=0)
    assert 200 / steps > 1.5
    assert max(len(t["accepted"]) for t in trace) == 4
    _, steps0, _ = loop.lookahead_decode(model, prompt, 0, 4, 0, 50, seed=0)
    assert steps0 == 50


@pytest.mark.parametrize("W,N,G", [(4, 3, 2), (4, 3, 0), (2, 5, 1)])
def test_step_layout_and_pool_cap(W, N, G):
    model = loop.ToyModel(1)
    _, _, trace = loop.lookahead_decode(model, [0, 2, 4], W, N, G, 60, seed=3)
    for t in trace:
        n_cand = (len(t["tokens"]) - 1 - W * (N - 1)) // (N - 1)
        assert 0 <= n_cand <= G
        assert len(t["tokens"]) == 1 + (W + n_cand) * (N - 1)
        assert len(t["window"]) == W
        assert t["best"] == -1 or 0 <= t["best"] < n_cand


def test_expected_tokens_formula_of_the_scaling_section():
    """Eq. 5 reduces to Eq. 4 for b = 1, and with the setting quoted for Fig. 4(b)
    (alpha = 0.425, f = 3.106, b = W = G = 15, gamma = N - 1 = 4) Eq. 7 gives S close to the
    compression reported for that configuration (1.96, Table 3)."""
    def e_tokens(alpha, gamma, b):
        return (gamma + 1) - sum((1 - alpha ** i) ** b for i in range(1, gamma + 1))
    for alpha in (0.1, 0.425, 0.9):
        for gamma in (1, 4, 9):
            assert abs(e_tokens(alpha, gamma, 1) - (1 - alpha ** (gamma + 1)) / (1 - alpha)) < 1e-12
    s = (3.106 - 1 + e_tokens(0.425, 4, 15)) / 3.106
    assert abs(s - 1.96) < 0.05


def test_random_window_tokens_are_valid_and_spread():
    toks = [wl.window_random_token(s, i, j) for s in range(3) for i in range(-4, 60) for j in range(8)]
    assert min(toks) >= 1 and max(toks) < wl.TOY_VOCAB
    assert len(set(toks)) == wl.TOY_VOCAB - 1


def test_prompt_as_reference_changes_the_steps_but_never_the_output():
    """Sec. 5.4: the prompt's own n-grams as candidates.  With no lookahead branch (W = 0) the pool
    holds nothing else: a prompt that already contains the continuation compresses the steps, any
    other prompt leaves one token per step; the tokens are the greedy ones either way."""
    model = loop.ToyModel(3)
    head = [0, 5, 9]
    seen = loop.greedy_decode(model, head, 80)
    prompt = head + seen                          # the continuation goes on cycling through these
    want = loop.greedy_decode(model, prompt, 60)
    plain, steps_plain, _ = loop.lookahead_decode(model, prompt, 0, 4, 3, 60, seed=3)
    assert plain == want and steps_plain == 60
    got, steps, trace = loop.lookahead_decode(model, prompt, 0, 4, 3, 60, seed=3, prompt_as_reference=True)
    assert got == want and steps < 40
    assert all(len(t["tokens"]) == 1 + len(t["tokens"][1:]) and (len(t["tokens"]) - 1) % 3 == 0 for t in trace)
    # with a lookahead branch as well: still the same tokens
    got, steps_both, _ = loop.lookahead_decode(model, prompt, 5, 4, 5, 60, seed=3, prompt_as_reference=True)
    assert got == want and steps_both <= 60
