"""Pins of the oracle's attention over a row subset, and of lookahead parallelism's claim
(Sec. 3.4): a device that holds the current token, the oldest window level, its own columns of the
newer levels and its own candidates needs nothing from the other devices - what it computes for
its rows is what the full step computes for them."""
import numpy as np
import pytest

from oracle import la_oracle as orc
from paper_2402_02057_amd import workloads as wl


def rand_inputs(seed, P, T, H, KV, d):
    rng = np.random.default_rng(seed)
    bf = lambda shape: wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))
    return dict(q=bf((T, H, d)), k_cache=bf((KV, P, d)), v_cache=bf((KV, P, d)), step_k=bf((T, KV, d)), step_v=bf((T, KV, d)))


def share(W, N, G, parts, part):
    """Sec. 3.4 / its figure, written out: current token and oldest level everywhere (computed
    redundantly), columns and candidates dealt round-robin."""
    rows = [0] + [1 + j for j in range(W)]
    for l in range(1, N - 1):
        rows += [1 + l * W + j for j in range(W) if j % parts == part]
    for g in range(G):
        if g % parts == part:
            rows += [1 + W * (N - 1) + g * (N - 1) + k for k in range(N - 1)]
    return rows


@pytest.mark.parametrize("P,W,N,G,H,KV,d", [(7, 4, 3, 2, 2, 2, 8), (0, 3, 4, 3, 4, 2, 8), (20, 5, 5, 5, 2, 1, 16)])
def test_all_rows_is_the_plain_step(P, W, N, G, H, KV, d):
    T = 1 + (W + G) * (N - 1)
    x = rand_inputs(P + W, P, T, H, KV, d)
    want = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], P, W, N, G, H, KV, d)
    got = orc.step_attention_rows(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], np.arange(T), P, W, N, G, H, KV, d)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("W,N,G,parts", [(4, 3, 2, 2), (5, 4, 5, 4), (15, 5, 15, 4), (7, 5, 7, 8), (3, 2, 3, 2), (6, 4, 0, 3)])
def test_a_share_needs_nothing_from_the_others(W, N, G, parts):
    P, H, KV, d = 9, 2, 2, 8
    T = 1 + (W + G) * (N - 1)
    x = rand_inputs(W * 100 + G, P, T, H, KV, d)
    full = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], P, W, N, G, H, KV, d)
    mask = orc.step_mask(W, N, G)
    owned = np.zeros(T, dtype=int)
    for part in range(parts):
        ids = np.array(share(W, N, G, parts, part))
        assert (np.diff(ids) > 0).all()
        # closed: whatever a row of the share may see lies in the share
        assert not mask[ids][:, np.setdiff1d(np.arange(T), ids)].any()
        got = orc.step_attention_rows(x["q"][ids], x["k_cache"], x["v_cache"], x["step_k"][ids], x["step_v"][ids],
                                      ids, P, W, N, G, H, KV, d)
        np.testing.assert_allclose(got, full[ids], rtol=0, atol=1e-12)
        owned[ids] += 1
    # every row is computed somewhere; only the current token and the oldest level more than once
    assert (owned >= 1).all()
    assert (owned[1 + W:] == 1).all() and (owned[:1 + W] == parts).all()


def test_a_subset_that_is_not_closed_changes_the_result():
    """The restriction matters: dropping a visible key from the subset changes the row."""
    P, W, N, G, H, KV, d = 0, 3, 3, 1, 1, 1, 8
    T = 1 + (W + G) * (N - 1)
    x = rand_inputs(1, P, T, H, KV, d)
    full = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], P, W, N, G, H, KV, d)
    ids = np.array([0, 2, 5])               # level-1 column 1 without level-0 column 0 (which it sees)
    got = orc.step_attention_rows(x["q"][ids], x["k_cache"], x["v_cache"], x["step_k"][ids], x["step_v"][ids], ids,
                                  P, W, N, G, H, KV, d)
    assert np.abs(got[2] - full[5]).max() > 1e-3
    np.testing.assert_allclose(got[0], full[0], atol=1e-12)


@pytest.mark.parametrize("W,N,G,parts", [(4, 3, 2, 2), (15, 5, 15, 4), (7, 5, 7, 8), (6, 4, 0, 3), (0, 3, 5, 2), (30, 5, 30, 16)])
def test_the_products_share_helper(W, N, G, parts):
    """paper_2402_02057_amd.lookahead.lp_share (host logic, no GPU): the shares written out above."""
    from paper_2402_02057_amd import lookahead
    mask = orc.step_mask(W, N, G)
    T = 1 + (W + G) * (N - 1)
    for part in range(parts):
        ids = lookahead.lp_share(W, N, G, parts, part)
        assert ids == share(W, N, G, parts, part)
        assert not mask[ids][:, np.setdiff1d(np.arange(T), ids)].any()
