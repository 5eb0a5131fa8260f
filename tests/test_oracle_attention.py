"""Pins of the oracle's attention arithmetic (Sec. 2 causal attention + Sec. 3.3 mask).

Nothing here retypes the oracle's formula: every expected value comes from a library
softmax-attention (torch.nn.functional.scaled_dot_product_attention, fp64, CPU) run on an
ordinary causal sequence, or from an invariant of softmax attention.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import la_oracle as orc
from paper_2402_02057_amd import workloads as wl
from test_oracle_mask import parent


def rand_bf16(rng, shape):
    return wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


def f64(bits):
    return torch.from_numpy(wl.bf16_bits_to_f32(bits).astype(np.float64))


def make_inputs(rng, P, W, N, G, H, KV, d):
    T = 1 + (W + G) * (N - 1)
    return dict(q=rand_bf16(rng, (T, H, d)), k_cache=rand_bf16(rng, (KV, P, d)),
                v_cache=rand_bf16(rng, (KV, P, d)), step_k=rand_bf16(rng, (T, KV, d)),
                step_v=rand_bf16(rng, (T, KV, d)))


def run_oracle(x, P, W, N, G, H, KV, d):
    return orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"],
                              P, W, N, G, H, KV, d)


def chain_of(r, W, N, G):
    """Step rows on row r's trajectory, oldest first, ending with r itself."""
    chain = []
    c = r
    while c is not None:
        chain.append(c)
        c = parent(c, W, N, G)
    return chain[::-1]


def causal_reference(x, P, W, N, G, H, KV, d):
    """Each row = last row of textbook causal attention over prefix + its own token chain."""
    T = 1 + (W + G) * (N - 1)
    g = H // KV
    out = np.zeros((T, H, d))
    q, kc, vc, sk, sv = (f64(x[k]) for k in ("q", "k_cache", "v_cache", "step_k", "step_v"))
    for r in range(T):
        chain = chain_of(r, W, N, G)
        n = len(chain)
        for h in range(H):
            kvh = h // g
            keys = torch.cat([kc[kvh], sk[chain, kvh]], dim=0)            # [P+n, d]
            vals = torch.cat([vc[kvh], sv[chain, kvh]], dim=0)
            # queries of the prefix positions are irrelevant to the last row: use zeros
            qs = torch.zeros(P + n, d, dtype=torch.float64)
            qs[-1] = q[r, h]
            o = F.scaled_dot_product_attention(qs[None, None], keys[None, None], vals[None, None],
                                               is_causal=True)
            out[r, h] = o[0, 0, -1].numpy()
    return out


BRUTE = [(P, W, N, G) for P in (0, 1, 5) for W in (0, 1, 3, 4) for N in (2, 3, 4) for G in (0, 1, 3)]


@pytest.mark.parametrize("P,W,N,G", BRUTE)
def test_rows_equal_causal_attention_over_their_chain(P, W, N, G):
    rng = np.random.default_rng(1000 + 97 * P + 13 * W + 5 * N + G)
    H, KV, d = 2, 1, 8
    x = make_inputs(rng, P, W, N, G, H, KV, d)
    got = run_oracle(x, P, W, N, G, H, KV, d)
    want = causal_reference(x, P, W, N, G, H, KV, d)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_rows_equal_causal_attention_gqa_tiny_shape():
    s = wl.TINY
    x = wl.attention_inputs(s)
    got = run_oracle(x, s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim)
    want = causal_reference(x, s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # grouped-query layout: 4 query heads on 2 KV heads
    rng = np.random.default_rng(7)
    x = make_inputs(rng, 9, 3, 3, 2, 4, 2, 16)
    got = run_oracle(x, 9, 3, 3, 2, 4, 2, 16)
    want = causal_reference(x, 9, 3, 3, 2, 4, 2, 16)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("P,H,KV,d", [(1, 1, 1, 4), (33, 4, 2, 16), (257, 8, 8, 64)])
def test_reduces_to_one_token_decode(P, H, KV, d):
    """W = 0, G = 0: one query row over P + 1 keys, a plain decode step."""
    rng = np.random.default_rng(P)
    x = make_inputs(rng, P, 0, 3, 0, H, KV, d)
    got = run_oracle(x, P, 0, 3, 0, H, KV, d)
    assert got.shape == (1, H, d)
    g = H // KV
    q, kc, vc, sk, sv = (f64(x[k]) for k in ("q", "k_cache", "v_cache", "step_k", "step_v"))
    for h in range(H):
        kvh = h // g
        keys = torch.cat([kc[kvh], sk[:, kvh]], dim=0)
        vals = torch.cat([vc[kvh], sv[:, kvh]], dim=0)
        o = F.scaled_dot_product_attention(q[0, h][None, None, None], keys[None, None],
                                           vals[None, None])
        np.testing.assert_allclose(got[0, h], o[0, 0, 0].numpy(), rtol=0, atol=1e-12)


def test_empty_prefix_first_row_is_its_own_value():
    rng = np.random.default_rng(3)
    x = make_inputs(rng, 0, 2, 3, 1, 2, 2, 8)
    got = run_oracle(x, 0, 2, 3, 1, 2, 2, 8)
    np.testing.assert_array_equal(got[0], wl.bf16_bits_to_f32(x["step_v"][0]).astype(np.float64))


def test_scale_is_inverse_sqrt_head_dim():
    """Two keys, q.k = d for one and 0 for the other: weights are softmax([sqrt(d), 0])."""
    d = 16
    one = wl.f32_to_bf16_bits(np.ones((1, 1, d), dtype=np.float32))
    zero = wl.f32_to_bf16_bits(np.zeros((1, 1, d), dtype=np.float32))
    v_prefix = wl.f32_to_bf16_bits(np.full((1, 1, d), 2.0, dtype=np.float32))
    v_step = wl.f32_to_bf16_bits(np.full((1, 1, d), -1.0, dtype=np.float32))
    got = orc.step_attention(one, one, v_prefix, zero, v_step, 1, 0, 2, 0, 1, 1, d)
    w = 1.0 / (1.0 + np.exp(-np.sqrt(d)))   # weight of the prefix key
    np.testing.assert_allclose(got[0, 0], np.full(d, 2.0 * w - (1 - w)), rtol=0, atol=1e-13)


def test_branch_isolation_is_bit_exact():
    P, W, N, G, H, KV, d = 6, 4, 4, 3, 2, 2, 8
    rng = np.random.default_rng(11)
    x = make_inputs(rng, P, W, N, G, H, KV, d)
    base = run_oracle(x, P, W, N, G, H, KV, d)
    nl = W * (N - 1)
    n1 = N - 1
    # perturb every candidate key/value: current + lookahead rows unchanged
    y = {k: v.copy() for k, v in x.items()}
    y["step_k"][1 + nl:] = rand_bf16(rng, y["step_k"][1 + nl:].shape)
    y["step_v"][1 + nl:] = rand_bf16(rng, y["step_v"][1 + nl:].shape)
    got = run_oracle(y, P, W, N, G, H, KV, d)
    np.testing.assert_array_equal(got[:1 + nl], base[:1 + nl])
    assert np.abs(got[1 + nl:] - base[1 + nl:]).max() > 1e-3
    # perturb the lookahead window: current + candidate rows unchanged
    y = {k: v.copy() for k, v in x.items()}
    y["step_k"][1:1 + nl] = rand_bf16(rng, y["step_k"][1:1 + nl].shape)
    y["step_v"][1:1 + nl] = rand_bf16(rng, y["step_v"][1:1 + nl].shape)
    got = run_oracle(y, P, W, N, G, H, KV, d)
    np.testing.assert_array_equal(got[0], base[0])
    np.testing.assert_array_equal(got[1 + nl:], base[1 + nl:])
    # perturb candidate 1 only: candidates 0 and 2 unchanged
    y = {k: v.copy() for k, v in x.items()}
    sl = slice(1 + nl + n1, 1 + nl + 2 * n1)
    y["step_k"][sl] = rand_bf16(rng, y["step_k"][sl].shape)
    y["step_v"][sl] = rand_bf16(rng, y["step_v"][sl].shape)
    got = run_oracle(y, P, W, N, G, H, KV, d)
    keep = np.ones(base.shape[0], dtype=bool)
    keep[sl] = False
    np.testing.assert_array_equal(got[keep], base[keep])
    # perturb column 2 above the oldest level: only that column's rows at levels >= 1 move
    y = {k: v.copy() for k, v in x.items()}
    rows = [1 + l * W + 2 for l in range(1, N - 1)]
    y["step_k"][rows] = rand_bf16(rng, y["step_k"][rows].shape)
    y["step_v"][rows] = rand_bf16(rng, y["step_v"][rows].shape)
    got = run_oracle(y, P, W, N, G, H, KV, d)
    keep = np.ones(base.shape[0], dtype=bool)
    keep[rows] = False
    np.testing.assert_array_equal(got[keep], base[keep])


def test_mask_read_out_through_one_hot_values():
    """Prefix values 0 and step value c = e_c: out[r][c] > 0 exactly where r sees c."""
    s = wl.TINY
    x = wl.attention_inputs(s)
    T, d = s.T, s.head_dim
    assert d >= T
    x["v_cache"][:] = 0
    onehot = np.zeros((T, s.kv_heads, d), dtype=np.float32)
    for c in range(T):
        onehot[c, :, c] = 1.0
    x["step_v"] = wl.f32_to_bf16_bits(onehot)
    got = run_oracle(x, s.P, s.W, s.N, s.G, s.heads, s.kv_heads, d)
    m = orc.step_mask(s.W, s.N, s.G)
    for h in range(s.heads):
        np.testing.assert_array_equal(got[:, h, :T] > 0, m)
        assert np.all(got[:, h, T:] == 0)


def test_constant_values_and_prefix_permutation():
    P, W, N, G, H, KV, d = 40, 3, 4, 2, 4, 2, 16
    rng = np.random.default_rng(5)
    x = make_inputs(rng, P, W, N, G, H, KV, d)
    base = run_oracle(x, P, W, N, G, H, KV, d)
    # permuting prefix keys together with their values changes nothing but rounding order
    perm = rng.permutation(P)
    y = dict(x)
    y["k_cache"] = x["k_cache"][:, perm].copy()
    y["v_cache"] = x["v_cache"][:, perm].copy()
    np.testing.assert_allclose(run_oracle(y, P, W, N, G, H, KV, d), base, rtol=0, atol=1e-13)
    # all values equal to one vector: every output row is that vector
    v0 = rand_bf16(rng, (d,))
    y = dict(x)
    y["v_cache"] = np.broadcast_to(v0, (KV, P, d)).copy()
    y["step_v"] = np.broadcast_to(v0, x["step_v"].shape).copy()
    got = run_oracle(y, P, W, N, G, H, KV, d)
    want = wl.bf16_bits_to_f32(v0).astype(np.float64)
    np.testing.assert_allclose(got, np.broadcast_to(want, got.shape), rtol=0, atol=1e-13)


def test_bad_shapes_are_rejected():
    z = np.zeros((1, 3, 4), dtype=np.uint16)
    with pytest.raises(ValueError):
        orc.step_attention(z, np.zeros((2, 0, 4), np.uint16), np.zeros((2, 0, 4), np.uint16),
                           np.zeros((1, 2, 4), np.uint16), np.zeros((1, 2, 4), np.uint16),
                           0, 0, 2, 0, 3, 2, 4)
