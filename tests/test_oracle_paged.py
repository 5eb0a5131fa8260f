"""Pins of the oracle's paged-cache helpers: a paged cache stands for the packed cache obtained by
following the block table; scattering a packed cache into pages (written here, the inverse
direction) and gathering it back must be the identity, and the paged append must leave the same
sequence as the packed append."""
import numpy as np
import pytest

from oracle import la_oracle as orc


def scatter(packed, block_table, page_size, n_pages, fill):
    """Independent inverse: place key t of every head at (block_table[t // ps], head, t % ps)."""
    kv, P, d = packed.shape
    pages = np.full((n_pages, kv, page_size, d), fill, dtype=packed.dtype)
    for page_index, page in enumerate(block_table[:(P + page_size - 1) // page_size]):
        lo = page_index * page_size
        hi = min(P, lo + page_size)
        pages[page, :, :hi - lo] = packed[:, lo:hi]
    return pages


@pytest.mark.parametrize("P,page_size,kv,d", [(0, 64, 2, 4), (1, 64, 1, 4), (64, 64, 2, 4), (65, 64, 3, 2),
                                              (300, 128, 2, 4), (1000, 256, 1, 8)])
def test_gather_inverts_scatter(P, page_size, kv, d):
    rng = np.random.default_rng(P + page_size)
    n_used = (P + page_size - 1) // page_size
    n_pages = n_used + 3
    table = rng.permutation(n_pages)[:n_used + 1].astype(np.int32)   # one spare entry, never read
    packed = rng.standard_normal((kv, P, d)).astype(np.float32)
    pages = scatter(packed, table, page_size, n_pages, np.nan)
    got = orc.gather_pages(pages, table, P, page_size)
    np.testing.assert_array_equal(got, packed)          # (no NaN: nothing outside the prefix is read)


def test_by_hand():
    pages = np.arange(3 * 1 * 2 * 1, dtype=np.float32).reshape(3, 1, 2, 1)   # page p holds [2p, 2p+1]
    got = orc.gather_pages(pages, np.array([2, 0, 1], np.int32), 5, 2)
    assert got[0, :, 0].tolist() == [4, 5, 0, 1, 2]


@pytest.mark.parametrize("P,page_size", [(3, 4), (4, 4), (6, 4), (0, 8)])
def test_paged_append_leaves_the_sequence_of_the_packed_append(P, page_size):
    rng = np.random.default_rng(P * 10 + page_size)
    W, N, G, kv, d = 2, 4, 3, 2, 3
    T = 1 + (W + G) * (N - 1)
    step_k = rng.standard_normal((T, kv, d)).astype(np.float32)
    step_v = rng.standard_normal((T, kv, d)).astype(np.float32)
    cap = P + N
    n_pages = (cap + page_size - 1) // page_size + 2
    table = rng.permutation(n_pages).astype(np.int32)
    packed_k = np.zeros((kv, cap, d), np.float32)
    packed_v = np.zeros((kv, cap, d), np.float32)
    packed_k[:, :P] = rng.standard_normal((kv, P, d))
    packed_v[:, :P] = rng.standard_normal((kv, P, d))
    for best, n_out in [(0, 1), (1, 2), (2, 4), (0, 3)]:
        pk, pv = packed_k.copy(), packed_v.copy()
        kp = scatter(np.ascontiguousarray(pk[:, :P]), table, page_size, n_pages, 0.0)
        vp = scatter(np.ascontiguousarray(pv[:, :P]), table, page_size, n_pages, 0.0)
        assert orc.kv_commit(pk, pv, step_k, step_v, P, W, N, G, best, n_out) == P + n_out
        assert orc.kv_commit_paged(kp, vp, table, page_size, step_k, step_v, P, W, N, G, best, n_out) == P + n_out
        np.testing.assert_array_equal(orc.gather_pages(kp, table, P + n_out, page_size), pk[:, :P + n_out])
        np.testing.assert_array_equal(orc.gather_pages(vp, table, P + n_out, page_size), pv[:, :P + n_out])
