"""GPU parity: la_verify_sample (HIP, through the C ABI) against the CPU oracle.

The kernel's arithmetic is fp32, the oracle's fp64: a uniform draw within rounding of the
probability it is compared with (or of a step of the cumulative distribution) may legitimately
fall on either side.  The tests therefore compute, with an independent fp64 walk, how close the
closest decision of a case was, require exact agreement whenever that margin is not tiny, and
require most cases to agree exactly."""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def dev(x):
    x = np.ascontiguousarray(x)
    return torch.from_numpy(x).cuda() if x.size else None


def run_hip(cur, cnd, cand, u_test, u_final, temperature, N, G, V):
    out = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    n_out = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    binding.la_verify_sample(torch.from_numpy(cur).cuda(), dev(cnd.reshape(G, N - 1, V)), dev(cand.reshape(G, N - 1)),
                             dev(u_test.reshape(N - 1, G)), torch.from_numpy(u_final).cuda(), temperature, N, G, V,
                             out, n_out)
    torch.cuda.synchronize()
    return out.cpu().numpy()[:int(n_out.item())].tolist()


def walk_with_margin(cur, cnd, cand, u_test, u_final, temperature, N, G, V):
    """Algorithm 4 in fp64 with the smallest distance between a draw and what it was compared to."""
    n1 = N - 1
    margin = 1.0
    alive, out = list(range(G)), []

    def dist(row):
        return scipy.special.softmax(row.astype(np.float64) / temperature)

    def draw(P, u):
        nonlocal margin
        cdf = np.cumsum(P)
        v = min(int(np.searchsorted(cdf, u, side="right")), V - 1)
        while P[v] == 0.0 and v > 0:
            v -= 1
        margin = min(margin, abs(cdf[v] - u), abs((cdf[v - 1] if v > 0 else 0.0) - u) if v > 0 else 1.0)
        return v
    for i in range(n1):
        if not alive:
            break
        P = dist(cur if i == 0 else cnd[alive[0], i - 1])
        accepted = False
        for j, g in enumerate(alive):
            s = int(cand[g, i])
            if not 0 <= s < V:     # outside the vocabulary: probability zero, nothing ruled out
                continue
            margin = min(margin, abs(float(u_test[i, j]) - P[s]))
            if u_test[i, j] < P[s]:
                out.append(s)
                alive = [k for k in alive[j:] if cand[k, i] == s]
                accepted = True
                break
            P[s] = 0.0
            P = P / P.sum()
        if not accepted:
            return out + [draw(P, float(u_final[0]))], margin
    P = dist(cur if not out else cnd[alive[0], len(out) - 1])
    return out + [draw(P, float(u_final[0]))], margin


def check(cur, cnd, cand, u_test, u_final, temperature, N, G, V, tag=""):
    print("case", tag, dict(N=N, G=G, V=V, T=temperature), flush=True)
    got = run_hip(cur, cnd, cand, u_test, u_final, temperature, N, G, V)
    want = orc.verify_sample(cur, cnd, cand, u_test, float(u_final[0]), temperature, N, G, V)
    ref, margin = walk_with_margin(cur, cnd, cand, u_test, u_final, temperature, N, G, V)
    assert ref == want or margin < 1e-9
    assert 1 <= len(got) <= N
    if got != want:
        assert margin < 2e-5, (got, want, margin)
        return False
    return True


@pytest.mark.parametrize("shape", [wl.LLAMA2_7B, wl.LLAMA2_13B, wl.LLAMA2_70B, wl.ragged_shape(0, 30)],
                         ids=lambda s: s.name)
def test_paper_configs(shape):
    s = shape
    exact = 0
    lengths = set()
    for extra in range(12):
        for temperature in (1.0, 0.7):
            x = wl.verify_sample_inputs(s, extra)
            exact += check(*x, temperature, s.N, s.G, s.V, "%s/%d" % (s.name, extra))
            lengths.add(len(orc.verify_sample(*x[:4], float(x[4][0]), temperature, s.N, s.G, s.V)))
    assert exact >= 22          # near-ties are rare
    assert len(lengths) >= 2    # the cases exercise both rejection and acceptance


@pytest.mark.parametrize("V", [1, 2, 3, 5, 63, 64, 65, 1000, 1023, 4096, 4097, 32001, 50257, 70001])
def test_odd_vocabulary_sizes(V):
    rng = np.random.default_rng(V)
    N, G = 4, 5
    cur = (rng.standard_normal(V) * 3).astype(np.float32)
    cnd = (rng.standard_normal((G, N - 1, V)) * 3).astype(np.float32)
    cand = rng.integers(0, V, size=(G, N - 1)).astype(np.int32)
    cand[0, 0] = int(np.argmax(cur))
    cand[1, 0] = int(np.argmax(cur))
    cand[1, 1] = int(np.argmax(cnd[1, 0]))
    exact = 0
    for t in range(6):
        u_test = rng.random((N - 1, G), dtype=np.float32)
        u_final = rng.random(1, dtype=np.float32)
        exact += check(cur, cnd, cand, u_test, u_final, 0.9, N, G, V)
    assert exact >= 5


@pytest.mark.parametrize("N,G", [(2, 0), (5, 0), (2, 1), (3, 7), (8, 3), (2, 64), (4, 200)])
def test_shapes_and_degenerate_cases(N, G):
    rng = np.random.default_rng(N * 100 + G)
    V = 501
    cur = (rng.standard_normal(V) * 4).astype(np.float32)
    cnd = (rng.standard_normal((G, N - 1, V)) * 4).astype(np.float32)
    cand = rng.integers(0, V, size=(G, N - 1)).astype(np.int32)
    if G:
        cand[:, 0] = np.argsort(cur)[::-1][rng.integers(0, 3, size=G)]     # likely tokens, with repeats
    exact = 0
    for t in range(5):
        u_test = rng.random((N - 1, G), dtype=np.float32)
        u_final = rng.random(1, dtype=np.float32)
        exact += check(cur, cnd, cand, u_test, u_final, 1.3, N, G, V)
    assert exact >= 4


@pytest.mark.parametrize("bad", [-1, 501, 2**31 - 1, -2**31])
def test_tokens_outside_the_vocabulary_are_never_accepted_and_never_read(bad):
    """Padding ids among the candidate tokens: probability zero, no logit read (the logits sit at
    the very end of their allocation here, and in front of it)."""
    rng = np.random.default_rng(5)
    N, G, V = 4, 6, 501
    cur = (rng.standard_normal(V) * 4).astype(np.float32)
    cnd = (rng.standard_normal((G, N - 1, V)) * 4).astype(np.float32)
    cand = rng.integers(0, V, size=(G, N - 1)).astype(np.int32)
    cand[:, 0] = np.argsort(cur)[::-1][rng.integers(0, 2, size=G)]
    cand[0, :] = bad              # a whole candidate of padding
    cand[2, 1] = bad              # padding after a real first token
    cand[4, 0] = bad
    exact = 0
    for t in range(6):
        u_test = rng.random((N - 1, G), dtype=np.float32) * 0.5   # low draws: accept often
        u_final = rng.random(1, dtype=np.float32)
        exact += check(cur, cnd, cand, u_test, u_final, 1.0, N, G, V, "bad token %d" % bad)
        got = run_hip(cur, cnd, cand, u_test, u_final, 1.0, N, G, V)
        assert all(0 <= t < V for t in got)
    assert exact >= 5


def test_draw_extremes_and_sharp_distributions():
    rng = np.random.default_rng(3)
    V, N, G = 32000, 3, 2
    cur = rng.standard_normal(V).astype(np.float32)
    cnd = rng.standard_normal((G, N - 1, V)).astype(np.float32)
    cand = rng.integers(0, V, size=(G, N - 1)).astype(np.int32)
    for u in (0.0, 1.0 - 2.0 ** -24):
        # all candidates rejected (their tokens are improbable): the draw decides alone
        u_test = np.full((N - 1, G), 0.5, dtype=np.float32)
        got = run_hip(cur, cnd, cand, u_test, np.array([u], np.float32), 1.0, N, G, V)
        assert len(got) == 1
        P = scipy.special.softmax(cur.astype(np.float64))
        P[cand[:, 0]] = 0.0
        nz = np.nonzero(P)[0]
        assert got[0] == (nz[0] if u == 0.0 else nz[-1]) or abs(np.cumsum(P / P.sum())[got[0]] - u) < 1e-4
    # a one-hot distribution: the peaked token is accepted whatever the draw
    cur[:] = 0.0
    cur[123] = 80.0
    cand[0, 0] = 5
    cand[1, 0] = 123
    got = run_hip(cur, cnd, cand, np.full((N - 1, G), 0.999, dtype=np.float32), np.array([0.3], np.float32),
                  1.0, N, G, V)
    assert got[0] == 123


def test_zero_temperature_limit_equals_the_greedy_step():
    s = wl.LLAMA2_7B
    cur, look, cnd, cand, lens = wl.verify_step_inputs(s)
    want, _, _, _ = orc.verify_step(cur, look, cnd, cand, s.W, s.N, s.G, s.V)
    rng = np.random.default_rng(8)
    # planted peaks of 12 against N(0,1) noise at temperature 0.05: one-hot to fp32 precision.
    # Greedy judges every candidate by its own rows; sampling by the first survivor's: they agree
    # when the surviving candidates' rows agree, which holds for the winner's accepted run here.
    u_test = (rng.random((s.N - 1, s.G), dtype=np.float32) * 0.9 + 0.05).astype(np.float32)
    got = run_hip(cur, cnd, cand, u_test, np.array([0.5], np.float32), 0.05, s.N, s.G, s.V)
    ref = orc.verify_sample(cur, cnd, cand, u_test, 0.5, 0.05, s.N, s.G, s.V)
    assert got == ref
    assert got[:1] == want[:1]


def test_repeated_calls_leave_the_workspace_clean():
    s = wl.LLAMA2_13B
    x = wl.verify_sample_inputs(s, 1)
    for _ in range(3):
        check(*x, 1.0, s.N, s.G, s.V, "again")
    logits, cand, lens = wl.verify_inputs(s)
    alen = torch.empty((s.G,), dtype=torch.int32, device="cuda")
    acc = torch.empty((s.G, s.N - 1), dtype=torch.int32, device="cuda")
    binding.la_verify(torch.from_numpy(logits).cuda(), torch.from_numpy(cand).cuda(), s.G, s.N, s.V, alen, acc)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(alen.cpu().numpy(), lens)


def test_errors():
    z = torch.zeros((8,), dtype=torch.float32, device="cuda")
    u = torch.zeros((1,), dtype=torch.float32, device="cuda")
    i1 = torch.zeros((1,), dtype=torch.int32, device="cuda")
    i2 = torch.zeros((2,), dtype=torch.int32, device="cuda")
    with pytest.raises(binding.LaError) as e:
        binding.la_verify_sample(z, None, None, None, u, 0.0, 2, 0, 8, i2, i1)
    assert e.value.code == -1
