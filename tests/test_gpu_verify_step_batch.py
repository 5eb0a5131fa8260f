"""GPU parity: la_verify_step_batch (the ends of several sequences' steps in one launch, through the
C ABI) against the CPU oracle's verify_step sequence by sequence, bit-exact."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda() if x.size else None


def run_batch(inputs, W, N, G, V, want_len=True):
    seqs = []
    for cur, look, cnd, cand in inputs:
        seqs.append(dict(logits_cur=torch.from_numpy(cur).cuda(), logits_look=dev(look.reshape(W, V)),
                         logits_cand=dev(cnd.reshape(G, N - 1, V)), cand_tokens=dev(cand.reshape(G, N - 1)),
                         out_tokens=torch.full((N,), -7, dtype=torch.int32, device="cuda"),
                         n_out=torch.full((1,), -7, dtype=torch.int32, device="cuda"),
                         best=torch.full((1,), -7, dtype=torch.int32, device="cuda"),
                         new_window=torch.full((W,), -7, dtype=torch.int32, device="cuda") if W else None,
                         accept_len=torch.full((G,), -7, dtype=torch.int32, device="cuda") if (want_len and G) else None))
    binding.la_verify_step_batch(seqs, W, N, G, V)
    torch.cuda.synchronize()
    return seqs


def check_batch(inputs, W, N, G, V, want_len=True):
    seqs = run_batch(inputs, W, N, G, V, want_len)
    for i, (x, (cur, look, cnd, cand)) in enumerate(zip(seqs, inputs)):
        w_out, w_best, w_window, w_len = orc.verify_step(cur, look, cnd, cand, W, N, G, V)
        n = int(x["n_out"].item())
        assert x["out_tokens"].cpu().numpy()[:n].tolist() == w_out, i
        assert int(x["best"].item()) == w_best, i
        if W:
            np.testing.assert_array_equal(x["new_window"].cpu().numpy(), w_window)
        if want_len and G:
            np.testing.assert_array_equal(x["accept_len"].cpu().numpy(), w_len)


@pytest.mark.parametrize("shape,n", [(wl.TINY, 5), (wl.LLAMA2_7B, 8), (wl.LLAMA2_13B, 3), (wl.LLAMA2_70B, 40),
                                     (wl.ragged_shape(0, 30), 2)], ids=lambda x: getattr(x, "name", str(x)))
def test_paper_configs(shape, n):
    """n sequences with different planted outcomes each; 40 is more than one launch carries."""
    s = shape
    print("case", s.name, n, flush=True)
    inputs = [wl.verify_step_inputs(s, extra)[:4] for extra in range(n)]
    check_batch(inputs, s.W, s.N, s.G, s.V)
    # the single call right after, on the same workspace
    cur, look, cnd, cand = inputs[0]
    check_batch([inputs[0]], s.W, s.N, s.G, s.V, want_len=False)


@pytest.mark.parametrize("V", [1, 3, 65, 1000, 4097, 50257])
def test_odd_vocabulary_sizes_and_ties(V):
    rng = np.random.default_rng(V)
    W, N, G, n = 3, 4, 4, 6
    inputs = []
    for i in range(n):
        cur = rng.standard_normal(V).astype(np.float32)
        look = np.round(rng.standard_normal((W, V))).astype(np.float32)          # many exact ties
        cnd = rng.standard_normal((G, N - 1, V)).astype(np.float32)
        cand = np.stack([np.concatenate([[int(np.argmax(cur))], np.argmax(cnd[g, :-1], axis=-1)]) for g in range(G)])
        cand = cand.astype(np.int32)
        if V > 1:
            cand[i % G, i % (N - 1)] = (cand[i % G, i % (N - 1)] + 1) % V          # one planted mismatch
        inputs.append((cur, look, cnd, cand))
    print("case", dict(V=V), flush=True)
    check_batch(inputs, W, N, G, V)


@pytest.mark.parametrize("W,N,G", [(0, 3, 2), (4, 2, 0), (0, 2, 0), (2, 2, 3)])
def test_degenerate_steps(W, N, G):
    V = 777
    rng = np.random.default_rng(W * 9 + N * 3 + G)
    inputs = []
    for _ in range(4):
        cur = rng.standard_normal(V).astype(np.float32)
        look = rng.standard_normal((W, V)).astype(np.float32)
        cnd = rng.standard_normal((G, N - 1, V)).astype(np.float32)
        cand = rng.integers(0, V, size=(G, N - 1)).astype(np.int32)
        if G:
            cand[0, 0] = int(np.argmax(cur))
        inputs.append((cur, look, cnd, cand))
    print("case", dict(W=W, N=N, G=G), flush=True)
    check_batch(inputs, W, N, G, V)


def test_equals_the_single_calls():
    s = wl.LLAMA2_7B
    inputs = [wl.verify_step_inputs(s, extra)[:4] for extra in range(16)]
    seqs = run_batch(inputs, s.W, s.N, s.G, s.V)
    for x in seqs:
        outs = [torch.full_like(x[k], -9) for k in ("out_tokens", "n_out", "best", "new_window", "accept_len")]
        binding.la_verify_step(x["logits_cur"], x["logits_look"], x["logits_cand"], x["cand_tokens"], s.W, s.N, s.G,
                               s.V, *outs)
        torch.cuda.synchronize()
        n = int(outs[1].item())
        assert n == int(x["n_out"].item())
        assert torch.equal(outs[0][:n], x["out_tokens"][:n]) and torch.equal(outs[2], x["best"])
        assert torch.equal(outs[3], x["new_window"]) and torch.equal(outs[4], x["accept_len"])
