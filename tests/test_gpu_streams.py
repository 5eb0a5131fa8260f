"""Calls on two streams at once, each with its own workspace set (la_select_workspace): the results
are those of the same calls one after the other.  Both streams run split attention steps and
verification steps, which keep tickets, keys and partial results in the library's workspace - the
state that calls sharing a set would trample on."""
import numpy as np
import pytest
import torch

from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def test_two_streams_with_their_own_workspace_sets():
    s = wl.LLAMA2_7B
    W, N, G, V, H, KV, d, T = s.W, s.N, s.G, s.V, s.heads, s.kv_heads, s.head_dim, s.T
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)

    def rb(*shape):
        return torch.randn(shape, device="cuda", generator=gen).bfloat16()

    def job(P):
        x = dict(q=rb(T, H, d), kc=rb(KV, P, d), vc=rb(KV, P, d), sk=rb(T, KV, d), sv=rb(T, KV, d), P=P,
                 cur=torch.randn(V, device="cuda", generator=gen), look=torch.randn(W, V, device="cuda", generator=gen),
                 cnd=torch.randn(G, N - 1, V, device="cuda", generator=gen),
                 cand=torch.randint(0, V, (G, N - 1), device="cuda", generator=gen, dtype=torch.int32))
        x["cur"][x["cand"][0, 0].long()] = 30.0
        return x

    def outputs():
        i32 = dict(dtype=torch.int32, device="cuda")
        return [torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda"), torch.empty(N, **i32), torch.empty(1, **i32),
                torch.empty(1, **i32), torch.empty(W, **i32), torch.empty(G, **i32)]

    def run(x, o, rounds):
        for _ in range(rounds):
            binding.la_step_attention(x["q"], x["kc"], x["vc"], x["sk"], x["sv"], x["P"], W, N, G, H, KV, d, o[0])
            binding.la_verify_step(x["cur"], x["look"], x["cnd"], x["cand"], W, N, G, V, *o[1:])

    jobs = [job(1024), job(1800)]
    want = [outputs(), outputs()]
    for x, o in zip(jobs, want):                # one after the other, on the current stream, set 0
        run(x, o, 1)
    torch.cuda.synchronize()

    got = [outputs(), outputs()]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    try:
        for rounds in (1, 20):                  # 20: long enough for the two streams to overlap for certain
            for o in got:
                for t in o:
                    t.zero_()
            torch.cuda.synchronize()
            for i, (x, o, st) in enumerate(zip(jobs, got, streams)):
                binding.la_select_workspace(1 + i)
                with torch.cuda.stream(st):
                    run(x, o, rounds)
            torch.cuda.synchronize()
            for i in range(2):
                assert torch.equal(got[i][0].view(torch.int16), want[i][0].view(torch.int16)), (rounds, i)
                n = int(want[i][2].item())
                assert int(got[i][2].item()) == n and torch.equal(got[i][1][:n], want[i][1][:n]), (rounds, i)
                for a, b in zip(got[i][3:], want[i][3:]):
                    assert torch.equal(a, b), (rounds, i)
    finally:
        binding.la_select_workspace(0)
    with pytest.raises(binding.LaError, match="0..15"):
        binding.la_select_workspace(16)
