"""The entry points inside a HIP graph: every replay, with other work and new input contents
between the replays, must give what the same calls give eagerly (the tickets and packed keys the
kernels keep in the library's workspace have to come back to zero after every launch, also when
the launch is a graph node)."""
import numpy as np
import pytest
import torch

from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def test_replays_equal_eager_calls():
    s = wl.LLAMA2_7B
    W, N, G, V, H, KV, d, P, T = s.W, s.N, s.G, s.V, s.heads, s.kv_heads, s.head_dim, s.P, s.T
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)

    def rb(*shape):
        return torch.randn(shape, device="cuda", generator=gen).bfloat16()
    q, kc, vc, sk, sv = rb(T, H, d), rb(KV, P, d), rb(KV, P, d), rb(T, KV, d), rb(T, KV, d)
    q2, kc2, vc2, sk2, sv2 = rb(T, H, d), rb(KV, 700, d), rb(KV, 700, d), rb(T, KV, d), rb(T, KV, d)
    logits_cur = torch.randn(V, device="cuda", generator=gen)
    logits_look = torch.randn(W, V, device="cuda", generator=gen)
    logits_cand = torch.randn(G, N - 1, V, device="cuda", generator=gen)
    cand = torch.randint(0, V, (G, N - 1), device="cuda", generator=gen, dtype=torch.int32)
    u_test = torch.rand(N - 1, G, device="cuda", generator=gen)
    u_final = torch.rand(1, device="cuda", generator=gen)
    cap = P + 16
    kcap, vcap = torch.zeros((KV, cap, d), dtype=torch.bfloat16, device="cuda"), torch.zeros((KV, cap, d), dtype=torch.bfloat16, device="cuda")
    i32 = dict(dtype=torch.int32, device="cuda")

    def outputs():
        return dict(out=torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda"),
                    b0=torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda"),
                    b1=torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda"),
                    alen=torch.empty(G, **i32), acc=torch.empty((G, N - 1), **i32),
                    toks=torch.empty(N, **i32), n_out=torch.empty(1, **i32), best=torch.empty(1, **i32),
                    new=torch.empty(W, **i32), alen2=torch.empty(G, **i32),
                    stoks=torch.empty(N, **i32), sn=torch.empty(1, **i32))

    def calls(o):
        binding.la_step_attention(q, kc, vc, sk, sv, P, W, N, G, H, KV, d, o["out"])
        binding.la_step_attention_batch([dict(q=q, k_cache=kc, v_cache=vc, step_k=sk, step_v=sv, out=o["b0"], P=P),
                                         dict(q=q2, k_cache=kc2, v_cache=vc2, step_k=sk2, step_v=sv2, out=o["b1"], P=700)],
                                        W, N, G, H, KV, d)
        binding.la_verify(logits_cand, cand, G, N, V, o["alen"], o["acc"])
        binding.la_verify_step(logits_cur, logits_look, logits_cand, cand, W, N, G, V, o["toks"], o["n_out"], o["best"],
                               o["new"], o["alen2"])
        binding.la_verify_sample(logits_cur, logits_cand, cand, u_test, u_final, 1.0, N, G, V, o["stoks"], o["sn"])
        binding.la_kv_commit(kcap, vcap, sk, sv, P, W, N, G, KV, d, o["best"], o["n_out"])

    def plant():
        """New contents in the same buffers: random logits with a few candidate tokens made greedy."""
        for t in (q, kc, vc, sk, sv, q2, kc2, sk2):
            t.copy_(torch.randn(t.shape, device="cuda", generator=gen).bfloat16())
        for t in (logits_cur, logits_look, logits_cand):
            t.copy_(torch.randn(t.shape, device="cuda", generator=gen))
        u_test.copy_(torch.rand(u_test.shape, device="cuda", generator=gen))
        logits_cur[cand[0, 0].long()] = 30.0
        logits_cand[0, 0, cand[0, 1].long()] = 30.0
        kcap.zero_()
        vcap.zero_()

    eager = outputs()
    calls(eager)                      # (the first call sizes the library's workspace: not under capture)
    torch.cuda.synchronize()
    captured = outputs()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls(captured)
    for replay in range(4):
        plant()
        calls(eager)
        torch.cuda.synchronize()
        want_cache = kcap.clone()
        kcap.zero_()
        vcap.zero_()
        scratch = torch.randn(1 << 20, device="cuda", generator=gen).sum()     # unrelated work in between
        graph.replay()
        torch.cuda.synchronize()
        for name in eager:
            a, b = eager[name], captured[name]
            if name in ("toks", "stoks"):
                n = int(eager["n_out" if name == "toks" else "sn"].item())
                a, b = a[:n], b[:n]
            assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.int16) if b.dtype == torch.bfloat16 else b), (replay, name)
        assert torch.equal(kcap.view(torch.int16), want_cache.view(torch.int16)), replay
        assert int(eager["n_out"].item()) >= 2
        del scratch


def test_a_recorded_graph_survives_the_growth_of_the_workspace():
    """A graph names the workspace blocks of the time it was recorded.  Larger calls afterwards
    make the library allocate bigger blocks; the old ones must stay valid (and clean) for the
    graph's replays."""
    torch.cuda.synchronize()
    binding.la_shutdown()                       # start from an empty workspace
    s = wl.LLAMA2_7B
    W, N, G, V, H, KV, d, P, T = s.W, s.N, s.G, s.V, s.heads, s.kv_heads, s.head_dim, s.P, s.T
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)

    def rb(*shape):
        return torch.randn(shape, device="cuda", generator=gen).bfloat16()
    q, kc, vc, sk, sv = rb(T, H, d), rb(KV, P, d), rb(KV, P, d), rb(T, KV, d), rb(T, KV, d)
    logits = [torch.randn(shape, device="cuda", generator=gen) for shape in ((V,), (W, V), (G, N - 1, V))]
    cand = torch.randint(0, V, (G, N - 1), device="cuda", generator=gen, dtype=torch.int32)
    i32 = dict(dtype=torch.int32, device="cuda")

    def outputs():
        return [torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda"), torch.empty(N, **i32), torch.empty(1, **i32),
                torch.empty(1, **i32), torch.empty(W, **i32), torch.empty(G, **i32)]

    def calls(o):
        binding.la_step_attention(q, kc, vc, sk, sv, P, W, N, G, H, KV, d, o[0])
        binding.la_verify_step(*logits, cand, W, N, G, V, *o[1:])

    eager = outputs()
    calls(eager)
    torch.cuda.synchronize()
    captured = outputs()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls(captured)
    before = binding.la_step_attention_workspace_bytes(P, W, N, G, H, KV, d)

    # partial results of a much longer step, and the keys of 32 wide verification steps at once
    P2, W2 = 16000, 30
    T2 = 1 + 2 * W2 * (N - 1)
    assert binding.la_step_attention_workspace_bytes(P2, W2, N, W2, 64, 8, d) > max(before, 8 << 20)
    big = torch.empty((T2, 64, d), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention(rb(T2, 64, d), rb(8, P2, d), rb(8, P2, d), rb(T2, 8, d), rb(T2, 8, d), P2, W2, N, W2, 64, 8,
                              d, big)
    Wv, Gv, Vv = 1500, 1500, 16
    seqs = [dict(logits_cur=torch.randn(Vv, device="cuda", generator=gen),
                 logits_look=torch.randn(Wv, Vv, device="cuda", generator=gen),
                 logits_cand=torch.randn(Gv, N - 1, Vv, device="cuda", generator=gen),
                 cand_tokens=torch.randint(0, Vv, (Gv, N - 1), device="cuda", generator=gen, dtype=torch.int32),
                 out_tokens=torch.empty(N, **i32), n_out=torch.empty(1, **i32), best=torch.empty(1, **i32),
                 new_window=torch.empty(Wv, **i32)) for _ in range(32)]
    binding.la_verify_step_batch(seqs, Wv, N, Gv, Vv)          # 32 x 7501 keys: beyond the first block
    torch.cuda.synchronize()

    for replay in range(3):
        for t in (q, sk, sv):
            t.copy_(torch.randn(t.shape, device="cuda", generator=gen).bfloat16())
        logits[0].copy_(torch.randn(V, device="cuda", generator=gen))
        calls(eager)                                           # (uses the new blocks)
        graph.replay()                                         # (uses the old ones)
        torch.cuda.synchronize()
        assert torch.equal(eager[0].view(torch.int16), captured[0].view(torch.int16)), replay
        n = int(eager[2].item())
        assert int(captured[2].item()) == n and torch.equal(eager[1][:n], captured[1][:n]), replay
        for a, b in zip(eager[3:], captured[3:]):
            assert torch.equal(a, b), replay


def test_a_capture_that_would_have_to_grow_the_workspace_is_refused():
    """Growing the workspace allocates (and clears on the stream), which must not happen while the
    stream is being captured: such a call returns LA_EUNSUPPORTED, launches nothing and leaves the
    capture usable; after one call of the shape outside a capture, recording works."""
    torch.cuda.synchronize()
    binding.la_shutdown()                       # an empty workspace: any split step has to grow it
    s = wl.LLAMA2_7B
    W, N, G, H, KV, d, P, T = s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, s.P, s.T
    gen = torch.Generator(device="cuda")
    gen.manual_seed(13)

    def rb(*shape):
        return torch.randn(shape, device="cuda", generator=gen).bfloat16()
    q, kc, vc, sk, sv = rb(T, H, d), rb(KV, P, d), rb(KV, P, d), rb(T, KV, d), rb(T, KV, d)
    out = torch.zeros((T, H, d), dtype=torch.bfloat16, device="cuda")
    tiny_q, tiny_kv, tiny_out = rb(1, 1, 64), rb(1, 1, 64), torch.zeros((1, 1, 64), dtype=torch.bfloat16, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        with pytest.raises(binding.LaError) as e:
            binding.la_step_attention(q, kc, vc, sk, sv, P, W, N, G, H, KV, d, out)
        # a step that needs no workspace can still be recorded after the refusal
        binding.la_step_attention(tiny_q, None, None, tiny_kv, tiny_kv, 0, 0, 2, 0, 1, 1, 64, tiny_out)
    assert e.value.code == binding.LA_EUNSUPPORTED and "captured" in str(e.value)
    graph.replay()
    torch.cuda.synchronize()
    assert not out.any().item()                 # nothing of the refused call ran
    assert torch.equal(tiny_out, tiny_kv)       # one row that sees only itself: out = v
    eager = torch.empty_like(out)
    binding.la_step_attention(q, kc, vc, sk, sv, P, W, N, G, H, KV, d, eager)   # sizes the workspace
    torch.cuda.synchronize()
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph2):
        binding.la_step_attention(q, kc, vc, sk, sv, P, W, N, G, H, KV, d, out)
    graph2.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, eager)


def test_the_row_tile_kernel_in_a_graph_with_an_empty_workspace():
    """A short-prefix step takes the kernel that needs no workspace: it can be recorded with nothing
    allocated, and every replay (with eager work of the same library between the replays) gives the
    eager result, rotating form included."""
    torch.cuda.synchronize()
    binding.la_shutdown()
    s = wl.LLAMA2_7B_P256
    W, N, G, H, KV, d, P, T = s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, s.P, s.T
    assert binding.la_step_attention_kernel(P, W, N, G, H, KV, d) == 1
    gen = torch.Generator(device="cuda")
    gen.manual_seed(17)

    def rb(*shape):
        return torch.randn(shape, device="cuda", generator=gen).bfloat16()
    q, kc, vc, sk, sv = rb(T, H, d), rb(KV, P, d), rb(KV, P, d), rb(T, KV, d), rb(T, KV, d)
    cos, sin = [torch.from_numpy(t).cuda() for t in wl.rope_tables(P + W + N, d)]
    out, out_r = [torch.zeros((T, H, d), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.la_step_attention(q, kc, vc, sk, sv, P, W, N, G, H, KV, d, out)
        binding.la_step_attention_rope(q, kc, vc, sk, sv, cos, sin, P, W, N, G, H, KV, d, out_r, rotate_keys=True)
    eager, eager_r = torch.empty_like(out), torch.empty_like(out)
    binding.la_step_attention(q, kc, vc, sk, sv, P, W, N, G, H, KV, d, eager)
    binding.la_step_attention_rope(q, kc, vc, sk, sv, cos, sin, P, W, N, G, H, KV, d, eager_r, rotate_keys=True)
    torch.cuda.synchronize()
    for rep in range(4):
        out.zero_()
        out_r.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager) and torch.equal(out_r, eager_r), "replay %d" % rep
        binding.la_step_attention(q, kc, vc, sk, sv, P, W, N, G, H, KV, d, torch.empty_like(out))  # eager work between
        torch.cuda.synchronize()
    assert not torch.equal(eager, eager_r)
