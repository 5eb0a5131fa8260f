"""GPU parity of the paged-cache entry points: la_step_attention_paged against the oracle's
attention over the packed cache the block table stands for, la_kv_commit_paged bit-exactly against
the oracle's paged append."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2
NAN_BITS = np.uint16(0x7FC0)


def bits(rng, shape):
    return wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


def paged_copy(packed, table, page_size, n_pages):
    """Pages holding `packed` [kv, P, d] at the places `table` names; everything else is NaN."""
    kv, P, d = packed.shape
    pages = np.full((n_pages, kv, page_size, d), NAN_BITS, dtype=np.uint16)
    for i in range((P + page_size - 1) // page_size):
        lo, hi = i * page_size, min(P, (i + 1) * page_size)
        pages[table[i], :, :hi - lo] = packed[:, lo:hi]
    return pages


@pytest.mark.parametrize("P,page_size,W,N,G,H,KV,d", [
    (64, 64, 4, 3, 2, 4, 4, 64),
    (65, 64, 5, 4, 2, 4, 2, 128),          # one key in the second page
    (1024, 64, 15, 5, 15, 32, 32, 128),    # the 7B shape, a page per chunk
    (1024, 256, 15, 5, 15, 32, 32, 128),
    (1000, 128, 10, 5, 10, 8, 8, 128),     # ragged last page
    (4096, 512, 7, 5, 7, 64, 8, 128),      # the 70B shape
    (2500, 192, 5, 5, 5, 32, 8, 128),      # page of three chunks
    (333, 128, 3, 3, 3, 4, 2, 64),
    (0, 64, 3, 3, 1, 2, 2, 64),            # empty prefix: the table is not read
    (1, 64, 0, 2, 0, 2, 1, 64),
])
def test_paged_attention_matches_the_oracle(P, page_size, W, N, G, H, KV, d):
    print("case", dict(P=P, page=page_size, W=W, N=N, G=G, H=H, KV=KV, d=d), flush=True)
    rng = np.random.default_rng(P * 7 + page_size)
    T = 1 + (W + G) * (N - 1)
    x = dict(q=bits(rng, (T, H, d)), k_cache=bits(rng, (KV, P, d)), v_cache=bits(rng, (KV, P, d)),
             step_k=bits(rng, (T, KV, d)), step_v=bits(rng, (T, KV, d)))
    n_used = (P + page_size - 1) // page_size
    n_pages = n_used + 5
    table = rng.permutation(n_pages).astype(np.int32)        # entries past n_used are never read ...
    table_dev = table.copy()
    table_dev[n_used:] = 2 ** 30                              # ... so make them poisonous
    kp, vp = paged_copy(x["k_cache"], table, page_size, n_pages), paged_copy(x["v_cache"], table, page_size, n_pages)
    # the oracle sees the packed cache the pages stand for
    np.testing.assert_array_equal(orc.gather_pages(kp, table, P, page_size), x["k_cache"])
    want = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], P, W, N, G, H, KV, d)
    out = torch.full((T, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention_paged(binding.bf16_tensor(x["q"]), binding.bf16_tensor(kp), binding.bf16_tensor(vp),
                                    torch.from_numpy(table_dev).cuda() if P else None,
                                    binding.bf16_tensor(x["step_k"]), binding.bf16_tensor(x["step_v"]),
                                    P, W, N, G, H, KV, d, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= TOL


def test_paged_equals_packed_bit_for_bit():
    """Same keys, same plan: the paged and the packed call must give identical bits."""
    s = wl.LLAMA2_13B
    x = wl.attention_inputs(s)
    rng = np.random.default_rng(5)
    page_size = 128
    n_used = (s.P + page_size - 1) // page_size
    table = rng.permutation(n_used + 2).astype(np.int32)
    kp, vp = paged_copy(x["k_cache"], table, page_size, n_used + 2), paged_copy(x["v_cache"], table, page_size, n_used + 2)
    dev = {k: binding.bf16_tensor(v) for k, v in x.items()}
    a = torch.empty((s.T, s.heads, s.head_dim), dtype=torch.bfloat16, device="cuda")
    b = torch.empty_like(a)
    binding.la_step_attention(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"], s.P, s.W, s.N,
                              s.G, s.heads, s.kv_heads, s.head_dim, a)
    binding.la_step_attention_paged(dev["q"], binding.bf16_tensor(kp), binding.bf16_tensor(vp),
                                    torch.from_numpy(table).cuda(), dev["step_k"], dev["step_v"], s.P, s.W, s.N, s.G,
                                    s.heads, s.kv_heads, s.head_dim, b)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("W,N,G,KV,d,P,page_size", [
    (15, 5, 15, 32, 128, 1024, 64),     # the append starts a new page
    (15, 5, 15, 32, 128, 1022, 64),     # ... straddles two pages
    (7, 5, 7, 8, 128, 4000, 256),
    (4, 3, 2, 4, 64, 60, 64),
    (0, 4, 3, 1, 64, 0, 64),
])
def test_paged_commit_matches_the_oracle(W, N, G, KV, d, P, page_size):
    rng = np.random.default_rng(W + N + G + P)
    T = 1 + (W + G) * (N - 1)
    step_k, step_v = bits(rng, (T, KV, d)), bits(rng, (T, KV, d))
    n_used = (P + N + page_size - 1) // page_size
    n_pages = n_used + 3
    table = rng.permutation(n_pages).astype(np.int32)
    base_k, base_v = bits(rng, (n_pages, KV, page_size, d)), bits(rng, (n_pages, KV, page_size, d))
    sk, sv = binding.bf16_tensor(step_k), binding.bf16_tensor(step_v)
    tab = torch.from_numpy(table).cuda()
    outcomes = [(0 if G else -1, 1)] + [(g, n) for g in sorted({0, G - 1}) for n in range(2, N + 1)]
    for best, n_out in outcomes:
        print("case", dict(W=W, N=N, G=G, KV=KV, d=d, P=P, page=page_size, best=best, n_out=n_out), flush=True)
        want_k, want_v = base_k.copy(), base_v.copy()
        orc.kv_commit_paged(want_k, want_v, table, page_size, step_k, step_v, P, W, N, G, best, n_out)
        kp, vp = binding.bf16_tensor(base_k), binding.bf16_tensor(base_v)
        binding.la_kv_commit_paged(kp, vp, tab, sk, sv, P, W, N, G, KV, d,
                                   torch.tensor([best], dtype=torch.int32, device="cuda"),
                                   torch.tensor([n_out], dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(binding.bf16_bits(kp), want_k)
        np.testing.assert_array_equal(binding.bf16_bits(vp), want_v)


def test_argument_errors():
    z = torch.zeros((2, 2, 64, 64), dtype=torch.bfloat16, device="cuda")
    bad = torch.zeros((2, 2, 96, 64), dtype=torch.bfloat16, device="cuda")      # page of 96 keys
    st = torch.zeros((5, 2, 64), dtype=torch.bfloat16, device="cuda")
    tab = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.LaError):
        binding.la_step_attention_paged(st, bad, bad, tab, st, st, 10, 1, 3, 1, 2, 2, 64, st.clone())
    with pytest.raises(ValueError):                                             # table too short for P
        binding.la_step_attention_paged(st, z, z, tab[:1], st, st, 100, 1, 3, 1, 2, 2, 64, st.clone())


def test_every_paged_plan():
    """Every kernel variant compiled for a paged cache (a plan that is not compiled for it, the
    first one here, falls back to the default), with a page per chunk and all stages up front."""
    import os
    P, page_size, W, N, G, H, KV, d = 1500, 64, 5, 5, 5, 8, 8, 128
    rng = np.random.default_rng(3)
    T = 1 + (W + G) * (N - 1)
    x = dict(q=bits(rng, (T, H, d)), k_cache=bits(rng, (KV, P, d)), v_cache=bits(rng, (KV, P, d)),
             step_k=bits(rng, (T, KV, d)), step_v=bits(rng, (T, KV, d)))
    n_used = (P + page_size - 1) // page_size
    table = rng.permutation(n_used + 4).astype(np.int32)
    kp, vp = paged_copy(x["k_cache"], table, page_size, n_used + 4), paged_copy(x["v_cache"], table, page_size, n_used + 4)
    want = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], P, W, N, G, H, KV, d)
    for plan in ("2,2,2,9,32,9", "2,4,1,4,64,4", "4,2,2,4,64,4", "1,2,3,4,64"):
        print("case plan", plan, flush=True)
        binding.la_debug_override("attn_plan", plan)
        try:
            out = torch.full((T, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
            binding.la_step_attention_paged(binding.bf16_tensor(x["q"]), binding.bf16_tensor(kp), binding.bf16_tensor(vp),
                                            torch.from_numpy(table).cuda(), binding.bf16_tensor(x["step_k"]),
                                            binding.bf16_tensor(x["step_v"]), P, W, N, G, H, KV, d, out)
            torch.cuda.synchronize()
        finally:
            binding.la_debug_override("attn_plan", None)
        got = out.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all() and np.abs(got - want).max() <= TOL, plan


def test_paged_recompute_path(override):
    """The fallback of a split group that is not on one XCD (the last workgroup walks every chunk
    again, through the block table) with a paged cache."""
    override("force_recompute", "1")
    test_paged_attention_matches_the_oracle(1000, 128, 10, 5, 10, 8, 8, 128)
    test_paged_attention_matches_the_oracle(1024, 64, 15, 5, 15, 32, 32, 128)
