"""GPU parity of la_step_attention_rows (the step over a subset of its rows: one device's share
under lookahead parallelism, Sec. 3.4) against the oracle, and against the full step."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, lookahead, workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


def bits(rng, shape):
    return wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


def run_rows(x, ids, P, W, N, G, H, KV, d):
    n = len(ids)
    out = torch.full((n, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention_rows(binding.bf16_tensor(x["q"][ids]), binding.bf16_tensor(x["k_cache"]) if P else None,
                                   binding.bf16_tensor(x["v_cache"]) if P else None,
                                   binding.bf16_tensor(x["step_k"][ids]), binding.bf16_tensor(x["step_v"][ids]),
                                   torch.from_numpy(np.asarray(ids, dtype=np.int32)).cuda(), P, W, N, G, H, KV, d, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    return got


@pytest.mark.parametrize("P,W,N,G,H,KV,d,parts", [
    (64, 4, 3, 2, 4, 4, 64, 2),
    (1024, 15, 5, 15, 32, 32, 128, 4),     # the 7B step on four devices
    (1024, 15, 5, 15, 32, 32, 128, 8),
    (4096, 7, 5, 7, 64, 8, 128, 2),        # the 70B step, grouped-query heads
    (300, 30, 5, 30, 8, 2, 128, 4),        # a wide window: shares of 95 rows
    (0, 6, 4, 6, 4, 2, 64, 3),
    (77, 5, 2, 5, 2, 1, 128, 5),           # N = 2: one level
])
def test_every_share_equals_the_full_step_on_its_rows(P, W, N, G, H, KV, d, parts):
    rng = np.random.default_rng(P + W * 10 + parts)
    T = 1 + (W + G) * (N - 1)
    x = dict(q=bits(rng, (T, H, d)), k_cache=bits(rng, (KV, P, d)), v_cache=bits(rng, (KV, P, d)),
             step_k=bits(rng, (T, KV, d)), step_v=bits(rng, (T, KV, d)))
    full = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], P, W, N, G, H, KV, d)
    seen = np.zeros(T, dtype=bool)
    for part in range(parts):
        ids = np.array(lookahead.lp_share(W, N, G, parts, part))
        print("case", dict(P=P, W=W, N=N, G=G, H=H, KV=KV, d=d, part="%d/%d" % (part, parts), rows=len(ids)), flush=True)
        got = run_rows(x, ids, P, W, N, G, H, KV, d)
        want = orc.step_attention_rows(x["q"][ids], x["k_cache"], x["v_cache"], x["step_k"][ids], x["step_v"][ids],
                                       ids, P, W, N, G, H, KV, d)
        assert np.abs(got - want).max() <= TOL
        assert np.abs(got - full[ids]).max() <= TOL          # nothing was needed from the other shares
        seen[ids] = True
    assert seen.all()


def test_arbitrary_subsets_and_orders():
    """Any subset in any order: the mask is evaluated pair by pair from the ids."""
    rng = np.random.default_rng(9)
    P, W, N, G, H, KV, d = 130, 9, 4, 6, 4, 2, 128
    T = 1 + (W + G) * (N - 1)
    x = dict(q=bits(rng, (T, H, d)), k_cache=bits(rng, (KV, P, d)), v_cache=bits(rng, (KV, P, d)),
             step_k=bits(rng, (T, KV, d)), step_v=bits(rng, (T, KV, d)))
    for n in (1, 2, 31, 33, T):
        ids = rng.permutation(T)[:n]
        if 0 not in ids:
            ids[0] = 0          # (a row that sees no key at all has no softmax)
        print("case rows", n, flush=True)
        got = run_rows(x, ids, P, W, N, G, H, KV, d)
        want = orc.step_attention_rows(x["q"][ids], x["k_cache"], x["v_cache"], x["step_k"][ids], x["step_v"][ids],
                                       ids, P, W, N, G, H, KV, d)
        assert np.abs(got - want).max() <= TOL


def test_all_rows_in_order_is_the_plain_step():
    s = wl.LLAMA2_13B
    x = wl.attention_inputs(s)
    dev = {k: binding.bf16_tensor(v) for k, v in x.items()}
    a = torch.empty((s.T, s.heads, s.head_dim), dtype=torch.bfloat16, device="cuda")
    b = torch.empty_like(a)
    binding.la_step_attention(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"], s.P, s.W, s.N,
                              s.G, s.heads, s.kv_heads, s.head_dim, a)
    binding.la_step_attention_rows(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"],
                                   torch.arange(s.T, dtype=torch.int32, device="cuda"), s.P, s.W, s.N, s.G, s.heads,
                                   s.kv_heads, s.head_dim, b)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_argument_errors():
    z = torch.zeros((5, 2, 64), dtype=torch.bfloat16, device="cuda")
    ids = torch.zeros(5, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.LaError):       # more rows than the layout has
        binding.la_step_attention_rows(z, None, None, z, z, ids, 0, 1, 2, 1, 2, 2, 64, z.clone())


def test_rows_recompute_path(override):
    """The same with the fallback of a split group that is not on one XCD forced."""
    override("force_recompute", "1")
    test_every_share_equals_the_full_step_on_its_rows(1024, 15, 5, 15, 32, 32, 128, 4)
    test_every_share_equals_the_full_step_on_its_rows(300, 30, 5, 30, 8, 2, 128, 4)
