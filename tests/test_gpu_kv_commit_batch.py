"""GPU parity of la_kv_commit_batch (several appends in one launch: the layers of a model after a
step, several sequences, packed and paged caches side by side) bit-exactly against the oracle's
append applied descriptor by descriptor."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def bits(rng, shape):
    return wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


def as_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("layers,W,N,G,KV,d,P,cap", [
    (32, 15, 5, 15, 32, 128, 1024, 1040),   # every layer of the 7B shape, one launch
    (80, 7, 5, 7, 8, 128, 300, 305),        # more layers than one launch carries; exactly room for N
    (3, 4, 3, 2, 4, 64, 0, 8),
    (1, 5, 2, 5, 2, 256, 10, 64),
])
@pytest.mark.parametrize("outcome", ["first", "full", "middle"])
def test_layers_share_one_result(layers, W, N, G, KV, d, P, cap, outcome):
    """One (best, n_out) on the device drives the append of every layer."""
    best, n_out = {"first": (0, 1), "full": (G - 1, N), "middle": (G // 2, max(1, N // 2))}[outcome]
    print("case", dict(layers=layers, W=W, N=N, G=G, KV=KV, d=d, P=P, cap=cap, best=best, n_out=n_out), flush=True)
    rng = np.random.default_rng(layers * 7 + N)
    T = 1 + (W + G) * (N - 1)
    b = torch.tensor([best], dtype=torch.int32, device="cuda")
    n = torch.tensor([n_out], dtype=torch.int32, device="cuda")
    appends, want = [], []
    for _ in range(layers):
        step_k, step_v = bits(rng, (T, KV, d)), bits(rng, (T, KV, d))
        base_k, base_v = bits(rng, (KV, cap, d)), bits(rng, (KV, cap, d))
        wk, wv = base_k.copy(), base_v.copy()
        orc.kv_commit(wk, wv, step_k, step_v, P, W, N, G, best, n_out)
        want.append((wk, wv))
        appends.append(dict(k_cache=binding.bf16_tensor(base_k), v_cache=binding.bf16_tensor(base_v),
                            step_k=binding.bf16_tensor(step_k), step_v=binding.bf16_tensor(step_v),
                            best=b, n_out=n, P=P))
    binding.la_kv_commit_batch(appends, W, N, G, KV, d)
    torch.cuda.synchronize()
    for x, (wk, wv) in zip(appends, want):
        np.testing.assert_array_equal(as_bits(x["k_cache"]), wk)
        np.testing.assert_array_equal(as_bits(x["v_cache"]), wv)


def test_sequences_with_their_own_results_packed_and_paged():
    """Every descriptor its own prefix length and its own (best, n_out); even ones packed, odd
    ones in a shared pool of shuffled pages."""
    W, N, G, KV, d, page = 5, 4, 3, 2, 128, 64
    T = 1 + (W + G) * (N - 1)
    rng = np.random.default_rng(11)
    n_seq, n_pages = 9, 40
    pool_k, pool_v = bits(rng, (n_pages, KV, page, d)), bits(rng, (n_pages, KV, page, d))
    want_pk, want_pv = pool_k.copy(), pool_v.copy()
    pk, pv = binding.bf16_tensor(pool_k), binding.bf16_tensor(pool_v)
    free = list(rng.permutation(n_pages))
    appends, checks = [], []
    for s in range(n_seq):
        P = int(rng.integers(0, 3 * page - N))
        best, n_out = int(rng.integers(0, G)), int(rng.integers(1, N + 1))
        step_k, step_v = bits(rng, (T, KV, d)), bits(rng, (T, KV, d))
        x = dict(step_k=binding.bf16_tensor(step_k), step_v=binding.bf16_tensor(step_v), P=P,
                 best=torch.tensor([best], dtype=torch.int32, device="cuda"),
                 n_out=torch.tensor([n_out], dtype=torch.int32, device="cuda"))
        print("case", dict(seq=s, P=P, best=best, n_out=n_out, paged=bool(s % 2)), flush=True)
        if s % 2:
            table = np.array([free.pop() for _ in range((P + N + page - 1) // page)], dtype=np.int32)
            orc.kv_commit_paged(want_pk, want_pv, table, page, step_k, step_v, P, W, N, G, best, n_out)
            x.update(k_cache=pk, v_cache=pv, block_table=torch.from_numpy(table).cuda())
        else:
            cap = P + N + int(rng.integers(0, 5))
            base_k, base_v = bits(rng, (KV, cap, d)), bits(rng, (KV, cap, d))
            wk, wv = base_k.copy(), base_v.copy()
            orc.kv_commit(wk, wv, step_k, step_v, P, W, N, G, best, n_out)
            x.update(k_cache=binding.bf16_tensor(base_k), v_cache=binding.bf16_tensor(base_v))
            checks.append((x, wk, wv))
        appends.append(x)
    binding.la_kv_commit_batch(appends, W, N, G, KV, d)
    torch.cuda.synchronize()
    for x, wk, wv in checks:
        np.testing.assert_array_equal(as_bits(x["k_cache"]), wk)
        np.testing.assert_array_equal(as_bits(x["v_cache"]), wv)
    np.testing.assert_array_equal(as_bits(pk), want_pk)     # pages no table names are untouched
    np.testing.assert_array_equal(as_bits(pv), want_pv)


def test_equals_the_single_calls_after_a_real_verification():
    """la_verify_step's device-side result drives one batched append and, on copies, one
    la_kv_commit per layer: the caches agree bit for bit."""
    s = wl.LLAMA2_13B
    layers = 5
    cur, look, cnd, cand, _ = wl.verify_step_inputs(s)
    outs = [torch.empty((n,), dtype=torch.int32, device="cuda") for n in (s.N, 1, 1, s.W, s.G)]
    binding.la_verify_step(*[torch.from_numpy(a).cuda() for a in (cur, look, cnd, cand)], s.W, s.N, s.G, s.V, *outs)
    rng = np.random.default_rng(3)
    cap = s.P + s.N
    appends, singles = [], []
    for _ in range(layers):
        sk = binding.bf16_tensor(bits(rng, (s.T, s.kv_heads, s.head_dim)))
        sv = binding.bf16_tensor(bits(rng, (s.T, s.kv_heads, s.head_dim)))
        kc = binding.bf16_tensor(bits(rng, (s.kv_heads, cap, s.head_dim)))
        vc = binding.bf16_tensor(bits(rng, (s.kv_heads, cap, s.head_dim)))
        singles.append((kc.clone(), vc.clone(), sk, sv))
        appends.append(dict(k_cache=kc, v_cache=vc, step_k=sk, step_v=sv, best=outs[2], n_out=outs[1], P=s.P))
    binding.la_kv_commit_batch(appends, s.W, s.N, s.G, s.kv_heads, s.head_dim)
    for kc, vc, sk, sv in singles:
        binding.la_kv_commit(kc, vc, sk, sv, s.P, s.W, s.N, s.G, s.kv_heads, s.head_dim, outs[2], outs[1])
    torch.cuda.synchronize()
    for x, (kc, vc, _, _) in zip(appends, singles):
        assert torch.equal(x["k_cache"].view(torch.int16), kc.view(torch.int16))
        assert torch.equal(x["v_cache"].view(torch.int16), vc.view(torch.int16))
