"""GPU parity of la_step_attention_batch: several steps in one launch must give, per sequence,
the oracle's step (and agree with one la_step_attention call per sequence)."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


def bits(rng, shape):
    return wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


def make_seq(rng, P, T, H, KV, d):
    x = dict(q=bits(rng, (T, H, d)), k_cache=bits(rng, (KV, P, d)), v_cache=bits(rng, (KV, P, d)),
             step_k=bits(rng, (T, KV, d)), step_v=bits(rng, (T, KV, d)))
    dev = {k: (binding.bf16_tensor(v) if v.size else None) for k, v in x.items()}
    dev["P"] = P
    dev["out"] = torch.full((T, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    return x, dev


def run_batch(prefixes, W, N, G, H, KV, d, seed, check_oracle):
    rng = np.random.default_rng(seed)
    T = 1 + (W + G) * (N - 1)
    seqs = [make_seq(rng, P, T, H, KV, d) for P in prefixes]
    binding.la_step_attention_batch([dev for _, dev in seqs], W, N, G, H, KV, d)
    torch.cuda.synchronize()
    for i, (x, dev) in enumerate(seqs):
        got = dev["out"].float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all(), i
        single = torch.empty_like(dev["out"])
        binding.la_step_attention(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"], dev["P"],
                                  W, N, G, H, KV, d, single)
        torch.cuda.synchronize()
        assert np.abs(got - single.float().cpu().numpy()).max() <= TOL, i
        if i in check_oracle:
            want = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], dev["P"], W, N, G,
                                      H, KV, d)
            assert np.abs(got - want).max() <= TOL, i
            print("  sequence %d (P=%d): oracle agrees" % (i, dev["P"]), flush=True)


@pytest.mark.parametrize("prefixes,W,N,G,H,KV,d", [
    ([1024] * 8, 15, 5, 15, 32, 32, 128),                       # eight 7B-shaped steps
    (wl.ragged_prefix_lengths(), 5, 5, 5, 32, 8, 128),           # the ragged sweep, W = 5
    (wl.ragged_prefix_lengths(), 15, 5, 15, 32, 8, 128),
    ([300], 4, 3, 2, 4, 4, 64),                                  # a batch of one
    ([0, 64, 1, 65, 700], 4, 3, 2, 4, 2, 64),                    # empty and tiny prefixes, head_dim 64
    ([100 * i + 7 for i in range(11)], 7, 5, 7, 8, 2, 128),      # more than one launch (eight at a time)
    ([5000, 13], 10, 5, 10, 16, 16, 128),
    ([16000, 16000, 9000], 30, 5, 30, 32, 8, 128),               # the 128-row plan for all
])
def test_batch_matches_the_oracle_and_the_single_calls(prefixes, W, N, G, H, KV, d):
    print("case", dict(prefixes=list(prefixes), W=W, N=N, G=G, H=H, KV=KV, d=d), flush=True)
    # the oracle on the shortest and the longest sequence (it is slow on long prefixes)
    order = np.argsort(prefixes)
    run_batch(list(prefixes), W, N, G, H, KV, d, seed=len(prefixes) + W, check_oracle={int(order[0]), int(order[-1])})


@pytest.mark.timeout(600)
@pytest.mark.parametrize("W", list(wl.RAGGED_W))
def test_ragged_sweep_every_sequence_against_the_oracle(W):
    """Every point of the ragged sweep (8 sequences x 5 window widths): one launch over all eight
    sequences per width, the oracle on each of them."""
    prefixes = list(wl.ragged_prefix_lengths())
    print("case", dict(prefixes=prefixes, W=W), flush=True)
    run_batch(prefixes, W, 5, W, 32, 8, 128, seed=40 + W, check_oracle=set(range(len(prefixes))))


def test_batch_recompute_path(override):
    override("force_recompute", "1")
    run_batch([2492, 13246, 1253], 5, 5, 5, 32, 8, 128, seed=1, check_oracle={2})


def test_argument_errors():
    q = torch.zeros((5, 3, 64), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((5, 2, 64), dtype=torch.bfloat16, device="cuda")
    seq = dict(q=q, k_cache=None, v_cache=None, step_k=kv, step_v=kv, out=q.clone(), P=0)
    with pytest.raises(binding.LaError):
        binding.la_step_attention_batch([seq], 1, 3, 1, 3, 2, 64)      # 3 query heads on 2 KV heads
    with pytest.raises(binding.LaError):
        binding.la_step_attention_batch([], 1, 3, 1, 2, 2, 64)         # no descriptors


@pytest.mark.parametrize("plan", ["2", "4"])
def test_both_batch_decompositions(override, plan):
    """64-row and 128-row workgroups (the batch_plan hook overrides the choice the library makes)."""
    override("batch_plan", plan)
    run_batch([1024, 900, 64, 3000], 15, 5, 15, 32, 32, 128, seed=3, check_oracle={2, 3})
    run_batch([500, 2000], 4, 5, 4, 32, 8, 128, seed=4, check_oracle={0})


@pytest.mark.parametrize("prefixes,page_size,W,N,G,H,KV,d", [
    ([1024] * 8, 64, 15, 5, 15, 32, 32, 128),
    ([2492, 13246, 1253, 7849], 256, 5, 5, 5, 32, 8, 128),
    ([0, 64, 1, 65, 700], 64, 4, 3, 2, 4, 2, 64),
    ([900, 10], 128, 10, 5, 10, 16, 16, 128),
])
def test_paged_batch(prefixes, page_size, W, N, G, H, KV, d):
    """All sequences in one pool of pages, each with its own block table: per sequence the oracle's
    step over the packed cache its table stands for, and the bits of the packed batch."""
    print("case", dict(prefixes=prefixes, page=page_size, W=W, N=N, G=G, H=H, KV=KV, d=d), flush=True)
    rng = np.random.default_rng(sum(prefixes) + page_size)
    T = 1 + (W + G) * (N - 1)
    seqs = [make_seq(rng, P, T, H, KV, d) for P in prefixes]
    used = [(P + page_size - 1) // page_size for P in prefixes]
    n_pages = sum(used) + 3
    perm = rng.permutation(n_pages).astype(np.int32)
    kp = np.full((n_pages, KV, page_size, d), 0x7FC0, dtype=np.uint16)       # NaN wherever nothing was put
    vp = kp.copy()
    tables, at = [], 0
    for (x, _), P, n in zip(seqs, prefixes, used):
        table = perm[at:at + n]
        at += n
        for i in range(n):
            lo, hi = i * page_size, min(P, (i + 1) * page_size)
            kp[table[i], :, :hi - lo] = x["k_cache"][:, lo:hi]
            vp[table[i], :, :hi - lo] = x["v_cache"][:, lo:hi]
        np.testing.assert_array_equal(orc.gather_pages(kp, table, P, page_size), x["k_cache"])
        tables.append(torch.from_numpy(np.ascontiguousarray(table)).cuda() if n else None)
    packed_out = []
    binding.la_step_attention_batch([dev for _, dev in seqs], W, N, G, H, KV, d)
    torch.cuda.synchronize()
    for _, dev in seqs:
        packed_out.append(dev["out"].clone())
        dev["out"].fill_(float("nan"))
    descs = [dict(q=dev["q"], block_table=t, step_k=dev["step_k"], step_v=dev["step_v"], out=dev["out"], P=dev["P"])
             for (_, dev), t in zip(seqs, tables)]
    binding.la_step_attention_batch_paged(descs, binding.bf16_tensor(kp), binding.bf16_tensor(vp), W, N, G, H, KV, d)
    torch.cuda.synchronize()
    order = np.argsort(prefixes)
    for i, (x, dev) in enumerate(seqs):
        assert torch.equal(dev["out"].view(torch.int16), packed_out[i].view(torch.int16)), i
        if i in (int(order[0]), int(order[-1])):
            want = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], dev["P"], W, N, G,
                                      H, KV, d)
            assert np.abs(dev["out"].float().cpu().numpy() - want).max() <= TOL, i
