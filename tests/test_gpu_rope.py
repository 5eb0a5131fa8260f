"""GPU parity: la_step_rope (HIP, through the C ABI) against the oracle's step_rope.  Inputs are
bf16, the kernel computes in fp32 and rounds once: the result must be the oracle's fp64 value up
to that rounding (half a unit in the last place of bf16: at most 2^-8 of the value, which is no
larger than the pair's norm) plus fp32 arithmetic."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu


def run_case(P, W, N, G, H, KV, d, interleaved, max_pos=None, seed=0):
    print("case", dict(P=P, W=W, N=N, G=G, H=H, KV=KV, d=d, interleaved=interleaved), flush=True)
    rng = np.random.default_rng(seed + P + d)
    T = 1 + (W + G) * (N - 1)
    reach = P + max(W + N - 2 if W else 0, N - 1 if (W or G) else 0)
    max_pos = max_pos or reach + 1
    cos, sin = wl.rope_tables(max_pos, d)
    qb = wl.f32_to_bf16_bits(rng.standard_normal((T, H, d), dtype=np.float32) * 3)
    kb = wl.f32_to_bf16_bits(rng.standard_normal((T, KV, d), dtype=np.float32) * 3)
    q, k = binding.bf16_tensor(qb), binding.bf16_tensor(kb)
    binding.la_step_rope(q, k, torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda(), P, W, N, G, H, KV, d,
                         interleaved)
    torch.cuda.synchronize()
    x64, k64 = orc.bf16_to_f64(qb), orc.bf16_to_f64(kb)
    want_q, want_k = orc.step_rope(x64, k64, cos, sin, P, W, N, G, interleaved)
    for got, want, x in ((q, want_q, x64), (k, want_k, k64)):
        got = got.float().cpu().numpy().astype(np.float64)
        if interleaved:
            norm = np.repeat(np.hypot(x[..., 0::2], x[..., 1::2]), 2, axis=-1)
        else:
            h = np.hypot(x[..., :d // 2], x[..., d // 2:])
            norm = np.concatenate([h, h], axis=-1)
        assert (np.abs(got - want) <= norm * (2.0 ** -8 + 1e-6) + 1e-30).all()
        # sharper: nearly every element IS the oracle's value rounded to bf16 (fp32 arithmetic can
        # land on the other side of a rounding boundary now and then, one unit away at most)
        nearest = orc.bf16_to_f64(wl.f32_to_bf16_bits(want.astype(np.float32)))
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(nearest), 1e-30))) - 7)
        assert (np.abs(got - nearest) <= ulp + norm * 2.0 ** -21).all()   # (a result near zero has a tiny ulp;
        #                                                                   the fp32 products do not)
        assert (got == nearest).mean() > 0.99


@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("P,W,N,G,H,KV,d", [
    (1024, 15, 5, 15, 32, 32, 128),          # the 7B shape
    (4096, 7, 5, 7, 64, 8, 128),             # GQA
    (0, 5, 4, 2, 2, 1, 64),                  # the layout of Fig. 2(b), empty prefix
    (17, 0, 3, 4, 3, 3, 16),                 # no window
    (17, 4, 2, 0, 3, 1, 32),                 # no candidates, N = 2
    (5, 0, 2, 0, 1, 1, 256),                 # a plain decode token
    (300, 30, 5, 30, 8, 2, 128),
])
def test_against_the_oracle(P, W, N, G, H, KV, d, interleaved):
    run_case(P, W, N, G, H, KV, d, interleaved)


def test_tables_longer_than_needed_and_argument_errors():
    run_case(10, 3, 3, 2, 2, 2, 64, False, max_pos=4096)
    T = 1 + 5 * 2
    q = torch.zeros((T, 2, 64), dtype=torch.bfloat16, device="cuda")
    cos = torch.zeros((12, 32), device="cuda")
    with pytest.raises(binding.LaError, match="positions"):        # the step reaches position 10 + 4
        binding.la_step_rope(q, q.clone(), cos, cos, 10, 3, 3, 2, 2, 2, 64)


def test_rope_then_attention_scores_do_not_depend_on_the_prefix_length():
    """End to end through two kernels: rotate q and keys, attend with an EMPTY prefix (only step
    keys), once at P = 0 and once 'at' P = 777 (the tables shifted): the outputs agree, because
    every score depends on the distance of the two rows only."""
    W, N, G, H, KV, d = 5, 4, 2, 4, 2, 128
    T = 1 + (W + G) * (N - 1)
    rng = np.random.default_rng(5)
    qb = wl.f32_to_bf16_bits(rng.standard_normal((T, H, d), dtype=np.float32))
    kb = wl.f32_to_bf16_bits(rng.standard_normal((T, KV, d), dtype=np.float32))
    vb = wl.f32_to_bf16_bits(rng.standard_normal((T, KV, d), dtype=np.float32))
    cos, sin = [torch.from_numpy(x).cuda() for x in wl.rope_tables(1024, d)]
    outs = []
    for P in (0, 777):
        q, k, v = binding.bf16_tensor(qb), binding.bf16_tensor(kb), binding.bf16_tensor(vb)
        binding.la_step_rope(q, k, cos, sin, P, W, N, G, H, KV, d)
        out = torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda")
        binding.la_step_attention(q, None, None, k, v, 0, W, N, G, H, KV, d, out)
        torch.cuda.synchronize()
        outs.append(out.float().cpu().numpy())
    assert np.abs(outs[0] - outs[1]).max() <= 2e-2
