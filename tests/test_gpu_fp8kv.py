"""GPU parity: la_step_attention_fp8kv (8-bit float keys and values with one scale per KV head, through
the C ABI) against the fp64 oracle of the same step.

Bar: max abs error <= 2e-2, the bar of the 16-bit step: the codes are converted exactly, so the
kernel's rounding is the same (scores and sums in fp32, probabilities and outputs in bf16)."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


def run_hip(x, P, W, N, G, H, KV, d):
    T = 1 + (W + G) * (N - 1)
    dev = {k: torch.from_numpy(np.ascontiguousarray(x[k])).cuda() for k in ("k_cache", "v_cache", "step_k", "step_v",
                                                                             "k_scale", "v_scale")}
    q = binding.bf16_tensor(x["q"])
    out = torch.full((T, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention_fp8kv(q, dev["k_cache"] if P else None, dev["v_cache"] if P else None, dev["step_k"],
                                    dev["step_v"], dev["k_scale"], dev["v_scale"], P, W, N, G, H, KV, d, out)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


def run_oracle(x, P, W, N, G, H, KV, d):
    return orc.step_attention_fp8kv(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], x["k_scale"],
                                    x["v_scale"], P, W, N, G, H, KV, d)


def rand_inputs(seed, P, W, N, G, H, KV, d):
    """N(0,1) draws quantised per KV head as the seeded workloads are (largest magnitude -> 448)."""
    rng = np.random.default_rng(seed)
    T = 1 + (W + G) * (N - 1)
    f = lambda shape: rng.standard_normal(size=shape, dtype=np.float32)
    kc, vc, sk, sv = f((KV, P, d)), f((KV, P, d)), f((T, KV, d)), f((T, KV, d))
    ks = (np.maximum(np.abs(kc).max(axis=(1, 2), initial=0.0), np.abs(sk).max(axis=(0, 2))) / wl.FP8_MAX).astype(np.float32)
    vs = (np.maximum(np.abs(vc).max(axis=(1, 2), initial=0.0), np.abs(sv).max(axis=(0, 2))) / wl.FP8_MAX).astype(np.float32)
    return dict(q=wl.f32_to_bf16_bits(f((T, H, d))),
                k_cache=wl.quantize_fp8(kc, ks[:, None, None]), v_cache=wl.quantize_fp8(vc, vs[:, None, None]),
                step_k=wl.quantize_fp8(sk, ks[None, :, None]), step_v=wl.quantize_fp8(sv, vs[None, :, None]),
                k_scale=ks, v_scale=vs)


def check(x, P, W, N, G, H, KV, d, tag=""):
    print("case", tag, dict(P=P, W=W, N=N, G=G, H=H, KV=KV, d=d), flush=True)
    got = run_hip(x, P, W, N, G, H, KV, d)
    want = run_oracle(x, P, W, N, G, H, KV, d)
    assert np.isfinite(got).all(), "non-finite or unwritten output"
    err = np.abs(got - want).max()
    assert err <= TOL, "max abs err %g" % err
    return err


def test_tiny_config():
    s = wl.TINY
    check(wl.attention_inputs_fp8(s), s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, "tiny")


SMALL = [
    # P, W, N, G, H, KV, d
    (0, 0, 2, 0, 1, 1, 64),      # a single row that sees only itself
    (0, 3, 3, 2, 2, 2, 64),      # no prefix at all
    (1, 0, 2, 0, 4, 2, 128),     # one-token decode over 2 keys, grouped heads
    (63, 4, 3, 2, 4, 4, 64),
    (64, 4, 3, 2, 4, 4, 128),
    (65, 5, 4, 2, 4, 2, 128),    # ragged last prefix chunk
    (200, 0, 5, 6, 8, 2, 128),   # verification branch only
    (200, 7, 5, 0, 8, 2, 128),   # lookahead branch only
    (333, 15, 5, 15, 4, 4, 128), # T = 121: several row tiles, two step chunks
    (517, 3, 7, 3, 16, 2, 128),  # group of 8 heads per KV head
    (129, 30, 5, 30, 2, 2, 64),  # T = 241, head_dim 64
    (1000, 1, 3, 1, 24, 8, 128),
    (4200, 20, 5, 20, 32, 2, 128),  # many rows per KV head on a long prefix: the 128-row workgroups
]


@pytest.mark.parametrize("P,W,N,G,H,KV,d", SMALL)
def test_small_shapes(P, W, N, G, H, KV, d):
    check(rand_inputs(P * 7 + W * 3 + G + d, P, W, N, G, H, KV, d), P, W, N, G, H, KV, d)


@pytest.mark.parametrize("shape", [wl.LLAMA2_7B, wl.LLAMA2_13B, wl.LLAMA2_70B], ids=lambda s: s.name)
def test_paper_configs_full_size(shape):
    s = shape
    check(wl.attention_inputs_fp8(s), s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, s.name)


@pytest.mark.parametrize("seq,W", [(2, 5), (7, 30)])
def test_ragged_sweep_points(seq, W):
    """The shortest sequence at the narrowest window and the longest at the widest."""
    s = wl.ragged_shape(seq, W)
    check(wl.attention_inputs_fp8(s, extra=seq), s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, s.name)


def test_exactly_representable_case_is_the_16_bit_step(override):
    """Scales that are powers of two: the same numbers as bf16 tensors through la_step_attention give the
    same output bits (the conversion of the codes is exact and the scales only move exponents)."""
    override("attn_rowtile", "0")  # the 16-bit step through the staged kernel, which the 8-bit one is a variant of
    P, W, N, G, H, KV, d = 300, 6, 4, 3, 8, 4, 128
    x = rand_inputs(8, P, W, N, G, H, KV, d)
    x["k_scale"] = np.ldexp(1.0, np.array([-6, -5, -7, -6])).astype(np.float32)
    x["v_scale"] = np.ldexp(1.0, np.array([-7, -6, -6, -5])).astype(np.float32)
    got = run_hip(x, P, W, N, G, H, KV, d)
    dec = lambda c, s, axis: (orc.fp8_e4m3_decode(c) * np.expand_dims(s.astype(np.float64), tuple(a for a in range(3) if a != axis))).astype(np.float32)
    y = dict(q=x["q"], k_cache=wl.f32_to_bf16_bits(dec(x["k_cache"], x["k_scale"], 0)),
             v_cache=wl.f32_to_bf16_bits(dec(x["v_cache"], x["v_scale"], 0)),
             step_k=wl.f32_to_bf16_bits(dec(x["step_k"], x["k_scale"], 1)),
             step_v=wl.f32_to_bf16_bits(dec(x["step_v"], x["v_scale"], 1)))
    dev = {k: binding.bf16_tensor(v) for k, v in y.items()}
    out = torch.empty((1 + (W + G) * (N - 1), H, d), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"], P, W, N, G, H,
                              KV, d, out)
    torch.cuda.synchronize()
    ref = out.float().cpu().numpy().astype(np.float64)
    # the reference of the running maximum moves at the same blocks in both, so only the last
    # rounding (scale applied before or after the division) can differ: one bf16 step
    assert np.abs(got - ref).max() <= 2.0 ** -8 * max(1.0, np.abs(ref).max())
    assert np.abs(got - run_oracle(x, P, W, N, G, H, KV, d)).max() <= TOL


def test_every_code_point_as_a_value():
    """A key that dominates hands the row its value row: 256 value rows holding every code (NaN codes
    replaced) come back as code * scale, rounded to bf16."""
    P, H, KV, d = 256, 2, 2, 128
    rng = np.random.default_rng(3)
    x = rand_inputs(4, P, 0, 2, 0, H, KV, d)
    codes = np.arange(256, dtype=np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x00
    for kvh in range(KV):
        x["v_cache"][kvh] = np.roll(codes, kvh * 17)[(np.arange(P)[:, None] + np.arange(d)[None, :]) % 256]
    x["v_scale"] = np.array([0.75, 1.5], dtype=np.float32)
    want = run_oracle(x, P, 0, 2, 0, H, KV, d)
    got = run_hip(x, P, 0, 2, 0, H, KV, d)
    assert np.abs(got - want).max() <= TOL * max(1.0, np.abs(want).max())
    # and one row read out exactly: make key 100 of every head dominate
    x["k_cache"][:] = 0
    x["step_k"][:] = 0
    qf = np.zeros((1, H, d), dtype=np.float32)
    qf[0, :, 5] = 256.0
    x["q"] = wl.f32_to_bf16_bits(qf)
    x["k_cache"][:, 100, 5] = 0x7E   # 448
    x["k_scale"] = np.array([1.0, 1.0], dtype=np.float32)
    got = run_hip(x, P, 0, 2, 0, H, KV, d)
    for h in range(H):
        want_row = orc.fp8_e4m3_decode(x["v_cache"][h, 100]) * float(x["v_scale"][h])
        np.testing.assert_array_equal(got[0, h], wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(want_row.astype(np.float32))))


@pytest.mark.parametrize("plan", ["2,2,0,4,64", "2,4,2,4,64", "2,4,7,4,64", "1,2,0,4,64", "4,2,0,4,64"])
def test_other_decompositions(override, plan):
    override("attn_plan", plan)
    P, W, N, G, H, KV, d = 700, 10, 5, 10, 8, 4, 128
    check(rand_inputs(21, P, W, N, G, H, KV, d), P, W, N, G, H, KV, d, plan)


def test_recompute_path(override):
    override("force_recompute", "1")
    P, W, N, G, H, KV, d = 900, 15, 5, 15, 8, 8, 128
    check(rand_inputs(22, P, W, N, G, H, KV, d), P, W, N, G, H, KV, d, "recompute")


def test_argument_errors():
    s = wl.TINY
    x = wl.attention_inputs_fp8(s)
    T = s.T
    q = binding.bf16_tensor(x["q"])
    dev = {k: torch.from_numpy(x[k]).cuda() for k in ("k_cache", "v_cache", "step_k", "step_v", "k_scale", "v_scale")}
    out = torch.empty((T, s.heads, s.head_dim), dtype=torch.bfloat16, device="cuda")
    lib = binding.load()
    rc = lib.la_step_attention_fp8kv(q.data_ptr(), dev["k_cache"].data_ptr(), dev["v_cache"].data_ptr(),
                                     dev["step_k"].data_ptr(), dev["step_v"].data_ptr(), None, dev["v_scale"].data_ptr(),
                                     s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, out.data_ptr(), None)
    assert rc == binding.LA_EINVAL and b"k_scale" in lib.la_last_error()
    rc = lib.la_step_attention_fp8kv(q.data_ptr(), dev["k_cache"].data_ptr(), dev["v_cache"].data_ptr(),
                                     dev["step_k"].data_ptr(), dev["step_v"].data_ptr(), dev["k_scale"].data_ptr(),
                                     dev["v_scale"].data_ptr(), s.P, s.W, s.N, s.G, s.heads, s.kv_heads, 96,
                                     out.data_ptr(), None)
    assert rc == binding.LA_EUNSUPPORTED


def test_committed_rows_are_read_back_as_the_step_saw_them():
    """A step over a quantised cache, the append of its accepted rows (la_kv_commit moves bytes: rows of
    head_dim bytes are head_dim / 2 sixteen-bit elements to it), and the next step over the longer
    prefix: the appended cache equals the oracle's append bit for bit, and the next step equals the
    oracle's over that cache."""
    P, W, N, G, H, KV, d = 200, 4, 3, 2, 4, 2, 128
    T = 1 + (W + G) * (N - 1)
    x = rand_inputs(77, P, W, N, G, H, KV, d)
    cap = P + N
    best, n_out = 1, 3                      # candidate 1 accepted in full: rows 0, and its two tokens
    kc = torch.zeros((KV, cap, d), dtype=torch.uint8, device="cuda")
    vc = torch.zeros_like(kc)
    kc[:, :P], vc[:, :P] = torch.from_numpy(x["k_cache"]).cuda(), torch.from_numpy(x["v_cache"]).cuda()
    sk, sv = torch.from_numpy(x["step_k"]).cuda(), torch.from_numpy(x["step_v"]).cuda()
    as16 = lambda t: t.view(torch.bfloat16)
    binding.la_kv_commit(as16(kc), as16(vc), as16(sk), as16(sv), P, W, N, G, KV, d // 2,
                         torch.tensor([best], dtype=torch.int32, device="cuda"),
                         torch.tensor([n_out], dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    ok = np.zeros((KV, cap, d // 2), np.uint16)
    ov = np.zeros_like(ok)
    ok[:, :P], ov[:, :P] = x["k_cache"].view(np.uint16), x["v_cache"].view(np.uint16)
    orc.kv_commit(ok, ov, x["step_k"].view(np.uint16), x["step_v"].view(np.uint16), P, W, N, G, best, n_out)
    np.testing.assert_array_equal(kc.cpu().numpy().view(np.uint16), ok)
    np.testing.assert_array_equal(vc.cpu().numpy().view(np.uint16), ov)
    # the appended keys are step rows 0, 1 + W(N-1) + best(N-1), ... as codes, unchanged
    rows = [0] + [1 + W * (N - 1) + best * (N - 1) + i for i in range(n_out - 1)]
    np.testing.assert_array_equal(kc.cpu().numpy()[:, P:P + n_out], x["step_k"][rows].transpose(1, 0, 2))
    # next step over the longer prefix (a fresh draw for its own rows, the same scales)
    P2 = P + n_out
    y = rand_inputs(78, P2, W, N, G, H, KV, d)
    y["k_cache"], y["v_cache"] = kc.cpu().numpy()[:, :P2].copy(), vc.cpu().numpy()[:, :P2].copy()
    y["k_scale"], y["v_scale"] = x["k_scale"], x["v_scale"]
    check(y, P2, W, N, G, H, KV, d, "after the append")
