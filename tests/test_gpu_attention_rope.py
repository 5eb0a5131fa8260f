"""GPU parity of la_step_attention_rope (query rows, and on request the step's keys, rotated inside
the attention kernel), of the keys-only mode of la_step_rope and of la_kv_commit_rope.

Two bars: against the oracle (step_rope in fp64, rounded to bf16 as the tensors in memory are, then
step_attention) within 2e-2; and against the library's own two-pass path (la_step_rope on q and
step_k, then la_step_attention), whose output bits it must reproduce exactly, because both rotate
with the same arithmetic."""
import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


def make(seed, P, W, N, G, H, KV, d):
    rng = np.random.default_rng(seed)
    T = 1 + (W + G) * (N - 1)
    bf = lambda shape: wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))
    x = dict(q=bf((T, H, d)), k_cache=bf((KV, P, d)), v_cache=bf((KV, P, d)), step_k=bf((T, KV, d)), step_v=bf((T, KV, d)))
    reach = P + max(W + N - 2 if W else 0, N - 1 if (W or G) else 0)
    cos, sin = wl.rope_tables(reach + 5, d)
    return x, cos, sin


@pytest.fixture(autouse=True, params=["auto", "staged", "rowtile"])
def kernel_choice(request, override):
    """Both attention kernels have a rotating form, picked by the same rule as the plain step's kernel:
    every test runs with the library's choice and with each kernel forced, so that the rotating entry
    point and the plain step it is compared with bit by bit always take the same kernel."""
    if request.param != "auto":
        override("attn_rowtile", "1" if request.param == "rowtile" else "0")
    return request.param


def run_case(seed, P, W, N, G, H, KV, d, interleaved, oracle=True):
    print("case", dict(P=P, W=W, N=N, G=G, H=H, KV=KV, d=d, interleaved=interleaved), flush=True)
    x, cos, sin = make(seed, P, W, N, G, H, KV, d)
    T = 1 + (W + G) * (N - 1)
    dev = {k: binding.bf16_tensor(v) for k, v in x.items()}
    dcos, dsin = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()

    # two passes: rotate q and the keys in memory, then the plain step
    q2, k2 = dev["q"].clone(), dev["step_k"].clone()
    binding.la_step_rope(q2, k2, dcos, dsin, P, W, N, G, H, KV, d, interleaved)
    two = torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention(q2, dev["k_cache"], dev["v_cache"], k2, dev["step_v"], P, W, N, G, H, KV, d, two)

    # fused: the keys alone in memory, q rotated inside the attention kernel
    k1 = dev["step_k"].clone()
    binding.la_step_rope(None, k1, dcos, dsin, P, W, N, G, H, KV, d, interleaved)
    q_before = dev["q"].clone()
    one = torch.full((T, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention_rope(dev["q"], dev["k_cache"], dev["v_cache"], k1, dev["step_v"], dcos, dsin, P, W, N, G,
                                   H, KV, d, one, interleaved)
    torch.cuda.synchronize()
    assert torch.equal(k1.view(torch.int16), k2.view(torch.int16)), "keys-only rotation differs from the full pass"
    assert torch.equal(dev["q"].view(torch.int16), q_before.view(torch.int16)), "q was modified"
    assert torch.equal(one.view(torch.int16), two.view(torch.int16)), "fused and two-pass outputs differ"

    # nothing rotated in memory: q and the step keys are turned inside the attention kernel
    k_before = dev["step_k"].clone()
    none = torch.full((T, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention_rope(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"], dcos, dsin,
                                   P, W, N, G, H, KV, d, none, interleaved, rotate_keys=True)
    torch.cuda.synchronize()
    assert torch.equal(dev["step_k"].view(torch.int16), k_before.view(torch.int16)), "step_k was modified"
    assert torch.equal(dev["q"].view(torch.int16), q_before.view(torch.int16)), "q was modified"
    assert torch.equal(none.view(torch.int16), two.view(torch.int16)), "keys rotated in the kernel: output differs"

    if oracle:
        rq, rk = orc.step_rope(orc.bf16_to_f64(x["q"]), orc.bf16_to_f64(x["step_k"]), cos, sin, P, W, N, G, interleaved)
        want = orc.step_attention(wl.f32_to_bf16_bits(rq.astype(np.float32)), x["k_cache"], x["v_cache"],
                                  wl.f32_to_bf16_bits(rk.astype(np.float32)), x["step_v"], P, W, N, G, H, KV, d)
        got = one.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        err = np.abs(got - want).max()
        assert err <= TOL, "max abs err %g" % err


@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("P,W,N,G,H,KV,d", [
    (64, 4, 3, 2, 4, 4, 64),          # the tiny shape
    (0, 5, 4, 2, 2, 1, 64),           # the layout of Fig. 2(b), empty prefix
    (17, 0, 3, 4, 4, 2, 128),         # no window
    (17, 4, 2, 0, 3, 1, 128),         # no candidates, N = 2
    (5, 0, 2, 0, 1, 1, 128),          # a plain decode token
    (333, 15, 5, 15, 4, 4, 128),      # several row tiles, ragged last one
    (517, 3, 7, 3, 16, 2, 128),       # group of 8 heads per KV head
    (129, 20, 5, 20, 2, 2, 64),       # head_dim 64, 24 positions
    (1000, 28, 5, 3, 8, 8, 128),      # 32 positions: the most that fit beside the ring at head_dim 128
])
def test_small_shapes(P, W, N, G, H, KV, d, interleaved):
    run_case(P + W + d, P, W, N, G, H, KV, d, interleaved)


@pytest.mark.parametrize("shape", [wl.LLAMA2_7B, wl.LLAMA2_13B, wl.LLAMA2_70B], ids=lambda s: s.name)
def test_paper_configs_full_size(shape):
    s = shape
    run_case(7, s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, False)


def test_long_ragged_sequence_takes_the_64_row_workgroups():
    """A shape whose plain step uses 128-row workgroups (no LDS left for the tables): the rotating entry
    point falls back to 64-row ones, so the output bits may differ from the two-pass path; the oracle decides."""
    s = wl.ragged_shape(7, 15)
    x, cos, sin = make(3, s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim)
    dev = {k: binding.bf16_tensor(v) for k, v in x.items()}
    dcos, dsin = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    binding.la_step_rope(None, dev["step_k"], dcos, dsin, s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim)
    out = torch.full((s.T, s.heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    binding.la_step_attention_rope(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"], dcos, dsin,
                                   s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim, out)
    torch.cuda.synchronize()
    rq, rk = orc.step_rope(orc.bf16_to_f64(x["q"]), orc.bf16_to_f64(x["step_k"]), cos, sin, s.P, s.W, s.N, s.G)
    want = orc.step_attention(wl.f32_to_bf16_bits(rq.astype(np.float32)), x["k_cache"], x["v_cache"],
                              wl.f32_to_bf16_bits(rk.astype(np.float32)), x["step_v"], s.P, s.W, s.N, s.G, s.heads,
                              s.kv_heads, s.head_dim)
    assert np.abs(out.float().cpu().numpy().astype(np.float64) - want).max() <= TOL


@pytest.mark.parametrize("plan", ["2,2,0,4,64", "1,2,0,4,64", "2,4,2,4,64"])
def test_other_decompositions(override, plan):
    override("attn_plan", plan)
    run_case(31, 700, 10, 5, 10, 8, 4, 128, False)


def test_recompute_path(override):
    override("force_recompute", "1")
    run_case(32, 900, 15, 5, 15, 8, 8, 128, False)


def test_limits_and_argument_errors(kernel_choice, override):
    if kernel_choice != "auto":
        pytest.skip("sets the kernel itself")
    # 34 positions (W = 30, N = 5) do not fit beside the staged kernel's ring at head_dim 128 (the
    # row-tile kernel, which this short prefix would take, has room for 64: see the next test)
    override("attn_rowtile", "0")
    P, W, N, G, H, KV, d = 300, 30, 5, 30, 8, 2, 128
    x, cos, sin = make(1, P, W, N, G, H, KV, d)
    dev = {k: binding.bf16_tensor(v) for k, v in x.items()}
    dcos, dsin = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    out = torch.empty((1 + (W + G) * (N - 1), H, d), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.LaError, match="positions"):
        binding.la_step_attention_rope(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"], dcos,
                                       dsin, P, W, N, G, H, KV, d, out)
    # tables that end before the step's furthest position
    with pytest.raises(binding.LaError, match="positions"):
        binding.la_step_attention_rope(dev["q"], dev["k_cache"], dev["v_cache"], dev["step_k"], dev["step_v"],
                                       dcos[:P + 10].contiguous(), dsin[:P + 10].contiguous(), P, W, N, G, H, KV, d, out)


@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("P,W,N,G,KV,d,best,n_out", [
    (64, 4, 3, 2, 4, 64, 1, 3),        # a full match of the second candidate
    (0, 5, 4, 2, 1, 64, 0, 2),         # empty prefix, one candidate token accepted
    (333, 15, 5, 15, 4, 128, 7, 5),    # the 7B step, full match
    (333, 15, 5, 15, 4, 128, -1, 1),   # nothing accepted: the current token alone
    (17, 4, 2, 0, 1, 128, -1, 1),      # no candidates at all
    (100, 3, 7, 3, 2, 256, 2, 4),      # head_dim 256
])
def test_commit_rope_leaves_the_bits_of_rotate_then_commit(P, W, N, G, KV, d, best, n_out, interleaved):
    """The appended key rows, turned by their cache positions, against la_step_rope on the whole step
    followed by la_kv_commit; values and everything outside the appended rows untouched.  The oracle's
    rotation and append decide the values (keys within one bf16 rounding of the fp64 rotation)."""
    print("case", dict(P=P, W=W, N=N, G=G, KV=KV, d=d, best=best, n_out=n_out, interleaved=interleaved), flush=True)
    rng = np.random.default_rng(P + W + d + n_out)
    T = 1 + (W + G) * (N - 1)
    cap = P + N + 3
    bf = lambda shape: wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))
    kc, vc, sk, sv = bf((KV, cap, d)), bf((KV, cap, d)), bf((T, KV, d)), bf((T, KV, d))
    cos, sin = wl.rope_tables(P + W + N + 5, d)
    dcos, dsin = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    dbest = torch.tensor([best], dtype=torch.int32, device="cuda")
    dn = torch.tensor([n_out], dtype=torch.int32, device="cuda")

    k_a, v_a = binding.bf16_tensor(kc), binding.bf16_tensor(vc)
    sk_rot = binding.bf16_tensor(sk)
    binding.la_step_rope(None, sk_rot, dcos, dsin, P, W, N, G, 1, KV, d, interleaved)
    binding.la_kv_commit(k_a, v_a, sk_rot, binding.bf16_tensor(sv), P, W, N, G, KV, d, dbest, dn)

    k_b, v_b = binding.bf16_tensor(kc), binding.bf16_tensor(vc)
    dsk = binding.bf16_tensor(sk)
    binding.la_kv_commit_rope(k_b, v_b, dsk, binding.bf16_tensor(sv), dcos, dsin, P, W, N, G, KV, d, dbest, dn,
                              interleaved)
    torch.cuda.synchronize()
    assert torch.equal(dsk.view(torch.int16).cpu(), torch.from_numpy(sk.view(np.int16))), "step_k was modified"
    assert torch.equal(k_a.view(torch.int16), k_b.view(torch.int16))
    assert torch.equal(v_a.view(torch.int16), v_b.view(torch.int16))

    # the oracle: rotate the step's keys in fp64, append the rows the result names
    _, rk = orc.step_rope(np.zeros((T, 1, d)), orc.bf16_to_f64(sk), cos, sin, P, W, N, G, interleaved)
    want_k, want_v = orc.bf16_to_f64(kc), orc.bf16_to_f64(vc)
    assert orc.kv_commit(want_k, want_v, rk, orc.bf16_to_f64(sv), P, W, N, G, best, n_out) == P + n_out
    got_k = k_b.float().cpu().numpy().astype(np.float64)
    got_v = v_b.float().cpu().numpy().astype(np.float64)
    np.testing.assert_array_equal(got_v, want_v)
    np.testing.assert_array_equal(got_k[:, :P], want_k[:, :P])
    np.testing.assert_array_equal(got_k[:, P + n_out:], want_k[:, P + n_out:])
    new = slice(P, P + n_out)
    assert np.abs(got_k[:, new] - want_k[:, new]).max() <= 2.0 ** -8 * max(1.0, np.abs(want_k[:, new]).max()) + 1e-6


def test_commit_rope_argument_errors():
    P, W, N, G, KV, d = 10, 2, 3, 2, 2, 64
    T = 1 + (W + G) * (N - 1)
    z = lambda *shape: torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
    cos, sin = wl.rope_tables(P + N + 4, d)
    dcos, dsin = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    one = torch.ones(1, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.LaError, match="capacity"):
        binding.la_kv_commit_rope(z(KV, P + 1, d), z(KV, P + 1, d), z(T, KV, d), z(T, KV, d), dcos, dsin, P, W, N, G,
                                  KV, d, one, one)
    with pytest.raises(binding.LaError, match="positions"):
        binding.la_kv_commit_rope(z(KV, P + N, d), z(KV, P + N, d), z(T, KV, d), z(T, KV, d), dcos[:P + 1].contiguous(),
                                  dsin[:P + 1].contiguous(), P, W, N, G, KV, d, one, one)
    with pytest.raises(binding.LaError, match="multiple of 16"):
        t24 = torch.zeros((P + N + 4, 12), dtype=torch.float32, device="cuda")
        binding.la_kv_commit_rope(z(KV, P + N, 24), z(KV, P + N, 24), z(T, KV, 24), z(T, KV, 24), t24, t24, P, W, N, G,
                                  KV, 24, one, one)


def test_wide_window_on_a_short_prefix_takes_the_row_tile_kernel(kernel_choice):
    """34 positions: more than the staged kernel stages, fewer than the row-tile kernel's 64."""
    if kernel_choice == "staged":
        pytest.skip("the staged kernel refuses this step (test_limits_and_argument_errors)")
    P, W, N, G, H, KV, d = 300, 30, 5, 30, 8, 2, 128
    assert binding.la_step_attention_kernel(P, W, N, G, H, KV, d) == 1
    run_case(41, P, W, N, G, H, KV, d, False)


def test_recompute_and_forced_decompositions_stay_with_the_staged_kernel(kernel_choice):
    """(run_case compares bits: with a forced decomposition both sides are the staged kernel)"""
    if kernel_choice != "rowtile":
        pytest.skip("covered by test_other_decompositions")
    binding.la_debug_override("attn_plan", "2,4,2,4,64")
    try:
        run_case(31, 200, 10, 5, 10, 8, 4, 128, False)
    finally:
        binding.la_debug_override("attn_plan", None)
