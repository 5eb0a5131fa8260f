"""Pins of the oracle's step over a quantised KV cache (8-bit float keys and values, one scale per KV
head).  The paper computes in 16 bits; this extension only changes what a stored key or value stands
for, so the pins are: the decoding of every code against a library's cast, equality with the pinned
16-bit step wherever both formats hold the same numbers, what the scales must do (values: linear;
keys: the same as scaling the scores), a library attention on the one-token decode, and a read-out
of single value rows that fails on any wrong index."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import la_oracle as orc
from paper_2402_02057_amd import workloads as wl


def finite_codes(rng, shape):
    """Random codes without the two NaN patterns."""
    c = rng.integers(0, 256, size=shape, dtype=np.uint16).astype(np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x3A
    return c


def make_inputs(rng, P, W, N, G, H, KV, d, pow2_scales=False):
    T = 1 + (W + G) * (N - 1)
    if pow2_scales:
        ks = np.ldexp(1.0, rng.integers(-6, 1, size=KV)).astype(np.float32)
        vs = np.ldexp(1.0, rng.integers(-6, 1, size=KV)).astype(np.float32)
    else:
        ks = rng.uniform(0.004, 0.02, size=KV).astype(np.float32)
        vs = rng.uniform(0.004, 0.02, size=KV).astype(np.float32)
    # codes of moderate magnitude (exponent field <= 10), so that scores stay in a sane range
    def codes(shape):
        c = finite_codes(rng, shape)
        return np.where(((c >> 3) & 15) > 10, c & 0xD7, c).astype(np.uint8)
    return dict(q=wl.f32_to_bf16_bits(rng.standard_normal(size=(T, H, d), dtype=np.float32)),
                k_cache=codes((KV, P, d)), v_cache=codes((KV, P, d)), step_k=codes((T, KV, d)),
                step_v=codes((T, KV, d)), k_scale=ks, v_scale=vs)


def run(x, P, W, N, G, H, KV, d):
    return orc.step_attention_fp8kv(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], x["k_scale"],
                                    x["v_scale"], P, W, N, G, H, KV, d)


def library_decode(codes):
    return torch.from_numpy(np.ascontiguousarray(codes)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def test_every_code_point_against_the_library_cast_and_the_format_definition():
    codes = np.arange(256, dtype=np.uint8)
    got = orc.fp8_e4m3_decode(codes)
    want = library_decode(codes)
    nan = np.isnan(want)
    assert list(codes[nan]) == [0x7F, 0xFF] and np.isnan(got[nan]).all()
    np.testing.assert_array_equal(got[~nan], want[~nan])
    # corners of the format, from its definition: largest, smallest normal, smallest subnormal, one, signs
    assert got[0x7E] == 448.0 and got[0xFE] == -448.0
    assert got[0x08] == 2.0 ** -6 and got[0x01] == 2.0 ** -9 and got[0x07] == 7 * 2.0 ** -9
    assert got[0x38] == 1.0 and got[0xB8] == -1.0 and got[0x00] == 0.0 and got[0x80] == 0.0
    assert np.signbit(got[0x80])
    # 8 values per binade, evenly spaced
    assert np.allclose(np.diff(got[0x40:0x49]), 0.25)


@pytest.mark.parametrize("P,W,N,G,H,KV,d", [(5, 3, 4, 2, 4, 2, 16), (0, 2, 3, 1, 2, 2, 8), (40, 4, 3, 2, 4, 4, 64)])
def test_equals_the_16_bit_step_where_both_formats_hold_the_same_numbers(P, W, N, G, H, KV, d):
    """An 8-bit float times a power of two is a bf16 number: the same step through the 16-bit oracle
    (pinned on its own) must give the same bits."""
    rng = np.random.default_rng(P + d)
    x = make_inputs(rng, P, W, N, G, H, KV, d, pow2_scales=True)
    got = run(x, P, W, N, G, H, KV, d)
    def as_bf16(codes, scale, head_axis):
        shape = [1, 1, 1]
        shape[head_axis] = KV
        val = (library_decode(codes) * scale.astype(np.float64).reshape(shape)).astype(np.float32)
        bits = wl.f32_to_bf16_bits(val)
        np.testing.assert_array_equal(wl.bf16_bits_to_f32(bits), val)  # exact in bf16
        return bits
    want = orc.step_attention(x["q"], as_bf16(x["k_cache"], x["k_scale"], 0), as_bf16(x["v_cache"], x["v_scale"], 0),
                              as_bf16(x["step_k"], x["k_scale"], 1), as_bf16(x["step_v"], x["v_scale"], 1),
                              P, W, N, G, H, KV, d)
    np.testing.assert_array_equal(got, want)


def test_value_scale_is_linear_and_per_head():
    P, W, N, G, H, KV, d = 7, 2, 3, 2, 4, 2, 8
    rng = np.random.default_rng(11)
    x = make_inputs(rng, P, W, N, G, H, KV, d)
    base = run(x, P, W, N, G, H, KV, d)
    y = dict(x)
    y["v_scale"] = (x["v_scale"] * np.array([3.0, 1.0], dtype=np.float32)).astype(np.float32)
    got = run(y, P, W, N, G, H, KV, d)
    ratio = y["v_scale"].astype(np.float64) / x["v_scale"].astype(np.float64)
    np.testing.assert_allclose(got[:, :2], base[:, :2] * ratio[0], rtol=1e-13)   # heads 0, 1 read KV head 0
    np.testing.assert_array_equal(got[:, 2:], base[:, 2:])                        # heads 2, 3 read KV head 1


def test_key_scale_acts_on_the_scores_of_its_head_only():
    """Doubling the key scale of a head is the same as doubling its queries (a power of two: exact in bf16)."""
    P, W, N, G, H, KV, d = 6, 3, 3, 1, 4, 2, 8
    rng = np.random.default_rng(12)
    x = make_inputs(rng, P, W, N, G, H, KV, d)
    y = dict(x)
    y["k_scale"] = (x["k_scale"] * np.array([1.0, 2.0], dtype=np.float32)).astype(np.float32)
    z = dict(x)
    qf = wl.bf16_bits_to_f32(x["q"]).copy()
    qf[:, 2:] *= 2.0
    z["q"] = wl.f32_to_bf16_bits(qf)
    a, b = run(y, P, W, N, G, H, KV, d), run(z, P, W, N, G, H, KV, d)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-15)
    assert np.abs(a[:, 2:] - run(x, P, W, N, G, H, KV, d)[:, 2:]).max() > 1e-3  # and it does something


@pytest.mark.parametrize("P,H,KV,d", [(9, 4, 2, 16), (33, 2, 2, 64), (0, 3, 1, 8)])
def test_one_token_decode_against_a_library_attention(P, H, KV, d):
    rng = np.random.default_rng(P + 1)
    x = make_inputs(rng, P, 0, 3, 0, H, KV, d)
    got = run(x, P, 0, 3, 0, H, KV, d)
    g = H // KV
    q = torch.from_numpy(wl.bf16_bits_to_f32(x["q"]).astype(np.float64))
    for h in range(H):
        kvh = h // g
        deq = lambda c, s: torch.from_numpy(library_decode(c) * float(s))
        keys = torch.cat([deq(x["k_cache"][kvh], x["k_scale"][kvh]), deq(x["step_k"][:, kvh], x["k_scale"][kvh])])
        vals = torch.cat([deq(x["v_cache"][kvh], x["v_scale"][kvh]), deq(x["step_v"][:, kvh], x["v_scale"][kvh])])
        o = F.scaled_dot_product_attention(q[0, h][None, None, None], keys[None, None], vals[None, None])
        np.testing.assert_allclose(got[0, h], o[0, 0, 0].numpy(), rtol=0, atol=1e-12)


def test_read_out_of_single_value_rows():
    """A key that dominates a row's softmax hands the row that key's value row: checks which cache row,
    which KV head and which scale an output element comes from."""
    P, W, N, G, H, KV, d = 12, 0, 2, 0, 4, 2, 8
    rng = np.random.default_rng(5)
    x = make_inputs(rng, P, W, N, G, H, KV, d)
    x["k_cache"][:] = 0x00
    x["step_k"][:] = 0x00
    qf = np.zeros((1, H, d), dtype=np.float32)
    qf[0, :, 0] = 64.0
    x["q"] = wl.f32_to_bf16_bits(qf)
    x["k_scale"] = np.array([1.0, 0.5], dtype=np.float32)
    target = {0: 3, 1: 10}                      # KV head -> the prefix key its queries single out
    for kvh, row in target.items():
        x["k_cache"][kvh, row, 0] = 0x58        # 16.0: score 64 * 16 * scale / sqrt(8), far above the zeros
    got = run(x, P, W, N, G, H, KV, d)
    for h in range(H):
        kvh = h // 2
        want = library_decode(x["v_cache"][kvh, target[kvh]]) * float(x["v_scale"][kvh])
        np.testing.assert_allclose(got[0, h], want, rtol=0, atol=1e-9)


def test_missing_scales_and_bad_shapes_are_rejected():
    rng = np.random.default_rng(2)
    x = make_inputs(rng, 3, 1, 3, 1, 2, 2, 8)
    import ctypes
    lib = orc._load()
    out = np.zeros((5, 2, 8))
    args = [x[k].ctypes.data for k in ("q", "k_cache", "v_cache", "step_k", "step_v")]
    assert lib.la_oracle_step_attention_fp8kv(*args, None, x["v_scale"].ctypes.data, 3, 1, 3, 1, 2, 2, 8,
                                              out.ctypes.data) == -1
    assert lib.la_oracle_step_attention_fp8kv(*args, x["k_scale"].ctypes.data, x["v_scale"].ctypes.data, 3, 1, 1, 1,
                                              2, 2, 8, out.ctypes.data) == -1


def test_the_quantised_workload_stays_close_to_the_16_bit_one():
    """The seeded 8-bit workload is the 16-bit one quantised: the two steps differ by the quantisation
    error only (3 mantissa bits: a few percent of the output's scale), nowhere near a wrong scale."""
    s = wl.TINY
    x = wl.attention_inputs_fp8(s)
    y = wl.attention_inputs(s)
    a = run(x, s.P, s.W, s.N, s.G, s.heads, s.kv_heads, s.head_dim)
    b = orc.step_attention(y["q"], y["k_cache"], y["v_cache"], y["step_k"], y["step_v"], s.P, s.W, s.N, s.G, s.heads,
                           s.kv_heads, s.head_dim)
    assert np.abs(a - b).max() < 0.1 * np.abs(b).max()
    assert not np.isnan(library_decode(x["k_cache"])).any() and np.abs(library_decode(x["k_cache"])).max() == 448.0
