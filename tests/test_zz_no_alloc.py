"""GPU: la_step_attention_noalloc (fixed scratch block inside the library, no allocation)
against la_step_attention, through the raw C ABI, on two calls in a row, the second smaller.

Bar: the two entry points share their kernels and their decomposition, so the outputs must be
the same bits; the smaller case is also compared with the fp64 oracle (max abs error <= 2e-2).
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import la_oracle as orc
from paper_2402_02057_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


def rand_inputs(seed, P, W, N, G, H, KV, d):
    rng = np.random.default_rng(seed)
    T = 1 + (W + G) * (N - 1)

    def bf(shape):
        return wl.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))
    return dict(q=bf((T, H, d)), k_cache=bf((KV, P, d)), v_cache=bf((KV, P, d)),
                step_k=bf((T, KV, d)), step_v=bf((T, KV, d)))


def call_raw(name, dev, shape, out):
    """The entry point `name` through ctypes, nothing of the Python binding in between."""
    P, W, N, G, H, KV, d = shape
    lib = binding.load()
    fn = getattr(lib, name)
    fn.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int] * 7 + [ctypes.c_void_p, ctypes.c_void_p]
    fn.restype = ctypes.c_int
    rc = fn(dev["q"].data_ptr(), dev["k_cache"].data_ptr(), dev["v_cache"].data_ptr(), dev["step_k"].data_ptr(),
            dev["step_v"].data_ptr(), P, W, N, G, H, KV, d, out.data_ptr(),
            torch.cuda.current_stream().cuda_stream)
    assert rc == 0, lib.la_last_error().decode()


def both(shape, seed):
    P, W, N, G, H, KV, d = shape
    T = 1 + (W + G) * (N - 1)
    x = rand_inputs(seed, *shape)
    dev = {k: binding.bf16_tensor(v) for k, v in x.items()}
    outs = []
    for name in ("la_step_attention_noalloc", "la_step_attention"):
        out = torch.full((T, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        print("call", name, shape, flush=True)
        call_raw(name, dev, shape, out)
        torch.cuda.synchronize()
        outs.append(binding.bf16_bits(out))
    return x, outs


def test_two_calls_second_smaller():
    torch.cuda.set_device(0)
    big = (1024, 15, 5, 15, 32, 32, 128)     # the 7B shape: 256 workgroups, four-way key split
    small = (900, 4, 3, 2, 8, 4, 128)        # fewer split groups, shorter partials (15 chunks: still the
                                             # staged kernel, the one that uses the scratch block)
    assert binding.la_step_attention_kernel(*small) == 0 and binding.la_step_attention_workspace_bytes(*small) > 0
    _, (fixed, pooled) = both(big, 11)
    assert np.array_equal(fixed, pooled), "7B shape: noalloc differs from la_step_attention"
    x, (fixed, pooled) = both(small, 12)
    assert np.array_equal(fixed, pooled), "small shape after the large one: noalloc differs"
    P, W, N, G, H, KV, d = small
    want = orc.step_attention(x["q"], x["k_cache"], x["v_cache"], x["step_k"], x["step_v"], P, W, N, G, H, KV, d)
    got = wl.bf16_bits_to_f32(fixed).astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= TOL
    # and once more at the large shape: the block keeps the small call's contents
    _, (fixed, pooled) = both(big, 13)
    assert np.array_equal(fixed, pooled)
    # a step short enough for the kernel that needs no scratch memory at all goes through as well
    tiny = (333, 4, 3, 2, 8, 4, 128)
    assert binding.la_step_attention_kernel(*tiny) == 1
    _, (fixed, pooled) = both(tiny, 14)
    assert np.array_equal(fixed, pooled)


def test_refuses_what_does_not_fit(override):
    """A decomposition whose partials exceed the fixed block is refused before anything is launched
    (the library's own choice never needs more than 5 MiB; a 64-way split forced by hand does).
    The buffers are real and of the right size all the same."""
    torch.cuda.set_device(0)
    override("attn_plan", "2,4,64,4,64")
    shape = (4096, 15, 5, 15, 32, 32, 128)
    P, W, N, G, H, KV, d = shape
    T = 1 + (W + G) * (N - 1)
    x = rand_inputs(14, *shape)
    dev = {k: binding.bf16_tensor(v) for k, v in x.items()}
    out = torch.zeros((T, H, d), dtype=torch.bfloat16, device="cuda")
    lib = binding.load()
    rc = lib.la_step_attention_noalloc(dev["q"].data_ptr(), dev["k_cache"].data_ptr(), dev["v_cache"].data_ptr(),
                                       dev["step_k"].data_ptr(), dev["step_v"].data_ptr(), P, W, N, G, H, KV, d,
                                       out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == binding.LA_EUNSUPPORTED, rc
    assert b"scratch" in lib.la_last_error()
    assert not out.any().item()   # nothing was launched
