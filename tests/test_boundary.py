"""The C-ABI library builds, loads without a GPU and exports what include/la.h declares."""
import os
import re

import pytest

from paper_2402_02057_amd import binding, buildlib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if buildlib.is_stale():
        buildlib.build()
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "la.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(la_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_error_string(lib):
    assert binding.la_version() >= 1000
    assert isinstance(lib.la_last_error(), bytes)


def test_argument_errors_are_reported_without_a_gpu(lib):
    # validation happens before any HIP call
    rc = lib.la_step_attention(None, None, None, None, None, 0, 1, 1, 1, 1, 1, 128, None, None)
    assert rc == -1 and b"N >= 2" in lib.la_last_error()
    rc = lib.la_step_attention(None, None, None, None, None, 0, 1, 3, 1, 4, 4, 96, None, None)
    assert rc == -2 and b"head_dim" in lib.la_last_error()
    rc = lib.la_step_attention(None, None, None, None, None, 0, 1, 3, 1, 6, 4, 128, None, None)
    assert rc == -2
    rc = lib.la_step_attention(None, None, None, None, None, 0, 1, 3, 1, 4, 4, 128, None, None)
    assert rc == -1 and b"null" in lib.la_last_error()
    rc = lib.la_step_attention(16, None, None, 16, 24, 0, 1, 3, 1, 4, 4, 128, 16, None)
    assert rc == -1 and b"aligned" in lib.la_last_error()
    assert lib.la_verify(None, None, 0, 3, 10, None, None, None) == 0      # G = 0: no-op
    assert lib.la_verify(None, None, 2, 3, 10, None, None, None) == -1
    assert lib.la_verify(None, None, 2, 1, 10, None, None, None) == -1
    assert lib.la_verify_step(None, None, None, None, 0, 3, 0, 10, None, None, None, None, None, None) == -1
    assert b"null" in lib.la_last_error()
    assert lib.la_verify_step(None, None, None, None, 0, 1, 0, 10, None, None, None, None, None, None) == -1
    assert b"N >= 2" in lib.la_last_error()
    assert lib.la_verify_sample(None, None, None, None, None, 1.0, 3, 0, 10, None, None, None) == -1
    assert b"null" in lib.la_last_error()
    assert lib.la_verify_sample(None, None, None, None, None, 0.0, 3, 0, 10, None, None, None) == -1
    assert b"temperature" in lib.la_last_error()


def test_cache_forms_report_argument_errors_without_a_gpu(lib):
    A = 4096    # any aligned non-null value: nothing is dereferenced before validation ends
    # in-place cache: capacity below the prefix, and no room for N more rows
    rc = lib.la_step_attention_cap(A, A, A, 10, A, A, 11, 1, 3, 1, 4, 4, 128, A, None)
    assert rc == -1 and b"capacity" in lib.la_last_error()
    rc = lib.la_kv_commit(A, A, 12, A, A, 10, 1, 3, 1, 4, 128, A, A, None)
    assert rc == -1 and b"capacity" in lib.la_last_error()
    assert lib.la_kv_commit(A, A, 64, A, A, 10, 1, 1, 1, 4, 128, A, A, None) == -1      # N < 2
    assert lib.la_kv_commit(A, A, 64, A, A, 10, 1, 3, 1, 4, 100, A, A, None) == -2      # head_dim % 8
    assert lib.la_kv_commit(A, A, 64, A, A, 10, 1, 3, 1, 4, 128, None, A, None) == -1   # best is null
    assert lib.la_kv_commit(A, A + 8, 64, A, A, 10, 1, 3, 1, 4, 128, A, A, None) == -1  # misaligned cache
    # paged cache: page size, page count, table
    rc = lib.la_step_attention_paged(A, A, A, A, 96, 4, A, A, 10, 1, 3, 1, 4, 4, 128, A, None)
    assert rc == -2 and b"page_size" in lib.la_last_error()
    rc = lib.la_step_attention_paged(A, A, A, A, 64, 0, A, A, 10, 1, 3, 1, 4, 4, 128, A, None)
    assert rc == -1 and b"n_pages" in lib.la_last_error()
    rc = lib.la_step_attention_paged(A, A, A, None, 64, 4, A, A, 10, 1, 3, 1, 4, 4, 128, A, None)
    assert rc == -1 and b"block_table" in lib.la_last_error()
    rc = lib.la_kv_commit_paged(A, A, None, 64, 4, A, A, 0, 1, 3, 1, 4, 128, A, A, None)
    assert rc == -1 and b"block_table" in lib.la_last_error()      # the append always reads the table
    assert lib.la_kv_commit_paged(A, A, A, 48, 4, A, A, 0, 1, 3, 1, 4, 128, A, A, None) == -2


def test_quantised_and_rotating_forms_report_argument_errors_without_a_gpu(lib):
    A = 4096
    # 8-bit cache: scales are required and must be aligned
    rc = lib.la_step_attention_fp8kv(A, A, A, A, A, None, A, 10, 1, 3, 1, 4, 4, 128, A, None)
    assert rc == -1 and b"k_scale" in lib.la_last_error()
    rc = lib.la_step_attention_fp8kv(A, A, A, A, A, A, A + 2, 10, 1, 3, 1, 4, 4, 128, A, None)
    assert rc == -1 and b"aligned" in lib.la_last_error()
    rc = lib.la_step_attention_fp8kv(A, A, A, A, A, A, A, 10, 1, 1, 1, 4, 4, 128, A, None)
    assert rc == -1 and b"N >= 2" in lib.la_last_error()
    rc = lib.la_step_attention_fp8kv(A, A, A, A, A, A, A, 10, 1, 3, 1, 4, 4, 96, A, None)
    assert rc == -2 and b"head_dim" in lib.la_last_error()
    # rotation inside the kernel: tables present, aligned, and long enough for the step's furthest position
    args = (1, 10, 3, 4, 2, 4, 4, 128, A, None)   # rotate_keys, P, W, N, G, heads, kv_heads, head_dim, out, stream
    rc = lib.la_step_attention_rope(A, A, A, A, A, None, A, 64, 0, *args)
    assert rc == -1 and b"cos" in lib.la_last_error()
    rc = lib.la_step_attention_rope(A, A, A, A, A, A + 4, A, 64, 0, *args)
    assert rc == -1 and b"aligned" in lib.la_last_error()
    rc = lib.la_step_attention_rope(A, A, A, A, A, A, A, 15, 0, *args)       # reaches 10 + 3 + 4 - 2 = 15
    assert rc == -1 and b"positions" in lib.la_last_error()
    rc = lib.la_step_attention_rope(A, A, A, A, A, A, A, 16, 0, 0, 10, 3, 1, 2, 4, 4, 128, A, None)
    assert rc == -1 and b"N >= 2" in lib.la_last_error()
    rc = lib.la_step_attention_rope(A, A, A, None, A, A, A, 16, 0, *args)
    assert rc == -1 and b"null" in lib.la_last_error()
    # the rotating append: room for N rows, tables up to position P + N - 1, whole units of eight pairs
    c = (10, 3, 4, 2, 4, 128, A, A, None)                # P, W, N, G, kv_heads, head_dim, best, n_out, stream
    rc = lib.la_kv_commit_rope(A, A, 13, A, A, A, A, 64, 0, *c)
    assert rc == -1 and b"capacity" in lib.la_last_error()
    rc = lib.la_kv_commit_rope(A, A, 64, A, A, A, A, 13, 0, *c)              # reaches 10 + 4 - 1 = 13
    assert rc == -1 and b"positions" in lib.la_last_error()
    assert lib.la_kv_commit_rope(A, A, 64, A, A, A, A, 14, 0, 10, 3, 4, 2, 4, 128, None, A, None) == -1  # null best
    assert lib.la_kv_commit_rope(A, A, 64, A, A, A + 8, A, 14, 0, *c) == -1  # misaligned table
    rc = lib.la_kv_commit_rope(A, A, 64, A, A, A, A, 14, 0, 10, 3, 4, 2, 4, 24, A, A, None)
    assert rc == -2 and b"multiple of 16" in lib.la_last_error()
    # the rope pass takes a null q (keys alone) but not null keys or tables
    rc = lib.la_step_rope(None, None, A, A, 64, 10, 3, 4, 2, 4, 4, 128, 0, None)
    assert rc == -1 and b"null" in lib.la_last_error()
    # testing hooks: unknown keys and malformed plans are refused
    assert lib.la_debug_override(b"no_such_key", b"1") == -1
    assert lib.la_debug_override(b"attn_plan", b"2,4") == -1
    assert lib.la_debug_override(b"attn_plan", None) == 0


def test_batch_reports_argument_errors_without_a_gpu(lib):
    import ctypes
    A = 4096
    d = (binding.StepDesc * 2)()
    for x in d:
        x.q = x.step_k = x.step_v = x.out = x.k_cache = x.v_cache = A
        x.P, x.reserved = 10, 0
    ptr = ctypes.cast(d, ctypes.c_void_p)
    assert lib.la_step_attention_batch(ptr, 0, 1, 3, 1, 4, 4, 128, None) == -1
    assert lib.la_step_attention_batch(None, 2, 1, 3, 1, 4, 4, 128, None) == -1
    assert lib.la_step_attention_batch(ptr, 2, 1, 1, 1, 4, 4, 128, None) == -1          # N < 2
    assert lib.la_step_attention_batch(ptr, 2, 1, 3, 1, 4, 4, 96, None) == -2           # head_dim
    d[1].P = -1
    rc = lib.la_step_attention_batch(ptr, 2, 1, 3, 1, 4, 4, 128, None)
    assert rc == -1 and b"descriptor 1" in lib.la_last_error()
    d[1].P = 10
    d[1].out = A + 2
    rc = lib.la_step_attention_batch(ptr, 2, 1, 3, 1, 4, 4, 128, None)
    assert rc == -1 and b"aligned" in lib.la_last_error()
    d[1].out = A
    d[0].k_cache = None
    rc = lib.la_step_attention_batch(ptr, 2, 1, 3, 1, 4, 4, 128, None)
    assert rc == -1 and b"descriptor 0" in lib.la_last_error()


def test_paged_batch_reports_argument_errors_without_a_gpu(lib):
    import ctypes
    A = 4096
    d = (binding.StepDescPaged * 1)()
    d[0].q = d[0].step_k = d[0].step_v = d[0].out = d[0].block_table = A
    d[0].P, d[0].reserved = 10, 0
    ptr = ctypes.cast(d, ctypes.c_void_p)
    assert lib.la_step_attention_batch_paged(ptr, 1, A, A, 96, 4, 1, 3, 1, 4, 4, 128, None) == -2     # page size
    assert lib.la_step_attention_batch_paged(ptr, 1, None, A, 64, 4, 1, 3, 1, 4, 4, 128, None) == -1  # no pool
    d[0].block_table = None
    rc = lib.la_step_attention_batch_paged(ptr, 1, A, A, 64, 4, 1, 3, 1, 4, 4, 128, None)
    assert rc == -1 and b"descriptor 0" in lib.la_last_error()


def test_commit_batch_reports_argument_errors_without_a_gpu(lib):
    import ctypes
    A = 4096
    d = (binding.CommitDesc * 2)()
    for x in d:
        x.k_cache = x.v_cache = x.step_k = x.step_v = x.best = x.n_out = A
        x.block_table = None
        x.capacity, x.P, x.reserved = 64, 10, 0
    ptr = ctypes.cast(d, ctypes.c_void_p)
    assert lib.la_kv_commit_batch(ptr, 0, 0, 0, 1, 3, 1, 4, 128, None) == -1
    assert lib.la_kv_commit_batch(None, 2, 0, 0, 1, 3, 1, 4, 128, None) == -1
    assert lib.la_kv_commit_batch(ptr, 2, 0, 0, 1, 1, 1, 4, 128, None) == -1            # N < 2
    assert lib.la_kv_commit_batch(ptr, 2, 0, 0, 1, 3, 1, 4, 100, None) == -2            # head_dim % 8
    d[1].capacity = 12
    rc = lib.la_kv_commit_batch(ptr, 2, 0, 0, 1, 3, 1, 4, 128, None)
    assert rc == -1 and b"descriptor 1" in lib.la_last_error() and b"capacity" in lib.la_last_error()
    d[1].capacity = 64
    d[0].n_out = None
    rc = lib.la_kv_commit_batch(ptr, 2, 0, 0, 1, 3, 1, 4, 128, None)
    assert rc == -1 and b"descriptor 0" in lib.la_last_error()
    d[0].n_out = A
    d[1].v_cache = A + 8
    rc = lib.la_kv_commit_batch(ptr, 2, 0, 0, 1, 3, 1, 4, 128, None)
    assert rc == -1 and b"aligned" in lib.la_last_error()
    d[1].v_cache = A
    d[1].block_table = A                     # a paged descriptor needs the launch's page geometry
    rc = lib.la_kv_commit_batch(ptr, 2, 48, 4, 1, 3, 1, 4, 128, None)
    assert rc == -2 and b"page_size" in lib.la_last_error()
    rc = lib.la_kv_commit_batch(ptr, 2, 64, 0, 1, 3, 1, 4, 128, None)
    assert rc == -1 and b"n_pages" in lib.la_last_error()


def test_verify_step_batch_reports_argument_errors_without_a_gpu(lib):
    import ctypes
    A = 4096
    d = (binding.VerifyDesc * 2)()
    for x in d:
        for name, _ in binding.VerifyDesc._fields_:
            setattr(x, name, A)
    ptr = ctypes.cast(d, ctypes.c_void_p)
    assert lib.la_verify_step_batch(ptr, 0, 1, 3, 1, 10, None) == -1
    assert lib.la_verify_step_batch(None, 2, 1, 3, 1, 10, None) == -1
    assert lib.la_verify_step_batch(ptr, 2, 1, 1, 1, 10, None) == -1 and b"N >= 2" in lib.la_last_error()
    d[1].best = None
    rc = lib.la_verify_step_batch(ptr, 2, 1, 3, 1, 10, None)
    assert rc == -1 and b"descriptor 1" in lib.la_last_error() and b"null" in lib.la_last_error()
    d[1].best = A
    d[0].logits_cand = A + 2
    rc = lib.la_verify_step_batch(ptr, 2, 1, 3, 1, 10, None)
    assert rc == -1 and b"descriptor 0" in lib.la_last_error() and b"aligned" in lib.la_last_error()
    d[0].logits_cand = None                  # allowed without candidates only
    assert lib.la_verify_step_batch(ptr, 2, 1, 3, 1, 10, None) == -1


def test_rope_reports_argument_errors_without_a_gpu(lib):
    A = 4096
    assert lib.la_step_rope(A, A, A, A, 64, 10, 1, 1, 1, 4, 4, 128, 0, None) == -1      # N < 2
    assert lib.la_step_rope(A, A, A, A, 64, 10, 1, 3, 1, 4, 4, 72, 0, None) == -2       # head_dim % 16
    rc = lib.la_step_rope(A, A, A, A, 12, 10, 3, 3, 1, 4, 4, 128, 0, None)              # reaches 10 + 4
    assert rc == -1 and b"positions" in lib.la_last_error()
    assert lib.la_step_rope(A, None, A, A, 64, 10, 1, 3, 1, 4, 4, 128, 0, None) == -1   # null
    assert lib.la_step_rope(A, A, A + 4, A, 64, 10, 1, 3, 1, 4, 4, 128, 0, None) == -1  # misaligned table


def test_verify_sample_batch_reports_argument_errors_without_a_gpu(lib):
    import ctypes
    A = 4096
    d = (binding.SampleDesc * 2)()
    for x in d:
        for name in ("logits_cur", "logits_cand", "cand_tokens", "u_test", "u_final", "out_tokens", "n_out"):
            setattr(x, name, A)
        x.temperature, x.reserved = 1.0, 0
    ptr = ctypes.cast(d, ctypes.c_void_p)
    assert lib.la_verify_sample_batch(ptr, 0, 3, 1, 10, None) == -1
    assert lib.la_verify_sample_batch(None, 2, 3, 1, 10, None) == -1
    assert lib.la_verify_sample_batch(ptr, 2, 1, 1, 10, None) == -1 and b"N >= 2" in lib.la_last_error()
    assert lib.la_verify_sample_batch(ptr, 2, 3, 2000, 10, None) == -2
    d[1].temperature = -1.0
    rc = lib.la_verify_sample_batch(ptr, 2, 3, 1, 10, None)
    assert rc == -1 and b"descriptor 1" in lib.la_last_error() and b"temperature" in lib.la_last_error()
    d[1].temperature = 1.0
    d[0].u_test = None
    rc = lib.la_verify_sample_batch(ptr, 2, 3, 1, 10, None)
    assert rc == -1 and b"descriptor 0" in lib.la_last_error() and b"null" in lib.la_last_error()


def test_workspace_sets_are_range_checked(lib):
    assert lib.la_select_workspace(-1) == -1 and b"0..15" in lib.la_last_error()
    assert lib.la_select_workspace(16) == -1
    assert lib.la_select_workspace(15) == 0
    assert lib.la_select_workspace(0) == 0


def test_workspace_query(lib):
    assert binding.la_step_attention_workspace_bytes(1024, 15, 5, 15, 32, 32, 128) > 0
    assert binding.la_step_attention_workspace_bytes(0, 0, 2, 0, 1, 1, 128) == 0
    assert binding.la_step_attention_workspace_bytes(0, 0, 2, 0, 3, 2, 128) == 0


def test_binding_rejects_host_tensors():
    import torch
    z = torch.zeros((1, 1, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        binding.la_step_attention(z, None, None, z, z, 0, 0, 2, 0, 1, 1, 64, z)


def test_kernel_choice_is_a_host_side_query(lib):
    """Which kernel a plain step takes, without a GPU: the benchmark's shapes keep the staged kernel,
    the 7B step on a short prefix takes the row-tile one; the hooks force either."""
    k = lib.la_step_attention_kernel
    assert k(1024, 15, 5, 15, 32, 32, 128) == 0        # the 7B configuration
    assert k(2048, 10, 5, 10, 40, 40, 128) == 0
    assert k(4096, 7, 5, 7, 64, 8, 128) == 0
    assert k(256, 15, 5, 15, 32, 32, 128) == 1         # 6 chunks, 256 workgroups
    assert k(640, 15, 5, 15, 32, 32, 128) == 1         # 12 chunks: the last one it takes
    assert k(704, 15, 5, 15, 32, 32, 128) == 0
    assert k(256, 30, 5, 30, 32, 32, 128) == 0         # 512 workgroups: more than one round
    assert k(64, 4, 3, 2, 4, 4, 64) == 0               # head_dim 64: the staged kernel only
    assert k(64, 4, 1, 2, 4, 4, 128) == -1 and k(64, 4, 3, 2, 4, 3, 128) == -1
    try:
        assert lib.la_debug_override(b"attn_rowtile", b"1") == 0
        assert k(1024, 15, 5, 15, 32, 32, 128) == 1 and k(64, 4, 3, 2, 4, 4, 64) == 0
        assert lib.la_debug_override(b"attn_plan", b"2,4,0,4,64") == 0
        assert k(256, 15, 5, 15, 32, 32, 128) == 0     # a forced decomposition is the staged kernel
        assert lib.la_debug_override(b"attn_plan", None) == 0
        assert lib.la_debug_override(b"attn_rowtile", b"0") == 0
        assert k(256, 15, 5, 15, 32, 32, 128) == 0
    finally:
        lib.la_debug_override(b"attn_plan", None)
        lib.la_debug_override(b"attn_rowtile", None)
    assert k(256, 15, 5, 15, 32, 32, 128) == 1
