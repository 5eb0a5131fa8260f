"""Thin ctypes binding of the C-ABI HIP library (include/la.h): argument marshalling only.

Every step of the hot path runs in the library's kernels.  There is no fallback: if the
library has not been built (python -m paper_2402_02057_amd.buildlib, or
__graft_entry__.build()) loading fails loudly.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libla_hip.so")

LA_OK = 0
LA_EINVAL, LA_EUNSUPPORTED, LA_ENOMEM, LA_EHIP = -1, -2, -3, -4
_lib = None


class StepDesc(ctypes.Structure):
    """la_step_desc of include/la.h."""
    _fields_ = [("q", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("step_k", ctypes.c_void_p), ("step_v", ctypes.c_void_p), ("out", ctypes.c_void_p),
                ("P", ctypes.c_int), ("reserved", ctypes.c_int)]


class StepDescPaged(ctypes.Structure):
    """la_step_desc_paged of include/la.h."""
    _fields_ = [("q", ctypes.c_void_p), ("block_table", ctypes.c_void_p), ("step_k", ctypes.c_void_p),
                ("step_v", ctypes.c_void_p), ("out", ctypes.c_void_p), ("P", ctypes.c_int), ("reserved", ctypes.c_int)]


class CommitDesc(ctypes.Structure):
    """la_commit_desc of include/la.h."""
    _fields_ = [("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
                ("step_k", ctypes.c_void_p), ("step_v", ctypes.c_void_p), ("best", ctypes.c_void_p),
                ("n_out", ctypes.c_void_p), ("capacity", ctypes.c_longlong), ("P", ctypes.c_int),
                ("reserved", ctypes.c_int)]


class VerifyDesc(ctypes.Structure):
    """la_verify_desc of include/la.h."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("logits_cur", "logits_look", "logits_cand", "cand_tokens",
                                                "out_tokens", "n_out", "best", "new_window", "accept_len")]


class SampleDesc(ctypes.Structure):
    """la_sample_desc of include/la.h."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("logits_cur", "logits_cand", "cand_tokens", "u_test", "u_final",
                                                "out_tokens", "n_out")] + \
               [("temperature", ctypes.c_float), ("reserved", ctypes.c_int)]


class LaError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("la error %d: %s" % (code, message))
        self.code = code


def load():
    """Open libla_hip.so (once).  Raises if it is missing: the HIP path is the only path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library %s is not built; run __graft_entry__.build()" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    i, p = ctypes.c_int, ctypes.c_void_p
    lib.la_step_attention.argtypes = [p, p, p, p, p, i, i, i, i, i, i, i, p, p]
    lib.la_step_attention.restype = i
    lib.la_step_attention_noalloc.argtypes = [p, p, p, p, p, i, i, i, i, i, i, i, p, p]
    lib.la_step_attention_noalloc.restype = i
    lib.la_step_attention_fp8kv.argtypes = [p, p, p, p, p, p, p, i, i, i, i, i, i, i, p, p]
    lib.la_step_attention_fp8kv.restype = i
    lib.la_step_attention_rope.argtypes = [p, p, p, p, p, p, p, i, i, i, i, i, i, i, i, i, i, p, p]
    lib.la_step_attention_rope.restype = i
    ll = ctypes.c_longlong
    lib.la_step_attention_cap.argtypes = [p, p, p, ll, p, p, i, i, i, i, i, i, i, p, p]
    lib.la_step_attention_cap.restype = i
    lib.la_kv_commit.argtypes = [p, p, ll, p, p, i, i, i, i, i, i, p, p, p]
    lib.la_kv_commit.restype = i
    lib.la_kv_commit_rope.argtypes = [p, p, ll, p, p, p, p, i, i, i, i, i, i, i, i, p, p, p]
    lib.la_kv_commit_rope.restype = i
    lib.la_verify_sample_batch.argtypes = [p, i, i, i, i, p]
    lib.la_verify_sample_batch.restype = i
    lib.la_step_rope.argtypes = [p, p, p, p, i, i, i, i, i, i, i, i, i, p]
    lib.la_step_rope.restype = i
    lib.la_verify_step_batch.argtypes = [p, i, i, i, i, i, p]
    lib.la_verify_step_batch.restype = i
    lib.la_kv_commit_batch.argtypes = [p, i, i, i, i, i, i, i, i, p]
    lib.la_kv_commit_batch.restype = i
    lib.la_step_attention_batch.argtypes = [p, i, i, i, i, i, i, i, p]
    lib.la_step_attention_batch.restype = i
    lib.la_step_attention_batch_paged.argtypes = [p, i, p, p, i, i, i, i, i, i, i, i, p]
    lib.la_step_attention_batch_paged.restype = i
    lib.la_step_attention_rows.argtypes = [p, p, p, p, p, p, i, i, i, i, i, i, i, i, p, p]
    lib.la_step_attention_rows.restype = i
    lib.la_step_attention_paged.argtypes = [p, p, p, p, i, i, p, p, i, i, i, i, i, i, i, p, p]
    lib.la_step_attention_paged.restype = i
    lib.la_kv_commit_paged.argtypes = [p, p, p, i, i, p, p, i, i, i, i, i, i, p, p, p]
    lib.la_kv_commit_paged.restype = i
    lib.la_verify.argtypes = [p, p, i, i, i, p, p, p]
    lib.la_verify.restype = i
    lib.la_verify_step.argtypes = [p, p, p, p, i, i, i, i, p, p, p, p, p, p]
    lib.la_verify_step.restype = i
    lib.la_verify_sample.argtypes = [p, p, p, p, p, ctypes.c_float, i, i, i, p, p, p]
    lib.la_verify_sample.restype = i
    lib.la_step_attention_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    lib.la_step_attention_workspace_bytes.restype = ctypes.c_longlong
    lib.la_step_attention_kernel.argtypes = [i, i, i, i, i, i, i]
    lib.la_step_attention_kernel.restype = i
    lib.la_shutdown.argtypes = []
    lib.la_shutdown.restype = None
    lib.la_last_error.argtypes = []
    lib.la_last_error.restype = ctypes.c_char_p
    lib.la_probe_stream_read.argtypes = [p, ll, p, p]
    lib.la_probe_stream_read.restype = i
    lib.la_probe_mfma.argtypes = [i, p, p]
    lib.la_probe_mfma.restype = ll
    lib.la_debug_override.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    lib.la_debug_override.restype = i
    lib.la_select_workspace.argtypes = [i]
    lib.la_select_workspace.restype = i
    lib.la_version.argtypes = []
    lib.la_version.restype = i
    _lib = lib
    return lib


EXPORTS = ("la_step_rope", "la_step_attention", "la_step_attention_noalloc", "la_step_attention_fp8kv", "la_step_attention_rope", "la_step_attention_cap", "la_kv_commit", "la_kv_commit_rope", "la_step_attention_paged", "la_kv_commit_paged", "la_kv_commit_batch", "la_step_attention_rows", "la_step_attention_batch", "la_step_attention_batch_paged", "la_verify", "la_verify_step", "la_verify_step_batch", "la_verify_sample", "la_verify_sample_batch", "la_step_attention_workspace_bytes", "la_step_attention_kernel", "la_shutdown", "la_select_workspace", "la_debug_override", "la_probe_stream_read", "la_probe_mfma",
           "la_last_error", "la_version")


def _check(rc):
    if rc != LA_OK:
        raise LaError(rc, load().la_last_error().decode())


def _ptr(x, dtype, shape, name, allow_empty_null=False):
    """Device pointer of a contiguous CUDA tensor of the expected dtype and shape."""
    if x is None:
        if allow_empty_null:
            return None
        raise ValueError("%s is None" % name)
    if not isinstance(x, torch.Tensor):
        raise TypeError("%s must be a torch.Tensor" % name)
    if not x.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if x.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, x.dtype))
    if tuple(x.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(x.shape)))
    if not x.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return x.data_ptr() if x.numel() else None


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def la_step_attention(q, k_cache, v_cache, step_k, step_v, P, W, N, G, heads, kv_heads, head_dim,
                      out, stream=None):
    """out[T, heads, head_dim] (bf16) <- lookahead-step attention; asynchronous on `stream`."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    rc = load().la_step_attention(
        _ptr(q, bf, (T, heads, head_dim), "q"),
        _ptr(k_cache, bf, (kv_heads, P, head_dim), "k_cache", allow_empty_null=True),
        _ptr(v_cache, bf, (kv_heads, P, head_dim), "v_cache", allow_empty_null=True),
        _ptr(step_k, bf, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (T, kv_heads, head_dim), "step_v"),
        P, W, N, G, heads, kv_heads, head_dim,
        _ptr(out, bf, (T, heads, head_dim), "out"), _stream(stream))
    _check(rc)
    return out


def la_step_attention_noalloc(q, k_cache, v_cache, step_k, step_v, P, W, N, G, heads, kv_heads, head_dim,
                              out, stream=None):
    """la_step_attention through the entry point that allocates nothing (fixed scratch block)."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    rc = load().la_step_attention_noalloc(
        _ptr(q, bf, (T, heads, head_dim), "q"),
        _ptr(k_cache, bf, (kv_heads, P, head_dim), "k_cache", allow_empty_null=True),
        _ptr(v_cache, bf, (kv_heads, P, head_dim), "v_cache", allow_empty_null=True),
        _ptr(step_k, bf, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (T, kv_heads, head_dim), "step_v"),
        P, W, N, G, heads, kv_heads, head_dim,
        _ptr(out, bf, (T, heads, head_dim), "out"), _stream(stream))
    _check(rc)
    return out


def la_step_attention_fp8kv(q, k_cache, v_cache, step_k, step_v, k_scale, v_scale, P, W, N, G, heads, kv_heads,
                            head_dim, out, stream=None):
    """The step over a cache of 8-bit floats (uint8 codes, cache and step rows) with one fp32 scale per
    KV head for the keys and one for the values; q and out are bf16.  Asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf, u8 = torch.bfloat16, torch.uint8
    rc = load().la_step_attention_fp8kv(
        _ptr(q, bf, (T, heads, head_dim), "q"),
        _ptr(k_cache, u8, (kv_heads, P, head_dim), "k_cache", allow_empty_null=True),
        _ptr(v_cache, u8, (kv_heads, P, head_dim), "v_cache", allow_empty_null=True),
        _ptr(step_k, u8, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, u8, (T, kv_heads, head_dim), "step_v"),
        _ptr(k_scale, torch.float32, (kv_heads,), "k_scale"),
        _ptr(v_scale, torch.float32, (kv_heads,), "v_scale"),
        P, W, N, G, heads, kv_heads, head_dim,
        _ptr(out, bf, (T, heads, head_dim), "out"), _stream(stream))
    _check(rc)
    return out


def la_step_attention_cap(q, k_cache, v_cache, step_k, step_v, P, W, N, G, heads, kv_heads, head_dim, out,
                          stream=None):
    """la_step_attention over caches [kv_heads, capacity, head_dim] whose first P rows per head are
    the prefix (capacity is read from the tensors); asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    capacity = int(k_cache.shape[1])
    rc = load().la_step_attention_cap(
        _ptr(q, bf, (T, heads, head_dim), "q"),
        _ptr(k_cache, bf, (kv_heads, capacity, head_dim), "k_cache"),
        _ptr(v_cache, bf, (kv_heads, capacity, head_dim), "v_cache"), capacity,
        _ptr(step_k, bf, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (T, kv_heads, head_dim), "step_v"),
        P, W, N, G, heads, kv_heads, head_dim,
        _ptr(out, bf, (T, heads, head_dim), "out"), _stream(stream))
    _check(rc)
    return out


def la_step_rope(q, step_k, cos, sin, P, W, N, G, heads, kv_heads, head_dim, interleaved=False, stream=None):
    """Rotate q [T, heads, d] and step_k [T, kv_heads, d] (bf16, in place) by the step's positions with
    the fp32 tables cos, sin [max_pos, d/2]; asynchronous."""
    T = 1 + (W + G) * (N - 1)
    max_pos = int(cos.shape[0])
    rc = load().la_step_rope(
        _ptr(q, torch.bfloat16, (T, heads, head_dim), "q", allow_empty_null=True),   # None: the keys alone
        _ptr(step_k, torch.bfloat16, (T, kv_heads, head_dim), "step_k"),
        _ptr(cos, torch.float32, (max_pos, head_dim // 2), "cos"),
        _ptr(sin, torch.float32, (max_pos, head_dim // 2), "sin"),
        max_pos, P, W, N, G, heads, kv_heads, head_dim, 1 if interleaved else 0, _stream(stream))
    _check(rc)


def la_step_attention_rope(q, k_cache, v_cache, step_k, step_v, cos, sin, P, W, N, G, heads, kv_heads, head_dim, out,
                           interleaved=False, stream=None, rotate_keys=False):
    """la_step_attention with q rotated inside the kernel (q is left as it is).  rotate_keys False:
    step_k must be rotated already, e.g. by la_step_rope(None, step_k, ...); True: step_k comes
    unrotated too and the kernel turns the step keys it stages (append with la_kv_commit_rope then);
    asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    max_pos = int(cos.shape[0])
    rc = load().la_step_attention_rope(
        _ptr(q, bf, (T, heads, head_dim), "q"),
        _ptr(k_cache, bf, (kv_heads, P, head_dim), "k_cache", allow_empty_null=True),
        _ptr(v_cache, bf, (kv_heads, P, head_dim), "v_cache", allow_empty_null=True),
        _ptr(step_k, bf, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (T, kv_heads, head_dim), "step_v"),
        _ptr(cos, torch.float32, (max_pos, head_dim // 2), "cos"),
        _ptr(sin, torch.float32, (max_pos, head_dim // 2), "sin"),
        max_pos, 1 if interleaved else 0, 1 if rotate_keys else 0, P, W, N, G, heads, kv_heads, head_dim,
        _ptr(out, bf, (T, heads, head_dim), "out"), _stream(stream))
    _check(rc)
    return out


def la_kv_commit(k_cache, v_cache, step_k, step_v, P, W, N, G, kv_heads, head_dim, best, n_out, stream=None):
    """Append the rows of the tokens la_verify_step accepted (device-side best, n_out) to the caches
    [kv_heads, capacity, head_dim] at row P; asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    capacity = int(k_cache.shape[1])
    rc = load().la_kv_commit(
        _ptr(k_cache, bf, (kv_heads, capacity, head_dim), "k_cache"),
        _ptr(v_cache, bf, (kv_heads, capacity, head_dim), "v_cache"), capacity,
        _ptr(step_k, bf, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (T, kv_heads, head_dim), "step_v"),
        P, W, N, G, kv_heads, head_dim,
        _ptr(best, torch.int32, (1,), "best"), _ptr(n_out, torch.int32, (1,), "n_out"), _stream(stream))
    _check(rc)


def la_kv_commit_rope(k_cache, v_cache, step_k, step_v, cos, sin, P, W, N, G, kv_heads, head_dim, best, n_out,
                      interleaved=False, stream=None):
    """la_kv_commit for unrotated step keys: the appended key rows are turned by their cache positions
    (tables as for la_step_rope); asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    capacity = int(k_cache.shape[1])
    max_pos = int(cos.shape[0])
    rc = load().la_kv_commit_rope(
        _ptr(k_cache, bf, (kv_heads, capacity, head_dim), "k_cache"),
        _ptr(v_cache, bf, (kv_heads, capacity, head_dim), "v_cache"), capacity,
        _ptr(step_k, bf, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (T, kv_heads, head_dim), "step_v"),
        _ptr(cos, torch.float32, (max_pos, head_dim // 2), "cos"),
        _ptr(sin, torch.float32, (max_pos, head_dim // 2), "sin"),
        max_pos, 1 if interleaved else 0, P, W, N, G, kv_heads, head_dim,
        _ptr(best, torch.int32, (1,), "best"), _ptr(n_out, torch.int32, (1,), "n_out"), _stream(stream))
    _check(rc)


def la_step_attention_batch(seqs, W, N, G, heads, kv_heads, head_dim, stream=None):
    """Several steps in one launch.  `seqs` is a list of dicts with q, k_cache, v_cache, step_k,
    step_v, out (tensors as for la_step_attention) and P; asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    descs = (StepDesc * len(seqs))()
    for d, x in zip(descs, seqs):
        P = int(x["P"])
        d.q = _ptr(x["q"], bf, (T, heads, head_dim), "q")
        d.k_cache = _ptr(x["k_cache"], bf, (kv_heads, P, head_dim), "k_cache", allow_empty_null=True)
        d.v_cache = _ptr(x["v_cache"], bf, (kv_heads, P, head_dim), "v_cache", allow_empty_null=True)
        d.step_k = _ptr(x["step_k"], bf, (T, kv_heads, head_dim), "step_k")
        d.step_v = _ptr(x["step_v"], bf, (T, kv_heads, head_dim), "step_v")
        d.out = _ptr(x["out"], bf, (T, heads, head_dim), "out")
        d.P, d.reserved = P, 0
    _check(load().la_step_attention_batch(ctypes.cast(descs, ctypes.c_void_p), len(seqs), W, N, G, heads, kv_heads,
                                          head_dim, _stream(stream)))


def la_step_attention_batch_paged(seqs, k_pages, v_pages, W, N, G, heads, kv_heads, head_dim, stream=None):
    """Several steps over one paged cache in one launch.  `seqs`: dicts with q, block_table (int32
    tensor, >= ceil(P / page_size) entries, or None if P == 0), step_k, step_v, out, P; asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    n_pages, page_size = int(k_pages.shape[0]), int(k_pages.shape[2])
    shape = (n_pages, kv_heads, page_size, head_dim)
    descs = (StepDescPaged * len(seqs))()
    for d, x in zip(descs, seqs):
        P = int(x["P"])
        need = (P + page_size - 1) // page_size
        bt = x.get("block_table")
        if need > 0 and (bt is None or bt.numel() < need):
            raise ValueError("block_table must hold at least %d entries" % need)
        d.q = _ptr(x["q"], bf, (T, heads, head_dim), "q")
        d.block_table = None if bt is None else _ptr(bt, torch.int32, (bt.numel(),), "block_table", allow_empty_null=True)
        d.step_k = _ptr(x["step_k"], bf, (T, kv_heads, head_dim), "step_k")
        d.step_v = _ptr(x["step_v"], bf, (T, kv_heads, head_dim), "step_v")
        d.out = _ptr(x["out"], bf, (T, heads, head_dim), "out")
        d.P, d.reserved = P, 0
    _check(load().la_step_attention_batch_paged(ctypes.cast(descs, ctypes.c_void_p), len(seqs),
                                                _ptr(k_pages, bf, shape, "k_pages"), _ptr(v_pages, bf, shape, "v_pages"),
                                                page_size, n_pages, W, N, G, heads, kv_heads, head_dim, _stream(stream)))


def la_step_attention_rows(q, k_cache, v_cache, step_k, step_v, row_ids, P, W, N, G, heads, kv_heads, head_dim, out,
                           stream=None):
    """la_step_attention over the rows `row_ids` (int32 tensor) of the (W, N, G) layout: a device's
    share under lookahead parallelism; asynchronous."""
    n = int(row_ids.numel())
    bf = torch.bfloat16
    rc = load().la_step_attention_rows(
        _ptr(q, bf, (n, heads, head_dim), "q"),
        _ptr(k_cache, bf, (kv_heads, P, head_dim), "k_cache", allow_empty_null=True),
        _ptr(v_cache, bf, (kv_heads, P, head_dim), "v_cache", allow_empty_null=True),
        _ptr(step_k, bf, (n, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (n, kv_heads, head_dim), "step_v"),
        _ptr(row_ids, torch.int32, (n,), "row_ids"), n, P, W, N, G, heads, kv_heads, head_dim,
        _ptr(out, bf, (n, heads, head_dim), "out"), _stream(stream))
    _check(rc)
    return out


def _pages(k_pages, v_pages, block_table, kv_heads, head_dim, rows):
    n_pages, page_size = int(k_pages.shape[0]), int(k_pages.shape[2])
    shape = (n_pages, kv_heads, page_size, head_dim)
    need = (rows + page_size - 1) // page_size
    if need > 0 and (block_table is None or block_table.numel() < need):
        raise ValueError("block_table must hold at least %d entries" % need)
    bt = None if block_table is None else _ptr(block_table, torch.int32, (block_table.numel(),), "block_table",
                                               allow_empty_null=True)
    return (_ptr(k_pages, torch.bfloat16, shape, "k_pages"), _ptr(v_pages, torch.bfloat16, shape, "v_pages"), bt,
            page_size, n_pages)


def la_step_attention_paged(q, k_pages, v_pages, block_table, step_k, step_v, P, W, N, G, heads, kv_heads,
                            head_dim, out, stream=None):
    """la_step_attention over pages [n_pages, kv_heads, page_size, head_dim] named by the int32
    block_table (>= ceil(P / page_size) entries); asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    kp, vp, bt, page_size, n_pages = _pages(k_pages, v_pages, block_table, kv_heads, head_dim, P)
    rc = load().la_step_attention_paged(
        _ptr(q, bf, (T, heads, head_dim), "q"), kp, vp, bt, page_size, n_pages,
        _ptr(step_k, bf, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (T, kv_heads, head_dim), "step_v"),
        P, W, N, G, heads, kv_heads, head_dim,
        _ptr(out, bf, (T, heads, head_dim), "out"), _stream(stream))
    _check(rc)
    return out


def la_kv_commit_paged(k_pages, v_pages, block_table, step_k, step_v, P, W, N, G, kv_heads, head_dim, best,
                       n_out, stream=None):
    """la_kv_commit into pages; block_table needs >= ceil((P + N) / page_size) entries; asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    kp, vp, bt, page_size, n_pages = _pages(k_pages, v_pages, block_table, kv_heads, head_dim, P + N)
    rc = load().la_kv_commit_paged(
        kp, vp, bt, page_size, n_pages,
        _ptr(step_k, bf, (T, kv_heads, head_dim), "step_k"),
        _ptr(step_v, bf, (T, kv_heads, head_dim), "step_v"),
        P, W, N, G, kv_heads, head_dim,
        _ptr(best, torch.int32, (1,), "best"), _ptr(n_out, torch.int32, (1,), "n_out"), _stream(stream))
    _check(rc)


def la_kv_commit_batch(appends, W, N, G, kv_heads, head_dim, stream=None):
    """Several appends in one launch.  `appends`: dicts with k_cache, v_cache, step_k, step_v, best,
    n_out, P and, for a paged cache, block_table (then k_cache / v_cache are the page pools
    [n_pages, kv_heads, page_size, head_dim], the same geometry in all of them); asynchronous."""
    T = 1 + (W + G) * (N - 1)
    bf = torch.bfloat16
    descs = (CommitDesc * len(appends))()
    page_size = n_pages = 0
    for d, x in zip(descs, appends):
        P = int(x["P"])
        bt = x.get("block_table")
        if bt is not None:
            kp, vp, btp, ps, npg = _pages(x["k_cache"], x["v_cache"], bt, kv_heads, head_dim, P + N)
            if page_size and (ps, npg) != (page_size, n_pages):
                raise ValueError("all page pools of a launch must have the same geometry")
            page_size, n_pages = ps, npg
            d.k_cache, d.v_cache, d.block_table, d.capacity = kp, vp, btp, 0
        else:
            cap = int(x["k_cache"].shape[1])
            d.k_cache = _ptr(x["k_cache"], bf, (kv_heads, cap, head_dim), "k_cache")
            d.v_cache = _ptr(x["v_cache"], bf, (kv_heads, cap, head_dim), "v_cache")
            d.block_table, d.capacity = None, cap
        d.step_k = _ptr(x["step_k"], bf, (T, kv_heads, head_dim), "step_k")
        d.step_v = _ptr(x["step_v"], bf, (T, kv_heads, head_dim), "step_v")
        d.best = _ptr(x["best"], torch.int32, (1,), "best")
        d.n_out = _ptr(x["n_out"], torch.int32, (1,), "n_out")
        d.P, d.reserved = P, 0
    _check(load().la_kv_commit_batch(ctypes.cast(descs, ctypes.c_void_p), len(appends), page_size, n_pages, W, N, G,
                                     kv_heads, head_dim, _stream(stream)))


def la_verify(logits, cand_tokens, G, N, V, accept_len, accepted, stream=None):
    """accept_len[G], accepted[G, N-1] (int32) <- greedy verification; asynchronous."""
    rc = load().la_verify(
        _ptr(logits, torch.float32, (G, N - 1, V), "logits"),
        _ptr(cand_tokens, torch.int32, (G, N - 1), "cand_tokens"), G, N, V,
        _ptr(accept_len, torch.int32, (G,), "accept_len"),
        _ptr(accepted, torch.int32, (G, N - 1), "accepted"), _stream(stream))
    _check(rc)
    return accept_len, accepted


def la_verify_step(logits_cur, logits_look, logits_cand, cand_tokens, W, N, G, V, out_tokens, n_out, best,
                   new_window, accept_len=None, stream=None):
    """out_tokens[N], n_out[1], best[1], new_window[W], accept_len[G] (int32) <- the end of a greedy
    step (accepted tokens of the best candidate plus correction or bonus token; new window tokens);
    asynchronous."""
    rc = load().la_verify_step(
        _ptr(logits_cur, torch.float32, (V,), "logits_cur"),
        _ptr(logits_look, torch.float32, (W, V), "logits_look", allow_empty_null=True),
        _ptr(logits_cand, torch.float32, (G, N - 1, V), "logits_cand", allow_empty_null=True),
        _ptr(cand_tokens, torch.int32, (G, N - 1), "cand_tokens", allow_empty_null=True), W, N, G, V,
        _ptr(out_tokens, torch.int32, (N,), "out_tokens"), _ptr(n_out, torch.int32, (1,), "n_out"),
        _ptr(best, torch.int32, (1,), "best"),
        _ptr(new_window, torch.int32, (W,), "new_window", allow_empty_null=True),
        _ptr(accept_len, torch.int32, (G,), "accept_len", allow_empty_null=True), _stream(stream))
    _check(rc)
    return out_tokens, n_out, best, new_window, accept_len


def la_verify_step_batch(seqs, W, N, G, V, stream=None):
    """The ends of several sequences' steps in one launch.  `seqs`: dicts with logits_cur, logits_look,
    logits_cand, cand_tokens, out_tokens, n_out, best, new_window and optionally accept_len (tensors
    as for la_verify_step); asynchronous."""
    descs = (VerifyDesc * len(seqs))()
    f, i32 = torch.float32, torch.int32
    for d, x in zip(descs, seqs):
        d.logits_cur = _ptr(x["logits_cur"], f, (V,), "logits_cur")
        d.logits_look = _ptr(x.get("logits_look"), f, (W, V), "logits_look", allow_empty_null=True)
        d.logits_cand = _ptr(x.get("logits_cand"), f, (G, N - 1, V), "logits_cand", allow_empty_null=True)
        d.cand_tokens = _ptr(x.get("cand_tokens"), i32, (G, N - 1), "cand_tokens", allow_empty_null=True)
        d.out_tokens = _ptr(x["out_tokens"], i32, (N,), "out_tokens")
        d.n_out = _ptr(x["n_out"], i32, (1,), "n_out")
        d.best = _ptr(x["best"], i32, (1,), "best")
        d.new_window = _ptr(x.get("new_window"), i32, (W,), "new_window", allow_empty_null=True)
        d.accept_len = _ptr(x.get("accept_len"), i32, (G,), "accept_len", allow_empty_null=True)
    _check(load().la_verify_step_batch(ctypes.cast(descs, ctypes.c_void_p), len(seqs), W, N, G, V, _stream(stream)))


def la_verify_sample(logits_cur, logits_cand, cand_tokens, u_test, u_final, temperature, N, G, V, out_tokens,
                     n_out, stream=None):
    """out_tokens[N], n_out[1] (int32) <- sampling verification (Algorithm 4); asynchronous."""
    rc = load().la_verify_sample(
        _ptr(logits_cur, torch.float32, (V,), "logits_cur"),
        _ptr(logits_cand, torch.float32, (G, N - 1, V), "logits_cand", allow_empty_null=True),
        _ptr(cand_tokens, torch.int32, (G, N - 1), "cand_tokens", allow_empty_null=True),
        _ptr(u_test, torch.float32, (N - 1, G), "u_test", allow_empty_null=True),
        _ptr(u_final, torch.float32, (1,), "u_final"), float(temperature), N, G, V,
        _ptr(out_tokens, torch.int32, (N,), "out_tokens"), _ptr(n_out, torch.int32, (1,), "n_out"),
        _stream(stream))
    _check(rc)
    return out_tokens, n_out


def la_verify_sample_batch(seqs, N, G, V, stream=None):
    """Sampling verification of several sequences in one launch.  `seqs`: dicts with logits_cur,
    logits_cand, cand_tokens, u_test, u_final, temperature, out_tokens, n_out (tensors as for
    la_verify_sample); asynchronous."""
    descs = (SampleDesc * len(seqs))()
    f, i32 = torch.float32, torch.int32
    for d, x in zip(descs, seqs):
        d.logits_cur = _ptr(x["logits_cur"], f, (V,), "logits_cur")
        d.logits_cand = _ptr(x.get("logits_cand"), f, (G, N - 1, V), "logits_cand", allow_empty_null=True)
        d.cand_tokens = _ptr(x.get("cand_tokens"), i32, (G, N - 1), "cand_tokens", allow_empty_null=True)
        d.u_test = _ptr(x.get("u_test"), f, (N - 1, G), "u_test", allow_empty_null=True)
        d.u_final = _ptr(x["u_final"], f, (1,), "u_final")
        d.out_tokens = _ptr(x["out_tokens"], i32, (N,), "out_tokens")
        d.n_out = _ptr(x["n_out"], i32, (1,), "n_out")
        d.temperature, d.reserved = float(x["temperature"]), 0
    _check(load().la_verify_sample_batch(ctypes.cast(descs, ctypes.c_void_p), len(seqs), N, G, V, _stream(stream)))


def la_step_attention_kernel(P, W, N, G, heads, kv_heads, head_dim):
    """0: the staged kernel, 1: the row-tile kernel (what la_step_attention takes for this shape)."""
    return int(load().la_step_attention_kernel(P, W, N, G, heads, kv_heads, head_dim))


def la_step_attention_workspace_bytes(P, W, N, G, heads, kv_heads, head_dim):
    return int(load().la_step_attention_workspace_bytes(P, W, N, G, heads, kv_heads, head_dim))


def la_shutdown():
    load().la_shutdown()


def la_select_workspace(index):
    """The calling thread's next calls use workspace set `index` (0..15): calls on different streams
    that may overlap need different sets."""
    _check(load().la_select_workspace(int(index)))


def la_version():
    return int(load().la_version())


def bf16_tensor(bits, device="cuda"):
    """numpy uint16 bit patterns -> bf16 tensor on the device (no value conversion)."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).copy())
    return t.view(torch.bfloat16).to(device)


def bf16_bits(t):
    """bf16 tensor -> numpy uint16 bit patterns on the host."""
    import numpy as np
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def la_debug_override(key, value):
    """Testing hook: force a decomposition ("attn_plan", "batch_plan") or the recompute path
    ("force_recompute"); value None clears it."""
    _check(load().la_debug_override(key.encode(), None if value is None else str(value).encode()))


def la_probe_stream_read(buf, sink, stream=None):
    """Measurement aid: read every byte of the uint8 tensor `buf` once (asynchronous)."""
    _check(load().la_probe_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream(stream)))


def la_probe_mfma(iters, sink, stream=None):
    """Measurement aid: a register-resident bf16 MFMA loop; returns the flops of the launch."""
    flops = load().la_probe_mfma(int(iters), sink.data_ptr(), _stream(stream))
    if flops < 0:
        raise LaError(LA_EHIP, load().la_last_error().decode())
    return int(flops)
