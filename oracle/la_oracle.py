"""ctypes front end of the plain-C fp64 oracle, plus the paper's Algorithm 3 in Python.

Test infrastructure only (tests, the smoke check, the benchmark's cpu_baseline leg).
bf16 tensors travel as numpy uint16 bit patterns; nothing here touches the GPU library.
`kv_commit` (appending the accepted tokens to the KV cache) is plain numpy; its pin is that the
cache after any run of lookahead steps equals the cache of plain autoregressive decoding.
`step_attention_rows` is the step over a subset of its rows (one device's share under lookahead
parallelism), dense numpy with the explicit mask, pinned by equality with the full step on closed
subsets.  `gather_pages` / `kv_commit_paged` define what a paged cache stands for (pinned as the inverse of
a scatter written in the test, and against the packed append).
`step_attention_fp8kv` is the step over a KV cache quantised to 8-bit floats with one scale per KV head
(decode, scale, then the same dense definition); pins: every code point against a library's cast,
equality with the 16-bit step on inputs both formats hold exactly, linearity in the value scale, the
one-token decode against a library attention, and a hand-indexed read-out of one value row.
`step_rope` rotates the step's queries and keys by the positions of Fig. 2(b) (rotary position
embedding written out pair by pair in fp64); pins: the printed digits, norms, the dependence of a
score on the distance only, a quarter turn, and complex multiplication.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        i, p = ctypes.c_int, ctypes.c_void_p
        lib.la_oracle_num_rows.argtypes = [i, i, i]
        lib.la_oracle_num_rows.restype = i
        lib.la_oracle_position.argtypes = [i, i, i, i]
        lib.la_oracle_position.restype = i
        lib.la_oracle_visible.argtypes = [i, i, i, i, i]
        lib.la_oracle_visible.restype = i
        lib.la_oracle_step_mask.argtypes = [i, i, i, p]
        lib.la_oracle_step_mask.restype = None
        lib.la_oracle_threads.argtypes = []
        lib.la_oracle_threads.restype = i
        lib.la_oracle_step_attention.argtypes = [p, p, p, p, p, i, i, i, i, i, i, i, p]
        lib.la_oracle_step_attention.restype = i
        lib.la_oracle_step_attention_fp8kv.argtypes = [p, p, p, p, p, p, p, i, i, i, i, i, i, i, p]
        lib.la_oracle_step_attention_fp8kv.restype = i
        lib.la_oracle_fp8_e4m3_decode.argtypes = [p, ctypes.c_size_t, p]
        lib.la_oracle_fp8_e4m3_decode.restype = None
        lib.la_oracle_verify.argtypes = [p, p, i, i, i, p, p]
        lib.la_oracle_verify.restype = i
        lib.la_oracle_verify_step.argtypes = [p, p, p, p, i, i, i, i, p, p, p, p, p]
        lib.la_oracle_verify_step.restype = i
        f = ctypes.c_float
        lib.la_oracle_verify_sample.argtypes = [p, p, p, p, f, f, i, i, i, p, p]
        lib.la_oracle_verify_sample.restype = i
        _lib = lib
    return _lib


def num_rows(W, N, G):
    return _load().la_oracle_num_rows(W, N, G)


def position(r, W, N, G):
    return _load().la_oracle_position(r, W, N, G)


def threads():
    return _load().la_oracle_threads()


def set_threads(n):
    """Let the oracle's loops over heads use `n` threads from now on (for timing on one core)."""
    _load().la_oracle_set_threads(int(n))


def step_mask(W, N, G):
    """bool [T, T]: may step row r attend to step key c (Sec. 3.3)."""
    T = num_rows(W, N, G)
    m = np.zeros((T, T), dtype=np.uint8)
    _load().la_oracle_step_mask(W, N, G, m.ctypes.data)
    return m.astype(bool)


def _u16(a, shape):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def step_attention(q, k_cache, v_cache, step_k, step_v, P, W, N, G, heads, kv_heads, head_dim):
    """fp64 [T, heads, head_dim] from bf16 bit patterns (uint16 arrays)."""
    T = num_rows(W, N, G)
    q = _u16(q, (T, heads, head_dim))
    k_cache = _u16(k_cache, (kv_heads, P, head_dim))
    v_cache = _u16(v_cache, (kv_heads, P, head_dim))
    step_k = _u16(step_k, (T, kv_heads, head_dim))
    step_v = _u16(step_v, (T, kv_heads, head_dim))
    out = np.empty((T, heads, head_dim), dtype=np.float64)
    rc = _load().la_oracle_step_attention(q.ctypes.data, k_cache.ctypes.data, v_cache.ctypes.data,
                                          step_k.ctypes.data, step_v.ctypes.data, P, W, N, G,
                                          heads, kv_heads, head_dim, out.ctypes.data)
    if rc != 0:
        raise ValueError("la_oracle_step_attention: bad shape (rc=%d)" % rc)
    return out


def _u8(a, shape):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint8 and a.shape == tuple(shape), (a.dtype, a.shape, shape)
    return a


def fp8_e4m3_decode(codes):
    """fp64 values of 8-bit float codes (E4M3, finite-only: exponent bias 7, no infinities, 0x7f / 0xff NaN)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, dtype=np.float64)
    _load().la_oracle_fp8_e4m3_decode(codes.ctypes.data, ctypes.c_size_t(codes.size), out.ctypes.data)
    return out


def step_attention_fp8kv(q, k_cache, v_cache, step_k, step_v, k_scale, v_scale, P, W, N, G, heads, kv_heads,
                         head_dim):
    """The step over a quantised KV cache: fp64 [T, heads, head_dim] from a bf16 q (uint16 bit patterns),
    8-bit float keys and values (uint8 codes, cache and step rows alike) and one fp32 scale per KV head
    for the keys and one for the values."""
    T = num_rows(W, N, G)
    q = _u16(q, (T, heads, head_dim))
    k_cache = _u8(k_cache, (kv_heads, P, head_dim))
    v_cache = _u8(v_cache, (kv_heads, P, head_dim))
    step_k = _u8(step_k, (T, kv_heads, head_dim))
    step_v = _u8(step_v, (T, kv_heads, head_dim))
    k_scale = np.ascontiguousarray(k_scale)
    v_scale = np.ascontiguousarray(v_scale)
    assert k_scale.dtype == np.float32 and k_scale.shape == (kv_heads,)
    assert v_scale.dtype == np.float32 and v_scale.shape == (kv_heads,)
    out = np.empty((T, heads, head_dim), dtype=np.float64)
    rc = _load().la_oracle_step_attention_fp8kv(q.ctypes.data, k_cache.ctypes.data, v_cache.ctypes.data,
                                                step_k.ctypes.data, step_v.ctypes.data, k_scale.ctypes.data,
                                                v_scale.ctypes.data, P, W, N, G, heads, kv_heads, head_dim,
                                                out.ctypes.data)
    if rc != 0:
        raise ValueError("la_oracle_step_attention_fp8kv: bad shape (rc=%d)" % rc)
    return out


def verify(logits, cand_tokens, G, N, V):
    """(accept_len int32 [G], accepted int32 [G, N-1]) from fp32 logits [G, N-1, V]."""
    logits = np.ascontiguousarray(logits)
    cand = np.ascontiguousarray(cand_tokens)
    assert logits.dtype == np.float32 and logits.shape == (G, N - 1, V)
    assert cand.dtype == np.int32 and cand.shape == (G, N - 1)
    accept_len = np.zeros((G,), dtype=np.int32)
    accepted = np.zeros((G, N - 1), dtype=np.int32)
    rc = _load().la_oracle_verify(logits.ctypes.data, cand.ctypes.data, G, N, V,
                                  accept_len.ctypes.data, accepted.ctypes.data)
    if rc != 0:
        raise ValueError("la_oracle_verify: bad shape (rc=%d)" % rc)
    return accept_len, accepted


def verify_step(logits_cur, logits_look, logits_cand, cand_tokens, W, N, G, V):
    """The end of a greedy step: (out_tokens list, best, new_window int32 [W], accept_len int32 [G]).

    logits_cur fp32 [V], logits_look fp32 [W, V], logits_cand fp32 [G, N-1, V], cand_tokens int32
    [G, N-1]; see la_oracle_verify_step in la_oracle.c.
    """
    cur = np.ascontiguousarray(logits_cur)
    look = np.ascontiguousarray(logits_look).reshape(W, V)
    cnd = np.ascontiguousarray(logits_cand).reshape(G, N - 1, V)
    cand = np.ascontiguousarray(cand_tokens).reshape(G, N - 1)
    assert cur.dtype == look.dtype == cnd.dtype == np.float32 and cur.shape == (V,)
    assert cand.dtype == np.int32
    out = np.zeros((N,), dtype=np.int32)
    n_out = np.zeros((1,), dtype=np.int32)
    best = np.zeros((1,), dtype=np.int32)
    window = np.zeros((W,), dtype=np.int32)
    accept_len = np.zeros((G,), dtype=np.int32)
    rc = _load().la_oracle_verify_step(cur.ctypes.data, look.ctypes.data, cnd.ctypes.data, cand.ctypes.data,
                                       W, N, G, V, out.ctypes.data, n_out.ctypes.data, best.ctypes.data,
                                       window.ctypes.data, accept_len.ctypes.data)
    if rc != 0:
        raise ValueError("la_oracle_verify_step: bad shape (rc=%d)" % rc)
    return [int(t) for t in out[:int(n_out[0])]], int(best[0]), window, accept_len


def verify_sample(logits_cur, logits_cand, cand_tokens, u_test, u_final, temperature, N, G, V):
    """Algorithm 4 (sampling verification): the list of 1..N accepted tokens.

    logits_cur fp32 [V], logits_cand fp32 [G, N-1, V], cand_tokens int32 [G, N-1], u_test fp32
    [N-1, G] (draw of the j-th candidate examined at position i), u_final the draw of the last
    token; see la_oracle_verify_sample in la_oracle.c.
    """
    cur = np.ascontiguousarray(logits_cur)
    cnd = np.ascontiguousarray(logits_cand).reshape(G, N - 1, V)
    cand = np.ascontiguousarray(cand_tokens).reshape(G, N - 1)
    ut = np.ascontiguousarray(u_test, dtype=np.float32).reshape(N - 1, G)
    assert cur.dtype == cnd.dtype == np.float32 and cur.shape == (V,) and cand.dtype == np.int32
    out = np.zeros((N,), dtype=np.int32)
    n_out = np.zeros((1,), dtype=np.int32)
    rc = _load().la_oracle_verify_sample(cur.ctypes.data, cnd.ctypes.data, cand.ctypes.data, ut.ctypes.data,
                                         float(u_final), float(temperature), N, G, V, out.ctypes.data,
                                         n_out.ctypes.data)
    if rc != 0:
        raise ValueError("la_oracle_verify_sample: bad arguments (rc=%d)" % rc)
    return [int(t) for t in out[:int(n_out[0])]]


def verify_sample_margin(logits_cur, logits_cand, cand_tokens, u_test, u_final, temperature, N, G, V):
    """Algorithm 4 once more, in NumPy fp64, returning (tokens, margin): margin is the smallest
    distance between a uniform draw and the value it was compared with (an accept test against
    P(s), or a step of the cumulative distribution of the last draw).  An fp32 implementation may
    decide a comparison whose margin is within its rounding (about 1e-6) the other way; callers
    that check one against the oracle demand equality unless the margin is that small."""
    n1 = N - 1
    cur = np.asarray(logits_cur, dtype=np.float64)
    cnd = np.asarray(logits_cand, dtype=np.float64).reshape(G, n1, V)
    cand = np.asarray(cand_tokens).reshape(G, n1)
    ut = np.asarray(u_test, dtype=np.float64).reshape(n1, G)
    margin = [1.0]

    def dist(row):
        z = row / float(temperature)
        e = np.exp(z - z.max())
        return e / e.sum()

    def draw(P, u):
        cdf = np.cumsum(P)
        v = min(int(np.searchsorted(cdf, u, side="right")), V - 1)
        while P[v] == 0.0 and v > 0:
            v -= 1
        margin[0] = min(margin[0], abs(cdf[v] - u))
        if v > 0:
            margin[0] = min(margin[0], abs(cdf[v - 1] - u))
        return v
    alive, out = list(range(G)), []
    for i in range(n1):
        if not alive:
            break
        P = dist(cur if i == 0 else cnd[alive[0], i - 1])
        accepted = False
        for j, g in enumerate(alive):
            s = int(cand[g, i])
            if not 0 <= s < V:
                continue
            margin[0] = min(margin[0], abs(ut[i, j] - P[s]))
            if ut[i, j] < P[s]:
                out.append(s)
                alive = [k for k in alive[j:] if cand[k, i] == s]
                accepted = True
                break
            P[s] = 0.0
            P = P / P.sum()
        if not accepted:
            return out + [draw(P, float(u_final))], margin[0]
    P = dist(cur if not out else cnd[alive[0], len(out) - 1])
    return out + [draw(P, float(u_final))], margin[0]


def greedy_verification(candidates, dist_argmax):
    """The whole of Algorithm 3 (greedy verification of G disjoint n-gram tails), small inputs.

    candidates:  list of G tuples, the N-1 tokens of each n-gram after its first token.
    dist_argmax: dist_argmax[g][i] = greedy token of the i-th of the N distributions the model
                 returned for candidate g (i = 0: output at the last accepted token; i >= 1:
                 output at candidate token i-1).
    Returns the accepted tokens, between 1 and N of them.

    Position by position the surviving candidates are scanned in order; the first whose token
    equals the model's greedy token is accepted and only candidates sharing that token survive;
    if none matches, the model's own token is emitted and the walk stops; when every position
    was accepted the N-th distribution of the first survivor gives a bonus token.
    """
    alive = list(range(len(candidates)))
    assert alive, "Algorithm 3 needs at least one candidate"
    n1 = len(candidates[0])
    out = []
    for i in range(n1):
        target = dist_argmax[alive[0]][i]
        hit = None
        for pos, g in enumerate(alive):
            if candidates[g][i] == target:
                hit = pos
                break
        if hit is None:
            out.append(target)
            return out
        out.append(target)
        alive = [g for g in alive[hit:] if candidates[g][i] == target]
    out.append(dist_argmax[alive[0]][n1])
    return out


def kv_commit(k_cache, v_cache, step_k, step_v, P, W, N, G, best, n_out):
    """Append the accepted tokens of a greedy step to the KV cache, in place (numpy arrays
    [kv_heads, capacity, d] and step tensors [T, kv_heads, d] of any dtype).

    Sec. 3.3 evaluates every step token at the position it would hold in the sequence (the current
    token at 0, candidate token k at 1 + k), so the keys and values the step computed for the
    accepted tokens ARE their cache rows: the current token goes to row P, the i-th accepted
    candidate token (i = 1 .. n_out - 1) of candidate `best` to row P + i.  The last emitted token
    (Algorithm 3's correction or bonus token) has no keys yet.  Returns the new prefix length.
    """
    n1 = N - 1
    assert 1 <= n_out <= N and (n_out == 1 or 0 <= best < G)
    assert P + n_out <= k_cache.shape[1]
    for i in range(n_out):
        row = 0 if i == 0 else 1 + W * n1 + best * n1 + (i - 1)
        for h in range(k_cache.shape[0]):
            k_cache[h, P + i, :] = step_k[row, h, :]
            v_cache[h, P + i, :] = step_v[row, h, :]
    return P + n_out


def gather_pages(pages, block_table, P, page_size):
    """The packed prefix cache [kv_heads, P, d] that a paged cache stands for.

    pages is [n_pages, kv_heads, page_size, d] (any dtype); key t of the sequence lives in page
    block_table[t // page_size] at slot t % page_size.  Plain loops: this is the definition the
    paged entry points are checked against (attention over a paged cache = attention over the
    packed cache it stands for)."""
    n_pages, kv_heads, ps, d = pages.shape
    assert ps == page_size
    out = np.zeros((kv_heads, P, d), dtype=pages.dtype)
    for t in range(P):
        page = int(block_table[t // page_size])
        assert 0 <= page < n_pages
        for h in range(kv_heads):
            out[h, t, :] = pages[page, h, t % page_size, :]
    return out


def kv_commit_paged(k_pages, v_pages, block_table, page_size, step_k, step_v, P, W, N, G, best, n_out):
    """kv_commit for a paged cache, in place: row P + i of the sequence is slot (P + i) % page_size
    of page block_table[(P + i) // page_size].  Returns the new prefix length."""
    n1 = N - 1
    assert 1 <= n_out <= N and (n_out == 1 or 0 <= best < G)
    for i in range(n_out):
        row = 0 if i == 0 else 1 + W * n1 + best * n1 + (i - 1)
        t = P + i
        page = int(block_table[t // page_size])
        for h in range(k_pages.shape[1]):
            k_pages[page, h, t % page_size, :] = step_k[row, h, :]
            v_pages[page, h, t % page_size, :] = step_v[row, h, :]
    return P + n_out


def step_attention_rows(q, k_cache, v_cache, step_k, step_v, row_ids, P, W, N, G, heads, kv_heads, head_dim):
    """Lookahead-step attention over a SUBSET of the step's rows (one device's share under
    lookahead parallelism, Sec. 3.4): fp64 [n, heads, head_dim] from bf16 bit patterns.

    q is [n, heads, d] and step_k / step_v are [n, kv_heads, d]: local row a is row row_ids[a] of
    the full (W, N, G) layout and may see local key b iff full row row_ids[a] may see full row
    row_ids[b] (the mask of Sec. 3.3 restricted to the subset), plus all P prefix keys.  Dense
    numpy with the explicit boolean mask; no blocking."""
    ids = np.asarray(row_ids, dtype=np.int64)
    n = len(ids)
    mask = step_mask(W, N, G)[np.ix_(ids, ids)]
    f = lambda a, shape: bf16_to_f64(_u16(a, shape))
    qf = f(q, (n, heads, head_dim))
    kc, vc = f(k_cache, (kv_heads, P, head_dim)), f(v_cache, (kv_heads, P, head_dim))
    sk, sv = f(step_k, (n, kv_heads, head_dim)), f(step_v, (n, kv_heads, head_dim))
    group = heads // kv_heads
    out = np.zeros((n, heads, head_dim))
    scale = 1.0 / np.sqrt(head_dim)
    for h in range(heads):
        kv = h // group
        keys = np.concatenate([kc[kv], sk[:, kv]], axis=0)          # [P + n, d]
        vals = np.concatenate([vc[kv], sv[:, kv]], axis=0)
        s = qf[:, h] @ keys.T * scale                                # [n, P + n]
        vis = np.concatenate([np.ones((n, P), dtype=bool), mask], axis=1)
        s = np.where(vis, s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        out[:, h] = (p / p.sum(axis=1, keepdims=True)) @ vals
    return out


def bf16_to_f64(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def step_rope(q, step_k, cos, sin, P, W, N, G, interleaved=False):
    """Rotary position embedding of a step's queries and keys at the positions the step's tokens
    hold: row r sits at P + position(r), the relative positions being the digits printed on the
    tokens of Fig. 2(b) (current token 0, lookahead token of level l and column j at 1 + l + j,
    candidate token k at 1 + k; Sec. 3.1 and 3.3).  The rotation itself is the published one: the
    head dimension is cut into d/2 pairs, pair i of a vector at position t turns by the angle whose
    cosine and sine are cos[t, i], sin[t, i]:
        (a, b) -> (a cos - b sin, b cos + a sin).
    Pair i is (x[i], x[i + d/2]), or (x[2i], x[2i + 1]) with `interleaved`.

    q [T, heads, d], step_k [T, kv_heads, d]: float arrays (any float dtype); cos, sin
    [max_pos, d/2].  Returns the rotated (q, step_k) in float64; nothing is rounded here.
    """
    T = num_rows(W, N, G)
    out = []
    for x in (q, step_k):
        x = np.asarray(x, dtype=np.float64)
        assert x.shape[0] == T and x.shape[2] % 2 == 0
        half = x.shape[2] // 2
        y = np.empty_like(x)
        for r in range(T):
            t = P + position(r, W, N, G)
            c, s_ = np.asarray(cos[t], dtype=np.float64), np.asarray(sin[t], dtype=np.float64)
            assert c.shape == (half,)
            for h in range(x.shape[1]):
                for i in range(half):
                    ia, ib = (2 * i, 2 * i + 1) if interleaved else (i, i + half)
                    a, b = x[r, h, ia], x[r, h, ib]
                    y[r, h, ia] = a * c[i] - b * s_[i]
                    y[r, h, ib] = b * c[i] + a * s_[i]
        out.append(y)
    return out[0], out[1]

