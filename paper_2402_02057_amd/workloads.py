"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds shapes, seeds and random draws only: none of the method's arithmetic
(no mask, no attention, no argmax) lives here, so both the HIP path and the CPU oracle can
take their inputs from it without sharing anything else.

The shapes follow the (W, N, G) settings the paper reports as good for each model size
(Table 4: N = 5 and G = W, with W = 15 / 10 / 7) on LLaMA-2-shaped attention layers; the
tensors are N(0,1) draws rounded to bf16, standing in for real activations and KV caches.
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20240205
# tensor ids within a config
_Q, _KC, _VC, _SK, _SV, _LOGITS, _CAND, _PLAN, _PLIST = range(9)


@dataclass(frozen=True)
class StepShape:
    """One lookahead step of one sequence on one attention layer."""
    name: str
    config: int      # index used for seeding
    heads: int
    kv_heads: int
    head_dim: int
    P: int           # prefix (KV cache) length
    W: int           # lookahead window width
    N: int           # n-gram size
    G: int           # number of candidate n-grams verified this step
    V: int           # vocabulary size of the verification logits
    planted: bool    # whether verify logits carry planted accept lengths

    @property
    def T(self):
        return 1 + (self.W + self.G) * (self.N - 1)


TINY = StepShape("tiny", 0, 4, 4, 64, 64, 4, 3, 2, 512, False)
LLAMA2_7B = StepShape("llama2-7b", 1, 32, 32, 128, 1024, 15, 5, 15, 32000, True)
LLAMA2_13B = StepShape("llama2-13b", 2, 40, 40, 128, 2048, 10, 5, 10, 32000, True)
LLAMA2_70B = StepShape("llama2-70b-gqa", 3, 64, 8, 128, 4096, 7, 5, 7, 32000, True)
# the 7B step early in a sequence: the prefix of a short prompt (not one of the benchmark's configs;
# the shape the short-prefix kernel is measured and profiled on)
LLAMA2_7B_P256 = StepShape("llama2-7b-p256", 9, 32, 32, 128, 256, 15, 5, 15, 32000, True)
SHAPES = {s.name: s for s in (TINY, LLAMA2_7B, LLAMA2_13B, LLAMA2_70B, LLAMA2_7B_P256)}

RAGGED_W = (5, 10, 15, 20, 30)
RAGGED_SEQS = 8


def seed_for(config, tensor_id, extra=0):
    return BASE_SEED + 100 * config + tensor_id + 1000003 * extra


def ragged_prefix_lengths():
    """The 8 prefix lengths of the ragged long-context sweep, uniform in [512, 16384]."""
    rng = np.random.default_rng(seed_for(4, _PLIST))
    return [int(x) for x in rng.integers(512, 16384, endpoint=True, size=RAGGED_SEQS)]


def ragged_shape(seq, W):
    """Sequence `seq` (0..7) of the ragged sweep at window width W (N = 5, G = W, GQA 32/8)."""
    P = ragged_prefix_lengths()[seq]
    return StepShape("ragged-s%d-w%d" % (seq, W), 4, 32, 8, 128, P, W, 5, W, 32016, True)


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _normal_bf16(seed, shape):
    rng = np.random.default_rng(seed)
    return f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


def attention_inputs(s: StepShape, extra=0):
    """dict of bf16 bit-pattern (uint16) arrays: q, k_cache, v_cache, step_k, step_v.

    `extra` selects an independent draw of the same shape (distinct layers of one model).
    """
    T, H, KV, d, P = s.T, s.heads, s.kv_heads, s.head_dim, s.P
    return {
        "q": _normal_bf16(seed_for(s.config, _Q, extra), (T, H, d)),
        "k_cache": _normal_bf16(seed_for(s.config, _KC, extra), (KV, P, d)),
        "v_cache": _normal_bf16(seed_for(s.config, _VC, extra), (KV, P, d)),
        "step_k": _normal_bf16(seed_for(s.config, _SK, extra), (T, KV, d)),
        "step_v": _normal_bf16(seed_for(s.config, _SV, extra), (T, KV, d)),
    }


PLANT_VALUE = np.float32(12.0)   # far above the largest of 32000 N(0,1) draws (about 4.2)


def verify_inputs(s: StepShape, extra=0):
    """(logits fp32 [G, N-1, V], cand_tokens int32 [G, N-1], planted accept lengths or None).

    With `planted`, candidate g is given the accept length (g + shift) mod N: its first rows
    peak at the candidate token, the next row peaks elsewhere, and on odd g the later rows
    peak at the candidate token again, so that counting matches instead of the leading run
    gives a different answer.
    """
    G, n1, V = s.G, s.N - 1, s.V
    rng = np.random.default_rng(seed_for(s.config, _LOGITS, extra))
    logits = rng.standard_normal(size=(G, n1, V), dtype=np.float32)
    rng = np.random.default_rng(seed_for(s.config, _CAND, extra))
    cand = rng.integers(0, V, size=(G, n1)).astype(np.int32)
    if not s.planted:
        return logits, cand, None
    rng = np.random.default_rng(seed_for(s.config, _PLAN, extra))
    shift = int(rng.integers(0, s.N))
    lens = np.zeros((G,), dtype=np.int32)
    for g in range(G):
        L = (g + shift) % s.N
        lens[g] = L
        for k in range(n1):
            if k < L or (k > L and g % 2 == 1):
                logits[g, k, cand[g, k]] = PLANT_VALUE
            elif k == L:
                other = (int(cand[g, k]) + 1 + int(rng.integers(0, V - 1))) % V
                logits[g, k, other] = PLANT_VALUE
    return logits, cand, lens


def verify_step_inputs(s: StepShape, extra=0):
    """Inputs of the end-of-step reduction: (logits_cur fp32 [V], logits_look fp32 [W, V],
    logits_cand fp32 [G, N-1, V], cand_tokens int32 [G, N-1], planted accept lengths or None).

    Row (g, k) of logits_cand is the model output at candidate g's token k: it judges slot k + 1
    (slot 0 is judged by logits_cur, the same for every candidate) and row (g, N-2) is the bonus
    row.  With `planted`, candidate g gets the accept length (g + shift) mod N: its slot-0 token is
    the peak of logits_cur iff that length is positive, the rows judging its next slots peak at its
    tokens, the row judging the first rejected slot peaks elsewhere, and on odd g the later rows
    peak at the candidate's tokens again.
    """
    W, G, n1, V = s.W, s.G, s.N - 1, s.V
    rng = np.random.default_rng(seed_for(s.config, _LOGITS, extra + 7))
    cur = rng.standard_normal(size=(V,), dtype=np.float32)
    look = rng.standard_normal(size=(W, V), dtype=np.float32)
    cnd = rng.standard_normal(size=(G, n1, V), dtype=np.float32)
    rng = np.random.default_rng(seed_for(s.config, _CAND, extra + 7))
    cand = rng.integers(0, V, size=(G, n1)).astype(np.int32)
    if not s.planted:
        return cur, look, cnd, cand, None
    rng = np.random.default_rng(seed_for(s.config, _PLAN, extra + 7))
    shift = int(rng.integers(0, s.N))
    a0 = int(rng.integers(0, V))
    cur[a0] = PLANT_VALUE
    for j in range(W):
        look[j, int(rng.integers(0, V))] = PLANT_VALUE
    lens = np.zeros((G,), dtype=np.int32)
    for g in range(G):
        L = (g + shift) % s.N
        lens[g] = L
        if L >= 1:
            cand[g, 0] = a0
        elif cand[g, 0] == a0:
            cand[g, 0] = (a0 + 1) % V
        for slot in range(1, n1):            # judged by row (g, slot - 1)
            if slot < L or (slot > L and g % 2 == 1):
                cnd[g, slot - 1, cand[g, slot]] = PLANT_VALUE
            elif slot == L:
                other = (int(cand[g, slot]) + 1 + int(rng.integers(0, V - 1))) % V
                cnd[g, slot - 1, other] = PLANT_VALUE
        cnd[g, n1 - 1, int(rng.integers(0, V))] = PLANT_VALUE   # bonus row
    return cur, look, cnd, cand, lens



def verify_sample_inputs(s: StepShape, extra=0, temperature=1.0):
    """Inputs of sampling verification: (logits_cur fp32 [V], logits_cand fp32 [G, N-1, V],
    cand_tokens int32 [G, N-1], u_test fp32 [N-1, G], u_final fp32 [1]).

    Logits are N(0,1) draws with a few tokens per row raised so that a handful of tokens carry
    most of the probability (as a language model's rows do); candidate g follows the peaked
    tokens for (g + shift) mod N positions, so that accept tests meet both large and small
    probabilities.  Rows of candidates that share a token prefix are made identical, as a real
    model's would be.  Draws are uniform in [0, 1).
    """
    G, n1, V = s.G, s.N - 1, s.V
    rng = np.random.default_rng(seed_for(s.config, _LOGITS, extra + 13))
    top = min(V, 4)

    def peaked_row():
        row = rng.standard_normal(size=(V,), dtype=np.float32)
        idx = rng.choice(V, size=top, replace=False)
        row[idx] += np.float32(9.0) + rng.standard_normal(top).astype(np.float32)
        return row, idx
    cur, cur_top = peaked_row()
    cnd = np.zeros((G, n1, V), dtype=np.float32)
    cand = np.zeros((G, n1), dtype=np.int32)
    shift = int(rng.integers(0, s.N))
    rows_by_prefix = {}
    for g in range(G):
        follow = (g + shift) % s.N
        prefix, tops = (), cur_top
        for k in range(n1):
            tokn = int(tops[int(rng.integers(0, len(tops)))]) if k < follow else int(rng.integers(0, V))
            cand[g, k] = tokn
            prefix = prefix + (tokn,)
            if prefix not in rows_by_prefix:
                rows_by_prefix[prefix] = peaked_row()
            cnd[g, k], tops = rows_by_prefix[prefix]
    u_test = rng.random(size=(n1, G), dtype=np.float32)
    u_final = rng.random(size=(1,), dtype=np.float32)
    return cur, cnd, cand, u_test, u_final


# ---- a toy language model for driving the decoding loop end to end --------------------------

TOY_VOCAB = 32       # token 0 is the begin-of-sequence token and is never generated
TOY_HEAD_DIM = 64
TOY_SENTINEL = 32    # the coordinate of the key that only the begin-of-sequence token carries


def toy_lm_tables(seed=0):
    """Seeded tables of a one-layer attention-only toy language model (inputs, like weights).

    The model looks for one particular other token in what a position may see: `wanted[c]` is the
    token that position holding token c looks for, `next_token[2 c + found]` the greedy
    continuation, `logits[2 c + found]` an fp32 row of N(0,1) noise with a peak of 12 at that
    continuation.  `q`, `k`, `v` are the attention tables (float32 holding bf16-exact values,
    [vocab, 64]) with which one softmax-attention head computes `found`: a query matches the
    wanted token's key with score 32 and the begin-of-sequence key with score 16 (everything else
    0), values carry 1 in coordinate 0 for ordinary tokens and in coordinate 1 for the
    begin-of-sequence token, so that found <=> out[0] > 0.5 with a wide margin.
    """
    rng = np.random.default_rng(BASE_SEED + 9000 + seed)
    V, d = TOY_VOCAB, TOY_HEAD_DIM
    wanted = rng.integers(1, V, size=V).astype(np.int32)
    next_token = rng.integers(1, V, size=2 * V).astype(np.int32)
    logits = rng.standard_normal(size=(2 * V, V)).astype(np.float32)
    logits[np.arange(2 * V), next_token] = PLANT_VALUE
    q = np.zeros((V, d), dtype=np.float32)
    k = np.zeros((V, d), dtype=np.float32)
    v = np.zeros((V, d), dtype=np.float32)
    for c in range(V):
        q[c, wanted[c]] = 16.0
        q[c, TOY_SENTINEL] = 8.0
        if c == 0:
            k[c, TOY_SENTINEL] = 16.0
            v[c, 1] = 1.0
        else:
            k[c, c] = 16.0
            v[c, 0] = 1.0
    return {"wanted": wanted, "next_token": next_token, "logits": logits, "q": q, "k": k, "v": v}


def window_random_token(seed, step, column):
    """The "random" tokens Algorithm 2 fills the window with, as a counter-based generator so
    that every implementation of the loop draws the same ones: a token in [1, TOY_VOCAB)."""
    h = (seed * 0x9E3779B97F4A7C15 + step * 0xBF58476D1CE4E5B9 + column * 0x94D049BB133111EB) % (1 << 64)
    h ^= h >> 31
    h = (h * 0xD6E8FEB86659FD93) % (1 << 64)
    h ^= h >> 29
    return 1 + h % (TOY_VOCAB - 1)


def uniform_draw(seed, step, index):
    """The uniform draws of sampling verification inside a decoding loop, as a counter-based
    generator (every implementation of the loop makes the same ones): a float32 in [0, 1)."""
    h = (seed * 0xD1342543DE82EF95 + step * 0x9E3779B97F4A7C15 + index * 0xC2B2AE3D27D4EB4F + 0x165667B19E3779F9) % (1 << 64)
    h ^= h >> 32
    h = (h * 0xD6E8FEB86659FD93) % (1 << 64)
    h ^= h >> 32
    h = (h * 0xD6E8FEB86659FD93) % (1 << 64)
    h ^= h >> 32
    return np.float32((h >> 40) / float(1 << 24))


def rope_tables(max_pos, head_dim, base=10000.0):
    """cos, sin fp32 [max_pos, head_dim / 2] of rotary position embedding: entry [t, i] belongs to
    the angle t * base^(-2 i / head_dim).  Inputs like weights: a model brings its own tables."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    angle = np.arange(max_pos, dtype=np.float64)[:, None] * base ** (-2.0 * i / head_dim)[None, :]
    return np.cos(angle).astype(np.float32), np.sin(angle).astype(np.float32)



FP8_MAX = 448.0   # largest finite value of the 8-bit float (E4M3, finite-only) a quantised cache stores


def quantize_fp8(x, scale):
    """8-bit float codes (uint8) of x / scale, by the library's round-to-nearest cast (torch, CPU).

    Input preparation only: what a code stands for is defined by the consumer of the bytes."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x / scale, dtype=np.float32))
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def attention_inputs_fp8(s: StepShape, extra=0):
    """The draws of attention_inputs with keys and values (cache and step rows) quantised to 8-bit
    floats: per KV head one scale for the keys and one for the values, the head's largest magnitude
    over FP8_MAX, as an offline calibration of a quantised cache would choose them.

    dict: q (bf16 bits), k_cache / v_cache / step_k / step_v (uint8 codes), k_scale / v_scale (fp32 [kv_heads]).
    """
    x = {k: bf16_bits_to_f32(v) for k, v in attention_inputs(s, extra).items()}
    k_amax = np.maximum(np.abs(x["k_cache"]).max(axis=(1, 2), initial=0.0), np.abs(x["step_k"]).max(axis=(0, 2)))
    v_amax = np.maximum(np.abs(x["v_cache"]).max(axis=(1, 2), initial=0.0), np.abs(x["step_v"]).max(axis=(0, 2)))
    k_scale = (k_amax / FP8_MAX).astype(np.float32)
    v_scale = (v_amax / FP8_MAX).astype(np.float32)
    return {
        "q": f32_to_bf16_bits(x["q"]),
        "k_cache": quantize_fp8(x["k_cache"], k_scale[:, None, None]),
        "v_cache": quantize_fp8(x["v_cache"], v_scale[:, None, None]),
        "step_k": quantize_fp8(x["step_k"], k_scale[None, :, None]),
        "step_v": quantize_fp8(x["step_v"], v_scale[None, :, None]),
        "k_scale": k_scale,
        "v_scale": v_scale,
    }
