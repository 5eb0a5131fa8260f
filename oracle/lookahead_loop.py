"""The decoding loop of Lookahead Decoding (Algorithm 2) on the CPU, with a toy model.

THIS FILE IS TEST INFRASTRUCTURE, like the rest of oracle/: a plain statement of the loop written
from the paper, used to pin the method (its output must equal plain greedy decoding) and to check
the product's host loop step by step.  It shares no code with the product path; both take the toy
model's tables and the window's random tokens from the seeded generators in
paper_2402_02057_amd/workloads.py.

State, in the layout of one step (Sec. 3.1, with the window kept as a full W x (N-1) rectangle
behind the current token): `window[l][j]`, l = 0 (oldest) .. N-2, is the token at relative
position 1 + l + j produced by an earlier Jacobi iteration; `pool[t]` lists, oldest first, the
(N-1)-token tails of the n-grams collected so far whose first token is t (Sec. 3.2).

One step (Algorithm 2's loop body for an index i that has no token yet):
  lookahead branch     new[j] = greedy token of the model at the newest window token of column j,
                       which sees the prefix, the current token, level-0 columns <= j and its own
                       column (the mask of Sec. 3.3);
  verification branch  up to G pool n-grams that start with the current token (the most recent
                       ones) are verified greedily (Algorithm 3);
  pool update          column j yields the n-gram (window[0][j], ..., window[N-2][j], new[j]);
  window update        the oldest level is dropped and `new` appended; every further token accepted
                       in the same step stands for a loop index that is skipped with a window
                       level set "randomly" (the counter-based generator).
"""
import numpy as np

from paper_2402_02057_amd import workloads as wl

from . import la_oracle as orc


class ToyModel:
    """Greedy next-token logits as a function of the token at a position and the SET of tokens
    that position may see (itself included): row 2 c + found of the seeded table."""

    def __init__(self, seed=0):
        t = wl.toy_lm_tables(seed)
        self.wanted, self.table, self.vocab = t["wanted"], t["logits"], wl.TOY_VOCAB

    def logits(self, token, visible):
        found = int(self.wanted[token]) in visible
        return self.table[2 * int(token) + int(found)]


def greedy_decode(model, prompt, n_tokens):
    """Plain autoregressive greedy decoding: the sequence every lossless method must reproduce."""
    seq = list(prompt)
    out = []
    for _ in range(n_tokens):
        out.append(int(np.argmax(model.logits(seq[-1], set(seq)))))
        seq.append(out[-1])
    return out


def lookahead_decode(model, prompt, W, N, G, n_tokens, seed=0, prompt_as_reference=False, temperature=None):
    """(tokens, steps, trace): Algorithm 2 with greedy verification until n_tokens are out.

    trace is one record per step: the step's tokens in row order, the accepted tokens, the index
    of the winning candidate and the new window level, for step-by-step comparison.
    With a temperature the verification branch samples (Algorithm 4) while the lookahead branch
    stays greedy, as Sec. 3.2 prescribes: how the candidates were made does not matter to the
    output distribution.  The uniform draws come from the counter-based generator, indexed by the
    step and by (position, order of examination); `best` is then the first candidate that starts
    with the accepted tokens (-1 if none was accepted).
    With prompt_as_reference the pool starts with every n-gram of the prompt (the augmentation of
    the ablation study, Sec. 5.4): candidates may come from anywhere, the output cannot change.
    """
    n1 = N - 1
    V = model.vocab
    seq = list(prompt)                     # x^0 followed by the accepted tokens; seq[-1] is the current token
    window = [[wl.window_random_token(seed, l - n1, j) for j in range(W)] for l in range(n1)]
    pool = {}
    if prompt_as_reference:
        for i in range(len(prompt) - N + 1):
            bucket = pool.setdefault(int(prompt[i]), [])
            tail = tuple(int(t) for t in prompt[i + 1:i + N])
            if tail in bucket:
                bucket.remove(tail)
            bucket.append(tail)
    out, trace, steps = [], [], 0
    index = 0                              # Algorithm 2's loop index i - 1 (tokens decided so far, skips included)
    while len(out) < n_tokens:
        steps += 1
        cur = seq[-1]
        prefix_set = set(seq)              # prefix and current token: visible to every row
        tails = pool.get(cur, [])[-G:] if G > 0 else []   # at most G, the most recent
        # ---- lookahead branch: model output at the newest token of every column
        look = np.zeros((W, V), dtype=np.float32)
        for j in range(W):
            visible = prefix_set | set(window[0][:j + 1]) | {window[l][j] for l in range(n1)}
            look[j] = model.logits(window[n1 - 1][j], visible)
        # ---- verification branch: the N distributions of every candidate
        logits_cur = model.logits(cur, prefix_set)
        cand = np.array(tails, dtype=np.int32).reshape(len(tails), n1)
        cnd = np.zeros((len(tails), n1, V), dtype=np.float32)
        for g, tail in enumerate(tails):
            for k in range(n1):
                cnd[g, k] = model.logits(tail[k], prefix_set | set(tail[:k + 1]))
        if temperature is None:
            accepted, best, new, _ = orc.verify_step(logits_cur, look, cnd, cand, W, N, len(tails), V)
        else:
            g = len(tails)
            _, _, new, _ = orc.verify_step(logits_cur, look, cnd[:0], cand[:0], W, N, 0, V)   # window: greedy
            u_test = np.array([wl.uniform_draw(seed, steps, i * g + j) for i in range(n1) for j in range(g)],
                              dtype=np.float32).reshape(n1, g)
            u_final = wl.uniform_draw(seed, steps, 1 << 20)
            accepted = orc.verify_sample(logits_cur, cnd, cand, u_test, u_final, temperature, N, g, V)
            k = len(accepted) - 1
            best = next((i for i, tail in enumerate(tails) if list(tail[:k]) == accepted[:k]), -1) if k else -1
        step_tokens = [cur] + [t for level in window for t in level] + [t for tail in tails for t in tail]
        trace.append({"tokens": step_tokens, "accepted": list(accepted), "best": best, "window": new.tolist()})
        # ---- pool update: one n-gram per column
        for j in range(W):
            gram = tuple(window[l][j] for l in range(n1)) + (int(new[j]),)
            bucket = pool.setdefault(gram[0], [])
            if gram[1:] in bucket:
                bucket.remove(gram[1:])    # keep one copy, as the most recent
            bucket.append(gram[1:])
        # ---- window update
        window = window[1:] + [[int(t) for t in new]]
        for extra in range(1, len(accepted)):   # skipped loop indices: a random level each
            window = window[1:] + [[wl.window_random_token(seed, index + extra, j) for j in range(W)]]
        index += len(accepted)
        out.extend(accepted)
        seq.extend(accepted)
    return out[:n_tokens], steps, trace
