"""Host side of a Lookahead Decoding run (Algorithm 2 of arXiv 2402.02057) driving the HIP kernels.

Everything per-token runs on the device: the model's forward pass over the step's
T = 1 + (W + G)(N - 1) tokens (its attention is `la_step_attention`) and the end of the step
(`la_verify_step`: Algorithm 3 and the window's new tokens; `la_kv_commit`: the accepted tokens'
keys and values go to the KV cache).  The host keeps what the paper keeps
on the host: the 2D window of Jacobi iterates (Sec. 3.1) and the n-gram pool (Sec. 3.2).

`model` is any object with
    vocab                               vocabulary size
    forward_step(tokens, W, N, G)       fp32 device tensor [T, vocab]: the model output at every
                                        row of the step (row order of include/la.h), attending to
                                        its own KV cache as the prefix
    commit(best, n_out)                 append the accepted tokens of the step just run to the KV
                                        cache from the device-side result of la_verify_step
                                        (int32 tensors; `la_kv_commit`), without waiting for it
    advance(n)                          the host's count of what commit appended
    append(tokens)                      prefill: append tokens to the KV cache
`BatchedLookaheadDecoder` runs several sequences side by side through the batched entry points
(`ToyBatchLM` is its model).  `ToyAttentionLM` below is such a model: one attention head over seeded tables, enough to run the
loop end to end on the GPU and check it against plain greedy decoding.

    python -m paper_2402_02057_amd.lookahead      # demo: tokens per step and time per step
"""
import time

import torch

from . import binding, workloads as wl


def lp_share(W, N, G, parts, part):
    """Rows of the (W, N, G) step that device `part` of `parts` holds under lookahead parallelism
    (Sec. 3.4): the current token and the oldest window level on every device (computed
    redundantly, which spares all communication inside the forward pass), the columns of the newer
    levels and the candidates dealt round-robin.  For `la_step_attention_rows`."""
    n1 = N - 1
    rows = [0] + [1 + j for j in range(W)]
    for level in range(1, n1):
        rows += [1 + level * W + j for j in range(part, W, parts)]
    for g in range(part, G, parts):
        rows += [1 + W * n1 + g * n1 + k for k in range(n1)]
    return rows


class NgramPool:
    """n-grams collected from the Jacobi trajectory, by first token; most recent last."""

    def __init__(self):
        self._tails = {}

    def add(self, gram):
        bucket = self._tails.setdefault(gram[0], [])
        tail = tuple(gram[1:])
        if tail in bucket:
            bucket.remove(tail)
        bucket.append(tail)

    def lookup(self, first_token, limit):
        """At most `limit` tails of n-grams starting with first_token, the most recent ones."""
        return self._tails.get(first_token, [])[-limit:] if limit > 0 else []


class _Sequence:
    """What the host keeps per sequence: the current token, the 2D window of Jacobi iterates
    (Sec. 3.1), the n-gram pool (Sec. 3.2) and Algorithm 2's loop index."""

    def __init__(self, prompt, W, N, G, seed, random_token, prompt_as_reference):
        if N < 2 or W < 0 or G < 0 or not prompt:
            raise ValueError("need N >= 2, W >= 0, G >= 0 and a non-empty prompt")
        self.W, self.N, self.G, self.seed, self.random_token = W, N, G, seed, random_token
        n1 = N - 1
        self.window = [[random_token(seed, l - n1, j) for j in range(W)] for l in range(n1)]
        self.pool = NgramPool()
        if prompt_as_reference:     # the prompt's own n-grams as first candidates (ablation study, Sec. 5.4)
            for i in range(len(prompt) - N + 1):
                self.pool.add(tuple(int(t) for t in prompt[i:i + N]))
        self.current = int(prompt[-1])
        self.index = 0          # Algorithm 2's loop index: tokens decided so far
        self.steps = 0

    def candidates(self):
        return self.pool.lookup(self.current, self.G)

    def step_tokens(self, tails):
        return [self.current] + [t for level in self.window for t in level] + [t for tail in tails for t in tail]

    def absorb(self, accepted, new):
        """The step's outcome: the window's columns become n-grams of the pool, the window moves on."""
        W, n1, n = self.W, self.N - 1, len(accepted)
        for j in range(W):
            self.pool.add(tuple(self.window[l][j] for l in range(n1)) + (new[j],))
        self.window = self.window[1:] + [new]
        for extra in range(1, n):   # skipped loop indices: a "random" level each (Algorithm 2)
            self.window = self.window[1:] + [[self.random_token(self.seed, self.index + extra, j)
                                              for j in range(W)]]
        self.index += n
        self.current = accepted[-1]
        self.steps += 1


class LookaheadDecoder:
    """Greedy Lookahead Decoding.  `prompt` must hold at least one token; its last token is the
    first current token, the others go to the model's KV cache.  With prompt_as_reference the
    pool starts with the prompt's own n-grams.  With a temperature the candidates are verified by
    sampling (Algorithm 4, `la_verify_sample`) while the lookahead branch stays greedy (Sec. 3.2);
    `uniform(seed, step, index)` supplies the draws."""

    def __init__(self, model, prompt, W, N, G, seed=0, random_token=wl.window_random_token,
                 prompt_as_reference=False, temperature=None, uniform=wl.uniform_draw):
        self._seq = _Sequence(prompt, W, N, G, seed, random_token, prompt_as_reference)
        self.model, self.W, self.N, self.G, self.seed = model, W, N, G, seed
        self.temperature, self.uniform = temperature, uniform
        model.append([int(t) for t in prompt[:-1]])
        dev = "cuda"
        self._out = torch.empty((N,), dtype=torch.int32, device=dev)
        self._n_out = torch.empty((1,), dtype=torch.int32, device=dev)
        self._best = torch.empty((1,), dtype=torch.int32, device=dev)
        self._new = torch.empty((W,), dtype=torch.int32, device=dev)

    window = property(lambda self: self._seq.window)
    pool = property(lambda self: self._seq.pool)
    current = property(lambda self: self._seq.current)
    index = property(lambda self: self._seq.index)
    steps = property(lambda self: self._seq.steps)

    def step(self):
        """One decoding step; returns (accepted tokens, step tokens, winning candidate, new level)."""
        W, N, n1 = self.W, self.N, self.N - 1
        tails = self._seq.candidates()
        g = len(tails)
        tokens = self._seq.step_tokens(tails)
        logits = self.model.forward_step(tokens, W, N, g)
        V = self.model.vocab
        look = logits[1 + (n1 - 1) * W:1 + n1 * W] if W else None        # newest level of the window
        cand_logits = logits[1 + W * n1:].view(g, n1, V) if g else None
        cand = torch.tensor(tails, dtype=torch.int32, device=logits.device).view(g, n1) if g else None
        if self.temperature is None:
            binding.la_verify_step(logits[0], look, cand_logits, cand, W, N, g, V, self._out, self._n_out,
                                   self._best, self._new if W else None, None)
            self.model.commit(self._best, self._n_out)                    # queued behind the verification
            n = int(self._n_out.item())                                   # (synchronises)
            accepted = self._out[:n].tolist()
        else:
            # the window's new level: greedy tokens of the lookahead rows (no candidates in this call)
            binding.la_verify_step(logits[0], look, None, None, W, N, 0, V, self._out, self._n_out, self._best,
                                   self._new if W else None, None)
            step = self.steps + 1
            u_test = torch.tensor([float(self.uniform(self.seed, step, i * g + j)) for i in range(n1) for j in range(g)],
                                  dtype=torch.float32).view(n1, g).to(logits.device) if g else None
            u_final = torch.tensor([float(self.uniform(self.seed, step, 1 << 20))], dtype=torch.float32).to(logits.device)
            binding.la_verify_sample(logits[0], cand_logits, cand, u_test, u_final, self.temperature, N, g, V,
                                     self._out, self._n_out)
            n = int(self._n_out.item())
            accepted = self._out[:n].tolist()
            # any candidate that starts with the accepted tokens has their keys and values
            k = n - 1
            best = next((i for i, tail in enumerate(tails) if list(tail[:k]) == accepted[:k]), -1) if k else -1
            self._best.fill_(best)
            self.model.commit(self._best, self._n_out)
        new = self._new.tolist() if W else []
        self._seq.absorb(accepted, new)
        self.model.advance(n)       # the cache now holds cur and accepted[:-1]
        return accepted, tokens, int(self._best.item()), new

    def generate(self, n_tokens):
        out = []
        while len(out) < n_tokens:
            out.extend(self.step()[0])
        return out[:n_tokens]


class BatchedLookaheadDecoder:
    """Greedy Lookahead Decoding of several sequences side by side, one launch per operation and
    step: `la_step_attention_batch_paged` inside the model's forward pass, `la_verify_step_batch`,
    `la_kv_commit_batch`.  Those calls want one G for all sequences, and the pools answer with
    different numbers of candidates: a sequence with fewer gets copies of its first one (a copy
    never wins, the lowest index does), a sequence with none gets placeholders whose acceptance the
    host ignores - so every sequence moves exactly as it would alone.

    `model` as for LookaheadDecoder, with a leading sequence argument: append(i, tokens),
    forward_step(token lists, W, N, G) -> list of logits, commit(best tensors, n_out tensors),
    advance(i, n)."""

    def __init__(self, model, prompts, W, N, G, seeds=None, random_token=wl.window_random_token,
                 prompt_as_reference=False):
        n = len(prompts)
        seeds = list(range(n)) if seeds is None else list(seeds)
        self.model, self.W, self.N, self.G = model, W, N, G
        self.seqs = [_Sequence(p, W, N, G, sd, random_token, prompt_as_reference) for p, sd in zip(prompts, seeds)]
        for i, p in enumerate(prompts):
            model.append(i, [int(t) for t in p[:-1]])
        dev, i32 = "cuda", torch.int32
        self._out = torch.empty((n, N), dtype=i32, device=dev)
        self._n_out = torch.empty((n, 1), dtype=i32, device=dev)
        self._best = torch.empty((n, 1), dtype=i32, device=dev)
        self._new = torch.empty((n, W), dtype=i32, device=dev)

    def step(self):
        """One step of every sequence; returns per sequence (accepted tokens, step tokens without the
        padding, winning candidate, new level)."""
        W, N, n1, V = self.W, self.N, self.N - 1, self.model.vocab
        tails = [s.candidates() for s in self.seqs]
        g_step = max(len(t) for t in tails)
        placeholder = (0,) * n1
        padded = [t + [t[0] if t else placeholder] * (g_step - len(t)) for t in tails]
        tokens = [s.step_tokens(p) for s, p in zip(self.seqs, padded)]
        logits = self.model.forward_step(tokens, W, N, g_step)
        descs = []
        for i, lg in enumerate(logits):
            descs.append(dict(
                logits_cur=lg[0], logits_look=lg[1 + (n1 - 1) * W:1 + n1 * W] if W else None,
                logits_cand=lg[1 + W * n1:].view(g_step, n1, V) if g_step else None,
                cand_tokens=torch.tensor(padded[i], dtype=torch.int32, device=lg.device).view(g_step, n1) if g_step else None,
                out_tokens=self._out[i], n_out=self._n_out[i], best=self._best[i],
                new_window=self._new[i] if W else None))
        binding.la_verify_step_batch(descs, W, N, g_step, V)
        self.model.commit([self._best[i] for i in range(len(self.seqs))],
                          [self._n_out[i] for i in range(len(self.seqs))])   # queued behind the verification
        out, n_out = self._out.tolist(), self._n_out.view(-1).tolist()           # (synchronises)
        best, new = self._best.view(-1).tolist(), self._new.tolist()
        results = []
        for i, s in enumerate(self.seqs):
            real = len(tails[i])
            n = n_out[i] if real else 1          # a placeholder's acceptance does not count
            accepted = out[i][:n]
            s.absorb(accepted, new[i] if W else [])
            self.model.advance(i, n)            # (rows the device appended beyond that are never read)
            results.append((accepted, tokens[i][:1 + (W + real) * n1], best[i] if real else -1, new[i] if W else []))
        return results

    def generate(self, n_tokens):
        outs = [[] for _ in self.seqs]
        while min(len(o) for o in outs) < n_tokens:
            for o, r in zip(outs, self.step()):
                o.extend(r[0])
        return [o[:n_tokens] for o in outs]


class ToyAttentionLM:
    """One attention head over the seeded tables of workloads.toy_lm_tables: a position's output
    depends on its token and on whether the token it looks for is among the positions it may see,
    which the head finds out with `la_step_attention` (head_dim 64).  A sequence must start with
    token 0, the begin-of-sequence token the head falls back on.  The KV cache is kept in place
    (`la_step_attention_cap` / `la_kv_commit`) or, with page_size, in pages named by a shuffled
    block table (`la_step_attention_paged` / `la_kv_commit_paged`)."""

    def __init__(self, seed=0, max_len=8192, device="cuda", page_size=None):
        t = wl.toy_lm_tables(seed)
        self.vocab = wl.TOY_VOCAB
        d = wl.TOY_HEAD_DIM

        def table(x):
            return torch.from_numpy(x).to(device).to(torch.bfloat16).view(self.vocab, 1, d)
        self._q, self._k, self._v = table(t["q"]), table(t["k"]), table(t["v"])
        self._logits = torch.from_numpy(t["logits"]).to(device)
        self.page_size = page_size
        if page_size:
            n_pages = (max_len + page_size - 1) // page_size
            self.capacity = n_pages * page_size
            self._k_cache = torch.zeros((n_pages, 1, page_size, d), dtype=torch.bfloat16, device=device)
            self._v_cache = torch.zeros_like(self._k_cache)
            gen = torch.Generator().manual_seed(seed)
            self.block_table = torch.randperm(n_pages, generator=gen).to(torch.int32).to(device)
        else:
            self.capacity = max_len
            self._k_cache = torch.zeros((1, max_len, d), dtype=torch.bfloat16, device=device)
            self._v_cache = torch.zeros((1, max_len, d), dtype=torch.bfloat16, device=device)
        self.length = 0
        self.device = device

    def append(self, tokens):
        if not tokens:
            return
        idx = torch.tensor(tokens, dtype=torch.long, device=self.device)
        n = len(tokens)
        if self.length + n > self.capacity:
            raise ValueError("KV cache full")
        if self.page_size:
            pos = torch.arange(self.length, self.length + n, device=self.device)
            page = self.block_table[pos // self.page_size].long()
            self._k_cache[page, 0, pos % self.page_size] = self._k[idx, 0]
            self._v_cache[page, 0, pos % self.page_size] = self._v[idx, 0]
        else:
            self._k_cache[0, self.length:self.length + n] = self._k[idx, 0]
            self._v_cache[0, self.length:self.length + n] = self._v[idx, 0]
        self.length += n

    def forward_step(self, tokens, W, N, G):
        idx = torch.tensor(tokens, dtype=torch.long, device=self.device)
        T, P, d = len(tokens), self.length, wl.TOY_HEAD_DIM
        assert T == 1 + (W + G) * (N - 1)
        if P + N > self.capacity:
            raise ValueError("KV cache full")
        out = torch.empty((T, 1, d), dtype=torch.bfloat16, device=self.device)
        self._step = (self._k[idx].contiguous(), self._v[idx].contiguous(), W, N, G)
        if self.page_size:
            binding.la_step_attention_paged(self._q[idx].contiguous(), self._k_cache, self._v_cache,
                                            self.block_table, self._step[0], self._step[1], P, W, N, G, 1, 1, d, out)
        else:
            binding.la_step_attention_cap(self._q[idx].contiguous(), self._k_cache, self._v_cache, self._step[0],
                                          self._step[1], P, W, N, G, 1, 1, d, out)
        found = (out[:, 0, 0].float() > 0.5).long()
        return self._logits[idx * 2 + found].contiguous()

    def commit(self, best, n_out):
        step_k, step_v, W, N, G = self._step
        if self.page_size:
            binding.la_kv_commit_paged(self._k_cache, self._v_cache, self.block_table, step_k, step_v, self.length,
                                       W, N, G, 1, wl.TOY_HEAD_DIM, best, n_out)
        else:
            binding.la_kv_commit(self._k_cache, self._v_cache, step_k, step_v, self.length, W, N, G, 1,
                                 wl.TOY_HEAD_DIM, best, n_out)

    def advance(self, n):
        self.length += n


class ToyBatchLM:
    """ToyAttentionLM for several sequences side by side, as a serving system holds them: one pool
    of KV pages shared by all, a block table per sequence (shuffled, so that no two neighbours in a
    sequence are neighbours in memory), and one launch per operation for the whole batch."""

    def __init__(self, seed, n_seqs, max_len=4096, page_size=64, device="cuda"):
        t = wl.toy_lm_tables(seed)
        self.vocab = wl.TOY_VOCAB
        d = wl.TOY_HEAD_DIM

        def table(x):
            return torch.from_numpy(x).to(device).to(torch.bfloat16).view(self.vocab, 1, d)
        self._q, self._k, self._v = table(t["q"]), table(t["k"]), table(t["v"])
        self._logits = torch.from_numpy(t["logits"]).to(device)
        self.page_size, self.device = page_size, device
        per_seq = (max_len + page_size - 1) // page_size
        self.capacity = per_seq * page_size
        n_pages = per_seq * n_seqs
        self._k_pages = torch.zeros((n_pages, 1, page_size, d), dtype=torch.bfloat16, device=device)
        self._v_pages = torch.zeros_like(self._k_pages)
        perm = torch.randperm(n_pages, generator=torch.Generator().manual_seed(seed)).to(torch.int32)
        self.block_tables = [perm[i * per_seq:(i + 1) * per_seq].contiguous().to(device) for i in range(n_seqs)]
        self.lengths = [0] * n_seqs

    def append(self, i, tokens):
        if not tokens:
            return
        n = len(tokens)
        if self.lengths[i] + n > self.capacity:
            raise ValueError("KV cache full")
        idx = torch.tensor(tokens, dtype=torch.long, device=self.device)
        pos = torch.arange(self.lengths[i], self.lengths[i] + n, device=self.device)
        page = self.block_tables[i][pos // self.page_size].long()
        self._k_pages[page, 0, pos % self.page_size] = self._k[idx, 0]
        self._v_pages[page, 0, pos % self.page_size] = self._v[idx, 0]
        self.lengths[i] += n

    def forward_step(self, tokens, W, N, G):
        d = wl.TOY_HEAD_DIM
        T = 1 + (W + G) * (N - 1)
        seqs, idxs = [], []
        for i, toks in enumerate(tokens):
            assert len(toks) == T
            if self.lengths[i] + N > self.capacity:
                raise ValueError("KV cache full")
            idx = torch.tensor(toks, dtype=torch.long, device=self.device)
            idxs.append(idx)
            seqs.append(dict(q=self._q[idx].contiguous(), block_table=self.block_tables[i],
                             step_k=self._k[idx].contiguous(), step_v=self._v[idx].contiguous(),
                             out=torch.empty((T, 1, d), dtype=torch.bfloat16, device=self.device), P=self.lengths[i]))
        binding.la_step_attention_batch_paged(seqs, self._k_pages, self._v_pages, W, N, G, 1, 1, d)
        self._step = (seqs, W, N, G)
        return [self._logits[idx * 2 + (x["out"][:, 0, 0].float() > 0.5).long()].contiguous()
                for idx, x in zip(idxs, seqs)]

    def commit(self, bests, n_outs):
        seqs, W, N, G = self._step
        binding.la_kv_commit_batch(
            [dict(k_cache=self._k_pages, v_cache=self._v_pages, block_table=x["block_table"], step_k=x["step_k"],
                  step_v=x["step_v"], best=b, n_out=n, P=x["P"]) for x, b, n in zip(seqs, bests, n_outs)],
            W, N, G, 1, wl.TOY_HEAD_DIM)

    def advance(self, i, n):
        self.lengths[i] += n


def _demo():
    torch.cuda.set_device(0)
    for W, N, G in ((5, 4, 5), (15, 5, 15)):
        model = ToyAttentionLM(0)
        dec = LookaheadDecoder(model, [0, 5, 9], W, N, G)
        dec.generate(32)                      # warm-up
        torch.cuda.synchronize()
        t0, s0 = time.perf_counter(), dec.steps
        n = len(dec.generate(512))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        print("W=%d N=%d G=%d: %d tokens in %d steps (S = %.2f), %.0f us per step (host loop included)"
              % (W, N, G, n, dec.steps - s0, n / (dec.steps - s0), dt / (dec.steps - s0) * 1e6))


    n_seqs, (W, N, G) = 8, (15, 5, 15)
    dec = BatchedLookaheadDecoder(ToyBatchLM(0, n_seqs), [[0, 5 + i, 9] for i in range(n_seqs)], W, N, G)
    dec.generate(32)
    torch.cuda.synchronize()
    t0, s0 = time.perf_counter(), dec.seqs[0].steps
    n = sum(len(o) for o in dec.generate(256))
    torch.cuda.synchronize()
    dt, steps = time.perf_counter() - t0, dec.seqs[0].steps - s0
    print("%d sequences, W=%d N=%d G=%d: %d steps, %.0f us per step of the batch (host loop included)"
          % (n_seqs, W, N, G, steps, dt / steps * 1e6))


if __name__ == "__main__":
    _demo()
