/*
 * la.h - C ABI of the MI355X (gfx950) lookahead-decoding hot path.
 *
 * Lookahead Decoding (arXiv 2402.02057) evaluates, in ONE model forward per
 * decoding step, the current input token, a W x (N-1) window of Jacobi
 * lookahead tokens and G candidate n-grams against the prefix KV cache
 * (Sec. 3, Sec. 3.3), then
 * verifies the candidates greedily (Sec. 3.2, Algorithm 3).  This library is
 * the attention of that forward and the verification reduction.  The n-gram
 * pool, the window update, projections, RoPE and the LM head are the
 * caller's.
 *
 * Row order of one step (shared by q, step_k, step_v and out):
 *   row 0                              current input token        position 0
 *   row 1 + l*W + j                    lookahead level l in [0,N-2] (0 = oldest
 *                                      kept Jacobi iterate), column j in [0,W-1]
 *                                                                 position 1+l+j
 *   row 1 + W*(N-1) + g*(N-1) + k      candidate g in [0,G-1], its k-th token
 *                                      after the shared first one position 1+k
 *   T = 1 + (W + G) * (N - 1) rows.
 * "Position" is relative to the current token (the digits of Fig. 2(b)); the
 * library does not use it, the caller's RoPE does.
 *
 * Visibility (Fig. 2(b), Sec. 3.3; conditioning sets of Algorithm 2):
 *   - every row attends to all P prefix keys and to the current token;
 *   - lookahead row (l, j) also attends to level-0 columns <= j and to its
 *     own column at levels <= l (its Jacobi trajectory, itself included);
 *   - candidate row (g, k) also attends to tokens <= k of candidate g;
 *   - nothing else: the branches and distinct candidates are mutually
 *     invisible.
 * Compared with the figure, whose oldest level starts with the current token,
 * the window here is a full W x (N-1) rectangle behind a separate current-token
 * row (every position shifted by one); the trajectories are the same.
 *
 * All pointers are DEVICE pointers unless said otherwise.  The caller owns
 * every buffer; nothing is retained after the call's work has run.  Calls are
 * asynchronous on `stream` (a hipStream_t passed as void*, NULL = the default
 * stream) and never synchronise the device.  The library keeps a small device
 * workspace per device (split partials, tickets), grown on demand with
 * hipMalloc - so the first call at a new size may allocate - and shared by
 * all calls on that device: calls issued to one stream are ordered; calls on
 * different streams of the same device must not overlap in time unless they use
 * different workspace sets (la_select_workspace).  The calls may
 * be recorded into a HIP graph once a call of the same (or a larger) shape has
 * run outside the capture: that one sizes and clears the workspace, the kernels
 * leave it cleared.  A workspace block that a later, larger call replaces stays
 * allocated until la_shutdown, so graphs recorded before remain valid (do not
 * call la_shutdown while such a graph may still be launched).
 *
 * Errors are returned, never thrown; on error nothing has been launched.
 */
#ifndef LA_H
#define LA_H

#ifdef __cplusplus
extern "C" {
#endif

typedef int la_status;
#define LA_OK 0
#define LA_EINVAL (-1)       /* null pointer, negative size, N < 2, misaligned buffer */
#define LA_EUNSUPPORTED (-2) /* head_dim not 64 or 128, heads % kv_heads != 0, step too large */
#define LA_ENOMEM (-3)       /* workspace allocation failed */
#define LA_EHIP (-4)         /* a HIP call or the launch failed (see la_last_error) */

/*
 * Lookahead-step attention (Sec. 2 causal-attention definition with the mask
 * of Sec. 3.3):  out[r][h] = sum_c softmax_c(q[r][h].k[c] / sqrt(head_dim)) v[c]
 * over the P prefix keys of KV head h / (heads / kv_heads) and the step keys
 * row r may see.  bf16 in, fp32 accumulation and softmax, bf16 out (round to
 * nearest even).
 *
 *   q        bf16 [T][heads][head_dim]           16-byte aligned
 *   k_cache  bf16 [kv_heads][P][head_dim]        16-byte aligned; may be NULL iff P == 0
 *   v_cache  same shape as k_cache
 *   step_k   bf16 [T][kv_heads][head_dim]        this step's keys, row order as q
 *   step_v   same shape as step_k
 *   out      bf16 [T][heads][head_dim]
 *   P >= 0, W >= 0, G >= 0, N >= 2; head_dim in {64, 128}; heads % kv_heads == 0.
 */
la_status la_step_attention(const void* q, const void* k_cache, const void* v_cache,
                            const void* step_k, const void* step_v, int P, int W, int N, int G,
                            int heads, int kv_heads, int head_dim, void* out, void* stream);

/*
 * Rotary position embedding of a step's queries and keys, in place, at the positions the
 * step's tokens hold: row r of the layout above sits at P + (its relative position, the
 * digit printed on the token in Fig. 2(b)).  Run it on the projected q and step_k before
 * la_step_attention*; the keys la_kv_commit* appends afterwards are then the rotated ones,
 * as the cache needs them (an accepted token keeps the position it was evaluated at,
 * Sec. 3.3).  Pair i of a head turns by the angle whose cosine and sine are cos[t][i],
 * sin[t][i], t the row's position: (a, b) -> (a cos - b sin, b cos + a sin), computed in fp32
 * and rounded to bf16 once.
 *
 *   q            bf16 [T][heads][head_dim], in/out, or NULL: then only the keys are rotated
 *   step_k       bf16 [T][kv_heads][head_dim], in/out
 *   cos, sin     fp32 [max_pos][head_dim/2] on the device (the model's tables)
 *   max_pos      positions the tables hold; the step reaches P + max(W + N - 2, N - 1)
 *   interleaved  0: pair i is (x[i], x[i + head_dim/2]);  nonzero: (x[2i], x[2i + 1])
 *   head_dim: a multiple of 16 up to 1024.  All four pointers 16-byte aligned.
 * A separate pass rather than part of the attention kernel: there every row block and every
 * head of a group would rotate the same keys again.
 */
la_status la_step_rope(void* q, void* step_k, const float* cos, const float* sin, int max_pos, int P, int W, int N,
                       int G, int heads, int kv_heads, int head_dim, int interleaved, void* stream);

/*
 * The same step (Sec. 3.3 mask, Sec. 2 attention) over a KV cache quantised to 8-bit floats: an
 * extension for memory-bound decoding, the regime the method targets (Sec. 1, Sec. 4.2); the
 * paper itself computes in 16 bits.  A key or value element of KV head h is a code of the OCP
 * E4M3 format in its finite-only form (exponent bias 7, no infinities, largest value 448) and
 * stands for the code's value times k_scale[h] (keys) or v_scale[h] (values).  The step's own
 * keys and values arrive quantised the same way, so that a token committed to the cache later
 * is read back exactly as its step saw it.
 *
 *   q                 bf16 [T][heads][head_dim]
 *   k_cache, v_cache  8-bit [kv_heads][P][head_dim]
 *   step_k, step_v    8-bit [T][kv_heads][head_dim]
 *   k_scale, v_scale  fp32 [kv_heads], device memory, 4-byte aligned, finite and > 0
 *   out               bf16 [T][heads][head_dim]
 * Codes are converted exactly (every E4M3 value is a bf16 number), the products run on the
 * bf16 MFMA pipes with fp32 accumulation, the key scale multiplies the scores and the value
 * scale the finished rows.  The two NaN codes (0x7f, 0xff) give NaN outputs in the rows that
 * see them.  Everything else (row order, head mapping, alignment, errors, workspace) as
 * la_step_attention.  Packed caches and whole steps only.
 */
la_status la_step_attention_fp8kv(const void* q, const void* k_cache, const void* v_cache, const void* step_k,
                                  const void* step_v, const float* k_scale, const float* v_scale, int P, int W,
                                  int N, int G, int heads, int kv_heads, int head_dim, void* out, void* stream);

/*
 * la_step_attention with the rotary position embedding done inside the kernel: q arrives as
 * the projection left it and is not modified; the kernel stages its rows in on-chip memory,
 * turns them by the positions of Fig. 2(b) (row r sits at P + its digit) with the arithmetic
 * of la_step_rope, and goes on as la_step_attention does.
 *
 *   rotate_keys == 0: step_k is already rotated (la_step_rope with q == NULL rotates it alone).
 *     The result has the bits of la_step_rope on q followed by la_step_attention.
 *   rotate_keys != 0: step_k arrives unrotated as well and is not modified; every workgroup
 *     turns the step keys it has staged before it multiplies with them.  The result has the
 *     bits of la_step_rope on q and step_k followed by la_step_attention, with no pass over
 *     the step's tensors at all.  Append the accepted rows with la_kv_commit_rope then, which
 *     turns the few key rows it copies.
 *
 *   cos, sin     fp32 [max_pos][head_dim/2] on the device, 16-byte aligned
 *   max_pos      positions the tables hold; the step reaches P + max(W + N - 2, N - 1)
 *   interleaved  0: pair i is (x[i], x[i + head_dim/2]);  nonzero: (x[2i], x[2i + 1])
 * Everything else as la_step_attention (the choice between the two kernels included, see
 * la_step_attention_kernel).  Limit: the table rows of the step's positions are staged beside
 * the key/value ring; with head_dim 128 there is room for 32 positions (W + N - 2 <= 31) in the
 * staged kernel's common decomposition and for 64 in the row-tile kernel.  A step that needs
 * more is refused with LA_EUNSUPPORTED: rotate with la_step_rope then.
 */
la_status la_step_attention_rope(const void* q, const void* k_cache, const void* v_cache, const void* step_k,
                                 const void* step_v, const float* cos, const float* sin, int max_pos, int interleaved,
                                 int rotate_keys, int P, int W, int N, int G, int heads, int kv_heads, int head_dim,
                                 void* out, void* stream);

/*
 * The same step over a cache allocated for more keys than it holds, as a decoding loop keeps
 * it (rows are appended in place, see la_kv_commit):
 *   k_cache, v_cache  bf16 [kv_heads][capacity][head_dim]; rows 0..P-1 of every head are the
 *                     prefix, the rest is never read.  capacity >= P.
 * Everything else as la_step_attention, which is the case capacity == P.
 */
la_status la_step_attention_cap(const void* q, const void* k_cache, const void* v_cache, long long capacity,
                                const void* step_k, const void* step_v, int P, int W, int N, int G,
                                int heads, int kv_heads, int head_dim, void* out, void* stream);

/*
 * Append the tokens a greedy step accepted to the KV cache, on the device, from the result
 * la_verify_step left there.  The step's keys and values of those rows are already what the
 * next steps need (Sec. 3.3: candidate token k is evaluated at relative position 1+k, the
 * position it holds once accepted), so this is a copy:
 *   cache row P        <- step row 0 (the current token)
 *   cache row P + i    <- step row 1 + W(N-1) + best(N-1) + (i-1), i = 1 .. n_out-1
 * The last of the n_out emitted tokens is the next current token; its keys do not exist yet.
 * Afterwards the prefix holds P + n_out keys.
 *
 *   k_cache, v_cache  bf16 [kv_heads][capacity][head_dim], in/out; P + N <= capacity (the
 *                     count is known only on the device, so room for a full match is required)
 *   step_k, step_v    bf16 [T][kv_heads][head_dim] of the step just verified
 *   best, n_out       int32 [1] each, as written by la_verify_step (values outside -1..G-1
 *                     and 1..N are clamped, never followed out of bounds)
 *   head_dim: any multiple of 8 up to 1024.
 * Rows are moved as bytes (2 * head_dim of them) and never interpreted: for a cache of 8-bit
 * elements (la_step_attention_fp8kv) pass head_dim / 2, so that a row is head_dim bytes.
 */
la_status la_kv_commit(void* k_cache, void* v_cache, long long capacity, const void* step_k,
                       const void* step_v, int P, int W, int N, int G, int kv_heads, int head_dim,
                       const int* best, const int* n_out, void* stream);

/*
 * la_kv_commit for a step whose keys were left unrotated in memory (la_step_attention_rope
 * with rotate_keys != 0): the key row appended as cache row P + i is turned by position P + i,
 * the position its step evaluated it at (Sec. 3.3; Fig. 2(b): the current token at P, token
 * i - 1 of a candidate at P + i), with the arithmetic of la_step_rope, so the cache holds the
 * bits that la_step_rope followed by la_kv_commit would have left.  Values are copied.
 *
 *   cos, sin, max_pos, interleaved  as la_step_rope; the append reaches position P + N - 1
 *   head_dim: a multiple of 16 up to 1024.  Contiguous bf16 caches only.
 * Everything else as la_kv_commit.
 */
la_status la_kv_commit_rope(void* k_cache, void* v_cache, long long capacity, const void* step_k,
                            const void* step_v, const float* cos, const float* sin, int max_pos, int interleaved,
                            int P, int W, int N, int G, int kv_heads, int head_dim, const int* best,
                            const int* n_out, void* stream);

/*
 * The same step and the same append over a PAGED cache, as a serving system keeps it:
 *   k_pages, v_pages  bf16 [n_pages][kv_heads][page_size][head_dim]; 16-byte aligned
 *   block_table       int32 [ceil(P / page_size)] (for the append: ceil((P + N) / page_size)):
 *                     prefix key t of every KV head sits in page block_table[t / page_size] at
 *                     slot t % page_size.  Entries outside 0..n_pages-1 are clamped into that
 *                     range (wrong results, never an access outside the pages).
 *   page_size         a multiple of 64
 * The result is that of la_step_attention / la_kv_commit over the packed cache the table
 * stands for.  Pages the table does not name are never touched.
 */
la_status la_step_attention_paged(const void* q, const void* k_pages, const void* v_pages, const int* block_table,
                                  int page_size, int n_pages, const void* step_k, const void* step_v, int P,
                                  int W, int N, int G, int heads, int kv_heads, int head_dim, void* out,
                                  void* stream);
la_status la_kv_commit_paged(void* k_pages, void* v_pages, const int* block_table, int page_size, int n_pages,
                             const void* step_k, const void* step_v, int P, int W, int N, int G, int kv_heads,
                             int head_dim, const int* best, const int* n_out, void* stream);

/*
 * Several appends in ONE launch: the layers of a model after a step (every layer's step keys
 * and values go to that layer's cache, all following the same best / n_out), or several
 * sequences, or both.  The same result as n_descs calls of la_kv_commit / la_kv_commit_paged,
 * one per descriptor; a call costs a launch, and a step has as many appends as layers.
 *
 *   descs      HOST array of n_descs descriptors (read before the call returns), 1..1024
 *   page_size, n_pages   of the page pools of the descriptors that name a block table (ignored
 *                        if none does)
 * Destination rows of different descriptors must not overlap.
 */
typedef struct la_commit_desc {
    void* k_cache;           /* block_table NULL: bf16 [kv_heads][capacity][head_dim], P + N <= capacity; */
    void* v_cache;           /* else the page pool, bf16 [n_pages][kv_heads][page_size][head_dim]         */
    const int* block_table;  /* NULL, or int32 [ceil((P + N) / page_size)] on the device                  */
    const void* step_k;      /* bf16 [T][kv_heads][head_dim] of the step just verified                    */
    const void* step_v;
    const int* best;         /* int32 [1] each on the device, as la_verify_step wrote them;               */
    const int* n_out;        /* descriptors may share them                                                */
    long long capacity;      /* rows per KV head of a packed cache (not used with a block table)          */
    int P;                   /* keys the cache holds before the append                                    */
    int reserved;            /* must be 0 */
} la_commit_desc;

la_status la_kv_commit_batch(const la_commit_desc* descs, int n_descs, int page_size, int n_pages, int W, int N,
                             int G, int kv_heads, int head_dim, void* stream);

/*
 * The step over a SUBSET of its rows: one device's share under lookahead parallelism
 * (Sec. 3.4), which keeps the current token and the oldest window level everywhere and deals
 * the columns of the newer levels and the candidates out to the devices; such a share needs no
 * key of another share, so every device runs this call on its own rows and the outputs are
 * those of the full step.
 *   row_ids  int32 [n_rows]  which rows of the (W, N, G) layout the step holds, in the order of
 *                            q / step_k / step_v / out; 1 <= n_rows <= 1024.  Ids outside the
 *                            layout are clamped into it.
 *   q, out   bf16 [n_rows][heads][head_dim];  step_k, step_v  bf16 [n_rows][kv_heads][head_dim]
 * Local row a attends to the P prefix keys and to local key b iff row row_ids[a] of the full
 * layout may see row row_ids[b].  Everything else as la_step_attention (packed cache).
 */
la_status la_step_attention_rows(const void* q, const void* k_cache, const void* v_cache, const void* step_k,
                                 const void* step_v, const int* row_ids, int n_rows, int P, int W, int N, int G,
                                 int heads, int kv_heads, int head_dim, void* out, void* stream);

/*
 * Several independent steps (sequences decoding side by side, or the sequences of a ragged
 * batch) in ONE launch: the same result as n_seqs calls of la_step_attention with the same
 * W, N, G and head geometry, one per descriptor, in any order.  A single decode-sized step
 * cannot fill the GPU (it is bound by latencies, not by bandwidth); a batch can: key ranges are
 * split only as far as the whole batch needs, and one step's tail overlaps the next one's head.
 *
 *   seqs    HOST array of n_seqs descriptors (read before the call returns); the pointers in
 *           them are device pointers with the shapes and alignment la_step_attention asks for
 *   n_seqs  1..1024 (launched sixteen at a time, longest prefix first)
 * Outputs of different descriptors must not overlap.
 */
typedef struct la_step_desc {
    const void* q;        /* bf16 [T][heads][head_dim] */
    const void* k_cache;  /* bf16 [kv_heads][P][head_dim]; may be NULL iff P == 0 */
    const void* v_cache;
    const void* step_k;   /* bf16 [T][kv_heads][head_dim] */
    const void* step_v;
    void* out;            /* bf16 [T][heads][head_dim] */
    int P;                /* prefix length of this sequence */
    int reserved;         /* must be 0 */
} la_step_desc;

la_status la_step_attention_batch(const la_step_desc* seqs, int n_seqs, int W, int N, int G, int heads,
                                  int kv_heads, int head_dim, void* stream);

/*
 * The same over a paged cache, as a serving system holds it: all sequences share one pool of
 * pages (k_pages, v_pages, page_size, n_pages as for la_step_attention_paged) and every
 * descriptor names its sequence's block table.
 */
typedef struct la_step_desc_paged {
    const void* q;
    const int* block_table;  /* int32 [ceil(P / page_size)], device; may be NULL iff P == 0 */
    const void* step_k;
    const void* step_v;
    void* out;
    int P;
    int reserved;            /* must be 0 */
} la_step_desc_paged;

la_status la_step_attention_batch_paged(const la_step_desc_paged* seqs, int n_seqs, const void* k_pages,
                                        const void* v_pages, int page_size, int n_pages, int W, int N, int G,
                                        int heads, int kv_heads, int head_dim, void* stream);

/*
 * Greedy verification reduction (Sec. 2, the guess-and-verify paragraph: accept a draft
 * token while it equals the model's greedy token, stop at the first mismatch;
 * Algorithm 3 runs it over G candidates).
 *
 *   logits       fp32 [G][N-1][V]; row (g,k) is the model output that judges
 *                cand_tokens[g][k]: k = 0 the output at the current token,
 *                k >= 1 the output at candidate token k-1.  Values must not be NaN.
 *   cand_tokens  int32 [G][N-1]
 *   accept_len   int32 [G]       out: number of leading k with argmax == cand_tokens
 *   accepted     int32 [G][N-1]  out: argmax of every row, lowest index on ties
 *   G >= 0 (G == 0 is a no-op), N >= 2, V >= 1.
 */
la_status la_verify(const float* logits, const int* cand_tokens, int G, int N, int V,
                    int* accept_len, int* accepted, void* stream);

/*
 * The end of a greedy lookahead step in one launch: Algorithm 3 in full (Sec. 3.2: a
 * candidate's tokens are accepted while they equal the model's greedy tokens, the longest
 * run wins, and the model's own token at the first unaccepted slot follows - the
 * correction token, or the bonus token after a full match, so that a step always moves
 * by at least one token), and the new window tokens of Algorithm 2's lookahead branch
 * (the greedy token at each of the W newest lookahead positions).
 *
 *   logits_cur   fp32 [V]          model output at the current token: judges slot 0 of
 *                                  every candidate
 *   logits_look  fp32 [W][V]       outputs at the W newest lookahead tokens (level N-2,
 *                                  columns 0..W-1); may be NULL iff W == 0
 *   logits_cand  fp32 [G][N-1][V]  row (g,k): output at candidate g's token k: judges slot
 *                                  k+1; row (g,N-2) gives the bonus token; NULL iff G == 0
 *   cand_tokens  int32 [G][N-1]
 *   out_tokens   int32 [N]   out: the accepted tokens, n_out of them
 *   n_out        int32 [1]   out: 1..N
 *   best         int32 [1]   out: the winning candidate - the lowest index among those with
 *                            the longest accepted run (the order Algorithm 3 scans them in);
 *                            -1 if G == 0
 *   new_window   int32 [W]   out
 *   accept_len   int32 [G]   out: accepted run of every candidate; may be NULL
 * Argmax = lowest index of the maximum; values must not be NaN.  1 + W + G(N-1) <= 12288.
 */
la_status la_verify_step(const float* logits_cur, const float* logits_look, const float* logits_cand,
                         const int* cand_tokens, int W, int N, int G, int V, int* out_tokens, int* n_out,
                         int* best, int* new_window, int* accept_len, void* stream);

/*
 * The ends of several sequences' steps (same W, N, G, V) in ONE launch: the same result as
 * n_descs calls of la_verify_step, one per descriptor.  With la_step_attention_batch and
 * la_kv_commit_batch this keeps a step of a batch of sequences at one launch per operation.
 *
 *   descs    HOST array of n_descs descriptors (read before the call returns), 1..1024; the
 *            pointers in them are device pointers with the shapes la_verify_step asks for
 * Outputs of different descriptors must not overlap.
 */
typedef struct la_verify_desc {
    const float* logits_cur;   /* fp32 [V] */
    const float* logits_look;  /* fp32 [W][V]; may be NULL iff W == 0 */
    const float* logits_cand;  /* fp32 [G][N-1][V]; may be NULL iff G == 0 */
    const int* cand_tokens;    /* int32 [G][N-1] */
    int* out_tokens;           /* int32 [N] */
    int* n_out;                /* int32 [1] */
    int* best;                 /* int32 [1] */
    int* new_window;           /* int32 [W] */
    int* accept_len;           /* int32 [G]; may be NULL */
} la_verify_desc;

la_status la_verify_step_batch(const la_verify_desc* descs, int n_descs, int W, int N, int G, int V,
                               void* stream);

/*
 * Sampling verification in one launch (Algorithm 4; App. B shows that every token it emits
 * follows the model's own distribution).  Distributions are softmax(logits / temperature).
 * Position by position the surviving candidates are examined in order: candidate token s is
 * accepted if its draw is below P(s), where P starts as the first survivor's distribution at
 * that position and, after every rejection, has the rejected token's probability set to zero
 * and is renormalised; after an acceptance only the later candidates with the same token
 * survive.  If none is accepted one token is drawn from the residual P and the walk stops;
 * after N-1 acceptances one token is drawn from the first survivor's N-th distribution.
 *
 *   logits_cur   fp32 [V]          model output at the current token (distribution 1 of every
 *                                  candidate)
 *   logits_cand  fp32 [G][N-1][V]  row (g,k): output at candidate g's token k (its distribution
 *                                  k+2); NULL iff G == 0
 *   cand_tokens  int32 [G][N-1]    a token outside 0 .. V-1 (a padding id) is examined like any
 *                                  other - its draw is spent - and has probability zero: never
 *                                  accepted, nothing ruled out, no logit read
 *   u_test       fp32 [N-1][G]     uniform draws in [0,1): u_test[i][j] serves the j-th candidate
 *                                  examined at position i; NULL iff G == 0
 *   u_final      fp32 [1]          the draw for the last token (inverse CDF in index order)
 *   temperature  > 0 (host value)
 *   out_tokens   int32 [N]   out: n_out tokens
 *   n_out        int32 [1]   out: 1..N
 * The accept test is "draw < P(s)" (a token of probability zero is never accepted).  Arithmetic
 * is fp32: a draw within rounding of P(s), or of a step of the cumulative distribution, may fall
 * on either side.  G <= 1024.
 */
la_status la_verify_sample(const float* logits_cur, const float* logits_cand, const int* cand_tokens,
                           const float* u_test, const float* u_final, float temperature, int N, int G, int V,
                           int* out_tokens, int* n_out, void* stream);

/*
 * Sampling verification for several sequences (same N, G, V) in ONE launch: the same result as
 * n_descs calls of la_verify_sample, one per descriptor, each with its own draws and
 * temperature.
 *   descs    HOST array of n_descs descriptors (read before the call returns), 1..1024; device
 *            pointers with the shapes la_verify_sample asks for
 */
typedef struct la_sample_desc {
    const float* logits_cur;   /* fp32 [V] */
    const float* logits_cand;  /* fp32 [G][N-1][V]; may be NULL iff G == 0 */
    const int* cand_tokens;    /* int32 [G][N-1] */
    const float* u_test;       /* fp32 [N-1][G] */
    const float* u_final;      /* fp32 [1] */
    int* out_tokens;           /* int32 [N] */
    int* n_out;                /* int32 [1] */
    float temperature;         /* > 0 */
    int reserved;              /* must be 0 */
} la_sample_desc;

la_status la_verify_sample_batch(const la_sample_desc* descs, int n_descs, int N, int G, int V, void* stream);

/*
 * la_step_attention for callers that cannot allocate device memory: code under HIP graph
 * capture with no warm-up call, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels, same result as la_step_attention; the difference is where the
 * scratch memory (tickets and split partials) comes from: a fixed block of 128 KiB + 12 MiB
 * inside the library's own image, present once on every device the library runs on until the
 * process ends.  The call never calls hipMalloc, hipFree or any allocating routine.
 *
 * Limits: a step whose decomposition needs more than 128 KiB of tickets (128 split groups) or
 * more than 12 MiB of partials is refused with LA_EUNSUPPORTED (la_last_error says how much it
 * needs); the library's own decomposition needs at most 5 MiB.  Every call on a device shares that device's block:
 * the tickets are cleared by a small kernel in front of the step (no memset node, so the call
 * can be captured), the partials are overwritten; two such calls that overlap in time on one
 * device (different streams) race and give wrong results.  la_select_workspace does not apply.
 */
la_status la_step_attention_noalloc(const void* q, const void* k_cache, const void* v_cache,
                                    const void* step_k, const void* step_v, int P, int W, int N, int G,
                                    int heads, int kv_heads, int head_dim, void* out, void* stream);

/*
 * Testing hooks (host strings; not for production use).  They take their first values from the
 * environment variables named below, read once at the first attention call, and apply to the
 * whole process from then on:
 *   "attn_plan"        (LA_ATTN_PLAN)        "RT,KS,XS,NS,KC[,PRE]": the decomposition of the one-step
 *                                            entry points forced by hand (ignored where no such
 *                                            kernel is compiled); NULL or "" = the library's choice
 *                                            (a forced decomposition is one of the staged kernel)
 *   "attn_rowtile"     (no variable)         "1" / "0": the row-tile kernel forced on (where it
 *                                            applies) / off; NULL = the library's choice
 *   "batch_plan"       (LA_BATCH_PLAN)       "2" or "4": 32-row tiles per workgroup of a batched launch
 *   "force_recompute"  (LA_FORCE_RECOMPUTE)  "1": treat every split group as spread over several
 *                                            XCDs, so that the recompute path runs
 * Returns LA_EINVAL for an unknown key or a malformed plan.
 */
la_status la_debug_override(const char* key, const char* value);

/*
 * Measurement aids (not part of the method; Sec. 1 and Sec. 4.2 argue from the gap between what
 * decoding moves and what the device can compute, so a benchmark quotes both): what this device
 * reaches at best.  Time them with events on `stream`.
 *   la_probe_stream_read  reads `bytes` (a multiple of 16, 16-byte aligned) of device memory once;
 *                         `sink` (4 bytes of device memory) is never written in practice
 *   la_probe_mfma         `iters` x 8 bf16 MFMAs (32x32x16) per wave on register operands, 32 waves
 *                         per compute unit; returns the floating-point operations of the launch
 *                         (-1 on error).  `sink`: 24 bytes of device memory, 8-byte aligned; the
 *                         first wave leaves its elapsed shader-clock cycles in sink[0] and its
 *                         elapsed 100 MHz ticks in sink[1] (uint64 each): the clock it ran at
 */
la_status la_probe_stream_read(const void* src, long long bytes, void* sink, void* stream);
long long la_probe_mfma(int iters, void* sink, void* stream);

/*
 * Bytes of device workspace la_step_attention may need for this shape (0 if none; an upper
 * bound: a shape that takes the row-tile kernel, see la_step_attention_kernel, needs none).
 */
long long la_step_attention_workspace_bytes(int P, int W, int N, int G, int heads, int kv_heads,
                                            int head_dim);

/*
 * Which kernel la_step_attention, la_step_attention_cap and la_step_attention_noalloc take for
 * this shape: 0 the staged kernel (workgroups split the keys of a row block and combine partial
 * results; every shape), 1 the row-tile kernel (a workgroup walks all keys for 32 rows and half
 * of the value columns and writes `out` directly; head_dim 128, picked for short prefixes,
 * where it measures 10 to 28 % faster).  Both compute the step of Sec. 3.3 to the same bar; the
 * output bits may differ between them.  -1 for arguments la_step_attention would refuse.
 */
int la_step_attention_kernel(int P, int W, int N, int G, int heads, int kv_heads, int head_dim);

/* Free the per-device workspaces.  No call may be in flight.  Optional at exit. */
void la_shutdown(void);

/*
 * Which of the library's 16 workspace sets (per device) the calling thread's next calls use;
 * 0 until told otherwise.  Calls that may overlap in time on one device - issued to different
 * streams - must use different sets; a HIP graph keeps the set that was selected when it was
 * recorded.  A set costs memory only once it has been used.  LA_EINVAL outside 0..15.
 */
la_status la_select_workspace(int set);

/* Host string describing the most recent error on this thread ("" if none). */
const char* la_last_error(void);

/* Library version, major * 1000 + minor. */
int la_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LA_H */
