// Internal declarations shared by the translation units of the HIP library.
// Nothing here is part of the C ABI (include/la.h is).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "la.h"

namespace la {

// Record a message for la_last_error() and hand back `code`.
la_status fail(la_status code, const char* fmt, ...);
// The code of this thread's last fail(): what a caller returns when a helper that reports through
// a null pointer (the workspaces) has failed.
la_status last_failure();

// Per-device scratch memory.  `bytes` of zero-initialised device memory that every kernel
// leaves zeroed again (tickets, packed argmax keys), and `bytes` of uninitialised memory
// (split partials).  Grown on demand - never while `stream` is being captured; returns nullptr
// (and records the error) on failure.
void* zeroed_workspace(size_t bytes, hipStream_t stream);
void* scratch_workspace(size_t bytes, hipStream_t stream);
void free_workspaces();
la_status select_workspace(int set);
// Testing hooks of the attention launchers (la_debug_override).
la_status set_override(const char* key, const char* value);

// Launchers (defined next to their kernels).
la_status launch_verify(const float* logits, const int* cand_tokens, int G, int N, int V,
                        int* accept_len, int* accepted, hipStream_t stream);
la_status launch_verify_step(const float* logits_cur, const float* logits_look, const float* logits_cand,
                             const int* cand_tokens, int W, int N, int G, int V, int* out_tokens, int* n_out,
                             int* best, int* new_window, int* accept_len, hipStream_t stream);
// One sequence of a batched la_verify_step (pointers as for launch_verify_step).
struct VerifySeq {
    const float* logits_cur;
    const float* logits_look;
    const float* logits_cand;
    const int* cand_tokens;
    int* out_tokens;
    int* n_out;
    int* best;
    int* new_window;
    int* accept_len;
};
la_status launch_verify_step_batch(const VerifySeq* seqs, int n_seqs, int W, int N, int G, int V,
                                   hipStream_t stream);
la_status launch_verify_sample(const float* logits_cur, const float* logits_cand, const int* cand_tokens,
                               const float* u_test, const float* u_final, float temperature, int N, int G,
                               int V, int* out_tokens, int* n_out, hipStream_t stream);
// Scratch memory that the caller of launch_step_attention provides instead of the per-device
// pools (which grow with hipMalloc): tickets (cleared by the launcher) and room for partials.
struct FixedWorkspace {
    void* tickets;
    size_t ticket_bytes;
    void* partials;
    size_t partial_bytes;
};
// Rotary position embedding applied to the query rows inside the attention kernel: the model's
// tables, fp32 [max_pos][head_dim/2] on the device (the launcher takes the rows from P on).
struct RopeTables {
    const float* cos;
    const float* sin;
    bool interleaved;
    bool rotate_keys;  // the step keys come unrotated too: the kernel turns them as their chunks land
};
// The library's own fixed block on the current device (a file-scope device array; no allocation).
la_status fixed_workspace(FixedWorkspace* ws);
// `capacity`: rows between the caches of consecutive KV heads (P for a packed cache).
// `block_table` != nullptr: the caches are pages [n_pages][kv_heads][page_size][head_dim]
// (page_size a multiple of 64) and `capacity` is not used.  `row_ids` != nullptr: the step holds
// n_rows rows of the (W, N, G) layout (packed cache only).  `k_scale` != nullptr: keys and values
// (cache and step rows) are 8-bit floats with one scale per KV head each (packed cache, whole steps).
la_status launch_step_attention(const void* q, const void* k_cache, const void* v_cache,
                                long long capacity, const int* block_table, int page_size, int n_pages,
                                const int* row_ids, int n_rows, const void* step_k, const void* step_v, int P,
                                int W, int N, int G, int heads, int kv_heads, int head_dim, void* out,
                                hipStream_t stream, const FixedWorkspace* fixed = nullptr,
                                const float* k_scale = nullptr, const float* v_scale = nullptr,
                                const RopeTables* rope = nullptr);
// One step of a batched launch.  Packed caches: k_cache / v_cache per step, block_table null.  Paged
// (page_size > 0): k_cache / v_cache are the shared page pools, block_table the step's own table.
struct BatchSeq {
    const void* q;
    const void* k_cache;
    const void* v_cache;
    const int* block_table;
    const void* step_k;
    const void* step_v;
    void* out;
    int P;
};
// The decomposition without partial results between workgroups (la_attention_rowtile.hip): packed or
// in-place bf16 caches, whole steps, head_dim 128.
bool rowtile_supported(int head_dim, int group, int T);
// 1: la_step_attention / _cap / _noalloc take the row-tile kernel for this shape; 0: the staged one.
int step_attention_kernel_choice(int P, int W, int N, int G, int heads, int kv_heads, int head_dim);
int rowtile_rope_positions();
la_status launch_step_attention_rowtile(const void* q, const void* k_cache, const void* v_cache, long long capacity,
                                        const void* step_k, const void* step_v, int P, int W, int N, int G, int heads,
                                        int kv_heads, void* out, hipStream_t stream, const RopeTables* rope = nullptr);
la_status launch_step_attention_batch(const BatchSeq* seqs, int n_seqs, int page_size, int n_pages, int W, int N,
                                      int G, int heads, int kv_heads, int head_dim, hipStream_t stream);
la_status launch_kv_commit(void* k_cache, void* v_cache, long long capacity, const int* block_table,
                           int page_size, int n_pages, const void* step_k, const void* step_v, int P, int W,
                           int N, int G, int kv_heads, int head_dim, const int* best, const int* n_out,
                           hipStream_t stream);
// The append with the key rows turned by their cache positions (contiguous caches only).
la_status launch_kv_commit_rope(void* k_cache, void* v_cache, long long capacity, const void* step_k,
                                const void* step_v, const float* cos, const float* sin, int interleaved, int P,
                                int W, int N, int G, int kv_heads, int head_dim, const int* best, const int* n_out,
                                hipStream_t stream);
// One sequence of a batched la_verify_sample (pointers as for launch_verify_sample).
struct SampleSeq {
    const float* logits_cur;
    const float* logits_cand;
    const int* cand_tokens;
    const float* u_test;
    const float* u_final;
    int* out_tokens;
    int* n_out;
    float temperature;
};
la_status launch_verify_sample_batch(const SampleSeq* seqs, int n_seqs, int N, int G, int V, hipStream_t stream);
// One append of a batched launch: block_table null = packed cache with `capacity` rows per head,
// else the caches are page pools (page_size, n_pages common to the launch).
struct CommitSeq {
    void* k_cache;
    void* v_cache;
    const int* block_table;
    const void* step_k;
    const void* step_v;
    const int* best;
    const int* n_out;
    long long capacity;
    int P;
};
la_status launch_kv_commit_batch(const CommitSeq* seqs, int n_seqs, int page_size, int n_pages, int W, int N,
                                 int G, int kv_heads, int head_dim, hipStream_t stream);
la_status launch_step_rope(void* q, void* step_k, const float* cos, const float* sin, int P, int W, int N, int G,
                           int heads, int kv_heads, int head_dim, int interleaved, hipStream_t stream);
size_t step_attention_workspace_bytes(int P, int W, int N, int G, int heads, int kv_heads,
                                      int head_dim);

// Measurement aids (la_probe.hip).
la_status launch_probe_stream_read(const void* src, long long bytes, void* sink, hipStream_t stream);
long long launch_probe_mfma(int iters, void* sink, hipStream_t stream);  // flops of the launch, -1 on error

}  // namespace la
