// C-ABI entry points of the lookahead-decoding hot path (declared in include/la.h):
// argument validation, error reporting and the per-device workspaces.  The kernels
// live in la_attention.hip and la_verify.hip.
#include <stdarg.h>
#include <stdio.h>

#include <mutex>
#include <vector>

#include "la_internal.h"

namespace la {

static thread_local char g_error[512] = "";
static thread_local la_status g_last_code = LA_OK;

la_status fail(la_status code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    g_last_code = code;
    return code;
}

la_status last_failure() { return g_last_code; }

namespace {
constexpr int kMaxDevices = 16;
struct Pool {
    void* zeroed = nullptr;
    size_t zeroed_bytes = 0;
    void* scratch = nullptr;
    size_t scratch_bytes = 0;
    // Blocks that a growth replaced.  They are kept until la_shutdown: work already issued, and
    // HIP graphs recorded earlier, still name them (and no call has to wait for the device).
    std::vector<void*> retired;
};
// Per device, a few independent sets of blocks.  A thread's calls use the set it selected
// (la_select_workspace, set 0 unless told otherwise): calls that may overlap in time - on different
// streams - must use different sets, calls on one stream run in order and share one.
constexpr int kWorkspaceSets = 16;
Pool g_pools[kMaxDevices][kWorkspaceSets];
thread_local int g_set = 0;
std::mutex g_mutex;

Pool* current_pool()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        fail(LA_EHIP, "hipGetDevice failed or device index out of range");
        return nullptr;
    }
    return &g_pools[dev][g_set];
}
}  // namespace

la_status select_workspace(int set)
{
    if (set < 0 || set >= kWorkspaceSets)
        return fail(LA_EINVAL, "la_select_workspace: set %d is not in 0..%d", set, kWorkspaceSets - 1);
    g_set = set;
    return LA_OK;
}

namespace {
// Growing a block means hipMalloc (and a clear on the stream): neither may happen while the
// stream is being captured into a graph - the allocation would invalidate the capture, the
// clear would be recorded as a node of it.
bool growth_allowed(hipStream_t stream)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &status) == hipSuccess && status != hipStreamCaptureStatusNone) {
        fail(LA_EUNSUPPORTED, "the device workspace must grow for this shape, which cannot happen while the stream is "
                              "being captured: run a call of this (or a larger) shape outside the capture first");
        return false;
    }
    return true;
}
}  // namespace

void* zeroed_workspace(size_t bytes, hipStream_t stream)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    Pool* p = current_pool();
    if (!p) return nullptr;
    if (bytes <= p->zeroed_bytes) return p->zeroed;
    if (!growth_allowed(stream)) return nullptr;
    // Growing (only when a larger shape than any before is seen): a fresh block, cleared on
    // this stream ahead of the kernel that will use it; the old one is retired, not freed.
    size_t want = bytes < (1u << 16) ? (1u << 16) : bytes;
    void* fresh = nullptr;
    if (hipMalloc(&fresh, want) != hipSuccess) {
        fail(LA_ENOMEM, "hipMalloc of %zu bytes of ticket workspace failed", want);
        return nullptr;
    }
    if (hipMemsetAsync(fresh, 0, want, stream) != hipSuccess) {
        (void)hipFree(fresh);
        fail(LA_EHIP, "hipMemsetAsync on the ticket workspace failed");
        return nullptr;
    }
    if (p->zeroed) p->retired.push_back(p->zeroed);
    p->zeroed = fresh;
    p->zeroed_bytes = want;
    return fresh;
}

void* scratch_workspace(size_t bytes, hipStream_t stream)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    Pool* p = current_pool();
    if (!p) return nullptr;
    if (bytes <= p->scratch_bytes) return p->scratch;
    if (!growth_allowed(stream)) return nullptr;
    size_t want = bytes < (size_t(8) << 20) ? (size_t(8) << 20) : bytes + bytes / 4;
    void* fresh = nullptr;
    if (hipMalloc(&fresh, want) != hipSuccess) {
        fail(LA_ENOMEM, "hipMalloc of %zu bytes of partial-result workspace failed", want);
        return nullptr;
    }
    if (p->scratch) p->retired.push_back(p->scratch);
    p->scratch = fresh;
    p->scratch_bytes = want;
    return fresh;
}

void free_workspaces()
{
    std::lock_guard<std::mutex> lock(g_mutex);
    int saved = 0;
    (void)hipGetDevice(&saved);
    for (int d = 0; d < kMaxDevices; ++d) {
        bool any = false;
        for (const Pool& p : g_pools[d]) any = any || p.zeroed || p.scratch || !p.retired.empty();
        if (!any) continue;
        if (hipSetDevice(d) != hipSuccess) continue;
        (void)hipDeviceSynchronize();
        for (Pool& p : g_pools[d]) {
            if (p.zeroed) (void)hipFree(p.zeroed);
            if (p.scratch) (void)hipFree(p.scratch);
            for (void* block : p.retired) (void)hipFree(block);
            p = Pool();
        }
    }
    (void)hipSetDevice(saved);
}

}  // namespace la

extern "C" {

namespace {

// block_table == nullptr: packed caches with `capacity` rows per head; else pages.
la_status step_attention_checked(const char* name, const void* q, const void* k_cache, const void* v_cache,
                                 long long capacity, const int* block_table, int page_size, int n_pages,
                                 const void* step_k, const void* step_v, int P, int W, int N, int G, int heads,
                                 int kv_heads, int head_dim, void* out, void* stream, const int* row_ids = nullptr,
                                 int n_rows = 0, const la::FixedWorkspace* fixed = nullptr,
                                 const float* k_scale = nullptr, const float* v_scale = nullptr,
                                 const la::RopeTables* rope = nullptr)
{
    if (P < 0 || W < 0 || G < 0 || N < 2 || heads < 1 || kv_heads < 1)
        return la::fail(LA_EINVAL, "%s: need P,W,G >= 0, N >= 2, heads,kv_heads >= 1 "
                                   "(got P=%d W=%d N=%d G=%d heads=%d kv_heads=%d)",
                        name, P, W, N, G, heads, kv_heads);
    if (head_dim != 64 && head_dim != 128)
        return la::fail(LA_EUNSUPPORTED, "%s: head_dim %d is not 64 or 128", name, head_dim);
    if (heads % kv_heads != 0)
        return la::fail(LA_EUNSUPPORTED, "%s: heads %d not a multiple of kv_heads %d", name, heads, kv_heads);
    const long long T = 1 + (long long)(W + G) * (N - 1);
    if (T > (1 << 20) || (long long)P > (1ll << 30))
        return la::fail(LA_EINVAL, "%s: step of %lld rows / prefix %d too large", name, T, P);
    if (!block_table && (capacity < P || capacity > (1ll << 40)))
        return la::fail(LA_EINVAL, "%s: capacity %lld does not hold the %d prefix keys", name, capacity, P);
    if (!q || !step_k || !step_v || !out || (P > 0 && (!k_cache || !v_cache)))
        return la::fail(LA_EINVAL, "%s: null pointer", name);
    if (((uintptr_t)block_table) & 3) return la::fail(LA_EINVAL, "%s: block_table must be 4-byte aligned", name);
    const uintptr_t bits = (uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache |
                           (uintptr_t)step_k | (uintptr_t)step_v | (uintptr_t)out;
    if (bits & 15) return la::fail(LA_EINVAL, "%s: buffers must be 16-byte aligned", name);
    return la::launch_step_attention(q, k_cache, v_cache, capacity, block_table, page_size, n_pages, row_ids,
                                     n_rows, step_k, step_v, P, W, N, G, heads, kv_heads, head_dim, out,
                                     (hipStream_t)stream, fixed, k_scale, v_scale, rope);
}

// page geometry shared by the paged entry points
la_status check_pages(const char* name, const int* block_table, int page_size, int n_pages, long long rows)
{
    if (page_size < 64 || page_size % 64 != 0 || page_size > (1 << 20))
        return la::fail(LA_EUNSUPPORTED, "%s: page_size %d is not a multiple of 64 in 64..2^20", name, page_size);
    if (n_pages < 1) return la::fail(LA_EINVAL, "%s: n_pages %d < 1", name, n_pages);
    if (rows > 0 && !block_table) return la::fail(LA_EINVAL, "%s: block_table is null", name);
    return LA_OK;
}

}  // namespace

la_status la_step_attention(const void* q, const void* k_cache, const void* v_cache,
                            const void* step_k, const void* step_v, int P, int W, int N, int G,
                            int heads, int kv_heads, int head_dim, void* out, void* stream)
{
    return step_attention_checked("la_step_attention", q, k_cache, v_cache, P, nullptr, 0, 0, step_k, step_v,
                                  P, W, N, G, heads, kv_heads, head_dim, out, stream);
}

la_status la_step_attention_noalloc(const void* q, const void* k_cache, const void* v_cache,
                                    const void* step_k, const void* step_v, int P, int W, int N, int G,
                                    int heads, int kv_heads, int head_dim, void* out, void* stream)
{
    la::FixedWorkspace ws;
    const la_status st = la::fixed_workspace(&ws);
    if (st != LA_OK) return st;
    return step_attention_checked("la_step_attention_noalloc", q, k_cache, v_cache, P, nullptr, 0, 0, step_k, step_v,
                                  P, W, N, G, heads, kv_heads, head_dim, out, stream, nullptr, 0, &ws);
}

la_status la_step_attention_fp8kv(const void* q, const void* k_cache, const void* v_cache, const void* step_k,
                                  const void* step_v, const float* k_scale, const float* v_scale, int P, int W,
                                  int N, int G, int heads, int kv_heads, int head_dim, void* out, void* stream)
{
    if (!k_scale || !v_scale || (((uintptr_t)k_scale | (uintptr_t)v_scale) & 3))
        return la::fail(LA_EINVAL, "la_step_attention_fp8kv: k_scale / v_scale must be 4-byte aligned device arrays");
    return step_attention_checked("la_step_attention_fp8kv", q, k_cache, v_cache, P, nullptr, 0, 0, step_k, step_v,
                                  P, W, N, G, heads, kv_heads, head_dim, out, stream, nullptr, 0, nullptr, k_scale,
                                  v_scale);
}

la_status la_step_attention_rope(const void* q, const void* k_cache, const void* v_cache, const void* step_k,
                                 const void* step_v, const float* cos, const float* sin, int max_pos, int interleaved,
                                 int rotate_keys, int P, int W, int N, int G, int heads, int kv_heads, int head_dim,
                                 void* out, void* stream)
{
    if (P < 0 || W < 0 || G < 0 || N < 2)
        return la::fail(LA_EINVAL, "la_step_attention_rope: need P,W,G >= 0, N >= 2 (got P=%d W=%d N=%d G=%d)", P, W, N, G);
    if (!cos || !sin || (((uintptr_t)cos | (uintptr_t)sin) & 15))
        return la::fail(LA_EINVAL, "la_step_attention_rope: cos / sin must be 16-byte aligned device arrays");
    const long long furthest = (long long)P + (W > 0 && W + N - 2 > N - 1 ? W + N - 2 : (W > 0 || G > 0 ? N - 1 : 0));
    if (max_pos < 1 || furthest >= max_pos)
        return la::fail(LA_EINVAL, "la_step_attention_rope: the tables hold %d positions, the step reaches position %lld",
                        max_pos, furthest);
    const la::RopeTables rope = {cos, sin, interleaved != 0, rotate_keys != 0};
    return step_attention_checked("la_step_attention_rope", q, k_cache, v_cache, P, nullptr, 0, 0, step_k, step_v,
                                  P, W, N, G, heads, kv_heads, head_dim, out, stream, nullptr, 0, nullptr, nullptr,
                                  nullptr, &rope);
}

la_status la_step_attention_cap(const void* q, const void* k_cache, const void* v_cache, long long capacity,
                                const void* step_k, const void* step_v, int P, int W, int N, int G,
                                int heads, int kv_heads, int head_dim, void* out, void* stream)
{
    return step_attention_checked("la_step_attention_cap", q, k_cache, v_cache, capacity, nullptr, 0, 0, step_k,
                                  step_v, P, W, N, G, heads, kv_heads, head_dim, out, stream);
}

namespace {

la_status batch_common_checks(const char* name, const void* seqs, int n_seqs, int W, int N, int G, int heads,
                              int kv_heads, int head_dim)
{
    if (!seqs || n_seqs < 1 || n_seqs > 1024)
        return la::fail(LA_EINVAL, "%s: need 1..1024 descriptors (got %d)", name, n_seqs);
    if (W < 0 || G < 0 || N < 2 || heads < 1 || kv_heads < 1)
        return la::fail(LA_EINVAL, "%s: need W,G >= 0, N >= 2, heads,kv_heads >= 1 "
                                   "(got W=%d N=%d G=%d heads=%d kv_heads=%d)", name, W, N, G, heads, kv_heads);
    if (head_dim != 64 && head_dim != 128)
        return la::fail(LA_EUNSUPPORTED, "%s: head_dim %d is not 64 or 128", name, head_dim);
    if (heads % kv_heads != 0)
        return la::fail(LA_EUNSUPPORTED, "%s: heads %d not a multiple of kv_heads %d", name, heads, kv_heads);
    if (1 + (long long)(W + G) * (N - 1) > (1 << 20)) return la::fail(LA_EINVAL, "%s: step too large", name);
    return LA_OK;
}

}  // namespace

la_status la_step_attention_batch(const la_step_desc* seqs, int n_seqs, int W, int N, int G, int heads,
                                  int kv_heads, int head_dim, void* stream)
{
    const char* name = "la_step_attention_batch";
    la_status st = batch_common_checks(name, seqs, n_seqs, W, N, G, heads, kv_heads, head_dim);
    if (st != LA_OK) return st;
    la::BatchSeq b[1024];
    for (int i = 0; i < n_seqs; ++i) {
        const la_step_desc& d = seqs[i];
        if (d.P < 0 || (long long)d.P > (1ll << 30) || d.reserved != 0)
            return la::fail(LA_EINVAL, "%s: descriptor %d: bad P or reserved field", name, i);
        if (!d.q || !d.step_k || !d.step_v || !d.out || (d.P > 0 && (!d.k_cache || !d.v_cache)))
            return la::fail(LA_EINVAL, "%s: descriptor %d: null pointer", name, i);
        const uintptr_t bits = (uintptr_t)d.q | (uintptr_t)d.k_cache | (uintptr_t)d.v_cache | (uintptr_t)d.step_k |
                               (uintptr_t)d.step_v | (uintptr_t)d.out;
        if (bits & 15) return la::fail(LA_EINVAL, "%s: descriptor %d: buffers must be 16-byte aligned", name, i);
        b[i] = la::BatchSeq{d.q, d.k_cache, d.v_cache, nullptr, d.step_k, d.step_v, d.out, d.P};
    }
    return la::launch_step_attention_batch(b, n_seqs, 0, 0, W, N, G, heads, kv_heads, head_dim, (hipStream_t)stream);
}

la_status la_step_attention_batch_paged(const la_step_desc_paged* seqs, int n_seqs, const void* k_pages,
                                        const void* v_pages, int page_size, int n_pages, int W, int N, int G,
                                        int heads, int kv_heads, int head_dim, void* stream)
{
    const char* name = "la_step_attention_batch_paged";
    la_status st = batch_common_checks(name, seqs, n_seqs, W, N, G, heads, kv_heads, head_dim);
    if (st != LA_OK) return st;
    st = check_pages(name, nullptr, page_size, n_pages, 0);
    if (st != LA_OK) return st;
    if (!k_pages || !v_pages || (((uintptr_t)k_pages | (uintptr_t)v_pages) & 15))
        return la::fail(LA_EINVAL, "%s: page pools are null or not 16-byte aligned", name);
    la::BatchSeq b[1024];
    for (int i = 0; i < n_seqs; ++i) {
        const la_step_desc_paged& d = seqs[i];
        if (d.P < 0 || (long long)d.P > (1ll << 30) || d.reserved != 0)
            return la::fail(LA_EINVAL, "%s: descriptor %d: bad P or reserved field", name, i);
        if (!d.q || !d.step_k || !d.step_v || !d.out || (d.P > 0 && !d.block_table))
            return la::fail(LA_EINVAL, "%s: descriptor %d: null pointer", name, i);
        const uintptr_t bits = (uintptr_t)d.q | (uintptr_t)d.step_k | (uintptr_t)d.step_v | (uintptr_t)d.out;
        if ((bits & 15) || ((uintptr_t)d.block_table & 3))
            return la::fail(LA_EINVAL, "%s: descriptor %d: misaligned buffer", name, i);
        b[i] = la::BatchSeq{d.q, k_pages, v_pages, d.block_table, d.step_k, d.step_v, d.out, d.P};
    }
    return la::launch_step_attention_batch(b, n_seqs, page_size, n_pages, W, N, G, heads, kv_heads, head_dim,
                                           (hipStream_t)stream);
}

la_status la_step_attention_rows(const void* q, const void* k_cache, const void* v_cache, const void* step_k,
                                 const void* step_v, const int* row_ids, int n_rows, int P, int W, int N, int G,
                                 int heads, int kv_heads, int head_dim, void* out, void* stream)
{
    const long long T = 1 + (long long)(W > 0 ? W : 0) * (N - 1) + (long long)(G > 0 ? G : 0) * (N - 1);
    if (n_rows < 1 || n_rows > 1024 || (N >= 2 && n_rows > T))
        return la::fail(LA_EINVAL, "la_step_attention_rows: n_rows %d not in 1..min(1024, rows of the step)", n_rows);
    if (!row_ids || ((uintptr_t)row_ids & 3))
        return la::fail(LA_EINVAL, "la_step_attention_rows: row_ids is null or misaligned");
    return step_attention_checked("la_step_attention_rows", q, k_cache, v_cache, P, nullptr, 0, 0, step_k, step_v, P,
                                  W, N, G, heads, kv_heads, head_dim, out, stream, row_ids, n_rows);
}

la_status la_step_attention_paged(const void* q, const void* k_pages, const void* v_pages, const int* block_table,
                                  int page_size, int n_pages, const void* step_k, const void* step_v, int P,
                                  int W, int N, int G, int heads, int kv_heads, int head_dim, void* out,
                                  void* stream)
{
    const la_status st = check_pages("la_step_attention_paged", block_table, page_size, n_pages, P);
    if (st != LA_OK) return st;
    // with an empty prefix the table is never read
    return step_attention_checked("la_step_attention_paged", q, k_pages, v_pages, 0, P > 0 ? block_table : nullptr,
                                  page_size, n_pages, step_k, step_v, P, W, N, G, heads, kv_heads, head_dim, out,
                                  stream);
}

la_status la_kv_commit_paged(void* k_pages, void* v_pages, const int* block_table, int page_size, int n_pages,
                             const void* step_k, const void* step_v, int P, int W, int N, int G, int kv_heads,
                             int head_dim, const int* best, const int* n_out, void* stream)
{
    if (P < 0 || W < 0 || G < 0 || N < 2 || kv_heads < 1)
        return la::fail(LA_EINVAL, "la_kv_commit_paged: need P,W,G >= 0, N >= 2, kv_heads >= 1 "
                                   "(got P=%d W=%d N=%d G=%d kv_heads=%d)", P, W, N, G, kv_heads);
    if (head_dim < 8 || head_dim % 8 != 0 || head_dim > 1024)
        return la::fail(LA_EUNSUPPORTED, "la_kv_commit_paged: head_dim %d is not a multiple of 8 in 8..1024", head_dim);
    if (1 + (long long)(W + G) * (N - 1) > (1 << 20) || N > 65535 || (long long)P > (1ll << 30))
        return la::fail(LA_EINVAL, "la_kv_commit_paged: step or prefix too large");
    const la_status st = check_pages("la_kv_commit_paged", block_table, page_size, n_pages, (long long)P + N);
    if (st != LA_OK) return st;
    if (!k_pages || !v_pages || !step_k || !step_v || !best || !n_out)
        return la::fail(LA_EINVAL, "la_kv_commit_paged: null pointer");
    if (((uintptr_t)k_pages | (uintptr_t)v_pages | (uintptr_t)step_k | (uintptr_t)step_v) & 15)
        return la::fail(LA_EINVAL, "la_kv_commit_paged: pages and step tensors must be 16-byte aligned");
    if (((uintptr_t)best | (uintptr_t)n_out | (uintptr_t)block_table) & 3)
        return la::fail(LA_EINVAL, "la_kv_commit_paged: best, n_out and block_table must be 4-byte aligned");
    return la::launch_kv_commit(k_pages, v_pages, 0, block_table, page_size, n_pages, step_k, step_v, P, W, N, G,
                                kv_heads, head_dim, best, n_out, (hipStream_t)stream);
}

la_status la_kv_commit(void* k_cache, void* v_cache, long long capacity, const void* step_k,
                       const void* step_v, int P, int W, int N, int G, int kv_heads, int head_dim,
                       const int* best, const int* n_out, void* stream)
{
    if (P < 0 || W < 0 || G < 0 || N < 2 || kv_heads < 1)
        return la::fail(LA_EINVAL, "la_kv_commit: need P,W,G >= 0, N >= 2, kv_heads >= 1 "
                                   "(got P=%d W=%d N=%d G=%d kv_heads=%d)", P, W, N, G, kv_heads);
    if (head_dim < 8 || head_dim % 8 != 0 || head_dim > 1024)
        return la::fail(LA_EUNSUPPORTED, "la_kv_commit: head_dim %d is not a multiple of 8 in 8..1024", head_dim);
    if (1 + (long long)(W + G) * (N - 1) > (1 << 20) || N > 65535)
        return la::fail(LA_EINVAL, "la_kv_commit: step too large");
    // up to N rows are appended; the count is only known on the device
    if (capacity > (1ll << 40) || (long long)P + N > capacity)
        return la::fail(LA_EINVAL, "la_kv_commit: capacity %lld cannot take N = %d more rows after P = %d",
                        capacity, N, P);
    if (!k_cache || !v_cache || !step_k || !step_v || !best || !n_out)
        return la::fail(LA_EINVAL, "la_kv_commit: null pointer");
    if (((uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)step_k | (uintptr_t)step_v) & 15)
        return la::fail(LA_EINVAL, "la_kv_commit: caches and step tensors must be 16-byte aligned");
    if (((uintptr_t)best | (uintptr_t)n_out) & 3)
        return la::fail(LA_EINVAL, "la_kv_commit: best and n_out must be 4-byte aligned");
    return la::launch_kv_commit(k_cache, v_cache, capacity, nullptr, 0, 0, step_k, step_v, P, W, N, G, kv_heads,
                                head_dim, best, n_out, (hipStream_t)stream);
}

la_status la_kv_commit_rope(void* k_cache, void* v_cache, long long capacity, const void* step_k,
                            const void* step_v, const float* cos, const float* sin, int max_pos, int interleaved,
                            int P, int W, int N, int G, int kv_heads, int head_dim, const int* best,
                            const int* n_out, void* stream)
{
    if (P < 0 || W < 0 || G < 0 || N < 2 || kv_heads < 1)
        return la::fail(LA_EINVAL, "la_kv_commit_rope: need P,W,G >= 0, N >= 2, kv_heads >= 1 "
                                   "(got P=%d W=%d N=%d G=%d kv_heads=%d)", P, W, N, G, kv_heads);
    if (head_dim < 16 || head_dim % 16 != 0 || head_dim > 1024)
        return la::fail(LA_EUNSUPPORTED, "la_kv_commit_rope: head_dim %d is not a multiple of 16 in 16..1024", head_dim);
    if (1 + (long long)(W + G) * (N - 1) > (1 << 20) || N > 65535)
        return la::fail(LA_EINVAL, "la_kv_commit_rope: step too large");
    if (capacity > (1ll << 40) || (long long)P + N > capacity)
        return la::fail(LA_EINVAL, "la_kv_commit_rope: capacity %lld cannot take N = %d more rows after P = %d",
                        capacity, N, P);
    // row i of the append is turned by position P + i; a candidate's last token sits at P + N - 1
    const long long furthest = (long long)P + (G > 0 ? N - 1 : 0);
    if (max_pos < 1 || furthest >= max_pos)
        return la::fail(LA_EINVAL, "la_kv_commit_rope: the tables hold %d positions, the append reaches position %lld",
                        max_pos, furthest);
    if (!k_cache || !v_cache || !step_k || !step_v || !cos || !sin || !best || !n_out)
        return la::fail(LA_EINVAL, "la_kv_commit_rope: null pointer");
    if (((uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)step_k | (uintptr_t)step_v | (uintptr_t)cos |
         (uintptr_t)sin) & 15)
        return la::fail(LA_EINVAL, "la_kv_commit_rope: caches, step tensors and tables must be 16-byte aligned");
    if (((uintptr_t)best | (uintptr_t)n_out) & 3)
        return la::fail(LA_EINVAL, "la_kv_commit_rope: best and n_out must be 4-byte aligned");
    return la::launch_kv_commit_rope(k_cache, v_cache, capacity, step_k, step_v, cos, sin, interleaved != 0, P, W, N,
                                     G, kv_heads, head_dim, best, n_out, (hipStream_t)stream);
}

la_status la_kv_commit_batch(const la_commit_desc* descs, int n_descs, int page_size, int n_pages, int W, int N,
                             int G, int kv_heads, int head_dim, void* stream)
{
    const char* name = "la_kv_commit_batch";
    if (n_descs < 1 || n_descs > 1024 || !descs)
        return la::fail(LA_EINVAL, "%s: need 1..1024 descriptors (got %d)", name, n_descs);
    if (W < 0 || G < 0 || N < 2 || kv_heads < 1)
        return la::fail(LA_EINVAL, "%s: need W,G >= 0, N >= 2, kv_heads >= 1 (got W=%d N=%d G=%d kv_heads=%d)",
                        name, W, N, G, kv_heads);
    if (head_dim < 8 || head_dim % 8 != 0 || head_dim > 1024)
        return la::fail(LA_EUNSUPPORTED, "%s: head_dim %d is not a multiple of 8 in 8..1024", name, head_dim);
    if (1 + (long long)(W + G) * (N - 1) > (1 << 20) || N > 65535)
        return la::fail(LA_EINVAL, "%s: step too large", name);
    bool any_paged = false;
    for (int i = 0; i < n_descs; ++i) any_paged = any_paged || descs[i].block_table != nullptr;
    if (any_paged) {
        const la_status st = check_pages(name, nullptr, page_size, n_pages, 0);
        if (st != LA_OK) return st;
    }
    la::CommitSeq c[1024];
    for (int i = 0; i < n_descs; ++i) {
        const la_commit_desc& d = descs[i];
        if (d.P < 0 || (long long)d.P > (1ll << 30) || d.reserved != 0)
            return la::fail(LA_EINVAL, "%s: descriptor %d: bad P or reserved field", name, i);
        if (!d.k_cache || !d.v_cache || !d.step_k || !d.step_v || !d.best || !d.n_out)
            return la::fail(LA_EINVAL, "%s: descriptor %d: null pointer", name, i);
        if (((uintptr_t)d.k_cache | (uintptr_t)d.v_cache | (uintptr_t)d.step_k | (uintptr_t)d.step_v) & 15)
            return la::fail(LA_EINVAL, "%s: descriptor %d: caches and step tensors must be 16-byte aligned", name, i);
        if (((uintptr_t)d.best | (uintptr_t)d.n_out | (uintptr_t)d.block_table) & 3)
            return la::fail(LA_EINVAL, "%s: descriptor %d: best, n_out and block_table must be 4-byte aligned", name, i);
        // up to N rows are appended; the count is only known on the device
        if (!d.block_table && (d.capacity > (1ll << 40) || (long long)d.P + N > d.capacity))
            return la::fail(LA_EINVAL, "%s: descriptor %d: capacity %lld cannot take N = %d more rows after P = %d",
                            name, i, d.capacity, N, d.P);
        c[i] = la::CommitSeq{d.k_cache, d.v_cache, d.block_table, d.step_k, d.step_v, d.best, d.n_out,
                             d.block_table ? 0 : d.capacity, d.P};
    }
    return la::launch_kv_commit_batch(c, n_descs, any_paged ? page_size : 0, any_paged ? n_pages : 0, W, N, G,
                                      kv_heads, head_dim, (hipStream_t)stream);
}

la_status la_step_rope(void* q, void* step_k, const float* cos, const float* sin, int max_pos, int P, int W, int N,
                       int G, int heads, int kv_heads, int head_dim, int interleaved, void* stream)
{
    if (P < 0 || W < 0 || G < 0 || N < 2 || heads < 1 || kv_heads < 1)
        return la::fail(LA_EINVAL, "la_step_rope: need P,W,G >= 0, N >= 2, heads,kv_heads >= 1 "
                                   "(got P=%d W=%d N=%d G=%d heads=%d kv_heads=%d)", P, W, N, G, heads, kv_heads);
    if (head_dim < 16 || head_dim % 16 != 0 || head_dim > 1024)
        return la::fail(LA_EUNSUPPORTED, "la_step_rope: head_dim %d is not a multiple of 16 in 16..1024", head_dim);
    const long long T = 1 + (long long)(W + G) * (N - 1);
    if (T > (1 << 20) || (long long)heads + kv_heads > (1 << 16) || (long long)P > (1ll << 30))
        return la::fail(LA_EINVAL, "la_step_rope: step, heads or prefix too large");
    // the furthest position of the step: the newest window level's last column, or a candidate's last token
    const long long furthest = (long long)P + (W > 0 && W + N - 2 > N - 1 ? W + N - 2 : (W > 0 || G > 0 ? N - 1 : 0));
    if (max_pos < 1 || furthest >= max_pos)
        return la::fail(LA_EINVAL, "la_step_rope: the tables hold %d positions, the step reaches position %lld",
                        max_pos, furthest);
    if (!step_k || !cos || !sin) return la::fail(LA_EINVAL, "la_step_rope: null pointer");
    if (((uintptr_t)q | (uintptr_t)step_k | (uintptr_t)cos | (uintptr_t)sin) & 15)
        return la::fail(LA_EINVAL, "la_step_rope: q, step_k and the tables must be 16-byte aligned");
    return la::launch_step_rope(q, step_k, cos, sin, P, W, N, G, heads, kv_heads, head_dim, interleaved != 0,
                                (hipStream_t)stream);
}

la_status la_verify(const float* logits, const int* cand_tokens, int G, int N, int V,
                    int* accept_len, int* accepted, void* stream)
{
    if (G < 0 || N < 2 || V < 1)
        return la::fail(LA_EINVAL, "la_verify: need G >= 0, N >= 2, V >= 1 (got G=%d N=%d V=%d)", G,
                        N, V);
    if (G == 0) return LA_OK;
    if ((long long)G * (N - 1) > (1 << 20))
        return la::fail(LA_EINVAL, "la_verify: %lld rows is too many", (long long)G * (N - 1));
    if (!logits || !cand_tokens || !accept_len || !accepted)
        return la::fail(LA_EINVAL, "la_verify: null pointer");
    if (((uintptr_t)logits | (uintptr_t)cand_tokens | (uintptr_t)accept_len | (uintptr_t)accepted) & 3)
        return la::fail(LA_EINVAL, "la_verify: buffers must be 4-byte aligned");
    return la::launch_verify(logits, cand_tokens, G, N, V, accept_len, accepted, (hipStream_t)stream);
}

la_status la_verify_step(const float* logits_cur, const float* logits_look, const float* logits_cand,
                         const int* cand_tokens, int W, int N, int G, int V, int* out_tokens, int* n_out,
                         int* best, int* new_window, int* accept_len, void* stream)
{
    if (W < 0 || G < 0 || N < 2 || V < 1)
        return la::fail(LA_EINVAL, "la_verify_step: need W >= 0, G >= 0, N >= 2, V >= 1 (got W=%d G=%d N=%d V=%d)",
                        W, G, N, V);
    if (!logits_cur || !out_tokens || !n_out || !best || (W > 0 && (!logits_look || !new_window)) ||
        (G > 0 && (!logits_cand || !cand_tokens)))
        return la::fail(LA_EINVAL, "la_verify_step: null pointer");
    if (((uintptr_t)logits_cur | (uintptr_t)logits_look | (uintptr_t)logits_cand | (uintptr_t)cand_tokens |
         (uintptr_t)out_tokens | (uintptr_t)n_out | (uintptr_t)best | (uintptr_t)new_window |
         (uintptr_t)accept_len) & 3)
        return la::fail(LA_EINVAL, "la_verify_step: buffers must be 4-byte aligned");
    return la::launch_verify_step(logits_cur, logits_look, logits_cand, cand_tokens, W, N, G, V, out_tokens,
                                  n_out, best, new_window, accept_len, (hipStream_t)stream);
}

la_status la_verify_step_batch(const la_verify_desc* descs, int n_descs, int W, int N, int G, int V, void* stream)
{
    const char* name = "la_verify_step_batch";
    if (n_descs < 1 || n_descs > 1024 || !descs)
        return la::fail(LA_EINVAL, "%s: need 1..1024 descriptors (got %d)", name, n_descs);
    if (W < 0 || G < 0 || N < 2 || V < 1)
        return la::fail(LA_EINVAL, "%s: need W >= 0, G >= 0, N >= 2, V >= 1 (got W=%d G=%d N=%d V=%d)", name, W, G,
                        N, V);
    la::VerifySeq v[1024];
    for (int i = 0; i < n_descs; ++i) {
        const la_verify_desc& d = descs[i];
        if (!d.logits_cur || !d.out_tokens || !d.n_out || !d.best || (W > 0 && (!d.logits_look || !d.new_window)) ||
            (G > 0 && (!d.logits_cand || !d.cand_tokens)))
            return la::fail(LA_EINVAL, "%s: descriptor %d: null pointer", name, i);
        if (((uintptr_t)d.logits_cur | (uintptr_t)d.logits_look | (uintptr_t)d.logits_cand |
             (uintptr_t)d.cand_tokens | (uintptr_t)d.out_tokens | (uintptr_t)d.n_out | (uintptr_t)d.best |
             (uintptr_t)d.new_window | (uintptr_t)d.accept_len) & 3)
            return la::fail(LA_EINVAL, "%s: descriptor %d: buffers must be 4-byte aligned", name, i);
        v[i] = la::VerifySeq{d.logits_cur, d.logits_look, d.logits_cand, d.cand_tokens, d.out_tokens,
                             d.n_out,      d.best,        d.new_window,  d.accept_len};
    }
    return la::launch_verify_step_batch(v, n_descs, W, N, G, V, (hipStream_t)stream);
}

la_status la_verify_sample(const float* logits_cur, const float* logits_cand, const int* cand_tokens,
                           const float* u_test, const float* u_final, float temperature, int N, int G, int V,
                           int* out_tokens, int* n_out, void* stream)
{
    if (G < 0 || N < 2 || V < 1 || !(temperature > 0.0f))
        return la::fail(LA_EINVAL,
                        "la_verify_sample: need G >= 0, N >= 2, V >= 1, temperature > 0 (got G=%d N=%d V=%d T=%g)",
                        G, N, V, (double)temperature);
    if (G > 1024) return la::fail(LA_EUNSUPPORTED, "la_verify_sample: at most 1024 candidates (got %d)", G);
    if (!logits_cur || !u_final || !out_tokens || !n_out || (G > 0 && (!logits_cand || !cand_tokens || !u_test)))
        return la::fail(LA_EINVAL, "la_verify_sample: null pointer");
    if (((uintptr_t)logits_cur | (uintptr_t)logits_cand | (uintptr_t)cand_tokens | (uintptr_t)u_test |
         (uintptr_t)u_final | (uintptr_t)out_tokens | (uintptr_t)n_out) & 3)
        return la::fail(LA_EINVAL, "la_verify_sample: buffers must be 4-byte aligned");
    return la::launch_verify_sample(logits_cur, logits_cand, cand_tokens, u_test, u_final, temperature, N, G, V,
                                    out_tokens, n_out, (hipStream_t)stream);
}

la_status la_verify_sample_batch(const la_sample_desc* descs, int n_descs, int N, int G, int V, void* stream)
{
    const char* name = "la_verify_sample_batch";
    if (n_descs < 1 || n_descs > 1024 || !descs)
        return la::fail(LA_EINVAL, "%s: need 1..1024 descriptors (got %d)", name, n_descs);
    if (G < 0 || N < 2 || V < 1)
        return la::fail(LA_EINVAL, "%s: need G >= 0, N >= 2, V >= 1 (got G=%d N=%d V=%d)", name, G, N, V);
    if (G > 1024) return la::fail(LA_EUNSUPPORTED, "%s: at most 1024 candidates (got %d)", name, G);
    la::SampleSeq v[1024];
    for (int i = 0; i < n_descs; ++i) {
        const la_sample_desc& d = descs[i];
        if (!(d.temperature > 0.0f) || d.reserved != 0)
            return la::fail(LA_EINVAL, "%s: descriptor %d: temperature must be positive, reserved 0", name, i);
        if (!d.logits_cur || !d.u_final || !d.out_tokens || !d.n_out ||
            (G > 0 && (!d.logits_cand || !d.cand_tokens || !d.u_test)))
            return la::fail(LA_EINVAL, "%s: descriptor %d: null pointer", name, i);
        if (((uintptr_t)d.logits_cur | (uintptr_t)d.logits_cand | (uintptr_t)d.cand_tokens | (uintptr_t)d.u_test |
             (uintptr_t)d.u_final | (uintptr_t)d.out_tokens | (uintptr_t)d.n_out) & 3)
            return la::fail(LA_EINVAL, "%s: descriptor %d: buffers must be 4-byte aligned", name, i);
        v[i] = la::SampleSeq{d.logits_cur, d.logits_cand, d.cand_tokens, d.u_test,
                             d.u_final,    d.out_tokens,  d.n_out,       d.temperature};
    }
    return la::launch_verify_sample_batch(v, n_descs, N, G, V, (hipStream_t)stream);
}

long long la_step_attention_workspace_bytes(int P, int W, int N, int G, int heads, int kv_heads,
                                            int head_dim)
{
    if (P < 0 || W < 0 || G < 0 || N < 2 || heads < 1 || kv_heads < 1 || heads % kv_heads != 0 ||
        (head_dim != 64 && head_dim != 128))
        return 0;
    return (long long)la::step_attention_workspace_bytes(P, W, N, G, heads, kv_heads, head_dim);
}

int la_step_attention_kernel(int P, int W, int N, int G, int heads, int kv_heads, int head_dim)
{
    if (P < 0 || W < 0 || G < 0 || N < 2 || heads < 1 || kv_heads < 1 || heads % kv_heads != 0 ||
        (head_dim != 64 && head_dim != 128))
        return -1;
    return la::step_attention_kernel_choice(P, W, N, G, heads, kv_heads, head_dim);
}

la_status la_probe_stream_read(const void* src, long long bytes, void* sink, void* stream)
{
    if (!src || !sink || bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)sink & 3))
        return la::fail(LA_EINVAL, "la_probe_stream_read: need a 16-byte aligned buffer of a multiple of 16 bytes and a sink");
    return la::launch_probe_stream_read(src, bytes, sink, (hipStream_t)stream);
}

long long la_probe_mfma(int iters, void* sink, void* stream)
{
    if (iters < 1 || iters > (1 << 24) || !sink || ((uintptr_t)sink & 7)) {
        la::fail(LA_EINVAL, "la_probe_mfma: need 1 <= iters <= 2^24 and an 8-byte aligned sink of 24 bytes");
        return -1;
    }
    return la::launch_probe_mfma(iters, sink, (hipStream_t)stream);
}

void la_shutdown(void) { la::free_workspaces(); }

la_status la_select_workspace(int set) { return la::select_workspace(set); }

la_status la_debug_override(const char* key, const char* value) { return la::set_override(key, value); }

const char* la_last_error(void) { return la::g_error; }

int la_version(void) { return 1013; }

}  // extern "C"
